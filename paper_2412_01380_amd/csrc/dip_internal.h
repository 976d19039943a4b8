// Internal declarations shared by the libdip translation units (not part of the C ABI).
#ifndef DIP_INTERNAL_H_
#define DIP_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "dip.h"
#include "dip_devtools.h"

namespace dip {

// ---- error reporting -------------------------------------------------------------------
int32_t fail(int32_t status, const char* fmt, ...);
int32_t check_hip(hipError_t e, const char* what);

// ---- optional per-launch timing ---------------------------------------------------------
// Hands out the next (start, stop) event pair for a launch of `kind`, or false when timing
// is off or the pool is used up.
bool prof_next(int kind, hipEvent_t* start, hipEvent_t* stop);

// Launch `kernel`, with timing events bound to the dispatch when the profiler provides them.
template <typename K, typename P>
inline hipError_t launch_timed(K kernel, dim3 grid, dim3 block, hipStream_t stream, int prof_kind,
                               const P& params) {
    hipEvent_t e0, e1;
    if (prof_kind >= 0 && prof_next(prof_kind, &e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, e0, e1, 0, params);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, params);
    }
    return hipGetLastError();
}

// ---- selection kernel (scores -> top-K -> cache update), one workgroup ------------------
constexpr int kSelThreads = 1024;

struct SelectParams {
    const float* v;               // input vector (x or h~), n floats
    int n;
    int k;
    const uint32_t* score_bits;   // residency used for scoring (Eq. 10), or null for |v|
    float gamma;
    const uint32_t* mask_in;      // non-null: take the mask from here instead of selecting
    int scores_only;              // 1: write s_out and return
    float* s_out;                 // nullable
    uint32_t* mask_out;           // nullable
    int32_t* idx_out;             // nullable, k entries
    float* val_out;               // nullable, k entries: v at the selected indices
    // cache update (all null/0 -> none)
    uint32_t* c_bits;
    uint32_t* c_stamp;
    uint32_t* c_meta;
    int capacity;
    int policy;
    // counters the following GEMV launch expects to be zero
    uint32_t* zero_ptr;
    int zero_n;
    // words of the columns this update evicted / inserted (nullable; only with a cache update)
    uint32_t* evicted_out;
    uint32_t* inserted_out;
    // rows > 1: one workgroup per row; row b reads v + b*v_row_stride and writes its mask at
    // mask_out + b*words_row_stride (the other outputs and the cache update must be off)
    int rows;
    int64_t v_row_stride;
    int64_t words_row_stride;
    // nullable: row b (one workgroup per row; row 0 otherwise) writes the bit pattern of max |v| here
    uint32_t* rowmax_out;
};

hipError_t launch_select(const SelectParams& p, hipStream_t stream, int prof_kind);
// The row selections of a small batch (rows >= 1, one workgroup per row): mask_out and, if
// given, rowmax_out only; every other output of SelectParams must be off.
hipError_t launch_select_rows(const SelectParams& p, hipStream_t stream, int prof_kind);

// Cache updates of several caches in one launch, one workgroup each (nothing in the token
// that produced the masks waits for them).
struct UpdatePiece {
    const uint32_t* mask;         // this token's mask words
    uint32_t* bits;
    uint32_t* stamp;
    uint32_t* meta;
    int n;
    int capacity;
    int policy;
    int pad;
};
hipError_t launch_update_batch(const UpdatePiece* pieces, int count, hipStream_t stream, int prof_kind);

struct CacheInitParams {
    uint32_t* bits;
    uint32_t* stamp;
    uint32_t* meta;
    const uint32_t* initial_bits;
    int n;
};
hipError_t launch_cache_init(const CacheInitParams& p, hipStream_t stream);
hipError_t launch_zero_u32(uint32_t* p, int n, hipStream_t stream);

// ---- gathered GEMV -----------------------------------------------------------------------
struct GemvShape {
    int lpr;     // lanes per stored row
    int waves;   // wavefronts per workgroup
    int ksplit;  // workgroups per output strip
    int unroll;  // rows in flight per lane group
};

struct GemvParams {
    const void* w;            // feature-major weights
    int64_t row_stride;       // bytes
    const uint16_t* scales;   // DIP_INT4_G128: fp16 bit patterns, scale_stride per stored row
    int scale_stride;
    int dtype;                // DIP_F32 | DIP_BF16
    int n_in;                 // stored rows
    int n_out;                // elements per row actually produced per segment
    int nseg;                 // 1: plain GEMV;  2: bundled [up ; gate] with SwiGLU epilogue
    const int32_t* idx;       // k ascending row indices (16-byte aligned); null: rows 0..k-1
    const float* val;         // val[t] multiplies row idx[t] (16-byte aligned)
    int k;
    int rows_per_split;       // ceil(k / ksplit), filled in by launch_gemv
    float* out;               // n_out floats (nseg == 2: the GLU output, n_out = d_ff)
    float* partial;           // [ksplit][nseg][n_out] when ksplit > 1
    uint32_t* counters;       // [strips], zero on entry, when ksplit > 1
    int act;                  // nseg == 1 only: 0 writes the sums, 1 writes SiLU of the sums
    const void* w_alt;        // second matrix for list entries r < 0 (stored row ~r), same dtype and
    int n_alt;                // row stride, n_alt rows; null / 0 when there is none
};

// ---- row-gathered dot products (Sec. 3.2, Gate / Up pruning) ---------------------------------
struct RowdotParams {
    const void* w;            // neuron-major: stored row j = row j of the paper's matrix
    int64_t row_stride;       // bytes
    const uint16_t* scales;
    int scale_stride;
    int dtype;
    int n_rows;
    int n_cols;
    const int32_t* idx;       // k ascending stored-row indices
    int k;
    const float* x;           // n_cols
    const float* a;           // n_rows partial activations, or null when mode == 0
    int mode;                 // 0: out[t] = w[idx[t]] . x
                              // 1: out[t] = (w[idx[t]] . x) * a[idx[t]]
                              // 2: out[t] = a[idx[t]] * SiLU(w[idx[t]] . x)
    float* out;               // k
};
hipError_t launch_rowdot(const RowdotParams& p, hipStream_t stream, int prof_kind);

GemvShape choose_gemv_shape(int dtype, int n_out, int nseg, int k);
int gemv_strips(const GemvShape& s, int dtype, int n_out);
hipError_t launch_gemv(const GemvParams& p, const GemvShape& s, hipStream_t stream, int prof_kind);
// val[t] = x[idx[t]] (0 for an index outside [0, n)) and idx_copy[t] = idx[t], for t < k
hipError_t launch_gather(const float* x, const int32_t* idx, int k, int n, float* val, int32_t* idx_copy,
                         hipStream_t stream);

extern GemvShape g_gemv_override;
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream, int prof_kind);

// ---- gathered product with the selection at its head (one launch for Alg. 1 steps 1, 2, 4) ----
constexpr int kFusedListCap = 2048;   // rows of one workgroup's share (index + multiplier in LDS)
constexpr int kFusedMaxIn = 8192;     // longest input vector of the bundled up/gate product
struct FusedSelect {
    const float* v;               // the vector the mask is taken from (x or h~), n floats
    int n;
    const uint32_t* score_bits;   // residency for Eq. 10 scores, or null for |v|
    float gamma;
    // launch-wide outputs, written by one workgroup (mask, scores) or the workgroups of strip 0
    // (index list); each may be null
    uint32_t* mask_out;
    int32_t* idx_out;
    float* s_out;
};
struct FusedParams {
    GemvParams g;                 // idx / val are ignored: the lists live in LDS
    FusedSelect s;
};
// false when no kernel covers the shape (then the caller launches selection and product apart)
bool fused_shape(int dtype, int n_sel, int n_out, int nseg, int k, GemvShape* shape);
hipError_t launch_fused(const FusedParams& p, const GemvShape& s, hipStream_t stream, int prof_kind);
hipError_t launch_fused_1_0(const FusedParams&, const GemvShape&, hipStream_t, int);
hipError_t launch_fused_1_1(const FusedParams&, const GemvShape&, hipStream_t, int);
hipError_t launch_fused_1_2(const FusedParams&, const GemvShape&, hipStream_t, int);
hipError_t launch_fused_2_0(const FusedParams&, const GemvShape&, hipStream_t, int);
hipError_t launch_fused_2_1(const FusedParams&, const GemvShape&, hipStream_t, int);
hipError_t launch_fused_2_2(const FusedParams&, const GemvShape&, hipStream_t, int);
extern int g_fusion;              // 0: always launch selection and product apart

// ---- small batches: union of row masks, batched gathered product, reduction ------------------
struct UnionParams {
    const uint32_t* masks;     // [batch][words_stride]
    int64_t words_stride;
    const float* x;            // [batch][x_stride] activations the masks were taken from
    int64_t x_stride;
    int n;
    int batch;
    uint32_t* union_words;     // ceil(n/32)
    int32_t* uidx;             // ascending indices of the union, up to min(n, batch*k)
    float* uval;               // [listed][batch]: x[b][i] if row b selected i, else 0
    uint32_t* count_out;       // number of listed indices
};
struct BatchedGemvParams {
    const void* w;
    int64_t row_stride;
    const uint16_t* scales;
    int scale_stride;
    int dtype;
    int n_in;
    int n_out;                 // full stored row width
    const int32_t* uidx;
    const float* uval;
    const uint32_t* k_dev;     // listed columns (device)
    int k_max;                 // capacity of the lists
    int batch;
    float* partial;            // [shares][batch][n_out]
    const uint32_t* rowmax;    // [batch] bit patterns of max |x[b]| from the row selection (matrix-core product only)
};
struct BatchedReduceParams {
    const float* partial;
    int shares;
    int batch;
    int n_out;
    int glu;                   // 1: out = up * SiLU(gate) over the two halves of a row
    float* out;
    int64_t out_stride;
};
bool batched_on_matrix_cores(int dtype, int batch, int64_t n_in, int64_t row_stride);
int batched_strip_cols(int dtype, int batch, bool mc);
int batched_shares(int dtype, int batch, int n_out, int k_max, bool mc);
hipError_t launch_union(const UnionParams& p, hipStream_t stream);
hipError_t launch_batched_gemv(const BatchedGemvParams& p, int shares, bool mc, hipStream_t stream, int prof_kind);
hipError_t launch_batched_reduce(const BatchedReduceParams& p, hipStream_t stream);

// ---- two-tier residency: slot map of the HBM cache, fill list, encoded row list -----------------
struct TierParams {
    const uint32_t* evicted;   // words from the cache update of this token
    const uint32_t* inserted;
    const uint32_t* meta;      // the cache's counters after that update
    int n;                     // columns
    int capacity;              // slots
    int32_t* slot_of;          // [n]: slot of a resident column, -1 otherwise
    int32_t* fill_col;         // [<= capacity] inserted columns ...
    int32_t* fill_slot;        // ... and the slots they were given
    uint32_t* fill_count;
    const int32_t* idx;        // this token's selected columns (k ascending), or null
    int k;
    int32_t* src;              // [k]: slot s >= 0 of a resident column, ~column otherwise
};
struct TierFillParams {
    const void* host_rows;     // full matrix, device-accessible host memory
    void* slots;               // HBM cache
    int64_t row_stride;        // bytes, both tiers
    int64_t row_bytes;
    const int32_t* fill_col;
    const int32_t* fill_slot;
    const uint32_t* fill_count;
    int max_rows;
};
struct TierInitParams {
    const uint32_t* bits;      // residency words
    int n;
    int32_t* slot_of;
    int32_t* fill_col;
    int32_t* fill_slot;
    uint32_t* fill_count;
};
hipError_t launch_tier_update(const TierParams& p, hipStream_t stream);
hipError_t launch_tier_fill(const TierFillParams& p, hipStream_t stream, int prof_kind);
hipError_t launch_tier_init(const TierInitParams& p, hipStream_t stream);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace dip

#endif  // DIP_INTERNAL_H_
