// Column-gathered GEMV (Alg. 1 step 4 applied to x; Sec. 4 for the bundled up/gate case):
//     y[j] = sum_{t<k} W[j, idx[t]] * x[idx[t]]
// over a feature-major matrix, so each selected column is one contiguous row in HBM.
//
// Decode at batch 1 reads every selected weight exactly once and does two flops per
// element: the kernel is bound by HBM bandwidth, not arithmetic, so there are no matrix
// cores here -- only wide coalesced loads, many of them in flight, and fp32 FMAs.
//
// Work split.  The outputs are cut into strips of LPR*EPL columns (EPL = elements per
// 16-byte load).  A workgroup owns one strip (both the up and the gate strip when the
// matrix is the bundled pair) and a contiguous share of the k selected rows; inside it
// every wavefront handles 64/LPR rows per step, LPR lanes side by side on one row, each
// lane loading 16 bytes.  Sums are combined in a fixed order: lane groups inside a
// wavefront (xor butterfly), wavefronts through LDS in index order, workgroups of one
// strip through a partial buffer that the last workgroup to arrive adds in index order.
// The result is bit-repeatable for a given launch shape.

#include "dip_internal.h"

namespace dip {

GemvShape g_gemv_override = {0, 0, 0, 0};
constexpr int kComputeUnits = 256;   // MI355X

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename WT>
struct Elem;
struct q4_t {};  // tag: signed 4-bit codes, one fp16 scale per 128 consecutive elements of a row

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <>
struct Elem<float> {
    typedef u32x4 raw_t;
    static constexpr int kPerLoad = 4;
    static constexpr int kBits = 32;
    static constexpr bool kScaled = false;
    __device__ static __forceinline__ void widen(const u32x4& q, float (&f)[4]) {
        f[0] = __uint_as_float(q.x);
        f[1] = __uint_as_float(q.y);
        f[2] = __uint_as_float(q.z);
        f[3] = __uint_as_float(q.w);
    }
};
template <>
struct Elem<uint16_t> {  // bfloat16: the upper half of an fp32 pattern
    typedef u32x4 raw_t;
    static constexpr int kPerLoad = 8;
    static constexpr int kBits = 16;
    static constexpr bool kScaled = false;
    __device__ static __forceinline__ void widen(const u32x4& q, float (&f)[8]) {
        f[0] = __uint_as_float(q.x << 16);
        f[1] = __uint_as_float(q.x & 0xffff0000u);
        f[2] = __uint_as_float(q.y << 16);
        f[3] = __uint_as_float(q.y & 0xffff0000u);
        f[4] = __uint_as_float(q.z << 16);
        f[5] = __uint_as_float(q.z & 0xffff0000u);
        f[6] = __uint_as_float(q.w << 16);
        f[7] = __uint_as_float(q.w & 0xffff0000u);
    }
};

template <>
struct Elem<q4_t> {
    // 32 codes per 16-byte load, low nibble = even element.  Flipping bit 3 of every nibble
    // turns the two's-complement code q into q + 8 in [0, 15]; masking even and odd nibbles
    // apart leaves them as bytes, which convert to float in one instruction each.  The
    // caller removes the offset: sum (q + 8) m - 8 sum m.
    typedef u32x4 raw_t;
    static constexpr int kPerLoad = 32;
    static constexpr int kBits = 4;
    static constexpr bool kScaled = true;
    __device__ static __forceinline__ void widen(const u32x4& q, float (&f)[32]) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t o = w[i] ^ 0x88888888u;
            uint32_t ev = o & 0x0f0f0f0fu, od = (o >> 4) & 0x0f0f0f0fu;
            // keep the compiler from narrowing the byte extracts below into bit-field
            // extracts: a byte of a register converts to float in one instruction
            asm volatile("" : "+v"(ev), "+v"(od));
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f[i * 8 + 2 * b] = (float)((ev >> (8 * b)) & 0xffu);
                f[i * 8 + 2 * b + 1] = (float)((od >> (8 * b)) & 0xffu);
            }
        }
    }
};

struct q4n_t {};  // tag: the same 4-bit format read 8 bytes (16 codes) per lane
template <>
struct Elem<q4n_t> {
    // The column-gathered product keeps one accumulator per code and output segment in
    // registers; with 32 codes per lane that is 64 accumulators and 163 registers, one
    // workgroup per compute unit, and every latency of a workgroup's prologue and reduction
    // is exposed (about 8 us per workgroup).  Half the codes per lane halve the
    // accumulators, and two to three workgroups share a compute unit.
    typedef u32x2 raw_t;
    static constexpr int kPerLoad = 16;
    static constexpr int kBits = 4;
    static constexpr bool kScaled = true;
    __device__ static __forceinline__ void widen(const u32x2& q, float (&f)[16]) {
        const uint32_t w[2] = {q.x, q.y};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t o = w[i] ^ 0x88888888u;
            uint32_t ev = o & 0x0f0f0f0fu, od = (o >> 4) & 0x0f0f0f0fu;
            asm volatile("" : "+v"(ev), "+v"(od));
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f[i * 8 + 2 * b] = (float)((ev >> (8 * b)) & 0xffu);
                f[i * 8 + 2 * b + 1] = (float)((od >> (8 * b)) & 0xffu);
            }
        }
    }
};

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
    _Float16 v;
    __builtin_memcpy(&v, &h, 2);
    return (float)v;
}

__device__ __forceinline__ u32x4 load16(const char* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
template <typename RAW>
__device__ __forceinline__ RAW load_raw(const char* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const RAW*>(p));
}

__device__ __forceinline__ float silu(float g) { return g / (1.0f + expf(-g)); }

template <typename WT, int LPR, int WAVES, int UNROLL, int NSEG>
__global__ __launch_bounds__(WAVES * 64) void gemv_kernel(GemvParams p) {
    constexpr int EPL = Elem<WT>::kPerLoad;
    constexpr int RPW = 64 / LPR;          // rows per wavefront step
    constexpr int SC = LPR * EPL;          // strip columns
    __shared__ float red[WAVES][NSEG][SC];
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, l = lane % LPR;
    const int strip = blockIdx.x;
    const int g = blockIdx.y, G = gridDim.y;
    const int col_raw = strip * SC + l * EPL;
    const bool col_ok = col_raw < p.n_out;
    // lanes past the right edge of a ragged last strip re-read its last 16 bytes; they own no output
    const int col = col_ok ? col_raw : p.n_out - EPL;

    // this workgroup's share of the selected rows
    const int kb = min(p.k, g * p.rows_per_split);   // rows_per_split is a multiple of 8
    const int ke = min(p.k, kb + p.rows_per_split);

    float acc[NSEG][EPL];
    float msum[NSEG];   // quantised rows: sum of the row multipliers, for the code offset
#pragma unroll
    for (int s = 0; s < NSEG; ++s) {
        msum[s] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[s][e] = 0.f;
    }

    const char* wbase = static_cast<const char*>(p.w) + (size_t)col * Elem<WT>::kBits / 8;
    const char* abase = p.w_alt ? static_cast<const char*>(p.w_alt) + (size_t)col * Elem<WT>::kBits / 8 : wbase;
    const size_t seg_bytes = (size_t)p.n_out * Elem<WT>::kBits / 8;
    // quantised rows: the scale of this lane's 32 codes (all inside one group of 128)
    const int sgroup = col >> 7, sgroups_per_seg = p.n_out >> 7;
    constexpr int NG = WAVES * RPW;            // lane groups per workgroup
    constexpr int ROWS_PER_ITER = UNROLL * NG;

    // Every lane group takes UNROLL consecutive selected rows per iteration, so their
    // indices and multipliers arrive as one vector load each.  Full iterations need no
    // predicates; the pairs of the next iteration are requested right after this
    // iteration's weight loads so that their latency hides behind the weights.
    const int gid = wave * RPW + sub;
    const int n_full = (ke - kb) / ROWS_PER_ITER;   // the same for every lane
    const bool ident = p.idx == nullptr;       // every stored row in order (a dense product)
    int t0 = kb + gid * UNROLL;

    auto fetch_pairs = [&](int t, int (&row)[UNROLL], float (&xv)[UNROLL]) {
        if constexpr (UNROLL % 4 == 0) {
#pragma unroll
            for (int u = 0; u < UNROLL; u += 4) {
                const float4 x4 = *reinterpret_cast<const float4*>(p.val + t + u);
                int4 r4 = make_int4(t + u, t + u + 1, t + u + 2, t + u + 3);
                if (!ident) r4 = *reinterpret_cast<const int4*>(p.idx + t + u);
                row[u] = r4.x; row[u + 1] = r4.y; row[u + 2] = r4.z; row[u + 3] = r4.w;
                xv[u] = x4.x; xv[u + 1] = x4.y; xv[u + 2] = x4.z; xv[u + 3] = x4.w;
            }
        } else if constexpr (UNROLL == 2) {
            const float2 x2 = *reinterpret_cast<const float2*>(p.val + t);
            int2 r2 = make_int2(t, t + 1);
            if (!ident) r2 = *reinterpret_cast<const int2*>(p.idx + t);
            row[0] = r2.x; row[1] = r2.y;
            xv[0] = x2.x; xv[1] = x2.y;
        } else {
            xv[0] = p.val[t];
            row[0] = t;
            if (!ident) row[0] = p.idx[t];
        }
    };
    // A list entry r >= 0 is stored row r of p.w; an entry r < 0 is stored row ~r of the second
    // matrix p.w_alt (two-tier residency: the copy of the full matrix in host memory).  An
    // entry outside its matrix reads row 0 with multiplier 0.
    auto settle_pairs = [&](int (&row)[UNROLL], float (&xv)[UNROLL], uint32_t& alt) {
        alt = 0u;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const bool second = row[u] < 0;
            const int r = second ? ~row[u] : row[u];
            const bool inside = (unsigned)r < (unsigned)(second ? p.n_alt : p.n_in);
            row[u] = inside ? r : 0;
            xv[u] = inside ? xv[u] : 0.f;
            alt |= (inside && second) ? (1u << u) : 0u;
        }
    };
    int row[UNROLL];
    float xv[UNROLL];
    uint32_t alt = 0u;
    auto fetch_full = [&](int t) { fetch_pairs(t, row, xv); settle_pairs(row, xv, alt); };

    if (n_full > 0) fetch_full(t0);
    for (int it = 0; it < n_full; ++it) {
        typename Elem<WT>::raw_t q[UNROLL][NSEG];
        uint16_t sc[UNROLL][NSEG];
        float xc[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t off = (size_t)row[u] * (size_t)p.row_stride;
            const char* src = ((alt >> u) & 1u) ? abase : wbase;
            xc[u] = xv[u];
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                q[u][s] = load_raw<typename Elem<WT>::raw_t>(src + off + s * seg_bytes);
                if constexpr (Elem<WT>::kScaled)
                    sc[u][s] = p.scales[(size_t)row[u] * p.scale_stride + s * sgroups_per_seg + sgroup];
            }
        }
        t0 += ROWS_PER_ITER;
        if (it + 1 < n_full) fetch_full(t0);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                float f[EPL];
                Elem<WT>::widen(q[u][s], f);
                float mult = xc[u];
                if constexpr (Elem<WT>::kScaled) {
                    mult *= half_bits_to_float(sc[u][s]);
                    msum[s] += mult;
                }
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[s][e] = fmaf(f[e], mult, acc[s][e]);
            }
        }
    }
    // Tail: fewer than ROWS_PER_ITER rows are left; rows past the end are skipped.
    if (col_ok && t0 < ke) {
        typename Elem<WT>::raw_t q[UNROLL][NSEG];
        uint16_t sc[UNROLL][NSEG];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int t = t0 + u;
            row[u] = -1;
            xv[u] = 0.f;
            if (t < ke) {
                const int e = ident ? t : p.idx[t];
                const bool second = e < 0;
                const int r = second ? ~e : e;
                if ((unsigned)r < (unsigned)(second ? p.n_alt : p.n_in)) {
                    row[u] = r;
                    xv[u] = p.val[t];
                    alt = second ? (alt | (1u << u)) : (alt & ~(1u << u));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                q[u][s] = typename Elem<WT>::raw_t{};
                sc[u][s] = 0;
                if (row[u] >= 0) {
                    const char* src = ((alt >> u) & 1u) ? abase : wbase;
                    q[u][s] = load_raw<typename Elem<WT>::raw_t>(src + (size_t)row[u] * (size_t)p.row_stride + s * seg_bytes);
                    if constexpr (Elem<WT>::kScaled)
                        sc[u][s] = p.scales[(size_t)row[u] * p.scale_stride + s * sgroups_per_seg + sgroup];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                float f[EPL];
                Elem<WT>::widen(q[u][s], f);
                float mult = xv[u];
                if constexpr (Elem<WT>::kScaled) {
                    mult *= half_bits_to_float(sc[u][s]);
                    msum[s] += mult;
                }
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[s][e] = fmaf(f[e], mult, acc[s][e]);
            }
        }
    }

    if constexpr (Elem<WT>::kScaled) {
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[s][e] = fmaf(-8.0f, msum[s], acc[s][e]);
    }

    // lane groups of one wavefront
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[s][e] += __shfl_xor(acc[s][e], off);
    }
    if (sub == 0) {
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
#pragma unroll
            for (int e = 0; e < EPL; ++e) red[wave][s][l * EPL + e] = acc[s][e];
    }
    __syncthreads();

    // wavefronts of one workgroup: lane c of the first NSEG*SC lanes owns one output
    constexpr int NOUT = NSEG * SC;
    static_assert(NOUT <= WAVES * 64, "strip wider than the workgroup");  // launch_nseg guards this
    const int oseg = tid / SC, ocol = tid % SC;
    const int gcol = strip * SC + ocol;
    const bool owner = tid < NOUT && gcol < p.n_out;
    float sum = 0.f;
    if (owner) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[w][oseg][ocol];
    }

    if (G > 1) {
        // Workgroups of one strip.  Partial sums travel through agent-scope atomics, which
        // are written through to (and read from) the memory side where all eight L2s agree,
        // so no L2 write-back or invalidate is needed: waiting for the stores to be
        // acknowledged (vmcnt = 0) before this workgroup's ticket is taken orders them
        // before any read by the workgroup that draws the last ticket.
        float* part = p.partial + ((size_t)g * NSEG + oseg) * (size_t)p.n_out + gcol;
        if (owner) __hip_atomic_store(part, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(&p.counters[strip], 1u, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            s_last = (prev == (uint32_t)(G - 1));
        }
        __syncthreads();
        if (!s_last) return;
        // eight partial sums in flight at a time, added in workgroup order
        sum = 0.f;
        if (owner) {
            const float* src0 = p.partial + (size_t)oseg * (size_t)p.n_out + gcol;
            const size_t gstride = (size_t)NSEG * (size_t)p.n_out;
            for (int g0 = 0; g0 < G; g0 += 8) {
                float part8[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int gg = g0 + j < G ? g0 + j : G - 1;
                    part8[j] = __hip_atomic_load(src0 + (size_t)gg * gstride, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (g0 + j < G) sum += part8[j];
            }
        }
    }

    if constexpr (NSEG == 2) {
        // Sec. 3 Eq. 2: GLU = up (.) SiLU(gate); the gate sums sit SC lanes further on
        __syncthreads();
        if (owner) red[0][oseg][ocol] = sum;
        __syncthreads();
        if (owner && oseg == 0) p.out[gcol] = red[0][0][ocol] * silu(red[0][1][ocol]);
    } else {
        if (owner) p.out[gcol] = p.act == 1 ? silu(sum) : sum;
    }
}

// ---------------------------------------------------------------------------------------
// Row-gathered dot products (Sec. 3.2, Gate / Up pruning): the matrix whose rows a mask
// removes is stored neuron-major, so the selected neuron j is one contiguous row and
//     out[t] = W[idx[t], :] . x
// streams k whole rows.  One wavefront takes one row at a time, 16 bytes per lane.  A row is
// cut into chunks of P loads per lane (one chunk when the row fits); the loads of the next
// chunk are issued into a second set of registers before the current chunk is multiplied,
// so a wavefront always has one to two chunks outstanding.  The steady-state step has no
// lane-dependent branch -- columns past the end of a row are re-read from its last 16
// bytes and dropped by a select -- which lets the compiler wait for exactly the older
// chunk.  x sits in LDS, laid out in planes of 64 x 16 bytes so that the lanes of a
// wavefront read consecutive 16-byte pieces.  The sum runs over this lane's elements in
// column order, then across lanes in a fixed butterfly: bit-repeatable.
// ---------------------------------------------------------------------------------------
constexpr int kRowdotWaves = 4;

template <typename WT, int P, bool SINGLE>
__global__ __launch_bounds__(kRowdotWaves * 64) void rowdot_kernel(RowdotParams p, int rows_per_wg, int nchunks) {
    extern __shared__ __align__(16) float xs[];
    constexpr int EPL = Elem<WT>::kPerLoad;
    constexpr int PLANES = EPL / 4;          // 16-byte pieces of x per weight load
    constexpr int STEP = 64 * EPL;
    constexpr int CHUNK = P * STEP;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int t_begin = blockIdx.x * rows_per_wg;
    const int t_end = min(p.k, t_begin + rows_per_wg);

    // element j of x: load group g = j / EPL (one lane's 16 bytes of weights), piece h of it
    for (int j = tid * 4; j < p.n_cols; j += kRowdotWaves * 64 * 4) {
        const int g = j / EPL, h = (j % EPL) / 4;
        *reinterpret_cast<float4*>(xs + ((g >> 6) * PLANES + h) * 256 + (g & 63) * 4) =
            *reinterpret_cast<const float4*>(p.x + j);
    }
    __syncthreads();

    // This wavefront's rows: list positions t0, t0 + 4, ... (at most 64 of them: lane i holds
    // the index and the partial activation of the i-th, fetched once, handed out with
    // readlane so that everything that steers the loop sits in scalar registers).
    // A unit is one chunk of one row.
    const int t0 = t_begin + wave;
    if (t0 >= t_end) return;
    const int n_rows_w = (t_end - t0 + kRowdotWaves - 1) / kRowdotWaves;
    const int n_units = SINGLE ? n_rows_w : n_rows_w * nchunks;
    const int last_col = p.n_cols - EPL;
    int my_r = 0;
    float my_av = 0.f;
    bool my_ok = false;
    if (lane < n_rows_w) {
        my_r = p.idx[t0 + kRowdotWaves * lane];
        my_ok = (unsigned)my_r < (unsigned)p.n_rows;   // a row outside the matrix contributes nothing
        if (!my_ok) my_r = 0;
        if (p.a) my_av = p.a[my_r];
    }
    const uint64_t ok_rows = __ballot(my_ok);

    struct Buf {
        u32x4 q[P];
        uint16_t sc[P];
    };
    auto issue = [&](int u, Buf& b) {
        const int i = SINGLE ? u : u / nchunks;
        const int c0 = SINGLE ? 0 : (u - i * nchunks) * CHUNK;
        const int r = __builtin_amdgcn_readlane(my_r, i);
        const char* row = static_cast<const char*>(p.w) + (size_t)r * (size_t)p.row_stride;
#pragma unroll
        for (int v = 0; v < P; ++v) {
            const int c = min(c0 + v * STEP + lane * EPL, last_col);
            b.q[v] = load16(row + (size_t)c * Elem<WT>::kBits / 8);
            b.sc[v] = 0;
            if constexpr (Elem<WT>::kScaled) b.sc[v] = p.scales[(size_t)r * p.scale_stride + (c >> 7)];
        }
    };
    float dot = 0.f;
    auto consume = [&](int u, const Buf& b) {
        const int i = SINGLE ? u : u / nchunks;
        const int cc = SINGLE ? 0 : u - i * nchunks;
        const int c0 = cc * CHUNK;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < P; ++v) {
            const int craw = c0 + v * STEP + lane * EPL;
            const int c = min(craw, last_col);
            const int g = c / EPL;
            const float* xp = xs + (g >> 6) * (PLANES * 256) + (g & 63) * 4;
            float f[EPL];
            Elem<WT>::widen(b.q[v], f);
            float part[4] = {0.f, 0.f, 0.f, 0.f}, xsum = 0.f;
#pragma unroll
            for (int h = 0; h < PLANES; ++h) {
                const float4 xv = *reinterpret_cast<const float4*>(xp + h * 256);
                part[0] = fmaf(f[4 * h], xv.x, part[0]);
                part[1] = fmaf(f[4 * h + 1], xv.y, part[1]);
                part[2] = fmaf(f[4 * h + 2], xv.z, part[2]);
                part[3] = fmaf(f[4 * h + 3], xv.w, part[3]);
                if constexpr (Elem<WT>::kScaled) xsum += (xv.x + xv.y) + (xv.z + xv.w);
            }
            const bool live = craw < p.n_cols;
            if constexpr (Elem<WT>::kScaled) {
                // codes arrive offset by 8 (see Elem<q4_t>)
                const float sv = half_bits_to_float(b.sc[v]);
                const float val = ((part[0] + part[1]) + (part[2] + part[3])) - 8.0f * xsum;
                acc[v & 3] += live ? sv * val : 0.f;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += live ? part[e] : 0.f;
            }
        }
        dot += (acc[0] + acc[1]) + (acc[2] + acc[3]);
        if (!SINGLE && cc != nchunks - 1) return;
        // the last chunk of row i has been added
        float total = dot;
        dot = 0.f;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) total += __shfl_xor(total, off);
        const float av = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_av), i));
        float o = total;
        if (p.mode == 1) o = total * av;
        if (p.mode == 2) o = av * silu(total);
        if (!((ok_rows >> i) & 1ull)) o = 0.f;
        if (lane == 0) p.out[t0 + kRowdotWaves * i] = o;
    };

    Buf A, B;
    issue(0, A);
    int u = 0;
    while (true) {
        if (u + 1 == n_units) { consume(u, A); break; }
        issue(u + 1, B);
        consume(u, A);
        ++u;
        if (u + 1 == n_units) { consume(u, B); break; }
        issue(u + 1, A);
        consume(u, B);
        ++u;
    }
}

template <typename WT, int P, bool SINGLE>
hipError_t launch_rowdot_p(const RowdotParams& p, int nchunks, hipStream_t stream, int pk) {
    // one resident generation of workgroups (two per compute unit), whole rows per wavefront
    int rows_per_wg = (p.k + 511) / 512;
    rows_per_wg = (rows_per_wg + kRowdotWaves - 1) / kRowdotWaves * kRowdotWaves;
    if (rows_per_wg > 64 * kRowdotWaves) rows_per_wg = 64 * kRowdotWaves;   // one row per lane of a wavefront at most
    const int grid = (p.k + rows_per_wg - 1) / rows_per_wg;
    constexpr int STEP = 64 * Elem<WT>::kPerLoad;
    const size_t lds = sizeof(float) * (size_t)((p.n_cols + STEP - 1) / STEP) * STEP;
    auto kernel = rowdot_kernel<WT, P, SINGLE>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipEvent_t e0, e1;
    if (pk >= 0 && prof_next(pk, &e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(kRowdotWaves * 64), lds, stream, e0, e1, 0, p,
                              rows_per_wg, nchunks);
    } else {
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(kRowdotWaves * 64), lds, stream, p, rows_per_wg, nchunks);
    }
    return hipGetLastError();
}

template <typename WT>
hipError_t launch_rowdot_t(const RowdotParams& p, hipStream_t stream, int pk) {
    const int step = 64 * Elem<WT>::kPerLoad;
    const int passes = (p.n_cols + step - 1) / step;
    // whole row in flight, twice (x then stays in registers) ...
    if (passes <= 2) return launch_rowdot_p<WT, 2, true>(p, 1, stream, pk);
    if (passes <= 4) return launch_rowdot_p<WT, 4, true>(p, 1, stream, pk);
    if (passes <= 6) return launch_rowdot_p<WT, 6, true>(p, 1, stream, pk);
    if (passes <= 8) return launch_rowdot_p<WT, 8, true>(p, 1, stream, pk);
    // ... or in two or more chunks when that would not fit the register file
    if (passes <= 10) return launch_rowdot_p<WT, 5, false>(p, 2, stream, pk);
    if (passes <= 12) return launch_rowdot_p<WT, 6, false>(p, 2, stream, pk);
    return launch_rowdot_p<WT, 8, false>(p, (passes + 7) / 8, stream, pk);
}

template <typename WT, int LPR, int WAVES, int UNROLL>
hipError_t launch_nseg(const GemvParams& p, const GemvShape& s, hipStream_t stream, int pk) {
    constexpr int SC = LPR * Elem<WT>::kPerLoad;
    const int strips = (p.n_out + SC - 1) / SC;
    dim3 grid(strips, s.ksplit), block(WAVES * 64);
    if (p.nseg == 2) {
        if constexpr (2 * SC <= WAVES * 64) {
            return launch_timed(gemv_kernel<WT, LPR, WAVES, UNROLL, 2>, grid, block, stream, pk, p);
        } else {
            return hipErrorInvalidConfiguration;
        }
    } else {
        if constexpr (SC <= WAVES * 64) {
            return launch_timed(gemv_kernel<WT, LPR, WAVES, UNROLL, 1>, grid, block, stream, pk, p);
        } else {
            return hipErrorInvalidConfiguration;
        }
    }
}

template <typename WT, int LPR, int WAVES>
hipError_t launch_unroll(const GemvParams& p, const GemvShape& s, hipStream_t stream, int pk) {
    switch (s.unroll) {
        case 1: return launch_nseg<WT, LPR, WAVES, 1>(p, s, stream, pk);
        case 2: return launch_nseg<WT, LPR, WAVES, 2>(p, s, stream, pk);
        case 4: return launch_nseg<WT, LPR, WAVES, 4>(p, s, stream, pk);
        case 8: return launch_nseg<WT, LPR, WAVES, 8>(p, s, stream, pk);
    }
    return hipErrorInvalidConfiguration;
}

template <typename WT, int LPR>
hipError_t launch_waves(const GemvParams& p, const GemvShape& s, hipStream_t stream, int pk) {
    switch (s.waves) {
        case 2: return launch_unroll<WT, LPR, 2>(p, s, stream, pk);
        case 4: return launch_unroll<WT, LPR, 4>(p, s, stream, pk);
        case 8: return launch_unroll<WT, LPR, 8>(p, s, stream, pk);
        case 16: return launch_unroll<WT, LPR, 16>(p, s, stream, pk);
    }
    return hipErrorInvalidConfiguration;
}

template <typename WT>
hipError_t launch_lpr(const GemvParams& p, const GemvShape& s, hipStream_t stream, int pk) {
    switch (s.lpr) {
        case 8: return launch_waves<WT, 8>(p, s, stream, pk);
        case 16: return launch_waves<WT, 16>(p, s, stream, pk);
        case 32: return launch_waves<WT, 32>(p, s, stream, pk);
        case 64: return launch_waves<WT, 64>(p, s, stream, pk);
    }
    return hipErrorInvalidConfiguration;
}

}  // namespace

static int elems_per_load(int dtype) { return dtype == DIP_F32 ? 4 : (dtype == DIP_BF16 ? 8 : 16); }

int gemv_strips(const GemvShape& s, int dtype, int n_out) {
    const int epl = elems_per_load(dtype);
    const int sc = s.lpr * epl;
    return (n_out + sc - 1) / sc;
}

GemvShape choose_gemv_shape(int dtype, int n_out, int nseg, int k) {
    // Defaults from launch-shape sweeps and same-box comparisons on MI355X (Phi-3-Mini,
    // Llama-3-8B and Phi-3-Medium shaped layers): 8 wavefronts, 4 rows in flight per lane
    // group, 16 lanes per row (32 for the bundled up/gate matrix when that gives whole
    // rounds), and row shares of a few hundred rows -- long enough to amortise a workgroup's
    // prologue and reduction, short enough to fill 256 compute units.
    GemvShape s;
    const bool q4 = dtype == DIP_INT4_G128;
    const int epl = elems_per_load(dtype);
    s.lpr = g_gemv_override.lpr ? g_gemv_override.lpr : 16;
    s.waves = g_gemv_override.waves ? g_gemv_override.waves : 8;
    s.unroll = g_gemv_override.unroll ? g_gemv_override.unroll : 4;
    int ks = 0;
    // Whole rounds of workgroups: with strips * ksplit just below one or two times the 256
    // compute units no unit is left with an extra workgroup while the others idle (280
    // workgroups take as long as 512).  Take the fewest rounds whose row shares fall into
    // the given range.
    auto whole_rounds = [&](int lpr, int min_share, int max_share) {
        const int strips = (n_out + lpr * epl - 1) / (lpr * epl);
        for (int m = 1; m <= 2; ++m) {
            const int cand = kComputeUnits * m / strips;
            if (cand < 1) continue;
            const int share = (k + cand - 1) / cand;
            if (share >= min_share && share <= max_share) return cand;
        }
        return 0;
    };
    if (!g_gemv_override.lpr && !g_gemv_override.ksplit) {
        if (q4) {
            // 4-bit rows are a quarter of the bytes while a workgroup's fixed costs (prologue,
            // 32 or 64 accumulators through the cross-lane reduction, the ticket protocol) are
            // the same: longer shares
            ks = whole_rounds(16, 256, 640);
        } else if (nseg == 2) {
            // bundled up/gate: the widest strip whose shares come out between 200 and 400 rows
            const int lprs[2] = {32, 16};
            for (int li = 0; li < 2 && !ks; ++li) {
                ks = whole_rounds(lprs[li], 200, 400);
                if (ks) s.lpr = lprs[li];
            }
        } else {
            // single matrix (down): whole rounds when the shares come out at 420-700 rows
            ks = whole_rounds(16, 420, 700);
        }
    }
    // a bundled strip needs 2*SC lanes for its epilogue
    while (nseg * s.lpr * epl > s.waves * 64 && s.waves < 16) s.waves *= 2;
    if (g_gemv_override.ksplit) {
        s.ksplit = g_gemv_override.ksplit;
    } else {
        if (!ks) {
            const int strips = gemv_strips(s, dtype, n_out);
            // (int4 rows are a quarter of the bytes and the reduction costs the same: longer shares)
            const int rows_per_wg = q4 ? (nseg == 2 ? 768 : 640) : (nseg == 2 ? 384 : 512);
            ks = (k + rows_per_wg / 2) / rows_per_wg;
            if (ks < 1) ks = 1;
            const int min_wgs = q4 ? 128 : 192;
            if (strips * ks < min_wgs) ks = (min_wgs + strips - 1) / strips;
        }
        // but keep at least one full iteration of rows per workgroup
        const int rows_per_iter = s.waves * (64 / s.lpr) * s.unroll;
        while (ks > 1 && k / ks < rows_per_iter) --ks;
        s.ksplit = ks;
    }
    if (s.ksplit > k) s.ksplit = k;
    if (s.ksplit < 1) s.ksplit = 1;
    return s;
}

hipError_t launch_gemv(const GemvParams& p0, const GemvShape& s, hipStream_t stream, int pk) {
    GemvParams p = p0;
    p.rows_per_split = ((p.k + s.ksplit - 1) / s.ksplit + 7) / 8 * 8;   // keeps vector index loads aligned
    if (p.dtype == DIP_F32) return launch_lpr<float>(p, s, stream, pk);
    if (p.dtype == DIP_BF16) return launch_lpr<uint16_t>(p, s, stream, pk);
    if (p.dtype == DIP_INT4_G128) return launch_lpr<q4n_t>(p, s, stream, pk);
    return hipErrorInvalidValue;
}

__global__ void gather_kernel(const float* x, const int32_t* idx, int k, int n, float* val, int32_t* idx_copy) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= k) return;
    const int r = idx[t];
    idx_copy[t] = r;
    val[t] = (unsigned)r < (unsigned)n ? x[r] : 0.f;
}

hipError_t launch_gather(const float* x, const int32_t* idx, int k, int n, float* val, int32_t* idx_copy,
                         hipStream_t stream) {
    hipLaunchKernelGGL(gather_kernel, dim3((k + 255) / 256), dim3(256), 0, stream, x, idx, k, n, val, idx_copy);
    return hipGetLastError();
}

hipError_t launch_rowdot(const RowdotParams& p, hipStream_t stream, int prof_kind) {
    if (p.k <= 0) return hipSuccess;
    if (p.dtype == DIP_F32) return launch_rowdot_t<float>(p, stream, prof_kind);
    if (p.dtype == DIP_BF16) return launch_rowdot_t<uint16_t>(p, stream, prof_kind);
    if (p.dtype == DIP_INT4_G128) return launch_rowdot_t<q4_t>(p, stream, prof_kind);
    return hipErrorInvalidValue;
}

}  // namespace dip
