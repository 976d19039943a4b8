/*
 * libdip -- Dynamic Input Pruning (DIP) and cache-aware masking (DIP-CA) for the
 * batch-1 SwiGLU MLP forward, native on AMD MI355X (gfx950).
 *
 * Paper notation used throughout (Sec. 3-5):
 *   x        input activations of a linear layer (fp32 here)
 *   W^u,W^g  up / gate matrices in R^{d_ff x d_model}; W^d down matrix in R^{d_model x d_ff}
 *   GLU(x)   = W^u x (.) SiLU(W^g x)                                   (Sec. 3, Eq. 2)
 *   m        binary column mask with exactly k ones, m = topK(s, k)    (Alg. 1)
 *   c        binary residency mask: which columns are in the cache     (Sec. 5.2)
 *   s        = |x| (c + gamma (1 - c)) / ||x||_inf                     (Sec. 5.2, Eq. 10)
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is a DEVICE pointer unless its comment says "host".
 *     Descriptor structs (dip_weight, dip_cache, dip_mlp, dip_debug) are host structs
 *     holding device pointers; the library reads them during the call only.
 *   - The library allocates nothing on the device: outputs, cache state and workspace
 *     belong to the caller, and it never frees caller memory.  The calls declared in this
 *     header keep no state between calls, with one exception that says so
 *     (dip_swiglu_mlp_forward_noalloc and its built-in scratch).  The process-wide
 *     switches for tuning and per-kernel timing live in dip_devtools.h.
 *   - All work is enqueued on the caller's stream (a hipStream_t passed as void*, NULL =
 *     the default stream).  No call synchronises with the host or reads device memory
 *     back.  Calls on one stream are ordered; calls that share a workspace or a cache on
 *     different streams race.  The scoring, selection, cache-update, product and forward
 *     calls enqueue kernel launches only (no allocation, no memset, no copy), so they may
 *     be captured into a HIP graph and replayed; dip_profile_enable must be off then.
 *   - Arguments are validated on the host before any HIP call.  On an error nothing is
 *     enqueued and no state changes.  Every function returns a dip_status; the message
 *     of the last failure on the calling thread is available from dip_last_error().
 *   - Bit masks: uint32_t[ceil(n/32)], feature i is bit (i & 31) of word (i >> 5); the
 *     padding bits of the last word are written as zero.  Index lists: int32_t, strictly
 *     ascending.
 *   - Weight layout is FEATURE-MAJOR: a matrix the paper writes as W in R^{n_out x n_in}
 *     is stored as n_in rows of n_out elements; stored row i is the paper's column
 *     W[:, i], everything that input feature i multiplies, so one selected column is one
 *     contiguous burst.  Row starts and row_stride_bytes must be multiples of 16.
 *   - Inputs must be finite.  Non-finite inputs never hang or fault; results are then
 *     unspecified.
 */
#ifndef DIP_H_
#define DIP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DIP_VERSION_MAJOR 0
#define DIP_VERSION_MINOR 1

typedef enum dip_status {
    DIP_OK = 0,
    DIP_ERR_INVALID_ARG = 1, /* null pointer, k outside [1, n], gamma outside [0, 1], ...   */
    DIP_ERR_UNSUPPORTED = 2, /* dtype / size / alignment the kernels do not handle          */
    DIP_ERR_WORKSPACE = 3,   /* workspace pointer null or smaller than *_workspace_bytes()  */
    DIP_ERR_HIP = 4          /* the HIP runtime reported an error at launch                 */
} dip_status;

typedef enum dip_dtype {
    DIP_F32 = 0,      /* fp32 weights                                                       */
    DIP_BF16 = 1,     /* bfloat16 weights, widened exactly to fp32 before the multiply      */
    DIP_INT4_G128 = 2 /* signed 4-bit codes, one fp16 scale per 128 consecutive elements of
                         a stored row (dip_weight.scales: n_out/128 per row, rows back to
                         back), w = scale * q; two codes per byte, low nibble = even
                         element; n_out must be a multiple of 128                           */
} dip_dtype;

typedef enum dip_policy {
    DIP_LRU = 0, /* evict the resident whose last use lies farthest back   (Sec. 5.1)       */
    DIP_LFU = 1  /* evict the resident with the smallest use counter       (Sec. 5.1)       */
} dip_policy;

/* Largest vector length the selection kernels handle (one workgroup keeps all keys in registers). */
#define DIP_MAX_N 32768

/* A feature-major weight matrix (see "Weight layout" above). */
typedef struct dip_weight {
    const void* data;         /* device; n_in rows                                          */
    const void* scales;       /* device; fp16 scales for DIP_INT4_G128, otherwise NULL      */
    int32_t dtype;            /* dip_dtype                                                   */
    int32_t n_in;             /* input features = stored rows                               */
    int32_t n_out;            /* outputs = elements per stored row                          */
    int32_t reserved;         /* must be 0                                                  */
    int64_t row_stride_bytes; /* distance between stored rows, >= n_out * element size      */
} dip_weight;

/* The three matrices of one SwiGLU MLP (Sec. 3, Eq. 1-2).  Up and gate are bundled per
 * input feature: stored row i of w_ug is [ W^u[:, i] ; W^g[:, i] ], 2*d_ff elements, so
 * w_ug.n_in = d_model, w_ug.n_out = 2*d_ff, and w_d.n_in = d_ff, w_d.n_out = d_model. */
typedef struct dip_mlp {
    dip_weight w_ug;
    dip_weight w_d;
} dip_mlp;

#define DIP_CACHE_META_WORDS 8
/* meta[] layout (device, uint32): */
#define DIP_META_STEP 0      /* 1-based step counter t; advanced by one per update          */
#define DIP_META_RESIDENT 1  /* number of resident columns after the last update            */
#define DIP_META_HITS 2      /* |m & c| of the last update                                  */
#define DIP_META_INSERTED 3  /* misses brought into the cache by the last update            */
#define DIP_META_EVICTED 4   /* residents evicted by the last update                        */
#define DIP_META_BYPASSED 5  /* misses that found no room and were not cached               */
#define DIP_META_CUM_HITS 6  /* running sum of hits   (wraps at 2^32)                       */
#define DIP_META_CUM_LOOKUPS 7 /* running sum of |m|  (wraps at 2^32)                       */

/* Residency state of one linear layer's columns (the paper's c, Sec. 5.2), owned by the caller. */
typedef struct dip_cache {
    uint32_t* bits;   /* device; ceil(n/32) words; bit set = column resident                */
    uint32_t* stamp;  /* device; n words; LRU: step of last use, LFU: use count             */
    uint32_t* meta;   /* device; DIP_CACHE_META_WORDS words                                 */
    int32_t n;        /* number of columns (input features of the layer)                   */
    int32_t capacity; /* at most this many columns resident, 0 <= capacity <= n             */
    int32_t policy;   /* dip_policy                                                         */
    int32_t reserved; /* must be 0                                                          */
} dip_cache;

/* Optional per-stage outputs of dip_swiglu_mlp_forward for stage-wise comparison; every
 * member may be NULL. */
typedef struct dip_debug {
    float* s_in;        /* d_model scores at pruning point 1                                */
    uint32_t* mask_in;  /* ceil(d_model/32) words                                           */
    int32_t* idx_in;    /* k_in ascending indices (16-byte aligned)                         */
    float* h;           /* d_ff: the sparse GLU output  GLU~(x)                             */
    float* s_mid;       /* d_ff scores at pruning point 2                                   */
    uint32_t* mask_mid; /* ceil(d_ff/32) words                                              */
    int32_t* idx_mid;   /* k_mid ascending indices (16-byte aligned)                        */
} dip_debug;

/* The sibling schemes of Sec. 3.2 that prune on a partial activation. */
typedef enum dip_scheme {
    DIP_GATE_PRUNING = 1, /* a = SiLU(W^g x) dense; topK(|a|) removes rows of W^u, columns of W^d */
    DIP_UP_PRUNING = 2    /* a = W^u x dense;       topK(|a|) removes rows of W^g, columns of W^d */
} dip_scheme;

/* The three matrices of one SwiGLU MLP stored for Gate / Up pruning.  The matrix that is
 * multiplied densely (W^g for gate pruning, W^u for up pruning) is feature-major like every
 * other matrix here.  The one whose ROWS the mask removes is NEURON-MAJOR: stored row j is
 * row j of the paper's matrix, the d_model weights of GLU unit j, so that a kept unit is one
 * contiguous burst; in its descriptor n_in = d_ff (stored rows) and n_out = d_model
 * (elements per stored row). */
typedef struct dip_mlp_split {
    dip_weight w_dense; /* feature-major, n_in = d_model, n_out = d_ff                      */
    dip_weight w_rows;  /* neuron-major,  n_in = d_ff,    n_out = d_model                   */
    dip_weight w_d;     /* feature-major, n_in = d_ff,    n_out = d_model                   */
} dip_mlp_split;

/* Optional stage outputs of dip_partial_pruning_forward; every member may be NULL. */
typedef struct dip_partial_debug {
    float* a;       /* d_ff: the partial activation the mask is taken from                  */
    uint32_t* mask; /* ceil(d_ff/32) words                                                  */
    int32_t* idx;   /* k ascending kept GLU units (16-byte aligned)                         */
    float* h_sel;   /* k values of GLU~(x) at those units (16-byte aligned)                 */
} dip_partial_debug;

/* A weight matrix kept in two tiers (Sec. 5: a small fast memory caching columns of a large
 * slow one).  `full` describes the whole feature-major matrix in PINNED HOST memory that the
 * GPU can read directly (full.data is that device-accessible host pointer); `slots` is the
 * fast tier: `capacity` rows of full.row_stride_bytes in HBM.  Column i is resident -- bit i
 * of the cache's residency mask -- exactly when slot_of[i] >= 0, and then slots row
 * slot_of[i] holds a copy of stored row i.  F32 and BF16 only. */
typedef struct dip_tiered_weight {
    dip_weight full;     /* data: host memory, device-accessible                            */
    void* slots;         /* device; capacity rows, 16-byte aligned                          */
    int32_t* slot_of;    /* device; full.n_in entries                                       */
    int32_t capacity;    /* slots; must equal the capacity of the cache used with it        */
    int32_t reserved;    /* must be 0                                                       */
} dip_tiered_weight;

typedef struct dip_tiered_mlp {
    dip_tiered_weight w_ug; /* bundled up/gate, as in dip_mlp                              */
    dip_tiered_weight w_d;
} dip_tiered_mlp;

/* (major << 16) | minor. */
int32_t dip_version(void);

/* Message of the last failing call on this thread (host string, never NULL, owned by the library). */
const char* dip_last_error(void);

/*
 * Cache-aware scores, Sec. 5.2 Eq. 10 / Alg. 1 step 1, in fp32 with this exact operation
 * order (round to nearest even, no fused operations, denormals kept):
 *     a = |x_i| ;  p = c_i ? a : fl(a * gamma) ;  s_i = fl(p / M),  M = max_i |x_i| ;
 *     M == 0  ->  s = 0.
 * cache_bits == NULL selects the plain DIP key of Sec. 4:  s_i = |x_i|  (gamma ignored).
 *   x          n floats          cache_bits  ceil(n/32) words or NULL
 *   s_out      n floats          1 <= n <= DIP_MAX_N,  0 <= gamma <= 1
 */
int32_t dip_ca_scores(const float* x, int32_t n, const uint32_t* cache_bits, float gamma,
                      float* s_out, void* stream);

/*
 * m = topK(s, k), Alg. 1 step 2 (per-token top-K thresholding, Sec. 3.1): exactly k
 * features with the largest keys; among equal keys the lowest index wins.  Keys must be
 * non-negative (scores are).
 *   s         n floats, 1 <= k <= n <= DIP_MAX_N
 *   mask_out  ceil(n/32) words, or NULL
 *   idx_out   k ascending indices, or NULL      (at least one of the two outputs is required)
 */
int32_t dip_prune_topk(const float* s, int32_t n, int32_t k, uint32_t* mask_out,
                       int32_t* idx_out, void* stream);

/*
 * Start a cache: step counter 1, all counters 0, stamps 0, residency = initial_bits
 * (ceil(n/32) words with at most `capacity` bits set -- not checked on the device; padding
 * bits must be zero) or empty when initial_bits is NULL.
 */
int32_t dip_cache_init(const dip_cache* cache, const uint32_t* initial_bits, void* stream);

/*
 * c' = cache_update(c, m), Alg. 1 step 3, for one token's mask m (ceil(n/32) words).
 * The mask is a set, so the update is set-valued and deterministic:
 *   hits   = m & c   keep their place; LRU stamps them with the current step
 *   misses = m & ~c  in ascending index order
 *   free   = capacity - |c| ;  victims V = c & ~m  (a column this token uses is never evicted)
 *   n_ins  = min(|misses|, free + |V|) ;  evict the max(0, n_ins - free) members of V with
 *            the smallest (stamp, index) ;  insert the first n_ins misses ;  the remaining
 *            misses bypass the cache (Sec. 6.4: when the active set does not fit, part of
 *            it is used without being cached).
 *   LFU: stamp counts every selection of a column, resident or not, and survives eviction.
 * Advances meta[DIP_META_STEP] and refreshes the other meta counters.
 */
int32_t dip_cache_update(const dip_cache* cache, const uint32_t* mask_bits, void* stream);

/*
 * Checkpoint helpers for a cache (the state survives between tokens, Alg. 1 returns c^(t)).
 * dip_cache_state_bytes: sizes of the three caller-owned arrays for n columns (host outputs,
 * each may be NULL).  dip_cache_export / dip_cache_import copy the whole state to / from one
 * contiguous blob of dip_cache_blob_bytes(n) bytes laid out [bits | stamp | meta], each part
 * starting on a 256-byte boundary; the blob may be device memory or host memory (pinned
 * host memory keeps the copy asynchronous).  Copies are enqueued on the stream.
 */
int32_t dip_cache_state_bytes(int32_t n, size_t* bits_bytes /* host */, size_t* stamp_bytes /* host */,
                              size_t* meta_bytes /* host */);
size_t dip_cache_blob_bytes(int32_t n);
int32_t dip_cache_export(const dip_cache* cache, void* blob, size_t blob_bytes, void* stream);
int32_t dip_cache_import(const dip_cache* cache, const void* blob, size_t blob_bytes, void* stream);

/*
 * Column-gathered matrix-vector product, Alg. 1 step 4 (W~ = W (.) m) applied to x:
 *     y[j] = sum_{t<k} W[j, idx[t]] * x[idx[t]]        fp32 accumulation.
 * The summation order is fixed by the launch configuration, so results are bit-repeatable.
 *   w        feature-major matrix (F32, BF16 or INT4_G128); a row is whole 16-byte loads
 *   x        w->n_in floats        idx   k ascending indices in [0, n_in), 1 <= k <= n_in
 *   y_out    w->n_out floats       ws    dip_gathered_gemv_workspace_bytes() bytes, 256-aligned
 */
size_t dip_gathered_gemv_workspace_bytes(const dip_weight* w, int32_t k);
int32_t dip_gathered_gemv(const dip_weight* w, const float* x, const int32_t* idx, int32_t k,
                          float* y_out, void* ws, size_t ws_bytes, void* stream);

/*
 * One token through one DIP / DIP-CA SwiGLU MLP (Sec. 4 composed with Alg. 1 at both
 * pruning points):
 *   1. s1 = score(x, c_in)          m1 = topK(s1, k_in)       c_in  <- cache_update(c_in,  m1)
 *   2. h~ = (sum_{i in m1} W^u[:,i] x_i) (.) SiLU(sum_{i in m1} W^g[:,i] x_i)
 *   3. s2 = score(h~, c_mid)        m2 = topK(s2, k_mid)      c_mid <- cache_update(c_mid, m2)
 *   4. y  = sum_{i in m2} W^d[:,i] h~_i
 * Scoring uses the cache state from before this token (the paper's c^(t-1)).  With a NULL
 * cache the key is |.| (DIP); a cache pointer switches that point to Eq. 10 (DIP-CA) and its
 * state is updated in place.
 *   x      d_model floats       y_out   d_model floats
 *   1 <= k_in <= d_model, 1 <= k_mid <= d_ff;  d_model, d_ff <= DIP_MAX_N
 *   dbg    NULL or stage outputs           ws   *_workspace_bytes() bytes, 256-aligned
 */
size_t dip_swiglu_mlp_forward_workspace_bytes(const dip_mlp* mlp, int32_t k_in, int32_t k_mid);
int32_t dip_swiglu_mlp_forward(const dip_mlp* mlp, const float* x, int32_t k_in, int32_t k_mid,
                               const dip_cache* cache_in, const dip_cache* cache_mid,
                               float gamma, float* y_out, const dip_debug* dbg, void* ws,
                               size_t ws_bytes, void* stream);

/*
 * dip_swiglu_mlp_forward for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and ordering rules as dip_swiglu_mlp_forward, minus
 * the workspace: the scratch (index lists, h~, split-K partial sums, ticket counters) lives
 * in a device array built into the library, DIP_STATIC_SCRATCH_BYTES per GPU, held from
 * library load until the process ends.  The call allocates and frees nothing.  A layer
 * whose dip_swiglu_mlp_forward_workspace_bytes() exceeds DIP_STATIC_SCRATCH_BYTES is
 * rejected with DIP_ERR_WORKSPACE and nothing is enqueued.  All calls on one GPU share that
 * GPU's array (it keeps the previous call's contents; what must start at zero is cleared by
 * the call's own kernels): calls that overlap on one GPU -- different streams, or replays
 * of graphs that contain it running concurrently -- race.
 */
#define DIP_STATIC_SCRATCH_BYTES (4u << 20)
int32_t dip_swiglu_mlp_forward_noalloc(const dip_mlp* mlp, const float* x, int32_t k_in, int32_t k_mid,
                                       const dip_cache* cache_in, const dip_cache* cache_mid,
                                       float gamma, float* y_out, const dip_debug* dbg, void* stream);

/*
 * The same forward for n_layers independent layers in one call (a decode step over a
 * stack): layer l reads x + l * x_stride and writes y_out + l * y_stride (strides in
 * floats) and keeps k_in[l] of its inputs and k_mid[l] of its GLU units (host arrays of
 * n_layers entries: Sec. 4 allows different sparsity levels per matrix and layer).
 * mlps / caches_in / caches_mid are host arrays of n_layers descriptors; the cache arrays
 * may be NULL (DIP).  Every layer and pruning point needs a dip_cache of its own (the call
 * rejects shared state): all caches are scored in their layers' launches and updated
 * together in one launch at the end of the call.
 * ws: dip_swiglu_mlp_forward_stack_workspace_bytes() bytes, 256-aligned.
 */
size_t dip_swiglu_mlp_forward_stack_workspace_bytes(const dip_mlp* mlps, int32_t n_layers,
                                                    const int32_t* k_in /* host */,
                                                    const int32_t* k_mid /* host */);
int32_t dip_swiglu_mlp_forward_stack(const dip_mlp* mlps, int32_t n_layers, const float* x,
                                     int64_t x_stride, const int32_t* k_in /* host */,
                                     const int32_t* k_mid /* host */, const dip_cache* caches_in,
                                     const dip_cache* caches_mid, float gamma, float* y_out,
                                     int64_t y_stride, void* ws, size_t ws_bytes, void* stream);

/*
 * A small decode batch through one layer: `batch` (1..8) rows X[b] (row stride d_model)
 * give `batch` independent batch-1 results Y[b] of dip_swiglu_mlp_forward -- every row has
 * its own two top-K masks -- while each stored column is read once if any row selected it
 * (the union of the row masks) and is accumulated only into the rows that selected it.
 * All rows are scored against the cache state from before the step; each cache is then
 * updated once with the union mask (Alg. 1 step 3).  The paper itself is batch 1 (Sec. 1).
 * Optional outputs for stage-wise comparison (each may be NULL):
 *   mask_in_out   [batch][ceil(d_model/32)] words     h_out  [batch][d_ff] floats
 *   mask_mid_out  [batch][ceil(d_ff/32)] words
 * Summation order is fixed by the launch configuration (bit-repeatable).
 * DIP_INT4_G128 weights with batch >= 3 are multiplied on the matrix cores (matrices of up to
 * 4 GiB; larger ones take the vector path): every row's activations are first scaled by a
 * power of two into [8, 16) -- exact, and undone exactly on the partial sums, so the result
 * does not depend on the magnitude of the activations -- and activation times group scale
 * enters as two fp16 terms (about 21 significant bits of the row's largest product); this
 * needs group scales of at most 4094 (|w| up to 28658; beyond that the sums overflow to
 * inf).  The sums are fp32 as everywhere else.
 */
size_t dip_swiglu_mlp_forward_batched_workspace_bytes(const dip_mlp* mlp, int32_t batch,
                                                      int32_t k_in, int32_t k_mid);
int32_t dip_swiglu_mlp_forward_batched(const dip_mlp* mlp, const float* X, int32_t batch,
                                       int32_t k_in, int32_t k_mid, const dip_cache* cache_in,
                                       const dip_cache* cache_mid, float gamma, float* Y,
                                       uint32_t* mask_in_out, float* h_out, uint32_t* mask_mid_out,
                                       void* ws, size_t ws_bytes, void* stream);

/*
 * The batched forward for n_layers independent layers in one call: layer l reads its `batch`
 * rows at X + l * x_stride ([batch][d_model], contiguous) and writes Y + l * y_stride (strides
 * in floats), with k_in[l] / k_mid[l] kept per row (host arrays).  Cache rules as in
 * dip_swiglu_mlp_forward_stack: one dip_cache per layer and point, all updated -- once each,
 * with the union of the layer's row masks -- in one launch at the end of the call.
 */
size_t dip_swiglu_mlp_forward_batched_stack_workspace_bytes(const dip_mlp* mlps, int32_t n_layers, int32_t batch,
                                                            const int32_t* k_in /* host */,
                                                            const int32_t* k_mid /* host */);
int32_t dip_swiglu_mlp_forward_batched_stack(const dip_mlp* mlps, int32_t n_layers, const float* X,
                                             int64_t x_stride, int32_t batch, const int32_t* k_in /* host */,
                                             const int32_t* k_mid /* host */, const dip_cache* caches_in,
                                             const dip_cache* caches_mid, float gamma, float* Y,
                                             int64_t y_stride, void* ws, size_t ws_bytes, void* stream);

/*
 * GLU pruning, Sec. 3.2: W^u x and W^g x are dense, m = topK(|GLU(x)|, k) removes columns
 * of W^d:  y = sum_{i in m} W^d[:, i] GLU(x)_i.  Same matrices, layout and workspace rules
 * as dip_swiglu_mlp_forward; x must be 16-byte aligned; the point-1 members of dbg must be NULL.
 */
size_t dip_glu_pruning_forward_workspace_bytes(const dip_mlp* mlp, int32_t k);
int32_t dip_glu_pruning_forward(const dip_mlp* mlp, const float* x, int32_t k, float* y_out,
                                const dip_debug* dbg, void* ws, size_t ws_bytes, void* stream);

/*
 * Row-gathered dot products: out[t] = W[idx[t], :] . x  for t < k, fp32 accumulation in a
 * fixed order -- what is left of W x when a mask removes rows of W (Sec. 3.2, the W^u of
 * gate pruning).
 *   w_rows   neuron-major matrix: n_in stored rows of n_out elements (n_out <= DIP_MAX_N)
 *   x        n_out floats, 16-byte aligned     idx   k ascending stored-row indices
 *   out      k floats
 */
int32_t dip_gathered_rowdot(const dip_weight* w_rows, const float* x, const int32_t* idx, int32_t k,
                            float* out, void* stream);

/*
 * Gate pruning and Up pruning, Sec. 3.2, one token through one MLP:
 *   1. a = SiLU(W^g x)  (gate)   or   a = W^u x  (up)        dense, all d_ff units, fp32
 *   2. m = topK(|a|, k)                                       lowest index wins ties
 *   3. h_j = (W^u x)_j a_j  (gate)   or   a_j SiLU((W^g x)_j)  (up)      for j in m only
 *   4. y = sum_{j in m} W^d[:, j] h_j
 * The fp32 array a is both the selection key and the factor in step 3.
 *   x     d_model floats, 16-byte aligned      y_out   d_model floats     1 <= k <= d_ff
 *   dbg   NULL or stage outputs                ws      *_workspace_bytes() bytes, 256-aligned
 */
size_t dip_partial_pruning_forward_workspace_bytes(const dip_mlp_split* mlp, int32_t k);
int32_t dip_partial_pruning_forward(const dip_mlp_split* mlp, int32_t scheme, const float* x,
                                    int32_t k, float* y_out, const dip_partial_debug* dbg,
                                    void* ws, size_t ws_bytes, void* stream);

/*
 * Two-tier residency made real (Sec. 5, Fig. 4; Alg. 1's c decides what the fast tier holds).
 * dip_tier_init: after dip_cache_init, give every resident column a slot (the r-th resident
 * column, ascending, gets slot r), copy those rows host -> HBM, mark the others slot_of = -1.
 * dip_tiered_mlp_forward: dip_swiglu_mlp_forward with both caches mandatory, where after each
 * cache update the inserted columns take over the slots of the evicted ones (i-th inserted,
 * ascending, <- slot of the i-th evicted; the rest get slots never used before), their rows
 * are copied host -> HBM, and the gathered product reads resident columns from their slots
 * and the misses that found no room (Sec. 6.4) straight from host memory.  y is bit-identical
 * to dip_swiglu_mlp_forward on the same inputs and cache states.
 */
size_t dip_tier_init_workspace_bytes(const dip_tiered_weight* tw);
int32_t dip_tier_init(const dip_tiered_weight* tw, const dip_cache* cache, void* ws, size_t ws_bytes,
                      void* stream);
size_t dip_tiered_mlp_forward_workspace_bytes(const dip_tiered_mlp* mlp, int32_t k_in, int32_t k_mid);
int32_t dip_tiered_mlp_forward(const dip_tiered_mlp* mlp, const float* x, int32_t k_in, int32_t k_mid,
                               const dip_cache* cache_in, const dip_cache* cache_mid, float gamma,
                               float* y_out, const dip_debug* dbg, void* ws, size_t ws_bytes,
                               void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DIP_H_ */
