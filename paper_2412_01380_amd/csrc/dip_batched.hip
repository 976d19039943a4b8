// Small decode batches (B = 1..8 rows per step) through one DIP / DIP-CA layer.
//
// The paper is strictly batch 1 (every product is a matrix-vector product, Sec. 1); a batch
// here is B independent batch-1 results that share the weight reads: each row keeps its own
// top-K masks (Alg. 1 step 2 per row), a stored column is read once if any row selected it
// (the union of the row masks) and is accumulated only into the rows that did select it
// (their multiplier is the row's activation, the others' is zero), and the cache sees one
// update per step with the union mask (Alg. 1 step 3).
//
// Kernels in this file:
//   union_kernel     union of the B row masks -> ascending index list, its length, and the
//                    B multipliers of every listed column (lists padded by 16 entries)
//   bgemv_kernel     column-gathered product for all B rows at once, partial sums per
//                    row share; the number of listed columns is read from device memory
//   bgemv_q4_mfma_kernel  the same product for int4 weights and three or more rows, as a
//                    dense contraction on the matrix cores
//   breduce_kernel   adds the partial sums in share order and applies the epilogue
//                    (SwiGLU for the bundled up/gate matrix, Sec. 3 Eq. 2)

#include "dip_internal.h"
#include "dip_select_device.h"

namespace dip {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// union of the row masks
// ---------------------------------------------------------------------------------------
constexpr int kUnionThreads = 512;
constexpr int kUnionWordsPerWg = kUnionThreads / 32;   // one lane per feature of 16 mask words

// Every workgroup scans the popcounts of all union words (two words per thread, at most 1024
// words), which gives each word the number of listed indices before it; it then lists the
// features of its own 16 words, one lane per feature, so the reads of x are coalesced.
// Everything a lane will need -- the words it counts, the word of its own feature in every
// row and the feature's activations -- is requested before anything is waited for: the kernel
// is one memory round trip, a scan and the stores.
__global__ __launch_bounds__(kUnionThreads) void union_kernel(UnionParams p) {
    __shared__ uint32_t s_base[2 * kUnionThreads];
    __shared__ uint32_t s_wave[kUnionThreads / 64];
    constexpr int kMaxBatch = 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int B = p.batch;
    const int nwords = (p.n + 31) >> 5;
    const int w0 = 2 * tid, w1 = 2 * tid + 1;
    const int w = blockIdx.x * kUnionWordsPerWg + (tid >> 5), bit = tid & 31;
    // (reads past the end are redirected to the last word / feature and dropped)
    const int w0c = min(w0, nwords - 1), w1c = min(w1, nwords - 1), wc = min(w, nwords - 1);
    const int i = w * 32 + bit, ic = min(i, p.n - 1);
    uint32_t a0[kMaxBatch], a1[kMaxBatch], mw[kMaxBatch];
    float xv[kMaxBatch];
#pragma unroll
    for (int b = 0; b < kMaxBatch; ++b) {
        a0[b] = 0u; a1[b] = 0u; mw[b] = 0u; xv[b] = 0.f;
        if (b < B) {    // (uniform)
            const uint32_t* mrow = p.masks + (size_t)b * p.words_stride;
            a0[b] = mrow[w0c];
            a1[b] = mrow[w1c];
            mw[b] = mrow[wc];
            xv[b] = p.x[(size_t)b * p.x_stride + ic];
        }
    }
    uint32_t u0 = 0u, u1 = 0u;
#pragma unroll
    for (int b = 0; b < kMaxBatch; ++b) {
        u0 |= a0[b];
        u1 |= a1[b];
    }
    if (w0 >= nwords) u0 = 0u;
    if (w1 >= nwords) u1 = 0u;
    const uint32_t c0 = (uint32_t)__popc(u0), c1 = (uint32_t)__popc(u1);
    const uint32_t inc = sel::wave_incl_scan(c0 + c1);
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int ww = 0; ww < kUnionThreads / 64; ++ww) {
        const uint32_t t = s_wave[ww];
        if (ww < wave) before += t;
        total += t;
    }
    const uint32_t excl = before + inc - (c0 + c1);
    s_base[w0] = excl;
    s_base[w1] = excl + c0;
    if (blockIdx.x == 0) {
        if (w0 < nwords) p.union_words[w0] = u0;
        if (w1 < nwords) p.union_words[w1] = u1;
        if (tid == 0) p.count_out[0] = total;
    }
    __syncthreads();

    if (w >= nwords) return;
    uint32_t rows = 0, uw = 0;    // bit b of rows: row b selected this feature
#pragma unroll
    for (int b = 0; b < kMaxBatch; ++b) {
        uw |= mw[b];
        rows |= ((mw[b] >> bit) & 1u) << b;
    }
    if (!rows) return;
    const uint32_t pos = s_base[w] + (uint32_t)__popc(uw & ((1u << bit) - 1u));
    p.uidx[pos] = i;
    float m[kMaxBatch];
#pragma unroll
    for (int b = 0; b < kMaxBatch; ++b) m[b] = ((rows >> b) & 1u) ? xv[b] : 0.f;
    float* dst = p.uval + (size_t)pos * B;
    if (B == 8) {
        reinterpret_cast<float4*>(dst)[0] = make_float4(m[0], m[1], m[2], m[3]);
        reinterpret_cast<float4*>(dst)[1] = make_float4(m[4], m[5], m[6], m[7]);
    } else if (B == 4) {
        reinterpret_cast<float4*>(dst)[0] = make_float4(m[0], m[1], m[2], m[3]);
    } else {
#pragma unroll
        for (int b = 0; b < kMaxBatch; ++b)
            if (b < B) dst[b] = m[b];
    }
}

// ---------------------------------------------------------------------------------------
// batched gathered product
// ---------------------------------------------------------------------------------------
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int DT>
struct BElem;
template <>
struct BElem<DIP_F32> {   // 16-byte load, 4 values
    static constexpr int kElems = 4, kBits = 32, kLanes = 16;
    static constexpr bool kScaled = false;
    typedef u32x4 raw_t;
    __device__ static __forceinline__ raw_t load(const char* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    }
    __device__ static __forceinline__ void widen(const raw_t& q, float (&f)[4]) {
        f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y);
        f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
    }
};
template <>
struct BElem<DIP_BF16> {  // 16-byte load, 8 values
    static constexpr int kElems = 8, kBits = 16, kLanes = 16;
    static constexpr bool kScaled = false;
    typedef u32x4 raw_t;
    __device__ static __forceinline__ raw_t load(const char* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    }
    __device__ static __forceinline__ void widen(const raw_t& q, float (&f)[8]) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <>
struct BElem<DIP_INT4_G128> {
    // 8-byte load, 16 codes: a batch multiplies every code B times, so fewer codes per lane
    // keep the B x 16 accumulators in registers.  Flipping bit 3 of every nibble turns the
    // two's-complement code q into q + 8 in [0, 15]; even and odd nibbles, masked apart, are
    // bytes that convert to float in one instruction each.  The caller removes the offset:
    // sum (q + 8) m - 8 sum m.
    static constexpr int kElems = 16, kBits = 4, kLanes = 32;
    static constexpr bool kScaled = true;
    typedef u32x2 raw_t;
    __device__ static __forceinline__ raw_t load(const char* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    }
    __device__ static __forceinline__ void widen(const raw_t& q, float (&f)[16]) {
        const uint32_t w[2] = {q.x, q.y};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t o = w[i] ^ 0x88888888u;
            uint32_t ev = o & 0x0f0f0f0fu, od = (o >> 4) & 0x0f0f0f0fu;
            // keeps the byte extracts below from being narrowed into bit-field extracts
            asm volatile("" : "+v"(ev), "+v"(od));
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f[i * 8 + 2 * b] = (float)((ev >> (8 * b)) & 0xffu);
                f[i * 8 + 2 * b + 1] = (float)((od >> (8 * b)) & 0xffu);
            }
        }
    }
};

struct BElemQ4Narrow {
    // 4-byte load, 8 codes, all 64 lanes on one stored row: for the larger batches, whose
    // B x 16 accumulators would not leave registers for anything else
    static constexpr int kElems = 8, kBits = 4, kLanes = 64;
    static constexpr bool kScaled = true;
    typedef uint32_t raw_t;
    __device__ static __forceinline__ raw_t load(const char* p) {
        return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
    }
    __device__ static __forceinline__ void widen(const raw_t& q, float (&f)[8]) {
        const uint32_t o = q ^ 0x88888888u;
        uint32_t ev = o & 0x0f0f0f0fu, od = (o >> 4) & 0x0f0f0f0fu;
        asm volatile("" : "+v"(ev), "+v"(od));
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            f[2 * b] = (float)((ev >> (8 * b)) & 0xffu);
            f[2 * b + 1] = (float)((od >> (8 * b)) & 0xffu);
        }
    }
};

template <int DT, int B>
struct BPick { using type = BElem<DT>; };
template <> struct BPick<DIP_INT4_G128, 5> { using type = BElemQ4Narrow; };
template <> struct BPick<DIP_INT4_G128, 6> { using type = BElemQ4Narrow; };
template <> struct BPick<DIP_INT4_G128, 7> { using type = BElemQ4Narrow; };
template <> struct BPick<DIP_INT4_G128, 8> { using type = BElemQ4Narrow; };

// B consecutive multipliers of one listed column
template <int B>
__device__ __forceinline__ void load_mult(const float* p, float (&m)[B]) {
    if constexpr (B % 4 == 0) {
#pragma unroll
        for (int b = 0; b < B; b += 4) {
            const float4 v = *reinterpret_cast<const float4*>(p + b);
            m[b] = v.x; m[b + 1] = v.y; m[b + 2] = v.z; m[b + 3] = v.w;
        }
    } else if constexpr (B % 2 == 0) {
#pragma unroll
        for (int b = 0; b < B; b += 2) {
            const float2 v = *reinterpret_cast<const float2*>(p + b);
            m[b] = v.x; m[b + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int b = 0; b < B; ++b) m[b] = p[b];
    }
}

constexpr int kBWaves = 4;
constexpr int kBUnroll = 4;   // listed columns in flight per lane group

template <int DT, int B>
__global__ __launch_bounds__(kBWaves * 64) void bgemv_kernel(BatchedGemvParams p) {
    using E = typename BPick<DT, B>::type;
    constexpr int EPL = E::kElems;
    constexpr int LPR = E::kLanes;
    constexpr int RPW = 64 / LPR;
    constexpr int SC = LPR * EPL;
    constexpr int NG = kBWaves * RPW;
    constexpr int U = kBUnroll;
    __shared__ float red[B][SC];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, l = lane % LPR;
    const int strip = blockIdx.x, g = blockIdx.y, G = gridDim.y;
    const int col_raw = strip * SC + l * EPL;
    // lanes past the right edge of a ragged last strip re-read its last piece; they own no output
    const int col = col_raw < p.n_out ? col_raw : p.n_out - EPL;

    const int k = min((int)p.k_dev[0], p.k_max);
    const int share = ((k + G - 1) / G + U - 1) / U * U;
    const int kb = min(k, g * share), ke = min(k, kb + share);

    float acc[B][EPL];
    float msum[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        msum[b] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[b][e] = 0.f;
    }

    const char* wbase = static_cast<const char*>(p.w) + (size_t)col * E::kBits / 8;
    const int sgroup = col >> 7;
    // a lane group takes U consecutive listed columns per step; the lists are padded so that
    // whole vectors can be read past position k, and what lies past the share is dropped
    for (int t0 = kb + (wave * RPW + sub) * U; t0 < ke; t0 += NG * U) {
        const int4 r4 = *reinterpret_cast<const int4*>(p.uidx + t0);
        const int r[U] = {r4.x, r4.y, r4.z, r4.w};
        typename E::raw_t q[U];
        float scale[U];
        bool live[U];
        float m[U][B];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            live[u] = t0 + u < ke && (unsigned)r[u] < (unsigned)p.n_in;
            const int rr = live[u] ? r[u] : 0;
            q[u] = E::load(wbase + (size_t)rr * (size_t)p.row_stride);
            scale[u] = 1.f;
            if constexpr (E::kScaled) {
                _Float16 hs;
                const uint16_t raw = p.scales[(size_t)rr * p.scale_stride + sgroup];
                __builtin_memcpy(&hs, &raw, 2);
                scale[u] = (float)hs;
            }
            load_mult<B>(p.uval + (size_t)(t0 + u) * B, m[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float f[EPL];
            E::widen(q[u], f);
#pragma unroll
            for (int b = 0; b < B; ++b) {
                // entries past the share hold whatever the list memory held: select, never multiply
                const float mb = live[u] ? m[u][b] * scale[u] : 0.f;
                if constexpr (E::kScaled) msum[b] += mb;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[b][e] = fmaf(f[e], mb, acc[b][e]);
            }
        }
    }
    if constexpr (E::kScaled) {
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[b][e] = fmaf(-8.0f, msum[b], acc[b][e]);
    }
    // lane groups of one wavefront, then wavefronts through LDS, both in a fixed order
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[b][e] += __shfl_xor(acc[b][e], off);
    // (one wavefront after the other adds its sums into the same LDS strip)
    for (int w = 0; w < kBWaves; ++w) {
        if (wave == w && sub == 0) {
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    float* dst = &red[b][l * EPL + e];
                    *dst = w == 0 ? acc[b][e] : *dst + acc[b][e];
                }
        }
        __syncthreads();
    }
    for (int o = tid; o < B * SC; o += kBWaves * 64) {
        const int b = o / SC, c = o % SC;
        const int gcol = strip * SC + c;
        if (gcol >= p.n_out) continue;
        p.partial[((size_t)g * B + b) * (size_t)p.n_out + gcol] = red[b][c];
    }
}

// ---------------------------------------------------------------------------------------
// int4-g128 weights, more than kMfmaMinBatch rows: the product on the matrix cores.
//
// With B rows the union columns times the row multipliers is a dense contraction
//     P[b][j] = sum_u  m[b][u] * scale[u][j / 128] * q[u][j],
// B x K_union x n_out, and on the vector ALU every 4-bit code costs B multiply-adds plus its
// unpacking.  v_mfma_f32_16x16x16_f16 takes it instead: M = batch row (16, the rows past B are
// zero), K = 16 listed columns, N = 16 stored columns.  The scale belongs to (u, 128-column
// group), so it goes into the left operand next to the multiplier: m * scale enters as the
// sum of two fp16 numbers (its rounded value and the rounded rest; each tile is multiplied
// twice).  fp16 has a fixed range, and the re-weighting of Sec. 5.2 normalises by ||x||_inf
// precisely so that the dynamic range of the activations does not matter: every batch row is
// therefore multiplied by the power of two that brings its largest |activation| into [8, 16)
// before the split -- exact in fp32 -- and the partial sums are multiplied by the inverse
// power when they are stored, also exact.  The product then depends on the weights only:
// with |m| < 16 it stays inside the fp16 range for group scales up to 4094, and the second
// term (an fp16 denormal as a rule, absolute step 6e-8) carries m * scale to about 2^-21 of
// the row's largest product whatever the magnitude of the activations.  The right operand
// holds the codes q + 8 in [0, 15], exact in fp16.  Sums are fp32; the offset leaves as
// -8 * sum_u m*scale, which a product with an all-ones right operand supplies.
//
// Lane l of a wavefront: k-block r = l / 16 (listed columns 4r .. 4r+3 of the 16), c = l % 16.
// Right operand: the lane loads one dword = 8 codes of each of its 4 stored rows at byte 4c of
// the group's 64-byte piece; product number t (0..7) takes code t of the four dwords, so it
// yields the stored columns 8c + t.  Left operand: the lane is batch row c; it multiplies that
// row's multiplier of its 4 listed columns by the scale of (column, group).
// A workgroup covers two groups (256 stored columns, one 128-byte piece per row) and a share
// of the listed columns; its wavefronts take sets of 16 listed columns in turn.
// ---------------------------------------------------------------------------------------
typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
typedef float f4_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaMinBatch = 3;
constexpr int kMWaves = 4;
constexpr int kMGroups = 2;
constexpr int kMStripCols = 128 * kMGroups;
constexpr int kMRowSet = 16;

__device__ __forceinline__ h4_t pack_h4(float a, float b, float c, float d) {
    // round-toward-zero packing is exact here: the values are integers in [0, 15]
    struct { decltype(__builtin_amdgcn_cvt_pkrtz(0.f, 0.f)) lo, hi; } v = {__builtin_amdgcn_cvt_pkrtz(a, b),
                                                                         __builtin_amdgcn_cvt_pkrtz(c, d)};
    return __builtin_bit_cast(h4_t, v);
}

// The power of two that brings a row's largest |activation| (given as its bit pattern) into
// [8, 16); 1 for an all-zero row.  Denormal and near-overflow maxima are clamped to factors
// fp32 can hold; such rows only lose the part of the range fp16 could not carry anyway.
__device__ __forceinline__ float row_scale_up(uint32_t max_bits) {
    const int e = (int)((max_bits >> 23) & 0xffu);       // biased exponent of the maximum
    if (max_bits == 0u) return 1.0f;
    int up = 127 + 3 - (e - 127);                        // biased exponent of 2^(3 - unbiased e)
    up = up < 1 ? 1 : (up > 254 ? 254 : up);
    return __uint_as_float((uint32_t)up << 23);
}

__global__ __launch_bounds__(kMWaves * 64) void bgemv_q4_mfma_kernel(BatchedGemvParams p) {
    __shared__ float red[kMGroups][8][8][16];    // [group][code position][batch row][lane column]
    __shared__ float red1[kMGroups][8];          // sum of m*scale per (group, batch row)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 4, c = lane & 15;
    const int strip = blockIdx.x, g = blockIdx.y, G = gridDim.y;
    const int B = p.batch;
    const int ngroups = p.n_out >> 7;

    const int k = min((int)p.k_dev[0], p.k_max);
    const int share = ((k + G - 1) / G + kMRowSet - 1) / kMRowSet * kMRowSet;
    const int kb = min(k, g * share), ke = min(k, kb + share);

    f4_t acc[kMGroups][8], acc1[kMGroups];
#pragma unroll
    for (int gg = 0; gg < kMGroups; ++gg) {
        acc1[gg] = f4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[gg][t] = f4_t{0.f, 0.f, 0.f, 0.f};
    }
    // a ragged last strip has one group only: the second is re-read from the first and dropped
    int grp[kMGroups];
#pragma unroll
    for (int gg = 0; gg < kMGroups; ++gg) grp[gg] = min(strip * kMGroups + gg, ngroups - 1);
    const h4_t ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f};
    const bool row_live = c < B;

    // One set of 16 listed columns per step; the index vector of the next set is requested
    // before the current one is multiplied.  Nothing branches on a lane: positions past the
    // share read stored row 0 and are masked out of the left operand.  Offsets are 32-bit
    // (a stored matrix is far below 4 GB) on top of scalar base pointers.
    constexpr int STEP = kMWaves * kMRowSet;
    // (the lists carry 16 spare entries past k_max, so whole index vectors may be read there)
    auto load_idx = [&](int t) {
        return *reinterpret_cast<const int4*>(p.uidx + min(t, p.k_max) + 4 * r);
    };
    const char* wbytes = static_cast<const char*>(p.w);
    const uint32_t row_stride = (uint32_t)p.row_stride;
    const uint32_t wcol[kMGroups] = {(uint32_t)(grp[0] * 64 + 4 * c), (uint32_t)(grp[1] * 64 + 4 * c)};
    const uint32_t cb = (uint32_t)min(c, B - 1);
    const float row_up = row_scale_up(p.rowmax[cb]);     // this lane's batch row, into [8, 16)
    int4 rn = load_idx(kb + wave * kMRowSet);
    for (int t0 = kb + wave * kMRowSet; t0 < ke; t0 += STEP) {
        const int rows[4] = {rn.x, rn.y, rn.z, rn.w};
        rn = load_idx(t0 + STEP);
        uint32_t wq[kMGroups][4];
        uint16_t sc[kMGroups][4];
        float mv[4];
        uint32_t keep[2] = {0u, 0u};    // bit masks over the two fp16 pairs of the left operand
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = t0 + 4 * r + i;
            const bool live = u < ke && (unsigned)rows[i] < (unsigned)p.n_in;
            const uint32_t rr = live ? (uint32_t)rows[i] : 0u;
            // entries past the share hold whatever the list memory held: they are masked out
            // of the left operand bit-wise (never multiplied away), and the mask is plain
            // arithmetic so that the load stays unconditional
            mv[i] = p.uval[(uint32_t)min(u, p.k_max - 1) * (uint32_t)B + cb] * row_up;
            if (live && row_live) keep[i >> 1] |= (i & 1) ? 0xffff0000u : 0x0000ffffu;
            const uint32_t wrow = rr * row_stride;
            const uint32_t srow = rr * (uint32_t)p.scale_stride;
#pragma unroll
            for (int gg = 0; gg < kMGroups; ++gg) {
                wq[gg][i] = *reinterpret_cast<const uint32_t*>(wbytes + (wrow + wcol[gg]));
                sc[gg][i] = p.scales[srow + (uint32_t)grp[gg]];
            }
        }
#pragma unroll
        for (int gg = 0; gg < kMGroups; ++gg) {
            float ms[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                _Float16 hs;
                __builtin_memcpy(&hs, &sc[gg][i], 2);
                ms[i] = mv[i] * (float)hs;
            }
            // m * scale as a sum of two fp16 numbers: the rounded value and the rounded rest
            // (a denormal, which the matrix cores keep): 22 significant bits instead of 11
            _Float16 top[4], rest[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                top[i] = (_Float16)ms[i];
                rest[i] = (_Float16)(ms[i] - (float)top[i]);
            }
            struct Pair { uint32_t lo, hi; };
            Pair pa = __builtin_bit_cast(Pair, h4_t{top[0], top[1], top[2], top[3]});
            Pair pb = __builtin_bit_cast(Pair, h4_t{rest[0], rest[1], rest[2], rest[3]});
            pa.lo &= keep[0]; pa.hi &= keep[1];
            pb.lo &= keep[0]; pb.hi &= keep[1];
            const h4_t a = __builtin_bit_cast(h4_t, pa), a2 = __builtin_bit_cast(h4_t, pb);
            uint32_t ev[4], od[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t o = wq[gg][i] ^ 0x88888888u;     // q -> q + 8
                ev[i] = o & 0x0f0f0f0fu;
                od[i] = (o >> 4) & 0x0f0f0f0fu;
                // keeps the byte extracts below from being narrowed into bit-field extracts
                asm volatile("" : "+v"(ev[i]), "+v"(od[i]));
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int sh = 8 * (t >> 1);
                float f[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) f[i] = (float)((((t & 1) ? od[i] : ev[i]) >> sh) & 0xffu);
                const h4_t codes = pack_h4(f[0], f[1], f[2], f[3]);
                acc[gg][t] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, codes, acc[gg][t], 0, 0, 0);
                acc[gg][t] = __builtin_amdgcn_mfma_f32_16x16x16f16(a2, codes, acc[gg][t], 0, 0, 0);
            }
            acc1[gg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, ones, acc1[gg], 0, 0, 0);
            acc1[gg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a2, ones, acc1[gg], 0, 0, 0);
        }
    }
    // A result register i of lane l is batch row 4 * (l / 16) + i, lane column l % 16: the
    // first 32 lanes hold the 8 real rows.  One wavefront after the other adds its sums into
    // the same LDS tile (fixed order).
    for (int w = 0; w < kMWaves; ++w) {
        if (wave == w && lane < 32) {
#pragma unroll
            for (int gg = 0; gg < kMGroups; ++gg) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int b = 4 * r + i;
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        float* dst = &red[gg][t][b][c];
                        *dst = w == 0 ? acc[gg][t][i] : *dst + acc[gg][t][i];
                    }
                    if (c == 0) {
                        float* dst = &red1[gg][b];
                        *dst = w == 0 ? acc1[gg][i] : *dst + acc1[gg][i];
                    }
                }
            }
        }
        __syncthreads();
    }
    for (int o = tid; o < B * kMStripCols; o += kMWaves * 64) {
        const int b = o / kMStripCols, cc = o % kMStripCols;
        const int gcol = strip * kMStripCols + cc;
        if (gcol >= p.n_out) continue;
        const int gg = cc >> 7, cl = (cc & 127) >> 3, t = cc & 7;
        const float row_down = 1.0f / row_scale_up(p.rowmax[b]);     // a power of two: exact
        p.partial[((size_t)g * B + b) * (size_t)p.n_out + gcol] = fmaf(-8.0f, red1[gg][b], red[gg][t][b][cl]) * row_down;
    }
}

// out[b][j] = sum over shares of partial[g][b][j]   (glu == 0), or
// out[b][j] = up * SiLU(gate), up = sum partial[g][b][j], gate = sum partial[g][b][half + j];
// up to 20 shares in flight at a time (one or two memory round trips for the usual numbers
// of shares), added in share order
__global__ void breduce_kernel(BatchedReduceParams p) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int b = blockIdx.y;
    const int width = p.glu ? p.n_out / 2 : p.n_out;
    if (j >= width) return;
    const size_t gstride = (size_t)p.batch * (size_t)p.n_out;
    const float* src = p.partial + (size_t)b * (size_t)p.n_out + j;
    float s0 = 0.f, s1 = 0.f;
    // (loads past the last share re-read it and are dropped: a load under a branch would be
    //  waited for where the branch ends, one round trip each)
    constexpr int kInFlight = 20;
    const size_t goff = p.glu ? (size_t)width : 0;
    for (int g0 = 0; g0 < p.shares; g0 += kInFlight) {
        float a8[kInFlight], b8[kInFlight];
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) {
            const int gg = g0 + i < p.shares ? g0 + i : p.shares - 1;
            a8[i] = src[(size_t)gg * gstride];
            b8[i] = src[(size_t)gg * gstride + goff];
        }
#pragma unroll
        for (int i = 0; i < kInFlight; ++i)
            if (g0 + i < p.shares) { s0 += a8[i]; s1 += b8[i]; }
    }
    p.out[(size_t)b * p.out_stride + j] = p.glu ? s0 * (s1 / (1.0f + expf(-s1))) : s0;
}

template <int DT>
hipError_t launch_dt(const BatchedGemvParams& p, dim3 grid, hipStream_t stream, int pk) {
    const dim3 block(kBWaves * 64);
    switch (p.batch) {
        case 1: return launch_timed(bgemv_kernel<DT, 1>, grid, block, stream, pk, p);
        case 2: return launch_timed(bgemv_kernel<DT, 2>, grid, block, stream, pk, p);
        case 3: return launch_timed(bgemv_kernel<DT, 3>, grid, block, stream, pk, p);
        case 4: return launch_timed(bgemv_kernel<DT, 4>, grid, block, stream, pk, p);
        case 5: return launch_timed(bgemv_kernel<DT, 5>, grid, block, stream, pk, p);
        case 6: return launch_timed(bgemv_kernel<DT, 6>, grid, block, stream, pk, p);
        case 7: return launch_timed(bgemv_kernel<DT, 7>, grid, block, stream, pk, p);
        case 8: return launch_timed(bgemv_kernel<DT, 8>, grid, block, stream, pk, p);
    }
    return hipErrorInvalidValue;
}

}  // namespace

bool batched_on_matrix_cores(int dtype, int batch, int64_t n_in, int64_t row_stride) {
    // the matrix-core kernel addresses the stored matrix with 32-bit byte offsets
    return dtype == DIP_INT4_G128 && batch >= kMfmaMinBatch && n_in * row_stride < ((int64_t)1 << 32);
}

int batched_strip_cols(int dtype, int batch, bool mc) {
    if (mc) return kMStripCols;
    (void)batch;
    return dtype == DIP_F32 ? 16 * 4 : (dtype == DIP_BF16 ? 16 * 8 : 32 * 16);
}

int batched_shares(int dtype, int batch, int n_out, int k_max, bool mc) {
    // Vector-ALU product: about 1024 workgroups, at least 32 listed columns each.
    // Matrix-core product: one round of workgroups -- three of them fit a compute unit, 768
    // in all; 840 take as long as 1536 -- and at least one set of 16 per wavefront.
    const int sc = batched_strip_cols(dtype, batch, mc);
    const int strips = (n_out + sc - 1) / sc;
    const int min_rows = mc ? kMWaves * kMRowSet : 32;
    int g = mc ? 768 / strips : (1024 + strips - 1) / strips;
    while (g > 1 && k_max / g < min_rows) --g;
    return g < 1 ? 1 : g;
}

hipError_t launch_union(const UnionParams& p, hipStream_t stream) {
    const int nwords = (p.n + 31) >> 5;
    hipLaunchKernelGGL(union_kernel, dim3((nwords + kUnionWordsPerWg - 1) / kUnionWordsPerWg),
                       dim3(kUnionThreads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_batched_gemv(const BatchedGemvParams& p, int shares, bool mc, hipStream_t stream, int pk) {
    const int sc = batched_strip_cols(p.dtype, p.batch, mc);
    dim3 grid((p.n_out + sc - 1) / sc, shares);
    if (mc) {
        if (!p.rowmax || p.dtype != DIP_INT4_G128 || (int64_t)p.n_in * p.row_stride >= ((int64_t)1 << 32))
            return hipErrorInvalidValue;
        return launch_timed(bgemv_q4_mfma_kernel, grid, dim3(kMWaves * 64), stream, pk, p);
    }
    if (p.dtype == DIP_F32) return launch_dt<DIP_F32>(p, grid, stream, pk);
    if (p.dtype == DIP_BF16) return launch_dt<DIP_BF16>(p, grid, stream, pk);
    if (p.dtype == DIP_INT4_G128) return launch_dt<DIP_INT4_G128>(p, grid, stream, pk);
    return hipErrorInvalidValue;
}

hipError_t launch_batched_reduce(const BatchedReduceParams& p, hipStream_t stream) {
    const int width = p.glu ? p.n_out / 2 : p.n_out;
    hipLaunchKernelGGL(breduce_kernel, dim3((width + 255) / 256, p.batch), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace dip
