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
//                    B multipliers of every listed column (lists padded by 8 entries)
//   bgemv_kernel     column-gathered product for all B rows at once, partial sums per
//                    row share; the number of listed columns is read from device memory
//   breduce_kernel   adds the partial sums in share order and applies the epilogue
//                    (SwiGLU for the bundled up/gate matrix, Sec. 3 Eq. 2)

#include "dip_internal.h"

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
__global__ __launch_bounds__(kUnionThreads) void union_kernel(UnionParams p) {
    __shared__ uint32_t s_base[2 * kUnionThreads];
    __shared__ uint32_t s_wave[kUnionThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwords = (p.n + 31) >> 5;
    const int w0 = 2 * tid, w1 = 2 * tid + 1;
    uint32_t u0 = 0, u1 = 0;
    for (int b = 0; b < p.batch; ++b) {
        if (w0 < nwords) u0 |= p.masks[(size_t)b * p.words_stride + w0];
        if (w1 < nwords) u1 |= p.masks[(size_t)b * p.words_stride + w1];
    }
    const uint32_t c0 = (uint32_t)__popc(u0), c1 = (uint32_t)__popc(u1);
    uint32_t inc = c0 + c1;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kUnionThreads / 64; ++w) {
        const uint32_t t = s_wave[w];
        if (w < wave) before += t;
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

    const int w = blockIdx.x * kUnionWordsPerWg + (tid >> 5), bit = tid & 31;
    if (w >= nwords) return;
    uint32_t rows = 0, uw = 0;    // bit b of rows: row b selected this feature
    for (int b = 0; b < p.batch; ++b) {
        const uint32_t m = p.masks[(size_t)b * p.words_stride + w];
        uw |= m;
        rows |= ((m >> bit) & 1u) << b;
    }
    if (!rows) return;
    const uint32_t pos = s_base[w] + (uint32_t)__popc(uw & ((1u << bit) - 1u));
    const int i = w * 32 + bit;
    p.uidx[pos] = i;
    for (int b = 0; b < p.batch; ++b)
        p.uval[(size_t)pos * p.batch + b] = ((rows >> b) & 1u) ? p.x[(size_t)b * p.x_stride + i] : 0.f;
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

// out[b][j] = sum over shares of partial[g][b][j]   (glu == 0), or
// out[b][j] = up * SiLU(gate), up = sum partial[g][b][j], gate = sum partial[g][b][half + j];
// eight partial sums in flight at a time, added in share order
__global__ void breduce_kernel(BatchedReduceParams p) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int b = blockIdx.y;
    const int width = p.glu ? p.n_out / 2 : p.n_out;
    if (j >= width) return;
    const size_t gstride = (size_t)p.batch * (size_t)p.n_out;
    const float* src = p.partial + (size_t)b * (size_t)p.n_out + j;
    float s0 = 0.f, s1 = 0.f;
    for (int g0 = 0; g0 < p.shares; g0 += 8) {
        float a8[8], b8[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int gg = g0 + i < p.shares ? g0 + i : p.shares - 1;
            a8[i] = src[(size_t)gg * gstride];
            b8[i] = p.glu ? src[(size_t)gg * gstride + width] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
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

int batched_strip_cols(int dtype) {
    return dtype == DIP_F32 ? 16 * 4 : (dtype == DIP_BF16 ? 16 * 8 : 32 * 16);
}

int batched_shares(int dtype, int n_out, int k_max) {
    // about 1024 workgroups, at least 32 listed columns each
    const int strips = (n_out + batched_strip_cols(dtype) - 1) / batched_strip_cols(dtype);
    int g = (1024 + strips - 1) / strips;
    while (g > 1 && k_max / g < 32) --g;
    return g < 1 ? 1 : g;
}

hipError_t launch_union(const UnionParams& p, hipStream_t stream) {
    const int nwords = (p.n + 31) >> 5;
    hipLaunchKernelGGL(union_kernel, dim3((nwords + kUnionWordsPerWg - 1) / kUnionWordsPerWg),
                       dim3(kUnionThreads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_batched_gemv(const BatchedGemvParams& p, int shares, hipStream_t stream, int pk) {
    const int sc = batched_strip_cols(p.dtype);
    dim3 grid((p.n_out + sc - 1) / sc, shares);
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
