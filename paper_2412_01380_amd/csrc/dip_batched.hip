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
//                    B multipliers of every listed column
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
constexpr int kUnionThreads = 1024;   // one mask word per lane; n <= 32768

__global__ __launch_bounds__(kUnionThreads) void union_kernel(UnionParams p) {
    __shared__ uint32_t wave_tot[kUnionThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwords = (p.n + 31) >> 5;
    uint32_t rowbits[8];
    uint32_t u = 0;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        rowbits[b] = (b < p.batch && tid < nwords) ? p.masks[(size_t)b * p.words_stride + tid] : 0u;
        u |= rowbits[b];
    }
    if (tid < nwords) p.union_words[tid] = u;
    // exclusive prefix of the popcounts over the words (ascending index order)
    const uint32_t cnt = (uint32_t)__popc(u);
    uint32_t inc = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kUnionThreads / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) base += t;
        total += t;
    }
    if (tid == 0) p.count_out[0] = total;
    uint32_t pos = base + inc - cnt;
    uint32_t rest = u;
    while (rest) {
        const int bit = __ffs((int)rest) - 1;
        rest &= rest - 1u;
        const int i = tid * 32 + bit;
        p.uidx[pos] = i;
        for (int b = 0; b < p.batch; ++b)
            p.uval[(size_t)pos * p.batch + b] = ((rowbits[b] >> bit) & 1u) ? p.x[(size_t)b * p.x_stride + i] : 0.f;
        ++pos;
    }
}

// ---------------------------------------------------------------------------------------
// batched gathered product
// ---------------------------------------------------------------------------------------
template <int DT>
struct BElem;
template <>
struct BElem<DIP_F32> {   // 16-byte load, 4 values
    static constexpr int kElems = 4, kBits = 32;
    static constexpr bool kScaled = false;
    __device__ static __forceinline__ void load(const char* p, float (&f)[4]) {
        const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y);
        f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
    }
};
template <>
struct BElem<DIP_BF16> {  // 16-byte load, 8 values
    static constexpr int kElems = 8, kBits = 16;
    static constexpr bool kScaled = false;
    __device__ static __forceinline__ void load(const char* p, float (&f)[8]) {
        const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <>
struct BElem<DIP_INT4_G128> {  // 4-byte load, 8 codes (a batch multiplies every code B times,
                               // so fewer codes per lane keep the B x 8 accumulators in registers)
    static constexpr int kElems = 8, kBits = 4;
    static constexpr bool kScaled = true;
    __device__ static __forceinline__ void load(const char* p, float (&f)[8]) {
        const uint32_t w = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
#pragma unroll
        for (int n = 0; n < 8; ++n) f[n] = (float)(((int)(w << (28 - 4 * n))) >> 28);
    }
};

constexpr int kBWaves = 4;

template <int DT, int B, int LPR>
__global__ __launch_bounds__(kBWaves * 64) void bgemv_kernel(BatchedGemvParams p) {
    using E = BElem<DT>;
    constexpr int EPL = E::kElems;
    constexpr int RPW = 64 / LPR;
    constexpr int SC = LPR * EPL;
    constexpr int NG = kBWaves * RPW;
    __shared__ float red[kBWaves][B][SC];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, l = lane % LPR;
    const int strip = blockIdx.x, g = blockIdx.y, G = gridDim.y;
    const int col = strip * SC + l * EPL;
    const bool col_ok = col < p.n_out;

    const int k = min((int)p.k_dev[0], p.k_max);
    const int share = ((k + G - 1) / G + 3) / 4 * 4;
    const int kb = min(k, g * share), ke = min(k, kb + share);

    float acc[B][EPL];
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[b][e] = 0.f;

    const char* wbase = static_cast<const char*>(p.w) + (size_t)col * E::kBits / 8;
    const int sgroup = col >> 7;
    if (col_ok) {
        for (int t = kb + wave * RPW + sub; t < ke; t += NG) {
            const int r = p.uidx[t];
            if ((unsigned)r >= (unsigned)p.n_in) continue;
            float f[EPL];
            E::load(wbase + (size_t)r * (size_t)p.row_stride, f);
            float scale = 1.f;
            if constexpr (E::kScaled) {
                _Float16 hs;
                const uint16_t raw = p.scales[(size_t)r * p.scale_stride + sgroup];
                __builtin_memcpy(&hs, &raw, 2);
                scale = (float)hs;
            }
            float m[B];
#pragma unroll
            for (int b = 0; b < B; ++b) m[b] = p.uval[(size_t)t * B + b] * scale;
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[b][e] = fmaf(f[e], m[b], acc[b][e]);
        }
    }
    // lane groups of one wavefront, then wavefronts through LDS, both in a fixed order
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[b][e] += __shfl_xor(acc[b][e], off);
    if (sub == 0) {
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
            for (int e = 0; e < EPL; ++e) red[wave][b][l * EPL + e] = acc[b][e];
    }
    __syncthreads();
    for (int o = tid; o < B * SC; o += kBWaves * 64) {
        const int b = o / SC, c = o % SC;
        const int gcol = strip * SC + c;
        if (gcol >= p.n_out) continue;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kBWaves; ++w) sum += red[w][b][c];
        p.partial[((size_t)g * B + b) * (size_t)p.n_out + gcol] = sum;
    }
}

// out[b][j] = sum over shares of partial[g][b][j]   (glu == 0), or
// out[b][j] = up * SiLU(gate), up = sum partial[g][b][j], gate = sum partial[g][b][half + j]
__global__ void breduce_kernel(BatchedReduceParams p) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int b = blockIdx.y;
    const int width = p.glu ? p.n_out / 2 : p.n_out;
    if (j >= width) return;
    float s0 = 0.f, s1 = 0.f;
    for (int g = 0; g < p.shares; ++g) {
        const float* src = p.partial + ((size_t)g * p.batch + b) * (size_t)p.n_out;
        s0 += src[j];
        if (p.glu) s1 += src[width + j];
    }
    p.out[(size_t)b * p.out_stride + j] = p.glu ? s0 * (s1 / (1.0f + expf(-s1))) : s0;
}

template <int DT, int B>
hipError_t launch_b(const BatchedGemvParams& p, dim3 grid, hipStream_t stream, int pk) {
    constexpr int LPR = DT == DIP_INT4_G128 ? 32 : 16;
    return launch_timed(bgemv_kernel<DT, B, LPR>, grid, dim3(kBWaves * 64), stream, pk, p);
}

template <int DT>
hipError_t launch_dt(const BatchedGemvParams& p, dim3 grid, hipStream_t stream, int pk) {
    switch (p.batch) {
        case 1: return launch_b<DT, 1>(p, grid, stream, pk);
        case 2: return launch_b<DT, 2>(p, grid, stream, pk);
        case 3: return launch_b<DT, 3>(p, grid, stream, pk);
        case 4: return launch_b<DT, 4>(p, grid, stream, pk);
        case 5: return launch_b<DT, 5>(p, grid, stream, pk);
        case 6: return launch_b<DT, 6>(p, grid, stream, pk);
        case 7: return launch_b<DT, 7>(p, grid, stream, pk);
        case 8: return launch_b<DT, 8>(p, grid, stream, pk);
    }
    return hipErrorInvalidValue;
}

}  // namespace

int batched_strip_cols(int dtype) {
    return dtype == DIP_F32 ? 16 * 4 : (dtype == DIP_BF16 ? 16 * 8 : 32 * 8);
}

int batched_shares(int dtype, int n_out, int k_max) {
    // about 1024 workgroups, at least 32 listed columns each
    const int strips = (n_out + batched_strip_cols(dtype) - 1) / batched_strip_cols(dtype);
    int g = (1024 + strips - 1) / strips;
    while (g > 1 && k_max / g < 32) --g;
    return g < 1 ? 1 : g;
}

hipError_t launch_union(const UnionParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(union_kernel, dim3(1), dim3(kUnionThreads), 0, stream, p);
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
