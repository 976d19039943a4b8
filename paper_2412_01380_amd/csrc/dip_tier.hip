// Two-tier residency (Sec. 5, Fig. 4 of the paper: a small fast memory in front of a large slow
// one).  On this machine the slow tier is pinned host memory behind PCIe and the fast tier a
// fixed number of row slots in HBM; the residency mask c of Alg. 1 says which columns have a
// slot.  After cache_update has produced c^(t), the kernels here
//   tier_update_kernel  hand the slots of the evicted columns to the inserted ones (the i-th
//                       inserted column, ascending, takes the slot of the i-th evicted one;
//                       the rest take slots never used before), list the rows to copy, and
//                       translate this token's selected columns into slot numbers (resident)
//                       or host row numbers (a miss that found no room and bypasses the cache);
//   tier_fill_kernel    copy the inserted columns host -> slot, one wavefront per row;
//   tier_init_kernel    give the r-th resident column (ascending) slot r at start-up.
// The gathered product then reads resident columns from HBM and bypassing ones over PCIe.

#include "dip_internal.h"

namespace dip {
namespace {

constexpr int kTierThreads = 1024;   // one lane per word of the 32768-column masks

// exclusive prefix over the workgroup of two 16-bit counts packed into one word
__device__ __forceinline__ uint32_t block_excl_scan_packed(uint32_t v, uint32_t* wave_tot, uint32_t& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kTierThreads / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) before += t;
        total += t;
    }
    return before + inc - v;
}

__global__ __launch_bounds__(kTierThreads) void tier_update_kernel(TierParams p) {
    __shared__ uint16_t freed[DIP_MAX_N];          // slots given up by the evicted columns, in column order
    __shared__ uint32_t wave_tot[kTierThreads / 64];
    const int tid = threadIdx.x;
    const int nwords = (p.n + 31) >> 5;
    const uint32_t ew = tid < nwords ? p.evicted[tid] : 0u;
    const uint32_t iw = tid < nwords ? p.inserted[tid] : 0u;
    uint32_t total;
    const uint32_t ex = block_excl_scan_packed((uint32_t)__popc(ew) | ((uint32_t)__popc(iw) << 16), wave_tot, total);
    const uint32_t n_evict = total & 0xffffu, n_ins = total >> 16;
    const uint32_t resident_after = p.meta[DIP_META_RESIDENT];
    const uint32_t first_fresh = resident_after - (n_ins - n_evict);   // slots handed out so far

    uint32_t pos = ex & 0xffffu;
    for (uint32_t rest = ew; rest; rest &= rest - 1u) {
        const int col = tid * 32 + (__ffs((int)rest) - 1);
        const int s = p.slot_of[col];
        freed[pos++] = (uint16_t)(s < 0 ? 0 : s);
        p.slot_of[col] = -1;
    }
    __syncthreads();
    pos = ex >> 16;
    for (uint32_t rest = iw; rest; rest &= rest - 1u) {
        const int col = tid * 32 + (__ffs((int)rest) - 1);
        uint32_t slot = pos < n_evict ? (uint32_t)freed[pos] : first_fresh + (pos - n_evict);
        if (slot >= (uint32_t)p.capacity) slot = 0;   // cannot happen with a consistent cache state
        p.slot_of[col] = (int32_t)slot;
        p.fill_col[pos] = col;
        p.fill_slot[pos] = (int32_t)slot;
        ++pos;
    }
    if (tid == 0) p.fill_count[0] = n_ins;
    // the translation below reads slot_of entries written by other lanes of this workgroup
    __threadfence_block();
    __syncthreads();
    for (int t = tid; t < p.k; t += kTierThreads) {
        const int col = p.idx[t];
        int code = ~0;                                 // outside the matrix: host row 0 ... dropped by the product
        if ((unsigned)col < (unsigned)p.n) {
            const int s = __hip_atomic_load(&p.slot_of[col], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            code = s >= 0 ? s : ~col;
        }
        p.src[t] = code;
    }
}

constexpr int kFillWaves = 4;

__global__ __launch_bounds__(kFillWaves * 64) void tier_fill_kernel(TierFillParams p) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * kFillWaves + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * kFillWaves;
    const int count = min((int)p.fill_count[0], p.max_rows);
    for (int r = wave; r < count; r += nwaves) {
        const char* src = static_cast<const char*>(p.host_rows) + (size_t)p.fill_col[r] * (size_t)p.row_stride;
        char* dst = static_cast<char*>(p.slots) + (size_t)p.fill_slot[r] * (size_t)p.row_stride;
        for (int64_t o = (int64_t)lane * 16; o < p.row_bytes; o += 64 * 16)
            *reinterpret_cast<u32x4*>(dst + o) = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + o));
    }
}

__global__ __launch_bounds__(kTierThreads) void tier_init_kernel(TierInitParams p) {
    __shared__ uint32_t wave_tot[kTierThreads / 64];
    const int tid = threadIdx.x;
    const int nwords = (p.n + 31) >> 5;
    const uint32_t cw = tid < nwords ? p.bits[tid] : 0u;
    uint32_t total;
    uint32_t pos = block_excl_scan_packed((uint32_t)__popc(cw), wave_tot, total);
    for (int b = 0; b < 32; ++b) {
        const int col = tid * 32 + b;
        if (col >= p.n) break;
        if ((cw >> b) & 1u) {
            p.slot_of[col] = (int32_t)pos;
            p.fill_col[pos] = col;
            p.fill_slot[pos] = (int32_t)pos;
            ++pos;
        } else {
            p.slot_of[col] = -1;
        }
    }
    if (tid == 0) p.fill_count[0] = total;
}

}  // namespace

hipError_t launch_tier_update(const TierParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(tier_update_kernel, dim3(1), dim3(kTierThreads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_tier_fill(const TierFillParams& p, hipStream_t stream, int prof_kind) {
    if (p.max_rows <= 0) return hipSuccess;
    const int grid = min(1024, (p.max_rows + kFillWaves - 1) / kFillWaves);
    return launch_timed(tier_fill_kernel, dim3(grid), dim3(kFillWaves * 64), stream, prof_kind, p);
}

hipError_t launch_tier_init(const TierInitParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(tier_init_kernel, dim3(1), dim3(kTierThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace dip
