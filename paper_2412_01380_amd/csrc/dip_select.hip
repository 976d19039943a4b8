// Selection kernel: scores (Sec. 5.2 Eq. 6) -> m = topK(s, k) (Alg. 1 step 2) ->
// c' = cache_update(c, m) (Alg. 1 step 3), for one vector of up to 32768 features.
//
// One workgroup of 1024 lanes (16 wavefronts of 64) keeps every key in registers:
// lane `tid` owns features tid, tid+1024, tid+2048, ...  so that, for a fixed item
// slot j, wavefront w covers the 64 consecutive features [j*1024 + w*64, +64).  A
// 64-bit wave ballot over a slot is therefore exactly two words of an output bit
// mask, and (slot, wavefront) tiles in ascending (j, w) order are the features in
// ascending index order, which is what the lowest-index tie rule and the ascending
// index list need.
//
// top-K is a three-pass most-significant-digit radix select (12 + 10 + 10 bits) on the
// 32-bit key patterns with LDS histograms; non-negative floats order like their bit
// patterns.  The same routine, on the complement of the stamps, picks eviction victims
// (smallest (stamp, index) first).

#include "dip_internal.h"

namespace dip {
namespace {

constexpr int kWaves = kSelThreads / 64;  // 16
constexpr int kMaxItems = DIP_MAX_N / kSelThreads;  // 32
constexpr int kMaxTiles = kMaxItems * kWaves;       // 512

struct SelShared {
    uint32_t hist[4096];
    uint32_t tile[2][kMaxTiles];
    uint32_t wave_tot[kWaves];
    float wave_max[kWaves];
    uint32_t bcast[4];
    uint32_t cnt[8];
};

__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, SelShared& sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) sh.wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        uint32_t t = sh.wave_tot[w];
        if (w < wave) base += t;
    }
    __syncthreads();
    return base + inc - v;
}

// Add one count per active lane to hist[d].  The lanes that share the first active lane's
// digit are merged into a single LDS atomic (keeps tie storms and narrow exponent ranges
// from serialising on one bin); the others add individually.
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t d, bool act, int lane) {
    const uint64_t am = __ballot(act);
    if (am == 0) return;
    const int leader = __ffsll((long long)am) - 1;
    const uint32_t d0 = __shfl(d, leader);
    const uint64_t same = __ballot(act && d == d0);
    if (lane == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
    if (act && d != d0) atomicAdd(&hist[d], 1u);
}

// Among the participating items (bit j of `part` set) find T = the k-th largest key and
// need = how many keys equal to T belong to the k largest.  Requires 1 <= k <= participants.
template <int ITEMS>
__device__ __forceinline__ void block_select_largest(const uint32_t (&key)[ITEMS], uint32_t part,
                                                     uint32_t k, SelShared& sh, uint32_t& T,
                                                     uint32_t& need) {
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t prefix = 0, pmask = 0, remaining = k;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
        const int nb = pass == 0 ? 4096 : 1024;
        for (int b = tid; b < nb; b += kSelThreads) sh.hist[b] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const bool act = ((part >> j) & 1u) && ((key[j] & pmask) == prefix);
            const uint32_t d = (key[j] >> shift) & (uint32_t)(nb - 1);
            hist_add(sh.hist, d, act, lane);
        }
        __syncthreads();
        // lane tid owns `per` bins counted down from the top; bins above it come first
        const int per = nb / kSelThreads;
        const int top = nb - 1 - tid * per;
        uint32_t local = 0;
        for (int q = 0; q < per; ++q) local += sh.hist[top - q];
        const uint32_t above = block_excl_scan(local, sh);
        if (above < remaining && remaining <= above + local) {
            uint32_t acc = above;
            int b = top;
            for (int q = 0; q < per; ++q) {
                const uint32_t c = sh.hist[top - q];
                if (remaining <= acc + c) { b = top - q; break; }
                acc += c;
            }
            sh.bcast[0] = (uint32_t)b;
            sh.bcast[1] = acc;
        }
        __syncthreads();
        const uint32_t b = sh.bcast[0];
        remaining -= sh.bcast[1];
        prefix |= b << shift;
        pmask |= (uint32_t)(nb - 1) << shift;
        __syncthreads();
    }
    T = prefix;
    need = remaining;
}

// Exclusive prefix over the (slot, wavefront) tiles of sh.tile[which], in place.
template <int ITEMS>
__device__ __forceinline__ void scan_tiles(SelShared& sh, int which) {
    constexpr int ntiles = ITEMS * kWaves;
    const int tid = threadIdx.x;
    const uint32_t mine = tid < ntiles ? sh.tile[which][tid] : 0u;
    const uint32_t ex = block_excl_scan(mine, sh);
    if (tid < ntiles) sh.tile[which][tid] = ex;
    __syncthreads();
}

__device__ __forceinline__ void store_ballot_words(uint32_t* words, int nwords, int first_word,
                                                   uint64_t b, int lane) {
    if (lane == 0 && first_word < nwords) words[first_word] = (uint32_t)b;
    if (lane == 32 && first_word + 1 < nwords) words[first_word + 1] = (uint32_t)(b >> 32);
}

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectParams p) {
    __shared__ SelShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint64_t lt = (1ull << lane) - 1ull;
    const int nwords = (p.n + 31) >> 5;

    for (int i = tid; i < p.zero_n; i += kSelThreads) p.zero_ptr[i] = 0u;

    float v[ITEMS];
    uint32_t key[ITEMS];
    uint32_t valid = 0, cres = 0, sel = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int i = j * kSelThreads + tid;
        v[j] = 0.f;
        key[j] = 0u;
        if (i < p.n) {
            valid |= 1u << j;
            if (p.v) v[j] = p.v[i];
        }
    }
    const uint32_t* rb = p.c_bits ? p.c_bits : p.score_bits;
    if (rb) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = j * kSelThreads + tid;
            if ((valid >> j) & 1u) {
                if ((rb[i >> 5] >> (i & 31)) & 1u) cres |= 1u << j;
            }
        }
    }

    if (p.mask_in) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = j * kSelThreads + tid;
            if ((valid >> j) & 1u) {
                if ((p.mask_in[i >> 5] >> (i & 31)) & 1u) sel |= 1u << j;
            }
        }
    } else {
        // ---- Alg. 1 step 1: scores --------------------------------------------------
        if (p.score_bits) {
            float m = 0.f;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) m = fmaxf(m, fabsf(v[j]));
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
            if (lane == 0) sh.wave_max[wave] = m;
            __syncthreads();
            float M = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sh.wave_max[w]);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const float a = fabsf(v[j]);
                const float pn = ((cres >> j) & 1u) ? a : __fmul_rn(a, p.gamma);
                const float s = (M > 0.f) ? __fdiv_rn(pn, M) : 0.f;
                key[j] = __float_as_uint(s);
            }
        } else {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) key[j] = __float_as_uint(fabsf(v[j]));
        }
        if (p.s_out) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int i = j * kSelThreads + tid;
                if ((valid >> j) & 1u) p.s_out[i] = __uint_as_float(key[j]);
            }
        }
        if (p.scores_only) return;

        // ---- Alg. 1 step 2: m = topK(s, k) -------------------------------------------
        // the sign bit of a score is 0: shifting it out gives the exponent one more
        // histogram bit without changing the order
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) key[j] <<= 1;
        uint32_t T, need;
        block_select_largest<ITEMS>(key, valid, (uint32_t)p.k, sh, T, need);
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const bool ok = (valid >> j) & 1u;
            const uint64_t be = __ballot(ok && key[j] == T);
            const uint64_t bg = __ballot(ok && key[j] > T);
            if (lane == 0) {
                sh.tile[0][j * kWaves + wave] = (uint32_t)__popcll(be);
                sh.tile[1][j * kWaves + wave] = (uint32_t)__popcll(bg);
            }
        }
        __syncthreads();
        scan_tiles<ITEMS>(sh, 0);
        scan_tiles<ITEMS>(sh, 1);
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = j * kSelThreads + tid;
            const bool ok = (valid >> j) & 1u;
            const bool e = ok && key[j] == T;
            const bool g = ok && key[j] > T;
            const uint64_t be = __ballot(e);
            const uint32_t eq_before = sh.tile[0][j * kWaves + wave];
            const uint32_t gt_before = sh.tile[1][j * kWaves + wave];
            const uint32_t rank = eq_before + (uint32_t)__popcll(be & lt);
            const bool s = g || (e && rank < need);
            const uint64_t bs = __ballot(s);
            if (s) {
                sel |= 1u << j;
                const uint32_t pos = gt_before + min(eq_before, need) + (uint32_t)__popcll(bs & lt);
                if (pos < (uint32_t)p.k) {  // always true; keeps a logic slip from writing out of bounds
                    if (p.idx_out) p.idx_out[pos] = i;
                    if (p.val_out) p.val_out[pos] = v[j];
                }
            }
        }
    }

    if (p.mask_out) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint64_t bs = __ballot((sel >> j) & 1u);
            store_ballot_words(p.mask_out, nwords, (j * kSelThreads + wave * 64) >> 5, bs, lane);
        }
    }

    // ---- Alg. 1 step 3: c' = cache_update(c, m) ------------------------------------------
    if (p.c_bits) {
        const uint32_t t_now = p.c_meta[DIP_META_STEP];
        const uint32_t cum_hits = p.c_meta[DIP_META_CUM_HITS];
        const uint32_t cum_look = p.c_meta[DIP_META_CUM_LOOKUPS];
        if (tid < 8) sh.cnt[tid] = 0u;
        __syncthreads();
        uint32_t w_res = 0, w_hit = 0, w_miss = 0, w_vic = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const bool r = (cres >> j) & 1u, s = (sel >> j) & 1u;
            const uint64_t bmiss = __ballot(s && !r);
            w_res += (uint32_t)__popcll(__ballot(r));
            w_hit += (uint32_t)__popcll(__ballot(r && s));
            w_vic += (uint32_t)__popcll(__ballot(r && !s));
            w_miss += (uint32_t)__popcll(bmiss);
            if (lane == 0) sh.tile[0][j * kWaves + wave] = (uint32_t)__popcll(bmiss);
        }
        if (lane == 0) {
            atomicAdd(&sh.cnt[0], w_res);
            atomicAdd(&sh.cnt[1], w_hit);
            atomicAdd(&sh.cnt[2], w_miss);
            atomicAdd(&sh.cnt[3], w_vic);
        }
        __syncthreads();
        const uint32_t n_res = sh.cnt[0], n_hit = sh.cnt[1], n_miss = sh.cnt[2], n_vic = sh.cnt[3];
        const uint32_t cap = (uint32_t)p.capacity;
        const uint32_t n_free = cap > n_res ? cap - n_res : 0u;
        const uint32_t n_ins = min(n_miss, n_free + n_vic);
        const uint32_t n_evict = n_ins > n_free ? n_ins - n_free : 0u;
        scan_tiles<ITEMS>(sh, 0);  // misses before each tile

        // priority of every column; the complement makes "smallest stamp" the largest key
        uint32_t ek[ITEMS];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = j * kSelThreads + tid;
            ek[j] = ((valid >> j) & 1u) ? ~p.c_stamp[i] : 0u;
        }
        uint32_t evict = 0;
        if (n_evict > 0) {
            const uint32_t vicm = cres & ~sel;
            uint32_t T2, need2;
            block_select_largest<ITEMS>(ek, vicm, n_evict, sh, T2, need2);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const bool e = ((vicm >> j) & 1u) && ek[j] == T2;
                const uint64_t be = __ballot(e);
                if (lane == 0) sh.tile[1][j * kWaves + wave] = (uint32_t)__popcll(be);
            }
            __syncthreads();
            scan_tiles<ITEMS>(sh, 1);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const bool vj = (vicm >> j) & 1u;
                const bool e = vj && ek[j] == T2;
                const bool g = vj && ek[j] > T2;
                const uint64_t be = __ballot(e);
                const uint32_t rank = sh.tile[1][j * kWaves + wave] + (uint32_t)__popcll(be & lt);
                if (g || (e && rank < need2)) evict |= 1u << j;
            }
        }
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = j * kSelThreads + tid;
            const bool r = (cres >> j) & 1u, s = (sel >> j) & 1u;
            const bool miss = s && !r;
            const uint64_t bm = __ballot(miss);
            const uint32_t rank = sh.tile[0][j * kWaves + wave] + (uint32_t)__popcll(bm & lt);
            const bool ins = miss && rank < n_ins;
            const bool newc = (r && !((evict >> j) & 1u)) || ins;
            const uint64_t bn = __ballot(newc);
            store_ballot_words(p.c_bits, nwords, (j * kSelThreads + wave * 64) >> 5, bn, lane);
            if (p.policy == DIP_LFU) {
                if (s) p.c_stamp[i] = ~ek[j] + 1u;
            } else {
                if ((r && s) || ins) p.c_stamp[i] = t_now;
            }
        }
        if (tid == 0) {
            p.c_meta[DIP_META_STEP] = t_now + 1u;
            p.c_meta[DIP_META_RESIDENT] = n_res - n_evict + n_ins;
            p.c_meta[DIP_META_HITS] = n_hit;
            p.c_meta[DIP_META_INSERTED] = n_ins;
            p.c_meta[DIP_META_EVICTED] = n_evict;
            p.c_meta[DIP_META_BYPASSED] = n_miss - n_ins;
            p.c_meta[DIP_META_CUM_HITS] = cum_hits + n_hit;
            p.c_meta[DIP_META_CUM_LOOKUPS] = cum_look + n_hit + n_miss;
        }
    }
}

__global__ void cache_init_kernel(CacheInitParams p) {
    const int nwords = (p.n + 31) >> 5;
    const int stride = gridDim.x * blockDim.x;
    const int t0 = blockIdx.x * blockDim.x + threadIdx.x;
    for (int i = t0; i < p.n; i += stride) p.stamp[i] = 0u;
    for (int i = t0; i < nwords; i += stride) p.bits[i] = p.initial_bits ? p.initial_bits[i] : 0u;
    if (blockIdx.x == 0) {
        // resident count: one workgroup counts the initial bits
        __shared__ uint32_t total;
        if (threadIdx.x == 0) total = 0u;
        __syncthreads();
        uint32_t c = 0;
        if (p.initial_bits)
            for (int i = threadIdx.x; i < nwords; i += blockDim.x) c += (uint32_t)__popc(p.initial_bits[i]);
        if (c) atomicAdd(&total, c);
        __syncthreads();
        if (threadIdx.x < DIP_CACHE_META_WORDS) {
            uint32_t val = 0u;
            if (threadIdx.x == DIP_META_STEP) val = 1u;
            if (threadIdx.x == DIP_META_RESIDENT) val = total;
            p.meta[threadIdx.x] = val;
        }
    }
}

__global__ void zero_u32_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

template <int ITEMS>
hipError_t launch_items(const SelectParams& p, hipStream_t stream, int prof_kind) {
    return launch_timed(select_kernel<ITEMS>, dim3(1), dim3(kSelThreads), stream, prof_kind, p);
}

}  // namespace

hipError_t launch_select(const SelectParams& p, hipStream_t stream, int prof_kind) {
    const int items = (p.n + kSelThreads - 1) / kSelThreads;
    if (items <= 1) return launch_items<1>(p, stream, prof_kind);
    if (items <= 2) return launch_items<2>(p, stream, prof_kind);
    if (items <= 4) return launch_items<4>(p, stream, prof_kind);
    if (items <= 6) return launch_items<6>(p, stream, prof_kind);
    if (items <= 8) return launch_items<8>(p, stream, prof_kind);
    if (items <= 12) return launch_items<12>(p, stream, prof_kind);
    if (items <= 16) return launch_items<16>(p, stream, prof_kind);
    if (items <= 20) return launch_items<20>(p, stream, prof_kind);
    if (items <= 24) return launch_items<24>(p, stream, prof_kind);
    return launch_items<32>(p, stream, prof_kind);
}

hipError_t launch_cache_init(const CacheInitParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(cache_init_kernel, dim3(16), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_zero_u32(uint32_t* p, int n, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(zero_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
    return hipGetLastError();
}

}  // namespace dip
