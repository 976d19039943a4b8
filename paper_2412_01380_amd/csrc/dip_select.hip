// Selection kernel: scores (Sec. 5.2 Eq. 10) -> m = topK(s, k) (Alg. 1 step 2) ->
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
// top-K works on the 32-bit key patterns (non-negative floats order like their bit patterns):
// one histogram pass with bins laid from the largest possible key downwards, 512 per octave,
// then the few keys of the threshold bin are ranked in registers
// (block_select_largest_near_max); when the k-th largest key is not within eight octaves of
// the maximum, or many keys share its bin, a most-significant-digit radix select (12 + 10 + 10
// bits) takes over, whose two last digits only look at the keys of the threshold bin.
// Eviction victims (smallest (stamp, index) first) are the largest ages (current step -
// stamp) among the evictable columns, found by that radix select.
//
// The kernel runs on one compute unit and is bound by what that unit does in sequence: the
// instructions per key (16 wavefronts share 4 SIMDs: every instruction executed per key costs
// 16 cycles of the workgroup), the LDS adds of the histogram (with generic digits the keys of
// an activation vector crowd into a few dozen bins) and the barrier-separated LDS round
// trips.  Each stage is therefore written for the fewest instructions per key: plain histogram
// adds with the tie-storm handling hoisted out of the per-key path, branch-free clamped
// loads, one compare per key on the usual path where no tie is split at the threshold.
// The forward calls run the same selection at the head of the gathered products instead
// (dip_fused.hip); this kernel serves the stand-alone entry points, the batched rows, the
// two-tier path and, through update_batch_kernel, every cache update.
#include "dip_select_device.h"

namespace dip {
namespace {

using namespace sel;

constexpr int kVicCap = 12288;   // evictable columns whose (age, index) fit the LDS list

struct SelShared {
    uint32_t hist[kBinsA + kBinsB + kBinsC];
    uint32_t vkey[kVicCap];          // eviction keys of the evictable columns, ascending index
    uint16_t vidx[kVicCap];          // ... and their column indices
    uint32_t cw[kMaxWords];          // residency words (the paper's c)
    uint32_t mw[kMaxWords];          // mask words (m)
    uint32_t vpre[kMaxWords];        // evictable columns before each word
    uint32_t tile[2][kMaxTiles];
    uint32_t wave_tot[2][kWaves];
    float wave_max[kWaves];
    uint32_t bcast[4];
    uint32_t cnt[8];
    uint32_t cand[kNearCand];        // keys of the threshold bin
    uint32_t ncand;
};

__device__ __forceinline__ void store_ballot_words(uint32_t* words, int nwords, int first_word,
                                                   uint64_t b, int lane) {
    if (lane == 0 && first_word < nwords) words[first_word] = (uint32_t)b;
    if (lane == 32 && first_word + 1 < nwords) words[first_word + 1] = (uint32_t)(b >> 32);
}

// One slot of the selection `key >= T`: ballot, place in the index list, mask words.
// (A template recursion rather than a loop: the lane numbers must be constants.)
template <int J, int ITEMS, bool EMIT>
struct SelectGe {
    __device__ static __forceinline__ void run(const uint32_t (&key)[ITEMS], const float (&v)[ITEMS],
                                               uint32_t T, int pre, int32_t* idx_out, float* val_out,
                                               uint32_t k, uint32_t& sel, int& my_word) {
        const bool mine = key[J] >= T;
        const uint64_t bs = __ballot(mine);
        if (EMIT) {
            const uint32_t pos = (uint32_t)__builtin_amdgcn_readlane(pre, J) + lanes_below(bs);
            // pos < k always holds; the test keeps a logic slip from writing out of bounds
            // (and the mask tells the compiler that a 32-bit offset is enough)
            if (mine && pos < k) {
                idx_out[pos & (DIP_MAX_N - 1)] = J * kSelThreads + (int)threadIdx.x;
                val_out[pos & (DIP_MAX_N - 1)] = v[J];
            }
        }
        sel |= mine ? (1u << J) : 0u;
        write_lane<(2 * J) & 63>(my_word, (uint32_t)bs);
        write_lane<(2 * J + 1) & 63>(my_word, (uint32_t)(bs >> 32));
        if constexpr (J + 1 < ITEMS) SelectGe<J + 1, ITEMS, EMIT>::run(key, v, T, pre, idx_out, val_out, k, sel, my_word);
    }
};

template <int ITEMS>
__device__ __forceinline__ void select_body(SelectParams& p, SelShared& sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwords = (p.n + 31) >> 5;
    int phase = 0;

    for (int i = tid; i < p.zero_n; i += kSelThreads) p.zero_ptr[i] = 0u;

    // Features past n hold value 0 and key 0.  They sit at the highest indices, so the
    // lowest-index tie rule never picks them while k <= n, and they need no masking.
    float v[ITEMS];
    uint32_t key[ITEMS];
    uint32_t cres = 0, sel = 0;
    // this lane's features tid, tid + 1024, ... below n: the low `mine_n` slots
    const int mine_n = p.n > tid ? (p.n - tid - 1) / kSelThreads + 1 : 0;
    const uint32_t valid = mine_n >= 32 ? 0xffffffffu : (1u << mine_n) - 1u;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        v[j] = 0.f;
        key[j] = 0u;
    }
    if (p.v) {   // loads without branches: past the end the last element is read and dropped
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint32_t i = (uint32_t)(j * kSelThreads + tid);
            const float t = p.v[min(i, (uint32_t)p.n - 1u) & (DIP_MAX_N - 1)];
            v[j] = i < (uint32_t)p.n ? t : 0.f;
        }
    }
    // the radix histograms are cleared while the loads above are on their way
    if (!p.mask_in && !p.scores_only) {
        for (int b = tid; b < kBinsA + kBinsB + kBinsC; b += kSelThreads) sh.hist[b] = 0u;
        __syncthreads();
    }
    // residency and (when given) mask words: one per lane, then bit tests out of LDS
    const uint32_t* rb = p.c_bits ? p.c_bits : p.score_bits;
    if (rb || p.mask_in) {
        sh.cw[tid] = (rb && tid < nwords) ? rb[tid] : 0u;
        sh.mw[tid] = (p.mask_in && tid < nwords) ? p.mask_in[tid] : 0u;
        __syncthreads();
        if (rb) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                cres |= ((sh.cw[j * (kSelThreads / 32) + (tid >> 5)] >> (tid & 31)) & 1u) << j;
        }
        if (p.mask_in) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                sel |= ((sh.mw[j * (kSelThreads / 32) + (tid >> 5)] >> (tid & 31)) & 1u) << j;
        }
        cres &= valid;
        sel &= valid;
    }

    if (!p.mask_in) {
        // ---- Alg. 1 step 1: scores --------------------------------------------------
        // ||v||_inf: the denominator of Eq. 10, and the anchor of the selection's histogram
        float M;
        {
            float m = 0.f;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) m = fmaxf(m, fabsf(v[j]));
            m = wave_max_nonneg(m);
            if (lane == 0) sh.wave_max[wave] = m;
            __syncthreads();
            static_assert(kWaves == 16, "one wavefront maximum per lane of a 16-lane row");
            M = row_max_nonneg(sh.wave_max[lane & (kWaves - 1)]);
            if (p.rowmax_out && tid == 0) p.rowmax_out[0] = __float_as_uint(M);
        }
        if (p.score_bits) {
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
        uint32_t T, need, n_equal;
        // no key exceeds the score 1 (Eq. 10 divides by the maximum) or, without a cache, M
        const uint32_t max_key = (p.score_bits ? (M > 0.f ? __float_as_uint(1.0f) : 0u) : __float_as_uint(M)) << 1;
        block_select_largest_near_max<ITEMS>(key, max_key, (uint32_t)p.k, sh, phase, T, need, &n_equal);
        const bool want_words = p.mask_out || p.c_bits;
        // a wave ballot over slot j is two words of the mask: lane 2j keeps the low word and
        // lane 2j+1 the high word, stored to LDS once after the loop
        int my_word = 0;
        if (need == n_equal) {
            // No tie is split at the threshold (the usual case): the selection is key >= T and
            // a selected key's place in the list is the number of such keys before it.
            const int pre = (int)tile_prefix_ge<ITEMS>(key, T, sh, phase);
            const bool emit = p.idx_out && p.val_out;
            // (T is made opaque here: keeping the comparison masks of the counting pass in
            //  scalar registers for reuse costs more than comparing again)
            uint32_t Tv = T;
            asm volatile("" : "+v"(Tv));
            if (emit) SelectGe<0, ITEMS, true>::run(key, v, Tv, pre, p.idx_out, p.val_out, (uint32_t)p.k, sel, my_word);
            else SelectGe<0, ITEMS, false>::run(key, v, Tv, pre, p.idx_out, p.val_out, (uint32_t)p.k, sel, my_word);
            if (!emit && (p.idx_out || p.val_out)) {
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    const bool mine = (sel >> j) & 1u;
                    const uint32_t pos = (uint32_t)__builtin_amdgcn_readlane(pre, j) + lanes_below(__ballot(mine));
                    if (mine && pos < (uint32_t)p.k) {
                        if (p.idx_out) p.idx_out[pos] = j * kSelThreads + tid;
                        if (p.val_out) p.val_out[pos] = v[j];
                    }
                }
            }
        } else {
            const int pre = (int)tile_prefix_eq_gt<ITEMS>(key, T, sh, phase);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const int i = j * kSelThreads + tid;
                const uint32_t packed = (uint32_t)__builtin_amdgcn_readlane(pre, j);
                const uint32_t eq_before = packed & 0xffffu, gt_before = packed >> 16;
                const uint64_t be = __ballot(key[j] == T);
                bool mine = key[j] > T;
                if (be) {
                    // ties at the threshold: the `need` lowest indices among them are selected
                    mine = mine || (key[j] == T && eq_before + lanes_below(be) < need);
                }
                const uint64_t bs = __ballot(mine);
                const uint32_t pos = gt_before + min(eq_before, need) + lanes_below(bs);
                if (mine && pos < (uint32_t)p.k) {
                    if (p.idx_out) p.idx_out[pos] = i;
                    if (p.val_out) p.val_out[pos] = v[j];
                }
                sel |= mine ? (1u << j) : 0u;
                my_word = lane == 2 * j ? (int)(uint32_t)bs : my_word;
                my_word = lane == 2 * j + 1 ? (int)(uint32_t)(bs >> 32) : my_word;
            }
        }
        if (want_words && lane < 2 * ITEMS)
            sh.mw[(lane >> 1) * (kSelThreads / 32) + wave * 2 + (lane & 1)] = (uint32_t)my_word;
        if (want_words) __syncthreads();
        if (p.mask_out && tid < nwords) p.mask_out[tid] = sh.mw[tid];
    }

    // ---- Alg. 1 step 3: c' = cache_update(c, m) ------------------------------------------
    // Works on the 32-column words of c and m, one word per lane: hits, misses and
    // evictable columns are bit operations, their counts and running sums one packed
    // workgroup scan.  Only when something must be evicted are the stamps read and the
    // evictable columns listed (ascending) in LDS for the selection of the oldest.
    if (p.c_bits) {
        const uint32_t t_now = p.c_meta[DIP_META_STEP];
        const uint32_t cum_hits = p.c_meta[DIP_META_CUM_HITS];
        const uint32_t cum_look = p.c_meta[DIP_META_CUM_LOOKUPS];
        // words past nwords are zero; padding bits of the last word are ignored
        const uint32_t wmask = (tid == nwords - 1 && (p.n & 31)) ? (1u << (p.n & 31)) - 1u : 0xffffffffu;
        const uint32_t c = sh.cw[tid] & wmask, m = sh.mw[tid] & wmask;
        const uint32_t hitw = m & c, missw = m & ~c, vicw = c & ~m;
        const uint32_t n_missw = (uint32_t)__popc(missw);
        // two 16-bit counts per scan word: every total is at most 32768
        const uint32_t A = (uint32_t)__popc(c) | ((uint32_t)__popc(hitw) << 16);
        const uint32_t B = n_missw | ((uint32_t)__popc(vicw) << 16);
        const uint32_t exA = block_excl_scan(A, sh, phase);
        const uint32_t exB = block_excl_scan(B, sh, phase);
        sh.vpre[tid] = exB >> 16;
        if (tid == kSelThreads - 1) {
            sh.cnt[0] = exA + A;
            sh.cnt[1] = exB + B;
        }
        __syncthreads();
        const uint32_t n_res = sh.cnt[0] & 0xffffu, n_hit = sh.cnt[0] >> 16;
        const uint32_t n_miss = sh.cnt[1] & 0xffffu, n_vic = sh.cnt[1] >> 16;
        const uint32_t cap = (uint32_t)p.capacity;
        const uint32_t n_free = cap > n_res ? cap - n_res : 0u;
        const uint32_t n_ins = min(n_miss, n_free + n_vic);
        const uint32_t n_evict = n_ins > n_free ? n_ins - n_free : 0u;

        // the first n_ins misses (ascending index) are inserted
        const uint32_t miss_before = exB & 0xffffu;
        const uint32_t take = n_ins > miss_before ? min(n_ins - miss_before, n_missw) : 0u;
        uint32_t insw = missw;
        if (take < n_missw) {   // only the word(s) at the boundary
            insw = 0u;
            uint32_t mm = missw;
            for (uint32_t q = 0; q < take; ++q) {
                const uint32_t low = mm & (0u - mm);
                insw |= low;
                mm ^= low;
            }
        }

        // When the misses outnumber the room that evictions can make (the active set does not
        // fit: Sec. 6.4), every evictable column goes and nothing has to be ranked.
        const bool evict_all = n_evict > 0 && n_evict == n_vic;
        const bool need_stamps = (n_evict > 0 && !evict_all) || p.policy == DIP_LFU;
        uint32_t stamp_old[ITEMS];
        if (need_stamps) {
            // (slots past n read the last stamp; nothing below uses them: their residency and
            //  mask bits are zero)
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const uint32_t i = (uint32_t)(j * kSelThreads + tid);
                stamp_old[j] = p.c_stamp[min(i, (uint32_t)p.n - 1u) & (DIP_MAX_N - 1)];
            }
        }
        if (evict_all) {
            sh.cw[tid] = c & ~vicw;
            __syncthreads();
        } else if (n_evict > 0) {
            // Eviction key of an evictable column: its age t_now - stamp (LRU: steps since
            // last use, LFU: how far its use count lags the step counter), moved up so that
            // the top bit of t_now becomes bit 31.  The oldest / least used has the largest
            // key; equal keys go by the lowest index.
            const int age_shift = __clz((int)(t_now | 1u));
            const uint32_t vicm = cres & ~sel;
            uint32_t ek[ITEMS];
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const uint32_t age = t_now > stamp_old[j] ? t_now - stamp_old[j] : 1u;
                ek[j] = ((vicm >> j) & 1u) ? (age << age_shift) : 0u;
            }
            if (n_vic <= (uint32_t)kVicCap) {
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    const bool isv = (vicm >> j) & 1u;
                    const uint64_t bv = __ballot(isv);
                    if (isv) {
                        const uint32_t pos = sh.vpre[j * (kSelThreads / 32) + wave * 2] + lanes_below(bv);
                        if (pos < (uint32_t)kVicCap) {
                            sh.vkey[pos] = ek[j];
                            sh.vidx[pos] = (uint16_t)(j * kSelThreads + tid);
                        }
                    }
                }
                __syncthreads();
                const uint32_t chunk = (n_vic + kSelThreads - 1) / kSelThreads;
                const uint32_t lo = min(n_vic, (uint32_t)tid * chunk), hi = min(n_vic, lo + chunk);
                uint32_t T2, need2;
                list_select_largest(sh.vkey, lo, hi, n_evict, age_shift, sh, phase, T2, need2);
                uint32_t eqc = 0;
                for (uint32_t e = lo; e < hi; ++e) eqc += sh.vkey[e] == T2 ? 1u : 0u;
                uint32_t rank = block_excl_scan(eqc, sh, phase);
                for (uint32_t e = lo; e < hi; ++e) {
                    const uint32_t kk = sh.vkey[e];
                    bool ev = kk > T2;
                    if (kk == T2) ev = rank++ < need2;
                    if (ev) {
                        const uint32_t i = sh.vidx[e];
                        atomicAnd(&sh.cw[i >> 5], ~(1u << (i & 31u)));
                    }
                }
            } else {
                // more evictable columns than the list holds: select straight from the registers
                uint32_t T2, need2;
                block_select_largest<ITEMS, true>(ek, n_evict, sh, phase, T2, need2);
                const int pre2 = (int)tile_prefix_eq_gt<ITEMS>(ek, T2, sh, phase);
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    const uint32_t i = (uint32_t)(j * kSelThreads + tid);
                    const uint32_t eq_before = (uint32_t)__builtin_amdgcn_readlane(pre2, j) & 0xffffu;
                    const uint64_t be = __ballot(ek[j] == T2);
                    bool ev = ek[j] > T2;
                    if (be) ev = ev || (ek[j] == T2 && eq_before + lanes_below(be) < need2);
                    if (ev) atomicAnd(&sh.cw[i >> 5], ~(1u << (i & 31u)));
                }
            }
            __syncthreads();
        }
        const uint32_t kept = sh.cw[tid] & wmask;
        const uint32_t newc = kept | insw;
        if (tid < nwords) {
            if (p.evicted_out) p.evicted_out[tid] = c & ~kept;
            if (p.inserted_out) p.inserted_out[tid] = insw;
        }
        __syncthreads();          // every lane has read its word before any is replaced
        sh.cw[tid] = newc;
        if (tid < nwords) p.c_bits[tid] = newc;
        __syncthreads();
        // stamps: LRU marks everything used by this token that is resident afterwards
        // (hits and inserted columns); LFU counts every use
        if (p.policy == DIP_LFU) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                if ((sel >> j) & 1u) p.c_stamp[(uint32_t)(j * kSelThreads + tid) & (DIP_MAX_N - 1)] = stamp_old[j] + 1u;
        } else {
            uint32_t upd = 0u;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                upd |= ((sh.cw[j * (kSelThreads / 32) + (tid >> 5)] >> (tid & 31)) & 1u) << j;
            upd &= sel;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                if ((upd >> j) & 1u) p.c_stamp[(uint32_t)(j * kSelThreads + tid) & (DIP_MAX_N - 1)] = t_now;
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

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectParams p) {
    __shared__ SelShared sh;
    // one workgroup per row of a small batch (row 0 when there is no batch)
    if (p.v) p.v += (size_t)blockIdx.x * p.v_row_stride;
    if (p.mask_out) p.mask_out += (size_t)blockIdx.x * p.words_row_stride;
    if (p.rowmax_out) p.rowmax_out += blockIdx.x;
    select_body<ITEMS>(p, sh);
}

// pieces per launch: they travel in the kernel arguments (4 KB at most), and 80 is what a stack
// of 40 layers asks for in one call
constexpr int kUpdateBatch = 80;
struct UpdateWork {
    UpdatePiece piece[kUpdateBatch];
};
static_assert(sizeof(UpdateWork) <= 4096, "kernel arguments are limited to 4 KB");

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void update_batch_kernel(UpdateWork work) {
    __shared__ SelShared sh;
    const UpdatePiece u = work.piece[blockIdx.x];
    SelectParams p;
    p.v = nullptr; p.n = u.n; p.k = 1; p.score_bits = nullptr; p.gamma = 0.f;
    p.mask_in = u.mask; p.scores_only = 0; p.s_out = nullptr; p.mask_out = nullptr;
    p.idx_out = nullptr; p.val_out = nullptr;
    p.c_bits = u.bits; p.c_stamp = u.stamp; p.c_meta = u.meta; p.capacity = u.capacity; p.policy = u.policy;
    p.zero_ptr = nullptr; p.zero_n = 0; p.evicted_out = nullptr; p.inserted_out = nullptr;
    p.rows = 1; p.v_row_stride = 0; p.words_row_stride = 0; p.rowmax_out = nullptr;
    select_body<ITEMS>(p, sh);
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
    return launch_timed(select_kernel<ITEMS>, dim3(p.rows > 1 ? p.rows : 1), dim3(kSelThreads), stream, prof_kind, p);
}

template <int ITEMS>
hipError_t launch_update_items(const UpdateWork& work, int count, hipStream_t stream, int prof_kind) {
    return launch_timed(update_batch_kernel<ITEMS>, dim3(count), dim3(kSelThreads), stream, prof_kind, work);
}

}  // namespace

hipError_t launch_update_batch(const UpdatePiece* pieces, int count, hipStream_t stream, int prof_kind) {
    for (int first = 0; first < count; first += kUpdateBatch) {
        const int m = count - first < kUpdateBatch ? count - first : kUpdateBatch;
        UpdateWork work;
        int n = 1;
        for (int i = 0; i < kUpdateBatch; ++i) {
            work.piece[i] = pieces[first + (i < m ? i : 0)];
            if (i < m && work.piece[i].n > n) n = work.piece[i].n;
        }
        // all pieces of a launch run the instantiation that fits the longest cache
        const int items = (n + kSelThreads - 1) / kSelThreads;
        hipError_t e;
        if (items <= 4) e = launch_update_items<4>(work, m, stream, prof_kind);
        else if (items <= 8) e = launch_update_items<8>(work, m, stream, prof_kind);
        else if (items <= 14) e = launch_update_items<14>(work, m, stream, prof_kind);
        else if (items <= 18) e = launch_update_items<18>(work, m, stream, prof_kind);
        else if (items <= 24) e = launch_update_items<24>(work, m, stream, prof_kind);
        else e = launch_update_items<32>(work, m, stream, prof_kind);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_select(const SelectParams& p, hipStream_t stream, int prof_kind) {
    const int items = (p.n + kSelThreads - 1) / kSelThreads;
    switch (items) {
        case 1: return launch_items<1>(p, stream, prof_kind);
        case 2: return launch_items<2>(p, stream, prof_kind);
        case 3: return launch_items<3>(p, stream, prof_kind);
        case 4: return launch_items<4>(p, stream, prof_kind);
        case 5: return launch_items<5>(p, stream, prof_kind);
        case 6: return launch_items<6>(p, stream, prof_kind);
        case 7: case 8: return launch_items<8>(p, stream, prof_kind);
        case 9: case 10: return launch_items<10>(p, stream, prof_kind);
        case 11: case 12: return launch_items<12>(p, stream, prof_kind);
        case 13: case 14: return launch_items<14>(p, stream, prof_kind);
        case 15: case 16: return launch_items<16>(p, stream, prof_kind);
        case 17: case 18: return launch_items<18>(p, stream, prof_kind);
        case 19: case 20: return launch_items<20>(p, stream, prof_kind);
        case 21: case 22: case 23: case 24: return launch_items<24>(p, stream, prof_kind);
        case 25: case 26: case 27: case 28: return launch_items<28>(p, stream, prof_kind);
        default: return launch_items<32>(p, stream, prof_kind);
    }
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
