// Device-side building blocks of the selection (scores -> top-K) shared by the stand-alone
// selection kernel and by the gathered products that run the selection at their head.
// Everything here is written for a workgroup of kSelThreads = 1024 lanes (16 wavefronts);
// SH is the kernel's shared-memory struct and must provide
//     uint32_t hist[kBinsA + kBinsB + kBinsC], tile[2][kMaxTiles], wave_tot[2][kWaves], bcast[4].
#ifndef DIP_SELECT_DEVICE_H_
#define DIP_SELECT_DEVICE_H_

#include "dip_internal.h"

#ifndef SEL_WRITELANE
#define SEL_WRITELANE 1
#endif

namespace dip {
namespace sel {

constexpr int kWaves = kSelThreads / 64;            // 16
constexpr int kMaxItems = DIP_MAX_N / kSelThreads;  // 32
constexpr int kMaxTiles = kMaxItems * kWaves;       // 512
constexpr int kBinsA = 4096, kBinsB = 1024, kBinsC = 1024;

constexpr int kMaxWords = DIP_MAX_N / 32;  // 1024: one residency / mask word per lane


// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel primitives:
// shifts inside each row of 16 lanes, then the last lane of row 0/2 is added to row 1/3,
// then lane 31 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
    int v = (int)x;
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);  // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2, 3
    return (uint32_t)v;
}

// Maximum of a non-negative float over the lanes of a wavefront, with data-parallel
// primitives (non-negative floats order as their bit patterns; a lane without a source keeps
// 0).  wave_max_nonneg: all 64 lanes; row_max_nonneg: the 16 lanes of the caller's row.
// Every lane receives the result.
__device__ __forceinline__ float row_max_nonneg(float x) {
    int v = __float_as_int(x);
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false));  // row_shr:1
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false));  // row_shr:2
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false));  // row_shr:4
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false));  // row_shr:8
    return __int_as_float(__builtin_amdgcn_readlane(v, 15));
}
__device__ __forceinline__ float wave_max_nonneg(float x) {
    int v = __float_as_int(x);
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false));  // row_shr:1
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false));  // row_shr:2
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false));  // row_shr:4
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false));  // row_shr:8
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false));  // row_bcast:15 -> rows 1, 3
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false));  // row_bcast:31 -> rows 2, 3
    return __int_as_float(__builtin_amdgcn_readlane(v, 63));
}

// Exclusive prefix sum over the 1024 lanes of the workgroup (one barrier).  `phase`
// alternates between two LDS buffers so that back-to-back calls need no trailing barrier.
template <typename SH>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, SH& sh, int& phase) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t inc = wave_incl_scan(v);
    uint32_t* tot = sh.wave_tot[phase];
    phase ^= 1;
    if (lane == 63) tot[wave] = inc;
    __syncthreads();
    // Sum of the totals of the wavefronts before this one: lane w < wave takes tot[w], the 16
    // lanes of row 0 are added with shifts inside the row, and lane 15 holds the sum (a loop
    // over the 16 totals costs every wavefront four instructions per total).
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    int t = lane < wv ? (int)tot[lane & (kWaves - 1)] : 0;
    t += __builtin_amdgcn_update_dpp(0, t, 0x111, 0xf, 0xf, false);  // row_shr:1
    t += __builtin_amdgcn_update_dpp(0, t, 0x112, 0xf, 0xf, false);  // row_shr:2
    t += __builtin_amdgcn_update_dpp(0, t, 0x114, 0xf, 0xf, false);  // row_shr:4
    t += __builtin_amdgcn_update_dpp(0, t, 0x118, 0xf, 0xf, false);  // row_shr:8
    const uint32_t base = (uint32_t)__builtin_amdgcn_readlane(t, 15);
    return base + inc - v;
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    // number of set bits of `mask` at positions below the calling lane
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// One count into hist[d] for every lane whose key is not 0 (eviction keys: most lanes hold a
// column that does not take part).
__device__ __forceinline__ void hist_add_nonzero(uint32_t* hist, uint32_t d, uint32_t key) {
    if (key != 0u) atomicAdd(&hist[d], 1u);
}

// Scan the bins from the top: find the bin in which the running count reaches `want`.
// Returns the bin, the count in the bins above it, and the count inside it.  Ends with a
// barrier, so every lane holds the same answer and the histogram may be reused.
template <int PER, typename SH>
__device__ __forceinline__ void find_bin(const uint32_t* hist, uint32_t want, SH& sh,
                                         int& phase, uint32_t& bin, uint32_t& above,
                                         uint32_t& inbin) {
    constexpr int nb = PER * kSelThreads;
    const int top = nb - 1 - (int)threadIdx.x * PER;  // this lane owns bins top, top-1, ...
    uint32_t c[PER];
    uint32_t local = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        c[q] = hist[top - q];
        local += c[q];
    }
    const uint32_t ab = block_excl_scan(local, sh, phase);
    if (ab < want && want <= ab + local) {
        uint32_t acc = ab;
        bool done = false;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            if (!done && want <= acc + c[q]) {
                sh.bcast[0] = (uint32_t)(top - q);
                sh.bcast[1] = acc;
                sh.bcast[2] = c[q];
                done = true;
            }
            acc += c[q];
        }
    }
    __syncthreads();
    bin = sh.bcast[0];
    above = sh.bcast[1];
    inbin = sh.bcast[2];
}

// Find T = the k-th largest of all ITEMS*1024 keys held by the workgroup and need = how
// many keys equal to T belong to the k largest.  Keys that must not take part are 0 and
// the caller guarantees that at least k keys are larger than 0 or that zero keys at the
// highest indices are harmless (padding).  Requires k >= 1.
// `hist_is_zero`: the caller has cleared sh.hist and a barrier lies between that and this call.
template <int ITEMS, bool SKIP_ZERO, typename SH>
__device__ __forceinline__ void block_select_largest(const uint32_t (&key)[ITEMS], uint32_t k,
                                                     SH& sh, int& phase, uint32_t& T,
                                                     uint32_t& need, bool hist_is_zero = false,
                                                     uint32_t* n_equal = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t* histA = sh.hist;
    uint32_t* histB = sh.hist + kBinsA;
    uint32_t* histC = sh.hist + kBinsA + kBinsB;
    if (!hist_is_zero) {
        for (int b = tid; b < kBinsA + kBinsB + kBinsC; b += kSelThreads) sh.hist[b] = 0u;
        __syncthreads();
    }

    // Many equal keys ("tie storms": an all-zero vector, the high digits of stamps) would
    // serialise their LDS adds on one address.  Per key, merging equal digits costs more
    // instructions than the add itself, and this kernel is bound by instruction issue; so
    // the plain add is the default and the merged forms are chosen per wavefront (digit 1:
    // all of its keys share the digit) or per pass (digits 2, 3: the bin being refined holds
    // more than kStorm keys).
    constexpr uint32_t kStorm = 2048;

    // digit 1: bits 31..20, every key
    if (SKIP_ZERO) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) hist_add_nonzero(histA, key[j] >> 20, key[j]);
    } else {
        const uint32_t k0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)key[0]);
        uint32_t diff = 0u;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) diff |= key[j] ^ k0;
        if (__ballot((diff >> 20) != 0u) == 0ull) {      // wave-uniform branch
            if (lane == 0) atomicAdd(&histA[k0 >> 20], 64u * ITEMS);
        } else {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) atomicAdd(&histA[key[j] >> 20], 1u);
        }
    }
    __syncthreads();
    uint32_t b1, above, inbin;
    find_bin<kBinsA / kSelThreads>(histA, k, sh, phase, b1, above, inbin);
    uint32_t remaining = k - above;

    // digit 2: bits 19..10, only the keys of the threshold bin (a few per cent of the vector)
    if (inbin > kStorm || SKIP_ZERO) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            if ((key[j] >> 20) == b1 && (!SKIP_ZERO || key[j] != 0u)) {
                // merge the lanes of a wavefront that share the digit of its first caller
                const uint32_t d = (key[j] >> 10) & 1023u;
                const uint32_t d0 = __builtin_amdgcn_readfirstlane(d);
                const uint64_t same = __ballot(d == d0);
                if (d == d0) {
                    if (lanes_below(same) == 0u) atomicAdd(&histB[d0], (uint32_t)__popcll(same));
                } else {
                    atomicAdd(&histB[d], 1u);
                }
            }
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            if ((key[j] >> 20) == b1) atomicAdd(&histB[(key[j] >> 10) & 1023u], 1u);
    }
    __syncthreads();
    uint32_t b2;
    find_bin<1>(histB, remaining, sh, phase, b2, above, inbin);
    remaining -= above;
    const uint32_t hi = (b1 << 10) | b2;

    // digit 3: bits 9..0
    if (inbin > kStorm || SKIP_ZERO) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            if ((key[j] >> 10) == hi && (!SKIP_ZERO || key[j] != 0u)) {
                const uint32_t d = key[j] & 1023u;
                const uint32_t d0 = __builtin_amdgcn_readfirstlane(d);
                const uint64_t same = __ballot(d == d0);
                if (d == d0) {
                    if (lanes_below(same) == 0u) atomicAdd(&histC[d0], (uint32_t)__popcll(same));
                } else {
                    atomicAdd(&histC[d], 1u);
                }
            }
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            if ((key[j] >> 10) == hi) atomicAdd(&histC[key[j] & 1023u], 1u);
    }
    __syncthreads();
    uint32_t b3;
    find_bin<1>(histC, remaining, sh, phase, b3, above, inbin);
    T = (hi << 10) | b3;
    need = remaining - above;
    if (n_equal) *n_equal = inbin;   // the last digit's bin is one key value
}

// One count into hist[d] from inside divergent code: when all calling lanes of the
// wavefront carry the same digit, the first of them adds the whole count.
__device__ __forceinline__ void hist_add_callers(uint32_t* hist, uint32_t d) {
    const uint32_t d0 = __builtin_amdgcn_readfirstlane(d);
    const uint64_t callers = __ballot(true);
    const uint64_t same = __ballot(d == d0);
    if (same == callers) {
        if (lanes_below(callers) == 0u) atomicAdd(&hist[d0], (uint32_t)__popcll(callers));
    } else {
        atomicAdd(&hist[d], 1u);
    }
}

// The k-th largest key and its tie count as block_select_largest returns them, for keys that
// are bit patterns of non-negative floats (shifted left by one) and `max_key` >= every key,
// found with ONE histogram pass in the usual case.
//
// The first generic digit is sign, exponent and three mantissa bits: 16 bins per octave, the
// threshold bin holds a few per cent of the keys, and two more passes over all keys must
// refine it.  Here the bins are laid from the maximum downwards, 512 per octave over eight
// octaves (bin 4095 - ((max_key - key) >> 15); keys farther down are not counted): the
// threshold bin then holds about a thousandth of the keys.  Those are copied to a short list
// in LDS, and every wavefront ranks the list in registers -- no further pass, no further bin
// search.  When the k-th largest key is not within eight octaves of the maximum, or its bin
// holds more than kNearCand keys (many equal values), the generic digits are run instead.
// SH needs cand[kNearCand] and ncand besides the fields block_select_largest uses.
// Requires k >= 1 and sh.hist all zero behind a barrier.  `n_equal` (nullable): the number of
// keys equal to T.
constexpr int kNearCand = 64;

template <int ITEMS, typename SH>
__device__ __forceinline__ void block_select_largest_near_max(const uint32_t (&key)[ITEMS],
                                                              uint32_t max_key, uint32_t k, SH& sh,
                                                              int& phase, uint32_t& T, uint32_t& need,
                                                              uint32_t* n_equal = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t* histA = sh.hist;
    constexpr uint32_t kShift = 15;
    constexpr uint32_t kRange = (uint32_t)(kBinsA - 1) << kShift;   // bins 1..4095; bin 0 stays empty
    constexpr uint32_t kNone = 0xffffffffu;
    if (max_key == 0u) {        // every key is 0: they all tie (uniform over the workgroup)
        T = 0u;
        need = k;
        if (n_equal) *n_equal = (uint32_t)(ITEMS * kSelThreads);
        return;
    }
    if (tid == 0) {
        sh.bcast[0] = kNone;    // stays if the bins hold fewer than k keys
        sh.ncand = 0u;
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const uint32_t d = max_key - key[j];     // (a key above max_key -- a NaN -- wraps to "far")
        if (d < kRange) atomicAdd(&histA[(uint32_t)(kBinsA - 1) - (d >> kShift)], 1u);
    }
    __syncthreads();
    uint32_t b1, above, inbin;
    find_bin<kBinsA / kSelThreads>(histA, k, sh, phase, b1, above, inbin);
    // (read from LDS by every lane: the same everywhere; say so to the compiler)
    b1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)b1);
    above = (uint32_t)__builtin_amdgcn_readfirstlane((int)above);
    inbin = (uint32_t)__builtin_amdgcn_readfirstlane((int)inbin);
    if (b1 == kNone || inbin > (uint32_t)kNearCand) {
        // not near the maximum, or a crowd of equal keys
        for (int b = tid; b < kBinsA; b += kSelThreads) histA[b] = 0u;
        __syncthreads();
        block_select_largest<ITEMS, false>(key, k, sh, phase, T, need, true, n_equal);
        return;
    }
    const uint32_t remaining = k - above;        // 1 <= remaining <= inbin
    // the keys of the threshold bin: max_key - key in [q << kShift, (q + 1) << kShift)
    const uint32_t top = max_key - (((uint32_t)(kBinsA - 1) - b1) << kShift);
    // (a lane holds one only rarely: the distance of its nearest key below `top` decides with
    //  two instructions per key whether the lane looks at its keys one by one)
    uint32_t nearest = 0xffffffffu;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) nearest = min(nearest, top - key[j]);
    if (nearest < (1u << kShift)) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (top - key[j] < (1u << kShift)) {
                const uint32_t at = atomicAdd(&sh.ncand, 1u);
                if (at < (uint32_t)kNearCand) sh.cand[at] = key[j];
            }
        }
    }
    __syncthreads();
    // every wavefront ranks the candidates by itself: lane l holds candidate l and counts the
    // candidates above it and not below it
    const uint32_t c = lane < (int)inbin ? sh.cand[lane] : 0u;
    uint32_t gt = 0u, ge = 0u;
    for (uint32_t j = 0; j < inbin; ++j) {
        const uint32_t cj = (uint32_t)__builtin_amdgcn_readlane((int)c, (int)j);
        gt += cj > c ? 1u : 0u;
        ge += cj >= c ? 1u : 0u;
    }
    const uint64_t at_threshold = __ballot(lane < (int)inbin && gt < remaining && remaining <= ge);
    const int lt = at_threshold ? __builtin_ctzll(at_threshold) : 0;
    T = (uint32_t)__builtin_amdgcn_readlane((int)c, lt);
    const uint32_t gt_t = (uint32_t)__builtin_amdgcn_readlane((int)gt, lt);
    need = remaining - gt_t;
    if (n_equal) *n_equal = (uint32_t)__builtin_amdgcn_readlane((int)ge, lt) - gt_t;
}

// The same selection over a list of `count` keys in LDS; lane `tid` owns the entries
// [lo, hi).  Requires 1 <= k <= count.
// `zero_low` low bits of every key are zero; digits made only of such bits are skipped.
template <typename SH>
__device__ __forceinline__ void list_select_largest(const uint32_t* keys, uint32_t lo, uint32_t hi,
                                                    uint32_t k, int zero_low, SH& sh,
                                                    int& phase, uint32_t& T, uint32_t& need) {
    const int tid = threadIdx.x;
    uint32_t* histA = sh.hist;
    uint32_t* histB = sh.hist + kBinsA;
    uint32_t* histC = sh.hist + kBinsA + kBinsB;
    for (int b = tid; b < kBinsA + kBinsB + kBinsC; b += kSelThreads) sh.hist[b] = 0u;
    __syncthreads();
    for (uint32_t e = lo; e < hi; ++e) hist_add_callers(histA, keys[e] >> 20);
    __syncthreads();
    uint32_t b1, above, inbin;
    find_bin<kBinsA / kSelThreads>(histA, k, sh, phase, b1, above, inbin);
    uint32_t remaining = k - above;
    if (zero_low >= 20) {   // the first digit is the whole key
        T = b1 << 20;
        need = remaining;
        return;
    }
    for (uint32_t e = lo; e < hi; ++e) {
        const uint32_t kk = keys[e];
        if ((kk >> 20) == b1) hist_add_callers(histB, (kk >> 10) & 1023u);
    }
    __syncthreads();
    uint32_t b2;
    find_bin<1>(histB, remaining, sh, phase, b2, above, inbin);
    remaining -= above;
    const uint32_t hi2 = (b1 << 10) | b2;
    if (zero_low >= 10) {
        T = hi2 << 10;
        need = remaining;
        return;
    }
    for (uint32_t e = lo; e < hi; ++e) {
        const uint32_t kk = keys[e];
        if ((kk >> 10) == hi2) hist_add_callers(histC, kk & 1023u);
    }
    __syncthreads();
    uint32_t b3;
    find_bin<1>(histC, remaining, sh, phase, b3, above, inbin);
    T = (hi2 << 10) | b3;
    need = remaining - above;
}

// Put the wave-uniform value `val` into lane `LANE` of `dst` (one v_writelane).
template <int LANE>
__device__ __forceinline__ void write_lane(int& dst, uint32_t val) {
#if SEL_WRITELANE
    // The scalar source may have just been written by a vector instruction (a ballot): this
    // chip wants two wait states between that write and a vector instruction reading the
    // register, which the compiler inserts for its own code but not inside an asm statement.
    const int sval = __builtin_amdgcn_readfirstlane((int)val);
    asm("s_nop 1\n\tv_writelane_b32 %0, %1, %2" : "+v"(dst) : "s"(sval), "n"(LANE));
#else
    if ((threadIdx.x & 63) == LANE) dst = (int)val;
#endif
}

template <int J, int ITEMS>
struct TileCount {
    __device__ static __forceinline__ void eq_gt(const uint32_t (&key)[ITEMS], uint32_t T, int& mine) {
        const uint32_t ce = (uint32_t)__popcll(__ballot(key[J] == T));
        const uint32_t cg = (uint32_t)__popcll(__ballot(key[J] > T));
        write_lane<J>(mine, ce | (cg << 16));
        if constexpr (J + 1 < ITEMS) TileCount<J + 1, ITEMS>::eq_gt(key, T, mine);
    }
    __device__ static __forceinline__ void ge(const uint32_t (&key)[ITEMS], uint32_t T, int& mine) {
        write_lane<J>(mine, (uint32_t)__popcll(__ballot(key[J] >= T)));
        if constexpr (J + 1 < ITEMS) TileCount<J + 1, ITEMS>::ge(key, T, mine);
    }
    __device__ static __forceinline__ void flag(uint32_t flags, int& mine) {
        write_lane<J>(mine, (uint32_t)__popcll(__ballot((flags >> J) & 1u)));
        if constexpr (J + 1 < ITEMS) TileCount<J + 1, ITEMS>::flag(flags, mine);
    }
};

// For every (slot, wavefront) tile: how many keys are equal to T (low 16 bits) and larger
// than T (high 16 bits); then the exclusive prefix of those over the tiles in index order.
// Lane j of each wavefront returns the prefix of the wavefront's tile in slot j.
template <int ITEMS, typename SH>
__device__ __forceinline__ uint32_t tile_prefix_eq_gt(const uint32_t (&key)[ITEMS], uint32_t T,
                                                      SH& sh, int& phase) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int ntiles = ITEMS * kWaves;
    int mine = 0;
    TileCount<0, ITEMS>::eq_gt(key, T, mine);
    static_assert(ITEMS <= 64, "one lane per slot");
    if (lane < ITEMS) sh.tile[0][lane * kWaves + wave] = (uint32_t)mine;
    __syncthreads();
    const uint32_t t = tid < ntiles ? sh.tile[0][tid] : 0u;
    const uint32_t ex = block_excl_scan(t, sh, phase);
    if (tid < ntiles) sh.tile[0][tid] = ex;
    __syncthreads();
    return lane < ITEMS ? sh.tile[0][lane * kWaves + wave] : 0u;
}

// Same for the single count of keys >= T per tile.
template <int ITEMS, typename SH>
__device__ __forceinline__ uint32_t tile_prefix_ge(const uint32_t (&key)[ITEMS], uint32_t T,
                                                   SH& sh, int& phase) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int ntiles = ITEMS * kWaves;
    int mine = 0;
    TileCount<0, ITEMS>::ge(key, T, mine);
    if (lane < ITEMS) sh.tile[0][lane * kWaves + wave] = (uint32_t)mine;
    __syncthreads();
    const uint32_t t = tid < ntiles ? sh.tile[0][tid] : 0u;
    const uint32_t ex = block_excl_scan(t, sh, phase);
    if (tid < ntiles) sh.tile[0][tid] = ex;
    __syncthreads();
    return lane < ITEMS ? sh.tile[0][lane * kWaves + wave] : 0u;
}

// Same for a single flag per key (bit j of `flags`): tile counts, prefix, lane j holds slot j.
template <int ITEMS, typename SH>
__device__ __forceinline__ uint32_t tile_prefix_flag(uint32_t flags, int which, SH& sh,
                                                     int& phase) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int ntiles = ITEMS * kWaves;
    int mine = 0;
    TileCount<0, ITEMS>::flag(flags, mine);
    if (lane < ITEMS) sh.tile[which][lane * kWaves + wave] = (uint32_t)mine;
    __syncthreads();
    const uint32_t t = tid < ntiles ? sh.tile[which][tid] : 0u;
    const uint32_t ex = block_excl_scan(t, sh, phase);
    if (tid < ntiles) sh.tile[which][tid] = ex;
    __syncthreads();
    return lane < ITEMS ? sh.tile[which][lane * kWaves + wave] : 0u;
}

}  // namespace sel
}  // namespace dip

#endif  // DIP_SELECT_DEVICE_H_
