// Gathered products that run their own selection (Sec. 4 composed with Alg. 1 steps 1-2 and 4):
//     head   s = score(v, c) ; m = topK(s, k)              -- every workgroup, redundantly
//     body   sum_{i in m} W[:, i] v_i over this workgroup's share of m
//     tail   fixed-order reduction, SwiGLU epilogue for the bundled up/gate pair
// One launch instead of two.  A stand-alone selection is a single workgroup on one compute
// unit while 255 idle, and the product behind it cannot start before its index list is in
// memory; here every workgroup of the product derives the list itself from the (small,
// L2-resident) input vector and keeps only the part that falls into its own row share, in LDS.
//
// Workgroups are 1024 lanes (16 wavefronts), one per compute unit, so the redundant head is
// paid once per compute unit.  Lane `tid` owns features tid, tid+1024, ...: a 64-bit wave
// ballot over one slot is two words of the mask and (slot, wavefront) tiles in ascending
// order are the features in index order (lowest index wins ties; ascending list).
//
// Cache-aware scores without a division per key.  Eq. 10 of Sec. 5.2 is s = fl(p / M) with
// p = |v| for resident columns, fl(|v| * gamma) otherwise, and M = ||v||_inf.  q -> fl(q / M)
// is monotone, so the k-th largest score is T_s = fl(T_p / M) with T_p the k-th largest p, and
//     { s > T_s }  = { p >= P_hi },  P_hi = the smallest float with fl(P_hi / M) >  T_s
//     { s == T_s } = { P_lo <= p < P_hi },  P_lo = the smallest float with fl(P_lo / M) >= T_s.
// The selection therefore runs on the bit patterns of p, and only P_lo and P_hi need
// divisions: 64 candidates around T_p, one per lane, settle them in one step (a bisection
// over all floats covers the case that the window is too small, e.g. denormal scores).  The
// selected set is then exactly the top-K of the rounded scores with lowest-index ties -- the
// set the stand-alone selection kernel and the oracle produce from the emitted s.
#include "dip_gemv_device.h"
#include "dip_select_device.h"

namespace dip {
namespace {

using namespace sel;
using namespace gemv;

constexpr int kFusedWaves = kSelThreads / 64;   // 16

struct HeadShared {
    uint32_t hist[kBinsA + kBinsB + kBinsC];
    uint32_t cw[kMaxWords];          // residency words used for scoring
    uint32_t tile[2][kMaxTiles];
    uint32_t wave_tot[2][kWaves];
    float wave_max[kWaves];
    uint32_t bcast[4];
    uint32_t cand[kNearCand];        // keys of the threshold bin
    uint32_t ncand;
};
constexpr int kHeadHistWords = kBinsA + kBinsB + kBinsC;

// Exclusive running sums of the per-tile counts over the tiles in index order: lane j of each
// wavefront passes the count of the wavefront's tile in slot j and gets the sum over the tiles
// before it; `total` is the sum over all tiles.
template <int ITEMS>
__device__ __forceinline__ uint32_t tile_scan(uint32_t cnt, HeadShared& sh, int& phase, uint32_t& total) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int ntiles = ITEMS * kWaves;
    if (lane < ITEMS) sh.tile[0][lane * kWaves + wave] = cnt;
    __syncthreads();
    const uint32_t t = tid < ntiles ? sh.tile[0][tid] : 0u;
    const uint32_t ex = block_excl_scan(t, sh, phase);
    if (tid < ntiles) sh.tile[0][tid] = ex;
    if (tid == ntiles - 1) sh.bcast[3] = ex + t;
    __syncthreads();
    total = sh.bcast[3];
    return lane < ITEMS ? sh.tile[0][lane * kWaves + wave] : 0u;
}

// Smallest float bit pattern c in [lo, hi] with pred(fl(c / M)) true, where pred is monotone
// (false ... false true ... true) and true at hi.  Every lane runs the same bisection.
template <bool STRICT>
__device__ __forceinline__ uint32_t bisect_quotient(uint32_t lo, uint32_t hi, float M, float Ts) {
    while (lo < hi) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        const float q = __fdiv_rn(__uint_as_float(mid), M);
        const bool ok = STRICT ? (q > Ts) : (q >= Ts);
        if (ok) hi = mid; else lo = mid + 1u;
    }
    return lo;
}

// The keys that tie with the k-th largest score, and those above it (Eq. 10 without a division
// per key, see the head of this file): Tk is the k-th largest key (bits(p) << 1), M = ||v||_inf.
// Leaves K_lo, K_hi alone when M is 0 (all scores are 0).
__device__ __forceinline__ void score_window(uint32_t Tk, float M, int lane, uint32_t& K_lo, uint32_t& K_hi) {
    if (!(M > 0.f)) return;
    const uint32_t Tb = Tk >> 1;
    const float Ts = __fdiv_rn(__uint_as_float(Tb), M);
    constexpr uint32_t kInf = 0x7f800000u;
    const int64_t cand = (int64_t)Tb + lane - 31;
    const uint32_t cb = cand < 0 ? 0u : (cand > (int64_t)kInf ? kInf : (uint32_t)cand);
    const float qc = __fdiv_rn(__uint_as_float(cb), M);
    const uint64_t ge = __ballot(qc >= Ts), gt = __ballot(qc > Ts);   // lane 31 is T_p: in ge
    const uint32_t c0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cb);
    uint32_t Plo, Phi;
    if ((ge & 1ull) && c0 > 0u) {
        Plo = bisect_quotient<false>(0u, c0, M, Ts);
    } else {
        // (ge is never empty for finite inputs: lane 31 holds T_p itself)
        Plo = ge ? (uint32_t)__builtin_amdgcn_readlane((int)cb, __builtin_ctzll(ge)) : Tb;
    }
    if (gt == 0ull) {
        Phi = bisect_quotient<true>(Tb + 1u, kInf, M, Ts);
    } else {
        Phi = (uint32_t)__builtin_amdgcn_readlane((int)cb, __builtin_ctzll(gt));
    }
    K_lo = Plo << 1;
    K_hi = Phi << 1;
}

// Per-tile counts of the keys in [K_lo, K_hi) (low 16 bits) and >= K_hi (high 16 bits), their
// exclusive prefix over the tiles in index order (lane j of each wavefront returns the prefix
// of the wavefront's tile in slot j), and the totals.
template <int ITEMS>
__device__ __forceinline__ uint32_t tile_prefix_window(const uint32_t (&key)[ITEMS], uint32_t K_lo, uint32_t K_hi,
                                                       HeadShared& sh, int& phase, uint32_t& totals) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int ntiles = ITEMS * kWaves;
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const uint32_t ce = (uint32_t)__popcll(__ballot(key[j] >= K_lo && key[j] < K_hi));
        const uint32_t cg = (uint32_t)__popcll(__ballot(key[j] >= K_hi));
        mine = lane == j ? (ce | (cg << 16)) : mine;
    }
    __syncthreads();       // (the table may still be read by a slower wavefront)
    if (lane < ITEMS) sh.tile[0][lane * kWaves + wave] = mine;
    __syncthreads();
    const uint32_t t = tid < ntiles ? sh.tile[0][tid] : 0u;
    const uint32_t ex = block_excl_scan(t, sh, phase);
    if (tid < ntiles) sh.tile[0][tid] = ex;
    if (tid == kSelThreads - 1) sh.bcast[3] = ex + t;
    __syncthreads();
    totals = sh.bcast[3];
    return lane < ITEMS ? sh.tile[0][lane * kWaves + wave] : 0u;
}

// One slot of the selection `key >= T` into the workgroup's share of the list; slots whose
// bit of `active` is clear cost one scalar test.  (A template recursion rather than a loop:
// the lane numbers must be constants.)
template <int J, int ITEMS>
struct ListGe {
    __device__ static __forceinline__ void run(const uint32_t (&key)[ITEMS], const float (&v)[ITEMS], uint32_t T,
                                               int pre, uint64_t active, int kb, int ke, int32_t* l_idx,
                                               float* l_val) {
        if ((active >> J) & 1ull) {     // wave-uniform
            const bool mine = key[J] >= T;
            const uint64_t bs = __ballot(mine);
            const uint32_t at = (uint32_t)__builtin_amdgcn_readlane(pre, J) + lanes_below(bs) - (uint32_t)kb;
            // (at < ke - kb also rejects the places before kb, which wrap around)
            if (mine && at < (uint32_t)(ke - kb)) {
                l_idx[at & (kFusedListCap - 1)] = J * kSelThreads + (int)threadIdx.x;
                l_val[at & (kFusedListCap - 1)] = v[J];
            }
        }
        if constexpr (J + 1 < ITEMS) ListGe<J + 1, ITEMS>::run(key, v, T, pre, active, kb, ke, l_idx, l_val);
    }
};

// Mask words of the selection, slot by slot (a template recursion: the lane numbers are constants).
template <int J, int ITEMS>
struct MaskWords {
    __device__ static __forceinline__ void run(const uint32_t (&key)[ITEMS], uint32_t K_lo, uint32_t K_hi, bool fast,
                                               uint32_t take, uint32_t eq_seen, int next, int G, int& my_word) {
        // `next`: the next slot of this workgroup (g, g + G, ...; uniform, and no division)
        if (J == next) {
            slot(key, K_lo, K_hi, fast, take, eq_seen, my_word);
            next += G;
        }
        if constexpr (J + 1 < ITEMS) MaskWords<J + 1, ITEMS>::run(key, K_lo, K_hi, fast, take, eq_seen, next, G, my_word);
    }
    __device__ static __forceinline__ void slot(const uint32_t (&key)[ITEMS], uint32_t K_lo, uint32_t K_hi, bool fast,
                                                uint32_t take, uint32_t eq_seen, int& my_word) {
        bool mine;
        if (fast) {
            mine = key[J] >= K_lo;
        } else {
            // ties at the threshold: the `take` lowest indices among them are selected
            mine = key[J] >= K_hi;
            const bool tie = key[J] >= K_lo && !mine;
            const uint64_t be = __ballot(tie);
            const uint32_t eq_before = (uint32_t)__builtin_amdgcn_readlane((int)eq_seen, J) & 0xffffu;
            mine = mine || (tie && eq_before + lanes_below(be) < take);
        }
        const uint64_t bs = __ballot(mine);
        write_lane<(2 * J) & 63>(my_word, (uint32_t)bs);
        write_lane<(2 * J + 1) & 63>(my_word, (uint32_t)(bs >> 32));
    }
};

template <typename WT, int LPR, int NSEG>
struct FusedShared {
    typedef Tile<WT, LPR, kFusedWaves, 4, NSEG> T;
    int32_t l_idx[kFusedListCap];    // this workgroup's share of the index list ...
    float l_val[kFusedListCap];      // ... and of the multipliers
    union {
        HeadShared head;                              // selection
        float red[kFusedWaves][NSEG][T::SC];          // reduction across wavefronts
    } u;
    uint32_t mwords[kMaxWords];      // mask words on their way out (the workgroup that writes them)
    int s_last;
};

template <typename WT, int LPR, int NSEG, int ITEMS>
__global__ __launch_bounds__(kSelThreads) void fused_kernel(FusedParams fp) {
    constexpr int WAVES = kFusedWaves, UNROLL = 4;
    typedef Tile<WT, LPR, WAVES, UNROLL, NSEG> T;
    __shared__ __align__(16) FusedShared<WT, LPR, NSEG> sh;
    HeadShared& hs = sh.u.head;
    const GemvParams& p = fp.g;
    const FusedSelect& q = fp.s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int strip = blockIdx.x;
    const int g = blockIdx.y, G = gridDim.y;
    const int kb = min(p.k, g * p.rows_per_split);   // rows_per_split is a multiple of 8, <= kFusedListCap
    const int ke = min(p.k, kb + p.rows_per_split);
    // the workgroup that also writes the launch-wide outputs of the selection
    // ... of the scores (workgroup (0, 0)) and of the mask words (the workgroups of strip 0 take
    // the slots in turn: slot j belongs to the workgroup with g == j mod G)
    const bool scribe = strip == 0 && g == 0;
    const bool mask_scribe = strip == 0 && q.mask_out != nullptr;
    const int nwords = (q.n + 31) >> 5;
    int phase = 0;

    // ---- head: Alg. 1 steps 1-2 on q.v --------------------------------------------------------
    float v[ITEMS];
    uint32_t key[ITEMS];
    const int mine_n = q.n > tid ? (q.n - tid - 1) / kSelThreads + 1 : 0;
    const uint32_t valid = mine_n >= 32 ? 0xffffffffu : (1u << mine_n) - 1u;
    {
        const float* vp = q.v + tid;
        const int full = q.n >> 10;     // slots that lie inside the vector entirely (wave-uniform)
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (j < full) {
                v[j] = vp[j * kSelThreads];
            } else {
                const uint32_t i = (uint32_t)(j * kSelThreads + tid);
                v[j] = 0.f;
                if (i < (uint32_t)q.n) v[j] = q.v[i & (DIP_MAX_N - 1)];
            }
        }
    }
    static_assert(kHeadHistWords % (2 * kSelThreads) == 0, "the histograms are cleared in 8-byte pieces");
#pragma unroll
    for (int b = 0; b < kHeadHistWords / (2 * kSelThreads); ++b)
        reinterpret_cast<uint2*>(hs.hist)[b * kSelThreads + tid] = make_uint2(0u, 0u);
    hs.cw[tid] = (q.score_bits && tid < nwords) ? q.score_bits[tid] : 0u;
    {
        // ||v||_inf: the denominator of Eq. 10, and the anchor of the selection's histogram
        float vmax = 0.f;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) vmax = fmaxf(vmax, fabsf(v[j]));
        // (fmaxf drops a NaN operand: non-finite inputs leave M finite or infinite, never NaN)
        vmax = wave_max_nonneg(vmax);
        if (lane == 0) hs.wave_max[wave] = vmax;
    }
    __syncthreads();
    static_assert(kWaves == 16, "one wavefront maximum per lane of a 16-lane row");
    const float M = row_max_nonneg(hs.wave_max[lane & (kWaves - 1)]);

    // p = |v| for resident columns, fl(|v| * gamma) for the others (plain DIP: p = |v|); p <= M
    if (q.score_bits) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const float a = fabsf(v[j]);
            const uint32_t c = (hs.cw[j * (kSelThreads / 32) + (tid >> 5)] >> (tid & 31)) & 1u;
            key[j] = __float_as_uint(c ? a : __fmul_rn(a, q.gamma)) << 1;
        }
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) key[j] = __float_as_uint(fabsf(v[j])) << 1;
    }

    uint32_t Tk, need;
    block_select_largest_near_max<ITEMS>(key, __float_as_uint(M) << 1, (uint32_t)p.k, hs, phase, Tk, need);

    // keys in [K_lo, K_hi) tie at the k-th largest score, keys >= K_hi lie above it
    uint32_t K_lo = Tk, K_hi = Tk + 1u;
    if (q.score_bits) score_window(Tk, M, lane, K_lo, K_hi);

    // ---- this workgroup's share of the list ---------------------------------------------------
    // Counts of the keys >= K_lo per (slot, wavefront) tile and their running sums in index
    // order.  If exactly k keys reach K_lo, no tie is split at the threshold (the usual case):
    // the selection is key >= K_lo and a selected key's place in the list is the number of such
    // keys before it.  Only the tiles whose selected keys reach into [kb, ke) are visited: lane j
    // of a wavefront holds count and running sum of its tile in slot j, and a ballot over "my
    // tile overlaps the share" is a scalar bit mask that steers the unrolled loop with no vector
    // work for the tiles that do not.
    int cnt = 0;
    TileCount<0, ITEMS>::ge(key, K_lo, cnt);
    uint32_t n_ge;
    const uint32_t pre_ge = tile_scan<ITEMS>((uint32_t)cnt, hs, phase, n_ge);
    const bool fast = n_ge == (uint32_t)p.k;
    if (fast) {
        const bool overlap = lane < ITEMS && pre_ge < (uint32_t)ke && pre_ge + (uint32_t)cnt > (uint32_t)kb;
        const uint64_t active = __ballot(overlap);
        ListGe<0, ITEMS>::run(key, v, K_lo, (int)pre_ge, active, kb, ke, sh.l_idx, sh.l_val);
    } else {
        uint32_t totals;
        const int pre = (int)tile_prefix_window<ITEMS>(key, K_lo, K_hi, hs, phase, totals);
        const uint32_t n_gt = totals >> 16;
        const uint32_t take = (uint32_t)p.k > n_gt ? (uint32_t)p.k - n_gt : 0u;   // ties that are selected
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint32_t packed = (uint32_t)__builtin_amdgcn_readlane(pre, j);
            const uint32_t eq_before = packed & 0xffffu, gt_before = packed >> 16;
            const bool above = key[j] >= K_hi;
            const bool tie = key[j] >= K_lo && !above;
            const uint64_t be = __ballot(tie);
            // ties at the threshold: the `take` lowest indices among them are selected
            const bool mine = above || (tie && eq_before + lanes_below(be) < take);
            const uint64_t bs = __ballot(mine);
            const uint32_t pos = gt_before + min(eq_before, take) + lanes_below(bs);
            if (mine && pos >= (uint32_t)kb && pos < (uint32_t)ke) {
                sh.l_idx[(pos - kb) & (kFusedListCap - 1)] = j * kSelThreads + tid;
                sh.l_val[(pos - kb) & (kFusedListCap - 1)] = v[j];
            }
        }
    }

    // ---- launch-wide outputs of the selection (mask words, index list, scores): off the hot path
    const bool list_idx = q.idx_out && strip == 0;   // the workgroups of strip 0 cover all of [0, k)
    if (list_idx) {
        __syncthreads();
        for (int t = tid; t < ke - kb; t += kSelThreads) q.idx_out[kb + t] = sh.l_idx[t];
    }
    if (mask_scribe) {
        uint32_t take = 0u, eq_seen = 0u;
        if (!fast) {
            // recount: how many ties are selected, and how many ties precede each tile
            uint32_t totals;
            const int pre = (int)tile_prefix_window<ITEMS>(key, K_lo, K_hi, hs, phase, totals);
            take = (uint32_t)p.k > (totals >> 16) ? (uint32_t)p.k - (totals >> 16) : 0u;
            eq_seen = (uint32_t)pre;
        }
        // A wave ballot over slot j is two words of the mask: lane 2j keeps the low word and
        // lane 2j+1 the high word, and the words go to LDS once after the loop, to memory one
        // per lane behind the barrier below.  (A workgroup barrier waits for the stores issued
        // before it: stores from inside the loop would hold this workgroup back by
        // microseconds, and with it the launch, which ends with its slowest workgroup.)
        int my_word = 0;
        MaskWords<0, ITEMS>::run(key, K_lo, K_hi, fast, take, eq_seen, g, G, my_word);
        if (lane < 2 * ITEMS)
            sh.mwords[((lane >> 1) * (kSelThreads / 32) + wave * 2 + (lane & 1)) & (kMaxWords - 1)] = (uint32_t)my_word;
    }
    if (scribe && q.s_out) {
        // the scores themselves, for stage-wise comparison: Eq. 10 in its stated operation order
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const float pj = __uint_as_float(key[j] >> 1);
            const float s = q.score_bits ? (M > 0.f ? __fdiv_rn(pj, M) : 0.f) : pj;
            if ((valid >> j) & 1u) q.s_out[j * kSelThreads + tid] = s;
        }
    }
    __syncthreads();   // the list is complete; the selection's LDS may be reused
    if (mask_scribe) {
        // the 32 words of this workgroup's slots g, g + G, ...: 32 lanes per slot
        const int slot = g + (tid >> 5) * G, w = slot * (kSelThreads / 32) + (tid & 31);
        if (slot < ITEMS && w < nwords) q.mask_out[w] = sh.mwords[w & (kMaxWords - 1)];
    }

    // ---- body and tail: Alg. 1 step 4 on this workgroup's share ---------------------------------
    float acc[NSEG][T::EPL];
    accumulate<WT, LPR, WAVES, UNROLL, NSEG>(p, sh.l_idx, sh.l_val, kb, kb, ke, strip, acc);
    finish<WT, LPR, WAVES, UNROLL, NSEG, true>(p, acc, strip, g, G, sh.u.red, sh.s_last);
}

// ---- launch ---------------------------------------------------------------------------------
template <typename WT, int LPR, int NSEG, int ITEMS>
hipError_t launch_k(const FusedParams& fp, int ksplit, hipStream_t stream, int pk) {
    typedef Tile<WT, LPR, kFusedWaves, 4, NSEG> T;
    if constexpr (T::NOUT <= kSelThreads) {
        const int strips = (fp.g.n_out + T::SC - 1) / T::SC;
        return launch_timed(fused_kernel<WT, LPR, NSEG, ITEMS>, dim3(strips, ksplit), dim3(kSelThreads), stream, pk, fp);
    } else {
        return hipErrorInvalidConfiguration;
    }
}

template <typename WT, int LPR, int NSEG>
hipError_t launch_items(const FusedParams& fp, int ksplit, hipStream_t stream, int pk) {
    const int items = (fp.s.n + kSelThreads - 1) / kSelThreads;
    if constexpr (NSEG == 2) {
        // the input of the up/gate product is d_model long
        if (items <= 2) return launch_k<WT, LPR, NSEG, 2>(fp, ksplit, stream, pk);
        if (items <= 3) return launch_k<WT, LPR, NSEG, 3>(fp, ksplit, stream, pk);
        if (items <= 4) return launch_k<WT, LPR, NSEG, 4>(fp, ksplit, stream, pk);
        if (items <= 5) return launch_k<WT, LPR, NSEG, 5>(fp, ksplit, stream, pk);
        if (items <= 6) return launch_k<WT, LPR, NSEG, 6>(fp, ksplit, stream, pk);
        if (items <= 8) return launch_k<WT, LPR, NSEG, 8>(fp, ksplit, stream, pk);
        return hipErrorInvalidConfiguration;
    } else {
        if (items <= 2) return launch_k<WT, LPR, NSEG, 2>(fp, ksplit, stream, pk);
        if (items <= 4) return launch_k<WT, LPR, NSEG, 4>(fp, ksplit, stream, pk);
        if (items <= 6) return launch_k<WT, LPR, NSEG, 6>(fp, ksplit, stream, pk);
        if (items <= 8) return launch_k<WT, LPR, NSEG, 8>(fp, ksplit, stream, pk);
        if (items <= 11) return launch_k<WT, LPR, NSEG, 11>(fp, ksplit, stream, pk);
        if (items <= 14) return launch_k<WT, LPR, NSEG, 14>(fp, ksplit, stream, pk);
        if (items <= 18) return launch_k<WT, LPR, NSEG, 18>(fp, ksplit, stream, pk);
        if (items <= 24) return launch_k<WT, LPR, NSEG, 24>(fp, ksplit, stream, pk);
        return launch_k<WT, LPR, NSEG, 32>(fp, ksplit, stream, pk);
    }
}

template <typename WT, int NSEG>
hipError_t launch_lpr(const FusedParams& fp, const GemvShape& s, hipStream_t stream, int pk) {
    switch (s.lpr) {
        case 16: return launch_items<WT, 16, NSEG>(fp, s.ksplit, stream, pk);
        case 32: return launch_items<WT, 32, NSEG>(fp, s.ksplit, stream, pk);
        case 64: return launch_items<WT, 64, NSEG>(fp, s.ksplit, stream, pk);
    }
    return hipErrorInvalidConfiguration;
}


#if DIP_FUSED_NSEG == 1 && DIP_FUSED_DTYPE == 0
// ---- row selections of a small batch --------------------------------------------------------
// One workgroup per row runs the head above on that row -- keys without a division, one
// histogram pass, the exact-tie window -- and leaves the row's mask words (and the bit pattern
// of max |v|, which the matrix-core product scales by).  No lists: the union kernel builds
// them from the masks of all rows.
struct RowsShared {
    HeadShared head;
    uint32_t mwords[kMaxWords];
    uint32_t wave_cnt[kWaves];
};

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void rows_select_kernel(SelectParams p) {
    __shared__ __align__(16) RowsShared sh;
    HeadShared& hs = sh.head;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwords = (p.n + 31) >> 5;
    const float* vrow = p.v + (size_t)blockIdx.x * p.v_row_stride;
    uint32_t* mrow = p.mask_out + (size_t)blockIdx.x * p.words_row_stride;
    int phase = 0;

    float v[ITEMS];
    uint32_t key[ITEMS];
    {
        const float* vp = vrow + tid;
        const int full = p.n >> 10;     // slots that lie inside the vector entirely (wave-uniform)
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (j < full) {
                v[j] = vp[j * kSelThreads];
            } else {
                const uint32_t i = (uint32_t)(j * kSelThreads + tid);
                v[j] = 0.f;
                if (i < (uint32_t)p.n) v[j] = vrow[i & (DIP_MAX_N - 1)];
            }
        }
    }
#pragma unroll
    for (int b = 0; b < kHeadHistWords / (2 * kSelThreads); ++b)
        reinterpret_cast<uint2*>(hs.hist)[b * kSelThreads + tid] = make_uint2(0u, 0u);
    hs.cw[tid] = (p.score_bits && tid < nwords) ? p.score_bits[tid] : 0u;
    {
        float vmax = 0.f;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) vmax = fmaxf(vmax, fabsf(v[j]));
        vmax = wave_max_nonneg(vmax);
        if (lane == 0) hs.wave_max[wave] = vmax;
    }
    __syncthreads();
    const float M = row_max_nonneg(hs.wave_max[lane & (kWaves - 1)]);
    if (p.rowmax_out && tid == 0) p.rowmax_out[blockIdx.x] = __float_as_uint(M);
    if (p.score_bits) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const float a = fabsf(v[j]);
            const uint32_t c = (hs.cw[j * (kSelThreads / 32) + (tid >> 5)] >> (tid & 31)) & 1u;
            key[j] = __float_as_uint(c ? a : __fmul_rn(a, p.gamma)) << 1;
        }
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) key[j] = __float_as_uint(fabsf(v[j])) << 1;
    }
    uint32_t Tk, need;
    block_select_largest_near_max<ITEMS>(key, __float_as_uint(M) << 1, (uint32_t)p.k, hs, phase, Tk, need);
    uint32_t K_lo = Tk, K_hi = Tk + 1u;
    if (p.score_bits) score_window(Tk, M, lane, K_lo, K_hi);

    // how many keys reach K_lo: exactly k means no tie is split at the threshold
    uint32_t n_wave = 0u;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) n_wave += (uint32_t)__popcll(__ballot(key[j] >= K_lo));
    if (lane == 0) sh.wave_cnt[wave] = n_wave;
    __syncthreads();
    uint32_t n_ge = 0u;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) n_ge += sh.wave_cnt[w];
    const bool fast = n_ge == (uint32_t)p.k;
    uint32_t take = 0u, eq_seen = 0u;
    if (!fast) {
        uint32_t totals;
        const int pre = (int)tile_prefix_window<ITEMS>(key, K_lo, K_hi, hs, phase, totals);
        take = (uint32_t)p.k > (totals >> 16) ? (uint32_t)p.k - (totals >> 16) : 0u;
        eq_seen = (uint32_t)pre;
    }
    int my_word = 0;
    MaskWords<0, ITEMS>::run(key, K_lo, K_hi, fast, take, eq_seen, 0, 1, my_word);
    if (lane < 2 * ITEMS)
        sh.mwords[((lane >> 1) * (kSelThreads / 32) + wave * 2 + (lane & 1)) & (kMaxWords - 1)] = (uint32_t)my_word;
    __syncthreads();
    if (tid < nwords) mrow[tid] = sh.mwords[tid];
}

template <int ITEMS>
hipError_t launch_rows_items(const SelectParams& p, hipStream_t stream, int pk) {
    return launch_timed(rows_select_kernel<ITEMS>, dim3(p.rows), dim3(kSelThreads), stream, pk, p);
}
#endif

#ifndef DIP_FUSED_NSEG
#error "compile with -DDIP_FUSED_NSEG=1 or 2 and -DDIP_FUSED_DTYPE=0, 1 or 2"
#endif

}  // namespace

#define DIP_CAT3(a, b, c) a##b##_##c
#define DIP_FUSED_NAME(n, d) DIP_CAT3(launch_fused_, n, d)

// One translation unit per (segments, weight type): the instantiations compile in parallel.
hipError_t DIP_FUSED_NAME(DIP_FUSED_NSEG, DIP_FUSED_DTYPE)(const FusedParams& fp, const GemvShape& s,
                                                           hipStream_t stream, int pk) {
#if DIP_FUSED_DTYPE == 0
    return launch_lpr<float, DIP_FUSED_NSEG>(fp, s, stream, pk);
#elif DIP_FUSED_DTYPE == 1
    return launch_lpr<uint16_t, DIP_FUSED_NSEG>(fp, s, stream, pk);
#else
    return launch_lpr<q4n_t, DIP_FUSED_NSEG>(fp, s, stream, pk);
#endif
}


#if DIP_FUSED_NSEG == 1 && DIP_FUSED_DTYPE == 0
hipError_t launch_select_rows(const SelectParams& p, hipStream_t stream, int pk) {
    if (!p.v || !p.mask_out || p.rows < 1 || p.n < 1 || p.n > DIP_MAX_N || p.k < 1 || p.k > p.n)
        return hipErrorInvalidValue;
    const int items = (p.n + kSelThreads - 1) / kSelThreads;
    if (items <= 2) return launch_rows_items<2>(p, stream, pk);
    if (items <= 4) return launch_rows_items<4>(p, stream, pk);
    if (items <= 6) return launch_rows_items<6>(p, stream, pk);
    if (items <= 8) return launch_rows_items<8>(p, stream, pk);
    if (items <= 11) return launch_rows_items<11>(p, stream, pk);
    if (items <= 14) return launch_rows_items<14>(p, stream, pk);
    if (items <= 18) return launch_rows_items<18>(p, stream, pk);
    if (items <= 24) return launch_rows_items<24>(p, stream, pk);
    return launch_rows_items<32>(p, stream, pk);
}
#endif

}  // namespace dip
