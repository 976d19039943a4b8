// Device-side pieces of the column-gathered GEMV shared by its kernels: element types (how
// 16 loaded bytes widen to fp32), the row loop that accumulates a workgroup's share of the
// selected rows, and the fixed-order reduction (lane groups -> wavefronts -> workgroups of one
// strip) with its epilogue.
#ifndef DIP_GEMV_DEVICE_H_
#define DIP_GEMV_DEVICE_H_

#include "dip_internal.h"

namespace dip {
namespace gemv {

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
struct Tile {
    static constexpr int EPL = Elem<WT>::kPerLoad;   // elements per load
    static constexpr int RPW = 64 / LPR;             // rows per wavefront step
    static constexpr int SC = LPR * EPL;             // strip columns
    static constexpr int NG = WAVES * RPW;           // lane groups per workgroup
    static constexpr int ROWS_PER_ITER = UNROLL * NG;
    static constexpr int NOUT = NSEG * SC;           // outputs a workgroup owns
};

// Sum of val[t] * row idx[t] over the list positions [kb, ke) for this lane's 16 bytes of
// the strip (both segments of a bundled matrix).  The lists are read at position t - list_base:
// they are either the launch-wide lists in global memory (list_base = 0) or this workgroup's
// share of them in LDS (list_base = kb).  idx == nullptr means rows kb .. ke-1 themselves (a
// dense product).  kb - list_base must be a multiple of 4 and the lists 16-byte aligned.
template <typename WT, int LPR, int WAVES, int UNROLL, int NSEG>
__device__ __forceinline__ void accumulate(const GemvParams& p, const int32_t* idx, const float* val,
                                           int list_base, int kb, int ke, int strip,
                                           float (&acc)[NSEG][Elem<WT>::kPerLoad]) {
    typedef Tile<WT, LPR, WAVES, UNROLL, NSEG> T;
    constexpr int EPL = T::EPL, RPW = T::RPW, SC = T::SC, ROWS_PER_ITER = T::ROWS_PER_ITER;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, l = lane % LPR;
    const int col_raw = strip * SC + l * EPL;
    const bool col_ok = col_raw < p.n_out;
    // lanes past the right edge of a ragged last strip re-read its last 16 bytes; they own no output
    const int col = col_ok ? col_raw : p.n_out - EPL;

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
    // quantised rows: the scale of this lane's codes (all inside one group of 128)
    const int sgroup = col >> 7, sgroups_per_seg = p.n_out >> 7;

    // Every lane group takes UNROLL consecutive selected rows per iteration, so their
    // indices and multipliers arrive as one vector load each.  Full iterations need no
    // predicates; the pairs of the next iteration are requested right after this
    // iteration's weight loads so that their latency hides behind the weights.
    const int gid = wave * RPW + sub;
    const int n_full = (ke - kb) / ROWS_PER_ITER;   // the same for every lane
    const bool ident = idx == nullptr;         // every stored row in order (a dense product)
    int t0 = kb + gid * UNROLL;

    auto fetch_pairs = [&](int t, int (&row)[UNROLL], float (&xv)[UNROLL]) {
        const int q = t - list_base;
        if constexpr (UNROLL % 4 == 0) {
#pragma unroll
            for (int u = 0; u < UNROLL; u += 4) {
                const float4 x4 = *reinterpret_cast<const float4*>(val + q + u);
                int4 r4 = make_int4(t + u, t + u + 1, t + u + 2, t + u + 3);
                if (!ident) r4 = *reinterpret_cast<const int4*>(idx + q + u);
                row[u] = r4.x; row[u + 1] = r4.y; row[u + 2] = r4.z; row[u + 3] = r4.w;
                xv[u] = x4.x; xv[u + 1] = x4.y; xv[u + 2] = x4.z; xv[u + 3] = x4.w;
            }
        } else if constexpr (UNROLL == 2) {
            const float2 x2 = *reinterpret_cast<const float2*>(val + q);
            int2 r2 = make_int2(t, t + 1);
            if (!ident) r2 = *reinterpret_cast<const int2*>(idx + q);
            row[0] = r2.x; row[1] = r2.y;
            xv[0] = x2.x; xv[1] = x2.y;
        } else {
            xv[0] = val[q];
            row[0] = t;
            if (!ident) row[0] = idx[q];
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
                const int e = ident ? t : idx[t - list_base];
                const bool second = e < 0;
                const int r = second ? ~e : e;
                if ((unsigned)r < (unsigned)(second ? p.n_alt : p.n_in)) {
                    row[u] = r;
                    xv[u] = val[t - list_base];
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
}

// Combine the lanes' sums in a fixed order and write the strip's outputs: lane groups of one
// wavefront (xor butterfly), wavefronts through `red` in index order, and -- with G > 1
// workgroups per strip -- the workgroups through p.partial, added in workgroup order by the
// one that draws the last ticket of p.counters[strip]; then the epilogue.
// WRAP: the ticket counter returns to 0 with the last ticket (it must be 0 before the first
// launch only); otherwise it counts up and the caller resets it between launches.
// Returns after the outputs are written; `red` and `s_last` are LDS of the workgroup.
template <typename WT, int LPR, int WAVES, int UNROLL, int NSEG, bool WRAP>
__device__ __forceinline__ void finish(const GemvParams& p, float (&acc)[NSEG][Elem<WT>::kPerLoad],
                                       int strip, int g, int G,
                                       float (&red)[WAVES][NSEG][LPR * Elem<WT>::kPerLoad], int& s_last) {
    typedef Tile<WT, LPR, WAVES, UNROLL, NSEG> T;
    constexpr int EPL = T::EPL, SC = T::SC, NOUT = T::NOUT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, l = lane % LPR;

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
    static_assert(NOUT <= WAVES * 64, "strip wider than the workgroup");
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
            uint32_t prev;
            if constexpr (WRAP) {
                prev = atomicInc(&p.counters[strip], (uint32_t)(G - 1));
            } else {
                prev = __hip_atomic_fetch_add(&p.counters[strip], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            s_last = (prev == (uint32_t)(G - 1));
        }
        __syncthreads();
        if (!s_last) return;
        // the partial sums of all workgroups, up to 32 in flight at a time (one round trip to
        // memory for the usual numbers of workgroups per strip), added in workgroup order
        sum = 0.f;
        if (owner) {
            const float* src0 = p.partial + (size_t)oseg * (size_t)p.n_out + gcol;
            const size_t gstride = (size_t)NSEG * (size_t)p.n_out;
            constexpr int kInFlight = 32;
            for (int g0 = 0; g0 < G; g0 += kInFlight) {
                float part[kInFlight];
#pragma unroll
                for (int j = 0; j < kInFlight; ++j) {
                    part[j] = 0.f;
                    if (g0 + j < G)      // (uniform: G is the same for every lane)
                        part[j] = __hip_atomic_load(src0 + (size_t)(g0 + j) * gstride, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int j = 0; j < kInFlight; ++j)
                    if (g0 + j < G) sum += part[j];
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

}  // namespace gemv
}  // namespace dip

#endif  // DIP_GEMV_DEVICE_H_
