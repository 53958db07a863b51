// Scoring kernel: per (step, metric) cross-rank median and MAD by selection,
// robust z, exceedance, multi-signal combine and 8-GPU node scores
// (Section 4.2 peer-relative evaluation and multi-signal rule; Section 7.1
// 8-GPU nodes).
//
// Persistent workgroups: each takes a contiguous run of steps and scores them
// column after column.  For each of a step's M columns it
//   1. holds the column in registers (float4 per lane per row, loaded once from
//      HBM, coalesced, rank-contiguous; the next column is loaded row by row
//      while the current one is scored) -- a column is never read again;
//   2. finds the two middle order statistics by counting: a bracket (taken from
//      the previous step of the same metric, else from a sample of the column)
//      is counted into an LDS histogram of order-preserving integer keys, a
//      scan locates the bucket(s) holding the wanted ranks, a second pass
//      gathers that bucket's few values into LDS where they are ranked exactly;
//      a bracket that misses, or a bucket that is too full (ties), falls back
//      to wider or narrower ranges until the answer is exact;
//   3. gets the MAD from the same histogram (pairs of bucket edges around the
//      median bound the wanted distances; one pass counts and gathers), or by a
//      second selection on |x - med| when that does not apply;
//   4. computes z, the exceedance bits and the node scores from the registers.
// After the M columns the per-rank mask bytes, anomaly bits and node outputs
// are written.  HBM traffic is the 4 bytes per sample read plus ~1.8 bytes per
// rank and step of outputs.
#include <type_traits>

#include "gd_internal.h"

// This file is compiled twice, side by side: as it is (every launch without the
// optional z output, and the entry points) and, through score_z.hip, with
// GD_SCORE_WANT_Z = 1 (the launches that write z as well).
#ifndef GD_SCORE_WANT_Z
#define GD_SCORE_WANT_Z 0
#endif

namespace {

constexpr bool WANT_Z_HERE = GD_SCORE_WANT_Z != 0;

constexpr int WAVE = 64;
constexpr int CAND_CAP = 512;  // values ranked exactly in LDS per selection

__device__ __forceinline__ uint32_t rfl(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Order-preserving map fp32 -> u32 and back.
__device__ __forceinline__ uint32_t key_of(float f) {
    uint32_t b = __float_as_uint(f);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float float_of_key(uint32_t k) {
    uint32_t b = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(b);
}

template <int NT, int LOG_NB, int MAX_NODES>
struct Shared {
    static constexpr int NB = 1 << LOG_NB;
    // dlo, hist, dhi are one array of 64 + NB + 64 counters for the hinted counting pass
    // (keys under / inside / over the bracket); the other passes use hist alone.
    uint32_t dlo[64];
    uint32_t hist[NB];
    uint32_t dhi[64];
    uint32_t pref[NB + 4];     // exclusive prefix sums of hist (pref[NB] = total), for the MAD shortcut
    uint32_t cand[CAND_CAP + 4];   // 16-byte aligned; read four at a time when ranking
    uint32_t wpart[16];
    uint32_t below, ncand;
    uint32_t nkept;            // hinted MAD: candidates kept after the exact test
    uint32_t wcnt[16];         // hinted MAD: values gathered by each wave
    uint32_t mres[2][4];       // hinted MAD: edge indices found by the search and a found flag (two slots, used in turn)
    uint32_t smin, smax;       // extremes of the sample keys
    uint32_t d1, d2;           // MAD shortcut: distance interval holding the wanted ranks
    uint32_t umax[2];          // largest raw bit pattern of the column (double-buffered)
    uint32_t res[6];           // ba, prefix before ba, bb, prefix through bb, va, vb
    // Per metric, from the previous step scored by this workgroup: the median and how
    // far below / above it the counting histogram reached (hok = the hint is usable).
    float hmed[8], hwl[8], hwh[8], hmad[8];
    uint32_t hok[8];
    uint32_t hfast[8];         // the hinted selection below has not failed for this metric yet
    alignas(8) uint8_t nodeb[MAX_NODES];        // the step's node mask bytes, read eight at a time
    uint64_t ranka[MAX_NODES / 8 > 0 ? MAX_NODES / 8 : 1];     // the step's rank anomaly words (zero between steps)
};

// Cross-lane moves with immediate patterns (DPP): no address registers, nothing
// for the optimiser to hoist out of the column loop.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp0(uint32_t v) {   // lanes without a source read 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_keep(uint32_t v) {   // lanes without a source keep v
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, ROW_MASK, 0xF, false);
}
template <int J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);
    else if constexpr (J == 8) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true);
    else {
        static_assert(J == 4, "lane_xor");
        return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (J << 10));
    }
}
__device__ __forceinline__ float lane_xor1(float v) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_mov_dpp((int)__float_as_uint(v), 0xB1, 0xF, 0xF, true));
}

// Inclusive prefix sum across the wave (lane 63 ends with the total).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    v += dpp0<0x111>(v);          // row_shr:1
    v += dpp0<0x112>(v);          // row_shr:2
    v += dpp0<0x114>(v);          // row_shr:4
    v += dpp0<0x118>(v);          // row_shr:8
    v += dpp0<0x142, 0xA>(v);     // row_bcast:15 into rows 1 and 3
    v += dpp0<0x143, 0xC>(v);     // row_bcast:31 into rows 2 and 3
    return v;
}
// Minimum / maximum over the wave, valid in lane 63.
__device__ __forceinline__ uint32_t wave_min_to_last(uint32_t v) {
    v = min(v, dpp_keep<0x111>(v)); v = min(v, dpp_keep<0x112>(v));
    v = min(v, dpp_keep<0x114>(v)); v = min(v, dpp_keep<0x118>(v));
    v = min(v, dpp_keep<0x142, 0xA>(v)); v = min(v, dpp_keep<0x143, 0xC>(v));
    return v;
}
__device__ __forceinline__ uint32_t wave_max_to_last(uint32_t v) {
    v = max(v, dpp_keep<0x111>(v)); v = max(v, dpp_keep<0x112>(v));
    v = max(v, dpp_keep<0x114>(v)); v = max(v, dpp_keep<0x118>(v));
    v = max(v, dpp_keep<0x142, 0xA>(v)); v = max(v, dpp_keep<0x143, 0xC>(v));
    return v;
}

// Exclusive prefix sum of one value per thread over the workgroup; total in *tot.
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t tid, uint32_t* wpart,
                                                    uint32_t* tot) {
    const uint32_t lane = tid & (WAVE - 1), w = tid >> 6;
    const uint32_t inc = wave_incl_scan(v);
    if (NT == WAVE) {
        *tot = __builtin_amdgcn_readlane((int)inc, WAVE - 1);
        return inc - v;
    }
    if (lane == WAVE - 1) wpart[w] = inc;
    __syncthreads();
    // every wave scans the (at most 16) wave totals itself: one LDS read, a row scan
    uint32_t p = lane < (uint32_t)(NT / WAVE) ? wpart[lane] : 0u;
    p += dpp0<0x111>(p); p += dpp0<0x112>(p); p += dpp0<0x114>(p); p += dpp0<0x118>(p);
    const uint32_t total = __builtin_amdgcn_readlane((int)p, NT / WAVE - 1);
    const uint32_t wu = rfl(w);
    const uint32_t off = wu ? (uint32_t)__builtin_amdgcn_readlane((int)p, (int)(wu - 1)) : 0u;
    *tot = total;
    return off + inc - v;
}

// Values the optimiser cannot see through.  They stop it from keeping one
// pass's per-element temporaries, or values derived from the thread index,
// alive in registers across the whole column loop.
__device__ __forceinline__ uint32_t opaque_s(uint32_t v) {   // wave-uniform
    v = rfl(v);
    asm volatile("" : "+s"(v));
    return v;
}
__device__ __forceinline__ uint32_t opaque_v(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

// Keys of the median selection.  PLAIN: the column has no sign bit set, so the
// raw bits order like the values; otherwise the order-preserving image is used.
template <int ROWS, bool PLAIN>
struct XKeys {
    const float (&v)[ROWS][4];
    __device__ __forceinline__ uint32_t token() const { return opaque_s(31u); }
    __device__ __forceinline__ uint32_t key(float f, uint32_t tok) const {
        if (PLAIN) return __float_as_uint(f);
        // -0 reads as +0; the zero is derived from the opaque token so that the
        // sum is recomputed per pass instead of being kept for all 64 values
        const float g = f + __uint_as_float(tok - 31u);
        const uint32_t b = __float_as_uint(g);
        const uint32_t k = b ^ ((uint32_t)((int32_t)b >> tok) | 0x80000000u);   // tok is an opaque 31
        return g != g ? 0xFFFFFFFFu : k;     // a missing sample (NaN) lies above every value
    }
    __device__ __forceinline__ uint32_t at(int j, int i, uint32_t tok) const { return key(v[j][i], tok); }
    __device__ __forceinline__ float value(uint32_t k) const {
        return PLAIN ? __uint_as_float(k) : float_of_key(k);
    }
};

// Keys of the MAD selection: the bits of |x - med| (non-negative floats order as integers).
template <int ROWS>
struct DKeys {
    const float (&v)[ROWS][4];
    float med;
    __device__ __forceinline__ uint32_t token() const { return opaque_s(__float_as_uint(med)); }
    __device__ __forceinline__ uint32_t key(float f, uint32_t tok) const {
        return __float_as_uint(fabsf(f - __uint_as_float(tok)));     // tok is an opaque med
    }
    __device__ __forceinline__ uint32_t at(int j, int i, uint32_t tok) const { return key(v[j][i], tok); }
    __device__ __forceinline__ float value(uint32_t k) const { return __uint_as_float(k); }
};

// LDS protocol of the selection code.  Between uses the work area is kept in a
// known state, so that no phase has to clear it behind two barriers of its own:
// sh.hist all zero (locate() clears what it reads), sh.below = sh.ncand = 0,
// sh.smin = ~0, sh.smax = 0, sh.d1 = 0, sh.d2 = ~0.  Thread 0 restores a scalar
// after the barrier that follows its last read, and at least one more barrier
// precedes the next atomic update of it.

// After a counting pass: find the buckets holding ranks ka and kb (relative to
// everything; `sh.below` keys lie under the histogram's range, or none if
// !USE_BELOW).  Clears the histogram, leaves the results in sh.res, returns the
// below count and whether both ranks fall inside the histogram.  Ends with a barrier.
template <int NT, int LOG_NB, bool WRITE_PREF, bool USE_BELOW, typename SH>
__device__ __forceinline__ bool locate(SH& sh, uint32_t tid, uint32_t ka, uint32_t kb,
                                       uint32_t* below_out) {
    constexpr int BPT = (1 << LOG_NB) / NT;
    uint32_t loc[BPT], s = 0;
#pragma unroll
    for (int q = 0; q < BPT; ++q) { loc[q] = sh.hist[tid * BPT + q]; s += loc[q]; }
#pragma unroll
    for (int q = 0; q < BPT; ++q) sh.hist[tid * BPT + q] = 0;
    uint32_t total;
    const uint32_t excl = block_excl_scan<NT>(s, tid, sh.wpart, &total);
    const uint32_t below = USE_BELOW ? sh.below : 0u;
    const uint32_t ra = ka - below, rb = kb - below;   // wrap when not bracketed
    if (WRITE_PREF) {
        uint32_t p = excl;
#pragma unroll
        for (int q = 0; q < BPT; ++q) { sh.pref[tid * BPT + q] = p; p += loc[q]; }
        if (tid == NT - 1) sh.pref[1 << LOG_NB] = p;
    }
    if (ra - excl < s) {
        uint32_t p = excl;
        bool done = false;
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            if (!done && ra - p < loc[q]) { sh.res[0] = tid * BPT + q; sh.res[1] = p; done = true; }
            p += loc[q];
        }
    }
    if (rb - excl < s) {
        uint32_t p = excl;
        bool done = false;
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            if (!done && rb - p < loc[q]) { sh.res[2] = tid * BPT + q; sh.res[3] = p + loc[q]; done = true; }
            p += loc[q];
        }
    }
    __syncthreads();
    if (USE_BELOW && tid == 0) sh.below = 0;
    *below_out = rfl(below);
    return rfl(ka >= below && rb < total) != 0;
}

// Exact ranking of the cnt gathered candidates in sh.cand (ties broken by
// position): the candidates of rank wa and wb go to sh.res[4] and sh.res[5].
// Each wave takes every (NT/64)-th candidate; its lanes split the comparisons
// and the wave counts the lanes that answered yes.  Ends with a barrier.
template <int NT, typename SH>
__device__ __forceinline__ void rank_candidates(SH& sh, uint32_t tid, uint32_t cnt, uint32_t wa,
                                                uint32_t wb, const uint32_t* list = nullptr) {
    if (list == nullptr) list = sh.cand;
    const uint32_t lane = tid & (WAVE - 1), w = rfl(tid >> 6);
    if (cnt <= (uint32_t)WAVE) {
        // one LDS read per wave: lane j holds candidate j, candidate i is read from lane i
        // (read whatever the slot holds: the load then does not wait for cnt)
        const uint32_t cj = list[lane];
        for (uint32_t i = w; i < cnt; i += NT / WAVE) {
            const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)cj, (int)i);
            const uint32_t r = (uint32_t)__popcll(__ballot(lane < cnt && (cj < c || (cj == c && lane < i))));
            if (lane == 0) {
                if (r == wa) sh.res[4] = c;
                if (r == wb) sh.res[5] = c;
            }
        }
    } else {
        for (uint32_t i = w; i < cnt; i += NT / WAVE) {
            const uint32_t c = list[i];
            uint32_t r = 0;                      // wave-uniform: candidates ordered before candidate i
            for (uint32_t j0 = 0; j0 < cnt; j0 += WAVE) {
                const uint32_t j = j0 + lane;
                const uint32_t cj = j < cnt ? list[j] : 0xFFFFFFFFu;
                r += (uint32_t)__popcll(__ballot(j < cnt && (cj < c || (cj == c && j < i))));
            }
            if (lane == 0) {
                if (r == wa) sh.res[4] = c;
                if (r == wb) sh.res[5] = c;
            }
        }
    }
    __syncthreads();
}

template <int LOG_NB>
__device__ __forceinline__ int shift_for(uint32_t span) {
    const int width = 32 - __builtin_clz(span | 1u);
    return width > LOG_NB ? width - LOG_NB : 0;            // (span >> shift) < NB
}

// Exact selection of the order statistics k0 <= k1 (0-based, k1 - k0 <= 1) of
// the ROWS*4 keys per thread held in registers (padding keys compare above all
// real ones).
//   1. One sampled key per thread (skey, svalid; n of them valid) goes into a histogram over the
//      sample's own range; the sample ranks n/2 -+ 2*sqrt(n) give a bracket
//      [lo, hi] that holds the wanted ranks with high probability and only a
//      small share of the column.
//   2. Counting pass: keys inside the bracket go into the LDS histogram, keys
//      below it are counted.  If the wanted ranks are not inside, count again
//      over the full range.
//   3. The buckets holding the ranks are gathered into LDS and ranked exactly,
//      or, when they are crowded (ties), the range is narrowed to the bucket.
//
// WIDE: bracket the sample ranks n/2 -+ 0.34*n instead, so that the histogram also
// covers the values around median -+ MAD, and keep its prefix sums in sh.pref.  If
// the first counting pass settles the selection, *hist_lo / *hist_shift describe
// that histogram (bucket b holds keys hist_lo + b*2^shift ...) and the function
// returns true; the MAD shortcut then reads the prefix sums.
//
// umax_slot (with a handed-in bracket only): the first counting pass also finds the
// largest raw bit pattern of the column and leaves it in *umax_out.  Should it carry
// a sign bit or be a NaN's, the raw bits were no valid keys or the ranks asked for
// not the right ones: the selection stops after clearing its work area and the
// caller starts over.
template <int NT, int ROWS, int LOG_NB, bool WIDE, typename SH, typename Keys>
__device__ __forceinline__ bool block_select(SH& sh, const Keys& keys, uint32_t skey, bool svalid,
                                             uint32_t n, uint32_t k0, uint32_t k1, uint32_t* out0,
                                             uint32_t* out1, uint32_t* hist_lo = nullptr,
                                             uint32_t* hist_hi = nullptr, int* hist_shift = nullptr,
                                             bool hinted = false, uint32_t hint_lo = 0,
                                             uint32_t hint_hi = 0, uint32_t* umax_slot = nullptr,
                                             uint32_t* umax_out = nullptr) {
    constexpr int NB = 1 << LOG_NB;
    constexpr int BPT = NB / NT;
    static_assert(BPT >= 1 && (BPT % 4 == 0 || BPT < 4), "bucket split");
    uint32_t lo = hint_lo, hi = hint_hi;
    // Bracket from the sample (skipped while a bracket handed in by the caller holds).
    auto sample_bracket = [&]() {
        const uint32_t tid = opaque_v(threadIdx.x), lane = tid & (WAVE - 1);
        const uint32_t mn = wave_min_to_last(svalid ? skey : 0xFFFFFFFFu);
        const uint32_t mx = wave_max_to_last(svalid ? skey : 0u);
        if (lane == WAVE - 1) { atomicMin(&sh.smin, mn); atomicMax(&sh.smax, mx); }
        __syncthreads();
        const uint32_t smin = rfl(sh.smin), smax = rfl(sh.smax);
        const uint32_t sspan = smax - smin;                 // smin <= smax: some sample is valid
        const int sshift = shift_for<LOG_NB>(sspan);
        if (svalid) atomicAdd(&sh.hist[(skey - smin) >> sshift], 1u);
        __syncthreads();
        if (tid == 0) { sh.smin = 0xFFFFFFFFu; sh.smax = 0; }
        // n valid samples: the ranks n/2 -+ (2*sqrt(n) + 1) bracket the column's median
        const uint32_t delta = WIDE ? (n * 87u) >> 8 : (uint32_t)(2.0f * __builtin_sqrtf((float)n)) + 1u;
        const uint32_t half = n / 2;
        const uint32_t ra = half > delta ? half - 1 - delta : 0u;
        const uint32_t rb = min(n - 1, half + delta);
        uint32_t unused;
        const bool both = locate<NT, LOG_NB, false, false>(sh, tid, ra, rb, &unused);
        const uint32_t ba = rfl(sh.res[0]), bb = rfl(sh.res[2]);
        lo = ra == 0 ? 0u : smin + (ba << sshift);
        const uint64_t hend = (uint64_t)smin + ((uint64_t)(bb + 1) << sshift) - 1;
        hi = rb == n - 1 ? 0xFFFFFFFFu : (hend > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)hend);
        // Fewer samples than n went in when some were missing values: a sample rank
        // beyond them was not located, and the bracket is then left open.
        if (!both) { lo = 0; hi = 0xFFFFFFFFu; }
    };
    if (!hinted) sample_bracket();
    // mode 0: both statistics together; 1: k0 alone; 2: k1 alone (after a split)
    int mode = 0, rounds = 0;
    uint32_t ka = k0, kb = k1, v0 = 0, v1 = 0;
    for (;;) {
        ++rounds;
        const uint32_t span = hi - lo;
        const int shift = shift_for<LOG_NB>(span);
        // a fresh copy of the thread index per round: values derived from it (bucket
        // slots, LDS addresses) are then recomputed instead of living in registers
        const uint32_t tid = opaque_v(threadIdx.x);
        const uint32_t lane = tid & (WAVE - 1);
        // counting pass
        uint32_t nbelow = 0;   // per lane; summed over the wave after the pass
        const bool with_umax = umax_slot != nullptr && rounds == 1;
        uint32_t um = 0;
        {
            const uint32_t tok = keys.token();
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t kk = keys.at(j, i, tok);
                    nbelow += kk < lo ? 1u : 0u;
                    const uint32_t t = kk - lo;
                    if (t <= span) atomicAdd(&sh.hist[t >> shift], 1u);
                }
                if (umax_slot != nullptr) {     // (padding lanes never take this route: FULL tilings only)
                    // the row's registers are made opaque here, or the maxima, which do not
                    // depend on the round, are all computed ahead of the loop -- after
                    // waiting for the whole column instead of row by row
                    float(&row)[4] = const_cast<float(&)[4]>(keys.v[j]);
                    asm volatile("" : "+v"(row[0]), "+v"(row[1]), "+v"(row[2]), "+v"(row[3]));
                    um = max(um, max(keys.at(j, 0, tok), keys.at(j, 1, tok)));
                    um = max(um, max(keys.at(j, 2, tok), keys.at(j, 3, tok)));
                    asm volatile("" : "+v"(um));
                }
                asm volatile("" : "+v"(nbelow));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        nbelow = wave_incl_scan(nbelow);
        if (with_umax) um = wave_max_to_last(um);
        if (lane == WAVE - 1) {
            if (nbelow) atomicAdd(&sh.below, nbelow);
            if (with_umax) atomicMax(umax_slot, um);
        }
        __syncthreads();
        if (with_umax) {
            const uint32_t umax = rfl(*umax_slot);
            *umax_out = umax;
            if (umax > 0x7F800000u) {
                uint32_t unused;
                (void)locate<NT, LOG_NB, false, true>(sh, tid, ka, kb, &unused);   // clears the work area
                *out0 = 0; *out1 = 0;
                return false;
            }
        }
        uint32_t below;
        const bool bracketed = locate<NT, LOG_NB, WIDE, true>(sh, tid, ka, kb, &below);
        if (!bracketed) {
            // the bracket missed: a handed-in one is replaced by the sample's, the
            // sample's by the full key range
            if (hinted) { hinted = false; sample_bracket(); }
            else { lo = 0; hi = 0xFFFFFFFFu; __syncthreads(); }
            continue;
        }
        const uint32_t ba = rfl(sh.res[0]), pa = rfl(sh.res[1]);
        const uint32_t bb = rfl(sh.res[2]), pb = rfl(sh.res[3]);
        uint32_t va, vb;
        if (shift == 0) {               // one key per bucket: the bucket is the answer
            va = lo + ba; vb = lo + bb;
        } else if (pb - pa <= (uint32_t)CAND_CAP) {
            // gather the values of buckets ba..bb and rank them exactly
            const uint32_t clo = lo + (ba << shift);
            const uint64_t cend = (uint64_t)lo + ((uint64_t)(bb + 1) << shift) - 1;
            const uint32_t chi = cend > hi ? hi : (uint32_t)cend;
            const uint32_t cspan = chi - clo;
            const uint32_t tok = keys.token();
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
                // one test per register row (hits are rare): the smallest offset decides
                uint32_t off[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) off[i] = keys.at(j, i, tok) - clo;
                if (min(min(off[0], off[1]), min(off[2], off[3])) <= cspan) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (off[i] <= cspan) {
                            uint32_t pos = atomicAdd(&sh.ncand, 1u);
                            if (pos < (uint32_t)CAND_CAP) sh.cand[pos] = off[i] + clo;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            const uint32_t cnt = min(sh.ncand, (uint32_t)CAND_CAP);
            const uint32_t wa = ka - below - pa, wb = kb - below - pa;
            rank_candidates<NT>(sh, tid, cnt, wa, wb);
            if (tid == 0) sh.ncand = 0;
            va = rfl(sh.res[4]); vb = rfl(sh.res[5]);
        } else {
            // crowded (ties): look inside bucket ba; if the two statistics sit in
            // different crowded buckets, finish k0 first, then k1 on its own
            if (ba != bb) { mode = 1; kb = ka; }
            const uint32_t nlo = lo + (ba << shift);
            const uint64_t nend = (uint64_t)nlo + ((uint64_t)1 << shift) - 1;
            hi = nend > hi ? hi : (uint32_t)nend;
            lo = nlo;
            __syncthreads();
            continue;
        }
        if (mode == 0) {
            v0 = va; v1 = vb;
            if (WIDE && hist_lo) { *hist_lo = lo; *hist_hi = hi; *hist_shift = shift; }
            break;
        }
        if (mode == 1) {
            v0 = va; mode = 2; ka = kb = k1; lo = 0; hi = 0xFFFFFFFFu;
            __syncthreads();
            continue;
        }
        v1 = va;
        break;
    }
    *out0 = v0;
    *out1 = v1;
    return rounds == 1 && mode == 0;
}

// MAD shortcut for a sign-free column whose median selection left a histogram of
// the raw bits over [lo, hi] (2^shift keys per bucket, prefix sums in sh.pref)
// that reaches well beyond median -+ MAD.  From the prefix sums alone the threads
// find a distance interval [d1, d2] that must hold the wanted order statistics of
// |x - med| (see below); one pass then counts the distances below d1 exactly and
// gathers those inside the interval (a few dozen) for exact ranking.  The pass
// also verifies the interval; false is returned, and the caller selects in the
// ordinary way, if the histogram did not reach far enough or the check fails.
template <int NT, int ROWS, int LOG_NB, typename SH>
__device__ __forceinline__ bool mad_from_histogram(SH& sh, const float (&v)[ROWS][4], float med,
                                                   uint32_t lo, uint32_t hi, int shift, uint32_t k0,
                                                   uint32_t k1, float mad_hint, uint32_t* out0,
                                                   uint32_t* out1) {
    constexpr int NB = 1 << LOG_NB;
    const uint32_t tid = opaque_v(threadIdx.x), lane = tid & (WAVE - 1);
    const float xlo = __uint_as_float(lo), xhi = __uint_as_float(hi);
    const float dmax = fminf(med - xlo, xhi - med);
    if (!(dmax > 0.0f) || shift < 2) return false;
    // With the previous step's MAD of this metric as a hint only the edges whose
    // distance from the median is within an eighth of it are paired (a couple of
    // hundred, one per thread); if they do not enclose the ranks, all edges are.
    uint32_t d1 = 0, d2 = 0;
    auto grid = [&](bool near_hint_only) -> bool {
        // Pairs of bucket edges (eL, eR) with value(eL) <= med < value(eR): the set
        // S = {eL <= key < eR} is counted exactly by the prefix sums, every value
        // outside S is at least min(dL, dR) away from med and every value inside at
        // most max(dL, dR) (subtraction is monotone), where dL = med - value(eL) and
        // dR = value(eR) - med.  So |S| <= k0 makes min(dL, dR) a valid d1 and
        // |S| >= k1 + 1 makes max(dL, dR) a valid d2.  Each thread pairs its own
        // buckets' edges with the two edges that nearly mirror them.
        constexpr int BPT = NB / NT;
        uint32_t c1 = 0, c2 = 0xFFFFFFFFu;
        auto edge = [&](uint32_t b) { return __uint_as_float(lo + (b << shift)); };
        const uint32_t bmax = (hi - lo) >> shift;     // last bucket whose lower edge is <= hi
        auto eval = [&](uint32_t bL, uint32_t bR) {
            if (bL < bR && bR <= bmax) {
                const float xl = edge(bL), xr = edge(bR);
                if (xl <= med && xr > med) {
                    const float dl = med - xl, dr = xr - med;
                    const uint32_t cntS = sh.pref[bR] - sh.pref[bL];
                    if (cntS <= k0) c1 = max(c1, __float_as_uint(fminf(dl, dr)));
                    if (cntS >= k1 + 1) c2 = min(c2, __float_as_uint(fmaxf(dl, dr)));
                }
            }
        };
        auto pair_edge = [&](uint32_t b) {
            const float xe = edge(b);
            if (xe > med) {            // a right edge: mirror it to the left
                const uint32_t km = __float_as_uint(med - (xe - med));
                if (km >= lo && km <= hi) {
                    const uint32_t bl = (km - lo) >> shift;
                    eval(bl, b);
                    eval(bl + 1, b);
                }
            } else {                   // a left edge: mirror it to the right
                const uint32_t km = __float_as_uint(med + (med - xe));
                if (km >= lo && km <= hi) {
                    const uint32_t br = (km - lo) >> shift;
                    eval(b, br);
                    eval(b, br + 1);
                }
            }
        };
        if (near_hint_only) {
            // the edges within an eighth of the hint around med - hint and med + hint,
            // dealt out one per thread
            const float wl0 = med - 1.125f * mad_hint, wl1 = med - 0.875f * mad_hint;
            const float wr0 = med + 0.875f * mad_hint, wr1 = med + 1.125f * mad_hint;
            const uint32_t klo = __float_as_uint(fmaxf(wl0, xlo)), khi = __float_as_uint(fminf(wr1, xhi));
            const uint32_t bl0 = (klo - lo) >> shift, bl1 = (__float_as_uint(fmaxf(wl1, xlo)) - lo) >> shift;
            const uint32_t br0 = (__float_as_uint(fminf(wr0, xhi)) - lo) >> shift, br1 = (khi - lo) >> shift;
            // (at most NB edges a side whatever the hint and the bounds hold -- infinities, NaN
            // patterns, a window turned inside out: the loop below stays short, and eval()
            // checks every bucket index against bmax before it reads a prefix sum)
            const uint32_t nl = min(bl1 - bl0 + 1, (uint32_t)NB), nr = min(br1 - br0 + 1, (uint32_t)NB);
            for (uint32_t e = tid; e < nl + nr; e += NT) pair_edge(e < nl ? bl0 + e : br0 + (e - nl));
        } else {
#pragma unroll
            for (int q = 0; q < BPT; ++q) pair_edge(tid * BPT + q);
        }
        c1 = wave_max_to_last(c1);
        c2 = wave_min_to_last(c2);
        if (lane == WAVE - 1) { atomicMax(&sh.d1, c1); atomicMin(&sh.d2, c2); }
        __syncthreads();
        d1 = rfl(sh.d1); d2 = rfl(sh.d2);
        if (d2 != 0xFFFFFFFFu && d2 >= d1) return true;
        __syncthreads();                     // everyone has read d1, d2
        if (tid == 0) { sh.d1 = 0; sh.d2 = 0xFFFFFFFFu; }
        return false;
    };
    bool found = mad_hint > 0.0f && grid(true);
    if (!found) {
        if (mad_hint > 0.0f) __syncthreads();    // the reset above precedes the next proposals
        found = grid(false);
    }
    if (!found) return false;
    // exact pass: count |x - med| below d1, gather those in [d1, d2]
    const uint32_t span = d2 - d1;
    uint32_t nbelow = 0;
    {
        const uint32_t tok = opaque_s(__float_as_uint(med));
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            uint32_t off[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t kk = __float_as_uint(fabsf(v[j][i] - __uint_as_float(tok)));
                nbelow += kk < d1 ? 1u : 0u;
                off[i] = kk - d1;
            }
            // one test per register row (hits are rare): the smallest offset decides
            if (min(min(off[0], off[1]), min(off[2], off[3])) <= span) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (off[i] <= span) {
                        uint32_t pos = atomicAdd(&sh.ncand, 1u);
                        if (pos < (uint32_t)CAND_CAP) sh.cand[pos] = off[i] + d1;
                    }
                }
            }
            asm volatile("" : "+v"(nbelow));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    nbelow = wave_incl_scan(nbelow);
    if (lane == WAVE - 1 && nbelow) atomicAdd(&sh.below, nbelow);
    __syncthreads();
    if (tid == 0) { sh.d1 = 0; sh.d2 = 0xFFFFFFFFu; }
    const uint32_t below = rfl(sh.below), cnt = rfl(sh.ncand);
    if (cnt > (uint32_t)CAND_CAP || below > k0 || k1 >= below + cnt) {
        __syncthreads();                     // everyone has read the counters
        if (tid == 0) { sh.below = 0; sh.ncand = 0; }
        return false;
    }
    const uint32_t wa = k0 - below, wb = k1 - below;
    rank_candidates<NT>(sh, tid, cnt, wa, wb);
    if (tid == 0) { sh.below = 0; sh.ncand = 0; }
    *out0 = rfl(sh.res[4]);
    *out1 = rfl(sh.res[5]);
    return true;
}

// Hinted selection: median and MAD of a sign-free column whose predecessor (the same
// metric one step earlier) left a bracket [hint_lo, hint_hi] around its median that
// reaches past median -+ MAD, and its MAD.  Three passes over the registers instead of
// the four of the general route, each with less work per value:
//   1. counting: every key adds one to a counter -- its bucket inside the bracket, or a
//      lane-private word under / over it (no test, no branch: the bucket index is clamped);
//      the pass also finds the largest bit pattern of the column.
//   2. the median's bucket(s) are gathered and ranked as in the general route.
//   3. MAD: with the exact median, the threads search the prefix sums for the right edge
//      e and the left edge f with  #[f, e) <= k0 < #[f', e + 1) -- the wanted distances
//      end inside the few buckets around those edges.  One pass gathers the values whose
//      distance lies between the distances of those buckets' edges (a few dozen); the
//      values strictly between the two bucket ranges are known from the prefix sums, so
//      nothing is counted per value.  The gathered values are then classified exactly:
//        inner: all values of the buckets between the ranges, distance <= DI;
//        outer: all values beyond the ranges, distance >= DO;
//      a gathered value with distance < DI counts with the inner ones, those in
//      [DI, DO] are ranked, and the wanted ranks must fall among them -- else the
//      function reports failure and the caller selects in the general way.
// found = 2: median and MAD; 1: the median alone (MAD by the general route); 0: neither
// (the work area is at rest in every case, the column is never modified).  umax is
// valid in every case.
struct HintedResult {
    int found;                  // 2: median and MAD, 1: median alone, 0: neither
    uint32_t umax;              // largest raw bit pattern of the column
    uint32_t m0, m1;            // the two middle keys
    uint32_t q0, q1;            // the two middle distances (bit patterns)
};

template <int NT, int ROWS, int LOG_NB, typename SH>
__device__ __forceinline__ HintedResult hinted_select(SH& sh, const float (&v)[ROWS][4], uint32_t hint_lo,
                                                      uint32_t hint_hi, float mad_hint, uint32_t k0,
                                                      uint32_t k1, uint32_t* umax_slot, uint32_t par) {
    HintedResult out = {0, 0u, 0u, 0u, 0u, 0u};
    constexpr int NB = 1 << LOG_NB;
    constexpr uint32_t KEY_LIMIT = 0x7D000000u;    // beyond it the signed bucket arithmetic could wrap
    const uint32_t span0 = hint_hi - hint_lo;
    const int shift = shift_for<LOG_NB>(span0);
    // the bracket is widened to all NB buckets (less than twice the hint's span; the caller
    // has checked that this stays below KEY_LIMIT) and starts on a bucket boundary
    constexpr uint32_t bmax = (uint32_t)NB - 1u;
    const uint32_t lo = hint_lo & ~((1u << shift) - 1u);
    const uint32_t hi = lo + ((uint32_t)NB << shift) - 1u;
    uint32_t* const cnt = sh.dlo;                  // 64 + NB + 64 counters
    // ---- pass 1: count.  lo is a multiple of 2^shift, so a key's bucket is its own bits
    // shifted down, less lo's: the clamp works on the shifted bits and the subtraction
    // moves into the counter's address (three vector instructions per value).
    {
        const uint32_t tid = opaque_v(threadIdx.x), lane = tid & (WAVE - 1);
        const int ql = (int)(lo >> shift);                       // (below 2^30: shift < 2 gives the result up anyway)
        const int cl = ql - 1 - (int)lane, ch = ql + NB + (int)lane;
        const uint32_t kb = opaque_s((uint32_t)(64 - ql) * 4u);  // counter 64 is bucket 0 (bytes, mod 2^32)
        const uint32_t sh_s = opaque_s((uint32_t)shift);
        uint32_t um = 0;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            float(&row)[4] = const_cast<float(&)[4]>(v[j]);
            asm volatile("" : "+v"(row[0]), "+v"(row[1]), "+v"(row[2]), "+v"(row[3]));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = (int)(__float_as_uint(row[i]) >> sh_s);
                int c;          // q clamped to [cl, ch] (cl < ch): the median of the three
                asm("v_med3_i32 %0, %1, %2, %3" : "=v"(c) : "v"(q), "v"(cl), "v"(ch));
                // counter c - ql + 64, in [63 - lane, 64 + NB + lane]
                atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(cnt) + (((uint32_t)c << 2) + kb)), 1u);
            }
            um = max(max(um, __float_as_uint(row[0])), __float_as_uint(row[1]));
            um = max(max(um, __float_as_uint(row[2])), __float_as_uint(row[3]));
            asm volatile("" : "+v"(um));
            __builtin_amdgcn_sched_barrier(0);
        }
        um = wave_max_to_last(um);
        if (lane == WAVE - 1) atomicMax(umax_slot, um);
    }
    __syncthreads();
    const uint32_t tid = opaque_v(threadIdx.x), lane = tid & (WAVE - 1), w = rfl(tid >> 6);
    const uint32_t umax = rfl(*umax_slot);
    out.umax = umax;
    // the lane-private words: everything under the bracket is `below`
    if (w == 0) {
        uint32_t d = cnt[lane];
        cnt[lane] = 0;
        d = wave_incl_scan(d);
        if (lane == WAVE - 1) sh.below = d;
    }
    if (w == (NT > WAVE ? 1u : 0u)) cnt[64 + NB + lane] = 0;
    uint32_t below;
    const bool bracketed = locate<NT, LOG_NB, true, true>(sh, tid, k0, k1, &below);
    if (umax > KEY_LIMIT || !bracketed || shift < 2) return out;
    const uint32_t ba = rfl(sh.res[0]), pa = rfl(sh.res[1]);
    const uint32_t bb = rfl(sh.res[2]), pb = rfl(sh.res[3]);
    if (pb - pa > (uint32_t)CAND_CAP / 2 || bb - ba > 1u) return out;      // crowded (ties): the general route narrows
    // ---- pass 2: the median's bucket(s)
    {
        const uint32_t clo = lo + (ba << shift);
        const uint32_t cspan = ((bb - ba + 1u) << shift) - 1u;
        const uint32_t tok = opaque_s(clo);
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            uint32_t off[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) off[i] = __float_as_uint(v[j][i]) - tok;
            if (min(min(off[0], off[1]), min(off[2], off[3])) <= cspan) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (off[i] <= cspan) {
                        uint32_t pos = atomicAdd(&sh.ncand, 1u);
                        if (pos < (uint32_t)CAND_CAP) sh.cand[pos] = off[i] + tok;
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();
    {
        const uint32_t ncnt = min(sh.ncand, (uint32_t)CAND_CAP);
        rank_candidates<NT>(sh, tid, ncnt, k0 - below - pa, k1 - below - pa);
        if (tid == 0) sh.ncand = 0;
    }
    const uint32_t s0 = rfl(sh.res[4]), s1 = rfl(sh.res[5]);
    out.m0 = s0; out.m1 = s1;
    out.found = 1;
    const float med = 0.5f * (__uint_as_float(s0) + __uint_as_float(s1));
    if (!(mad_hint > 0.0f)) return out;
    // ---- MAD: search the prefix sums.  Candidate c is the right edge e_c (a bucket's lower
    // edge, e_c > bb); its distance from the median mirrored to the left gives the edge
    // f_c, the first one above the mirror point.  F_c = #[f_c, e_c) never decreases with c;
    // the thread that sees F_c <= k0 < F_{c+1} reports e_c, f_c, f_{c+1}.
    auto edge = [&](uint32_t e) { return __uint_as_float(lo + (e << shift)); };
    struct Inner { uint32_t count, f; };                 // count ~0u: not a candidate
    auto inner_count = [&](uint32_t e) -> Inner {
        if (e <= bb || e > bmax + 1u) return Inner{0xFFFFFFFFu, 0u};
        const float d = edge(e) - med;
        const uint32_t kl = __float_as_uint(med - d);
        if (!(d > 0.0f) || kl < lo || kl > hi) return Inner{0xFFFFFFFFu, 0u};
        const uint32_t f = ((kl - lo) >> shift) + 1u;
        return Inner{f <= e ? sh.pref[e] - sh.pref[f] : 0xFFFFFFFFu, f};
    };
    {
        const uint32_t kr = __float_as_uint(med + mad_hint);
        const uint32_t eh = kr >= lo && kr <= hi ? (kr - lo) >> shift : bmax;   // the edge the hint points at
        constexpr int CPT = NT >= 512 ? 1 : 512 / NT;          // candidates per thread: at least 512 in all
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const uint32_t e = eh - (uint32_t)(NT * CPT / 2) + tid * CPT + c;     // (wraps below 0: rejected as > bmax + 1)
            const Inner A = inner_count(e), B = inner_count(e + 1u);
            if (A.count != 0xFFFFFFFFu && B.count != 0xFFFFFFFFu && A.count <= k0 && B.count > k0) {
                sh.mres[par][0] = e; sh.mres[par][1] = A.f; sh.mres[par][2] = B.f; sh.mres[par][3] = 1;
            }
        }
    }
    __syncthreads();
    // (the caller clears the other slot's flag, which every thread read a column ago)
    const uint32_t found = rfl(sh.mres[par][3]);
    const uint32_t e_star = rfl(sh.mres[par][0]), f_star = rfl(sh.mres[par][1]), f_next = rfl(sh.mres[par][2]);
    if (!found) return out;
    // bucket ranges around the edges (one bucket of margin each side)
    const uint32_t Rb0 = e_star - 1u, Rb1 = min(e_star + 1u, bmax);
    const uint32_t Lb1 = f_star, Lb0 = f_next >= 2u ? f_next - 2u : 0u;
    if (Rb0 <= bb || Lb1 >= ba || Lb0 > Lb1) return out;          // ranges reach the median's buckets: general route
    const float dLi = med - edge(Lb1 + 1u), dLo = med - edge(Lb0);
    const float dRi = edge(Rb0) - med, dRo = edge(Rb1 + 1u) - med;
    const float DI = fmaxf(dLi, dRi), DO = fminf(dLo, dRo);
    const float Da = fminf(dLi, dRi), Db = fmaxf(dLo, dRo);
    const uint32_t n_in = rfl(sh.pref[Rb0] - sh.pref[Lb1 + 1u]);
    if (!(Da > 0.0f) || !(DO >= DI)) return out;
    // ---- pass 3: gather the values whose distance from the median lies in [Da, Db].  No
    // round trips: each wave appends to a list of its own inside sh.cand (free at this point),
    // at a position made of a count kept in a scalar register and the lanes' ballot.
    constexpr uint32_t NWAVES = NT / WAVE, SUB = (uint32_t)CAND_CAP / NWAVES;
    {
        const float tokm = __uint_as_float(opaque_s(__float_as_uint(med)));
        const float toka = __uint_as_float(opaque_s(__float_as_uint(Da)));
        const uint32_t wspan = __float_as_uint(Db - Da);
        uint32_t* const mine = sh.cand + w * SUB;
        uint32_t n = 0;                            // (wave-uniform)
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            uint32_t off[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) off[i] = __float_as_uint(fabsf(v[j][i] - tokm) - toka);   // negative: a large pattern
            // one test per register row (hits are rare): the smallest offset decides
            if (__builtin_expect(__ballot(min(min(off[0], off[1]), min(off[2], off[3])) <= wspan) != 0ull, 0)) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool hit = off[i] <= wspan;
                    const uint64_t hm = __ballot(hit);
                    if (hm != 0ull) {
                        const uint32_t pos = n + __builtin_amdgcn_mbcnt_hi((uint32_t)(hm >> 32),
                                                                           __builtin_amdgcn_mbcnt_lo((uint32_t)hm, 0u));
                        if (hit && pos < SUB) mine[pos] = __float_as_uint(v[j][i]);
                        n += (uint32_t)__popcll(hm);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (lane == 0) sh.wcnt[w] = n;
    }
    __syncthreads();
    // classify the gathered values exactly; those kept go to a second list, which takes the
    // place of the prefix sums (read for the last time above).  A wave whose list overflowed
    // fails the selection for everybody.
    static_assert(NB + 4 >= CAND_CAP + 4, "the prefix array holds the second list");
    uint32_t* const kept_list = sh.pref;
    const bool fits = __ballot(lane < NWAVES && sh.wcnt[lane < NWAVES ? lane : 0u] > SUB) == 0ull;
    if (fits) {
        uint32_t nlt = 0;
#pragma unroll
        for (int q = 0; q < (CAND_CAP + NT - 1) / NT; ++q) {
            const uint32_t slot = tid + q * NT;
            if (slot < (uint32_t)CAND_CAP && slot % SUB < sh.wcnt[slot / SUB]) {
                const uint32_t x = sh.cand[slot];
                const uint32_t b = (x - lo) >> shift;          // (values outside the bracket: b is huge)
                const bool in_l = x >= lo && b >= Lb0 && b <= Lb1, in_r = x >= lo && b >= Rb0 && b <= Rb1;
                const float d = fabsf(__uint_as_float(x) - med);
                if (in_l || in_r) {
                    if (d < DI) nlt += 1u;
                    else if (d <= DO) kept_list[atomicAdd(&sh.nkept, 1u)] = __float_as_uint(d);
                }
            }
        }
        if (nlt) atomicAdd(&sh.below, nlt);
    }
    __syncthreads();
    const uint32_t c_in = n_in + rfl(sh.below), kept = rfl(sh.nkept);
    const bool ok = fits && c_in <= k0 && k1 < c_in + kept;
    if (ok) rank_candidates<NT>(sh, tid, kept, k0 - c_in, k1 - c_in, kept_list);
    else __syncthreads();
    if (tid == 0) {          // (a zero made here: kept in registers for the whole kernel it ends up spilled)
        const uint32_t zero = opaque_v(0u);
        sh.nkept = zero; sh.below = zero;
    }
    if (!ok) return out;
    out.q0 = rfl(sh.res[4]);
    out.q1 = rfl(sh.res[5]);
    out.found = 2;
    return out;
}

// Hints for a column that has no predecessor to take them from (the first step of a
// workgroup's run): median and quartiles of a sample -- the four values of register row 0
// of every thread, which cover the whole rank range -- read off a histogram over the
// sample's own range.  Half the interquartile distance stands in for the MAD (equal to it
// for a symmetric spread).  Like all hints they are only trusted as far as the counting
// pass of the hinted selection confirms them, so raw bit patterns serve as keys whatever
// the column holds.  Thread 0 writes the hints of metric m; ends with a barrier, the work
// area at rest.
template <int NT, int LOG_NB, typename SH>
__device__ __forceinline__ void sample_hints(SH& sh, const float (&row)[4], uint32_t m) {
    constexpr int BPT = (1 << LOG_NB) / NT;
    constexpr uint32_t n = 4u * NT;
    const uint32_t tid = opaque_v(threadIdx.x), lane = tid & (WAVE - 1);
    uint32_t k[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) k[i] = __float_as_uint(row[i]);
    const uint32_t mn = wave_min_to_last(min(min(k[0], k[1]), min(k[2], k[3])));
    const uint32_t mx = wave_max_to_last(max(max(k[0], k[1]), max(k[2], k[3])));
    if (lane == WAVE - 1) { atomicMin(&sh.smin, mn); atomicMax(&sh.smax, mx); }
    __syncthreads();
    const uint32_t smin = rfl(sh.smin), smax = rfl(sh.smax);
    const int sshift = shift_for<LOG_NB>(smax - smin);
#pragma unroll
    for (int i = 0; i < 4; ++i) atomicAdd(&sh.hist[(k[i] - smin) >> sshift], 1u);
    __syncthreads();
    if (tid == 0) { sh.smin = 0xFFFFFFFFu; sh.smax = 0; }
    uint32_t loc[BPT], sum = 0;
#pragma unroll
    for (int q = 0; q < BPT; ++q) { loc[q] = sh.hist[tid * BPT + q]; sum += loc[q]; }
#pragma unroll
    for (int q = 0; q < BPT; ++q) sh.hist[tid * BPT + q] = 0;
    uint32_t total;
    const uint32_t excl = block_excl_scan<NT>(sum, tid, sh.wpart, &total);
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const uint32_t want = (uint32_t)(r + 1) * (n / 4) - excl;      // sample ranks n/4, n/2, 3n/4
        if (want < sum) {
            uint32_t p = 0;
            bool done = false;
#pragma unroll
            for (int q = 0; q < BPT; ++q) {
                if (!done && want - p < loc[q]) { sh.res[r] = tid * BPT + q; done = true; }
                p += loc[q];
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        const uint32_t half = (1u << sshift) >> 1;
        const float q25 = __uint_as_float(smin + (sh.res[0] << sshift) + half);
        const float q50 = __uint_as_float(smin + (sh.res[1] << sshift) + half);
        const float q75 = __uint_as_float(smin + (sh.res[2] << sshift) + half);
        const float hd = 0.5f * (q75 - q25);
        if (q50 > 0.0f && hd > 0.0f && q50 < 3.0e38f && hd < 3.0e38f) {      // (false for NaNs)
            sh.hmed[m] = q50;
            sh.hwl[m] = 1.25f * hd;          // (the reach a run keeps from step to step)
            sh.hwh[m] = 1.25f * hd;
            sh.hmad[m] = hd;
            sh.hok[m] = 1;
        }
    }
    __syncthreads();
}

// Signed score and node score of one register row, dividing with the IEEE
// operator.  AGG 0 = scaled pairwise sum, 1 = max.  This is the route of every
// column that holds a missing sample.
template <int AGG>
__device__ __forceinline__ void score_row(const float (&x)[4], float med, float s, uint32_t absmask,
                                          uint32_t sgnmask, float thr, float node_scale,
                                          uint32_t* e, float* nz) {
    float zs[4];
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float z = ((x[i] + 0.0f) - med) / s;      // -0 reads as +0
        const float zi = __uint_as_float((__float_as_uint(z) & absmask) ^ sgnmask);
        // A NaN is a missing sample and its score a NaN: it never exceeds (the
        // comparison is false) and adds nothing to its node.
        bits |= (zi > thr ? 1u : 0u) << (8 * i);
        zs[i] = zi == zi ? zi : 0.0f;
    }
    *e = bits;
    // lanes 2p and 2p+1 hold GPUs 0-3 and 4-7 of one node
    if (AGG == 0) {
        const float half = (zs[0] + zs[1]) + (zs[2] + zs[3]);
        const float other = lane_xor1(half);
        *nz = node_scale * (half + other);
    } else {
        const float half = fmaxf(fmaxf(zs[0], zs[1]), fmaxf(zs[2], zs[3]));
        const float other = lane_xor1(half);
        *nz = fmaxf(half, other) + 0.0f;
    }
}

// The same for the scaled sum, with the quotient d/s obtained from the
// column's reciprocal r = RN(1/s) by two residual corrections:
//   q0 = RN(d*r); q1 = RN(q0 + RN(d - q0*s)*r); q2 = RN(q1 + (d - q1*s)*r)
// q1 is within one ulp of d/s, for which the residual d - q1*s is exact in
// fp32 and the second correction returns the correctly rounded quotient
// (Markstein's division theorem), provided nothing under- or overflows --
// the caller checks the column's magnitudes for that.  ss is +s or -s (a
// lower-is-worse metric scores -z), TWO_SIDED scores |z|.
template <bool TWO_SIDED>
__device__ __forceinline__ void score_row_fast(const float (&x)[4], float med, float ss, float rs,
                                               float thr, float node_scale, uint32_t* e, float* nz) {
    float zs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float d = x[i] - med;
        const float q0 = d * rs;
        const float e0 = __builtin_fmaf(-q0, ss, d);
        const float q1 = __builtin_fmaf(e0, rs, q0);
        const float e1 = __builtin_fmaf(-q1, ss, d);
        const float q2 = __builtin_fmaf(e1, rs, q1);
        zs[i] = TWO_SIDED ? fabsf(q2) : q2;
    }
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) bits |= (zs[i] > thr ? 1u : 0u) << (8 * i);
    *e = bits;
    const float half = (zs[0] + zs[1]) + (zs[2] + zs[3]);
    const float other = lane_xor1(half);
    *nz = node_scale * (half + other);
}

// Supporting (non-primary) metric with a one-sided direction, sign-free column:
// only the decisions are needed, not the scores, so no division is done.
//   * A rank exceeds iff x >= xstar (higher is worse) or x <= xstar (lower is
//     worse): sub and divide are monotone, and xstar is the exact boundary found
//     by the caller with the very operations the definition uses.
//   * The node score scale*sum(z') is estimated as cc*sum(x) - kk with
//     cc ~ +-scale/s and kk ~ 8*med*cc.  All roundings of the exact chain and of
//     the estimate together stay below `margin` (see the caller), so the estimate
//     decides unless it falls within `margin` of the threshold.  The estimate is
//     monotone in sum(x), so the caller hands in a bound sthr on the sum itself,
//     checked by it against the estimate's own formula: on the far side of sthr the
//     node cannot exceed nor come near.  *cand is set for the lanes on the near side;
//     the caller then forms the estimate and, within `margin` of the threshold, the
//     exact score.
template <bool LOWER_IS_WORSE>
__device__ __forceinline__ void score_row_decide(const float (&x)[4], uint32_t xcut, uint32_t shift_m,
                                                 uint32_t mask_m, float sthr, uint32_t* e, bool* cand) {
    // Values and boundary are positive floats, which order like their bit patterns: with
    // xcut = bits(xstar) - 1 (higher is worse) or bits(xstar) + 1 (lower is worse) the sign of
    // one integer difference per value is the decision.  The four sign bytes are brought
    // together by byte permutes and land, shifted, on bit m of the four mask bytes.
    uint32_t d[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        d[i] = LOWER_IS_WORSE ? __float_as_uint(x[i]) - xcut : xcut - __float_as_uint(x[i]);
    const uint32_t lo2 = __builtin_amdgcn_perm(d[1], d[0], 0x0C0C0703u);     // bytes: d0.b3, d1.b3, 0, 0
    const uint32_t hi2 = __builtin_amdgcn_perm(d[3], d[2], 0x07030C0Cu);     // bytes: 0, 0, d2.b3, d3.b3
    *e = ((lo2 | hi2) >> shift_m) & mask_m;                  // (already in place for metric m)
    const float half = (x[0] + x[1]) + (x[2] + x[3]);
    const float sum = half + lane_xor1(half);
    *cand = LOWER_IS_WORSE ? sum <= sthr : sum >= sthr;
}

// FULL: R == NT*4*ROWS exactly, so no lane is padding and no bounds are checked.
// SPLIT (short batches, the streaming case): one workgroup per column instead of
// per run of steps, so that the M columns of a step are scored side by side.  The
// exceed bits of a column are then OR-ed into the (zeroed) mask outputs in global
// memory and combine_kernel applies the multi-signal rule afterwards.
template <int NT, int ROWS, int LOG_NB, bool FULL, bool SPLIT, bool WANT_Z>
__global__ __launch_bounds__(NT, 4) void score_kernel(const gd_score_args a) {   // <= 128 VGPRs: 16 waves per CU
    constexpr int BLK = NT * 4;               // ranks per register row
    constexpr int MAX_NODES = BLK * ROWS / 8;
    constexpr int NWAVES = NT / WAVE;
    using SH = Shared<NT, LOG_NB, MAX_NODES>;
    // Dynamic LDS: the selection's work area, then one word of exceed-mask bytes
    // per (row, thread) -- kept in LDS, not registers, across the M columns.
    extern __shared__ __align__(16) unsigned char lds_raw[];
    SH& sh = *reinterpret_cast<SH*>(lds_raw);
    uint32_t* emask = reinterpret_cast<uint32_t*>(lds_raw + ((sizeof(SH) + 15) & ~(size_t)15));

    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int w = rfl(tid >> 6);
    const uint32_t R = a.R, N = a.N, M = a.M;
    const uint32_t RW = (R + 63) / 64, NWD = (N + 63) / 64;
    const float thr = a.thr;
    // Each workgroup scores a contiguous run of steps, column after column, and
    // loads the next column while it scores the current one.
    const uint32_t spw = SPLIT ? 1u : (a.T + gridDim.x - 1) / gridDim.x;
    const uint32_t t_begin = SPLIT ? blockIdx.x / M : blockIdx.x * spw;
    const uint32_t t_end = min(a.T, t_begin + spw);
    if (t_begin >= t_end) return;
    const uint32_t m_begin = SPLIT ? blockIdx.x % M : 0u, m_end = SPLIT ? m_begin + 1u : M;

    // Row j of wave w covers rank block (j + w) % ROWS, so that the first
    // registers to arrive (row 0) sample the whole rank range.
    // The lane part (tid*4) is passed in so that each phase can use its own,
    // optimiser-opaque copy: otherwise every row's store and load address is
    // computed once and kept in registers for the whole kernel.
    auto rbase = [&](int j, uint32_t tid4) -> uint32_t {
        return (uint32_t)((j + w) & (ROWS - 1)) * BLK + tid4;
    };
    auto fresh_tid4 = [&]() -> uint32_t { return opaque_v((uint32_t)tid * 4); };

    uint32_t NE[(ROWS + 3) / 4]; // node mask byte per row, packed
    // the selection's work area starts in its rest state (see the LDS protocol)
    for (int i = tid; i < SH::NB + 128; i += NT) sh.dlo[i] = 0;      // dlo, hist, dhi
    for (int i = tid; i < (MAX_NODES / 8 > 0 ? MAX_NODES / 8 : 1); i += NT) sh.ranka[i] = 0;
    if (tid == 0) {
        sh.umax[0] = 0; sh.umax[1] = 0; sh.ncand = 0; sh.below = 0; sh.nkept = 0; sh.mres[0][3] = 0; sh.mres[1][3] = 0;
        sh.smin = 0xFFFFFFFFu; sh.smax = 0; sh.d1 = 0; sh.d2 = 0xFFFFFFFFu;
        for (int m = 0; m < 8; ++m) { sh.hok[m] = 0; sh.hfast[m] = 1; }
        // A one-step call may be told the medians and MADs of a recent step (usually the
        // previous call's outputs).  They take the place of the hints a run of steps builds
        // up for itself; like those they are only trusted as far as the counting pass
        // confirms them, so any content is safe.
        if (SPLIT && a.hint_med && a.hint_mad && a.T == 1) {
            const float hm = a.hint_med[m_begin], hd = a.hint_mad[m_begin];
            if (hm > 0.0f && hd > 0.0f && hm < 3.0e38f && hd < 3.0e38f) {      // (false for NaNs)
                sh.hmed[m_begin] = hm;
                sh.hwl[m_begin] = 1.25f * hd;
                sh.hwh[m_begin] = 1.25f * hd;
                sh.hmad[m_begin] = hd;
                sh.hok[m_begin] = 1;
            }
        }
    }
    __syncthreads();
    // number of threads whose sampled element (row 0) is a real rank
    uint32_t nsample = NT;
    if (!FULL) {
        const uint32_t c = __popcll(__ballot(rbase(0, (uint32_t)tid * 4) < R));
        if (lane == 0) atomicAdd(&sh.ncand, c);
        __syncthreads();
        nsample = rfl(sh.ncand);
        __syncthreads();
        if (tid == 0) sh.ncand = 0;
        __syncthreads();
    }

    const float inv_node_scale = 1.0f / a.node_scale;      // (only used where node_scale > 0)
    uint32_t dir_codes = 0;          // direction + 1 of metric i in bits 2i, 2i + 1
#pragma unroll
    for (int i = 0; i < 8; ++i) dir_codes |= (uint32_t)(a.dir[i] + 1) << (2 * i);
    dir_codes = rfl(dir_codes);
    const uint32_t k0_all = R / 2 - 1, k1_all = R / 2;   // the middle ranks when nothing is missing (R is even)
    uint32_t colpar = 0;                          // parity of the column count: which umax slot is in use

    float v[ROWS][4];
    // Issue the loads of one register row of a column (padding: a NaN, whose key
    // lies above every real key).
    auto load_row = [&](int j, const float* col, uint32_t tid4) {
        float4 q;
        if (FULL) {
            // (a uniform row pointer plus the lane's 32-bit offset: one address mode, no vector
            // arithmetic per row)
            const float* rowp = col + (uint32_t)((j + w) & (ROWS - 1)) * BLK;
            q = *reinterpret_cast<const float4*>(rowp + tid4);
        } else if (rbase(j, tid4) < R) {
            q = *reinterpret_cast<const float4*>(col + rbase(j, tid4));
        } else {
            const float pad = __uint_as_float(0x7FFFFFFFu);
            q = make_float4(pad, pad, pad, pad);
        }
        v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
    };
    {
        const uint32_t tl = fresh_tid4();
        const float* col = a.x + ((size_t)t_begin * M + m_begin) * R;
        // issued in row order, like the refills of the score loop: the waits of the
        // first pass over a column are then placed row by row
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            load_row(j, col, tl);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    for (size_t t = t_begin; t < t_end; ++t) {
#pragma unroll
    for (int j = 0; j < ROWS; ++j) emask[j * NT + tid] = 0;   // each slot is private to its thread
#pragma unroll
    for (int j = 0; j < (ROWS + 3) / 4; ++j) NE[j] = 0;
    for (uint32_t m = m_begin; m < m_end; ++m) {
        // the column after this one (next metric, or the next step's first metric)
        // (after the very last column the current one is simply read again: a
        // branch-free refill keeps the register allocation of the score loops simple)
        const bool have_next = !SPLIT && (m + 1 < M || t + 1 < t_end);
        const float* next_col = a.x + (t * M + m + (have_next ? 1 : 0)) * (size_t)R;
        const uint32_t tl = fresh_tid4();
        const bool svalid = FULL || rbase(0, tl) < R;
        // A workgroup scores consecutive steps, and telemetry moves little from one
        // step to the next: the previous step's median of this metric, with the
        // reach its histogram had, brackets this step's counting pass without
        // sampling.  A bracket that misses is noticed and replaced by the sample's.
        // (the first step of a run has no predecessor: a sample of the column stands in)
        bool boot = false;
        if (FULL && t == t_begin && rfl(sh.hok[m]) == 0) {
            sample_hints<NT, LOG_NB>(sh, v[0], m);
            boot = true;
        }
        bool hinted = rfl(sh.hok[m]) != 0;
        uint32_t hint_lo = 0, hint_hi = 0;
        if (hinted) {
            const float xl = sh.hmed[m] - sh.hwl[m], xh = sh.hmed[m] + sh.hwh[m];
            hint_lo = rfl(__float_as_uint(xl));
            hint_hi = rfl(__float_as_uint(xh));
            hinted = xl >= 0.0f && xh > xl && hint_hi < 0x7F800000u;
        }
        uint32_t* const umax_slot = &sh.umax[colpar];
        uint32_t umax = 0;
        uint32_t s0 = 0, s1 = 0;
        float med = 0.0f;
        bool have_mad = false;
        // The hinted selection (sign-free column, exact-fit tiling, a predecessor's bracket and
        // MAD): median and MAD in three light passes.  Whatever it does not settle goes
        // through the general route below.
        int hsel = 0;
        bool tried_fast = false;
        if (FULL && hinted && rfl(sh.hfast[m]) != 0 && hint_hi < 0x7D000000u - 2u * (hint_hi - hint_lo) &&
            hint_hi - hint_lo < 0x20000000u) {
            tried_fast = true;
            const HintedResult hr = hinted_select<NT, ROWS, LOG_NB>(sh, v, hint_lo, hint_hi, sh.hmad[m], k0_all,
                                                                    k1_all, umax_slot, colpar);
            hsel = hr.found;
            umax = hr.umax;
            if (hsel == 0) {
                hinted = false;                 // (and this metric goes the general way from now on,
                                                // unless the hint was only a sample's)
                if (tid == 0 && !boot) sh.hfast[m] = 0;
            } else {
                med = 0.5f * (__uint_as_float(hr.m0) + __uint_as_float(hr.m1));
                have_mad = hsel == 2;
                s0 = hr.q0; s1 = hr.q1;
                if (tid == 0) sh.hmed[m] = med;
            }
        }
        // Largest raw bit pattern of the column: >= 0x80000000 iff some value carries
        // a sign bit (negative or -0); otherwise it is the bit pattern of the maximum.
        // With a hint the column is taken to be sign-free like its predecessor and the
        // maximum is found by the median's counting pass itself, which starts on the
        // register rows as they arrive; otherwise it takes a pass of its own.
        const bool fused_umax = FULL && hinted && !tried_fast;
        if (__builtin_expect(!fused_umax && !tried_fast, 0)) {
            uint32_t um = 0;
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
                if (FULL || rbase(j, tl) < R) {
                    um = max(um, max(__float_as_uint(v[j][0]), __float_as_uint(v[j][1])));
                    um = max(um, max(__float_as_uint(v[j][2]), __float_as_uint(v[j][3])));
                }
            }
            um = wave_max_to_last(um);
            if (lane == WAVE - 1) atomicMax(umax_slot, um);
            __syncthreads();
            umax = rfl(*umax_slot);
        }
        // special: some value carries a sign bit or is a NaN.  The raw bits are then no
        // keys to select by, and a NaN is a missing sample that the ranks must not count.
        bool special = umax > 0x7F800000u;
        uint32_t k0 = k0_all, k1 = k1_all;

        if (hsel == 0 && !special) {
            uint32_t hlo = 0, hhi = 0;
            int hshift = 0;
            const bool one_round = block_select<NT, ROWS, LOG_NB, true>(
                sh, XKeys<ROWS, true>{v}, __float_as_uint(v[0][0]), svalid, nsample, k0_all, k1_all, &s0,
                &s1, &hlo, &hhi, &hshift, hinted, hint_lo, hint_hi, fused_umax ? umax_slot : nullptr, &umax);
            special = umax > 0x7F800000u;      // (only the fused pass can find this out here)
        if (!special) {
            med = 0.5f * (__uint_as_float(s0) + __uint_as_float(s1));
            if (one_round)
                have_mad = mad_from_histogram<NT, ROWS, LOG_NB>(sh, v, med, hlo, hhi, hshift, k0_all, k1_all,
                                                                hinted ? sh.hmad[m] : 0.0f, &s0, &s1);
            if (tid == 0) {
                if (have_mad) {                 // keep the reach, follow the median
                    if (!hinted) {
                        // the reach kept for the coming steps: median -+ 1.25 MAD (the edge
                        // pairing looks up to 1.125 MAD away) rather than the sample's wider
                        // bracket -- fewer keys to count, finer buckets, fewer candidates
                        const float madv = 0.5f * (__uint_as_float(s0) + __uint_as_float(s1));
                        sh.hwl[m] = fminf(med - __uint_as_float(hlo), 1.25f * madv);
                        sh.hwh[m] = fminf(__uint_as_float(hhi) - med, 1.25f * madv);
                    }
                    sh.hmed[m] = med;
                    sh.hmad[m] = 0.5f * (__uint_as_float(s0) + __uint_as_float(s1));
                    sh.hok[m] = 1;
                } else {
                    sh.hok[m] = 0;
                }
            }
        }
        }
        // the other slot is free again: every thread read it a column ago
        if (tid == 0) { sh.umax[colpar ^ 1u] = 0; sh.mres[colpar ^ 1u][3] = 0; }
        colpar ^= 1u;
        uint32_t present = R;
        if (__builtin_expect(special, 0)) {
            if (tid == 0) sh.hok[m] = 0;
            __syncthreads();    // (a counting pass given up above has just reset sh.below)
            // samples present (padding lanes hold NaNs too): median and MAD are taken
            // over them alone, the middle one(s) of `present`
            // (tested on the bit patterns, against an opaque constant: the score loop's own
            // tests of the same registers must not be merged with these and kept for later)
            uint32_t np = 0;
            const uint32_t absm = opaque_s(0x7FFFFFFFu);
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) np += (__float_as_uint(v[j][i]) & absm) <= 0x7F800000u ? 1u : 0u;
                asm volatile("" : "+v"(np));
                __builtin_amdgcn_sched_barrier(0);
            }
            np = wave_incl_scan(np);
            if (lane == WAVE - 1 && np) atomicAdd(&sh.below, np);
            __syncthreads();
            present = rfl(sh.below);
            __syncthreads();                    // everyone has read the count
            if (tid == 0) sh.below = 0;
            k0 = present ? (present - 1) / 2 : 0u;
            k1 = present / 2;
            if (present) {
                const bool sv = svalid && v[0][0] == v[0][0];
                block_select<NT, ROWS, LOG_NB, false>(sh, XKeys<ROWS, false>{v}, key_of(v[0][0] + 0.0f),
                                                      sv, nsample, k0, k1, &s0, &s1);
                // (an odd count has one middle value: no sum that could overflow)
                med = k0 == k1 ? float_of_key(s0) : 0.5f * (float_of_key(s0) + float_of_key(s1));
            }
        }
        if (__builtin_expect(!have_mad && present, 0))
            block_select<NT, ROWS, LOG_NB, false>(sh, DKeys<ROWS>{v, med},
                                                  __float_as_uint(fabsf(v[0][0] - med)),
                                                  svalid && v[0][0] == v[0][0], nsample, k0, k1, &s0, &s1);
        float mad = k0 == k1 ? __uint_as_float(s0) : 0.5f * (__uint_as_float(s0) + __uint_as_float(s1));
        if (!present) med = mad = __uint_as_float(0x7FC00000u);      // nothing to take a median of
        if (tid == 0) {
            a.med[t * M + m] = med;
            a.mad[t * M + m] = mad;
            if (hsel) sh.hmad[m] = mad;         // the hinted selection follows median and MAD step by step
            // (from here on the reach is the exact MAD's, as after the general route)
            if (boot && hsel == 2) { sh.hwl[m] = 1.25f * mad; sh.hwh[m] = 1.25f * mad; }
        }
        float s = 1.4826f * mad;
        s = fmaxf(s, a.rel_floor * fabsf(med));
        s = fmaxf(s, a.abs_floor);

        // z, exceedance and node scores
        // (all eight directions in one scalar word: indexing the argument array by m
        // would be a load from memory, and a wait for it, in every column)
        const int dir = (int)((dir_codes >> (2u * m)) & 3u) - 1;
        const bool prim = m == a.primary;
        const uint32_t tz = fresh_tid4();
        float* nzrow = a.node_z + t * N;
        // The reciprocal route is exact while no intermediate can leave the normal
        // range: all x in [0, 2^59], 2^-34 <= med, 2^-60 <= s <= 2^60 (then every
        // non-zero |x - med| lies in [2^-59, 2^59]).
        const bool exact_recip = !special && umax <= 0x5D000000u && med >= 0x1p-34f && s >= 0x1p-60f &&
                                 s <= 0x1p60f;
        const bool fast = exact_recip && a.node_agg == 0;
        // (the run-time test that is always true keeps the block a region of its own for the
        // register allocator, as it was when the output pointer decided: without it this
        // instantiation spills)
        if (WANT_Z && opaque_s(1u) != 0u) {   // optional full z output, recomputed so that the loops below stay lean
                     // (it must come first: they refill the registers with the next column)
            float* zcol = a.z + (t * M + m) * (size_t)R;
            // the quotient by the column's reciprocal and two residual corrections where that
            // is exact (see score_row_fast; no sign bits there, so no -0 to read as +0)
            const bool by_recip = opaque_s(exact_recip ? 1u : 0u) != 0u;
            // (optimiser-opaque copies of the median and the scale: the differences x - med of
            // this loop must not be kept for the score loop below, 64 registers' worth)
            const float medz = __uint_as_float(opaque_s(__float_as_uint(med)));
            const float sz = __uint_as_float(opaque_s(__float_as_uint(s)));
            const float rz = 1.0f / sz;
            auto quotient = [&](float x) -> float {
                const float d = x - medz;
                const float q0 = d * rz;
                const float e0 = __builtin_fmaf(-q0, sz, d);
                const float q1 = __builtin_fmaf(e0, rz, q0);
                const float e1 = __builtin_fmaf(-q1, sz, d);
                return __builtin_fmaf(e1, rz, q1);
            };
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
                if (FULL || rbase(j, tz) < R) {
                    float4 q;
                    if (by_recip) {
                        q.x = quotient(v[j][0]); q.y = quotient(v[j][1]);
                        q.z = quotient(v[j][2]); q.w = quotient(v[j][3]);
                    } else {
                        q.x = ((v[j][0] + 0.0f) - medz) / sz; q.y = ((v[j][1] + 0.0f) - medz) / sz;
                        q.z = ((v[j][2] + 0.0f) - medz) / sz; q.w = ((v[j][3] + 0.0f) - medz) / sz;
                    }
                    if (special) {              // a missing sample (NaN) scores 0
                        const uint32_t absm = opaque_s(0x7FFFFFFFu);
                        q.x = (__float_as_uint(v[j][0]) & absm) <= 0x7F800000u ? q.x : 0.0f;
                        q.y = (__float_as_uint(v[j][1]) & absm) <= 0x7F800000u ? q.y : 0.0f;
                        q.z = (__float_as_uint(v[j][2]) & absm) <= 0x7F800000u ? q.z : 0.0f;
                        q.w = (__float_as_uint(v[j][3]) & absm) <= 0x7F800000u ? q.w : 0.0f;
                    }
                    *reinterpret_cast<float4*>(zcol + rbase(j, tz)) = q;
                }
                __builtin_amdgcn_sched_barrier(0);      // row by row: nothing of a later row starts early
            }
        }
        // Decision-only route for supporting one-sided metrics: find the exact boundary
        // xstar of "this rank exceeds" by probing 64 consecutive floats around
        // med +- thr*s with the defining operations (IEEE subtract and divide).
        bool decide = fast && !prim && dir != 0 && a.node_scale > 0.0f;
        float xstar = 0.0f;
        // One vector division serves both: lanes 0..62 probe 63 consecutive floats around
        // med +- thr*s, lane 63 divides 1 by s (the reciprocal every exact route needs).
        const float ss = dir < 0 ? -s : s;
        float rs;
        {
            const float xc = dir > 0 ? med + thr * s : med - thr * s;
            const uint32_t kc = key_of(xc);
            decide = decide && kc >= 64u && kc <= 0xFF800000u - 64u;
            const float xl = float_of_key(kc + (uint32_t)lane - 31u);
            const float num = lane == WAVE - 1 ? 1.0f : (dir > 0 ? xl - med : med - xl);
            const float q = num / s;
            const float r1 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(q), WAVE - 1));
            rs = dir < 0 ? -r1 : r1;                         // 1/(-s) = -(1/s) exactly
            if (decide) {
                const uint64_t probes = ~(1ull << (WAVE - 1));
                const uint64_t mk = __ballot(q > thr) & probes;
                // higher is worse: lanes f..62 true; lower is worse: lanes 0..f-1 true
                const uint64_t want = dir > 0 ? mk : ~mk & probes;
                const int f = want ? __builtin_ctzll(want) : 64;
                decide = f >= 1 && f <= 62 && want == ((~0ull << f) & probes);
                if (decide) xstar = __uint_as_float((uint32_t)__builtin_amdgcn_readlane(
                                (int)__float_as_uint(xl), dir > 0 ? f : f - 1));
                decide = decide && xstar > 0.0f;             // (the bit-pattern comparison needs a positive boundary)
            }
        }
        // decision-only route:
        // |estimate - exact node score| < |cc| * (sum(x) + 8*med) * 2^-20 + |thr| * 2^-23
        // and sum(x) + 8*med <= 16 * max(x):
        const float cc = a.node_scale * rs;
        const float kk = (8.0f * med) * cc;
        const float margin = __builtin_fmaf(fabsf(cc) * __uint_as_float(umax), 0x1.01p-16f,
                                            fabsf(thr) * 0x1p-22f);
        // The bound on sum(x) beyond which the estimate stays under thr - margin: solved
        // from the estimate's formula (1/cc = ss / node_scale, closely enough) with a little
        // slack and then checked with the formula itself (the estimate rises with the sum when
        // higher is worse, cc > 0, and falls with it otherwise).  Without a bound that passes
        // the check every row is a candidate.
        float sthr = dir > 0 ? -__builtin_inff() : __builtin_inff();
        if (decide) {
            const float tl = (thr - margin) - fabsf(thr) * 0x1p-20f;
            const float s0 = (tl + kk) * (ss * inv_node_scale);
            const float slack = fabsf(s0) * 0x1p-18f + 0x1p-100f;
            const float sb = dir > 0 ? s0 - slack : s0 + slack;
            if (__builtin_fmaf(sb, cc, -kk) < tl) sthr = sb;
        }
        const uint32_t xcut = dir > 0 ? __float_as_uint(xstar) - 1u : __float_as_uint(xstar) + 1u;
        const uint32_t shift_m = 7u - m, mask_m = 0x01010101u << m;
        const uint32_t absmask = dir == 0 ? 0x7FFFFFFFu : 0xFFFFFFFFu;
        const uint32_t sgnmask = dir < 0 ? 0x80000000u : 0u;
        // 0/1 decision-only (higher / lower is worse), 2/3 exact by reciprocal
        // (one- / two-sided), 4/5 IEEE division (scaled sum / max)
        const uint32_t route = fast ? (decide ? (dir > 0 ? 0u : 1u) : (dir != 0 ? 2u : 3u))
                                    : (a.node_agg == 0 ? 4u : 5u);
        uint32_t* const emask_lane = emask + opaque_v((uint32_t)tid);      // (row j: a constant offset from here)
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const uint32_t rt = opaque_s(route);
            uint32_t e, eplaced;
            float nz;
            if (rt <= 1u) {
                bool cand;
                if (rt == 0u) score_row_decide<false>(v[j], xcut, shift_m, mask_m, sthr, &e, &cand);
                else score_row_decide<true>(v[j], xcut, shift_m, mask_m, sthr, &e, &cand);
                eplaced = e;                                // (its bits are on metric m already)
                nz = thr;                                   // (not above the threshold: no node bit)
                if (__builtin_expect(__ballot(cand) != 0, 0)) {       // some node may exceed: the estimate decides,
                    const float half = (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);     // or, too close, the exact chain
                    nz = __builtin_fmaf(half + lane_xor1(half), cc, -kk);
                    if (__builtin_expect(__ballot(fabsf(nz - thr) <= margin) != 0, 0)) {
                        uint32_t e2;
                        score_row_fast<false>(v[j], med, ss, rs, thr, a.node_scale, &e2, &nz);
                    }
                    NE[j / 4] |= (nz > thr ? 1u : 0u) << (8 * (j & 3) + m);
                }
            } else {
                if (rt == 2u) {
                    score_row_fast<false>(v[j], med, ss, rs, thr, a.node_scale, &e, &nz);
                } else if (rt == 3u) {
                    score_row_fast<true>(v[j], med, ss, rs, thr, a.node_scale, &e, &nz);
                } else if (__builtin_expect(rt == 4u, 0)) {
                    score_row<0>(v[j], med, s, absmask, sgnmask, thr, a.node_scale, &e, &nz);
                } else {
                    score_row<1>(v[j], med, s, absmask, sgnmask, thr, a.node_scale, &e, &nz);
                }
                NE[j / 4] |= (nz > thr ? 1u : 0u) << (8 * (j & 3) + m);
                eplaced = e << m;
            }
            __hip_atomic_fetch_or(&emask_lane[j * NT], eplaced, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (prim && (FULL || rbase(j, tz) < R) && !(tz & 4)) nzrow[rbase(j, tz) / 8] = nz;
            if (!SPLIT) load_row(j, next_col, tz);   // the row is done: refill it with the next column
            // pin the row's results here, or its scores stay live until the loop ends
            asm volatile("" : "+v"(NE[j / 4]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    const uint32_t to = fresh_tid4();
    uint8_t* erow = a.exceed_mask + t * R;
    if (SPLIT) {
        // this column's bits join those of the step's other columns in global memory
        // (R and N are multiples of 4 here, the outputs word-aligned: see the launcher)
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            if (!(FULL || rbase(j, to) < R)) continue;
            const uint32_t Ej = emask[j * NT + to / 4];
            if (Ej) atomicOr(reinterpret_cast<uint32_t*>(erow + rbase(j, to)), Ej);
            const uint32_t nb = (NE[j / 4] >> (8 * (j & 3))) & 0xFFu;
            if (nb && !(to & 4)) {
                const size_t nidx = t * N + rbase(j, to) / 8;
                atomicOr(reinterpret_cast<uint32_t*>(a.node_mask + (nidx & ~(size_t)3)),
                         nb << (8 * (uint32_t)(nidx & 3)));
            }
        }
        return;
    }
    // per-rank mask bytes and anomaly bits.  Anomalous ranks are rare: their bits are OR-ed
    // into the step's bit words in LDS (all zero between steps) only by the waves that
    // hold one, and the finished words are copied out below.
    const uint32_t min_signals = rfl(a.min_signals), others_mask = ~(0x01010101u << a.primary);
    // multi-signal rule on four mask bytes at once: primary bit set and at least min_signals
    // bits in the byte; the answer is bit 0 of each byte
    auto rule4 = [&](uint32_t E) -> uint32_t {
        const uint32_t prim_set = (E >> a.primary) & 0x01010101u;
        if (min_signals <= 2u) {
            // (two signals: the primary's and any other -- bit 7 of "low seven bits + 0x7F",
            // or bit 7 itself, says that a byte is not zero)
            const uint32_t others = E & others_mask;
            const uint32_t some = (((others & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | others) >> 7;
            return min_signals <= 1u ? prim_set : (prim_set & some);
        }
        // per-byte popcount >= min_signals (adding 0x80 - min_signals carries into bit 7)
        uint32_t pc = E - ((E >> 1) & 0x55555555u);
        pc = (pc & 0x33333333u) + ((pc >> 2) & 0x33333333u);
        pc = (pc + (pc >> 4)) & 0x0F0F0F0Fu;
        return prim_set & ((pc + (0x80u - min_signals) * 0x01010101u) >> 7);
    };
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const bool valid = FULL || rbase(j, to) < R;
        const uint32_t Ej = emask[j * NT + to / 4];
        if (valid) *reinterpret_cast<uint32_t*>(erow + rbase(j, to)) = Ej;
        uint32_t an = rule4(Ej);
        if (!valid) an = 0u;
        if (__builtin_expect(__ballot(an != 0u) != 0ull, 0)) {
            // the lane's four ranks are bits rbase % 32 .. + 3 of 32-bit word rbase / 32
            const uint32_t nib = (an | (an >> 7) | (an >> 14) | (an >> 21)) & 0xFu;
            const uint32_t r0 = rbase(j, to);
            if (nib) atomicOr(&reinterpret_cast<uint32_t*>(sh.ranka)[r0 >> 5], nib << (r0 & 31u));
        }
        if (valid && !(to & 4)) sh.nodeb[rbase(j, to) / 8] = (uint8_t)((NE[j / 4] >> (8 * (j & 3))) & 0xFFu);
    }
    __syncthreads();
    for (uint32_t q = tid; q < RW; q += NT) {       // (one round at most in the exact-fit tilings)
        a.rank_anom[t * RW + q] = sh.ranka[q];
        sh.ranka[q] = 0;
    }
    if (FULL && ROWS == 16) {
        // N == 8 * NT: eight nodes per thread -- one 8-byte read of the staged bytes and one
        // 8-byte store; the rule byte-parallel as for the ranks; eight consecutive lanes make
        // one 64-bit anomaly word
        const uint32_t tq = opaque_v((uint32_t)tid), sl = tq & 7u;
        const uint2 nb = *reinterpret_cast<const uint2*>(&sh.nodeb[8 * tq]);
        uint8_t* nm = a.node_mask + t * N + 8 * tq;
        if (((uintptr_t)a.node_mask & 7u) == 0) {
            *reinterpret_cast<uint2*>(nm) = nb;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) nm[i] = (uint8_t)((i < 4 ? nb.x : nb.y) >> (8 * (i & 3)));
        }
        const uint32_t a0 = rule4(nb.x), a1 = rule4(nb.y);
        const uint32_t ab = ((a0 | (a0 >> 7) | (a0 >> 14) | (a0 >> 21)) & 0xFu) |
                            (((a1 | (a1 >> 7) | (a1 >> 14) | (a1 >> 21)) & 0xFu) << 4);
        uint32_t wlo = sl < 4u ? ab << (8u * sl) : 0u;
        uint32_t whi = sl >= 4u ? ab << (8u * (sl - 4u)) : 0u;
        wlo |= lane_xor<1>(wlo); whi |= lane_xor<1>(whi);
        wlo |= lane_xor<2>(wlo); whi |= lane_xor<2>(whi);
        wlo |= lane_xor<4>(wlo); whi |= lane_xor<4>(whi);
        if (sl == 0u) a.node_anom[t * NWD + tq / 8u] = ((uint64_t)whi << 32) | wlo;
    } else {
        if (FULL) {                             // N == NT * ROWS / 2: a fixed number of rounds
#pragma unroll
            for (int q = 0; q < (ROWS + 1) / 2; ++q) {
                const uint32_t n = opaque_v((uint32_t)tid) + (uint32_t)q * NT;
                if (ROWS % 2 == 0 || n < N) a.node_mask[t * N + n] = sh.nodeb[n];
            }
        } else {
            for (uint32_t n = tid; n < N; n += NT) a.node_mask[t * N + n] = sh.nodeb[n];
        }
        for (uint32_t wd = w; wd < NWD; wd += NWAVES) {
            const uint32_t n = wd * 64 + lane;
            bool an = false;
            if (n < N) {
                const uint32_t b = sh.nodeb[n];
                an = ((b >> a.primary) & 1u) && (uint32_t)__popc(b) >= a.min_signals;
            }
            const uint64_t word = __ballot(an);
            if (lane == 0) a.node_anom[t * NWD + wd] = word;
        }
    }
    }   // steps of this workgroup
}

// Split route, before the columns are scored: the mask outputs start at zero.
// (A fill kernel rather than a memset, so that a caller may capture the call.)
__global__ __launch_bounds__(256) void zero_masks_kernel(uint32_t* exceed_words, size_t n_exceed,
                                                         uint32_t* node_words, size_t n_node) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_exceed) exceed_words[i] = 0;
    if (i < n_node) node_words[i] = 0;
}

// Split route, after the columns: the multi-signal rule (primary bit set and at
// least min_signals bits) on the finished mask bytes.  blockIdx.y = step; a
// thread takes four ranks (one mask word), 16 lanes make one 64-bit word.
__global__ __launch_bounds__(256) void combine_kernel(const gd_score_args a) {
    const uint32_t t = blockIdx.y, lane = threadIdx.x & (WAVE - 1);
    const uint32_t R = a.R, N = a.N;
    const uint32_t RW = (R + 63) / 64, NWD = (N + 63) / 64;
    const uint32_t q = blockIdx.x * 256 + threadIdx.x;          // mask word index in the step
    if ((q & ~63u) * 4 < R) {                                   // some lane of this wave has ranks
        const bool valid = q * 4 < R;
        const uint32_t Ej = valid ? reinterpret_cast<const uint32_t*>(a.exceed_mask + (size_t)t * R)[q] : 0u;
        const uint32_t prim_set = (Ej >> a.primary) & 0x01010101u;
        uint32_t pc = Ej - ((Ej >> 1) & 0x55555555u);
        pc = (pc & 0x33333333u) + ((pc >> 2) & 0x33333333u);
        pc = (pc + (pc >> 4)) & 0x0F0F0F0Fu;
        const uint32_t enough = ((pc + (0x80u - a.min_signals) * 0x01010101u) >> 7) & 0x01010101u;
        const uint32_t an = prim_set & enough;
        const uint32_t nib = (an | (an >> 7) | (an >> 14) | (an >> 21)) & 0xFu;
        const uint32_t sub = lane & 15;
        uint32_t wlo = sub < 8 ? nib << (4 * sub) : 0u;
        uint32_t whi = sub >= 8 ? nib << (4 * (sub - 8)) : 0u;
        wlo |= lane_xor<1>(wlo); whi |= lane_xor<1>(whi);
        wlo |= lane_xor<2>(wlo); whi |= lane_xor<2>(whi);
        wlo |= lane_xor<4>(wlo); whi |= lane_xor<4>(whi);
        wlo |= lane_xor<8>(wlo); whi |= lane_xor<8>(whi);
        if (sub == 0 && valid) a.rank_anom[(size_t)t * RW + q / 16] = ((uint64_t)whi << 32) | wlo;
    }
    const uint32_t n = blockIdx.x * 256 + threadIdx.x;
    if ((n & ~63u) < N) {
        bool an = false;
        if (n < N) {
            const uint32_t b = a.node_mask[(size_t)t * N + n];
            an = ((b >> a.primary) & 1u) && (uint32_t)__popc(b) >= a.min_signals;
        }
        const uint64_t word = __ballot(an);
        if (lane == 0) a.node_anom[(size_t)t * NWD + n / 64] = word;
    }
}

// Diagnostic: the scoring kernel's loads and nothing else -- persistent 1024-thread
// workgroups, each reading a contiguous run of 256 KB blocks, sixteen float4 loads
// per thread and block -- as the ceiling that a single pass over the data has.
__global__ __launch_bounds__(1024) void read_probe_kernel(const float* x, uint64_t n_blocks,
                                                          uint32_t* sink) {
    constexpr uint32_t BLOCK_FLOATS = 1024 * 4 * 16;
    const uint64_t per = (n_blocks + gridDim.x - 1) / gridDim.x;
    const uint64_t b0 = blockIdx.x * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
    uint32_t acc = 0;
    for (uint64_t b = b0; b < b1; ++b) {
        const float* p = x + b * BLOCK_FLOATS + threadIdx.x * 4;
        float4 q[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) q[j] = *reinterpret_cast<const float4*>(p + j * 4096);
#pragma unroll
        for (int j = 0; j < 16; ++j)
            acc = max(acc, max(max(__float_as_uint(q[j].x), __float_as_uint(q[j].y)),
                               max(__float_as_uint(q[j].z), __float_as_uint(q[j].w))));
    }
    if (acc == 0xFFFFFFFFu) *sink = acc;      // (keeps the loads alive; NaN patterns aside, never true)
}

int compute_units(hipError_t* err) {
    static int n_cu = 0;
    *err = hipSuccess;
    if (n_cu == 0) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) { *err = e; return 0; }
        if (n_cu <= 0) n_cu = 256;
    }
    return n_cu;
}

// One workgroup per column needs whole mask words per step (R, N multiples of 4,
// word-aligned outputs) and pays off while the columns fit the chip side by side.
bool use_split(const gd_score_args& a, int n_cu) {
    return a.split_steps > 0 && a.T <= a.split_steps && (uint64_t)a.T * a.M <= (uint64_t)n_cu &&
           a.R % 32 == 0 && ((uintptr_t)a.node_mask & 3) == 0;
}

template <int NT, int ROWS, int LOG_NB>
constexpr size_t lds_bytes() {
    using SH = Shared<NT, LOG_NB, NT * 4 * ROWS / 8>;
    return ((sizeof(SH) + 15) & ~(size_t)15) + (size_t)ROWS * NT * 4;
}

// A whole batch: enough workgroups to fill every CU once (as many as fit by LDS and
// wave slots); each takes a contiguous run of ceil(T / grid) steps.
template <int NT, int ROWS, int LOG_NB, bool FULL>
hipError_t launch_runs(const gd_score_args& a, int n_cu, hipStream_t s) {
    constexpr size_t lds = lds_bytes<NT, ROWS, LOG_NB>();
    static_assert(lds <= 160 * 1024, "LDS budget of one CU");
    auto kern = score_kernel<NT, ROWS, LOG_NB, FULL, false, WANT_Z_HERE>;
    static bool configured = false;      // a handle is single-threaded; a repeated set is harmless
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const size_t by_lds = (size_t)160 * 1024 / lds, by_waves = (size_t)16 / (NT / WAVE);
    const size_t per_cu = by_lds < by_waves ? (by_lds ? by_lds : 1) : by_waves;
    const size_t cap = (size_t)n_cu * per_cu;
    const uint32_t grid = (uint32_t)(a.T < cap ? a.T : cap);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, s, a);
    return hipGetLastError();
}

// A short batch: one workgroup per column between the fill and the combining kernel.
template <int NT, int ROWS, int LOG_NB, bool FULL>
hipError_t launch_columns(const gd_score_args& a, hipStream_t s) {
    constexpr size_t lds = lds_bytes<NT, ROWS, LOG_NB>();
    static_assert(lds <= 160 * 1024, "LDS budget of one CU");
    auto kern = score_kernel<NT, ROWS, LOG_NB, FULL, true, WANT_Z_HERE>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const size_t n_exceed = (size_t)a.T * a.R / 4, n_node = (size_t)a.T * a.N / 4;
    hipLaunchKernelGGL(zero_masks_kernel, dim3((uint32_t)((n_exceed + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<uint32_t*>(a.exceed_mask), n_exceed,
                       reinterpret_cast<uint32_t*>(a.node_mask), n_node);
    hipLaunchKernelGGL(kern, dim3(a.T * a.M), dim3(NT), lds, s, a);
    hipLaunchKernelGGL(combine_kernel, dim3((a.R / 4 + 255) / 256, a.T), dim3(256), 0, s, a);
    return hipGetLastError();
}

// NT x ROWS: the tiling of a batch; CNT x CROWS: that of the per-column route, where a
// column has the CU to itself and is spread over more threads (fewer rows per lane:
// shorter passes between the barriers).
template <int NT, int ROWS, int LOG_NB, int CNT = NT, int CROWS = ROWS, int CLOG_NB = LOG_NB>
hipError_t launch(const gd_score_args& a, hipStream_t s) {
    static_assert(NT * ROWS == CNT * CROWS, "both tilings hold the same number of ranks");
    hipError_t cu_err;
    const int n_cu = compute_units(&cu_err);
    if (cu_err != hipSuccess) return cu_err;
    const bool full = a.R == (uint32_t)NT * 4 * ROWS;
    if (use_split(a, n_cu))
        return full ? launch_columns<CNT, CROWS, CLOG_NB, true>(a, s) : launch_columns<CNT, CROWS, CLOG_NB, false>(a, s);
    return full ? launch_runs<NT, ROWS, LOG_NB, true>(a, n_cu, s) : launch_runs<NT, ROWS, LOG_NB, false>(a, n_cu, s);
}

// Pick the register tiling for R: NT threads x ROWS float4 rows hold NT*4*ROWS ranks.
hipError_t pick_tiling(const gd_score_args& a, hipStream_t s) {
    const uint32_t R = a.R;
    if (R <= 256) return launch<64, 1, 10>(a, s);
    if (R <= 1024) return launch<64, 4, 10>(a, s);
    // (the 256-thread tilings take 2048 buckets: four workgroups then share a CU's LDS, and
    // their barrier-bound phases overlap)
    if (R <= 4096) return launch<256, 4, 11>(a, s);
    static_assert(4 * lds_bytes<256, 16, 11>() <= 160 * 1024, "four workgroups of the 16 384-rank tiling share a CU's LDS");
    if (R <= 16384) return launch<256, 16, 11, 1024, 4, 12>(a, s);
    if (R <= 32768) return launch<512, 16, 12, 1024, 8, 12>(a, s);
    if (R <= 65536) return launch<1024, 16, 12>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace

#if GD_SCORE_WANT_Z

hipError_t gd_launch_score_with_z(const gd_score_args& a, hipStream_t s) { return pick_tiling(a, s); }

#else

hipError_t gd_launch_read_probe(const float* d_x, uint64_t n_bytes, uint32_t* d_sink, hipStream_t s) {
    const uint64_t n_blocks = n_bytes / (256 * 1024);
    if (n_blocks == 0) return hipSuccess;
    hipError_t e;
    const int n_cu = compute_units(&e);
    if (e != hipSuccess) return e;
    const uint32_t grid = (uint32_t)(n_blocks < (uint64_t)n_cu ? n_blocks : (uint64_t)n_cu);
    hipLaunchKernelGGL(read_probe_kernel, dim3(grid), dim3(1024), 0, s, d_x, n_blocks, d_sink);
    return hipGetLastError();
}

hipError_t gd_launch_score(const gd_score_args& a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    return a.z ? gd_launch_score_with_z(a, s) : pick_tiling(a, s);
}

#endif
