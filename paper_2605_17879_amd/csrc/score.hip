// Scoring kernel: per (step, metric) cross-rank median and MAD by selection,
// robust z, exceedance, multi-signal combine and 8-GPU node scores
// (Section 4.2 peer-relative evaluation and multi-signal rule; Section 7.1
// 8-GPU nodes).
//
// One workgroup scores one step.  For each of the step's M columns it
//   1. loads the column once from HBM into registers (float4 per lane per row,
//      coalesced, rank-contiguous) -- the column is never read again;
//   2. finds the two middle order statistics by counting: a sample taken from
//      the first-arriving registers brackets the median, one pass puts the
//      bracketed values into an LDS histogram of order-preserving integer keys,
//      a scan locates the bucket(s) holding the wanted ranks, a second pass
//      gathers that bucket's few values into LDS where they are ranked exactly;
//      a bracket that misses, or a bucket that is too full (ties), falls back
//      to wider or narrower ranges until the answer is exact;
//   3. does the same for |x - med| to get the MAD;
//   4. computes z, the exceedance bits and the node scores from the registers.
// After the M columns the per-rank mask bytes, anomaly bits and node outputs
// are written.  HBM traffic is the 4 bytes per sample read plus ~1.8 bytes per
// rank and step of outputs.
#include <type_traits>

#include "gd_internal.h"

namespace {

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
    uint32_t hist[NB];
    uint32_t cand[CAND_CAP];
    uint32_t wpart[16];
    uint32_t below, ncand;
    uint32_t qlo, qhi, dlo, dhi;
    uint32_t res[6];   // ba, prefix before ba, bb, prefix through bb, va, vb
    uint8_t nodeb[MAX_NODES];
};

// Cross-lane moves with immediate patterns (DPP, swizzle, permlane): no address
// registers, nothing for the optimiser to hoist out of the column loop.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp0(uint32_t v) {   // lanes without a source read 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}
template <int J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v, int lane) {
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);
    else if constexpr (J == 8) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true);
    else if constexpr (J == 4 || J == 16) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (J << 10));
    else {
        static_assert(J == 32, "lane_xor");
        auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return (lane & 32) ? r[0] : r[1];
    }
}
__device__ __forceinline__ float lane_xor1(float v) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_mov_dpp((int)__float_as_uint(v), 0xB1, 0xF, 0xF, true));
}

// Inclusive prefix sum across the wave.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    v += dpp0<0x111>(v);          // row_shr:1
    v += dpp0<0x112>(v);          // row_shr:2
    v += dpp0<0x114>(v);          // row_shr:4
    v += dpp0<0x118>(v);          // row_shr:8
    v += dpp0<0x142, 0xA>(v);     // row_bcast:15 into rows 1 and 3
    v += dpp0<0x143, 0xC>(v);     // row_bcast:31 into rows 2 and 3
    return v;
}

// Exclusive prefix sum of one value per thread over the workgroup; total in *tot.
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wpart, uint32_t* tot) {
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x >> 6;
    const uint32_t inc = wave_incl_scan(v);
    if (NT == WAVE) {
        *tot = __builtin_amdgcn_readlane((int)inc, WAVE - 1);
        return inc - v;
    }
    if (lane == WAVE - 1) wpart[w] = inc;
    __syncthreads();
    uint32_t off = 0, total = 0;
#pragma unroll
    for (int i = 0; i < NT / WAVE; ++i) {
        uint32_t p = wpart[i];
        if (i < w) off += p;
        total += p;
    }
    *tot = total;
    return off + inc - v;
}

template <int K, int J>
__device__ __forceinline__ uint32_t sort_step(uint32_t v, int lane) {
    const uint32_t o = lane_xor<J>(v, lane);
    const bool take_min = ((lane & K) == 0) == ((lane & J) == 0);
    const uint32_t mn = v < o ? v : o, mx = v < o ? o : v;
    return take_min ? mn : mx;
}
template <int K, int J>
__device__ __forceinline__ uint32_t sort_merge(uint32_t v, int lane) {
    v = sort_step<K, J>(v, lane);
    if constexpr (J > 1) v = sort_merge<K, J / 2>(v, lane);
    return v;
}
// Ascending bitonic sort of one value per lane across the wave.
__device__ __forceinline__ uint32_t wave_sort(uint32_t v, int lane) {
    v = sort_merge<2, 1>(v, lane);
    v = sort_merge<4, 2>(v, lane);
    v = sort_merge<8, 4>(v, lane);
    v = sort_merge<16, 8>(v, lane);
    v = sort_merge<32, 16>(v, lane);
    v = sort_merge<64, 32>(v, lane);
    return v;
}

// A value the optimiser cannot see through: stops it from keeping one pass's
// per-element temporaries alive for the next pass (64+ registers per lane).
__device__ __forceinline__ uint32_t opaque(uint32_t v) {
    v = rfl(v);
    asm volatile("" : "+s"(v));
    return v;
}

// Keys of the median selection: the order-preserving image of x itself.
template <int ROWS>
struct XKeys {
    static constexpr bool kSigned = true;
    const float (&v)[ROWS][4];
    __device__ __forceinline__ uint32_t token() const { return opaque(31u); }
    __device__ __forceinline__ uint32_t raw(int j, int i, uint32_t) const { return __float_as_uint(v[j][i]); }
    // full key from the raw bits; tok is an opaque 31
    __device__ __forceinline__ uint32_t full(uint32_t b, uint32_t tok) const {
        return b ^ ((uint32_t)((int32_t)b >> tok) | 0x80000000u);
    }
};

// Keys of the MAD selection: the bits of |x - med| (non-negative floats order as integers).
template <int ROWS>
struct DKeys {
    static constexpr bool kSigned = false;
    const float (&v)[ROWS][4];
    float med;
    __device__ __forceinline__ uint32_t token() const { return opaque(__float_as_uint(med)); }
    __device__ __forceinline__ uint32_t raw(int j, int i, uint32_t tok) const {
        return __float_as_uint(fabsf(v[j][i] - __uint_as_float(tok)));
    }
    __device__ __forceinline__ uint32_t full(uint32_t b, uint32_t) const { return b; }
};

// Exact selection of the order statistics k0 <= k1 (0-based, k1 - k0 <= 1) of
// ROWS*4 keys per thread held in registers.  [lo, hi] is a guess of a key range
// containing both; any guess is safe.  Keys of padding lanes (NaN) compare
// above every real key.  While the range holds only non-negative floats the
// key arithmetic is done on the raw bits (key - lo is the same number).
template <int NT, int ROWS, int LOG_NB, typename SH, typename Keys>
__device__ __forceinline__ void block_select(SH& sh, const Keys& keys, uint32_t k0, uint32_t k1,
                                             uint32_t lo, uint32_t hi, uint32_t* out0,
                                             uint32_t* out1) {
    constexpr int NB = 1 << LOG_NB;
    constexpr int BPT = NB / NT;
    static_assert(BPT >= 1 && (BPT % 4 == 0 || BPT < 4), "bucket split");
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    // mode 0: both statistics together; 1: k0 alone; 2: k1 alone (after a split)
    int mode = 0;
    uint32_t ka = k0, kb = k1, v0 = 0, v1 = 0;
    lo = rfl(lo);
    hi = rfl(hi);
    if (lo > hi) { lo = 0; hi = 0xFFFFFFFFu; }
    for (;;) {
        const uint32_t span = hi - lo;
        const int width = 32 - __builtin_clz(span | 1u);           // bits of span
        const int shift = width > LOG_NB ? width - LOG_NB : 0;      // (span >> shift) < NB
        const bool plain = !Keys::kSigned || lo >= 0x80000000u;     // raw-bit arithmetic is valid
        const uint32_t flip = Keys::kSigned ? 0x80000000u : 0u;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < BPT; ++q) sh.hist[tid * BPT + q] = 0;
        if (tid == 0) { sh.below = 0; sh.ncand = 0; }
        __syncthreads();
        // counting pass
        uint32_t nbelow = 0;   // per lane; summed over the wave after the pass
        {
            const uint32_t tok = keys.token();
            if (plain) {
                const uint32_t lor = lo ^ flip;
#pragma unroll
                for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t b = keys.raw(j, i, tok);
                        nbelow += (int32_t)b < (int32_t)lor ? 1u : 0u;
                        const uint32_t t = b - lor;
                        if (t <= span) atomicAdd(&sh.hist[t >> shift], 1u);
                    }
                    asm volatile("" : "+v"(nbelow));
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t kk = keys.full(keys.raw(j, i, tok), tok);
                        nbelow += kk < lo ? 1u : 0u;
                        const uint32_t t = kk - lo;
                        if (t <= span) atomicAdd(&sh.hist[t >> shift], 1u);
                    }
                    asm volatile("" : "+v"(nbelow));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        nbelow = wave_incl_scan(nbelow);
        if (lane == WAVE - 1 && nbelow) atomicAdd(&sh.below, nbelow);
        __syncthreads();
        // locate the buckets of ka and kb
        uint32_t loc[BPT], s = 0;
#pragma unroll
        for (int q = 0; q < BPT; ++q) { loc[q] = sh.hist[tid * BPT + q]; s += loc[q]; }
        uint32_t total;
        const uint32_t excl = block_excl_scan<NT>(s, sh.wpart, &total);
        const uint32_t below = sh.below;
        const uint32_t ra = ka - below, rb = kb - below;   // wraps when not bracketed
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
        const bool bracketed = rfl(ka >= below && rb < total);
        if (!bracketed) {               // the guess missed: count over all keys
            lo = 0; hi = 0xFFFFFFFFu;
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
            if (plain) {
                const uint32_t clor = clo ^ flip;
#pragma unroll
                for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t b = keys.raw(j, i, tok);
                        if (b - clor <= cspan) {
                            uint32_t pos = atomicAdd(&sh.ncand, 1u);
                            if (pos < (uint32_t)CAND_CAP) sh.cand[pos] = b;   // raw bits: same order as keys here
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t kk = keys.full(keys.raw(j, i, tok), tok);
                        if (kk - clo <= cspan) {
                            uint32_t pos = atomicAdd(&sh.ncand, 1u);
                            if (pos < (uint32_t)CAND_CAP) sh.cand[pos] = kk;
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __syncthreads();
            const uint32_t cnt = min(sh.ncand, (uint32_t)CAND_CAP);
            const uint32_t wa = ra - pa, wb = rb - pa;
            for (uint32_t i = tid; i < cnt; i += NT) {
                const uint32_t c = sh.cand[i];
                uint32_t r = 0;
                for (uint32_t j = 0; j < cnt; ++j) {
                    const uint32_t cj = sh.cand[j];
                    r += (cj < c || (cj == c && j < i)) ? 1u : 0u;
                }
                if (r == wa) sh.res[4] = c;
                if (r == wb) sh.res[5] = c;
            }
            __syncthreads();
            va = rfl(sh.res[4]) ^ (plain ? flip : 0u); vb = rfl(sh.res[5]) ^ (plain ? flip : 0u);
        } else {
            // crowded (ties): look inside bucket ba; if the two statistics sit in
            // different crowded buckets, finish k0 first, then k1 on its own
            if (ba != bb) { mode = 1; kb = ka; }
            const uint32_t nlo = lo + (ba << shift);
            const uint64_t nend = (uint64_t)nlo + ((uint64_t)1 << shift) - 1;
            hi = nend > hi ? hi : (uint32_t)nend;
            lo = nlo;
            continue;
        }
        if (mode == 0) { v0 = va; v1 = vb; break; }
        if (mode == 1) { v0 = va; mode = 2; ka = kb = k1; lo = 0; hi = 0xFFFFFFFFu; continue; }
        v1 = va;
        break;
    }
    *out0 = v0;
    *out1 = v1;
}

// z' and node score of one register row; AGG 0 = scaled pairwise sum, 1 = max.
template <int AGG>
__device__ __forceinline__ void score_row(const float (&x)[4], float med, float s, uint32_t absmask,
                                          uint32_t sgnmask, float thr, float node_scale,
                                          uint32_t* e, float* nz) {
    float zs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float z = (x[i] - med) / s;
        zs[i] = __uint_as_float((__float_as_uint(z) & absmask) ^ sgnmask);
    }
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) bits |= (zs[i] > thr ? 1u : 0u) << (8 * i);
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

// FULL: R == NT*4*ROWS exactly, so no lane is padding and no bounds are checked.
template <int NT, int ROWS, int LOG_NB, bool FULL>
__global__ __launch_bounds__(NT) void score_kernel(const gd_score_args a) {
    constexpr int BLK = NT * 4;               // ranks per register row
    constexpr int MAX_NODES = BLK * ROWS / 8;
    constexpr int NWAVES = NT / WAVE;
    using SH = Shared<NT, LOG_NB, MAX_NODES>;
    __shared__ SH sh;

    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int w = rfl(tid >> 6);
    const uint32_t R = a.R, N = a.N, M = a.M;
    const size_t t = blockIdx.x;
    const uint32_t RW = (R + 63) / 64, NWD = (N + 63) / 64;
    const float thr = a.thr;

    // Row j of wave w covers rank block (j + w) % ROWS, so that the first
    // registers to arrive (row 0) sample the whole rank range.
    // The lane part (tid*4) is passed in so that each phase can use its own,
    // optimiser-opaque copy: otherwise every row's store and load address is
    // computed once and kept in registers for the whole kernel.
    auto rbase = [&](int j, uint32_t tid4) -> uint32_t {
        return (uint32_t)((j + w) & (ROWS - 1)) * BLK + tid4;
    };
    auto fresh_tid4 = [&]() -> uint32_t {
        uint32_t v = (uint32_t)tid * 4;
        asm volatile("" : "+v"(v));
        return v;
    };

    uint32_t E[ROWS];            // exceed mask bytes of the lane's 4 ranks per row
    uint32_t NE[(ROWS + 3) / 4]; // node mask byte per row, packed
#pragma unroll
    for (int j = 0; j < ROWS; ++j) E[j] = 0;
#pragma unroll
    for (int j = 0; j < (ROWS + 3) / 4; ++j) NE[j] = 0;

    const uint32_t k0 = R / 2 - 1, k1 = R / 2;   // R is even

    for (uint32_t m = 0; m < M; ++m) {
        const float* col = a.x + (t * M + m) * (size_t)R;
        float v[ROWS][4];
        const uint32_t tl = fresh_tid4();
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            float4 q;
            if (FULL || rbase(j, tl) < R) {
                q = *reinterpret_cast<const float4*>(col + rbase(j, tl));
            } else {   // padding: a NaN, whose key lies above every real key
                const float pad = __uint_as_float(0x7FFFFFFFu);
                q = make_float4(pad, pad, pad, pad);
            }
            v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
        }
        if (tid == 0) { sh.qlo = 0xFFFFFFFFu; sh.qhi = 0; sh.dlo = 0xFFFFFFFFu; sh.dhi = 0; }
        __syncthreads();
        // -0 reads as +0 (x + 0 is exact for everything else)
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[j][i] += 0.0f;
        }
        // bracket the median from a sorted per-wave sample of row 0
        const bool svalid = FULL || rbase(0, tl) < R;
        const uint32_t nv = __popcll(__ballot(svalid));
        int lane_o = lane;                       // recomputed per column, so that the sort's
        asm volatile("" : "+v"(lane_o));         // lane predicates are not kept in registers
        const uint32_t sorted = wave_sort(svalid ? key_of(v[0][0]) : 0xFFFFFFFFu, lane_o);
        auto pick = [&](uint32_t idx) { return (uint32_t)__builtin_amdgcn_readlane((int)sorted, (int)rfl(idx)); };
        if (nv > 0) {
            const uint32_t q1 = pick(nv / 4);
            const uint32_t q3 = pick(min(nv - 1, (3 * nv) / 4));
            if (lane == 0) { atomicMin(&sh.qlo, q1); atomicMax(&sh.qhi, q3); }
        }
        __syncthreads();
        uint32_t s0, s1;
        block_select<NT, ROWS, LOG_NB>(sh, XKeys<ROWS>{v}, k0, k1, sh.qlo, sh.qhi, &s0, &s1);
        const float med = 0.5f * (float_of_key(s0) + float_of_key(s1));

        // bracket the MAD from the same sorted sample: inner and outer distances
        if (nv > 0) {
            const float fil = float_of_key(pick((3 * nv) / 8));
            const float fih = float_of_key(pick(min(nv - 1, (5 * nv) / 8)));
            const float fol = float_of_key(pick((5 * nv) / 32));
            const float foh = float_of_key(pick(min(nv - 1, (27 * nv) / 32)));
            float inner = fminf(med - fil, fih - med);
            float outer = fmaxf(med - fol, foh - med);
            inner = inner > 0.0f ? inner : 0.0f;
            outer = outer > 0.0f ? outer : 0.0f;
            if (lane == 0) {
                atomicMin(&sh.dlo, __float_as_uint(inner));
                atomicMax(&sh.dhi, __float_as_uint(outer));
            }
        }
        __syncthreads();
        block_select<NT, ROWS, LOG_NB>(sh, DKeys<ROWS>{v, med}, k0, k1, sh.dlo, sh.dhi, &s0, &s1);
        const float mad = 0.5f * (__uint_as_float(s0) + __uint_as_float(s1));
        if (tid == 0) {
            a.med[t * M + m] = med;
            a.mad[t * M + m] = mad;
        }
        float s = 1.4826f * mad;
        s = fmaxf(s, a.rel_floor * fabsf(med));
        s = fmaxf(s, a.abs_floor);

        // z, exceedance and node scores
        const int dir = a.dir[m];
        const uint32_t absmask = dir == 0 ? 0x7FFFFFFFu : 0xFFFFFFFFu;
        const uint32_t sgnmask = dir < 0 ? 0x80000000u : 0u;
        const bool prim = m == a.primary;
        const uint32_t tz = fresh_tid4();
        float* nzrow = a.node_z + t * N;
        auto zphase = [&](auto agg) {
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
                uint32_t e;
                float nz;
                score_row<decltype(agg)::value>(v[j], med, s, absmask, sgnmask, thr, a.node_scale, &e, &nz);
                E[j] |= e << m;
                NE[j / 4] |= (nz > thr ? 1u : 0u) << (8 * (j & 3) + m);
                if (prim && (FULL || rbase(j, tz) < R) && !(tz & 4)) nzrow[rbase(j, tz) / 8] = nz;
                // pin the row's results here, or its scores stay live until the loop ends
                asm volatile("" : "+v"(E[j]), "+v"(NE[j / 4]));
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (a.node_agg == 0) zphase(std::integral_constant<int, 0>{});
        else zphase(std::integral_constant<int, 1>{});
        if (a.z) {   // optional full z output, recomputed so that the loop above stays lean
            float* zcol = a.z + (t * M + m) * (size_t)R;
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
                if (FULL || rbase(j, tz) < R) {
                    float4 q;
                    q.x = (v[j][0] - med) / s; q.y = (v[j][1] - med) / s;
                    q.z = (v[j][2] - med) / s; q.w = (v[j][3] - med) / s;
                    *reinterpret_cast<float4*>(zcol + rbase(j, tz)) = q;
                }
            }
        }
    }

    // per-rank mask bytes and anomaly bits
    const uint32_t to = fresh_tid4();
    uint8_t* erow = a.exceed_mask + t * R;
    uint64_t* arow = a.rank_anom + t * RW;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const bool valid = FULL || rbase(j, to) < R;
        if (valid) *reinterpret_cast<uint32_t*>(erow + rbase(j, to)) = E[j];
        uint32_t nib = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t b = (E[j] >> (8 * i)) & 0xFFu;
            const bool an = ((b >> a.primary) & 1u) && (uint32_t)__popc(b) >= a.min_signals;
            nib |= (an && valid ? 1u : 0u) << i;
        }
        // 16 consecutive lanes hold one 64-bit word
        const int sub = lane & 15;
        uint32_t wlo = sub < 8 ? nib << (4 * sub) : 0u;
        uint32_t whi = sub >= 8 ? nib << (4 * (sub - 8)) : 0u;
        wlo |= lane_xor<1>(wlo, lane); whi |= lane_xor<1>(whi, lane);
        wlo |= lane_xor<2>(wlo, lane); whi |= lane_xor<2>(whi, lane);
        wlo |= lane_xor<4>(wlo, lane); whi |= lane_xor<4>(whi, lane);
        wlo |= lane_xor<8>(wlo, lane); whi |= lane_xor<8>(whi, lane);
        if (sub == 0 && valid)
            arow[rbase(j, to) / 64] = ((uint64_t)whi << 32) | wlo;
        if (valid && !(to & 4)) sh.nodeb[rbase(j, to) / 8] = (uint8_t)((NE[j / 4] >> (8 * (j & 3))) & 0xFFu);
    }
    __syncthreads();
    for (uint32_t n = tid; n < N; n += NT) a.node_mask[t * N + n] = sh.nodeb[n];
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

template <int NT, int ROWS, int LOG_NB>
hipError_t launch(const gd_score_args& a, hipStream_t s) {
    if (a.R == (uint32_t)NT * 4 * ROWS)
        hipLaunchKernelGGL((score_kernel<NT, ROWS, LOG_NB, true>), dim3(a.T), dim3(NT), 0, s, a);
    else
        hipLaunchKernelGGL((score_kernel<NT, ROWS, LOG_NB, false>), dim3(a.T), dim3(NT), 0, s, a);
    return hipGetLastError();
}

}  // namespace

// Pick the register tiling for R: NT threads x ROWS float4 rows hold NT*4*ROWS ranks.
hipError_t gd_launch_score(const gd_score_args& a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    const uint32_t R = a.R;
    if (R <= 256) return launch<64, 1, 10>(a, s);
    if (R <= 1024) return launch<64, 4, 10>(a, s);
    if (R <= 4096) return launch<256, 4, 12>(a, s);
    if (R <= 16384) return launch<256, 16, 12>(a, s);
    if (R <= 32768) return launch<512, 16, 12>(a, s);
    if (R <= 65536) return launch<1024, 16, 12>(a, s);
    return hipErrorInvalidValue;
}
