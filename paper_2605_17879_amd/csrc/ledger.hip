// The ledger: bookkeeping beyond the default decision rule.
//
//  * Persistence per indicator -- the other reading of Section 4.2's rule that
//    several indicators must deviate and keep deviating over successive evaluations:
//    every metric keeps its own k-of-W count per rank and per node, and the
//    multi-signal rule (primary among them, at least min_signals) is applied to
//    the metrics that are themselves sustained.
//  * The primary node score summed over the window as 16-bit integers, the key of
//    the ranking "by average score" (integer sums do not depend on the order of
//    addition, so the ring can be updated in any order).
//  * Recurrence: how many flag episodes of a node began within a horizon (a node
//    sent to triage three times within a week is terminally bad, Section 7).
//
// ledger_count_kernel: one thread per item (a node, or four ranks) and per chunk
// of steps.  The per-metric counts live in four registers as eight 16-bit fields,
// biased so that a field's top bit says "reached k"; a step adds the entering
// byte's bits and takes off the leaving byte's through a table in LDS (byte ->
// eight fields, and the same words negated), and the rule itself is evaluated
// only while the primary metric's top bit is on and no flagged step has been
// found yet.  A chunk other than the first rebuilds its starting counts from the
// W steps before it, so chunks are independent; the first flagged step is the
// minimum over chunks (an atomic max on 0xFFFFFFFF - step).  For nodes the kernel
// also follows the default rule's own flag and leaves one bit per (step, node)
// where an episode starts.
// ledger_finish_kernel, launched behind it: the rings take the batch's last
// steps, the score sums are brought up to date, and one thread per node walks the
// episode starts in step order.
#include "gd_internal.h"

namespace {

constexpr int WAVE = 64;
constexpr int LED_NT = 256;
constexpr int LED_AHEAD = 8;     // steps whose bytes are fetched together
constexpr int MAX_STARTS = 8;

// bits 2j and 2j+1 of an exceed byte as the two 16-bit fields of a word
__device__ __forceinline__ uint32_t spread2(uint32_t b, int j) {
    const uint32_t v = (b >> (2 * j)) & 3u;
    return (v | (v << 15)) & 0x00010001u;
}

// bit m set iff the count of metric m has reached K (counts <= 1024 < 0x8000 - K)
__device__ __forceinline__ uint32_t sustained(const uint32_t (&c)[4], uint32_t K) {
    const uint32_t bias = (0x8000u - K) * 0x00010001u;
    uint32_t pm = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t t = c[j] + bias;
        pm |= ((t >> 15) & 1u) << (2 * j);
        pm |= ((t >> 31) & 1u) << (2 * j + 1);
    }
    return pm;
}

// the multi-signal rule on a byte of metric bits
__device__ __forceinline__ uint32_t combine(uint32_t bits, uint32_t primary, uint32_t min_signals) {
    return ((bits >> primary) & 1u) && (uint32_t)__popc(bits) >= min_signals ? 1u : 0u;
}

// The rule on biased counts (each 16-bit field holds count + 0x8000 - K, so its top
// bit says "sustained"; the primary metric's field is the low half of word 0):
// primary sustained and at least min_signals fields are.
__device__ __forceinline__ uint32_t rule_on_biased(const uint32_t (&c)[4], uint32_t min_signals) {
    uint32_t n = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) n += (uint32_t)__popc(c[j] & 0x80008000u);
    return (c[0] & 0x8000u) && n >= min_signals ? 1u : 0u;
}

// Field f of the count words belongs to metric field_metric(f): the identity but for
// the primary metric and metric 0, which change places.
__device__ __forceinline__ uint32_t field_metric(uint32_t f, uint32_t primary) {
    return f == 0 ? primary : (f == primary ? 0u : f);
}

// IPT items per thread: ranks go four at a time (one 4-byte load per step), nodes
// singly, so that a wave's ballot is one word of the episode-start map.
// spread[b] (LDS) = the eight bits of byte b as eight 16-bit fields, spread[256 + b]
// the same words negated, so that one three-operand add per word takes a step.
template <bool NODE, int IPT>
__device__ __forceinline__ void count_items(const gd_ledger_args& a, uint32_t blk, const uint4* spread) {
    static_assert(IPT == 1 || IPT == 4, "count_items");
    static_assert(!NODE || IPT == 1, "count_items");
    const uint32_t n_items = NODE ? a.N : a.R;              // (R is a multiple of 8)
    const uint32_t item = (blk * LED_NT + threadIdx.x) * IPT;
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    if (item - lane * IPT >= n_items) return;               // whole wave out of range
    const bool live = item < n_items;
    const uint32_t i = live ? item : n_items - IPT;         // idle lanes repeat the last items, store nothing
    const uint8_t* mask = NODE ? a.node_mask : a.exceed_mask;
    const uint8_t* ring = a.led + (NODE ? a.lay.node_ring : a.lay.rank_ring);
    uint16_t* cnt = reinterpret_cast<uint16_t*>(a.led + (NODE ? a.lay.node_cnt : a.lay.rank_cnt));
    uint32_t* first = reinterpret_cast<uint32_t*>(a.led + (NODE ? a.lay.node_first : a.lay.rank_first));
    uint16_t* ccnt = reinterpret_cast<uint16_t*>(a.led + a.lay.node_ccnt);
    uint64_t* rise = a.rise;
    const uint32_t W = a.W, K = a.K, T = a.T;
    const uint32_t s0 = blockIdx.y * a.chunk;
    const uint32_t s1 = min(T, s0 + a.chunk);
    if (s0 >= s1) return;
    const uint32_t bias = (0x8000u - K) * 0x00010001u;      // counts <= 1024 and 1 <= K <= 1024: fields never wrap

    auto load = [&](const uint8_t* row) -> uint32_t {       // the IPT exceed bytes of this thread
        if (IPT == 4) return *reinterpret_cast<const uint32_t*>(row + i);
        return row[i];
    };
    // the exceed bytes of step s of the batch; s < 0 reaches back into the ring
    auto hist = [&](int64_t s) -> uint32_t {
        if (s >= 0) return load(mask + (size_t)s * n_items);
        const int64_t g = (int64_t)a.first_step + s;        // (below 2^31)
        return g >= 0 ? load(ring + (size_t)((uint32_t)g % W) * n_items) : 0u;
    };
    auto add_fields = [&](uint32_t (&c)[4], const uint4 v) { c[0] += v.x; c[1] += v.y; c[2] += v.z; c[3] += v.w; };

    uint32_t c[IPT][4];                                     // biased counts
    uint32_t cc = 0;                                        // the default rule's count (nodes)
    if (s0 == 0) {
#pragma unroll
        for (int k = 0; k < IPT; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                c[k][j] = ((uint32_t)cnt[(size_t)field_metric(2 * j, a.primary) * n_items + i + k] |
                           ((uint32_t)cnt[(size_t)field_metric(2 * j + 1, a.primary) * n_items + i + k] << 16)) + bias;
        if (NODE) cc = ccnt[i];
    } else {
#pragma unroll
        for (int k = 0; k < IPT; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) c[k][j] = bias;
        for (int64_t s = (int64_t)s0 - W; s < (int64_t)s0; s += LED_AHEAD) {
            uint32_t hb[LED_AHEAD];
#pragma unroll
            for (int q = 0; q < LED_AHEAD; ++q) hb[q] = s + q < (int64_t)s0 ? hist(s + q) : 0u;
#pragma unroll
            for (int q = 0; q < LED_AHEAD; ++q) {
#pragma unroll
                for (int k = 0; k < IPT; ++k) {
                    const uint32_t b = (hb[q] >> (8 * k)) & 0xFFu;
                    add_fields(c[k], spread[b]);
                    if (NODE) cc += combine(b, a.primary, a.min_signals);
                }
            }
        }
    }
    uint32_t best[IPT];                                     // 0xFFFFFFFF - first flagged step of the chunk
#pragma unroll
    for (int k = 0; k < IPT; ++k) best[k] = 0;
    bool cflag = NODE && cc >= K;                           // the default rule's flag one step earlier

    for (uint32_t s = s0; s < s1; s += LED_AHEAD) {
        uint32_t eb[LED_AHEAD], lb[LED_AHEAD];
#pragma unroll
        for (int q = 0; q < LED_AHEAD; ++q) {
            eb[q] = 0; lb[q] = 0;
            if (s + q < s1) {
                eb[q] = load(mask + (size_t)(s + q) * n_items);
                lb[q] = hist((int64_t)(s + q) - W);
            }
        }
#pragma unroll
        for (int q = 0; q < LED_AHEAD; ++q) {
            if (s + q >= s1) break;                         // uniform over the wave
            const uint32_t step_code = 0xFFFFFFFFu - (uint32_t)(a.first_step + s + q);
#pragma unroll
            for (int k = 0; k < IPT; ++k) {
                const uint32_t e = (eb[q] >> (8 * k)) & 0xFFu, l = (lb[q] >> (8 * k)) & 0xFFu;
                const uint4 se = spread[e], nl = spread[256 + l];
                c[k][0] += se.x + nl.x; c[k][1] += se.y + nl.y;
                c[k][2] += se.z + nl.z; c[k][3] += se.w + nl.w;
                // the rule needs the primary metric sustained, which it rarely is: only then look further
                if ((c[k][0] & 0x8000u) && !best[k] && rule_on_biased(c[k], a.min_signals)) best[k] = step_code;
                if (NODE) cc = cc + combine(e, a.primary, a.min_signals) - combine(l, a.primary, a.min_signals);
            }
            if (NODE) {
                const bool now = cc >= K;
                const uint64_t rb = __ballot(live && now && !cflag);
                cflag = now;
                // one word per (64 nodes, step), the steps of a word side by side
                if (lane == 0) rise[(size_t)(item / 64) * T + (s + q)] = rb;
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int k = 0; k < IPT; ++k)
        if (best[k]) atomicMax(&first[i + k], best[k]);
    if (s1 == T) {
        // With several chunks the first one may still have to read the old counts:
        // the new ones go to the staging span and the finishing kernel moves them.
        // (the staging span is laid out like the span of counts itself)
        const bool staged = gridDim.y > 1;
        uint16_t* cnt_out = staged ? reinterpret_cast<uint16_t*>(
                                         a.counts_new + ((NODE ? a.lay.node_cnt : a.lay.rank_cnt) - a.lay.rank_cnt))
                                   : cnt;
        uint16_t* ccnt_out = staged ? reinterpret_cast<uint16_t*>(a.counts_new + (a.lay.node_ccnt - a.lay.rank_cnt))
                                    : ccnt;
#pragma unroll
        for (int k = 0; k < IPT; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t v = c[k][j] - bias;
                cnt_out[(size_t)field_metric(2 * j, a.primary) * n_items + i + k] = (uint16_t)(v & 0xFFFFu);
                cnt_out[(size_t)field_metric(2 * j + 1, a.primary) * n_items + i + k] = (uint16_t)(v >> 16);
            }
        if (NODE) ccnt_out[i] = (uint16_t)cc;
    }
}

constexpr int RANK_IPT = 4;

// Blocks [0, rank_blocks) take ranks, the rest nodes; blockIdx.y is the chunk.
__global__ __launch_bounds__(LED_NT) void ledger_count_kernel(const gd_ledger_args a) {
    __shared__ uint4 spread[512];
    {
        const uint32_t b = threadIdx.x;                     // LED_NT == 256: one byte value per thread
        // bit 0 and the primary metric's bit change places: its field is the low half of word 0
        const uint32_t b0 = b & 1u, bp = (b >> a.primary) & 1u;
        const uint32_t v = (b & ~(1u | (1u << a.primary))) | bp | (b0 << a.primary);
        const uint4 f = make_uint4(spread2(v, 0), spread2(v, 1), spread2(v, 2), spread2(v, 3));
        spread[b] = f;
        spread[256 + b] = make_uint4(0u - f.x, 0u - f.y, 0u - f.z, 0u - f.w);
    }
    __syncthreads();
    const uint32_t rank_blocks = (a.R / RANK_IPT + LED_NT - 1) / LED_NT;
    if (blockIdx.x < rank_blocks) count_items<false, RANK_IPT>(a, blockIdx.x, spread);
    else count_items<true, 1>(a, blockIdx.x - rank_blocks, spread);
}

__device__ __forceinline__ int32_t quantise(float z, float quant) {
    const float v = z * quant;
    float r = __builtin_rintf(v);                           // ties to even
    r = fminf(fmaxf(r, -32768.0f), 32767.0f);
    return v == v ? (int32_t)r : 0;                         // a NaN counts as 0
}

// Blocks [0, node_blocks): one thread per node -- score ring and sum, then the
// episode starts in step order.  Blocks after them copy the batch's last
// min(T, W) exceed bytes into the rings, grid-stride.
__global__ __launch_bounds__(LED_NT) void ledger_finish_kernel(const gd_ledger_args a) {
    const uint32_t node_blocks = (a.N + LED_NT - 1) / LED_NT;
    const uint32_t W = a.W, T = a.T, N = a.N, R = a.R;
    const uint32_t keep = T < W ? T : W;
    if (blockIdx.x >= node_blocks) {
        uint8_t* rring = a.led + a.lay.rank_ring;
        uint8_t* nring = a.led + a.lay.node_ring;
        const size_t stride = (size_t)(gridDim.x - node_blocks) * LED_NT;
        const size_t me = (size_t)(blockIdx.x - node_blocks) * LED_NT + threadIdx.x;
        // ranks four at a time (R is a multiple of 8 and both arrays are word-aligned)
        const size_t rwords = (size_t)keep * (R / 4);
        for (size_t q = me; q < rwords; q += stride) {
            const uint32_t s = T - keep + (uint32_t)(q / (R / 4));
            const uint32_t r4 = (uint32_t)(q % (R / 4));
            const uint32_t v = reinterpret_cast<const uint32_t*>(a.exceed_mask + (size_t)s * R)[r4];
            reinterpret_cast<uint32_t*>(rring + (size_t)((a.first_step + s) % W) * R)[r4] = v;
        }
        const size_t nbytes = (size_t)keep * N;
        for (size_t q = me; q < nbytes; q += stride) {
            const uint32_t s = T - keep + (uint32_t)(q / N);
            const uint32_t n = (uint32_t)(q % N);
            nring[(size_t)((a.first_step + s) % W) * N + n] = a.node_mask[(size_t)s * N + n];
        }
        if (T > a.chunk) {       // the batch was cut into chunks: its final counts wait in the staging span
            const uint32_t* from = reinterpret_cast<const uint32_t*>(a.counts_new);
            uint32_t* to = reinterpret_cast<uint32_t*>(a.led + a.lay.rank_cnt);
            for (size_t q = me; q < a.lay.counts_bytes / 4; q += stride) to[q] = from[q];
        }
        return;
    }
    const uint32_t n = blockIdx.x * LED_NT + threadIdx.x;
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    if (n - lane >= N) return;
    const bool live = n < N;
    const uint32_t i = live ? n : N - 1;
    if (n == 0) reinterpret_cast<uint64_t*>(a.led + a.lay.head)[0] = a.first_step + T;

    // score ring and sum
    int16_t* qring = reinterpret_cast<int16_t*>(a.led + a.lay.node_qring);
    int32_t* qsum = reinterpret_cast<int32_t*>(a.led + a.lay.node_qsum);
    if (live) {
        int32_t sum = T >= W ? 0 : qsum[i];
        for (uint32_t s = T - keep; s < T; s += LED_AHEAD) {
            float z[LED_AHEAD];
            int32_t old[LED_AHEAD];
#pragma unroll
            for (int q = 0; q < LED_AHEAD; ++q) {
                z[q] = 0.0f; old[q] = 0;
                if (s + q < T) {
                    z[q] = a.node_z[(size_t)(s + q) * N + i];
                    // (zero while the window is still filling; a batch of W steps or more starts afresh)
                    if (T < W) old[q] = qring[(size_t)((a.first_step + s + q) % W) * N + i];
                }
            }
#pragma unroll
            for (int q = 0; q < LED_AHEAD; ++q) {
                if (s + q >= T) break;
                const int32_t v = quantise(z[q], a.quant);
                sum += v - old[q];
                qring[(size_t)((a.first_step + s + q) % W) * N + i] = (int16_t)v;
            }
        }
        qsum[i] = sum;
    }

    // episode starts, in step order: lane l fetches the word of step s + l, and the few
    // words that hold a start are handed round
    const uint64_t* rise = a.rise;
    int32_t* starts = reinterpret_cast<int32_t*>(a.led + a.lay.node_starts);
    int32_t* term = reinterpret_cast<int32_t*>(a.led + a.lay.node_term);
    const uint32_t word = __builtin_amdgcn_readfirstlane(n / 64);
    int32_t st[MAX_STARTS];
#pragma unroll
    for (int j = 0; j < MAX_STARTS; ++j) st[j] = starts[(size_t)j * N + i];
    int32_t tf = term[i];
    bool changed = false;
    constexpr int BLOCKS = 4;                               // 64-step words fetched together
    for (uint32_t s = 0; s < T; s += BLOCKS * WAVE) {
        uint64_t v[BLOCKS];
#pragma unroll
        for (int q = 0; q < BLOCKS; ++q) {
            const uint32_t sq = s + q * WAVE + lane;
            v[q] = sq < T ? rise[(size_t)word * T + sq] : 0ull;
        }
#pragma unroll
        for (int q = 0; q < BLOCKS; ++q) {
            uint64_t any = __ballot(v[q] != 0);
            while (any) {
                const int j = __builtin_ctzll(any);
                any &= any - 1;
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v[q], j);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v[q] >> 32), j);
                const uint64_t w = ((uint64_t)hi << 32) | lo;
                if (!((w >> lane) & 1ull)) continue;
                const int64_t t = (int64_t)(a.first_step + s + q * WAVE + j);
#pragma unroll
                for (int jj = MAX_STARTS - 1; jj > 0; --jj) st[jj] = st[jj - 1];
                st[0] = (int32_t)t + 1;
                changed = true;
                // episodes that began inside (t - horizon, t], this one included
                uint32_t inside = 0;
#pragma unroll
                for (int jj = 0; jj < MAX_STARTS; ++jj)
                    inside += (st[jj] != 0 && (int64_t)(st[jj] - 1) + (int64_t)a.horizon > t) ? 1u : 0u;
                if (inside >= a.limit && tf == 0) tf = (int32_t)t + 1;
            }
        }
    }
    if (live && changed) {
#pragma unroll
        for (int j = 0; j < MAX_STARTS; ++j) starts[(size_t)j * N + i] = st[j];
        term[i] = tf;
    }
}

__global__ __launch_bounds__(LED_NT) void ledger_flags_kernel(const gd_ledger_flags_args a) {
    const uint32_t i = blockIdx.x * LED_NT + threadIdx.x;
    auto read_out = [&](const uint16_t* cnt, const uint32_t* first, uint32_t n_items, uint8_t* pmask,
                        uint8_t* pflag, int32_t* pfirst) {
        uint32_t c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            c[j] = (uint32_t)cnt[(size_t)(2 * j) * n_items + i] |
                   ((uint32_t)cnt[(size_t)(2 * j + 1) * n_items + i] << 16);
        const uint32_t pm = sustained(c, a.K);
        if (pmask) pmask[i] = (uint8_t)pm;
        if (pflag) pflag[i] = (uint8_t)combine(pm, a.primary, a.min_signals);
        if (pfirst) pfirst[i] = first[i] ? (int32_t)(0xFFFFFFFFu - first[i]) : -1;
    };
    if (i < a.R)
        read_out(reinterpret_cast<const uint16_t*>(a.led + a.lay.rank_cnt),
                 reinterpret_cast<const uint32_t*>(a.led + a.lay.rank_first), a.R, a.rank_pmask,
                 a.rank_pflag, a.rank_pfirst);
    if (i < a.N) {
        read_out(reinterpret_cast<const uint16_t*>(a.led + a.lay.node_cnt),
                 reinterpret_cast<const uint32_t*>(a.led + a.lay.node_first), a.N, a.node_pmask,
                 a.node_pflag, a.node_pfirst);
        if (a.node_score_sum)
            a.node_score_sum[i] = reinterpret_cast<const int32_t*>(a.led + a.lay.node_qsum)[i];
        const int32_t* starts = reinterpret_cast<const int32_t*>(a.led + a.lay.node_starts);
        const uint64_t next = reinterpret_cast<const uint64_t*>(a.led + a.lay.head)[0];
        if (a.node_episodes) {
            uint32_t inside = 0;
            if (next > 0) {
                const int64_t t = (int64_t)next - 1;        // the last step taken in
#pragma unroll
                for (int j = 0; j < MAX_STARTS; ++j) {
                    const int32_t st = starts[(size_t)j * a.N + i];
                    inside += (st != 0 && (int64_t)(st - 1) + (int64_t)a.horizon > t) ? 1u : 0u;
                }
            }
            a.node_episodes[i] = (uint8_t)min(inside, a.limit);
        }
        if (a.node_terminal_first)
            a.node_terminal_first[i] = reinterpret_cast<const int32_t*>(a.led + a.lay.node_term)[i] - 1;
    }
}

}  // namespace

hipError_t gd_launch_ledger(const gd_ledger_args& a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    if (a.chunk == 0 || a.limit < 1 || a.limit > (uint32_t)MAX_STARTS) return hipErrorInvalidValue;
    const uint32_t item_blocks = (a.R / RANK_IPT + LED_NT - 1) / LED_NT + (a.N + LED_NT - 1) / LED_NT;
    const uint32_t chunks = (a.T + a.chunk - 1) / a.chunk;
    if (chunks > 65535u) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ledger_count_kernel, dim3(item_blocks, chunks), dim3(LED_NT), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint32_t node_blocks = (a.N + LED_NT - 1) / LED_NT;
    const size_t keep = a.T < a.W ? a.T : a.W;
    const size_t copy_units = keep * (a.R / 4);
    uint32_t copy_blocks = (uint32_t)((copy_units + LED_NT * 4 - 1) / (LED_NT * 4));
    copy_blocks = copy_blocks < 1 ? 1 : (copy_blocks > 2048 ? 2048 : copy_blocks);
    hipLaunchKernelGGL(ledger_finish_kernel, dim3(node_blocks + copy_blocks), dim3(LED_NT), 0, s, a);
    return hipGetLastError();
}

// Work spans for callers that may not allocate (code under graph capture, serving loops
// that forbid hipMalloc): one array per GPU, held from the first use until the process
// ends.  Host code never uses the array's name as an address: the device address is
// asked for once per device and kept.
constexpr size_t LEDGER_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[LEDGER_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_DEVICES];     // device address of `scratch` on each GPU, null = not asked yet
}  // namespace

size_t gd_ledger_static_bytes() { return LEDGER_SCRATCH_BYTES; }

hipError_t gd_launch_ledger_static(gd_ledger_args a, hipStream_t s, bool* fits) {
    *fits = true;
    if (a.T == 0) return hipSuccess;
    const size_t NW = ((size_t)a.N + 63) / 64;
    const size_t rise_bytes = ((size_t)a.T * NW * 8 + 255) & ~(size_t)255;
    if (rise_bytes + a.lay.counts_bytes > LEDGER_SCRATCH_BYTES) { *fits = false; return hipSuccess; }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    // Nothing in either span has to start at zero: the counting kernel writes every
    // (node word, step) of the map and every staged count before the finishing kernel,
    // behind it on the stream, reads them.
    a.rise = reinterpret_cast<uint64_t*>(g_scratch_ptr[dev]);
    a.counts_new = g_scratch_ptr[dev] + rise_bytes;
    return gd_launch_ledger(a, s);
}

hipError_t gd_launch_ledger_flags(const gd_ledger_flags_args& a, hipStream_t s) {
    const uint32_t blocks = (a.R + LED_NT - 1) / LED_NT;
    hipLaunchKernelGGL(ledger_flags_kernel, dim3(blocks), dim3(LED_NT), 0, s, a);
    return hipGetLastError();
}
