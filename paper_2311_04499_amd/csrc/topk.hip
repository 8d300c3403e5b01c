// Fine-grained top-k sparsifier with error feedback: the contrast point to the
// coarse filter (Sec. I and Table II: "most of the overhead in Top-k comes from
// the topk() operator").  Exact, deterministic, no sampling.
//
//   pass 1   A = fma(c, R, G); R <- A; histogram of key bits 30..20        (reads 2D, writes D)
//            -> the bin b1 that holds the k-th largest key
//   collect  one more read of R: every element whose bin is >= b1 is copied, in
//            index order, into a 32-entry slot array of its 1024-element tile, and
//            the histogram of bits 19..9 among bin b1 is taken on the way    (reads D)
//   then everything works on the slots only (about 0.3 % of the data): histogram
//   of bits 8..0 -> threshold key T and the number of ties to keep; per-tile
//   counts; 3-phase exclusive scan; ordered write of (value, index), R <- +0 there.
//
// If any tile has more than 32 such elements (heavily clustered or tied data) a
// flag is raised on the device and the general path runs instead: two more
// full histogram passes, a counting pass and a compaction pass over R (4 more
// reads of D).  The host launches both tails; every kernel of the tail that is
// not taken returns at once, so no host round trip is needed.  Both tails give
// the same bits.
//
// key = bit pattern of |A| as an unsigned integer: a total order on magnitudes
// (NaN above Inf).  Among keys equal to T the lowest indices are kept, which
// makes the result unique.  Every decision is integer work on bit patterns.
//
// Histograms live in LDS per workgroup (a copy per wave) and are flushed once
// per workgroup; compaction uses wavefront prefix sums (one-wave workgroups, so
// no barriers).  All scratch is in the caller's workspace; nothing is allocated.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBins12 = 2048;  // digits of levels 1 and 2: key bits 30..20 and 19..9
constexpr int kBins3 = 512;    // digit of level 3: key bits 8..0
constexpr int kHistThreads = 256;
constexpr int kHistWaves = kHistThreads / 64;
constexpr int kTile = 1024;        // elements per compaction tile: 64 lanes x 4 vectors x 4 elements
constexpr int kScanChunk = 1024;   // tile counts scanned per workgroup in phase A
constexpr uint32_t kAbs = 0x7fffffffu;

// Selection state, first words of the workspace.
struct topk_state {
    uint32_t prefix;     // key bits fixed so far (in place, low bits zero)
    uint32_t k_rem;      // how many are still to be taken from the current bin
    uint32_t threshold;  // T, valid after level 3
    uint32_t ties;       // number of keys == T to keep, valid after level 3
    uint32_t overflow;   // != 0: some tile did not fit its slots, the general tail runs
    uint32_t pad[3];
};

constexpr int kSlots = 32;  // slot entries per 1024-element tile
// Histograms may be kept as several partial copies ("slices") that the pick
// kernel adds up.  Global atomics run at about 1.5 G/s on this chip whatever the
// address spread (320 k of them cost 200 us), so the slot passes, whose entries are
// few, build LDS histograms and store them as slices without any global atomic;
// the full-data passes flush one LDS histogram per workgroup (a few dozen
// non-empty bins each) and need no slicing.
constexpr int kHistSlices = 1;    // full-data passes: workgroup w adds into slice w mod kHistSlices
constexpr int kSlotGrid = 64;     // slot passes: one slice per workgroup, written with plain stores
constexpr int kSlotThreads = 512;
constexpr int kHistRows = 3 * kHistSlices + 2 * kSlotGrid;  // rows of 2048 counters in the workspace
enum { kAlways = 0, kSlotTail = 1, kGeneralTail = 2 };

// True if a kernel of tail `gate` has nothing to do.
__device__ __forceinline__ bool skip_tail(const topk_state *st, int gate)
{
    const uint32_t ov = st->overflow;
    return (gate == kSlotTail && ov != 0u) || (gate == kGeneralTail && ov == 0u);
}

struct topk_ws {
    topk_state *state;
    uint32_t *hist;       // [kHistRows][2048]: level 1 | general tail levels 2, 3 | slot tail levels 2, 3
    uint32_t *slot_cnt;   // [ntiles]
    uint32_t *slot_idx;   // [ntiles][kSlots]
    uint32_t *slot_bits;  // [ntiles][kSlots]  bit patterns of A
    uint32_t *cnt_gt;     // [ntiles]  -> exclusive prefix after the scan
    uint32_t *cnt_eq;     // [ntiles]
    uint32_t *chunk_gt;   // [nchunks] -> exclusive prefix
    uint32_t *chunk_eq;   // [nchunks]
};

__host__ __device__ inline int64_t div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }

size_t ws_layout(int64_t n, void *base, topk_ws *out)
{
    const int64_t ntiles = div_up(n > 0 ? n : 1, kTile);
    const int64_t nchunks = div_up(ntiles, kScanChunk);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) / 256 * 256;
        return at;
    };
    const size_t o_state = take(sizeof(topk_state));
    const size_t o_hist = take((size_t)kHistRows * 2048 * sizeof(uint32_t));
    const size_t o_scnt = take((size_t)ntiles * 4);
    const size_t o_sidx = take((size_t)ntiles * kSlots * 4);
    const size_t o_sbits = take((size_t)ntiles * kSlots * 4);
    const size_t o_gt = take((size_t)ntiles * 4);
    const size_t o_eq = take((size_t)ntiles * 4);
    const size_t o_cgt = take((size_t)nchunks * 4);
    const size_t o_ceq = take((size_t)nchunks * 4);
    if (out) {
        char *b = (char *)base;
        out->state = (topk_state *)(b + o_state);
        out->hist = (uint32_t *)(b + o_hist);
        out->slot_cnt = (uint32_t *)(b + o_scnt);
        out->slot_idx = (uint32_t *)(b + o_sidx);
        out->slot_bits = (uint32_t *)(b + o_sbits);
        out->cnt_gt = (uint32_t *)(b + o_gt);
        out->cnt_eq = (uint32_t *)(b + o_eq);
        out->chunk_gt = (uint32_t *)(b + o_cgt);
        out->chunk_eq = (uint32_t *)(b + o_ceq);
    }
    return off;
}

// ---- wavefront helpers (64 lanes) ---------------------------------------------

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// ---- init ------------------------------------------------------------------------

__global__ void k_topk_init(topk_state *st, uint32_t *hist, uint32_t k)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kHistRows * 2048; i += gridDim.x * blockDim.x)
        hist[i] = 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->prefix = 0u;
        st->k_rem = k;
        st->threshold = 0u;
        st->ties = 0u;
        st->overflow = 0u;
    }
}

// ---- histogram passes ----------------------------------------------------------------

// LEVEL 1: error feedback + residual write + histogram of bits 30..20.
// LEVEL 2/3: histogram of the next digit among keys that match the prefix.
// Persistent workgroups: each walks tiles of kHistThreads vectors with a grid
// stride and keeps one LDS histogram per wave.
template <int LEVEL>
__global__ __launch_bounds__(kHistThreads) void k_topk_hist(const float *__restrict__ G, float *R,
                                                            int64_t n, float c,
                                                            const topk_state *__restrict__ st,
                                                            uint32_t *__restrict__ hist)
{
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int SHIFT = LEVEL == 1 ? 20 : (LEVEL == 2 ? 9 : 0);
    constexpr int HI_SHIFT = LEVEL == 2 ? 20 : 9;  // bits above this digit (levels 2, 3)
    __shared__ uint32_t lds[kHistWaves][BINS];
    const int tid = threadIdx.x;
    uint32_t want = 0u;
    if constexpr (LEVEL > 1) {
        if (skip_tail(st, kGeneralTail)) return;  // same answer for every thread of the grid
        want = st->prefix >> HI_SHIFT;
    }
    uint32_t *mine = lds[tid >> 6];
    for (int i = tid; i < kHistWaves * BINS; i += kHistThreads) (&lds[0][0])[i] = 0u;
    __syncthreads();

    const int64_t nvec = n / 4;
    const int64_t stride = (int64_t)gridDim.x * kHistThreads;
    for (int64_t v = (int64_t)blockIdx.x * kHistThreads + tid; v < nvec; v += stride) {
        u32x4 key;
        if constexpr (LEVEL == 1) {
            const f32x4 g = __builtin_nontemporal_load((const f32x4 *)G + v);
            const f32x4 r = __builtin_nontemporal_load((const f32x4 *)R + v);
            f32x4 a;
            a.x = __builtin_fmaf(c, r.x, g.x);
            a.y = __builtin_fmaf(c, r.y, g.y);
            a.z = __builtin_fmaf(c, r.z, g.z);
            a.w = __builtin_fmaf(c, r.w, g.w);
            ((f32x4 *)R)[v] = a;  // read again by the later passes: keep it cacheable
            key = __builtin_bit_cast(u32x4, a) & kAbs;
            atomicAdd(&mine[key.x >> SHIFT], 1u);
            atomicAdd(&mine[key.y >> SHIFT], 1u);
            atomicAdd(&mine[key.z >> SHIFT], 1u);
            atomicAdd(&mine[key.w >> SHIFT], 1u);
        } else {
            key = __builtin_nontemporal_load((const u32x4 *)R + v) & kAbs;
            if ((key.x >> HI_SHIFT) == want) atomicAdd(&mine[(key.x >> SHIFT) & (BINS - 1)], 1u);
            if ((key.y >> HI_SHIFT) == want) atomicAdd(&mine[(key.y >> SHIFT) & (BINS - 1)], 1u);
            if ((key.z >> HI_SHIFT) == want) atomicAdd(&mine[(key.z >> SHIFT) & (BINS - 1)], 1u);
            if ((key.w >> HI_SHIFT) == want) atomicAdd(&mine[(key.w >> SHIFT) & (BINS - 1)], 1u);
        }
    }
    // scalar tail (n mod 4 elements), one workgroup only
    if (blockIdx.x == 0 && tid < (int)(n - nvec * 4)) {
        const int64_t i = nvec * 4 + tid;
        uint32_t key;
        if constexpr (LEVEL == 1) {
            const float a = __builtin_fmaf(c, R[i], G[i]);
            R[i] = a;
            key = __float_as_uint(a) & kAbs;
            atomicAdd(&mine[key >> SHIFT], 1u);
        } else {
            key = __float_as_uint(R[i]) & kAbs;
            if ((key >> HI_SHIFT) == want) atomicAdd(&mine[(key >> SHIFT) & (BINS - 1)], 1u);
        }
    }
    __syncthreads();
    for (int b = tid; b < BINS; b += kHistThreads) {
        uint32_t s = 0u;
#pragma unroll
        for (int w = 0; w < kHistWaves; ++w) s += lds[w][b];
        if (s) atomicAdd(&hist[(blockIdx.x % kHistSlices) * 2048 + b], s);
    }
}

// Finds the digit at which the count from the top reaches k_rem: the largest b
// with sum_{j >= b} hist[j] >= k_rem.  One workgroup of 256 threads.
constexpr int kPickThreads = 1024;  // all of them add up the slices; the first 256 then scan

template <int LEVEL, int GATE>
__global__ __launch_bounds__(kPickThreads) void k_topk_pick(topk_state *st,
                                                           const uint32_t *__restrict__ hist,
                                                           int nslices)
{
    if (skip_tail(st, GATE)) return;
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int PER = BINS / 256;
    constexpr int SHIFT = LEVEL == 1 ? 20 : (LEVEL == 2 ? 9 : 0);
    __shared__ uint32_t part[256];
    __shared__ uint32_t total[BINS];
    const int tid = threadIdx.x;
    const uint32_t k_rem = st->k_rem;
    for (int bin = tid; bin < BINS; bin += kPickThreads) {  // neighbouring threads read neighbouring counters
        uint32_t c[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        int sl = 0;
        for (; sl + 8 <= nslices; sl += 8) {  // eight independent loads in flight
#pragma unroll
            for (int j = 0; j < 8; ++j) c[j] += hist[(sl + j) * 2048 + bin];
        }
        for (; sl < nslices; ++sl) c[0] += hist[sl * 2048 + bin];
        total[bin] = ((c[0] + c[1]) + (c[2] + c[3])) + ((c[4] + c[5]) + (c[6] + c[7]));
    }
    __syncthreads();
    // The scan is the work of the first 256 threads; the others only keep every
    // barrier complete (a barrier must be reached by all threads of the workgroup).
    const bool scanner = tid < 256;
    // scanner t owns bins [BINS - (t+1)*PER, BINS - t*PER): thread 0 the top ones
    uint32_t h[PER];
    uint32_t mine = 0u;
    if (scanner) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            h[j] = total[BINS - 1 - (tid * PER + j)];  // descending bin order
            mine += h[j];
        }
        part[tid] = mine;
    }
    __syncthreads();
    // inclusive scan over the scanners (Hillis-Steele in LDS)
    for (int d = 1; d < 256; d <<= 1) {
        const uint32_t y = (scanner && tid >= d) ? part[tid - d] : 0u;
        __syncthreads();
        if (scanner) part[tid] += y;
        __syncthreads();
    }
    if (!scanner) return;  // no barrier follows
    const uint32_t incl = part[tid], excl = incl - mine;
    if (k_rem > 0u && excl < k_rem && k_rem <= incl) {  // exactly one thread
        uint32_t above = excl;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (above + h[j] >= k_rem) {
                const uint32_t bin = (uint32_t)(BINS - 1 - (tid * PER + j));
                const uint32_t prefix = st->prefix | (bin << SHIFT);
                st->prefix = prefix;
                st->k_rem = k_rem - above;
                if (LEVEL == 3) {
                    st->threshold = prefix;
                    st->ties = k_rem - above;
                }
                break;
            }
            above += h[j];
        }
    }
}

// ---- per-tile counts, scan, compaction -------------------------------------------------

__device__ __forceinline__ u32x4 load_keys(const float *R, int64_t n, int64_t e, uint32_t *valid)
{
    // four keys starting at element e (e is a multiple of 4); lanes past n are
    // flagged invalid (their key reads as 0 but must not count as a tie at T = 0)
    u32x4 k = {0u, 0u, 0u, 0u};
    *valid = 0u;
    if (e + 4 <= n) {
        k = __builtin_nontemporal_load((const u32x4 *)(R + e)) & kAbs;
        *valid = 0xfu;
    } else {
        for (int j = 0; j < 4; ++j)
            if (e + j < n) {
                k[j] = __float_as_uint(R[e + j]) & kAbs;
                *valid |= 1u << j;
            }
    }
    return k;
}

__global__ __launch_bounds__(64) void k_topk_count(const float *__restrict__ R, int64_t n, int64_t ntiles,
                                                   const topk_state *__restrict__ st,
                                                   uint32_t *__restrict__ cnt_gt,
                                                   uint32_t *__restrict__ cnt_eq)
{
    if (skip_tail(st, kGeneralTail)) return;
    const uint32_t T = st->threshold;
    const int lane = threadIdx.x;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t base = tile * kTile;
        uint32_t gt = 0u, eq = 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
            uint32_t valid;
            const u32x4 k = load_keys(R, n, e, &valid);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool ok = (valid >> j) & 1u;
                gt += (ok && k[j] > T) ? 1u : 0u;
                eq += (ok && k[j] == T) ? 1u : 0u;
            }
        }
        gt = wave_sum(gt);
        eq = wave_sum(eq);
        if (lane == 0) {
            cnt_gt[tile] = gt;
            cnt_eq[tile] = eq;
        }
    }
}

// Phase A: each workgroup turns kScanChunk tile counts into chunk-local
// exclusive prefixes and writes the chunk totals.
__global__ __launch_bounds__(256) void k_topk_scan_a(uint32_t *cnt_gt, uint32_t *cnt_eq,
                                                     int64_t ntiles, uint32_t *chunk_gt,
                                                     uint32_t *chunk_eq)
{
    __shared__ uint32_t sg[256], se[256];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + tid * 4;
    uint32_t g[4], e[4], tg = 0u, te = 0u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool ok = base + j < ntiles;
        g[j] = ok ? cnt_gt[base + j] : 0u;
        e[j] = ok ? cnt_eq[base + j] : 0u;
        tg += g[j];
        te += e[j];
    }
    sg[tid] = tg;
    se[tid] = te;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {
        const uint32_t yg = tid >= d ? sg[tid - d] : 0u, ye = tid >= d ? se[tid - d] : 0u;
        __syncthreads();
        sg[tid] += yg;
        se[tid] += ye;
        __syncthreads();
    }
    uint32_t pg = sg[tid] - tg, pe = se[tid] - te;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (base + j < ntiles) {
            cnt_gt[base + j] = pg;
            cnt_eq[base + j] = pe;
        }
        pg += g[j];
        pe += e[j];
    }
    if (tid == 255) {
        chunk_gt[blockIdx.x] = sg[255];
        chunk_eq[blockIdx.x] = se[255];
    }
}

// Phase B: one workgroup scans the chunk totals in place (exclusive).
__global__ __launch_bounds__(256) void k_topk_scan_b(uint32_t *chunk_gt, uint32_t *chunk_eq,
                                                     int64_t nchunks)
{
    __shared__ uint32_t sg[256], se[256];
    __shared__ uint32_t carry_g, carry_e;
    const int tid = threadIdx.x;
    if (tid == 0) {
        carry_g = 0u;
        carry_e = 0u;
    }
    __syncthreads();
    for (int64_t base = 0; base < nchunks; base += 256) {
        const int64_t i = base + tid;
        const uint32_t g = i < nchunks ? chunk_gt[i] : 0u, e = i < nchunks ? chunk_eq[i] : 0u;
        sg[tid] = g;
        se[tid] = e;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const uint32_t yg = tid >= d ? sg[tid - d] : 0u, ye = tid >= d ? se[tid - d] : 0u;
            __syncthreads();
            sg[tid] += yg;
            se[tid] += ye;
            __syncthreads();
        }
        if (i < nchunks) {
            chunk_gt[i] = carry_g + sg[tid] - g;
            chunk_eq[i] = carry_e + se[tid] - e;
        }
        __syncthreads();
        if (tid == 255) {
            carry_g += sg[255];
            carry_e += se[255];
        }
        __syncthreads();
    }
}

// Pass 5: one wave per tile.  Element order inside a tile is (round u, lane,
// component), which is ascending index; ranks come from wavefront prefix sums.
__global__ __launch_bounds__(64) void k_topk_write(float *R, int64_t n,
                                                   const topk_state *__restrict__ st,
                                                   const uint32_t *__restrict__ cnt_gt,
                                                   const uint32_t *__restrict__ cnt_eq,
                                                   const uint32_t *__restrict__ chunk_gt,
                                                   const uint32_t *__restrict__ chunk_eq,
                                                   int64_t ntiles, float *__restrict__ vals,
                                                   uint32_t *__restrict__ idx, uint32_t kmax)
{
    if (skip_tail(st, kGeneralTail)) return;
    const uint32_t T = st->threshold, ties = st->ties;
    const int lane = threadIdx.x;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t chunk = tile / kScanChunk;
        const uint32_t gt_before = chunk_gt[chunk] + cnt_gt[tile];
        uint32_t eq_before = chunk_eq[chunk] + cnt_eq[tile];
        uint32_t out_pos = gt_before + (eq_before < ties ? eq_before : ties);
        const int64_t base = tile * kTile;
#pragma unroll 1
        for (int u = 0; u < 4; ++u) {
            const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
            uint32_t valid;
            const u32x4 k = load_keys(R, n, e, &valid);
            uint32_t gtm = 0u, eqm = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool ok = (valid >> j) & 1u;
                gtm |= (ok && k[j] > T) ? (1u << j) : 0u;
                eqm |= (ok && k[j] == T) ? (1u << j) : 0u;
            }
            if (__ballot((gtm | eqm) != 0u) == 0ull) continue;  // nothing to keep in this round
            const uint32_t eq_cnt = __popc(eqm);
            const uint32_t eq_incl = wave_incl_scan(eq_cnt);
            const uint32_t eq_total = __shfl(eq_incl, 63, 64);
            uint32_t eq_rank = eq_before + eq_incl - eq_cnt;  // rank of this lane's first tie
            uint32_t selm = gtm;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if ((eqm >> j) & 1u) {
                    if (eq_rank < ties) selm |= 1u << j;
                    ++eq_rank;
                }
            }
            const uint32_t sel_cnt = __popc(selm);
            const uint32_t sel_incl = wave_incl_scan(sel_cnt);
            const uint32_t sel_total = __shfl(sel_incl, 63, 64);
            uint32_t pos = out_pos + sel_incl - sel_cnt;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (((selm >> j) & 1u) && pos < kmax) {  // pos < kmax always holds (see above)
                    const int64_t i = e + j;
                    vals[pos] = R[i];
                    idx[pos] = (uint32_t)i;
                    R[i] = 0.0f;
                    ++pos;
                }
            }
            eq_before += eq_total;
            out_pos += sel_total;
        }
    }
}

// ---- slot tail -------------------------------------------------------------------------

// One wave per 1024-element tile: copies (index, bits) of every element whose
// level-1 bin is >= the bin of the k-th largest key into the tile's slots, in
// index order.
__global__ __launch_bounds__(64) void k_topk_collect(const float *__restrict__ R, int64_t n,
                                                     topk_state *st, uint32_t *__restrict__ slot_cnt,
                                                     uint32_t *__restrict__ slot_idx,
                                                     uint32_t *__restrict__ slot_bits)
{
    const uint32_t b1 = st->prefix >> 20;
    const int lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kTile;
    uint32_t running = 0u;
    u32x4 raws[4];
    uint32_t valids[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // all four loads are in flight before the first is used
        const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
        raws[u] = u32x4{0u, 0u, 0u, 0u};
        valids[u] = 0u;
        if (e + 4 <= n) {
            raws[u] = __builtin_nontemporal_load((const u32x4 *)(R + e));
            valids[u] = 0xfu;
        } else {
            for (int j = 0; j < 4; ++j)
                if (e + j < n) {
                    raws[u][j] = __float_as_uint(R[e + j]);
                    valids[u] |= 1u << j;
                }
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
        const u32x4 raw = raws[u];
        const uint32_t valid = valids[u];
        uint32_t m = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            m |= (((valid >> j) & 1u) && ((raw[j] & kAbs) >> 20) >= b1) ? (1u << j) : 0u;
        if (__ballot(m != 0u) == 0ull) continue;
        const uint32_t cnt = __popc(m);
        const uint32_t incl = wave_incl_scan(cnt);
        const uint32_t total = __shfl(incl, 63, 64);
        uint32_t pos = running + incl - cnt;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if ((m >> j) & 1u) {
                if (pos < (uint32_t)kSlots) {
                    slot_idx[tile * kSlots + pos] = (uint32_t)(e + j);
                    slot_bits[tile * kSlots + pos] = raw[j];
                }
                ++pos;
            }
        }
        running += total;
    }
    if (lane == 0) {
        slot_cnt[tile] = running < (uint32_t)kSlots ? running : (uint32_t)kSlots;
        if (running > (uint32_t)kSlots) atomicOr(&st->overflow, 1u);
    }
}

// The remaining slot-tail kernels give one thread to each tile (a tile holds
// four entries on average).

// Histogram of the next digit over the slot entries: a few large workgroups, each
// with an LDS histogram that it stores as its own slice.
template <int LEVEL>
__global__ __launch_bounds__(kSlotThreads) void k_topk_slots_hist(const topk_state *__restrict__ st,
                                                                  const uint32_t *__restrict__ slot_cnt,
                                                                  const uint32_t *__restrict__ slot_bits,
                                                                  int64_t ntiles,
                                                                  uint32_t *__restrict__ hist)
{
    if (skip_tail(st, kSlotTail)) return;
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int SHIFT = LEVEL == 2 ? 9 : 0;
    constexpr int HI_SHIFT = LEVEL == 2 ? 20 : 9;
    __shared__ uint32_t lds[BINS];
    const int tid = threadIdx.x;
    for (int i = tid; i < BINS; i += kSlotThreads) lds[i] = 0u;
    __syncthreads();
    const uint32_t want = st->prefix >> HI_SHIFT;
    for (int64_t tile = (int64_t)blockIdx.x * kSlotThreads + tid; tile < ntiles;
         tile += (int64_t)gridDim.x * kSlotThreads) {
        const uint32_t cnt = slot_cnt[tile];
        for (uint32_t i = 0; i < cnt; ++i) {
            const uint32_t key = slot_bits[tile * kSlots + i] & kAbs;
            if ((key >> HI_SHIFT) == want) atomicAdd(&lds[(key >> SHIFT) & (BINS - 1)], 1u);
        }
    }
    __syncthreads();
    for (int i = tid; i < BINS; i += kSlotThreads) hist[blockIdx.x * 2048 + i] = lds[i];
}

__global__ __launch_bounds__(256) void k_topk_slots_count(const topk_state *__restrict__ st,
                                                          const uint32_t *__restrict__ slot_cnt,
                                                          const uint32_t *__restrict__ slot_bits,
                                                          int64_t ntiles, uint32_t *__restrict__ cnt_gt,
                                                          uint32_t *__restrict__ cnt_eq)
{
    if (skip_tail(st, kSlotTail)) return;
    const int64_t tile = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tile >= ntiles) return;
    const uint32_t T = st->threshold;
    const uint32_t cnt = slot_cnt[tile];
    uint32_t gt = 0u, eq = 0u;
    for (uint32_t i = 0; i < cnt; ++i) {
        const uint32_t key = slot_bits[tile * kSlots + i] & kAbs;
        gt += key > T ? 1u : 0u;
        eq += key == T ? 1u : 0u;
    }
    cnt_gt[tile] = gt;
    cnt_eq[tile] = eq;
}

__global__ __launch_bounds__(256) void k_topk_slots_write(float *R, const topk_state *__restrict__ st,
                                                          const uint32_t *__restrict__ slot_cnt,
                                                          const uint32_t *__restrict__ slot_idx,
                                                          const uint32_t *__restrict__ slot_bits,
                                                          const uint32_t *__restrict__ cnt_gt,
                                                          const uint32_t *__restrict__ cnt_eq,
                                                          const uint32_t *__restrict__ chunk_gt,
                                                          const uint32_t *__restrict__ chunk_eq,
                                                          int64_t ntiles, float *__restrict__ vals,
                                                          uint32_t *__restrict__ idx, uint32_t kmax)
{
    if (skip_tail(st, kSlotTail)) return;
    const int64_t tile = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tile >= ntiles) return;
    const uint32_t cnt = slot_cnt[tile];
    if (cnt == 0u) return;
    const uint32_t T = st->threshold, ties = st->ties;
    const int64_t chunk = tile / kScanChunk;
    uint32_t eq_before = chunk_eq[chunk] + cnt_eq[tile];
    uint32_t pos = chunk_gt[chunk] + cnt_gt[tile] + (eq_before < ties ? eq_before : ties);
    for (uint32_t i = 0; i < cnt; ++i) {  // entries are in ascending index order
        const uint32_t bits = slot_bits[tile * kSlots + i];
        const uint32_t key = bits & kAbs;
        bool keep = key > T;
        if (key == T) {
            keep = eq_before < ties;
            ++eq_before;
        }
        if (keep && pos < kmax) {  // pos < kmax always holds; the test keeps a corrupted workspace harmless
            const uint32_t at = slot_idx[tile * kSlots + i];
            vals[pos] = __uint_as_float(bits);
            idx[pos] = at;
            R[at] = 0.0f;
            ++pos;
        }
    }
}

covap_status_t check(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return covap::fail(COVAP_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    return COVAP_OK;
}

}  // namespace

extern "C" {

size_t topk_workspace_bytes(int64_t n, int32_t dtype)
{
    if (n < 0) return 0;
    return ws_layout(n, nullptr, nullptr);
}

covap_status_t topk_compress(const void *grad, void *residual, int64_t n, int64_t k, int32_t dtype,
                             float ef_coeff, void *out_vals, uint32_t *out_idx, void *workspace,
                             size_t ws_bytes, void *stream)
{
    covap::clear_error();
    if (dtype != COVAP_F32) return covap::fail(COVAP_EUNSUPPORTED, "topk_compress: fp32 only");
    if (n < 0 || k < 0 || k > n) return covap::fail(COVAP_EINVAL, "topk_compress: need 0 <= k <= n");
    if (n >= ((int64_t)1 << 32)) return covap::fail(COVAP_EINVAL, "topk_compress: n >= 2^32");
    if (n == 0) return COVAP_OK;
    if (!grad || !residual || !workspace || (k > 0 && (!out_vals || !out_idx)))
        return covap::fail(COVAP_EINVAL, "topk_compress: null device pointer");
    if (((uintptr_t)grad & 15u) || ((uintptr_t)residual & 15u) || ((uintptr_t)workspace & 255u) ||
        ((uintptr_t)out_vals & 3u) || ((uintptr_t)out_idx & 3u))
        return covap::fail(COVAP_EINVAL, "topk_compress: misaligned device pointer");
    if (ws_bytes < ws_layout(n, nullptr, nullptr))
        return covap::fail(COVAP_EINVAL, "topk_compress: workspace too small");

    topk_ws ws;
    ws_layout(n, workspace, &ws);
    hipStream_t st = (hipStream_t)stream;
    const float *G = (const float *)grad;
    float *R = (float *)residual;
    const int64_t nvec = n / 4;
    const int64_t ntiles = div_up(n, kTile);
    const int64_t nchunks = div_up(ntiles, kScanChunk);
    // persistent histogram grid: enough workgroups to fill 256 CUs several times over
    int64_t hist_grid = div_up(nvec > 0 ? nvec : 1, kHistThreads);
    if (hist_grid > 2048) hist_grid = 2048;

    uint32_t *h1 = ws.hist, *h2g = h1 + kHistSlices * 2048, *h3g = h2g + kHistSlices * 2048,
             *h2s = h3g + kHistSlices * 2048, *h3s = h2s + kSlotGrid * 2048;
    const uint32_t per_tile_grid = (uint32_t)div_up(ntiles, 256);
    // the general tail's tile kernels walk the tiles with a bounded grid, so that
    // they cost next to nothing when they are not taken
    const uint32_t tail_grid = (uint32_t)(ntiles < 16384 ? ntiles : 16384);
    k_topk_init<<<64, 256, 0, st>>>(ws.state, ws.hist, (uint32_t)k);
    k_topk_hist<1><<<(uint32_t)hist_grid, kHistThreads, 0, st>>>(G, R, n, ef_coeff, ws.state, h1);
    if (k > 0) {
        k_topk_pick<1, kAlways><<<1, kPickThreads, 0, st>>>(ws.state, h1, kHistSlices);
        k_topk_collect<<<(uint32_t)ntiles, 64, 0, st>>>(R, n, ws.state, ws.slot_cnt, ws.slot_idx, ws.slot_bits);
        // slot tail (returns at once if a tile overflowed its slots)
        k_topk_slots_hist<2><<<kSlotGrid, kSlotThreads, 0, st>>>(ws.state, ws.slot_cnt, ws.slot_bits, ntiles, h2s);
        k_topk_pick<2, kSlotTail><<<1, kPickThreads, 0, st>>>(ws.state, h2s, kSlotGrid);
        k_topk_slots_hist<3><<<kSlotGrid, kSlotThreads, 0, st>>>(ws.state, ws.slot_cnt, ws.slot_bits, ntiles, h3s);
        k_topk_pick<3, kSlotTail><<<1, kPickThreads, 0, st>>>(ws.state, h3s, kSlotGrid);
        k_topk_slots_count<<<per_tile_grid, 256, 0, st>>>(ws.state, ws.slot_cnt, ws.slot_bits, ntiles, ws.cnt_gt, ws.cnt_eq);
        // general tail (returns at once otherwise)
        k_topk_hist<2><<<(uint32_t)hist_grid, kHistThreads, 0, st>>>(G, R, n, ef_coeff, ws.state, h2g);
        k_topk_pick<2, kGeneralTail><<<1, kPickThreads, 0, st>>>(ws.state, h2g, kHistSlices);
        k_topk_hist<3><<<(uint32_t)hist_grid, kHistThreads, 0, st>>>(G, R, n, ef_coeff, ws.state, h3g);
        k_topk_pick<3, kGeneralTail><<<1, kPickThreads, 0, st>>>(ws.state, h3g, kHistSlices);
        k_topk_count<<<tail_grid, 64, 0, st>>>(R, n, ntiles, ws.state, ws.cnt_gt, ws.cnt_eq);
        // common: exclusive scan of the per-tile counts, then the ordered write
        k_topk_scan_a<<<(uint32_t)nchunks, 256, 0, st>>>(ws.cnt_gt, ws.cnt_eq, ntiles, ws.chunk_gt, ws.chunk_eq);
        k_topk_scan_b<<<1, 256, 0, st>>>(ws.chunk_gt, ws.chunk_eq, nchunks);
        k_topk_slots_write<<<per_tile_grid, 256, 0, st>>>(R, ws.state, ws.slot_cnt, ws.slot_idx, ws.slot_bits, ws.cnt_gt,
                                                          ws.cnt_eq, ws.chunk_gt, ws.chunk_eq, ntiles,
                                                          (float *)out_vals, out_idx, (uint32_t)k);
        k_topk_write<<<tail_grid, 64, 0, st>>>(R, n, ws.state, ws.cnt_gt, ws.cnt_eq, ws.chunk_gt,
                                                     ws.chunk_eq, ntiles, (float *)out_vals, out_idx, (uint32_t)k);
    }
    return check("topk_compress");
}

}  // extern "C"
