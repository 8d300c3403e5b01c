// Fine-grained top-k sparsifier with error feedback: the contrast point to the
// coarse filter (Sec. I and Table II, where the selection operator accounts for
// nearly all of Top-k's compression time).  Exact and deterministic: a sample only
// decides how much work the exact selection has to do, never what it returns.
//
//   sample   A = fma(c, R, G) on 1024 evenly spread 256-element chunks; histogram of
//            key bits 30..20 -> a key t_lo that very probably lies at or below
//            the k-th largest key, with only a few times k keys at or above it                                          (reads 2 MB)
//   pass 1   A = fma(c, R, G); R <- A; every element whose key is >= t_lo is copied,
//            in index order, into a 32-entry slot array of its 1024-element tile
//                                                                (reads 2D, writes D)
//   then everything works on the slots only (a fraction of a percent of the data):
//   histograms of bits 30..20, 19..9 and 8..0 -> threshold key T and the number of
//   ties to keep; kept entries per chunk of 256 tiles and a scan of those totals;
//   ordered write of (value, index), R <- +0 there (positions inside a chunk from a
//   scan in the writing workgroup).
//
// A tile with more than 32 such elements (clustered data: a layer with a larger
// gradient scale, a few hot embedding rows) gets no slots: it is put on a list, and
// every kernel of the slot tail then also walks that list and reads those tiles
// from R, one wave per tile.
//
// If fewer than k keys turn out to be >= t_lo (the sample misled), or if
// the list grows beyond a quarter of the tiles (data full of ties, a very large k), a
// flag is raised on the device and the general path runs instead: three full
// histogram passes, a counting pass and a compaction pass over R (5 more reads of
// D).  The two tails exclude each other, so the host launches one sequence of kernels
// whose steps branch on the flag (surplus workgroups of the larger grid return at
// once), twelve launches in all; no host round trip is needed.  Both tails give the
// same bits.
//
// key = bit pattern of |A| as an unsigned integer: a total order on magnitudes
// (NaN above Inf).  Among keys equal to T the lowest indices are kept, which
// makes the result unique.  Every decision is integer work on bit patterns.
//
// Histograms live in LDS per workgroup and are written out once per workgroup;
// compaction uses lane masks and wavefront prefix sums.  All scratch is in the
// caller's workspace; nothing is allocated.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdio>

#include "launch.h"
#include "plan.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBins12 = 2048;  // digits of levels 1 and 2: key bits 30..20 and 19..9
constexpr int kBins3 = 512;    // digit of level 3: key bits 8..0
constexpr int kTile = 1024;        // elements per compaction tile: 64 lanes x 4 vectors x 4 elements
constexpr int kScanChunk = 256;    // tiles per chunk: one workgroup of kScanChunk threads counts, scans and writes a chunk
constexpr uint32_t kAbs = 0x7fffffffu;

// Selection state, first words of the workspace.
struct topk_state {
    uint32_t prefix;     // key bits fixed so far (in place, low bits zero)
    uint32_t k_rem;      // how many are still to be taken from the current bin
    uint32_t threshold;  // T, valid after level 3
    uint32_t ties;       // number of keys == T to keep, valid after level 3
    uint32_t overflow;   // != 0: the general tail runs (bit 0: too many tiles did not fit their
                         // slots, bit 1: fewer than k keys are >= t_lo)
    uint32_t t_lo;       // pass 1 looks only at keys >= t_lo
    uint32_t k;          // the k of this call
    uint32_t n_crowded;  // tiles that did not fit their slots; the slot tail reads those from R
    uint32_t tickets[3]; // general tail: workgroups that have added their share of the histogram of level 1, 2, 3
};

// Slot entries per 1024-element tile.  2 to 10 times the keys needed are >= t_lo for small k (1.5 to 2 times
// around k = 1 % of the data), i.e. a handful per tile: with 16 slots so many tiles went on the crowded list that the call
// took 0.95 ms instead of 0.81.
//
// Layout: "plane" q holds entries 8q .. 8q+7 of every tile, 32 bytes per tile: entry p of tile t is word
// ((p / 8) * ntiles + t) * 8 + p % 8 of the array.  Most tiles have at most eight entries, so the kernels
// of the slot tail (one thread per tile) read plane 0 densely and the others hardly at all -- a fraction of the
// bytes a tile-major layout makes them fetch, where the 32 entries of a tile are one 128-byte line and reading
// the first of them brings in the whole line -- while pass 1 still writes one short piece per tile and array
// (planes of four entries made it write two, which cost pass 1 more than the tail gained).
constexpr int kSlots = 32;
constexpr int kSlotVecs = kSlots / 4;
static_assert(kSlotVecs * 4 == kSlots && kSlots % 8 == 0, "whole planes of eight slot entries");
constexpr uint32_t kCrowded = 0xffffffffu;  // slot count of a tile that did not fit and is listed instead
// A histogram is either one row that workgroups add their non-empty LDS bins to,
// or several partial copies ("slices"), one per workgroup, that the pick kernel
// adds up.  Global atomics run at about 1.5 G/s on this chip whatever the address
// spread (320 k of them cost 200 us), so the passes of the usual path (the sample
// and the slot passes: 64 workgroups each) store slices; only the general tail's
// full-data passes, with 2048 workgroups, add to one row.
constexpr int kAtomicRows = 3;    // general tail levels 1, 2, 3: one row each, added to atomically
constexpr int kSlotGrid = 64;     // slot passes and the sample: one slice per workgroup, plain stores
constexpr int kSlotThreads = 1024;
constexpr int kHistRows = kAtomicRows + 3 * kSlotGrid;  // rows of 2048 counters in the workspace
constexpr int kSampleChunks = 1024;  // the sample: this many chunks of 64 vectors (256 elements)
constexpr int kSampleThreads = 256;
enum { kAlways = 0, kSlotTail = 1, kGeneralTail = 2 };

struct topk_ws {
    topk_state *state;
    uint32_t *hist;       // [kHistRows][2048]: general tail levels 1, 2, 3 | slot tail levels 1, 2, 3
                          // (the sample's slices share the rows of slot level 2, which comes later)
    uint32_t *slot_cnt;   // [ntiles]
    uint32_t *slot_idx;   // [kSlots / 8][ntiles][8]  (planes, see kSlots)
    uint32_t *slot_bits;  // [kSlots / 8][ntiles][8]  bit patterns of A
    uint32_t *cnt_gt;     // [ntiles]  -> exclusive prefix after the scan
    uint32_t *cnt_eq;     // [ntiles]
    uint32_t *chunk_gt;   // [nchunks] -> exclusive prefix
    uint32_t *chunk_eq;   // [nchunks]
    uint32_t *crowded;    // [ntiles]  list of the tiles that did not fit their slots (any order)
    uint32_t *pre_gt;     // [ntiles]  slot tail, crowded tiles only: kept entries of the regular tiles
    uint32_t *pre_eq;     //           before the tile in its chunk (above / at the threshold)
};

__host__ __device__ constexpr int64_t div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Byte offsets of the workspace's parts for n elements, each on a 256-byte boundary.
struct ws_offsets {
    size_t state, hist, slot_cnt, slot_idx, slot_bits, cnt_gt, cnt_eq, chunk_gt, chunk_eq, crowded, pre_gt, pre_eq, total;
};

constexpr size_t round256(size_t bytes) { return (bytes + 255) / 256 * 256; }

constexpr ws_offsets ws_offsets_for(int64_t n)
{
    const size_t ntiles = (size_t)div_up(n > 0 ? n : 1, kTile);
    const size_t nchunks = (size_t)div_up((int64_t)ntiles, kScanChunk);
    ws_offsets o{};
    size_t off = 0;
    o.state = off;     off += round256(sizeof(topk_state));
    o.hist = off;      off += round256((size_t)kHistRows * 2048 * sizeof(uint32_t));
    o.slot_cnt = off;  off += round256(ntiles * 4);
    o.slot_idx = off;  off += round256(ntiles * kSlots * 4);
    o.slot_bits = off; off += round256(ntiles * kSlots * 4);
    o.cnt_gt = off;    off += round256(ntiles * 4);
    o.cnt_eq = off;    off += round256(ntiles * 4);
    o.chunk_gt = off;  off += round256(nchunks * 4);
    o.chunk_eq = off;  off += round256(nchunks * 4);
    o.crowded = off;   off += round256(ntiles * 4);
    o.pre_gt = off;    off += round256(ntiles * 4);
    o.pre_eq = off;    off += round256(ntiles * 4);
    o.total = off;
    return o;
}

size_t ws_layout(int64_t n, void *base, topk_ws *out)
{
    const ws_offsets o = ws_offsets_for(n);
    if (out) {
        char *b = (char *)base;
        out->state = (topk_state *)(b + o.state);
        out->hist = (uint32_t *)(b + o.hist);
        out->slot_cnt = (uint32_t *)(b + o.slot_cnt);
        out->slot_idx = (uint32_t *)(b + o.slot_idx);
        out->slot_bits = (uint32_t *)(b + o.slot_bits);
        out->cnt_gt = (uint32_t *)(b + o.cnt_gt);
        out->cnt_eq = (uint32_t *)(b + o.cnt_eq);
        out->chunk_gt = (uint32_t *)(b + o.chunk_gt);
        out->chunk_eq = (uint32_t *)(b + o.chunk_eq);
        out->crowded = (uint32_t *)(b + o.crowded);
        out->pre_gt = (uint32_t *)(b + o.pre_gt);
        out->pre_eq = (uint32_t *)(b + o.pre_eq);
    }
    return o.total;
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

// ---- sample (and workspace reset) ---------------------------------------------------

// Resets the selection state, the atomically accumulated histogram rows and the chunk
// totals, and
// takes the level-1 histogram of A on `n_s` chunks of 64 vectors spread evenly
// over the `nchunks` full chunks of the data.  Each workgroup stores its LDS
// histogram as its own slice.  Grid: kSlotGrid workgroups of kSampleThreads.
__global__ __launch_bounds__(kSampleThreads) void k_topk_sample(const float *__restrict__ G,
                                                                const float *__restrict__ R, float c,
                                                                int64_t nchunks, int32_t n_s,
                                                                topk_state *st, uint32_t *hist_rows,
                                                                uint32_t *__restrict__ slices, uint32_t k,
                                                                uint32_t *chunk_gt, uint32_t *chunk_eq,
                                                                int32_t nchunks_scan)
{
    __shared__ uint32_t lds[kBins12];
    const int tid = threadIdx.x;
    const int gid = blockIdx.x * kSampleThreads + tid;
    for (int i = gid; i < kAtomicRows * 2048; i += kSlotGrid * kSampleThreads) hist_rows[i] = 0u;
    for (int i = gid; i < nchunks_scan; i += kSlotGrid * kSampleThreads) {  // the slot tail adds to these
        chunk_gt[i] = 0u;
        chunk_eq[i] = 0u;
    }
    if (gid == 0) {
        st->tickets[0] = 0u;
        st->tickets[1] = 0u;
        st->tickets[2] = 0u;
        st->prefix = 0u;
        st->k_rem = k;
        st->threshold = 0u;
        st->ties = 0u;
        st->overflow = 0u;
        st->t_lo = 0u;
        st->k = k;
        st->n_crowded = 0u;
    }
    for (int i = tid; i < kBins12; i += kSampleThreads) lds[i] = 0u;
    __syncthreads();
    const int lane = tid & 63;
    constexpr int kWaves = kSampleThreads / 64;
    for (int j = blockIdx.x * kWaves + (tid >> 6); j < n_s; j += kSlotGrid * kWaves) {
        const int64_t q = (int64_t)j * nchunks / n_s;  // < nchunks
        const int64_t v = q * 64 + lane;
        const f32x4 g = ((const f32x4 *)G)[v];
        const f32x4 r = ((const f32x4 *)R)[v];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = __float_as_uint(__builtin_fmaf(c, r[e], g[e])) & kAbs;
            atomicAdd(&lds[key >> 20], 1u);
        }
    }
    __syncthreads();
    for (int i = tid; i < kBins12; i += kSampleThreads) slices[blockIdx.x * 2048 + i] = lds[i];
}

// ---- pass 1 ------------------------------------------------------------------------------

// Four values of a tile round: element e .. e+3 (e a multiple of 4); `valid` has
// one bit per element that lies below n.
__device__ __forceinline__ f32x4 load4(const float *p, int64_t n, int64_t e, uint32_t *valid)
{
    f32x4 x = {0.0f, 0.0f, 0.0f, 0.0f};
    *valid = 0u;
    if (e + 4 <= n) {
        x = __builtin_nontemporal_load((const f32x4 *)(p + e));
        *valid = 0xfu;
    } else {
        for (int j = 0; j < 4; ++j)
            if (e + j < n) {
                x[j] = p[e + j];
                *valid |= 1u << j;
            }
    }
    return x;
}

// Number of set bits of `mask` that belong to lanes below this one.
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Error feedback, residual write, and the ordered copy of every key whose level-1
// key is >= t_lo into the slots of its tile.  One workgroup of WAVES waves per
// 1024-element tile, in four rounds of 64 lanes x 4 elements (ascending index
// order); a wave takes 4 / WAVES consecutive rounds.  Ranks inside a round come from
// the lane masks of the four components, ranks across waves through LDS.  A tile
// with more than 32 such elements (clustered data: a layer with a larger gradient
// scale, a few hot embedding rows) is put on a list instead.
template <int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_topk_pass1(const float *__restrict__ G, float *R,
                                                           int64_t n, int64_t ntiles, float c, topk_state *st,
                                                           uint32_t *__restrict__ slot_cnt,
                                                           uint32_t *__restrict__ slot_idx,
                                                           uint32_t *__restrict__ slot_bits,
                                                           uint32_t *__restrict__ crowded)
{
    constexpr int ROUNDS = 4 / WAVES;
    __shared__ uint32_t wave_total[WAVES];
    const uint32_t t_lo = st->t_lo;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t tile = blockIdx.x;  // one workgroup per tile
    const int64_t base = tile * kTile + (int64_t)wv * ROUNDS * 256;
    f32x4 g[ROUNDS], r[ROUNDS];
    uint32_t valids[ROUNDS];
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {  // all loads are in flight before the first is used
        const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
        g[u] = load4(G, n, e, &valids[u]);
        r[u] = load4(R, n, e, &valids[u]);
    }
    u32x4 raw[ROUNDS];
    uint32_t cand[ROUNDS], rank[ROUNDS];  // per round: 4-bit mask of kept components, rank of the first
    uint32_t running = 0u;
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
        const uint32_t valid = valids[u];
        f32x4 a;
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] = __builtin_fmaf(c, r[u][j], g[u][j]);
        if (valid == 0xfu) {
            __builtin_nontemporal_store(a, (f32x4 *)(R + e));  // only single elements are read again
        } else {
            for (int j = 0; j < 4; ++j)
                if ((valid >> j) & 1u) R[e + j] = a[j];
        }
        raw[u] = __builtin_bit_cast(u32x4, a);
        bool cj[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) cj[j] = ((valid >> j) & 1u) && (raw[u][j] & kAbs) >= t_lo;
        const uint64_t m0 = __ballot(cj[0]), m1 = __ballot(cj[1]), m2 = __ballot(cj[2]), m3 = __ballot(cj[3]);
        cand[u] = (cj[0] ? 1u : 0u) | (cj[1] ? 2u : 0u) | (cj[2] ? 4u : 0u) | (cj[3] ? 8u : 0u);
        rank[u] = running;
        if ((m0 | m1 | m2 | m3) != 0ull) {
            rank[u] += lanes_below(m0) + lanes_below(m1) + lanes_below(m2) + lanes_below(m3);
            running += (uint32_t)(__popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3));
        }
    }
    uint32_t before = 0u, total = running;
    if constexpr (WAVES > 1) {
        if (lane == 0) wave_total[wv] = running;
        __syncthreads();
        total = 0u;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const uint32_t t = wave_total[w];
            before += w < wv ? t : 0u;
            total += t;
        }
    }
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        if (cand[u] == 0u) continue;
        const int64_t e = base + (int64_t)(u * 64 + lane) * 4;
        uint32_t pos = before + rank[u];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if ((cand[u] >> j) & 1u) {
                if (pos < (uint32_t)kSlots) {
                    const int64_t at = ((int64_t)(pos >> 3) * ntiles + tile) * 8 + (pos & 7u);
                    slot_idx[at] = (uint32_t)(e + j);
                    slot_bits[at] = raw[u][j];
                }
                ++pos;
            }
        }
    }
    if (threadIdx.x == 0) {
        if (total > (uint32_t)kSlots) {  // the tile goes on the list; the tail reads it from R instead
            crowded[atomicAdd(&st->n_crowded, 1u)] = (uint32_t)tile;  // at most once per tile: never past ntiles
            slot_cnt[tile] = kCrowded;
        } else {
            slot_cnt[tile] = total;
        }
    }
}

// ---- full histogram passes (general tail only) --------------------------------------------

// Histogram of one digit of the keys in R: level 1 counts every key, levels 2 and 3
// the keys that match the prefix found so far.  Persistent workgroups: each walks
// tiles of NT vectors with a grid stride and keeps one LDS histogram per
// wave.
// NT threads per workgroup; `lds` holds 4 * BINS counters (one histogram per wave
// modulo four); the first `groups` workgroups of the grid take part.
template <int LEVEL, int NT>
__device__ __forceinline__ void general_hist(const float *__restrict__ R, int64_t n,
                                             const topk_state *__restrict__ st,
                                             uint32_t *__restrict__ hist, uint32_t *lds, uint32_t groups)
{
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int SHIFT = LEVEL == 1 ? 20 : (LEVEL == 2 ? 9 : 0);
    constexpr int HI_SHIFT = LEVEL == 1 ? 31 : (LEVEL == 2 ? 20 : 9);  // bits above this digit
    const int tid = threadIdx.x;
    const uint32_t want = LEVEL == 1 ? 0u : st->prefix >> HI_SHIFT;  // keys have bit 31 clear
    uint32_t *mine = lds + ((tid >> 6) & 3) * BINS;
    for (int i = tid; i < 4 * BINS; i += NT) lds[i] = 0u;
    __syncthreads();

    const int64_t nvec = n / 4;
    const int64_t stride = (int64_t)groups * NT;
    for (int64_t v = (int64_t)blockIdx.x * NT + tid; v < nvec; v += stride) {
        const u32x4 key = __builtin_nontemporal_load((const u32x4 *)R + v) & kAbs;
        if ((key.x >> HI_SHIFT) == want) atomicAdd(&mine[(key.x >> SHIFT) & (BINS - 1)], 1u);
        if ((key.y >> HI_SHIFT) == want) atomicAdd(&mine[(key.y >> SHIFT) & (BINS - 1)], 1u);
        if ((key.z >> HI_SHIFT) == want) atomicAdd(&mine[(key.z >> SHIFT) & (BINS - 1)], 1u);
        if ((key.w >> HI_SHIFT) == want) atomicAdd(&mine[(key.w >> SHIFT) & (BINS - 1)], 1u);
    }
    // scalar tail (n mod 4 elements), one workgroup only
    if (blockIdx.x == 0 && tid < (int)(n - nvec * 4)) {
        const uint32_t key = __float_as_uint(R[nvec * 4 + tid]) & kAbs;
        if ((key >> HI_SHIFT) == want) atomicAdd(&mine[(key >> SHIFT) & (BINS - 1)], 1u);
    }
    __syncthreads();
    for (int b = tid; b < BINS; b += NT) {
        const uint32_t s = (lds[b] + lds[BINS + b]) + (lds[2 * BINS + b] + lds[3 * BINS + b]);
        if (s) atomicAdd(&hist[b], s);
    }
}

// Finds the digit at which the count from the top reaches the wanted count: the
// largest b with sum_{j >= b} hist[j] >= wanted.  One workgroup.
//   LEVEL 0     on the sample: wanted = `target`; the digit's lowest key (GATE 0) or a key inside
//               its bin found by interpolation (GATE 1) becomes t_lo (0 if the sample is too
//               small to tell)
//   LEVEL 1     wanted = k; the digit opens the prefix.  On the slots (GATE kSlotTail)
//               a total below k means that t_lo was too high, and a crowded list
//               longer than `target` that too many tiles missed their slots: either
//               switches the general tail on.
//   LEVEL 2, 3  wanted = k_rem; the digit extends the prefix; level 3 fixes T.
// One workgroup of NT threads runs it.  All of them add up the slices: a thread takes four
// neighbouring counters (one 16-byte load per slice) of every G-th slice, G = NT / (BINS / 4),
// with up to 16 loads in flight, and the G partial sums meet in LDS.  The first 256 threads
// then scan.  `lds` holds kPickLds words.  Barriers inside: every thread of the workgroup
// must call it, and nothing that needs a barrier may follow.
constexpr int kPickThreads = 1024;
constexpr int kPickLds = 4 + 4 * kPickThreads;  // words; the array must be 16-byte aligned

template <int LEVEL, int GATE, int NT>
__device__ __forceinline__ void pick(topk_state *st, const uint32_t *hist, int nslices, uint32_t target,
                                     uint32_t *lds)
{
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int PER = BINS / 256;
    constexpr int SHIFT = LEVEL <= 1 ? 20 : (LEVEL == 2 ? 9 : 0);
    constexpr int Q = BINS / 4, G = NT / Q;
    static_assert(NT % Q == 0 && G >= 1 && G * BINS <= 4 * kPickThreads, "slice groups fill the workgroup");
    uint32_t *wave_tot = lds, *sums = lds + 4;  // sums: [G][BINS], 16-byte aligned
    const int tid = threadIdx.x;
    const uint32_t k_rem = LEVEL == 0 ? target : (LEVEL == 1 ? st->k : st->k_rem);
    const uint32_t base_prefix = LEVEL <= 1 ? 0u : st->prefix;
    {
        const int quad = tid % Q, grp = tid / Q;
        const u32x4 *col = (const u32x4 *)hist + quad;  // rows are 2048 counters = 512 vectors apart
        u32x4 acc = {0u, 0u, 0u, 0u};
        int sl = grp;
        for (; sl + 15 * G < nslices; sl += 16 * G) {
            u32x4 x[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) x[j] = col[(sl + j * G) * 512];
#pragma unroll
            for (int j = 0; j < 16; ++j) acc += x[j];
        }
        for (; sl + 7 * G < nslices; sl += 8 * G) {
            u32x4 x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = col[(sl + j * G) * 512];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += x[j];
        }
        for (; sl < nslices; sl += G) acc += col[sl * 512];
        ((u32x4 *)sums)[grp * Q + quad] = acc;
    }
    __syncthreads();
    // The scan is the work of the first 256 threads (four waves); the others only keep
    // every barrier complete (a barrier must be reached by all threads of the workgroup).
    const bool scanner = tid < 256;
    // scanner t owns bins [BINS - (t+1)*PER, BINS - t*PER): thread 0 the top ones
    uint32_t h[PER];
    uint32_t mine = 0u, incl = 0u;
    if (scanner) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int bin = BINS - 1 - (tid * PER + j);  // descending bin order
            uint32_t c = 0u;
#pragma unroll
            for (int g = 0; g < G; ++g) c += sums[g * BINS + bin];
            h[j] = c;
            mine += c;
        }
        incl = wave_incl_scan(mine);  // whole waves: 256 is a multiple of 64
        if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
    }
    __syncthreads();
    if (!scanner) return;  // no barrier follows
    for (int w = 0; w < (tid >> 6); ++w) incl += wave_tot[w];
    const uint32_t excl = incl - mine;
    if (LEVEL == 1 && GATE == kSlotTail && tid == 255) {
        if (incl < k_rem) atomicOr(&st->overflow, 2u);
        if (st->n_crowded > target) atomicOr(&st->overflow, 1u);  // target: the longest list the slot tail takes
    }
    if (k_rem > 0u && excl < k_rem && k_rem <= incl) {  // at most one thread
        uint32_t above = excl;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (above + h[j] >= k_rem) {
                const uint32_t bin = (uint32_t)(BINS - 1 - (tid * PER + j));
                if (LEVEL == 0) {
                    // GATE != 0: the key inside the bin above which the wanted count lies, taking the
                    // bin's keys as evenly spread; otherwise the bin's lowest key, which can only admit
                    // more.  (A heuristic bound either way: nothing exact depends on it.)
                    uint32_t inside = 0u;  // offset of the key above the bin's lower edge
                    if (GATE != 0) {
                        // The count from the top grows geometrically through a bin of a smooth tail, and
                        // faster than that towards the lower edge when keys crowd below the k-th largest:
                        // a geometric fit between the counts at the two edges errs low, the safe side.
                        // (Linear in the count when nothing lies above the bin.)
                        const float total = (float)(above + h[j]), want_f = (float)k_rem;
                        const float s = above > 0u ? __log2f(want_f / (float)above) / __log2f(total / (float)above)
                                                   : (want_f / total);  // share of the bin's width, from its top
                        const float down = fminf(fmaxf(s, 0.0f), 1.0f) * 1048576.0f;
                        inside = 1048576u - (uint32_t)down;
                        if (inside > 1048575u) inside = 1048575u;
                    }
                    st->t_lo = (bin << 20) + inside;
                    break;
                }
                const uint32_t prefix = base_prefix | (bin << SHIFT);
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

// Numbers of keys above and at the threshold in one 1024-element tile of R.  One wave;
// every lane gets both sums.
__device__ __forceinline__ void tile_counts(const float *__restrict__ R, int64_t n, int64_t tile, uint32_t T,
                                            int lane, uint32_t *gt_out, uint32_t *eq_out)
{
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
    *gt_out = wave_sum(gt);
    *eq_out = wave_sum(eq);
}

// Exclusive prefix sum of x over the NT threads of a workgroup; *total gets the sum.
// `ldsw` holds one word per wave.  Barriers inside: every thread must call it.
template <int NT = kScanChunk>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t x, uint32_t *ldsw, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan(x);
    if (lane == 63) ldsw[wv] = incl;
    __syncthreads();
    uint32_t before = 0u, all = 0u;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const uint32_t t = ldsw[w];
        before += w < wv ? t : 0u;
        all += t;
    }
    __syncthreads();  // ldsw is free again
    *total = all;
    return before + incl - x;
}

// General tail: per-tile counts over the residual, one wave per tile; the first `groups`
// workgroups (kSlotThreads threads each) walk the tiles.
__device__ __forceinline__ void general_count(const float *__restrict__ R, int64_t n, int64_t ntiles,
                                              const topk_state *__restrict__ st, uint32_t *__restrict__ cnt_gt,
                                              uint32_t *__restrict__ cnt_eq, uint32_t groups)
{
    constexpr int kWaves = kSlotThreads / 64;
    const uint32_t T = st->threshold;
    const int lane = threadIdx.x & 63;
    for (int64_t tile = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6); tile < ntiles;
         tile += (int64_t)groups * kWaves) {
        uint32_t gt, eq;
        tile_counts(R, n, tile, T, lane, &gt, &eq);
        if (lane == 0) {
            cnt_gt[tile] = gt;
            cnt_eq[tile] = eq;
        }
    }
}

// General tail, scan phase A: workgroup c turns the counts of the kScanChunk tiles of
// chunk c into chunk-local exclusive prefixes and writes the chunk's totals.
__device__ __forceinline__ void general_scan_a(uint32_t *cnt_gt, uint32_t *cnt_eq, int64_t ntiles,
                                               uint32_t *chunk_gt, uint32_t *chunk_eq, uint32_t *lds16)
{
    const int64_t tile = (int64_t)blockIdx.x * kScanChunk + threadIdx.x;  // kScanChunk threads
    const bool in = tile < ntiles;
    const uint32_t g = in ? cnt_gt[tile] : 0u, e = in ? cnt_eq[tile] : 0u;
    uint32_t tg, te;
    const uint32_t pg = block_excl_scan(g, lds16, &tg), pe = block_excl_scan(e, lds16, &te);
    if (in) {
        cnt_gt[tile] = pg;
        cnt_eq[tile] = pe;
    }
    if (threadIdx.x == 0) {
        chunk_gt[blockIdx.x] = tg;
        chunk_eq[blockIdx.x] = te;
    }
}

// Phase B: one workgroup scans the chunk totals in place (exclusive).
__global__ __launch_bounds__(kSlotThreads) void k_topk_scan_b(uint32_t *chunk_gt, uint32_t *chunk_eq,
                                                              int64_t nchunks)
{
    __shared__ uint32_t ldsw[kSlotThreads / 64];
    uint32_t carry_g = 0u, carry_e = 0u;  // the same in every thread
    for (int64_t base = 0; base < nchunks; base += kSlotThreads) {
        const int64_t i = base + threadIdx.x;
        const uint32_t g = i < nchunks ? chunk_gt[i] : 0u, e = i < nchunks ? chunk_eq[i] : 0u;
        uint32_t tg, te;
        const uint32_t pg = block_excl_scan<kSlotThreads>(g, ldsw, &tg);
        const uint32_t pe = block_excl_scan<kSlotThreads>(e, ldsw, &te);
        if (i < nchunks) {
            chunk_gt[i] = carry_g + pg;
            chunk_eq[i] = carry_e + pe;
        }
        carry_g += tg;
        carry_e += te;
    }
}

// Ordered write of one tile's kept elements, read from R (one wave): gt_before keys above
// the threshold and eq_before keys at it lie before the tile.  Element order inside a
// tile is (round u, lane, component), which is ascending index; ranks come from wavefront
// prefix sums.
__device__ __forceinline__ void write_tile(float *R, int64_t n, int64_t tile, uint32_t T, uint32_t ties,
                                           int lane, uint32_t gt_before, uint32_t eq_before,
                                           float *__restrict__ vals, uint32_t *__restrict__ idx,
                                           uint32_t kmax)
{
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
            if (((selm >> j) & 1u) && pos < kmax) {  // pos < kmax always holds; the test keeps a corrupted workspace harmless
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

// General tail: the ordered write, one wave per tile; the first `groups` workgroups
// (NT threads each) walk the tiles.
template <int NT>
__device__ __forceinline__ void general_write(float *R, int64_t n, int64_t ntiles,
                                              const topk_state *__restrict__ st,
                                              const uint32_t *__restrict__ cnt_gt,
                                              const uint32_t *__restrict__ cnt_eq,
                                              const uint32_t *__restrict__ chunk_gt,
                                              const uint32_t *__restrict__ chunk_eq, float *__restrict__ vals,
                                              uint32_t *__restrict__ idx, uint32_t kmax, uint32_t groups)
{
    constexpr int kWaves = NT / 64;
    const uint32_t T = st->threshold, ties = st->ties;
    for (int64_t tile = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6); tile < ntiles;
         tile += (int64_t)groups * kWaves) {
        const int64_t chunk = tile / kScanChunk;
        write_tile(R, n, tile, T, ties, threadIdx.x & 63, chunk_gt[chunk] + cnt_gt[tile],
                   chunk_eq[chunk] + cnt_eq[tile], vals, idx, kmax);
    }
}

// ---- slot tail -------------------------------------------------------------------------

// The slot-tail kernels give one thread to each tile: neighbouring threads read
// neighbouring counts and neighbouring vectors of a plane.  The tiles on the crowded
// list have no slots: every slot-tail kernel then walks the list, one wave per tile, and
// reads those tiles from R.  When the list grows beyond a small share of the tiles (data
// full of ties, a very large k) the general tail takes over instead.
__host__ __device__ inline uint32_t crowded_limit(int64_t ntiles)
{
    const int64_t share = ntiles / 4;
    return (uint32_t)(share > 1024 ? share : 1024);
}

// Entries 4q .. 4q+3 of tile `tile` in a slot array (half of the tile's 32 bytes in plane q / 2).
__device__ __forceinline__ u32x4 slot_vec(const uint32_t *__restrict__ slots, int64_t ntiles, int q, int64_t tile)
{
    return ((const u32x4 *)slots)[((int64_t)(q >> 1) * ntiles + tile) * 2 + (q & 1)];
}

// Histogram of one digit over the slot entries (level 1: all of them; levels 2, 3:
// those that match the prefix): a few large workgroups, each with an LDS histogram
// that it stores as its own slice.
// The first kSlotGrid workgroups of the grid take part (kSlotThreads threads each);
// `lds` holds 4 * BINS counters.
template <int LEVEL>
__device__ __forceinline__ void slots_hist(const topk_state *__restrict__ st,
                                           const uint32_t *__restrict__ slot_cnt,
                                           const uint32_t *__restrict__ slot_bits, int64_t ntiles,
                                           const uint32_t *__restrict__ crowded,
                                           const float *__restrict__ R, int64_t n,
                                           uint32_t *__restrict__ hist, uint32_t *lds)
{
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int SHIFT = LEVEL == 1 ? 20 : (LEVEL == 2 ? 9 : 0);
    constexpr int HI_SHIFT = LEVEL == 1 ? 31 : (LEVEL == 2 ? 20 : 9);
    // Level 1 sees every entry, and nearly all of them fall into the eight bins from t_lo's up
    // (one octave): a thread counts those in the eight 8-bit fields of a register, and a wave
    // adds its fields up and makes eight LDS additions every six tiles per lane (at most 192
    // entries, so no field overflows).  The other bins, and the other levels, add to LDS
    // entry by entry; four copies of the level-1 histogram, picked by lane, spread those.
    constexpr int COPIES = LEVEL == 1 ? 4 : 1;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < COPIES * BINS; i += kSlotThreads) lds[i] = 0u;
    __syncthreads();
    uint32_t *mine = lds + (tid & (COPIES - 1)) * BINS;
    const uint32_t want = LEVEL == 1 ? 0u : st->prefix >> HI_SHIFT;  // keys have bit 31 clear
    const uint32_t t_lo = st->t_lo, b_lo = t_lo >> 20;
    uint64_t packed = 0ull;
    auto count = [&](uint32_t key) {  // key: bit 31 clear, matches the prefix
        if constexpr (LEVEL == 1) {
            const uint32_t rel = (key >> 20) - b_lo;  // >= 0: only keys at or above t_lo are looked at
            if (rel < 8u)
                packed += 1ull << (rel * 8u);
            else
                atomicAdd(&mine[key >> 20], 1u);
        } else {
            atomicAdd(&mine[(key >> SHIFT) & (BINS - 1)], 1u);
        }
    };
    auto flush = [&]() {  // whole waves only
        if constexpr (LEVEL == 1) {
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                const uint32_t c = wave_sum((uint32_t)(packed >> (8 * f)) & 255u);
                if (lane == f && c != 0u) atomicAdd(&mine[b_lo + f], c);  // c != 0: the bin exists
            }
            packed = 0ull;
        }
    };
    auto add = [&](const u32x4 v, uint32_t first, uint32_t c) {  // entries first .. first+3 of a tile with c entries
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = v[j] & kAbs;
            if (first + j < c && (key >> HI_SHIFT) == want) count(key);
        }
    };
    const int64_t stride = (int64_t)kSlotGrid * kSlotThreads;
    constexpr int U = 6;  // tiles in flight per thread (6 x kSlots = 192 entries: below the 255 a field holds)
    // the loop runs on the wave's first tile, so that a wave stays whole (flush needs all lanes)
    for (int64_t w0 = (int64_t)blockIdx.x * kSlotThreads + (tid - lane); w0 < ntiles; w0 += U * stride) {
        const int64_t t0 = w0 + lane;
        uint32_t c[U];
        u32x4 v[U];
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int64_t tile = t0 + i * stride;
            c[i] = tile < ntiles ? slot_cnt[tile] : 0u;
            if (c[i] == kCrowded) c[i] = 0u;
        }
#pragma unroll
        for (int i = 0; i < U; ++i) {
            v[i] = u32x4{0u, 0u, 0u, 0u};
            if (c[i] != 0u) v[i] = slot_vec(slot_bits, ntiles, 0, t0 + i * stride);
        }
#pragma unroll
        for (int i = 0; i < U; ++i) add(v[i], 0u, c[i]);
#pragma unroll
        for (int i = 0; i < U; ++i)
            for (int q = 1; (uint32_t)q * 4u < c[i]; ++q)  // c <= kSlots: at most kSlotVecs - 1 more
                add(slot_vec(slot_bits, ntiles, q, t0 + i * stride), (uint32_t)q * 4u, c[i]);
        flush();
    }
    // the crowded tiles, from R: one wave per tile.  Level 1 counts, like the slots do,
    // only the keys at or above t_lo.
    const uint32_t n_crowded = st->n_crowded;
    if (n_crowded <= crowded_limit(ntiles)) {
        constexpr int kWaves = kSlotThreads / 64;
        for (uint32_t i = blockIdx.x * kWaves + (tid >> 6); i < n_crowded; i += kSlotGrid * kWaves) {
            const int64_t base = (int64_t)crowded[i] * kTile;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint32_t valid;
                const u32x4 key = load_keys(R, n, base + (int64_t)(u * 64 + lane) * 4, &valid);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool ok = ((valid >> j) & 1u) && (key[j] >> HI_SHIFT) == want &&
                                    (LEVEL != 1 || key[j] >= t_lo);
                    if (ok) count(key[j]);
                }
            }
            flush();  // 16 keys per lane and tile
        }
    }
    __syncthreads();
    for (int i = tid; i < BINS; i += kSlotThreads) {
        uint32_t sum = 0u;
#pragma unroll
        for (int c = 0; c < COPIES; ++c) sum += lds[c * BINS + i];
        hist[blockIdx.x * 2048 + i] = sum;
    }
}

// Numbers of a tile's slot entries above and at the threshold (one thread).
__device__ __forceinline__ void slot_counts(const uint32_t *__restrict__ slot_bits, int64_t ntiles, int64_t tile,
                                            uint32_t cnt, uint32_t T, uint32_t *gt_out, uint32_t *eq_out)
{
    uint32_t gt = 0u, eq = 0u;
    for (int q = 0; (uint32_t)q * 4u < cnt; ++q) {
        const u32x4 v = slot_vec(slot_bits, ntiles, q, tile);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = v[j] & kAbs;
            const bool in = (uint32_t)q * 4u + j < cnt;
            gt += (in && key > T) ? 1u : 0u;
            eq += (in && key == T) ? 1u : 0u;
        }
    }
    *gt_out = gt;
    *eq_out = eq;
}

// Slot tail, counting step.  Workgroup c (kScanChunk threads, one per tile) owns the
// tiles of chunk c: it counts their slot entries above and at the threshold and adds the
// chunk's totals to chunk_gt / chunk_eq (zeroed by the first kernel of the call).  A
// crowded tile has no slots: its thread records how many kept entries of the chunk's
// REGULAR tiles lie before it (pre_gt / pre_eq); its own counts come from the residual,
// taken by the waves of the whole grid walking the crowded list (so that a cluster of such
// tiles is shared out evenly), stored per tile and added to the chunk totals as well.
__device__ __forceinline__ void slots_count(const topk_state *__restrict__ st,
                                            const uint32_t *__restrict__ slot_cnt,
                                            const uint32_t *__restrict__ slot_bits, int64_t ntiles,
                                            const uint32_t *__restrict__ crowded,
                                            const float *__restrict__ R, int64_t n,
                                            uint32_t *__restrict__ cnt_gt, uint32_t *__restrict__ cnt_eq,
                                            uint32_t *__restrict__ pre_gt, uint32_t *__restrict__ pre_eq,
                                            uint32_t *chunk_gt, uint32_t *chunk_eq, uint32_t groups,
                                            uint32_t *lds16)
{
    const int64_t tile = (int64_t)blockIdx.x * kScanChunk + threadIdx.x;
    const uint32_t T = st->threshold;
    uint32_t gt = 0u, eq = 0u;
    bool listed = false;
    if (tile < ntiles) {
        const uint32_t cnt = slot_cnt[tile];
        listed = cnt == kCrowded;
        if (!listed) slot_counts(slot_bits, ntiles, tile, cnt, T, &gt, &eq);
    }
    uint32_t tg, te;
    const uint32_t pg = block_excl_scan(gt, lds16, &tg), pe = block_excl_scan(eq, lds16, &te);
    if (listed) {
        pre_gt[tile] = pg;
        pre_eq[tile] = pe;
    }
    if (threadIdx.x == 0) {
        if (tg) atomicAdd(&chunk_gt[blockIdx.x], tg);
        if (te) atomicAdd(&chunk_eq[blockIdx.x], te);
    }
    // the crowded tiles, from R: one wave per tile
    constexpr int kWaves = kScanChunk / 64;
    const uint32_t n_crowded = st->n_crowded;
    const int lane = threadIdx.x & 63;
    for (uint32_t i = blockIdx.x * kWaves + (threadIdx.x >> 6); i < n_crowded; i += groups * kWaves) {
        const int64_t t = crowded[i];
        uint32_t g, e;
        tile_counts(R, n, t, T, lane, &g, &e);
        if (lane == 0) {
            cnt_gt[t] = g;
            cnt_eq[t] = e;
            if (g) atomicAdd(&chunk_gt[t / kScanChunk], g);
            if (e) atomicAdd(&chunk_eq[t / kScanChunk], e);
        }
    }
}

// Slot tail, ordered write.  Workgroup c owns the tiles of chunk c again: every thread
// recounts its tile (a crowded tile's counts are read back), a scan over the workgroup
// gives each tile its position, and a thread then walks the entries of its tile, which
// are in ascending index order.  The crowded tiles are written from the residual by the
// waves of the whole grid walking the list; such a wave puts the tile's position together
// from the chunk's offset, the regular tiles before it (pre_gt / pre_eq) and the crowded
// tiles before it in the chunk, which it finds by reading the chunk's slot counts.
// chunk_gt / chunk_eq hold exclusive prefixes by now.
__device__ __forceinline__ void slots_write(float *R, int64_t n, const topk_state *__restrict__ st,
                                            const uint32_t *__restrict__ slot_cnt,
                                            const uint32_t *__restrict__ slot_idx,
                                            const uint32_t *__restrict__ slot_bits,
                                            const uint32_t *__restrict__ crowded,
                                            const uint32_t *__restrict__ cnt_gt,
                                            const uint32_t *__restrict__ cnt_eq,
                                            const uint32_t *__restrict__ pre_gt,
                                            const uint32_t *__restrict__ pre_eq,
                                            const uint32_t *__restrict__ chunk_gt,
                                            const uint32_t *__restrict__ chunk_eq, int64_t ntiles,
                                            float *__restrict__ vals, uint32_t *__restrict__ idx,
                                            uint32_t kmax, uint32_t groups, uint32_t *lds16)
{
    const int64_t tile = (int64_t)blockIdx.x * kScanChunk + threadIdx.x;
    const uint32_t T = st->threshold, ties = st->ties;
    uint32_t cnt = 0u, gt = 0u, eq = 0u;
    if (tile < ntiles) {
        cnt = slot_cnt[tile];
        if (cnt == kCrowded) {
            gt = cnt_gt[tile];
            eq = cnt_eq[tile];
        } else {
            slot_counts(slot_bits, ntiles, tile, cnt, T, &gt, &eq);
        }
    }
    uint32_t tg, te;
    const uint32_t pg = block_excl_scan(gt, lds16, &tg), pe = block_excl_scan(eq, lds16, &te);
    if (cnt != kCrowded && (gt | eq) != 0u) {
        uint32_t eq_rank = chunk_eq[blockIdx.x] + pe;  // ties before this tile's first
        uint32_t pos = chunk_gt[blockIdx.x] + pg + (eq_rank < ties ? eq_rank : ties);
        for (int q = 0; (uint32_t)q * 4u < cnt; ++q) {
            const u32x4 v = slot_vec(slot_bits, ntiles, q, tile);
            uint32_t selm = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t key = v[j] & kAbs;
                if ((uint32_t)q * 4u + j < cnt) {
                    if (key > T) selm |= 1u << j;
                    if (key == T) {
                        if (eq_rank < ties) selm |= 1u << j;
                        ++eq_rank;
                    }
                }
            }
            if (selm == 0u) continue;
            const u32x4 at = slot_vec(slot_idx, ntiles, q, tile);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (((selm >> j) & 1u) && pos < kmax) {  // pos < kmax always holds; the test keeps a corrupted workspace harmless
                    vals[pos] = __uint_as_float(v[j]);
                    idx[pos] = at[j];
                    R[at[j]] = 0.0f;
                    ++pos;
                }
            }
        }
    }
    // the crowded tiles, from R: one wave per tile (the waves arrive here whole: the
    // branches above have closed)
    constexpr int kWaves = kScanChunk / 64;
    const uint32_t n_crowded = st->n_crowded;
    const int lane = threadIdx.x & 63;
    for (uint32_t i = blockIdx.x * kWaves + (threadIdx.x >> 6); i < n_crowded; i += groups * kWaves) {
        const int64_t t = crowded[i];
        const int64_t chunk = t / kScanChunk, first = chunk * kScanChunk;
        uint32_t g = 0u, e = 0u;
        for (int64_t u = first + lane; u < t; u += 64) {  // crowded tiles before t in its chunk
            if (slot_cnt[u] == kCrowded) {
                g += cnt_gt[u];
                e += cnt_eq[u];
            }
        }
        g = wave_sum(g);
        e = wave_sum(e);
        write_tile(R, n, t, T, ties, lane, chunk_gt[chunk] + pre_gt[t] + g, chunk_eq[chunk] + pre_eq[t] + e, vals,
                   idx, kmax);
    }
}

// ---- the kernels of the tail --------------------------------------------------------------
//
// The slot tail and the general tail exclude each other (a device flag, set by the pick
// that follows the first histogram below, says which runs), and the host cannot know which:
// every step is one kernel that branches on the flag, with a grid large enough for either
// and the surplus workgroups returning at once.  So that neither tail adds launches to the
// other, the general tail is shaped to the slot tail's seven steps:
//
//     step          slot tail                       general tail
//     hist_step<2>  histogram of digit 2, slots     histogram of digit 1 over R + its pick
//     pick_step<2>  pick of digit 2                 histogram of digit 2 over R + its pick
//     hist_step<3>  histogram of digit 3, slots     histogram of digit 3 over R + its pick
//     pick_step<3>  pick of digit 3                 per-tile counts over R
//     count         counts + totals per chunk       scan of the tile counts, chunk by chunk
//     scan_b        scan of the chunk totals        the same
//     emit          ordered write from the slots    ordered write from R
//
// In the general tail the workgroup that adds its share of a histogram last does the pick
// (a ticket counter).  On the slot tail, the usual one, the picks stay kernels of their
// own: the device-scope release that must precede a ticket writes back the L2 of the
// workgroup's XCD, which costs 10-12 us per kernel on this chip -- more than the 4-5 us of
// the launch it saves -- and that price is only worth paying where it keeps the rare tail
// from adding three launches to every call.

constexpr int kGenGrid = 256;  // general-tail passes over R: workgroups of kSlotThreads threads

// General tail: histogram of digit LEVEL over R by the first `groups` workgroups, then
// the pick by whichever of them finishes last.  `lds` holds 4 * 2048 words.
template <int LEVEL>
__device__ __forceinline__ void general_hist_pick(const float *__restrict__ R, int64_t n, topk_state *st,
                                                  uint32_t *row, uint32_t *lds, uint32_t groups)
{
    __shared__ uint32_t last;
    general_hist<LEVEL, kSlotThreads>(R, n, st, row, lds, groups);
    __threadfence();  // this thread's additions to the row are visible device-wide ...
    __syncthreads();  // ... for every thread of the workgroup, before the workgroup's ticket
    if (threadIdx.x == 0) last = atomicAdd(&st->tickets[LEVEL - 1], 1u) == groups - 1u ? 1u : 0u;
    __syncthreads();
    if (last == 0u) return;  // the whole workgroup leaves
    __threadfence();  // the other workgroups' additions are visible to this one
    pick<LEVEL, kGeneralTail, kSlotThreads>(st, row, 1, 0u, lds);
}

// INTERPOLATE: the bound is placed inside the level-1 bin (for larger k, see run_topk).
template <bool INTERPOLATE>
__global__ __launch_bounds__(kPickThreads) void k_topk_pick_sample(topk_state *st, const uint32_t *hist,
                                                                   uint32_t target)
{
    __shared__ __align__(16) uint32_t lds[kPickLds];
    pick<0, INTERPOLATE ? 1 : 0, kPickThreads>(st, hist, kSlotGrid, target, lds);
}

// Level-1 histogram of the slots (the pick that follows decides which tail runs).
__global__ __launch_bounds__(kSlotThreads) void k_topk_digit1(const topk_state *__restrict__ st,
                                                              const uint32_t *__restrict__ slot_cnt,
                                                              const uint32_t *__restrict__ slot_bits,
                                                              int64_t ntiles,
                                                              const uint32_t *__restrict__ crowded,
                                                              const float *__restrict__ R, int64_t n,
                                                              uint32_t *__restrict__ slices)
{
    __shared__ __align__(16) uint32_t lds[4 * kBins12];
    slots_hist<1>(st, slot_cnt, slot_bits, ntiles, crowded, R, n, slices, lds);
}

__global__ __launch_bounds__(kPickThreads) void k_topk_pick1(topk_state *st, const uint32_t *slices,
                                                             uint32_t crowded_max)
{
    __shared__ __align__(16) uint32_t lds[kPickLds];
    pick<1, kSlotTail, kPickThreads>(st, slices, kSlotGrid, crowded_max, lds);
}

// Slot tail: histogram of digit LEVEL (2 or 3) over the slots.  General tail: histogram
// and pick of digit 1 (LEVEL 2) or 3 (LEVEL 3) over the whole residual.
template <int LEVEL>
__global__ __launch_bounds__(kSlotThreads) void k_topk_hist_step(topk_state *st,
                                                                 const uint32_t *__restrict__ slot_cnt,
                                                                 const uint32_t *__restrict__ slot_bits,
                                                                 int64_t ntiles,
                                                                 const uint32_t *__restrict__ crowded,
                                                                 const float *__restrict__ R, int64_t n,
                                                                 uint32_t *__restrict__ slices, uint32_t *row,
                                                                 uint32_t gen_groups)
{
    __shared__ __align__(16) uint32_t lds[4 * kBins12];
    if (st->overflow == 0u) {  // the same answer in every workgroup: it was fixed by an earlier kernel
        if (blockIdx.x >= (uint32_t)kSlotGrid) return;
        slots_hist<LEVEL>(st, slot_cnt, slot_bits, ntiles, crowded, R, n, slices, lds);
    } else {
        if (blockIdx.x >= gen_groups) return;
        general_hist_pick<LEVEL == 2 ? 1 : 3>(R, n, st, row, lds, gen_groups);
    }
}

// Slot tail: the pick after k_topk_hist_step<LEVEL> (one workgroup).  General tail:
// histogram and pick of digit 2 (LEVEL 2), or the per-tile counts over the residual (LEVEL 3).
template <int LEVEL>
__global__ __launch_bounds__(kSlotThreads) void k_topk_pick_step(topk_state *st, const uint32_t *slices,
                                                                 const float *__restrict__ R, int64_t n,
                                                                 int64_t ntiles, uint32_t *row,
                                                                 uint32_t *__restrict__ cnt_gt,
                                                                 uint32_t *__restrict__ cnt_eq,
                                                                 uint32_t gen_groups)
{
    __shared__ __align__(16) uint32_t lds[4 * kBins12];
    if (st->overflow == 0u) {
        if (blockIdx.x != 0u) return;
        pick<LEVEL, kSlotTail, kSlotThreads>(st, slices, kSlotGrid, 0u, lds);
    } else {
        if (blockIdx.x >= gen_groups) return;
        if constexpr (LEVEL == 2)
            general_hist_pick<2>(R, n, st, row, lds, gen_groups);
        else
            general_count(R, n, ntiles, st, cnt_gt, cnt_eq, gen_groups);
    }
}

// One workgroup per chunk of kScanChunk tiles.  Slot tail: counts and chunk totals.
// General tail: first phase of the scan of the per-tile counts.
__global__ __launch_bounds__(kScanChunk) void k_topk_count(const topk_state *__restrict__ st,
                                                             const uint32_t *__restrict__ slot_cnt,
                                                             const uint32_t *__restrict__ slot_bits,
                                                             int64_t ntiles,
                                                             const uint32_t *__restrict__ crowded,
                                                             const float *__restrict__ R, int64_t n,
                                                             uint32_t *cnt_gt, uint32_t *cnt_eq,
                                                             uint32_t *__restrict__ pre_gt,
                                                             uint32_t *__restrict__ pre_eq, uint32_t *chunk_gt,
                                                             uint32_t *chunk_eq)
{
    __shared__ uint32_t lds16[kScanChunk / 64];
    if (st->overflow == 0u)
        slots_count(st, slot_cnt, slot_bits, ntiles, crowded, R, n, cnt_gt, cnt_eq, pre_gt, pre_eq, chunk_gt,
                    chunk_eq, gridDim.x, lds16);
    else
        general_scan_a(cnt_gt, cnt_eq, ntiles, chunk_gt, chunk_eq, lds16);
}

// The ordered write of (value, index), and +0 into the residual there: from the slots
// (one workgroup per chunk), or (general tail) from the residual, one wave per tile.
__global__ __launch_bounds__(kScanChunk) void k_topk_emit(float *R, int64_t n, const topk_state *__restrict__ st,
                                                            const uint32_t *__restrict__ slot_cnt,
                                                            const uint32_t *__restrict__ slot_idx,
                                                            const uint32_t *__restrict__ slot_bits,
                                                            const uint32_t *__restrict__ crowded,
                                                            const uint32_t *__restrict__ cnt_gt,
                                                            const uint32_t *__restrict__ cnt_eq,
                                                            const uint32_t *__restrict__ pre_gt,
                                                            const uint32_t *__restrict__ pre_eq,
                                                            const uint32_t *__restrict__ chunk_gt,
                                                            const uint32_t *__restrict__ chunk_eq, int64_t ntiles,
                                                            float *__restrict__ vals, uint32_t *__restrict__ idx,
                                                            uint32_t kmax, uint32_t slot_groups, uint32_t gen_groups)
{
    __shared__ uint32_t lds16[kScanChunk / 64];
    if (st->overflow == 0u) {
        if (blockIdx.x >= slot_groups) return;
        slots_write(R, n, st, slot_cnt, slot_idx, slot_bits, crowded, cnt_gt, cnt_eq, pre_gt, pre_eq, chunk_gt,
                    chunk_eq, ntiles, vals, idx, kmax, slot_groups, lds16);
    } else {
        if (blockIdx.x >= gen_groups) return;
        general_write<kScanChunk>(R, n, ntiles, st, cnt_gt, cnt_eq, chunk_gt, chunk_eq, vals, idx, kmax, gen_groups);
    }
}

// Argument checks shared by the entry points; `what` names the caller in the message.
covap_status_t check_topk_args(const char *what, const void *grad, const void *residual, int64_t n, int64_t k,
                               int32_t dtype, const void *out_vals, const uint32_t *out_idx)
{
    char msg[160];
    if (dtype != COVAP_F32) {
        std::snprintf(msg, sizeof msg, "%s: fp32 only", what);
        return covap::fail(COVAP_EUNSUPPORTED, msg);
    }
    if (n < 0 || k < 0 || k > n) {
        std::snprintf(msg, sizeof msg, "%s: need 0 <= k <= n", what);
        return covap::fail(COVAP_EINVAL, msg);
    }
    if (n >= ((int64_t)1 << 32)) {
        std::snprintf(msg, sizeof msg, "%s: n >= 2^32", what);
        return covap::fail(COVAP_EINVAL, msg);
    }
    if (n == 0) return COVAP_OK;
    if (!grad || !residual || (k > 0 && (!out_vals || !out_idx))) {
        std::snprintf(msg, sizeof msg, "%s: null device pointer", what);
        return covap::fail(COVAP_EINVAL, msg);
    }
    if (((uintptr_t)grad & 15u) || ((uintptr_t)residual & 15u) || ((uintptr_t)out_vals & 3u) ||
        ((uintptr_t)out_idx & 3u)) {
        std::snprintf(msg, sizeof msg, "%s: misaligned device pointer", what);
        return covap::fail(COVAP_EINVAL, msg);
    }
    return COVAP_OK;
}

// Enqueues the whole selection on `st`.  Arguments are already validated;
// `workspace` holds at least ws_layout(n) bytes on a 256-byte boundary.  The first
// kernel resets every part of the workspace that a later one adds to, so stale
// contents are harmless.
covap::launch_status run_topk(const void *grad, void *residual, int64_t n, int64_t k, float ef_coeff,
                              void *out_vals, uint32_t *out_idx, void *workspace, hipStream_t st)
{
    covap::launch_status ls;
    topk_ws ws;
    ws_layout(n, workspace, &ws);
    const float *G = (const float *)grad;
    float *R = (float *)residual;
    const int64_t nvec = n / 4;
    const int64_t ntiles = div_up(n, kTile);
    const uint32_t nchunks = (uint32_t)div_up(ntiles, kScanChunk);

    uint32_t *h1g = ws.hist, *h2g = h1g + 2048, *h3g = h2g + 2048, *h1s = ws.hist + kAtomicRows * 2048,
             *h2s = h1s + kSlotGrid * 2048, *h3s = h2s + kSlotGrid * 2048, *hs = h2s;
    // The sample: n_s of the full 256-element chunks; it proposes a key with `want` of the sample's keys
    // at or above it.  While the sample's share of k is small, `want` is twice that share plus a floor
    // and the key is the lower edge of a level-1 bin (an eighth of an octave): 2 to 10 times k keys are
    // then at or above it, and only more when the keys crowd just below the k-th largest (as they do
    // under error feedback), which errs on the safe side and which the 32 slots of a tile absorb.  For
    // k around 1 % of the data that many keys no longer fit the slots, so the margin falls to 1.5 times
    // the share and the key is placed inside the bin by interpolation; where that misjudges, the general
    // tail takes over, as it would have anyway.
    const int64_t nchunks_s = nvec / 64;
    const int32_t n_s = (int32_t)(nchunks_s < kSampleChunks ? nchunks_s : kSampleChunks);
    const int64_t m = (int64_t)n_s * 256;
    const int64_t ks = div_up(k * m, n);  // the sample's share of k
    const bool interpolate = ks > 512;
    const int64_t quarters = ks <= 512 ? 8 : (ks >= 2048 ? 6 : 8 - (ks - 512) * 2 / 1536);  // margin in quarters
    const int64_t want = div_up(ks * quarters, 4) + 32;
    const uint32_t target = (uint32_t)(want < ((int64_t)1 << 31) ? want : ((int64_t)1 << 31));
    ls += covap::launch(k_topk_sample, dim3(kSlotGrid), dim3(kSampleThreads), 0, st, G, R, ef_coeff, nchunks_s, n_s,
                        ws.state, ws.hist, hs, (uint32_t)k, ws.chunk_gt, ws.chunk_eq, (int32_t)nchunks);
    ls += covap::launch(interpolate ? k_topk_pick_sample<true> : k_topk_pick_sample<false>, dim3(1), dim3(kPickThreads), 0,
                        st, ws.state, hs, target);
    const covap::tuning tn = covap::tune();
    const auto pass1 = tn.topk_pass1_waves == 4 ? k_topk_pass1<4> : (tn.topk_pass1_waves == 2 ? k_topk_pass1<2> : k_topk_pass1<1>);
    ls += covap::launch(pass1, dim3((uint32_t)ntiles), dim3(64 * tn.topk_pass1_waves),
                        (size_t)tn.topk_pass1_lds_pad, st, G, R, n, ntiles, ef_coeff, ws.state, ws.slot_cnt,
                        ws.slot_idx, ws.slot_bits, ws.crowded);
    if (k > 0) {
        // every kernel from here on serves whichever tail the first pick switches on; the general
        // tail's passes walk the data with bounded grids
        const uint32_t gen_hist = (uint32_t)std::min<int64_t>(kGenGrid, div_up(nvec > 0 ? nvec : 1, kSlotThreads));
        const uint32_t gen_tiles = (uint32_t)std::min<int64_t>(4 * kGenGrid, div_up(ntiles, kSlotThreads / 64));
        const uint32_t hist_grid = gen_hist > (uint32_t)kSlotGrid ? gen_hist : (uint32_t)kSlotGrid;
        ls += covap::launch(k_topk_digit1, dim3(kSlotGrid), dim3(kSlotThreads), 0, st, ws.state, ws.slot_cnt,
                            ws.slot_bits, ntiles, ws.crowded, R, n, h1s);
        ls += covap::launch(k_topk_pick1, dim3(1), dim3(kPickThreads), 0, st, ws.state, h1s, crowded_limit(ntiles));
        ls += covap::launch(k_topk_hist_step<2>, dim3(hist_grid), dim3(kSlotThreads), 0, st, ws.state, ws.slot_cnt,
                            ws.slot_bits, ntiles, ws.crowded, R, n, h2s, h1g, gen_hist);
        ls += covap::launch(k_topk_pick_step<2>, dim3(gen_hist), dim3(kSlotThreads), 0, st, ws.state, h2s, R, n,
                            ntiles, h2g, ws.cnt_gt, ws.cnt_eq, gen_hist);
        ls += covap::launch(k_topk_hist_step<3>, dim3(hist_grid), dim3(kSlotThreads), 0, st, ws.state, ws.slot_cnt,
                            ws.slot_bits, ntiles, ws.crowded, R, n, h3s, h3g, gen_hist);
        ls += covap::launch(k_topk_pick_step<3>, dim3(gen_tiles), dim3(kSlotThreads), 0, st, ws.state, h3s, R, n,
                            ntiles, h3g, ws.cnt_gt, ws.cnt_eq, gen_tiles);
        ls += covap::launch(k_topk_count, dim3(nchunks), dim3(kScanChunk), 0, st, ws.state, ws.slot_cnt,
                            ws.slot_bits, ntiles, ws.crowded, R, n, ws.cnt_gt, ws.cnt_eq, ws.pre_gt, ws.pre_eq,
                            ws.chunk_gt, ws.chunk_eq);
        ls += covap::launch(k_topk_scan_b, dim3(1), dim3(kSlotThreads), 0, st, ws.chunk_gt, ws.chunk_eq, (int64_t)nchunks);
        const uint32_t gen_emit = (uint32_t)std::min<int64_t>(16 * kGenGrid, div_up(ntiles, kScanChunk / 64));
        ls += covap::launch(k_topk_emit, dim3(nchunks > gen_emit ? nchunks : gen_emit), dim3(kScanChunk), 0, st, R, n,
                            ws.state, ws.slot_cnt, ws.slot_idx, ws.slot_bits, ws.crowded, ws.cnt_gt, ws.cnt_eq,
                            ws.pre_gt, ws.pre_eq, ws.chunk_gt, ws.chunk_eq, ntiles, (float *)out_vals, out_idx,
                            (uint32_t)k, nchunks, gen_emit);
    }
    return ls;
}

// ---- the workspace of topk_compress_static ----------------------------------------------
//
// Callers that may not allocate (HIP graph capture, serving loops) get the workspace
// from a fixed array in the code object.  Every GPU the library runs on holds its own
// copy at its own address until the process ends; host code must not use the array's
// name as an address, only what hipGetSymbolAddress returns for the current device.
constexpr int64_t kStaticMaxN = (int64_t)1 << 24;  // 16 Mi elements: about 6.2 MB of workspace
constexpr size_t kStaticBytes = ws_offsets_for(kStaticMaxN).total;
constexpr int kMaxDevices = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

std::atomic<void *> g_scratch_ptr[kMaxDevices];  // device address of `scratch`, by device ordinal

// Device address of the current device's copy of `scratch`; looked up once per device.
// Two threads that race here both get the same address.
covap_status_t static_workspace(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        char msg[200];
        std::snprintf(msg, sizeof msg, "topk_compress_static: hipGetDevice: %s", hipGetErrorString(e));
        return covap::fail(COVAP_EHIP, msg);
    }
    if (dev < 0 || dev >= kMaxDevices)
        return covap::fail(COVAP_EUNSUPPORTED, "topk_compress_static: device ordinal beyond 63");
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            char msg[200];
            std::snprintf(msg, sizeof msg, "topk_compress_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
            return covap::fail(COVAP_EHIP, msg);
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return COVAP_OK;
}

}  // namespace

extern "C" {

size_t topk_workspace_bytes(int64_t n, int32_t dtype)
{
    if (n < 0 || dtype != COVAP_F32) return 0;  // fp32 only, as topk_compress
    return ws_layout(n, nullptr, nullptr);
}

covap_status_t topk_compress(const void *grad, void *residual, int64_t n, int64_t k, int32_t dtype,
                             float ef_coeff, void *out_vals, uint32_t *out_idx, void *workspace,
                             size_t ws_bytes, void *stream)
{
    covap::clear_error();
    const covap_status_t rs = check_topk_args("topk_compress", grad, residual, n, k, dtype, out_vals, out_idx);
    if (rs != COVAP_OK || n == 0) return rs;
    if (!workspace) return covap::fail(COVAP_EINVAL, "topk_compress: null device pointer");
    if ((uintptr_t)workspace & 255u) return covap::fail(COVAP_EINVAL, "topk_compress: misaligned device pointer");
    if (ws_bytes < ws_layout(n, nullptr, nullptr))
        return covap::fail(COVAP_EINVAL, "topk_compress: workspace too small");
    return run_topk(grad, residual, n, k, ef_coeff, out_vals, out_idx, workspace, (hipStream_t)stream)
        .report("topk_compress");
}

int64_t topk_static_max_elems(void) { return kStaticMaxN; }

covap_status_t topk_compress_static(const void *grad, void *residual, int64_t n, int64_t k, int32_t dtype,
                                    float ef_coeff, void *out_vals, uint32_t *out_idx, void *stream)
{
    covap::clear_error();
    const covap_status_t rs =
        check_topk_args("topk_compress_static", grad, residual, n, k, dtype, out_vals, out_idx);
    if (rs != COVAP_OK || n == 0) return rs;
    if (n > kStaticMaxN)
        return covap::fail(COVAP_EINVAL,
                           "topk_compress_static: n exceeds topk_static_max_elems() (2^24); use topk_compress "
                           "with a caller-owned workspace");
    static_assert(ws_offsets_for(kStaticMaxN).total <= kStaticBytes, "scratch holds the largest layout");
    void *workspace = nullptr;
    const covap_status_t ws = static_workspace(&workspace);
    if (ws != COVAP_OK) return ws;
    return run_topk(grad, residual, n, k, ef_coeff, out_vals, out_idx, workspace, (hipStream_t)stream)
        .report("topk_compress_static");
}

}  // extern "C"
