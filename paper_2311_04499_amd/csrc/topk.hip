// Fine-grained top-k sparsifier with error feedback: the contrast point to the
// coarse filter (Sec. I and Table II: "most of the overhead in Top-k comes from
// the topk() operator").  Exact, deterministic, no sampling:
//
//   pass 1   A = fma(c, R, G); R <- A; histogram of key bits 30..20        (reads 2D, writes D)
//   pass 2   histogram of bits 19..9 among keys whose bits 30..20 match    (reads D)
//   pass 3   histogram of bits 8..0 among keys whose bits 30..9 match      (reads D)
//            -> threshold key T and the number of ties to keep
//   pass 4   per tile: how many keys > T, how many == T                    (reads D)
//            3-phase exclusive scan of the tile counts (tiny)
//   pass 5   ordered compaction: (value, index) in ascending index,
//            R <- +0 at kept entries                                       (reads the tiles that keep something)
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
};

struct topk_ws {
    topk_state *state;
    uint32_t *hist;       // [3][2048]
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
    const size_t o_hist = take(3 * 2048 * sizeof(uint32_t));
    const size_t o_gt = take((size_t)ntiles * 4);
    const size_t o_eq = take((size_t)ntiles * 4);
    const size_t o_cgt = take((size_t)nchunks * 4);
    const size_t o_ceq = take((size_t)nchunks * 4);
    if (out) {
        char *b = (char *)base;
        out->state = (topk_state *)(b + o_state);
        out->hist = (uint32_t *)(b + o_hist);
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
    for (int i = threadIdx.x; i < 3 * 2048; i += blockDim.x) hist[i] = 0u;
    if (threadIdx.x == 0) {
        st->prefix = 0u;
        st->k_rem = k;
        st->threshold = 0u;
        st->ties = 0u;
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
    uint32_t *mine = lds[tid >> 6];
    for (int i = tid; i < kHistWaves * BINS; i += kHistThreads) (&lds[0][0])[i] = 0u;
    __syncthreads();

    uint32_t want = 0u;
    if constexpr (LEVEL > 1) want = st->prefix >> HI_SHIFT;

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
        if (s) atomicAdd(&hist[b], s);
    }
}

// Finds the digit at which the count from the top reaches k_rem: the largest b
// with sum_{j >= b} hist[j] >= k_rem.  One workgroup of 256 threads.
template <int LEVEL>
__global__ __launch_bounds__(256) void k_topk_pick(topk_state *st, const uint32_t *__restrict__ hist)
{
    constexpr int BINS = LEVEL == 3 ? kBins3 : kBins12;
    constexpr int PER = BINS / 256;
    constexpr int SHIFT = LEVEL == 1 ? 20 : (LEVEL == 2 ? 9 : 0);
    __shared__ uint32_t part[256];
    const int tid = threadIdx.x;
    const uint32_t k_rem = st->k_rem;
    // thread t owns bins [BINS - (t+1)*PER, BINS - t*PER): thread 0 the top ones
    uint32_t h[PER];
    uint32_t mine = 0u;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        h[j] = hist[BINS - 1 - (tid * PER + j)];  // descending bin order
        mine += h[j];
    }
    part[tid] = mine;
    __syncthreads();
    // inclusive scan over threads (Hillis-Steele in LDS)
    for (int d = 1; d < 256; d <<= 1) {
        const uint32_t y = tid >= d ? part[tid - d] : 0u;
        __syncthreads();
        part[tid] += y;
        __syncthreads();
    }
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

__global__ __launch_bounds__(64) void k_topk_count(const float *__restrict__ R, int64_t n,
                                                   const topk_state *__restrict__ st,
                                                   uint32_t *__restrict__ cnt_gt,
                                                   uint32_t *__restrict__ cnt_eq)
{
    const uint32_t T = st->threshold;
    const int lane = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kTile;
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
        cnt_gt[blockIdx.x] = gt;
        cnt_eq[blockIdx.x] = eq;
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
                                                   uint32_t *__restrict__ idx)
{
    const uint32_t T = st->threshold, ties = st->ties;
    const int lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int64_t chunk = tile / kScanChunk;
    const uint32_t gt_before = chunk_gt[chunk] + cnt_gt[tile];
    uint32_t eq_before = chunk_eq[chunk] + cnt_eq[tile];
    // how many this tile keeps: known from the prefixes of the next tile, but a
    // cheap local test is enough to skip tiles that hold nothing at or above T
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
            if ((selm >> j) & 1u) {
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

    k_topk_init<<<1, 256, 0, st>>>(ws.state, ws.hist, (uint32_t)k);
    k_topk_hist<1><<<(uint32_t)hist_grid, kHistThreads, 0, st>>>(G, R, n, ef_coeff, ws.state, ws.hist);
    if (k > 0) {
        k_topk_pick<1><<<1, 256, 0, st>>>(ws.state, ws.hist);
        k_topk_hist<2><<<(uint32_t)hist_grid, kHistThreads, 0, st>>>(G, R, n, ef_coeff, ws.state, ws.hist + 2048);
        k_topk_pick<2><<<1, 256, 0, st>>>(ws.state, ws.hist + 2048);
        k_topk_hist<3><<<(uint32_t)hist_grid, kHistThreads, 0, st>>>(G, R, n, ef_coeff, ws.state, ws.hist + 4096);
        k_topk_pick<3><<<1, 256, 0, st>>>(ws.state, ws.hist + 4096);
        k_topk_count<<<(uint32_t)ntiles, 64, 0, st>>>(R, n, ws.state, ws.cnt_gt, ws.cnt_eq);
        k_topk_scan_a<<<(uint32_t)nchunks, 256, 0, st>>>(ws.cnt_gt, ws.cnt_eq, ntiles, ws.chunk_gt, ws.chunk_eq);
        k_topk_scan_b<<<1, 256, 0, st>>>(ws.chunk_gt, ws.chunk_eq, nchunks);
        k_topk_write<<<(uint32_t)ntiles, 64, 0, st>>>(R, n, ws.state, ws.cnt_gt, ws.cnt_eq, ws.chunk_gt,
                                                     ws.chunk_eq, ntiles, (float *)out_vals, out_idx);
    }
    return check("topk_compress");
}

}  // extern "C"
