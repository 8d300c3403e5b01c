// Further contrast points on the same buffers as the COVAP path: the two
// schemes the paper singles out as free of data dependencies (Sec. II-C,
// Table III) -- Random-k and FP16 -- each with the error feedback of Algorithm 1,
// and the matching decompress sides (N-way mean of sparse / half payloads).
// Like top-k they are here to be measured against, not to be the product:
// plain streaming kernels with 16-byte accesses and streaming cache hints.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "half_util.h"
#include "launch.h"
#include "plan.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 64;  // one wave per workgroup, one vector per thread (measured best)

using covap_dev::half_hi;
using covap_dev::half_lo;
using covap_dev::pack_half2;
using covap_dev::pinned;

// R <- fma(c, R, G) over n fp32 elements (Algorithm 1 line 2 alone).
__global__ __launch_bounds__(kThreads) void k_ef_accumulate(const float *__restrict__ G, float *R,
                                                            int64_t n, float c)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t nvec = n / 4;
    if (v < nvec) {
        const f32x4 g = __builtin_nontemporal_load((const f32x4 *)G + v);
        const f32x4 r = __builtin_nontemporal_load((const f32x4 *)R + v);
        f32x4 a;
        a.x = __builtin_fmaf(c, r.x, g.x);
        a.y = __builtin_fmaf(c, r.y, g.y);
        a.z = __builtin_fmaf(c, r.z, g.z);
        a.w = __builtin_fmaf(c, r.w, g.w);
        __builtin_nontemporal_store(a, (f32x4 *)R + v);  // streaming: the gather that follows touches 1 % of it
    }
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - nvec * 4) {
        const int64_t i = nvec * 4 + threadIdx.x;
        R[i] = __builtin_fmaf(c, R[i], G[i]);
    }
}

// vals[j] = R[idx[j]]; R[idx[j]] = +0 (the sent coordinates leave no residual).
__global__ __launch_bounds__(256) void k_gather_clear(float *R, const uint32_t *__restrict__ idx,
                                                      int64_t k, float *__restrict__ vals)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < k) {
        const uint32_t i = idx[j];
        vals[j] = R[i];
        R[i] = 0.0f;
    }
}

// FP16 quantiser: h = fp16(A), residual = A - h.
__global__ __launch_bounds__(kThreads) void k_fp16_compress(const float *__restrict__ G, float *R,
                                                            int64_t n, float c,
                                                            uint16_t *__restrict__ out)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t nvec = n / 4;
    if (v < nvec) {
        const f32x4 g = __builtin_nontemporal_load((const f32x4 *)G + v);
        const f32x4 r = __builtin_nontemporal_load((const f32x4 *)R + v);
        f32x4 a;
        a.x = pinned(__builtin_fmaf(c, r.x, g.x));
        a.y = pinned(__builtin_fmaf(c, r.y, g.y));
        a.z = pinned(__builtin_fmaf(c, r.z, g.z));
        a.w = pinned(__builtin_fmaf(c, r.w, g.w));
        u32x2 h;
        h.x = pack_half2(a.x, a.y);
        h.y = pack_half2(a.z, a.w);
        a.x -= half_lo(h.x);
        a.y -= half_hi(h.x);
        a.z -= half_lo(h.y);
        a.w -= half_hi(h.y);
        __builtin_nontemporal_store(h, (u32x2 *)out + v);
        __builtin_nontemporal_store(a, (f32x4 *)R + v);
    }
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - nvec * 4) {
        const int64_t i = nvec * 4 + threadIdx.x;
        const float a = pinned(__builtin_fmaf(c, R[i], G[i]));
        const __half h = __float2half_rn(a);
        out[i] = __half_as_ushort(h);
        R[i] = a - __half2float(h);
    }
}

// out[i] = (sum over rows w = 0..N-1, in that order, of float(recv[w][i])) / N
__global__ __launch_bounds__(kThreads) void k_fp16_decompress(const uint16_t *__restrict__ recv,
                                                              int32_t N, int64_t stride, int64_t n,
                                                              float *__restrict__ out, float n_f,
                                                              float inv_n, int pow2)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // 8 elements each
    const int64_t nvec = n / 8;
    if (v < nvec) {
        const u32x4 *p = (const u32x4 *)recv + v;
        const int64_t stride_vec = stride / 8;
        float acc[8];
        {
            const u32x4 x = __builtin_nontemporal_load(p);
            acc[0] = half_lo(x.x); acc[1] = half_hi(x.x); acc[2] = half_lo(x.y); acc[3] = half_hi(x.y);
            acc[4] = half_lo(x.z); acc[5] = half_hi(x.z); acc[6] = half_lo(x.w); acc[7] = half_hi(x.w);
        }
        for (int32_t w = 1; w < N; ++w) {
            const u32x4 x = __builtin_nontemporal_load(p + (int64_t)w * stride_vec);
            acc[0] += half_lo(x.x); acc[1] += half_hi(x.x); acc[2] += half_lo(x.y); acc[3] += half_hi(x.y);
            acc[4] += half_lo(x.z); acc[5] += half_hi(x.z); acc[6] += half_lo(x.w); acc[7] += half_hi(x.w);
        }
        f32x4 o0, o1;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = pow2 ? acc[j] * inv_n : __fdiv_rn(acc[j], n_f);
        o0.x = acc[0]; o0.y = acc[1]; o0.z = acc[2]; o0.w = acc[3];
        o1.x = acc[4]; o1.y = acc[5]; o1.z = acc[6]; o1.w = acc[7];
        __builtin_nontemporal_store(o0, (f32x4 *)out + 2 * v);
        __builtin_nontemporal_store(o1, (f32x4 *)out + 2 * v + 1);
    }
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - nvec * 8) {
        const int64_t i = nvec * 8 + threadIdx.x;
        float acc = __half2float(__ushort_as_half(recv[i]));
        for (int32_t w = 1; w < N; ++w) acc += __half2float(__ushort_as_half(recv[(int64_t)w * stride + i]));
        out[i] = pow2 ? acc * inv_n : __fdiv_rn(acc, n_f);
    }
}

__global__ __launch_bounds__(kThreads) void k_zero(float *__restrict__ out, int64_t n)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t nvec = n / 4;
    const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
    if (v < nvec) __builtin_nontemporal_store(z, (f32x4 *)out + v);
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - nvec * 4) out[nvec * 4 + threadIdx.x] = 0.0f;
}

// One worker's sparse payload added into the dense buffer.  Indices inside one
// payload are distinct, so the plain read-add-write has no race; payloads are
// applied by successive launches, which fixes the order of the additions.
__global__ __launch_bounds__(256) void k_scatter_add(float *out, const uint32_t *__restrict__ idx,
                                                     const float *__restrict__ vals, int64_t k)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < k) {
        const uint32_t i = idx[j];
        out[i] = out[i] + vals[j];
    }
}

__global__ __launch_bounds__(kThreads) void k_scale(float *out, int64_t n, float n_f, float inv_n, int pow2)
{
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t nvec = n / 4;
    if (v < nvec) {
        f32x4 x = ((const f32x4 *)out)[v];
        x.x = pow2 ? x.x * inv_n : __fdiv_rn(x.x, n_f);
        x.y = pow2 ? x.y * inv_n : __fdiv_rn(x.y, n_f);
        x.z = pow2 ? x.z * inv_n : __fdiv_rn(x.z, n_f);
        x.w = pow2 ? x.w * inv_n : __fdiv_rn(x.w, n_f);
        __builtin_nontemporal_store(x, (f32x4 *)out + v);
    }
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - nvec * 4) {
        const int64_t i = nvec * 4 + threadIdx.x;
        out[i] = pow2 ? out[i] * inv_n : __fdiv_rn(out[i], n_f);
    }
}

constexpr int kSpTile = 4096;
constexpr int kSpRows = 64;

__device__ __forceinline__ void lds_add(float *p, float v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);  // ds_add_f32
}

// Mean of N <= 64 sparse payloads whose indices ascend inside every row (what
// topk_compress writes), in one pass over the dense result, as a pipeline of four waves.
// A workgroup walks one run of consecutive 4096-element tiles with four tile buffers in
// LDS.  Wave w owns a quarter of the payload rows (rows in worker order: wave 0 the first
// quarter) and in phase p adds its rows into tile p - w, so a tile passes through the
// waves in row order, one phase apart, with a barrier between phases.  The tile that has
// passed the last wave is scaled, written out and cleared by all four waves together.
//
// Inside a wave: every row has a cursor (found by a binary search at the start of the run
// and carried forward).  Per tile one load instruction fetches the 16 entries after the
// cursor of four rows at a time (lane = 16 * row-in-group + entry); those that fall into
// the tile are added with LDS float adds, one instruction per row and the rows in
// ascending order.  That is the worker order the definition asks for: LDS operations of
// one wave are carried out in program order, the waves follow each other across barriers,
// entries of one row are distinct (no two lanes of an instruction meet), and the LDS adder
// rounds to nearest even with subnormals like the vector unit (the parity tests cover
// both).  The common case is straight-line code -- every load of a tile is unconditional
// (clamped addresses, masked results), and the next tile's windows are in flight before
// this tile's adds; a tile in which some row has 16 or more entries takes a plain loop
// instead.  Unsorted rows give an unspecified result but no access outside the buffers.
//
// Against one wave doing all of this for a tile (which is how this kernel started: 0.39 ms
// on the GPT-2-medium-shaped set, this form 0.28 ms): the write-out is four 16-byte stores
// per lane from four waves instead of sixteen from one, the payload work of a tile is
// spread over four waves with a quarter of the rows and of the registers each (107
// instead of 229), and a compute unit holds eight such waves instead of five.
// ROWS = 16, 32 or 64 (the smallest that holds N); a wave has ROWS / 4 rows.
template <int ROWS, bool FULL>  // FULL: N == ROWS
__global__ __launch_bounds__(256) void k_sparse_mean_pipe(const float *__restrict__ vals,
                                                          const uint32_t *__restrict__ idx, int32_t N,
                                                          uint32_t k, int64_t stride, int64_t n,
                                                          float *__restrict__ out, int64_t tiles_per_wg,
                                                          float n_f, float inv_n, int pow2)
{
    constexpr int RW = ROWS / 4;     // rows of a wave
    constexpr int GROUPS = RW / 4;   // groups of four rows: one load instruction each
    static_assert(GROUPS >= 1 && (RW & (RW - 1)) == 0, "4, 8 or 16 rows per wave");
    __shared__ __align__(16) float tiles[4][kSpTile];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int q = lane >> 4, e = lane & 15;  // row inside a group of four, entry inside the window
    const int64_t ntiles = (n + kSpTile - 1) / kSpTile;
    const int64_t tile_lo = (int64_t)blockIdx.x * tiles_per_wg;
    int64_t tile_hi = tile_lo + tiles_per_wg;
    if (tile_hi > ntiles) tile_hi = ntiles;
    if (tile_lo >= tile_hi) return;  // the whole workgroup; k >= 1 from here on (the host handles empty payloads)
    const int64_t nrun = tile_hi - tile_lo;
    const int row0 = wv * RW;  // this wave's rows: row0 .. row0 + RW - 1

    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int v = 0; v < 4 * kSpTile / 4 / 256; ++v) ((f32x4 *)&tiles[0][0])[v * 256 + tid] = zero;

    // Cursor of row row0 + (lane mod RW): first entry whose index is >= the start of the run.
    uint32_t start = 0u;
    {
        const int my_row = row0 + (lane & (RW - 1));
        if (my_row < N) {
            const uint32_t *my_idx = idx + (int64_t)my_row * stride;
            const uint32_t first = (uint32_t)(tile_lo * kSpTile);
            uint32_t lo = 0u, hi = k;
            while (lo < hi) {
                const uint32_t mid = lo + ((hi - lo) >> 1);
                if (my_idx[mid] < first)
                    lo = mid + 1u;
                else
                    hi = mid;
            }
            start = lo;
        }
    }
    // Every lane carries, for each group g, the cursor and the row base of the row it
    // loads for: row0 + 4g + q.  The 16 lanes of a row hold the same cursor.
    uint32_t cur[GROUPS];
    uint32_t row_off[GROUPS];  // first entry of the row in idx / vals (the host checks that it fits 32 bits)
    bool row_live[GROUPS];
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const int w = row0 + 4 * g + q;
        cur[g] = (uint32_t)__shfl((int)start, 4 * g + q, 64);
        row_live[g] = FULL || w < N;
        row_off[g] = (uint32_t)(row_live[g] ? w : 0) * (uint32_t)stride;
    }
    const uint32_t k_last = k - 1u;

    // Window [cursor, cursor + 16) of every row: raw index and value, loaded unconditionally
    // (addresses clamped to the row); what lies outside the row or the tile is masked out.
    uint32_t raw[GROUPS];
    float val[GROUPS];
    auto load_windows = [&]() {
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            const uint32_t j = cur[g] + (uint32_t)e;  // no wrap: cursor <= k <= n < 2^32 - 16 (checked on the host)
            const uint64_t at = (uint64_t)row_off[g] + (j < k ? j : k_last);
            raw[g] = idx[at];
            val[g] = vals[at];
        }
    };
    load_windows();
    __syncthreads();  // the buffers are clear

    for (int64_t p = 0; p < nrun + 3; ++p) {
        const int64_t ti = p - wv;  // this wave's tile in this phase, counted from the start of the run
        if (ti >= 0 && ti < nrun) {  // the same in every lane of the wave
            float *tile = tiles[ti & 3];
            const int64_t T0 = (tile_lo + ti) * kSpTile;
            const int64_t left = n - T0;
            const uint32_t len = (uint32_t)(left < kSpTile ? left : kSpTile);
            uint32_t rel[GROUPS];
            float now[GROUPS];
            bool full_window = false;  // a row whose 16th entry is in the tile may have more there
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const uint32_t j = cur[g] + (uint32_t)e;
                const uint32_t r = raw[g] - (uint32_t)T0;  // wraps to a huge value below T0
                rel[g] = (row_live[g] && j < k) ? r : 0xffffffffu;
                now[g] = val[g];
                full_window |= e == 15 && rel[g] < len;
            }
            if (__ballot(full_window) == 0ull) {
#pragma unroll
                for (int g = 0; g < GROUPS; ++g) {
                    const uint64_t m = __ballot(rel[g] < len);
                    cur[g] += (uint32_t)__popcll((m >> (16 * q)) & 0xffffull);  // in-tile entries of this lane's row
                }
                load_windows();  // the next tile's, in flight during the adds and the phases in between
#pragma unroll
                for (int g = 0; g < GROUPS; ++g) {
                    const bool in = rel[g] < len;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {  // one add instruction per row, rows in order
                        if (q == r && in) lds_add(&tile[rel[g]], now[g]);
                    }
                }
            } else {
                // crowded tile: four rows at a time, the next 256 entries of each (four loads of
                // 64), all sixteen index and value loads in flight together; a row that still has
                // entries in the tile after that goes on alone, 64 at a time
                for (int g0 = 0; g0 < GROUPS; ++g0) {
                    const int w0 = row0 + 4 * g0;
                    uint32_t cg = 0u;
#pragma unroll
                    for (int g = 0; g < GROUPS; ++g) cg = g == g0 ? cur[g] : cg;
                    uint32_t base[4], rr[4][4];
                    float vv[4][4];
                    bool lv[4][4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int w = w0 + r;
                        const bool live = w < N;
                        base[r] = (uint32_t)__shfl((int)cg, r * 16, 64);
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int64_t j = (int64_t)base[r] + 64 * u + lane;
                            const int64_t at = (int64_t)(live ? w : 0) * stride + (j < (int64_t)k ? j : (int64_t)k - 1);
                            rr[r][u] = idx[at];
                            vv[r][u] = vals[at];
                            lv[r][u] = live && j < (int64_t)k;
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);  // all thirty-two loads first
                    uint32_t tot[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {  // rows in order
                        tot[r] = 0u;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const uint32_t rel_u = lv[r][u] ? rr[r][u] - (uint32_t)T0 : 0xffffffffu;
                            const bool in = rel_u < len;
                            tot[r] += (uint32_t)__popcll(__ballot(in));
                            if (in) lds_add(&tile[rel_u], vv[r][u]);
                        }
                        if (tot[r] == 256u) {
                            const int w = w0 + r;  // < N: a dead row has no entries
                            uint32_t cnt = 64u;
                            while (cnt == 64u) {
                                const int64_t j = (int64_t)base[r] + tot[r] + lane;
                                uint32_t rel_j = 0xffffffffu;
                                if (j < (int64_t)k) rel_j = idx[(int64_t)w * stride + j] - (uint32_t)T0;
                                const bool in = rel_j < len;
                                cnt = (uint32_t)__popcll(__ballot(in));
                                if (in) lds_add(&tile[rel_j], vals[(int64_t)w * stride + j]);
                                tot[r] += cnt;
                            }
                        }
                    }
                    const uint32_t add = q == 0 ? tot[0] : (q == 1 ? tot[1] : (q == 2 ? tot[2] : tot[3]));
#pragma unroll
                    for (int g = 0; g < GROUPS; ++g)
                        if (g == g0) cur[g] += add;
                }
                load_windows();
            }
        }
        __syncthreads();  // every wave's additions of this phase are in LDS

        // the tile that has passed all four waves: mean, write-out, and its buffer cleared
        const int64_t tw = p - 3;
        if (tw >= 0) {  // tw < nrun, since p < nrun + 3
            float *src = tiles[tw & 3];
            const int64_t T0 = (tile_lo + tw) * kSpTile;
            const int64_t left = n - T0;
            float *o = out + T0;
            if (left >= kSpTile) {
#pragma unroll
                for (int v = 0; v < kSpTile / 4 / 256; ++v) {
                    f32x4 x = ((const f32x4 *)src)[v * 256 + tid];
                    ((f32x4 *)src)[v * 256 + tid] = zero;
                    if (N > 1) {
                        x.x = pow2 ? x.x * inv_n : __fdiv_rn(x.x, n_f);
                        x.y = pow2 ? x.y * inv_n : __fdiv_rn(x.y, n_f);
                        x.z = pow2 ? x.z * inv_n : __fdiv_rn(x.z, n_f);
                        x.w = pow2 ? x.w * inv_n : __fdiv_rn(x.w, n_f);
                    }
                    __builtin_nontemporal_store(x, (f32x4 *)o + v * 256 + tid);
                }
            } else {  // the arena's last, short tile (the run ends here: the buffer is not used again)
                for (int64_t i = tid; i < left; i += 256) {
                    float x = src[i];
                    if (N > 1) x = pow2 ? x * inv_n : __fdiv_rn(x, n_f);
                    o[i] = x;
                }
            }
        }
        __syncthreads();  // the buffer is clear before a wave adds to it again
    }
}

bool al16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
uint32_t blocks(int64_t items, int per) { return (uint32_t)((items + per - 1) / per); }

}  // namespace

using covap::fail;

extern "C" {

covap_status_t randk_compress(const void *grad, void *residual, int64_t n, const uint32_t *idx,
                              int64_t k, float ef_coeff, void *out_vals, void *stream)
{
    covap::clear_error();
    if (n < 0 || k < 0 || k > n || n >= ((int64_t)1 << 32))
        return fail(COVAP_EINVAL, "randk_compress: need 0 <= k <= n < 2^32");
    if (n == 0) return COVAP_OK;
    if (!grad || !residual || (k > 0 && (!idx || !out_vals)))
        return fail(COVAP_EINVAL, "randk_compress: null device pointer");
    if (!al16(grad) || !al16(residual) || ((uintptr_t)idx & 3u) || ((uintptr_t)out_vals & 3u))
        return fail(COVAP_EINVAL, "randk_compress: misaligned device pointer");
    hipStream_t st = (hipStream_t)stream;
    covap::launch_status ls;
    ls += covap::launch(k_ef_accumulate, dim3(blocks(n / 4 > 0 ? n / 4 : 1, kThreads)), dim3(kThreads), 0, st,
                        (const float *)grad, (float *)residual, n, ef_coeff);
    if (k > 0)
        ls += covap::launch(k_gather_clear, dim3(blocks(k, 256)), dim3(256), 0, st, (float *)residual, idx, k,
                            (float *)out_vals);
    return ls.report("randk_compress");
}

covap_status_t fp16_compress(const void *grad, void *residual, int64_t n, float ef_coeff,
                             void *out_half, void *stream)
{
    covap::clear_error();
    if (n < 0) return fail(COVAP_EINVAL, "fp16_compress: n < 0");
    if (n == 0) return COVAP_OK;
    if (!grad || !residual || !out_half) return fail(COVAP_EINVAL, "fp16_compress: null device pointer");
    if (!al16(grad) || !al16(residual) || !al16(out_half))
        return fail(COVAP_EINVAL, "fp16_compress: device pointers must be 16-byte aligned");
    covap::launch_status ls;
    ls += covap::launch(k_fp16_compress, dim3(blocks(n / 4 > 0 ? n / 4 : 1, kThreads)), dim3(kThreads), 0,
                        (hipStream_t)stream, (const float *)grad, (float *)residual, n, ef_coeff,
                        (uint16_t *)out_half);
    return ls.report("fp16_compress");
}

covap_status_t fp16_decompress(const void *recv, int32_t n_workers, int64_t stride_elems, int64_t n,
                               void *dense_out, void *stream)
{
    covap::clear_error();
    if (n < 0 || n_workers < 1 || stride_elems < n)
        return fail(COVAP_EINVAL, "fp16_decompress: need n >= 0, n_workers >= 1, stride >= n");
    if (n_workers > 1 && stride_elems % 8 != 0)
        return fail(COVAP_EINVAL, "fp16_decompress: row stride must be a multiple of 16 bytes");
    if (n == 0) return COVAP_OK;
    if (!recv || !dense_out || !al16(recv) || !al16(dense_out))
        return fail(COVAP_EINVAL, "fp16_decompress: null or misaligned device pointer");
    const int pow2 = (n_workers & (n_workers - 1)) == 0;
    const float n_f = (float)n_workers;
    covap::launch_status ls;
    ls += covap::launch(k_fp16_decompress, dim3(blocks(n / 8 > 0 ? n / 8 : 1, kThreads)), dim3(kThreads), 0,
                        (hipStream_t)stream, (const uint16_t *)recv, n_workers, stride_elems, n, (float *)dense_out,
                        n_f, 1.0f / n_f, pow2);
    return ls.report("fp16_decompress");
}

covap_status_t sparse_decompress(const void *vals, const uint32_t *idx, int32_t n_workers, int64_t k,
                                 int64_t stride_elems, int64_t n, void *dense_out, void *stream)
{
    covap::clear_error();
    if (n < 0 || k < 0 || k > n || n_workers < 1 || stride_elems < k || n >= ((int64_t)1 << 32))
        return fail(COVAP_EINVAL, "sparse_decompress: need 0 <= k <= n < 2^32, n_workers >= 1, stride >= k");
    if (n == 0) return COVAP_OK;
    if (!dense_out || !al16(dense_out) || (k > 0 && (!vals || !idx)))
        return fail(COVAP_EINVAL, "sparse_decompress: null or misaligned device pointer");
    if (((uintptr_t)vals & 3u) || ((uintptr_t)idx & 3u))
        return fail(COVAP_EINVAL, "sparse_decompress: misaligned device pointer");
    hipStream_t st = (hipStream_t)stream;
    float *out = (float *)dense_out;
    const uint32_t dense_grid = blocks(n / 4 > 0 ? n / 4 : 1, kThreads);
    covap::launch_status ls;
    ls += covap::launch(k_zero, dim3(dense_grid), dim3(kThreads), 0, st, out, n);
    if (k > 0) {
        for (int32_t w = 0; w < n_workers; ++w)
            ls += covap::launch(k_scatter_add, dim3(blocks(k, 256)), dim3(256), 0, st, out,
                                idx + (int64_t)w * stride_elems, (const float *)vals + (int64_t)w * stride_elems, k);
        if (n_workers > 1) {
            const int pow2 = (n_workers & (n_workers - 1)) == 0;
            const float n_f = (float)n_workers;
            ls += covap::launch(k_scale, dim3(dense_grid), dim3(kThreads), 0, st, out, n, n_f, 1.0f / n_f, pow2);
        }
    }
    return ls.report("sparse_decompress");
}

covap_status_t sparse_decompress_sorted(const void *vals, const uint32_t *idx, int32_t n_workers,
                                        int64_t k, int64_t stride_elems, int64_t n, void *dense_out,
                                        void *stream)
{
    // the one-pass kernel keeps one cursor per lane, wants k >= 1 and 32-bit offsets into the payloads
    if (n_workers > kSpRows || k == 0 || (int64_t)n_workers * stride_elems >= ((int64_t)1 << 32))
        return sparse_decompress(vals, idx, n_workers, k, stride_elems, n, dense_out, stream);
    covap::clear_error();
    if (n < 0 || k < 0 || k > n || n_workers < 1 || stride_elems < k || n >= ((int64_t)1 << 32) - 16)
        return fail(COVAP_EINVAL,
                    "sparse_decompress_sorted: need 0 <= k <= n < 2^32 - 16, n_workers >= 1, stride >= k");
    if (n == 0) return COVAP_OK;
    if (!dense_out || !al16(dense_out) || (k > 0 && (!vals || !idx)))
        return fail(COVAP_EINVAL, "sparse_decompress_sorted: null or misaligned device pointer");
    if (((uintptr_t)vals & 3u) || ((uintptr_t)idx & 3u))
        return fail(COVAP_EINVAL, "sparse_decompress_sorted: misaligned device pointer");
    const int64_t ntiles = (n + kSpTile - 1) / kSpTile;
    // Two workgroups per CU (four tile buffers each fill the LDS), all resident at once, each
    // with one long run of tiles.
    int64_t tiles_per_wg = (ntiles + 511) / 512;
    if (tiles_per_wg < 1) tiles_per_wg = 1;
    const uint32_t grid = (uint32_t)((ntiles + tiles_per_wg - 1) / tiles_per_wg);
    const int pow2 = (n_workers & (n_workers - 1)) == 0;
    const float n_f = (float)n_workers;
    const auto kern = n_workers == 64   ? k_sparse_mean_pipe<64, true>
                      : n_workers > 32  ? k_sparse_mean_pipe<64, false>
                      : n_workers == 32 ? k_sparse_mean_pipe<32, true>
                      : n_workers > 16  ? k_sparse_mean_pipe<32, false>
                      : n_workers == 16 ? k_sparse_mean_pipe<16, true>
                                        : k_sparse_mean_pipe<16, false>;
    covap::launch_status ls;
    ls += covap::launch(kern, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const float *)vals, idx, n_workers,
                        (uint32_t)k, stride_elems, n, (float *)dense_out, tiles_per_wg, n_f, 1.0f / n_f, pow2);
    return ls.report("sparse_decompress_sorted");
}


}  // extern "C"
