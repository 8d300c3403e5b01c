// COVAP hot-path kernels for gfx950 (MI355X): covap_compress (also on a bounded,
// persistent grid), its aliased form, covap_decompress and covap_decompress_reduced
// (the same kernels on one summed row), plus the measurement probes (two plain
// streaming kernels and one that only keeps the matrix cores busy).
//
// Both kernels are pure HBM streaming (at most one FMA per 12 bytes moved), so
// the design is about memory access only:
//   * every thread moves 16-byte vectors; a workgroup of THREADS threads owns one
//     "tile" of THREADS * UNROLL consecutive vectors of ONE shard, so the filter's
//     decision (sent / kept) is uniform over the workgroup and costs a few
//     scalar integer operations per tile -- never per element.  The measured best
//     on MI355X is the smallest shape: one wave, one vector per thread (decompress
//     calls with few rows, which are bound by their stores, take 256 threads);
//   * all loads of a tile are issued before the first use; decompress walks the N
//     payload rows with one row in flight per wave (more was slower);
//   * data that is not read again in the same iteration (everything here) is
//     moved with streaming (non-temporal) hints;
//   * shard starts and packed offsets are multiples of the vector size, so the
//     vector path is always aligned; a shard's ragged tail (< one vector) goes
//     through a scalar path in the same launch.  Alignment to 1 KiB, one wave's
//     access, is faster still, which the planner provides for variable-length shards.
// How a workgroup index becomes a tile is in geom.h (shared with the host, which
// builds the launch geometry in plan.cpp and can replay it).  The hot path uses no LDS
// (beyond an unused reservation that caps occupancy) and no MFMA: there is no data
// reuse and no contraction.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <type_traits>

#include "half_util.h"
#include "launch.h"
#include "plan.h"

namespace {

using covap::fixed_geom;
using covap::table_geom;
using covap::tile_ref;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kProbeThreads = 64;

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <bool NT>
__device__ __forceinline__ void st16(u32x4 *p, u32x4 v)
{
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// ---- element types ---------------------------------------------------------

// fp32 elements: four per 16-byte vector.
struct ops_f32 {
    static constexpr int EPV = 4;
    static constexpr bool MIXED = false;
    static constexpr bool PAY16 = false;
    typedef float elem_t;
    typedef f32x4 acc_t;

    // A = fma(c, r, g): one rounding (Algorithm 1 line 2 with the scheduler's c)
    static __device__ __forceinline__ u32x4 ef(u32x4 g, u32x4 r, float c)
    {
        f32x4 gf = __builtin_bit_cast(f32x4, g), rf = __builtin_bit_cast(f32x4, r), a;
        a.x = __builtin_fmaf(c, rf.x, gf.x);
        a.y = __builtin_fmaf(c, rf.y, gf.y);
        a.z = __builtin_fmaf(c, rf.z, gf.z);
        a.w = __builtin_fmaf(c, rf.w, gf.w);
        return __builtin_bit_cast(u32x4, a);
    }
    static __device__ __forceinline__ float ef1(float g, float r, float c)
    {
        return __builtin_fmaf(c, r, g);
    }
    static __device__ __forceinline__ acc_t widen(u32x4 v) { return __builtin_bit_cast(f32x4, v); }
    static __device__ __forceinline__ void add(acc_t &acc, u32x4 v)
    {
        acc += __builtin_bit_cast(f32x4, v);
    }
    static __device__ __forceinline__ float mean1(float acc, float n, float inv, bool pow2)
    {
        // dividing by 2^m and multiplying by 2^-m round identically
        return pow2 ? acc * inv : __fdiv_rn(acc, n);
    }
    static __device__ __forceinline__ u32x4 mean(acc_t acc, float n, float inv, bool pow2)
    {
        f32x4 o;
        o.x = mean1(acc.x, n, inv, pow2);
        o.y = mean1(acc.y, n, inv, pow2);
        o.z = mean1(acc.z, n, inv, pow2);
        o.w = mean1(acc.w, n, inv, pow2);
        return __builtin_bit_cast(u32x4, o);
    }
    static __device__ __forceinline__ float widen1(float x) { return x; }
    static __device__ __forceinline__ float narrow1(float x) { return x; }
};

// bf16 elements stored as 16-bit patterns: eight per vector, arithmetic in
// fp32, one round-to-nearest-even back.
struct ops_bf16 {
    static constexpr int EPV = 8;
    static constexpr bool MIXED = false;
    static constexpr bool PAY16 = false;
    typedef uint16_t elem_t;
    struct acc_t {
        float v[8];
    };

    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    static __device__ __forceinline__ uint32_t rne(float f)
    {
        uint32_t u = __float_as_uint(f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    // two values at once with gfx950's own conversion (v_cvt_pk_bf16_f32: round to nearest
    // even, subnormals kept; the parity tests sweep the fp32 pattern space against rne())
    static __device__ __forceinline__ uint32_t pack(float a, float b)
    {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 v = {a, b};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }

    static __device__ __forceinline__ u32x4 ef(u32x4 g, u32x4 r, float c)
    {
        u32x4 a;
        a.x = pack(__builtin_fmaf(c, lo(r.x), lo(g.x)), __builtin_fmaf(c, hi(r.x), hi(g.x)));
        a.y = pack(__builtin_fmaf(c, lo(r.y), lo(g.y)), __builtin_fmaf(c, hi(r.y), hi(g.y)));
        a.z = pack(__builtin_fmaf(c, lo(r.z), lo(g.z)), __builtin_fmaf(c, hi(r.z), hi(g.z)));
        a.w = pack(__builtin_fmaf(c, lo(r.w), lo(g.w)), __builtin_fmaf(c, hi(r.w), hi(g.w)));
        return a;
    }
    static __device__ __forceinline__ uint16_t ef1(uint16_t g, uint16_t r, float c)
    {
        return (uint16_t)rne(__builtin_fmaf(c, lo(r), lo(g)));
    }
    static __device__ __forceinline__ acc_t widen(u32x4 v)
    {
        acc_t a;
        a.v[0] = lo(v.x); a.v[1] = hi(v.x); a.v[2] = lo(v.y); a.v[3] = hi(v.y);
        a.v[4] = lo(v.z); a.v[5] = hi(v.z); a.v[6] = lo(v.w); a.v[7] = hi(v.w);
        return a;
    }
    static __device__ __forceinline__ void add(acc_t &a, u32x4 v)
    {
        a.v[0] += lo(v.x); a.v[1] += hi(v.x); a.v[2] += lo(v.y); a.v[3] += hi(v.y);
        a.v[4] += lo(v.z); a.v[5] += hi(v.z); a.v[6] += lo(v.w); a.v[7] += hi(v.w);
    }
    static __device__ __forceinline__ float mean1(float acc, float n, float inv, bool pow2)
    {
        return pow2 ? acc * inv : __fdiv_rn(acc, n);
    }
    static __device__ __forceinline__ u32x4 mean(acc_t a, float n, float inv, bool pow2)
    {
        u32x4 o;
        o.x = pack(mean1(a.v[0], n, inv, pow2), mean1(a.v[1], n, inv, pow2));
        o.y = pack(mean1(a.v[2], n, inv, pow2), mean1(a.v[3], n, inv, pow2));
        o.z = pack(mean1(a.v[4], n, inv, pow2), mean1(a.v[5], n, inv, pow2));
        o.w = pack(mean1(a.v[6], n, inv, pow2), mean1(a.v[7], n, inv, pow2));
        return o;
    }
    static __device__ __forceinline__ float widen1(uint16_t x) { return lo(x); }
    static __device__ __forceinline__ uint16_t narrow1(float x) { return (uint16_t)rne(x); }
};

// bf16 gradients and payload with an fp32 residual.  Decompress is that of
// ops_bf16; compress has its own tile routine (compress_tile_mixed) because the
// residual stream is twice as wide as the other two.
struct ops_bf16_res32 : ops_bf16 {
    static constexpr bool MIXED = true;
};

// fp32 gradients, residual and dense output with an IEEE half-precision payload.
// Compress has its own tile routine (compress_tile_pay16: the payload stream is
// half as wide as the other two) and decompress its own kernel (k_decompress_pay16).
struct ops_f32_pay16 : ops_f32 {
    static constexpr bool PAY16 = true;
};

// ---- compress: error feedback + filter + pack + residual -----------------------

template <typename OPS, int kThreads, int UNROLL, bool NT>
__device__ __forceinline__ void compress_tile(const u32x4 *__restrict__ G, u32x4 *R,
                                              u32x4 *__restrict__ send, const tile_ref &t, float c)
{
    constexpr int EPV = OPS::EPV;
    constexpr int TILE = kThreads * EPV * UNROLL;
    const int tid = threadIdx.x;
    const u32x4 *gp = G + t.off / EPV;
    u32x4 *rp = R + t.off / EPV;
    u32x4 *sp = send + t.poff / EPV;
    const u32x4 zero = {0u, 0u, 0u, 0u};

    if (t.n == TILE) {
        u32x4 gv[UNROLL], rv[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) gv[u] = ld16<NT>(gp + u * kThreads + tid);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) rv[u] = ld16<NT>(rp + u * kThreads + tid);
        if (t.sel) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                st16<NT>(sp + u * kThreads + tid, OPS::ef(gv[u], rv[u], c));
                st16<NT>(rp + u * kThreads + tid, zero);
            }
        } else {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                st16<NT>(rp + u * kThreads + tid, OPS::ef(gv[u], rv[u], c));
        }
        return;
    }

    // ragged tile: whole vectors under a bound, then fewer than EPV scalars
    const int nv = t.n / EPV;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int v = u * kThreads + tid;
        if (v < nv) {
            const u32x4 a = OPS::ef(ld16<NT>(gp + v), ld16<NT>(rp + v), c);
            if (t.sel) {
                st16<NT>(sp + v, a);
                st16<NT>(rp + v, zero);
            } else {
                st16<NT>(rp + v, a);
            }
        }
    }
    const int rem = t.n - nv * EPV;
    if (tid < rem) {
        typedef typename OPS::elem_t E;
        const int64_t e = (int64_t)nv * EPV + tid;
        const E a = OPS::ef1(((const E *)gp)[e], ((const E *)rp)[e], c);
        if (t.sel) {
            ((E *)sp)[e] = a;
            ((E *)rp)[e] = (E)0;
        } else {
            ((E *)rp)[e] = a;
        }
    }
}

// Mixed precision tile: per step a thread owns four consecutive elements -- one
// 8-byte vector of bf16 gradients and one 16-byte vector of fp32 residuals -- so
// every load and store instruction of a wave still covers one contiguous run.
// A sent element leaves residual = A - bf16(A), the part rounding dropped
// (exact: both lie in the same or adjacent binade and share the low bits).
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int kThreads, int UNROLL, bool NT>
__device__ __forceinline__ void compress_tile_mixed(const uint16_t *__restrict__ G, float *R,
                                                    uint16_t *__restrict__ send,
                                                    const tile_ref &t, float c)
{
    constexpr int SLOTS = 2 * UNROLL;  // 4-element slots per thread; tile = kThreads * 8 * UNROLL
    const int tid = threadIdx.x;
    const u32x2 *gp = (const u32x2 *)(G + t.off);
    f32x4 *rp = (f32x4 *)(R + t.off);
    u32x2 *sp = (u32x2 *)(send + t.poff);
    const int nq = t.n / 4;
#pragma unroll
    for (int u = 0; u < SLOTS; ++u) {
        const int q = u * kThreads + tid;
        if (q < nq) {
            u32x2 g;
            f32x4 r;
            if constexpr (NT) {
                g = __builtin_nontemporal_load(gp + q);
                r = __builtin_nontemporal_load(rp + q);
            } else {
                g = gp[q];
                r = rp[q];
            }
            f32x4 a;
            a.x = __builtin_fmaf(c, r.x, ops_bf16::lo(g.x));
            a.y = __builtin_fmaf(c, r.y, ops_bf16::hi(g.x));
            a.z = __builtin_fmaf(c, r.z, ops_bf16::lo(g.y));
            a.w = __builtin_fmaf(c, r.w, ops_bf16::hi(g.y));
            if (t.sel) {
                u32x2 h;
                h.x = ops_bf16::pack(a.x, a.y);
                h.y = ops_bf16::pack(a.z, a.w);
                a.x -= ops_bf16::lo(h.x);
                a.y -= ops_bf16::hi(h.x);
                a.z -= ops_bf16::lo(h.y);
                a.w -= ops_bf16::hi(h.y);
                if constexpr (NT)
                    __builtin_nontemporal_store(h, sp + q);
                else
                    sp[q] = h;
            }
            if constexpr (NT)
                __builtin_nontemporal_store(a, rp + q);
            else
                rp[q] = a;
        }
    }
    const int rem = t.n - nq * 4;
    if (tid < rem) {
        const int64_t e = (int64_t)nq * 4 + tid;
        float a = __builtin_fmaf(c, R[t.off + e], ops_bf16::lo(G[t.off + e]));
        if (t.sel) {
            const uint16_t h = (uint16_t)ops_bf16::rne(a);
            send[t.poff + e] = h;
            a -= ops_bf16::lo(h);
        }
        R[t.off + e] = a;
    }
}

// Half-payload tile: per step a thread owns four consecutive elements -- 16-byte
// vectors of fp32 gradients and residuals, one 8-byte vector of halves -- so every
// load and store instruction of a wave covers one contiguous run.  A sent element
// leaves residual = A - fp16(A), what the quantiser dropped (Algorithm 1 line 4
// with the FP16 scheme of Table II as the compressor of line 3).
template <int kThreads, int UNROLL, bool NT>
__device__ __forceinline__ void compress_tile_pay16(const float *__restrict__ G, float *R,
                                                    uint16_t *__restrict__ send,
                                                    const tile_ref &t, float c)
{
    using covap_dev::half_hi;
    using covap_dev::half_lo;
    using covap_dev::pack_half2;
    using covap_dev::pinned;
    const int tid = threadIdx.x;
    const f32x4 *gp = (const f32x4 *)(G + t.off);
    f32x4 *rp = (f32x4 *)(R + t.off);
    u32x2 *sp = (u32x2 *)(send + t.poff);
    const int nq = t.n / 4;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int q = u * kThreads + tid;
        if (q < nq) {
            f32x4 g, r;
            if constexpr (NT) {
                g = __builtin_nontemporal_load(gp + q);
                r = __builtin_nontemporal_load(rp + q);
            } else {
                g = gp[q];
                r = rp[q];
            }
            f32x4 a;
            a.x = __builtin_fmaf(c, r.x, g.x);
            a.y = __builtin_fmaf(c, r.y, g.y);
            a.z = __builtin_fmaf(c, r.z, g.z);
            a.w = __builtin_fmaf(c, r.w, g.w);
            if (t.sel) {
                // the fp32 value must exist before it is narrowed (see pinned())
                a.x = pinned(a.x);
                a.y = pinned(a.y);
                a.z = pinned(a.z);
                a.w = pinned(a.w);
                u32x2 h;
                h.x = pack_half2(a.x, a.y);
                h.y = pack_half2(a.z, a.w);
                a.x -= half_lo(h.x);
                a.y -= half_hi(h.x);
                a.z -= half_lo(h.y);
                a.w -= half_hi(h.y);
                if constexpr (NT)
                    __builtin_nontemporal_store(h, sp + q);
                else
                    sp[q] = h;
            }
            if constexpr (NT)
                __builtin_nontemporal_store(a, rp + q);
            else
                rp[q] = a;
        }
    }
    const int rem = t.n - nq * 4;
    if (tid < rem) {
        const int64_t e = (int64_t)nq * 4 + tid;
        float a = pinned(__builtin_fmaf(c, R[t.off + e], G[t.off + e]));
        if (t.sel) {
            const __half h = __float2half_rn(a);
            send[t.poff + e] = __half_as_ushort(h);
            a -= __half2float(h);
        }
        R[t.off + e] = a;
    }
}

// PERSIST = false: one tile per workgroup, the grid holds exactly the tiles (the fastest
// shape when the kernel has the chip to itself).  PERSIST = true: a grid of a size the
// caller chose walks the n_tiles tiles with a grid stride; few resident waves leave the
// rest of every compute unit to a kernel of another stream (covap_compress_bounded).
template <typename OPS, typename GEOM, int kThreads, int UNROLL, bool NT, bool PERSIST>
__global__ __launch_bounds__(kThreads) void k_compress(const u32x4 *__restrict__ G, u32x4 *R,
                                                       u32x4 *__restrict__ send, GEOM g, float c,
                                                       uint32_t n_tiles)
{
    constexpr int TILE = kThreads * OPS::EPV * UNROLL;
    auto one = [&](uint32_t b) {
        tile_ref t;
        if (!covap::resolve_tile(g, b, (uint32_t)TILE, t)) return;
        if constexpr (OPS::MIXED)
            compress_tile_mixed<kThreads, UNROLL, NT>((const uint16_t *)G, (float *)R, (uint16_t *)send, t, c);
        else if constexpr (OPS::PAY16)
            compress_tile_pay16<kThreads, UNROLL, NT>((const float *)G, (float *)R, (uint16_t *)send, t, c);
        else
            compress_tile<OPS, kThreads, UNROLL, NT>(G, R, send, t, c);
    };
    if constexpr (PERSIST) {
        for (uint32_t b = blockIdx.x; b < n_tiles; b += gridDim.x) one(b);
    } else {
        one(blockIdx.x);
    }
}

// ---- take: aliased-residual form of compress ------------------------------------------
//
// When the caller's gradient-accumulation buffer doubles as the residual (the
// producer adds each new gradient into it, which is Algorithm 1 line 2 with
// c = 1), all that is left of compress is: move the sent shards to the payload
// and clear them.  Shards that are not sent are not touched at all, so the call
// moves 3 * P_t elements instead of 3 * D + P_t.  Pure byte movement: ESZ is the
// element size (4 or 2) and only matters for a shard's ragged tail.
template <typename GEOM, int ESZ, bool NT>
__global__ __launch_bounds__(64) void k_take(u32x4 *acc, u32x4 *__restrict__ send, GEOM g)
{
    constexpr int EPV = 16 / ESZ;
    constexpr int TILE = 64 * EPV;
    tile_ref t;
    if (!covap::resolve_tile(g, blockIdx.x, (uint32_t)TILE, t)) return;
    const int tid = threadIdx.x;
    u32x4 *ap = acc + t.off / EPV;
    u32x4 *sp = send + t.poff / EPV;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const int nv = t.n / EPV;
    if (tid < nv) {
        st16<NT>(sp + tid, ld16<NT>(ap + tid));
        st16<NT>(ap + tid, zero);
    }
    const int rem = t.n - nv * EPV;
    if (tid < rem) {
        const int64_t e = (int64_t)nv * EPV + tid;
        if constexpr (ESZ == 4) {
            ((uint32_t *)sp)[e] = ((const uint32_t *)ap)[e];
            ((uint32_t *)ap)[e] = 0u;
        } else {
            ((uint16_t *)sp)[e] = ((const uint16_t *)ap)[e];
            ((uint16_t *)ap)[e] = (uint16_t)0;
        }
    }
}

// ---- decompress: N-way mean + unpack + zero fill --------------------------------

// Sum of one packed vector position over the N payload rows, in row order.
// WU rows are loaded before the first of them is added, so WU 16-byte loads are
// in flight per thread; the additions keep the order w = 0, 1, ..., N-1.
template <typename OPS, int WU, bool NT>
__device__ __forceinline__ typename OPS::acc_t sum_rows(const u32x4 *p, int32_t N,
                                                        int64_t stride_vec)
{
    typename OPS::acc_t acc = OPS::widen(ld16<NT>(p));
    int32_t w = 1;
    for (; w + WU <= N; w += WU) {
        u32x4 x[WU];
#pragma unroll
        for (int j = 0; j < WU; ++j) x[j] = ld16<NT>(p + (int64_t)(w + j) * stride_vec);
#pragma unroll
        for (int j = 0; j < WU; ++j) OPS::add(acc, x[j]);
    }
    for (; w < N; ++w) OPS::add(acc, ld16<NT>(p + (int64_t)w * stride_vec));
    return acc;
}

template <typename OPS, int kThreads, int UNROLL, int WU, bool NT>
__device__ __forceinline__ void decompress_tile(const u32x4 *__restrict__ recv,
                                                u32x4 *__restrict__ out, const tile_ref &t,
                                                int32_t N, int64_t stride_elems, float n_f,
                                                float inv_n, int pow2)
{
    constexpr int EPV = OPS::EPV;
    constexpr int TILE = kThreads * EPV * UNROLL;
    typedef typename OPS::elem_t E;
    const int tid = threadIdx.x;
    u32x4 *op = out + t.off / EPV;
    const int nv = t.n / EPV;
    const int rem = t.n - nv * EPV;

    if (!t.sel) {  // nothing was sent for this shard: the dense result is +0
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int v = u * kThreads + tid;
            if (v < nv) st16<NT>(op + v, zero);
        }
        if (tid < rem) ((E *)op)[(int64_t)nv * EPV + tid] = (E)0;
        return;
    }

    const u32x4 *rp = recv + t.poff / EPV;
    const int64_t stride_vec = stride_elems / EPV;
    if (UNROLL > 1 && t.n == TILE) {
        // Full tile: walk the rows once for all UNROLL vector positions, so each
        // visit to a row reads UNROLL * kThreads * 16 contiguous bytes.
        typename OPS::acc_t acc[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc[u] = OPS::widen(ld16<NT>(rp + u * kThreads + tid));
        int32_t w = 1;
        for (; w + WU <= N; w += WU) {
            u32x4 x[WU][UNROLL];
#pragma unroll
            for (int j = 0; j < WU; ++j) {
                const u32x4 *row = rp + (int64_t)(w + j) * stride_vec + tid;
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) x[j][u] = ld16<NT>(row + u * kThreads);
            }
#pragma unroll
            for (int j = 0; j < WU; ++j)
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) OPS::add(acc[u], x[j][u]);
        }
        for (; w < N; ++w) {
            const u32x4 *row = rp + (int64_t)w * stride_vec + tid;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) OPS::add(acc[u], ld16<NT>(row + u * kThreads));
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            st16<NT>(op + u * kThreads + tid, OPS::mean(acc[u], n_f, inv_n, pow2 != 0));
        return;
    }
#pragma unroll 1
    for (int u = 0; u < UNROLL; ++u) {
        const int v = u * kThreads + tid;
        if (v < nv) {
            typename OPS::acc_t acc = sum_rows<OPS, WU, NT>(rp + v, N, stride_vec);
            st16<NT>(op + v, OPS::mean(acc, n_f, inv_n, pow2 != 0));
        }
    }
    if (tid < rem) {
        const int64_t e = (int64_t)nv * EPV + tid;
        const E *row = (const E *)rp + e;
        float acc = OPS::widen1(row[0]);
        for (int32_t w = 1; w < N; ++w) acc += OPS::widen1(row[(int64_t)w * stride_elems]);
        ((E *)op)[e] = OPS::narrow1(OPS::mean1(acc, n_f, inv_n, pow2 != 0));
    }
}

template <typename OPS, typename GEOM, int kThreads, int UNROLL, int WU, bool NT>
__global__ __launch_bounds__(kThreads) void k_decompress(const u32x4 *__restrict__ recv,
                                                         u32x4 *__restrict__ out, GEOM g,
                                                         int32_t N, int64_t stride_elems,
                                                         float n_f, float inv_n, int pow2)
{
    constexpr int TILE = kThreads * OPS::EPV * UNROLL;
    tile_ref t;
    if (!covap::resolve_tile(g, blockIdx.x, (uint32_t)TILE, t)) return;
    decompress_tile<OPS, kThreads, UNROLL, WU, NT>(recv, out, t, N, stride_elems, n_f, inv_n, pow2);
}

// Half payload into an fp32 dense result.  A tile is kThreads * 8 elements: a
// thread sums one 16-byte vector of eight halves over the N rows (fp32
// accumulators, row order) and writes two 16-byte vectors of means.
template <int kThreads, int WU, bool NT>
__device__ __forceinline__ void decompress_tile_pay16(const u32x4 *__restrict__ recv, float *__restrict__ out,
                                                      const tile_ref &t, int32_t N, int64_t stride_elems,
                                                      float n_f, float inv_n, int pow2)
{
    using covap_dev::half_hi;
    using covap_dev::half_lo;
    const int tid = threadIdx.x;
    float *o = out + t.off;
    if (!t.sel) {  // nothing was sent for this shard: the dense result is +0
        const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
        const int nv = t.n / 4;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int v = u * kThreads + tid;
            if (v < nv) {
                if constexpr (NT)
                    __builtin_nontemporal_store(zero, (f32x4 *)o + v);
                else
                    ((f32x4 *)o)[v] = zero;
            }
        }
        if (tid < t.n - nv * 4) o[nv * 4 + tid] = 0.0f;
        return;
    }
    const uint16_t *rp = (const uint16_t *)recv + t.poff;
    const int nv = t.n / 8;
    if (tid < nv) {
        const u32x4 *p = (const u32x4 *)rp + tid;
        const int64_t stride_vec = stride_elems / 8;
        float acc[8];
        {
            const u32x4 x = ld16<NT>(p);
            acc[0] = half_lo(x.x); acc[1] = half_hi(x.x); acc[2] = half_lo(x.y); acc[3] = half_hi(x.y);
            acc[4] = half_lo(x.z); acc[5] = half_hi(x.z); acc[6] = half_lo(x.w); acc[7] = half_hi(x.w);
        }
        auto add = [&](const u32x4 x) {
            acc[0] += half_lo(x.x); acc[1] += half_hi(x.x); acc[2] += half_lo(x.y); acc[3] += half_hi(x.y);
            acc[4] += half_lo(x.z); acc[5] += half_hi(x.z); acc[6] += half_lo(x.w); acc[7] += half_hi(x.w);
        };
        int32_t w = 1;
        for (; w + WU <= N; w += WU) {
            u32x4 x[WU];
#pragma unroll
            for (int j = 0; j < WU; ++j) x[j] = ld16<NT>(p + (int64_t)(w + j) * stride_vec);
#pragma unroll
            for (int j = 0; j < WU; ++j) add(x[j]);
        }
        for (; w < N; ++w) add(ld16<NT>(p + (int64_t)w * stride_vec));
        f32x4 lo4, hi4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lo4[j] = ops_f32::mean1(acc[j], n_f, inv_n, pow2 != 0);
            hi4[j] = ops_f32::mean1(acc[4 + j], n_f, inv_n, pow2 != 0);
        }
        if constexpr (NT) {
            __builtin_nontemporal_store(lo4, (f32x4 *)o + 2 * tid);
            __builtin_nontemporal_store(hi4, (f32x4 *)o + 2 * tid + 1);
        } else {
            ((f32x4 *)o)[2 * tid] = lo4;
            ((f32x4 *)o)[2 * tid + 1] = hi4;
        }
    }
    const int rem = t.n - nv * 8;
    if (tid < rem) {
        const int64_t e = (int64_t)nv * 8 + tid;
        const uint16_t *row = rp + e;
        float acc = __half2float(__ushort_as_half(row[0]));
        for (int32_t w = 1; w < N; ++w) acc += __half2float(__ushort_as_half(row[(int64_t)w * stride_elems]));
        o[e] = ops_f32::mean1(acc, n_f, inv_n, pow2 != 0);
    }
}

template <typename GEOM, int kThreads, int WU, bool NT>
__global__ __launch_bounds__(kThreads) void k_decompress_pay16(const u32x4 *__restrict__ recv,
                                                               float *__restrict__ out, GEOM g,
                                                               int32_t N, int64_t stride_elems,
                                                               float n_f, float inv_n, int pow2)
{
    tile_ref t;
    if (!covap::resolve_tile(g, blockIdx.x, (uint32_t)(kThreads * 8), t)) return;
    decompress_tile_pay16<kThreads, WU, NT>(recv, out, t, N, stride_elems, n_f, inv_n, pow2);
}

// The same with four elements per thread: an 8-byte load per row, one 16-byte store.
// For calls with few rows, which are bound by their stores: one store per thread from
// 256-thread workgroups is the shape that fills memory fastest (the loads are half as
// wide as they could be, which costs nothing when there are few of them).
template <typename GEOM, int kThreads, bool NT>
__global__ __launch_bounds__(kThreads) void k_decompress_pay16_narrow(const u32x2 *__restrict__ recv,
                                                                      float *__restrict__ out, GEOM g,
                                                                      int32_t N, int64_t stride_elems,
                                                                      float n_f, float inv_n, int pow2)
{
    using covap_dev::half_hi;
    using covap_dev::half_lo;
    tile_ref t;
    if (!covap::resolve_tile(g, blockIdx.x, (uint32_t)(kThreads * 4), t)) return;
    const int tid = threadIdx.x;
    float *o = out + t.off;
    const int nv = t.n / 4, rem = t.n - nv * 4;
    if (!t.sel) {  // nothing was sent for this shard: the dense result is +0
        const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
        if (tid < nv) {
            if constexpr (NT)
                __builtin_nontemporal_store(zero, (f32x4 *)o + tid);
            else
                ((f32x4 *)o)[tid] = zero;
        }
        if (tid < rem) o[nv * 4 + tid] = 0.0f;
        return;
    }
    const uint16_t *rp = (const uint16_t *)recv + t.poff;  // 16-byte aligned: 8-byte loads are aligned too
    if (tid < nv) {
        const u32x2 *p = (const u32x2 *)rp + tid;
        const int64_t stride_vec = stride_elems / 4;
        u32x2 x = NT ? __builtin_nontemporal_load(p) : *p;
        float acc[4] = {half_lo(x.x), half_hi(x.x), half_lo(x.y), half_hi(x.y)};
        for (int32_t w = 1; w < N; ++w) {
            const u32x2 *q = p + (int64_t)w * stride_vec;
            x = NT ? __builtin_nontemporal_load(q) : *q;
            acc[0] += half_lo(x.x); acc[1] += half_hi(x.x); acc[2] += half_lo(x.y); acc[3] += half_hi(x.y);
        }
        f32x4 m;
#pragma unroll
        for (int j = 0; j < 4; ++j) m[j] = ops_f32::mean1(acc[j], n_f, inv_n, pow2 != 0);
        if constexpr (NT)
            __builtin_nontemporal_store(m, (f32x4 *)o + tid);
        else
            ((f32x4 *)o)[tid] = m;
    }
    if (tid < rem) {
        const int64_t e = (int64_t)nv * 4 + tid;
        const uint16_t *row = rp + e;
        float acc = __half2float(__ushort_as_half(row[0]));
        for (int32_t w = 1; w < N; ++w) acc += __half2float(__ushort_as_half(row[(int64_t)w * stride_elems]));
        o[e] = ops_f32::mean1(acc, n_f, inv_n, pow2 != 0);
    }
}

// ---- probes ------------------------------------------------------------------------

// Both probes use the launch shape that the sweeps found best for the hot path:
// one-wave workgroups, one 16-byte vector per thread.
template <bool NT>
__global__ __launch_bounds__(kProbeThreads) void k_copy(u32x4 *__restrict__ dst,
                                                   const u32x4 *__restrict__ src, int64_t nvec)
{
    const int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    if (i < nvec) st16<NT>(dst + i, ld16<NT>(src + i));
}

template <bool NT>
__global__ __launch_bounds__(kProbeThreads) void k_triad(u32x4 *__restrict__ a,
                                                    const u32x4 *__restrict__ b,
                                                    const u32x4 *__restrict__ c, float s,
                                                    int64_t nvec)
{
    const int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    if (i < nvec) st16<NT>(a + i, ops_f32::ef(ld16<NT>(b + i), ld16<NT>(c + i), s));
}

// Matrix-core work on registers only: every wave issues 4 * iters MFMA instructions
// (32x32x8 bf16, four independent accumulators) and touches memory once, at the end.
// A stand-in for a purely compute-bound kernel of another stream: what the hot path
// costs next to it is contention for the compute units alone, not for the memory
// system.
typedef short bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void k_mfma_spin(float *__restrict__ out, int32_t iters)
{
    const int tid = threadIdx.x;
    const bf16x4_t a = {(short)(0x3f80 + (tid & 7)), (short)0x3f80, (short)0x3c00, (short)0x3f00};
    const bf16x4_t b = {(short)0x3f80, (short)(0x3c00 + (tid & 3)), (short)0x3f80, (short)0x3e00};
    f32x16_t acc0 = {}, acc1 = {}, acc2 = {}, acc3 = {};
    for (int32_t i = 0; i < iters; ++i) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(b, a, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, a, acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(b, b, acc3, 0, 0, 0);
    }
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) sum += (acc0[j] + acc1[j]) + (acc2[j] + acc3[j]);
    out[(int64_t)blockIdx.x * 256 + tid] = sum;
}

// ---- host-side launch helpers ----------------------------------------------------------

bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

bool overlap(const void *a, int64_t abytes, const void *b, int64_t bbytes)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + (uintptr_t)bbytes && b0 < a0 + (uintptr_t)abytes;
}

// Calls f(std::integral_constant<int, V>) for the V in Vs... that equals v.
template <int... Vs, typename F>
bool pick(int v, F &&f)
{
    return ((v == Vs ? (f(std::integral_constant<int, Vs>{}), true) : false) || ...);
}

// Runs f(geom, grid) once per launch the call needs: one launch for fixed-size
// shards, one per kMaxUnits list entries otherwise (the geometry is copied from the
// plan's tables; nothing is allocated).  sent_only: cover only the shards sent at
// this step.
template <typename F>
void for_each_launch(const covap_plan_s *plan, const covap::call_range &cr, int tile_elems,
                     bool sent_only, F &&f)
{
    if (plan->uniform) {
        uint32_t grid = 0;
        const fixed_geom g = covap::fixed_launch(plan, cr, (uint32_t)tile_elems, sent_only, &grid);
        if (grid) f(g, dim3(grid));
        return;
    }
    const int32_t n = covap::table_launches(plan, cr, sent_only);
    for (int32_t i = 0; i < n; ++i) {
        table_geom g;
        covap::table_launch(plan, cr, (uint32_t)tile_elems, sent_only, i, &g);
        const uint32_t grid = covap::grid_of(g);
        if (grid) f(g, dim3(grid));
    }
}

// max_groups = 0: one workgroup per tile; > 0: at most that many workgroups, persistent.
template <typename OPS>
bool launch_compress(const covap::tuning &tn, const covap_plan_s *plan, const covap::call_range &cr,
                     hipStream_t st, const void *G, void *R, void *send, float c, uint32_t max_groups,
                     covap::launch_status &ls)
{
    return pick<64, 256>(tn.compress_threads, [&](auto T) {
        pick<1, 2, 4>(tn.compress_unroll, [&](auto U) {
            pick<0, 1>(tn.nontemporal, [&](auto NT) {
                for_each_launch(plan, cr, T() * OPS::EPV * U(), false, [&](const auto &g, dim3 grid) {
                    typedef std::decay_t<decltype(g)> GEOM;
                    if (max_groups == 0u)
                        ls += covap::launch(k_compress<OPS, GEOM, T(), U(), NT() != 0, false>, grid, dim3(T()), 0,
                                            st, (const u32x4 *)G, (u32x4 *)R, (u32x4 *)send, g, c, grid.x);
                    else
                        ls += covap::launch(k_compress<OPS, GEOM, T(), U(), NT() != 0, true>,
                                            dim3(grid.x < max_groups ? grid.x : max_groups), dim3(T()), 0, st,
                                            (const u32x4 *)G, (u32x4 *)R, (u32x4 *)send, g, c, grid.x);
                });
            });
        });
    });
}

template <typename OPS>
bool launch_decompress(const covap::tuning &tn, const covap_plan_s *plan,
                       const covap::call_range &cr, hipStream_t st, const void *recv, void *out,
                       int32_t N, int32_t divisor, int64_t stride, covap::launch_status &ls)
{
    const int pow2 = (divisor & (divisor - 1)) == 0;
    const float n_f = (float)divisor, inv_n = 1.0f / n_f;
    return pick<64, 256>(tn.decompress_threads, [&](auto T) {
        pick<1, 2, 4>(tn.decompress_tile, [&](auto U) {
            pick<1, 2, 4>(tn.decompress_unroll, [&](auto WU) {
                pick<0, 1>(tn.nontemporal, [&](auto NT) {
                    for_each_launch(plan, cr, T() * OPS::EPV * U(), false, [&](const auto &g, dim3 grid) {
                        typedef std::decay_t<decltype(g)> GEOM;
                        // the LDS reservation is never touched: it only caps occupancy
                        ls += covap::launch(k_decompress<OPS, GEOM, T(), U(), WU(), NT() != 0>, grid, dim3(T()),
                                            (size_t)tn.decompress_lds_pad, st, (const u32x4 *)recv, (u32x4 *)out, g,
                                            N, stride, n_f, inv_n, pow2);
                    });
                });
            });
        });
    });
}

// Half-payload decompress: the tile knob does not apply (a tile is always one
// 16-byte payload vector per thread, or half of one in the store-bound form).
bool launch_decompress_pay16(const covap::tuning &tn, const covap_plan_s *plan,
                             const covap::call_range &cr, hipStream_t st, const void *recv, void *out,
                             int32_t N, int32_t divisor, int64_t stride, bool store_bound,
                             covap::launch_status &ls)
{
    const int pow2 = (divisor & (divisor - 1)) == 0;
    const float n_f = (float)divisor, inv_n = 1.0f / n_f;
    if (store_bound && plan->uniform && (N == 1 || stride % 4 == 0)) {
        return pick<0, 1>(tn.nontemporal, [&](auto NT) {
            for_each_launch(plan, cr, 256 * 4, false, [&](const auto &g, dim3 grid) {
                typedef std::decay_t<decltype(g)> GEOM;
                ls += covap::launch(k_decompress_pay16_narrow<GEOM, 256, NT() != 0>, grid, dim3(256), (size_t)0, st,
                                    (const u32x2 *)recv, (float *)out, g, N, stride, n_f, inv_n, pow2);
            });
        });
    }
    return pick<64, 256>(tn.decompress_threads, [&](auto T) {
        pick<1, 2, 4>(tn.decompress_unroll, [&](auto WU) {
            pick<0, 1>(tn.nontemporal, [&](auto NT) {
                for_each_launch(plan, cr, T() * 8, false, [&](const auto &g, dim3 grid) {
                    typedef std::decay_t<decltype(g)> GEOM;
                    ls += covap::launch(k_decompress_pay16<GEOM, T(), WU(), NT() != 0>, grid, dim3(T()),
                                        (size_t)tn.decompress_lds_pad, st, (const u32x4 *)recv, (float *)out, g, N,
                                        stride, n_f, inv_n, pow2);
                });
            });
        });
    });
}

// Element sizes in bytes of the four buffers of a plan's element type.
int64_t grad_esz(int32_t dtype) { return dtype == COVAP_F32 || dtype == COVAP_F32_PAY16 ? 4 : 2; }
int64_t residual_esz(int32_t dtype) { return dtype == COVAP_BF16 ? 2 : 4; }
int64_t payload_esz(int32_t dtype) { return dtype == COVAP_F32 ? 4 : 2; }

}  // namespace

using covap::fail;

namespace {

// covap_compress and covap_compress_bounded: argument checks and launches.
covap_status_t compress_call(const char *who, const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                    const void *grad, void *residual, void *send, int64_t send_cap_elems,
                                    float ef_coeff, uint32_t max_groups, void *stream)
{
    covap::clear_error();
    covap::call_range cr;
    const covap_status_t rs = covap::resolve(plan, step, bucket, &cr);
    if (rs != COVAP_OK) return rs;
    if (!grad || !residual || !send) return fail(COVAP_EINVAL, who, "null device pointer");
    if (!aligned16(grad) || !aligned16(residual) || !aligned16(send))
        return fail(COVAP_EINVAL, who, "device pointers must be 16-byte aligned");
    if (cr.packed_elems > 0 && send_cap_elems < cr.packed_base + cr.packed_elems)  // nothing sent: nothing written
        return fail(COVAP_EINVAL, who, "send buffer too small for this step");
    const int32_t dt = plan->opts.dtype;
    const int64_t abytes = plan->total_elems * grad_esz(dt), sbytes = send_cap_elems * payload_esz(dt);
    const int64_t rbytes = plan->total_elems * residual_esz(dt);
    if (overlap(grad, abytes, residual, rbytes) || overlap(grad, abytes, send, sbytes) ||
        overlap(residual, rbytes, send, sbytes))
        return fail(COVAP_EINVAL, who, "grad, residual and send must not overlap");
    if (cr.sh_hi == cr.sh_lo) return COVAP_OK;

    const covap::tuning tn = covap::tune();
    hipStream_t st = (hipStream_t)stream;
    covap::launch_status ls;
    bool ok;
    if (plan->opts.dtype == COVAP_F32)
        ok = launch_compress<ops_f32>(tn, plan, cr, st, grad, residual, send, ef_coeff, max_groups, ls);
    else if (plan->opts.dtype == COVAP_BF16)
        ok = launch_compress<ops_bf16>(tn, plan, cr, st, grad, residual, send, ef_coeff, max_groups, ls);
    else if (plan->opts.dtype == COVAP_BF16_RES32)
        ok = launch_compress<ops_bf16_res32>(tn, plan, cr, st, grad, residual, send, ef_coeff, max_groups, ls);
    else
        ok = launch_compress<ops_f32_pay16>(tn, plan, cr, st, grad, residual, send, ef_coeff, max_groups, ls);
    if (!ok) return fail(COVAP_EINVAL, who, "launch knobs select no kernel");
    return ls.report(who);
}


}  // namespace

extern "C" {

covap_status_t covap_compress(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                              const void *grad, void *residual, void *send,
                              int64_t send_cap_elems, float ef_coeff, void *stream)
{
    return compress_call("covap_compress", plan, step, bucket, grad, residual, send, send_cap_elems, ef_coeff, 0u,
                         stream);
}

covap_status_t covap_compress_bounded(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                      const void *grad, void *residual, void *send,
                                      int64_t send_cap_elems, float ef_coeff, int32_t max_workgroups,
                                      void *stream)
{
    if (max_workgroups < 1) {
        covap::clear_error();
        return fail(COVAP_EINVAL, "covap_compress_bounded", "max_workgroups < 1");
    }
    return compress_call("covap_compress_bounded", plan, step, bucket, grad, residual, send, send_cap_elems,
                         ef_coeff, (uint32_t)max_workgroups, stream);
}

covap_status_t covap_compress_aliased(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                      void *accum, void *send, int64_t send_cap_elems,
                                      void *stream)
{
    covap::clear_error();
    covap::call_range cr;
    const covap_status_t rs = covap::resolve(plan, step, bucket, &cr);
    if (rs != COVAP_OK) return rs;
    if (plan->opts.dtype == COVAP_BF16_RES32 || plan->opts.dtype == COVAP_F32_PAY16)
        return fail(COVAP_EUNSUPPORTED,
                    "covap_compress_aliased: gradient, residual and payload must share one element type");
    if (!accum || !send) return fail(COVAP_EINVAL, "covap_compress_aliased: null device pointer");
    if (!aligned16(accum) || !aligned16(send))
        return fail(COVAP_EINVAL, "covap_compress_aliased: device pointers must be 16-byte aligned");
    if (cr.packed_elems > 0 && send_cap_elems < cr.packed_base + cr.packed_elems)  // nothing sent: nothing written
        return fail(COVAP_EINVAL, "covap_compress_aliased: send buffer too small for this step");
    const int64_t esz = plan->opts.dtype == COVAP_F32 ? 4 : 2;
    if (overlap(accum, plan->total_elems * esz, send, send_cap_elems * esz))
        return fail(COVAP_EINVAL, "covap_compress_aliased: accum and send must not overlap");
    if (cr.sh_hi == cr.sh_lo) return COVAP_OK;
    hipStream_t st = (hipStream_t)stream;
    const bool nt = covap::tune().nontemporal != 0;
    covap::launch_status ls;
    for_each_launch(plan, cr, 64 * plan->elems_per_vec, true, [&](const auto &g, dim3 grid) {
        typedef std::decay_t<decltype(g)> GEOM;
        void (*kernel)(u32x4 *, u32x4 *, GEOM) =
            esz == 4 ? (nt ? k_take<GEOM, 4, true> : k_take<GEOM, 4, false>)
                     : (nt ? k_take<GEOM, 2, true> : k_take<GEOM, 2, false>);
        ls += covap::launch(kernel, grid, dim3(64), 0, st, (u32x4 *)accum, (u32x4 *)send, g);
    });
    return ls.report("covap_compress_aliased");
}

// Shared body of covap_decompress and covap_decompress_reduced: `rows` payload
// rows are added in row order and the sum is divided by `divisor`.
static covap_status_t decompress_call(const char *who, const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                      const void *recv, int32_t rows, int32_t divisor, int64_t stride_elems,
                                      void *dense_out, void *stream)
{
    covap::clear_error();
    covap::call_range cr;
    const covap_status_t rs = covap::resolve(plan, step, bucket, &cr);
    if (rs != COVAP_OK) return rs;
    if (!recv || !dense_out) return fail(COVAP_EINVAL, who, "null device pointer");
    if (!aligned16(recv) || !aligned16(dense_out))
        return fail(COVAP_EINVAL, who, "device pointers must be 16-byte aligned");
    if (rows < 1 || divisor < 1) return fail(COVAP_EINVAL, who, "n_workers < 1");
    if (rows == 1 && stride_elems < 0) stride_elems = cr.packed_base + cr.packed_elems;   // one row: its own length
    if (cr.packed_elems > 0 && stride_elems < cr.packed_base + cr.packed_elems)
        return fail(COVAP_EINVAL, who, "row stride smaller than the packed payload");
    if (rows > 1 && stride_elems % plan->elems_per_vec != 0)
        return fail(COVAP_EINVAL, who, "row stride must be a multiple of 16 bytes");
    const int32_t dt = plan->opts.dtype;
    if (overlap(recv, (int64_t)rows * stride_elems * payload_esz(dt), dense_out, plan->total_elems * grad_esz(dt)))
        return fail(COVAP_EINVAL, who, "the payload and dense_out must not overlap");
    if (cr.sh_hi == cr.sh_lo) return COVAP_OK;

    covap::tuning tn = covap::tune();
    // Few rows: the call writes more than it reads and is bound by its stores (measured
    // crossover: rows x packed elements = dense elements).  How fast memory fills depends on
    // how many stores the chip keeps in flight, with an optimum near 32 KB per compute unit:
    // fixed-size shards reach it with one 16-byte store per thread from 256-thread workgroups
    // at full occupancy; variable-length shards, where a wave spends part of its life
    // resolving its tile, with two stores per thread and an LDS reservation that holds a
    // compute unit to five such workgroups.  The one-wave shape that suits many rows is 40 %
    // slower here.
    const covap_shard_rec &first = plan->shards[cr.sh_lo], &last = plan->shards[cr.sh_hi - 1];
    const bool store_bound =
        tn.decompress_shape_unset && (int64_t)rows * cr.packed_elems < last.off + last.len - first.off;
    if (store_bound) {
        tn.decompress_threads = 256;
        tn.decompress_tile = plan->uniform ? 1 : 2;
        tn.decompress_lds_pad = plan->uniform ? 0 : 32768;
    }
    hipStream_t st = (hipStream_t)stream;
    covap::launch_status ls;
    bool ok;
    if (dt == COVAP_F32)
        ok = launch_decompress<ops_f32>(tn, plan, cr, st, recv, dense_out, rows, divisor, stride_elems, ls);
    else if (dt == COVAP_F32_PAY16)
        ok = launch_decompress_pay16(tn, plan, cr, st, recv, dense_out, rows, divisor, stride_elems, store_bound, ls);
    else
        ok = launch_decompress<ops_bf16>(tn, plan, cr, st, recv, dense_out, rows, divisor, stride_elems, ls);
    if (!ok) return fail(COVAP_EINVAL, who, "launch knobs select no kernel");
    return ls.report(who);
}

covap_status_t covap_decompress(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                const void *recv, int32_t n_workers, int64_t stride_elems,
                                void *dense_out, void *stream)
{
    if (stride_elems < 0) {
        covap::clear_error();
        return fail(COVAP_EINVAL, "covap_decompress", "row stride smaller than the packed payload");
    }
    return decompress_call("covap_decompress", plan, step, bucket, recv, n_workers, n_workers, stride_elems,
                           dense_out, stream);
}

covap_status_t covap_decompress_reduced(const covap_plan_t *plan, uint64_t step, int32_t bucket,
                                        const void *summed, int32_t n_workers, void *dense_out, void *stream)
{
    return decompress_call("covap_decompress_reduced", plan, step, bucket, summed, 1, n_workers, -1, dense_out,
                           stream);
}

covap_status_t covap_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    covap::clear_error();
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0)
        return fail(COVAP_EINVAL, "covap_probe_copy: pointers and size must be 16-byte multiples");
    if (bytes == 0) return COVAP_OK;
    const int64_t nvec = (int64_t)(bytes / 16);
    const int64_t per = kProbeThreads;
    const uint32_t grid = (uint32_t)((nvec + per - 1) / per);
    covap::launch_status ls;
    ls += covap::launch(covap::tune().nontemporal ? k_copy<true> : k_copy<false>, dim3(grid), dim3(kProbeThreads), 0,
                        (hipStream_t)stream, (u32x4 *)dst, (const u32x4 *)src, nvec);
    return ls.report("covap_probe_copy");
}

covap_status_t covap_probe_triad(float *a, const float *b, const float *c, float s, int64_t n,
                                 void *stream)
{
    covap::clear_error();
    if (!a || !b || !c || !aligned16(a) || !aligned16(b) || !aligned16(c) || n < 0 || n % 4 != 0)
        return fail(COVAP_EINVAL, "covap_probe_triad: pointers 16-byte aligned, n a multiple of 4");
    if (n == 0) return COVAP_OK;
    const int64_t nvec = n / 4;
    const int64_t per = kProbeThreads;
    const uint32_t grid = (uint32_t)((nvec + per - 1) / per);
    covap::launch_status ls;
    ls += covap::launch(covap::tune().nontemporal ? k_triad<true> : k_triad<false>, dim3(grid), dim3(kProbeThreads),
                        0, (hipStream_t)stream, (u32x4 *)a, (const u32x4 *)b, (const u32x4 *)c, s, nvec);
    return ls.report("covap_probe_triad");
}

covap_status_t covap_probe_mfma(float *out, int32_t workgroups, int32_t iters, int32_t lds_bytes, void *stream)
{
    covap::clear_error();
    if (!out || workgroups < 1 || workgroups > (1 << 20) || iters < 0 || lds_bytes < 0 || lds_bytes > 160 * 1024)
        return fail(COVAP_EINVAL, "covap_probe_mfma",
                    "need out, 1 <= workgroups <= 2^20, iters >= 0, 0 <= lds_bytes <= 160 KiB");
    covap::launch_status ls;
    ls += covap::launch(k_mfma_spin, dim3((uint32_t)workgroups), dim3(256), (size_t)lds_bytes, (hipStream_t)stream, out,
                        iters);
    return ls.report("covap_probe_mfma");
}

}  // extern "C"
