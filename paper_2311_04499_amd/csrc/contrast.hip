// Further contrast points on the same buffers as the COVAP path: the two
// schemes the paper singles out as free of data dependencies (Sec. II-C,
// Table III) -- Random-k and FP16 -- each with the error feedback of Algorithm 1,
// and the matching decompress sides (N-way mean of sparse / half payloads).
// Like top-k they are here to be measured against, not to be the product:
// plain streaming kernels with 16-byte accesses and streaming cache hints.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

#include "half_util.h"
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
        ((f32x4 *)R)[v] = a;  // the gather that follows reads a few of these again
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

covap_status_t check(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return covap::fail(COVAP_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    return COVAP_OK;
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
    k_ef_accumulate<<<blocks(n / 4 > 0 ? n / 4 : 1, kThreads), kThreads, 0, st>>>(
        (const float *)grad, (float *)residual, n, ef_coeff);
    if (k > 0)
        k_gather_clear<<<blocks(k, 256), 256, 0, st>>>((float *)residual, idx, k, (float *)out_vals);
    return check("randk_compress");
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
    k_fp16_compress<<<blocks(n / 4 > 0 ? n / 4 : 1, kThreads), kThreads, 0, (hipStream_t)stream>>>(
        (const float *)grad, (float *)residual, n, ef_coeff, (uint16_t *)out_half);
    return check("fp16_compress");
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
    k_fp16_decompress<<<blocks(n / 8 > 0 ? n / 8 : 1, kThreads), kThreads, 0, (hipStream_t)stream>>>(
        (const uint16_t *)recv, n_workers, stride_elems, n, (float *)dense_out, n_f, 1.0f / n_f, pow2);
    return check("fp16_decompress");
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
    k_zero<<<dense_grid, kThreads, 0, st>>>(out, n);
    if (k > 0) {
        for (int32_t w = 0; w < n_workers; ++w)
            k_scatter_add<<<blocks(k, 256), 256, 0, st>>>(out, idx + (int64_t)w * stride_elems,
                                                          (const float *)vals + (int64_t)w * stride_elems, k);
        if (n_workers > 1) {
            const int pow2 = (n_workers & (n_workers - 1)) == 0;
            const float n_f = (float)n_workers;
            k_scale<<<dense_grid, kThreads, 0, st>>>(out, n, n_f, 1.0f / n_f, pow2);
        }
    }
    return check("sparse_decompress");
}

}  // extern "C"
