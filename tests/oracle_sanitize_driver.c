/* Walks every routine of the CPU oracle on small ragged inputs held in heap buffers of
 * exactly the size each call may touch, so that AddressSanitizer sees any access past
 * an end and UBSan any undefined arithmetic.  Built together with oracle/covap_oracle.c
 * and run by tests/test_oracle_sanitize.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t orc_plan_offsets(const int64_t *, int32_t, int64_t *);
int64_t orc_plan_fixed_shards(int64_t, int64_t, int64_t *, int64_t *);
int32_t orc_plan_buckets(const int64_t *, int64_t, int64_t, int32_t *);
int32_t orc_plan_group_layers(const int64_t *, int32_t, int64_t, int32_t *);
int64_t orc_plan_median_parts(const int64_t *, int32_t, int64_t, int32_t, int32_t *);
int32_t orc_plan_even_slices(int64_t, int32_t, int64_t, int64_t *);
int64_t orc_plan_median_layout(const int64_t *, int32_t, int64_t, int32_t, int64_t, int64_t, int64_t *, int64_t *,
                               int64_t *, int32_t *, int64_t *);
int32_t orc_selected(int64_t, uint64_t, int32_t);
int64_t orc_packed_end(const int64_t *, int64_t, int32_t, uint64_t, int64_t);
uint16_t orc_f32_to_bf16(float);
float orc_bf16_to_f32(uint16_t);
uint16_t orc_f32_to_f16(float);
float orc_f16_to_f32(uint16_t);
int64_t orc_compress_f32(const float *, float *, float *, const int64_t *, const int64_t *, int64_t, int64_t, int32_t,
                         uint64_t, float, int64_t);
int64_t orc_compress_bf16(const uint16_t *, uint16_t *, uint16_t *, const int64_t *, const int64_t *, int64_t,
                          int64_t, int32_t, uint64_t, float, int64_t);
int64_t orc_compress_bf16_res32(const uint16_t *, float *, uint16_t *, const int64_t *, const int64_t *, int64_t,
                                int64_t, int32_t, uint64_t, float, int64_t);
int64_t orc_compress_f32_pay16(const float *, float *, uint16_t *, const int64_t *, const int64_t *, int64_t, int64_t,
                               int32_t, uint64_t, float, int64_t);
int64_t orc_compress_aliased(void *, void *, int32_t, const int64_t *, const int64_t *, int64_t, int64_t, int32_t,
                             uint64_t, int64_t);
void orc_decompress_f32(const float *, int32_t, int64_t, float *, const int64_t *, const int64_t *, int64_t, int64_t,
                        int32_t, uint64_t, int64_t);
void orc_decompress_bf16(const uint16_t *, int32_t, int64_t, uint16_t *, const int64_t *, const int64_t *, int64_t,
                         int64_t, int32_t, uint64_t, int64_t);
void orc_decompress_pay16(const uint16_t *, int32_t, int64_t, float *, const int64_t *, const int64_t *, int64_t,
                          int64_t, int32_t, uint64_t, int64_t);
void orc_unpack_mean_f32(const float *, int32_t, float *, const int64_t *, const int64_t *, int64_t, int64_t, int32_t,
                         uint64_t, int64_t);
void orc_unpack_mean_bf16(const uint16_t *, int32_t, uint16_t *, const int64_t *, const int64_t *, int64_t, int64_t,
                          int32_t, uint64_t, int64_t);
void orc_unpack_mean_pay16(const uint16_t *, int32_t, float *, const int64_t *, const int64_t *, int64_t, int64_t,
                           int32_t, uint64_t, int64_t);
int32_t orc_topk_f32(const float *, float *, int64_t, int64_t, float, float *, uint32_t *);
int32_t orc_randk_f32(const float *, float *, int64_t, const uint32_t *, int64_t, float, float *);
void orc_fp16_compress(const float *, float *, int64_t, float, uint16_t *);
void orc_fp16_mean(const uint16_t *, int32_t, int64_t, int64_t, float *);
void orc_sparse_mean(const float *, const uint32_t *, int32_t, int64_t, int64_t, int64_t, float *);
int32_t orc_ratio_from_ccr(double, int32_t *);
float orc_ef_coeff(float, uint64_t, uint64_t, float);

#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            fprintf(stderr, "CHECK failed: %s (line %d)\n", #c, __LINE__);        \
            return 1;                                                             \
        }                                                                         \
    } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
static float rndf(void) { return ((float)(rnd() % 2001) - 1000.0f) / 512.0f; }

/* One plan (shard table), every element type, every step of two periods, whole arena and
 * bucket by bucket. */
static int hot_path(const int64_t *off, const int64_t *len, const int32_t *bucket, int64_t n_sh, int64_t D,
                    int32_t I, int64_t align)
{
    const int32_t N = 3;
    int64_t pmax = 0;
    for (uint64_t t = 0; t < (uint64_t)I; ++t) {
        int64_t p = orc_packed_end(len, n_sh, I, t, align);
        if (p > pmax) pmax = p;
    }
    const int64_t stride = pmax; /* rows exactly as long as the longest payload */
    float *G = malloc(sizeof(float) * (size_t)(D ? D : 1)), *R = calloc((size_t)(D ? D : 1), sizeof(float));
    float *Rm = calloc((size_t)(D ? D : 1), sizeof(float)), *Rh = calloc((size_t)(D ? D : 1), sizeof(float));
    float *out = malloc(sizeof(float) * (size_t)(D ? D : 1));
    uint16_t *Gb = malloc(2 * (size_t)(D ? D : 1)), *Rb = calloc((size_t)(D ? D : 1), 2), *outb = malloc(2 * (size_t)(D ? D : 1));
    float *recv = malloc(sizeof(float) * (size_t)(N * stride ? N * stride : 1));
    uint16_t *recvb = malloc(2 * (size_t)(N * stride ? N * stride : 1));
    uint32_t *acc = malloc(4 * (size_t)(D ? D : 1)), *accs = malloc(4 * (size_t)(stride ? stride : 1));
    const int32_t n_buckets = n_sh ? bucket[n_sh - 1] + 1 : 0;
    for (uint64_t t = 0; t < (uint64_t)(2 * I + 1); ++t) {
        for (int64_t i = 0; i < D; ++i) {
            G[i] = rndf();
            Gb[i] = orc_f32_to_bf16(G[i]);
            acc[i] = (uint32_t)i + 1u;
        }
        for (int64_t i = 0; i < N * stride; ++i) {
            recv[i] = rndf();
            recvb[i] = orc_f32_to_bf16(recv[i]);
        }
        const int64_t P = orc_packed_end(len, n_sh, I, t, align);
        CHECK(P <= stride);
        int64_t sent = 0;
        for (int64_t s = 0; s < n_sh; ++s) sent += orc_selected(s, t, I) ? len[s] : 0;
        if (t % 2 == 0) { /* whole arena */
            CHECK(orc_compress_f32(G, R, recv, off, len, 0, n_sh, I, t, 0.5f, align) == sent);
            CHECK(orc_compress_bf16(Gb, Rb, recvb, off, len, 0, n_sh, I, t, 0.5f, align) == sent);
            CHECK(orc_compress_bf16_res32(Gb, Rm, recvb, off, len, 0, n_sh, I, t, 1.0f, align) == sent);
            CHECK(orc_compress_f32_pay16(G, Rh, recvb, off, len, 0, n_sh, I, t, 1.0f, align) == sent);
            CHECK(orc_compress_aliased(acc, accs, 4, off, len, 0, n_sh, I, t, align) == sent);
            orc_decompress_f32(recv, N, stride, out, off, len, 0, n_sh, I, t, align);
            orc_decompress_bf16(recvb, N, stride, outb, off, len, 0, n_sh, I, t, align);
            orc_decompress_pay16(recvb, N, stride, out, off, len, 0, n_sh, I, t, align);
            /* one summed row: the first row of the receive buffers stands in for it */
            orc_unpack_mean_f32(recv, N, out, off, len, 0, n_sh, I, t, align);
            orc_unpack_mean_bf16(recvb, N, outb, off, len, 0, n_sh, I, t, align);
            orc_unpack_mean_pay16(recvb, N, out, off, len, 0, n_sh, I, t, align);
        } else { /* bucket by bucket */
            int64_t total = 0, lo = 0;
            for (int32_t b = 0; b < n_buckets; ++b) {
                int64_t hi = lo;
                while (hi < n_sh && bucket[hi] == b) ++hi;
                total += orc_compress_f32(G, R, recv, off, len, lo, hi, I, t, 1.0f, align);
                orc_compress_bf16(Gb, Rb, recvb, off, len, lo, hi, I, t, 1.0f, align);
                orc_compress_aliased(acc, accs, 4, off, len, lo, hi, I, t, align);
                orc_decompress_f32(recv, N, stride, out, off, len, lo, hi, I, t, align);
                orc_decompress_bf16(recvb, N, stride, outb, off, len, lo, hi, I, t, align);
                orc_unpack_mean_f32(recv, N, out, off, len, lo, hi, I, t, align);
                orc_unpack_mean_bf16(recvb, N, outb, off, len, lo, hi, I, t, align);
                orc_unpack_mean_pay16(recvb, N, out, off, len, lo, hi, I, t, align);
                lo = hi;
            }
            CHECK(lo == n_sh && total == sent);
        }
    }
    free(G); free(R); free(Rm); free(Rh); free(out); free(Gb); free(Rb); free(outb); free(recv); free(recvb);
    free(acc); free(accs);
    return 0;
}

int main(void)
{
    /* planner: fixed shards over ragged arenas */
    const int64_t sizes[][8] = {{1003, 2001, 30007, 5, 4099, 17, 9001, 3}, {1, 0, 0, 0, 0, 0, 0, 0}, {0, 7, 0, 64, 0, 0, 0, 1}};
    for (int c = 0; c < 3; ++c) {
        int64_t offs[8];
        const int64_t D = orc_plan_offsets(sizes[c], 8, offs);
        for (int64_t S = 4; S <= 4096; S *= 8) {
            const int64_t n_sh = orc_plan_fixed_shards(D, S, NULL, NULL);
            int64_t *off = malloc(8 * (size_t)(n_sh ? n_sh : 1)), *len = malloc(8 * (size_t)(n_sh ? n_sh : 1));
            int32_t *bucket = malloc(4 * (size_t)(n_sh ? n_sh : 1));
            CHECK(orc_plan_fixed_shards(D, S, off, len) == n_sh);
            orc_plan_buckets(len, n_sh, 3 * S + 1, bucket);
            for (int32_t I = 1; I <= 7; I += 3)
                if (S >= 64 || D < 2000) CHECK(hot_path(off, len, bucket, n_sh, D, I, 1) == 0);
            free(off); free(len); free(bucket);
        }
        /* the paper's sharding on the same layers */
        for (int64_t cap = 1; cap <= 40000; cap *= 200) {
            for (int32_t I = 1; I <= 9; I += 4) {
                for (int64_t align = 4; align <= 256; align *= 64) {
                    int64_t toff[8], arena = 0;
                    const int64_t n_sh = orc_plan_median_layout(sizes[c], 8, cap, I, 0, align, toff, NULL, NULL, NULL, &arena);
                    int64_t *off = malloc(8 * (size_t)(n_sh ? n_sh : 1)), *len = malloc(8 * (size_t)(n_sh ? n_sh : 1));
                    int32_t *bucket = malloc(4 * (size_t)(n_sh ? n_sh : 1));
                    CHECK(orc_plan_median_layout(sizes[c], 8, cap, I, 0, align, toff, off, len, bucket, &arena) == n_sh);
                    int64_t covered = 0;
                    for (int64_t s = 0; s < n_sh; ++s) covered += len[s];
                    CHECK(covered == D && arena >= D);
                    CHECK(hot_path(off, len, bucket, n_sh, arena, I, align) == 0);
                    free(off); free(len); free(bucket);
                }
            }
        }
    }
    int32_t group_of[8], parts[8];
    int64_t piece[19];
    CHECK(orc_plan_group_layers(sizes[0], 8, 5000, group_of) >= 1);
    const int64_t vgg[6] = {4101096, 16781312, 107480576, 7079424, 7669760, 555072};
    CHECK(orc_plan_median_parts(vgg, 6, 5590260, 1000, parts) == 26);
    CHECK(orc_plan_median_parts(vgg, 6, 0, 2, parts) > 0 && orc_plan_median_parts(vgg, 0, 0, 2, parts) == 0);
    CHECK(orc_plan_even_slices(107480576, 19, 4, piece) == 19 && orc_plan_even_slices(10, 4, 4, piece) == 3);
    CHECK(orc_selected(0, 0, 4) == 1 && orc_selected(3, 0xffffffffffffffffull, 4) == (int32_t)((3 + 3) % 4 == 0));

    /* conversions over a sweep of bit patterns, incl. NaN, Inf, subnormals, both signs */
    for (uint32_t hi = 0; hi < 65536; hi += 7) {
        uint32_t u = (hi << 16) | (hi * 2654435761u >> 16);
        float f;
        memcpy(&f, &u, 4);
        (void)orc_f32_to_bf16(f);
        (void)orc_f32_to_f16(f);
        (void)orc_bf16_to_f32((uint16_t)hi);
        (void)orc_f16_to_f32((uint16_t)hi);
    }

    /* contrast routines */
    for (int64_t n = 0; n <= 1500; n = n * 3 + 1) {
        float *G = malloc(4 * (size_t)(n ? n : 1)), *R = malloc(4 * (size_t)(n ? n : 1));
        for (int64_t i = 0; i < n; ++i) {
            G[i] = (float)(rnd() % 7) - 3.0f; /* many ties */
            R[i] = rndf();
        }
        for (int64_t k = 0; k <= n; k = k * 2 + 1) {
            float *vals = malloc(4 * (size_t)(k ? k : 1));
            uint32_t *idx = malloc(4 * (size_t)(k ? k : 1));
            CHECK(orc_topk_f32(G, R, n, k, 0.5f, vals, idx) == 0);
            for (int64_t j = 0; j < k; ++j) idx[j] = (uint32_t)(n - 1 - j); /* distinct */
            CHECK(orc_randk_f32(G, R, n, idx, k, 1.0f, vals) == 0);
            free(vals); free(idx);
        }
        CHECK(orc_topk_f32(G, R, n, n + 1, 1.0f, NULL, NULL) == -1);
        uint16_t *h = malloc(2 * (size_t)(3 * n ? 3 * n : 1));
        float *m = malloc(4 * (size_t)(n ? n : 1));
        orc_fp16_compress(G, R, n, 0.25f, h);
        for (int64_t i = n; i < 3 * n; ++i) h[i] = h[i - n];
        orc_fp16_mean(h, 3, n, n, m);
        const int64_t k = n / 3;
        float *sv = malloc(4 * (size_t)(2 * k ? 2 * k : 1));
        uint32_t *si = malloc(4 * (size_t)(2 * k ? 2 * k : 1));
        for (int64_t j = 0; j < 2 * k; ++j) {
            sv[j] = rndf();
            si[j] = (uint32_t)((j % k) * 3 + (j >= k ? 1 : 0));
        }
        orc_sparse_mean(sv, si, 2, k, k, n, m);
        free(G); free(R); free(h); free(m); free(sv); free(si);
    }

    int32_t I = 0;
    CHECK(orc_ratio_from_ccr(3.1, &I) == 0 && I == 4 && orc_ratio_from_ccr(0.0, &I) == -1);
    CHECK(orc_ratio_from_ccr(NAN, &I) == -1 && orc_ratio_from_ccr(1e300, &I) == -1);
    CHECK(orc_ef_coeff(0.1f, 250, 100, 0.1f) > 0.29f && orc_ef_coeff(0.1f, 1u << 30, 1, 0.1f) == 1.0f);
    puts("oracle sanitize driver: ok");
    return 0;
}
