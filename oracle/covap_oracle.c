/*
 * covap_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded CPU statement of what the COVAP per-iteration
 * gradient-compression path computes, written from the paper
 * (arXiv 2311.04499).  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP library: it
 * has its own planner, its own filter, its own bf16 and fp16 conversions.
 *
 * Every function walks the data in the order the paper states the operation:
 * shard by shard, element by element, worker by worker.  No blocking, fusion
 * or reordering.  Compile with -ffp-contract=off so that the only fused
 * multiply-add is the one written as fmaf().
 *
 * Index conventions (the paper leaves the base open): shards ("tensors" after
 * sharding, Sec. III-C) and iterations (num_steps, Sec. III-A) are 0-based.
 *
 * Pins: tests/test_oracle_*.py check every function below against brute force,
 * closed forms and the figures the paper prints.  No function here is
 * "parity unpinned" except orc_plan_buckets (the paper gives no bucket rule;
 * buckets only partition launches and never change a result).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Planner                                                             */
/* ------------------------------------------------------------------ */

/* Flat arena: gradients of consecutive layers are laid end to end in one
 * communication buffer (Sec. II-B, Sec. III-A).  offsets[i] = sum of numel
 * before tensor i.  Returns the total D. */
int64_t orc_plan_offsets(const int64_t *numel, int32_t n, int64_t *offsets)
{
    int64_t d = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (offsets) offsets[i] = d;
        d += numel[i];
    }
    return d;
}

/* Fixed-size sharding of the arena: shard s covers [s*S, min((s+1)*S, D)).
 * After sharding every shard counts as one "tensor" for the filter
 * (Sec. III-C, last paragraph).  Returns the number of shards; fills off/len
 * when they are not NULL. */
int64_t orc_plan_fixed_shards(int64_t D, int64_t S, int64_t *off, int64_t *len)
{
    int64_t n = 0;
    for (int64_t b = 0; b < D; b += S) {
        int64_t l = D - b;
        if (l > S) l = S;
        if (off) off[n] = b;
        if (len) len[n] = l;
        ++n;
    }
    return n;
}

/* Buckets: consecutive shards are grouped greedily; a bucket is closed when
 * the next shard would push it over cap_elems (a shard larger than the cap is
 * a bucket by itself).  The paper only says communication tensors are about
 * 25 MB (Sec. III-A); this rule is this build's reading.  Returns the number
 * of buckets and writes the bucket id of each shard. */
int32_t orc_plan_buckets(const int64_t *len, int64_t n_sh, int64_t cap_elems,
                         int32_t *bucket_of)
{
    int32_t b = 0;
    int64_t fill = 0;
    for (int64_t s = 0; s < n_sh; ++s) {
        if (fill > 0 && fill + len[s] > cap_elems) {
            ++b;
            fill = 0;
        }
        bucket_of[s] = b;
        fill += len[s];
    }
    return n_sh > 0 ? b + 1 : 0;
}

/* Communication tensors from layers (Sec. II-B, Sec. III-A, Sec. III-C): whole
 * layers, in the given order, are merged greedily; a communication tensor is
 * closed when the next layer would push it over cap_elems, and it always holds
 * at least one layer (a layer larger than the cap is not split here).  Writes
 * the communication-tensor id of each layer; returns how many there are.  The
 * paper gives the target size only; the rule is this build's reading. */
int32_t orc_plan_group_layers(const int64_t *numel, int32_t n, int64_t cap_elems,
                              int32_t *group_of)
{
    int32_t g = 0;
    int64_t fill = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (fill > 0 && fill + numel[i] > cap_elems) {
            ++g;
            fill = 0;
        }
        group_of[i] = g;
        fill += numel[i];
    }
    return n > 0 ? g + 1 : 0;
}

/* Median-based tensor sharding (Sec. III-C): given the element counts of the
 * communication tensors, a tensor holding at least twice the reference count
 * is cut evenly into floor(numel/ref) parts, but never more than I parts.
 * ref <= 0 asks for the statistical median of numel[] (mean of the two middle
 * values for an even count).  parts[i] receives the number of pieces of
 * tensor i; the return value is the total number of units the filter then
 * sees. */
static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

int64_t orc_plan_median_parts(const int64_t *numel, int32_t n, int64_t ref,
                              int32_t I, int32_t *parts)
{
    if (n <= 0) return 0;
    if (ref <= 0) {
        int64_t *tmp = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
        memcpy(tmp, numel, sizeof(int64_t) * (size_t)n);
        qsort(tmp, (size_t)n, sizeof(int64_t), cmp_i64);
        ref = (n % 2) ? tmp[n / 2] : (tmp[n / 2 - 1] + tmp[n / 2]) / 2;
        free(tmp);
        if (ref <= 0) ref = 1;
    }
    int64_t total = 0;
    for (int32_t i = 0; i < n; ++i) {
        int64_t p = numel[i] / ref;
        if (p > I) p = I;
        if (p < 2) p = 1;
        parts[i] = (int32_t)p;
        total += p;
    }
    return total;
}

/* Even slicing of one tensor of `numel` elements into `parts` pieces: every
 * piece but the last has ceil(numel/parts) rounded up to a multiple of
 * `align` elements; the last takes the rest.  Writes piece lengths to len[]
 * and returns how many pieces are non-empty (always `parts` unless the
 * rounding used the tensor up early). */
int32_t orc_plan_even_slices(int64_t numel, int32_t parts, int64_t align,
                             int64_t *len)
{
    int64_t piece = (numel + parts - 1) / parts;
    piece = (piece + align - 1) / align * align;
    int32_t n = 0;
    int64_t left = numel;
    while (left > 0 && n < parts) {
        int64_t l = (n == parts - 1 || left < piece) ? left : piece;
        len[n++] = l;
        left -= l;
    }
    return n;
}

/* Sec. III-C end to end: the arena of a model under the paper's sharding rule.
 * Layers are merged into communication tensors (orc_plan_group_layers); the
 * median rule decides into how many pieces each is cut (orc_plan_median_parts)
 * and the even slicing how long the pieces are (orc_plan_even_slices).  Every
 * communication tensor starts at a multiple of `align` elements of the arena
 * (each is a buffer of its own in the framework the paper builds on), layers
 * inside it lie end to end; every piece is one shard for the filter, numbered
 * in arena order.  Fills tensor_off[n] (arena offset of each layer) and, when
 * sh_off is not NULL, the shards' offsets, lengths and communication-tensor
 * ids; returns the number of shards and writes the arena size to *arena. */
int64_t orc_plan_median_layout(const int64_t *numel, int32_t n, int64_t cap_elems, int32_t I,
                               int64_t ref, int64_t align, int64_t *tensor_off,
                               int64_t *sh_off, int64_t *sh_len, int32_t *sh_tensor,
                               int64_t *arena)
{
    *arena = 0;
    if (n <= 0) return 0;
    int32_t *group_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t n_groups = orc_plan_group_layers(numel, n, cap_elems, group_of);
    int64_t *group_numel = (int64_t *)calloc((size_t)n_groups, sizeof(int64_t));
    for (int32_t i = 0; i < n; ++i) group_numel[group_of[i]] += numel[i];
    int32_t *parts = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_groups);
    orc_plan_median_parts(group_numel, n_groups, ref, I, parts);
    int64_t *piece = (int64_t *)malloc(sizeof(int64_t) * (size_t)(I > 0 ? I : 1));
    int64_t n_shards = 0, end = 0;
    int32_t layer = 0;
    for (int32_t g = 0; g < n_groups; ++g) {
        int64_t begin = (end + align - 1) / align * align; /* the tensor's own buffer */
        int64_t at = begin;
        for (; layer < n && group_of[layer] == g; ++layer) { /* its layers, end to end */
            if (tensor_off) tensor_off[layer] = at;
            at += numel[layer];
        }
        end = at;
        int32_t m = orc_plan_even_slices(group_numel[g], parts[g], align, piece);
        int64_t o = begin;
        for (int32_t j = 0; j < m; ++j) {
            if (sh_off) {
                sh_off[n_shards] = o;
                sh_len[n_shards] = piece[j];
                sh_tensor[n_shards] = g;
            }
            o += piece[j];
            ++n_shards;
        }
    }
    *arena = end;
    free(piece);
    free(parts);
    free(group_numel);
    free(group_of);
    return n_shards;
}

/* ------------------------------------------------------------------ */
/* Coarse-grained filter (Sec. III-A; Definition 1)                    */
/* ------------------------------------------------------------------ */

/* Shard s is communicated in iteration t when (s + t) mod I == 0. */
int32_t orc_selected(int64_t s, uint64_t t, int32_t I)
{
    uint64_t a = (uint64_t)(s % I);
    uint64_t b = t % (uint64_t)I;
    return ((a + b) % (uint64_t)I) == 0 ? 1 : 0;
}

/* Packed layout of step t: the shards sent at t, in ascending order, one after
 * the other; each starts at the next multiple of `align` elements (align = 1:
 * plain concatenation; with equal-size shards that are multiples of `align`
 * the two coincide).  Returns the running position after shards [0, sh_hi). */
static int64_t round_up(int64_t x, int64_t align) { return (x + align - 1) / align * align; }

int64_t orc_packed_end(const int64_t *len, int64_t sh_hi, int32_t I, uint64_t t, int64_t align)
{
    int64_t p = 0;
    for (int64_t s = 0; s < sh_hi; ++s)
        if (orc_selected(s, t, I)) p = round_up(p, align) + len[s];
    return p;
}

/* ------------------------------------------------------------------ */
/* bf16 <-> fp32 (own implementation; round to nearest, ties to even)  */
/* ------------------------------------------------------------------ */

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) /* NaN: keep it a NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16;
    uint32_t drop = u & 0xffffu;
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) keep += 1u;
    return (uint16_t)keep;
}

uint16_t orc_f32_to_bf16(float f) { return f32_to_bf16(f); }
float orc_bf16_to_f32(uint16_t h) { return bf16_to_f32(h); }

/* ------------------------------------------------------------------ */
/* Compress: error feedback + filter + pack + residual (Algorithm 1)   */
/* ------------------------------------------------------------------ */

/*
 * For every element i of shards [sh_lo, sh_hi):
 *     a = G[i] + c * R[i]              Alg. 1 line 2, with the scheduler's
 *                                      coefficient c (one rounding: fmaf)
 *     selected shard:   send[p++] = a; R[i] = +0   (G' = a, so G - G' = 0)
 *     unselected shard: R[i] = a                   (G' = 0, Definition 1)
 * send is indexed from the start of the step's packed layout over ALL shards
 * (see orc_packed_end): p starts where shards [0, sh_lo) left it.  Returns the
 * number of elements written to send.
 */
int64_t orc_compress_f32(const float *G, float *R, float *send,
                          const int64_t *off, const int64_t *len,
                          int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                          float c, int64_t align)
{
    int64_t p = orc_packed_end(len, sh_lo, I, t, align);
    int64_t written = 0;
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) {
            p = round_up(p, align);
            written += len[s];
        }
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            float a = fmaf(c, R[i], G[i]);
            if (sel) {
                send[p++] = a;
                R[i] = 0.0f;
            } else {
                R[i] = a;
            }
        }
    }
    return written;
}

/* Same with bf16 storage: operands widen to fp32, one fmaf, one RNE back. */
int64_t orc_compress_bf16(const uint16_t *G, uint16_t *R, uint16_t *send,
                          const int64_t *off, const int64_t *len,
                          int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                          float c, int64_t align)
{
    int64_t p = orc_packed_end(len, sh_lo, I, t, align);
    int64_t written = 0;
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) {
            p = round_up(p, align);
            written += len[s];
        }
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            float a = fmaf(c, bf16_to_f32(R[i]), bf16_to_f32(G[i]));
            uint16_t h = f32_to_bf16(a);
            if (sel) {
                send[p++] = h;
                R[i] = 0;
            } else {
                R[i] = h;
            }
        }
    }
    return written;
}

/* Mixed precision: bf16 gradients and payload, fp32 residual.  Algorithm 1 with
 * the quantiser in line 3 made explicit:
 *     a  = G[i] + c * R[i]                 fp32, one rounding (fmaf)
 *     sent shard:   G' = bf16(a) (round to nearest even); send[p++] = G';
 *                   R[i] = a - G'          line 4: what rounding lost stays local
 *                                          (the difference is exact in fp32)
 *     kept shard:   R[i] = a               nothing is lost to rounding
 */
int64_t orc_compress_bf16_res32(const uint16_t *G, float *R, uint16_t *send,
                                const int64_t *off, const int64_t *len,
                                int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                                float c, int64_t align)
{
    int64_t p = orc_packed_end(len, sh_lo, I, t, align);
    int64_t written = 0;
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) {
            p = round_up(p, align);
            written += len[s];
        }
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            float a = fmaf(c, R[i], bf16_to_f32(G[i]));
            if (sel) {
                uint16_t h = f32_to_bf16(a);
                send[p++] = h;
                R[i] = a - bf16_to_f32(h);
            } else {
                R[i] = a;
            }
        }
    }
    return written;
}

/* Aliased-residual form: the caller's accumulation buffer already holds
 * G + residual (the producer added the new gradient into it: Algorithm 1 line 2
 * with c = 1).  Sent shards move to the payload and are cleared; the others are
 * left alone (their content IS the new residual).  esz = element size in bytes
 * (the operation only moves bit patterns). */
int64_t orc_compress_aliased(void *accum, void *send, int32_t esz,
                             const int64_t *off, const int64_t *len,
                             int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t, int64_t align)
{
    int64_t p = orc_packed_end(len, sh_lo, I, t, align);
    int64_t written = 0;
    unsigned char *a = (unsigned char *)accum, *o = (unsigned char *)send;
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        if (!orc_selected(s, t, I)) continue;
        p = round_up(p, align);
        written += len[s];
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            memcpy(o + p * esz, a + i * esz, (size_t)esz);
            memset(a + i * esz, 0, (size_t)esz);
            ++p;
        }
    }
    return written;
}

/* ------------------------------------------------------------------ */
/* Decompress: N-way average + unpack (Sec. II-A AllReduce + DP mean)  */
/* ------------------------------------------------------------------ */

/*
 * recv holds N workers' packed payloads, row w at recv + w*stride, each in
 * the layout orc_compress_* writes.  For shards [sh_lo, sh_hi):
 *     selected:   out[i] = (((recv[0][q] + recv[1][q]) + ...) + recv[N-1][q]) / N
 *     unselected: out[i] = +0                     (Definition 1, "otherwise")
 * The sum is a left fold over w = 0..N-1 in fp32; the division is IEEE.
 */
void orc_decompress_f32(const float *recv, int32_t N, int64_t stride,
                        float *out, const int64_t *off, const int64_t *len,
                        int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                        int64_t align)
{
    int64_t q = orc_packed_end(len, sh_lo, I, t, align);
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) q = round_up(q, align);
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            if (sel) {
                float acc = recv[q];
                for (int32_t w = 1; w < N; ++w) acc += recv[(int64_t)w * stride + q];
                out[i] = acc / (float)N;
                ++q;
            } else {
                out[i] = 0.0f;
            }
        }
    }
}

/* bf16 payloads: fp32 accumulator, one RNE at the end. */
void orc_decompress_bf16(const uint16_t *recv, int32_t N, int64_t stride,
                         uint16_t *out, const int64_t *off, const int64_t *len,
                         int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                         int64_t align)
{
    int64_t q = orc_packed_end(len, sh_lo, I, t, align);
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) q = round_up(q, align);
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            if (sel) {
                float acc = bf16_to_f32(recv[q]);
                for (int32_t w = 1; w < N; ++w)
                    acc += bf16_to_f32(recv[(int64_t)w * stride + q]);
                out[i] = f32_to_bf16(acc / (float)N);
                ++q;
            } else {
                out[i] = 0;
            }
        }
    }
}

/*
 * The same step when the exchange is a sum-AllReduce, which is how the paper
 * runs it (Sec. II-A: the gradients are aggregated by AllReduce and averaged;
 * Sec. III-B: COVAP keeps AllReduce because every worker sends the same
 * shards).  `summed` is ONE payload row, the element-wise sum of the N workers'
 * payloads as the collective delivered it, in the layout orc_compress_* writes.
 * For shards [sh_lo, sh_hi):
 *     selected:   out[i] = summed[q] / N
 *     unselected: out[i] = +0
 * The order in which the collective added the N payloads is its own; this
 * routine only divides.
 */
void orc_unpack_mean_f32(const float *summed, int32_t N, float *out,
                         const int64_t *off, const int64_t *len,
                         int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t, int64_t align)
{
    int64_t q = orc_packed_end(len, sh_lo, I, t, align);
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) q = round_up(q, align);
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i)
            out[i] = sel ? summed[q++] / (float)N : 0.0f;
    }
}

/* bf16 payload and result: widen, divide in fp32, one RNE back. */
void orc_unpack_mean_bf16(const uint16_t *summed, int32_t N, uint16_t *out,
                          const int64_t *off, const int64_t *len,
                          int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t, int64_t align)
{
    int64_t q = orc_packed_end(len, sh_lo, I, t, align);
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) q = round_up(q, align);
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i)
            out[i] = sel ? f32_to_bf16(bf16_to_f32(summed[q++]) / (float)N) : (uint16_t)0;
    }
}

/* ------------------------------------------------------------------ */
/* Top-k sparsifier with error feedback (contrast; Sec. I, Table II)   */
/* ------------------------------------------------------------------ */

typedef struct {
    uint32_t key;
    uint32_t idx;
} keyidx_t;

static int cmp_key_desc_idx_asc(const void *a, const void *b)
{
    const keyidx_t *x = (const keyidx_t *)a, *y = (const keyidx_t *)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

static int cmp_u32(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/*
 * a[i] = G[i] + c*R[i] (Alg. 1 line 2); keep the k entries of largest
 * magnitude.  Magnitudes are ordered by the bit pattern of |a| read as an
 * unsigned integer (a total order; NaN sorts above Inf); among equal
 * magnitudes the lower index wins.  Output: (vals, idx) in ascending index;
 * residual R = a with the kept entries set to +0 (Alg. 1 line 4).
 * The selection is a full sort: slow, and plainly the definition.
 * Returns 0, or -1 when k or n is out of range or memory runs out.
 */
int32_t orc_topk_f32(const float *G, float *R, int64_t n, int64_t k, float c,
                     float *vals, uint32_t *idx)
{
    if (n < 0 || k < 0 || k > n || n > (int64_t)0xffffffffLL) return -1;
    keyidx_t *ki = (keyidx_t *)malloc(sizeof(keyidx_t) * (size_t)(n ? n : 1));
    if (!ki) return -1;
    for (int64_t i = 0; i < n; ++i) {
        float a = fmaf(c, R[i], G[i]);
        R[i] = a;
        uint32_t u;
        memcpy(&u, &a, 4);
        ki[i].key = u & 0x7fffffffu;
        ki[i].idx = (uint32_t)i;
    }
    qsort(ki, (size_t)n, sizeof(keyidx_t), cmp_key_desc_idx_asc);
    for (int64_t j = 0; j < k; ++j) idx[j] = ki[j].idx;
    free(ki);
    qsort(idx, (size_t)k, sizeof(uint32_t), cmp_u32);
    for (int64_t j = 0; j < k; ++j) {
        vals[j] = R[idx[j]];
        R[idx[j]] = 0.0f;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Random-k and FP16 (contrast points without data dependency; Sec. II-C, */
/* Table III), each under Algorithm 1's error feedback, and their means  */
/* ------------------------------------------------------------------ */

/* Random-k: the k coordinates idx[] (distinct) are given -- all workers draw
 * them from a shared seed.  a = G + c*R; vals[j] = a[idx[j]]; R = a with the
 * sent coordinates set to +0. */
int32_t orc_randk_f32(const float *G, float *R, int64_t n, const uint32_t *idx, int64_t k,
                      float c, float *vals)
{
    if (n < 0 || k < 0 || k > n) return -1;
    for (int64_t i = 0; i < n; ++i) R[i] = fmaf(c, R[i], G[i]);
    for (int64_t j = 0; j < k; ++j) {
        vals[j] = R[idx[j]];
        R[idx[j]] = 0.0f;
    }
    return 0;
}

/* fp32 -> fp16, round to nearest even, with gradual underflow and overflow to
 * infinity (IEEE 754 binary16); own implementation. */
static uint16_t f32_to_f16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t mag = u & 0x7fffffffu;
    if (mag > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);            /* NaN */
    if (mag >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);           /* >= 65536 (and Inf) -> Inf */
    if (mag < 0x33000000u) return sign;                                  /* < 2^-25 -> 0 */
    int32_t e = (int32_t)(mag >> 23) - 127;                              /* unbiased exponent */
    uint32_t m = (mag & 0x7fffffu) | 0x800000u;                          /* 24-bit significand */
    int shift = e >= -14 ? 13 : 13 + (-14 - e);                          /* bits to drop */
    uint32_t keep = m >> shift;
    uint32_t drop = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (drop > half || (drop == half && (keep & 1u))) keep += 1u;
    uint32_t h;
    if (e >= -14)
        h = ((uint32_t)(e + 15) << 10) + (keep - 0x400u);                /* carry may bump the exponent: intended */
    else
        h = keep;                                                        /* subnormal (or the smallest normal on carry) */
    return (uint16_t)(sign | h);                                         /* 0x7c00 on overflow by rounding */
}

static float f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
    float v;
    if (e == 0x1fu) {
        uint32_t u = sign | 0x7f800000u | (m << 13);
        memcpy(&v, &u, 4);
        return v;
    }
    v = e ? ldexpf((float)(m | 0x400u), (int)e - 25) : ldexpf((float)m, -24);
    return sign ? -v : v;
}

uint16_t orc_f32_to_f16(float f) { return f32_to_f16(f); }
float orc_f16_to_f32(uint16_t h) { return f16_to_f32(h); }

/* FP16 quantiser: a = G + c*R; out[i] = fp16(a); R[i] = a - fp16(a). */
void orc_fp16_compress(const float *G, float *R, int64_t n, float c, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float a = fmaf(c, R[i], G[i]);
        uint16_t h = f32_to_f16(a);
        out[i] = h;
        R[i] = a - f16_to_f32(h);
    }
}

/* Mean of N fp16 payload rows: fp32 left fold over w = 0..N-1, then / N. */
void orc_fp16_mean(const uint16_t *recv, int32_t N, int64_t stride, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float acc = f16_to_f32(recv[i]);
        for (int32_t w = 1; w < N; ++w) acc += f16_to_f32(recv[(int64_t)w * stride + i]);
        out[i] = acc / (float)N;
    }
}

/*
 * Half-precision payload on the coarse filter: the FP16 scheme (Sec. II-C,
 * Table II) takes the place of the compressor in Algorithm 1 line 3 for the
 * shards the filter sends.  Gradients, residual and the dense result stay fp32.
 *     a = G[i] + c * R[i]                          (one rounding: fmaf)
 *     sent shard:   send[p++] = fp16(a)            round to nearest even
 *                   R[i] = a - fp32(send)          what the quantiser dropped
 *     kept shard:   R[i] = a
 * Packed layout as in orc_compress_f32.
 */
int64_t orc_compress_f32_pay16(const float *G, float *R, uint16_t *send,
                               const int64_t *off, const int64_t *len,
                               int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                               float c, int64_t align)
{
    int64_t p = orc_packed_end(len, sh_lo, I, t, align);
    int64_t written = 0;
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) {
            p = round_up(p, align);
            written += len[s];
        }
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            float a = fmaf(c, R[i], G[i]);
            if (sel) {
                uint16_t h = f32_to_f16(a);
                send[p++] = h;
                R[i] = a - f16_to_f32(h);
            } else {
                R[i] = a;
            }
        }
    }
    return written;
}

/* Matching dense mean: fp32 left fold over the widened halves of rows
 * w = 0..N-1, IEEE division by N; +0 where nothing was sent. */
void orc_decompress_pay16(const uint16_t *recv, int32_t N, int64_t stride,
                          float *out, const int64_t *off, const int64_t *len,
                          int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t,
                          int64_t align)
{
    int64_t q = orc_packed_end(len, sh_lo, I, t, align);
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) q = round_up(q, align);
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i) {
            if (sel) {
                float acc = f16_to_f32(recv[q]);
                for (int32_t w = 1; w < N; ++w)
                    acc += f16_to_f32(recv[(int64_t)w * stride + q]);
                out[i] = acc / (float)N;
                ++q;
            } else {
                out[i] = 0.0f;
            }
        }
    }
}

/* Half-precision payload summed by the collective (in half precision: that is
 * the collective's arithmetic, not this routine's); fp32 result = widened sum / N. */
void orc_unpack_mean_pay16(const uint16_t *summed, int32_t N, float *out,
                           const int64_t *off, const int64_t *len,
                           int64_t sh_lo, int64_t sh_hi, int32_t I, uint64_t t, int64_t align)
{
    int64_t q = orc_packed_end(len, sh_lo, I, t, align);
    for (int64_t s = sh_lo; s < sh_hi; ++s) {
        int sel = orc_selected(s, t, I);
        if (sel) q = round_up(q, align);
        for (int64_t i = off[s]; i < off[s] + len[s]; ++i)
            out[i] = sel ? f16_to_f32(summed[q++]) / (float)N : 0.0f;
    }
}

/* Mean of N sparse payloads of k (value, index) pairs: the dense sum is built
 * worker by worker (w = 0..N-1), then divided by N (not when N = 1). */
void orc_sparse_mean(const float *vals, const uint32_t *idx, int32_t N, int64_t k, int64_t stride,
                     int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = 0.0f;
    for (int32_t w = 0; w < N; ++w)
        for (int64_t j = 0; j < k; ++j) {
            int64_t at = (int64_t)w * stride + j;
            out[idx[at]] = out[idx[at]] + vals[at];
        }
    if (N > 1)
        for (int64_t i = 0; i < n; ++i) out[i] = out[i] / (float)N;
}

/* ------------------------------------------------------------------ */
/* Host policy                                                         */
/* ------------------------------------------------------------------ */

/* Interval from the communication-to-computation ratio: I = ceil(CCR), and
 * never below 1 (ratio 1 = no compression) (Sec. III-B).  Returns 0, or -1
 * for a CCR that is not a positive finite number. */
int32_t orc_ratio_from_ccr(double ccr, int32_t *I)
{
    if (!(ccr > 0.0) || isinf(ccr) || ccr > 2147483647.0) return -1;
    double c = ceil(ccr);
    *I = c < 1.0 ? 1 : (int32_t)c;
    return 0;
}

/* Error-feedback scheduler (Sec. III-D):
 *   coefficient = min(init_value + floor(num_steps/ascend_steps)*ascend_range, 1)
 * evaluated in double from the fp32 parameters, then rounded to fp32. */
float orc_ef_coeff(float init_value, uint64_t num_steps, uint64_t ascend_steps,
                   float ascend_range)
{
    double rises = (double)(num_steps / ascend_steps);
    double v = (double)init_value + rises * (double)ascend_range;
    if (v > 1.0) v = 1.0;
    return (float)v;
}
