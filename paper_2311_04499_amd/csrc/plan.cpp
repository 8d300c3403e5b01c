// Host side of libcovap: planner (arena layout, shards, buckets, interval),
// ratio policy and error-feedback scheduler.  Pure host code: nothing here
// touches the GPU, so plans can be built and queried on a machine without one.
#include "plan.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

namespace covap {

// The calling thread's last error text lives in a fixed buffer, so that reporting an
// error never allocates (and so can neither fail nor throw across the C boundary).
static thread_local char g_last_error[256] = "";

covap_status_t fail(covap_status_t st, const char *msg)
{
    std::snprintf(g_last_error, sizeof g_last_error, "%s", msg ? msg : "");
    return st;
}

covap_status_t fail(covap_status_t st, const std::string &msg) { return fail(st, msg.c_str()); }

void clear_error() { g_last_error[0] = '\0'; }

tuning &tune()
{
    static tuning t;
    return t;
}

covap_status_t resolve(const covap_plan_s *plan, uint64_t step, int32_t bucket, call_range *out)
{
    if (!plan) return fail(COVAP_EINVAL, "plan is null");
    const int32_t nb = (int32_t)plan->buckets.size();
    if (bucket < -1 || bucket >= nb) return fail(COVAP_ERANGE, "bucket out of range");
    const int32_t r = (int32_t)(step % (uint64_t)plan->K);
    out->first_sel = first_selected(step, plan->K);
    if (bucket < 0) {
        out->sh_lo = 0;
        out->sh_hi = (int32_t)plan->shards.size();
        out->packed_base = 0;
        out->packed_elems = plan->packed_total[r];
    } else {
        const covap_bucket_rec &b = plan->buckets[bucket];
        out->sh_lo = b.sh_lo;
        out->sh_hi = b.sh_hi;
        out->packed_base = b.packed_base[r];
        out->packed_elems = b.packed_elems[r];
    }
    return COVAP_OK;
}

// Shards -> buckets: consecutive shards are grouped greedily; a bucket closes
// when the next shard would push it past the cap (Sec. III-A gives only the
// target size of a communication tensor, about 25 MB).
static void assign_buckets(covap_plan_s *p, int64_t cap_elems)
{
    int32_t b = 0;
    int64_t fill = 0;
    for (auto &sh : p->shards) {
        if (fill > 0 && fill + sh.len > cap_elems) {
            ++b;
            fill = 0;
        }
        sh.bucket = b;
        fill += sh.len;
    }
}

static int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Packed layout: at any step the selected shards (one residue class mod K) are
// stored in ascending shard order, each starting at the next multiple of the
// plan's alignment unit.  A shard's packed offset therefore depends only on the
// earlier shards of its own class -- the same number at every step that sends
// it.  With fixed-size shards no padding ever appears (only the arena's last
// shard can be ragged).  Also fills the per-bucket and whole-arena packed
// extents by residue.
static void finish_tables(covap_plan_s *p)
{
    const int32_t K = p->K;
    const int64_t al = p->align_elems;
    const int32_t nb = p->shards.empty() ? 0 : p->shards.back().bucket + 1;
    p->buckets.assign((size_t)nb, covap_bucket_rec());
    for (auto &b : p->buckets) {
        b.sh_lo = -1;
        b.sh_hi = -1;
        b.packed_base.assign((size_t)K, 0);
        b.packed_elems.assign((size_t)K, 0);
    }
    std::vector<int64_t> end((size_t)K, 0);  // running end of each class's packed layout
    for (size_t s = 0; s < p->shards.size(); ++s) {
        covap_shard_rec &sh = p->shards[s];
        covap_bucket_rec &b = p->buckets[(size_t)sh.bucket];
        if (b.sh_lo < 0) {  // first shard of its bucket: where would each class continue?
            b.sh_lo = (int32_t)s;
            for (int32_t r = 0; r < K; ++r)  // r = step mod K sends class (K - r) mod K
                b.packed_base[(size_t)r] = round_up(end[(size_t)((K - r) % K)], al);
        }
        b.sh_hi = (int32_t)s + 1;
        const size_t cls = s % (size_t)K;
        sh.packed_off = round_up(end[cls], al);
        end[cls] = sh.packed_off + sh.len;
        const size_t r = (size_t)((K - (int32_t)cls) % K);
        b.packed_elems[r] = end[cls] - b.packed_base[r];
    }
    p->packed_total.assign((size_t)K, 0);
    p->packed_max = 0;
    for (int32_t r = 0; r < K; ++r) {
        p->packed_total[(size_t)r] = end[(size_t)((K - r) % K)];
        p->packed_max = std::max(p->packed_max, p->packed_total[(size_t)r]);
    }
}

// Fixed-size shards over a tightly packed arena.
static void build_fixed(covap_plan_s *p, const int64_t *numel, int32_t n, int64_t cap_elems)
{
    p->uniform = true;
    int64_t acc = 0;
    for (int32_t i = 0; i < n; ++i) {  // tight packing, in the caller's order
        p->tensor_off[(size_t)i] = acc;
        acc += numel[i];
    }
    p->total_elems = acc;
    const int64_t S = p->opts.shard_elems;
    for (int64_t b = 0; b < acc; b += S) {
        covap_shard_rec sh;
        sh.off = b;
        sh.len = std::min(S, acc - b);
        sh.packed_off = 0;
        sh.bucket = 0;
        p->shards.push_back(sh);
    }
    assign_buckets(p, cap_elems);
}

// Sec. III-C.  Layers are merged, in order, into communication tensors of about
// the cap (whole layers only; a layer above the cap stands alone).  The median of
// their element counts (or the caller's reference count) decides the cut: a
// tensor with at least twice that many elements is sliced evenly into
// floor(numel / ref) pieces, never more than K.  Every piece is one shard for the
// filter.  Each communication tensor starts on an alignment boundary of the arena
// (they are separate buffers in the framework the paper builds on), layers inside
// it are tight; pieces are multiples of the alignment unit except a tensor's last.
static void build_median(covap_plan_s *p, const int64_t *numel, int32_t n, int64_t cap_elems)
{
    p->uniform = false;
    const int64_t al = p->align_elems;
    std::vector<int32_t> group_of((size_t)n);
    std::vector<int64_t> group_numel;
    int64_t fill = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (group_numel.empty() || (fill > 0 && fill + numel[i] > cap_elems)) {
            group_numel.push_back(0);
            fill = 0;
        }
        group_of[(size_t)i] = (int32_t)group_numel.size() - 1;
        group_numel.back() += numel[i];
        fill += numel[i];
    }
    int64_t ref = p->opts.ref_elems;
    if (ref <= 0) {
        std::vector<int64_t> sorted(group_numel);
        std::sort(sorted.begin(), sorted.end());
        const size_t m = sorted.size();
        ref = (m % 2) ? sorted[m / 2] : (sorted[m / 2 - 1] + sorted[m / 2]) / 2;
        if (ref <= 0) ref = 1;
    }
    int64_t pos = 0;
    int32_t i = 0;
    for (size_t g = 0; g < group_numel.size(); ++g) {
        pos = round_up(pos, al);
        const int64_t start = pos;
        while (i < n && group_of[(size_t)i] == (int32_t)g) {
            p->tensor_off[(size_t)i] = pos;
            pos += numel[i];
            ++i;
        }
        const int64_t total = group_numel[g];
        int64_t parts = total / ref;
        if (parts > p->K) parts = p->K;
        if (parts < 2) parts = 1;
        const int64_t piece = round_up((total + parts - 1) / parts, al);
        int64_t left = total, o = start;
        for (int64_t k = 0; k < parts && left > 0; ++k) {
            covap_shard_rec sh;
            sh.off = o;
            sh.len = (k == parts - 1 || left < piece) ? left : piece;
            sh.packed_off = 0;
            sh.bucket = (int32_t)g;
            p->shards.push_back(sh);
            o += sh.len;
            left -= sh.len;
        }
    }
    p->total_elems = pos;
}

}  // namespace covap

using namespace covap;

extern "C" {

covap_status_t covap_plan(const int64_t *tensor_numel, int32_t n_tensors,
                          const covap_plan_opts_t *opts, covap_plan_t **out)
{
    clear_error();
    if (!tensor_numel || !opts || !out) return fail(COVAP_EINVAL, "covap_plan: null argument");
    *out = nullptr;
    if (n_tensors < 1) return fail(COVAP_EINVAL, "covap_plan: n_tensors < 1");
    if (opts->K < 1) return fail(COVAP_EINVAL, "covap_plan: K < 1");
    if (opts->reserved != 0) return fail(COVAP_EINVAL, "covap_plan: reserved must be 0");
    if (opts->dtype != COVAP_F32 && opts->dtype != COVAP_BF16 && opts->dtype != COVAP_BF16_RES32 &&
        opts->dtype != COVAP_F32_PAY16)
        return fail(COVAP_EINVAL, "covap_plan: unknown dtype");
    if (opts->bucket_cap_bytes <= 0) return fail(COVAP_EINVAL, "covap_plan: bucket_cap_bytes <= 0");
    // alignment unit of shard starts and packed offsets: 16 bytes of the narrowest buffer
    const int32_t epv = opts->dtype == COVAP_F32 ? 4 : 8;
    const int64_t esz = opts->dtype == COVAP_F32 || opts->dtype == COVAP_F32_PAY16 ? 4 : 2;  // gradient element
    int64_t total = 0;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (tensor_numel[i] < 0) return fail(COVAP_EINVAL, "covap_plan: negative element count");
        total += tensor_numel[i];
        if (total >= ((int64_t)1 << 38))  // keeps every grid below 2^31 workgroups
            return fail(COVAP_EINVAL, "covap_plan: total elements >= 2^38");
    }
    if (opts->mode != COVAP_SHARD_FIXED && opts->mode != COVAP_SHARD_MEDIAN)
        return fail(COVAP_EINVAL, "covap_plan: unknown mode");
    if (opts->mode == COVAP_SHARD_FIXED) {
        if (opts->shard_elems > ((int64_t)1 << 30))
            return fail(COVAP_EINVAL, "covap_plan: shard_elems > 2^30");
        if (opts->shard_elems <= 0 || opts->shard_elems % epv != 0)
            return fail(COVAP_EINVAL,
                        "covap_plan: shard_elems must be a positive multiple of the 16-byte vector");
        if ((total + opts->shard_elems - 1) / opts->shard_elems > (int64_t)0x7fffffff / 2)
            return fail(COVAP_EINVAL, "covap_plan: too many shards");
    } else if (opts->ref_elems < 0) {
        return fail(COVAP_EINVAL, "covap_plan: ref_elems < 0");
    }

    covap_plan_s *p = new (std::nothrow) covap_plan_s();
    if (!p) return fail(COVAP_ENOMEM, "covap_plan: out of host memory");
    try {
        p->opts = *opts;
        p->K = opts->K;
        p->elems_per_vec = epv;
        // Variable-length shards start on 1 KiB boundaries of every buffer (the
        // narrowest element decides), the size of one wave's access: measured on the
        // GPT-2-medium-shaped set, decompress runs 7 % faster than with 16-byte
        // alignment (it reads N rows at these offsets); 4 KiB gains nothing more.
        // Fixed-size shards need no padding; their alignment is that of shard_elems.
        p->align_elems = opts->mode == COVAP_SHARD_MEDIAN ? (opts->dtype == COVAP_F32 ? 256 : 512) : epv;
        p->tensor_off.resize((size_t)n_tensors);
        const int64_t cap_elems = std::max<int64_t>(1, opts->bucket_cap_bytes / esz);
        if (opts->mode == COVAP_SHARD_FIXED)
            build_fixed(p, tensor_numel, n_tensors, cap_elems);
        else
            build_median(p, tensor_numel, n_tensors, cap_elems);
        for (const covap_shard_rec &sh : p->shards)
            if (sh.len > ((int64_t)1 << 31) - 1) {
                delete p;
                return fail(COVAP_EINVAL, "covap_plan: a shard exceeds 2^31 - 1 elements");
            }
        finish_tables(p);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(COVAP_ENOMEM, "covap_plan: out of host memory");
    }
    *out = p;
    return COVAP_OK;
}

void covap_plan_free(covap_plan_t *plan) { delete plan; }

int64_t covap_plan_total_elems(const covap_plan_t *p) { return p ? p->total_elems : -1; }
int32_t covap_plan_num_tensors(const covap_plan_t *p) { return p ? (int32_t)p->tensor_off.size() : -1; }
int32_t covap_plan_num_shards(const covap_plan_t *p) { return p ? (int32_t)p->shards.size() : -1; }
int32_t covap_plan_num_buckets(const covap_plan_t *p) { return p ? (int32_t)p->buckets.size() : -1; }
int32_t covap_plan_interval(const covap_plan_t *p) { return p ? p->K : -1; }
int32_t covap_plan_align_elems(const covap_plan_t *p) { return p ? p->align_elems : -1; }

int64_t covap_plan_tensor_offset(const covap_plan_t *p, int32_t i)
{
    if (!p || i < 0 || i >= (int32_t)p->tensor_off.size()) return -1;
    return p->tensor_off[(size_t)i];
}

covap_status_t covap_plan_shard(const covap_plan_t *p, int32_t s, int64_t *off, int64_t *len,
                                int32_t *bucket)
{
    clear_error();
    if (!p) return fail(COVAP_EINVAL, "covap_plan_shard: plan is null");
    if (s < 0 || s >= (int32_t)p->shards.size())
        return fail(COVAP_ERANGE, "covap_plan_shard: shard out of range");
    const covap_shard_rec &sh = p->shards[(size_t)s];
    if (off) *off = sh.off;
    if (len) *len = sh.len;
    if (bucket) *bucket = sh.bucket;
    return COVAP_OK;
}

covap_status_t covap_plan_bucket(const covap_plan_t *p, int32_t b, int32_t *sh_lo, int32_t *sh_hi)
{
    clear_error();
    if (!p) return fail(COVAP_EINVAL, "covap_plan_bucket: plan is null");
    if (b < 0 || b >= (int32_t)p->buckets.size())
        return fail(COVAP_ERANGE, "covap_plan_bucket: bucket out of range");
    if (sh_lo) *sh_lo = p->buckets[(size_t)b].sh_lo;
    if (sh_hi) *sh_hi = p->buckets[(size_t)b].sh_hi;
    return COVAP_OK;
}

int32_t covap_plan_is_selected(const covap_plan_t *p, uint64_t step, int32_t s)
{
    if (!p || s < 0 || s >= (int32_t)p->shards.size()) return -1;
    return (s % p->K) == first_selected(step, p->K) ? 1 : 0;
}

int32_t covap_plan_selected(const covap_plan_t *p, uint64_t step, int32_t *ids, int32_t cap)
{
    if (!p) return -1;
    int32_t n = 0;
    const int32_t ns = (int32_t)p->shards.size();
    for (int32_t s = first_selected(step, p->K); s < ns; s += p->K) {
        if (ids && n < cap) ids[n] = s;
        ++n;
    }
    return n;
}

int64_t covap_plan_packed_elems(const covap_plan_t *p, uint64_t step, int32_t bucket)
{
    call_range cr;
    if (resolve(p, step, bucket, &cr) != COVAP_OK) return -1;
    return cr.packed_elems;
}

int64_t covap_plan_packed_base(const covap_plan_t *p, uint64_t step, int32_t bucket)
{
    call_range cr;
    if (resolve(p, step, bucket, &cr) != COVAP_OK) return -1;
    return cr.packed_base;
}

int64_t covap_plan_packed_elems_max(const covap_plan_t *p) { return p ? p->packed_max : -1; }

covap_status_t covap_ratio_from_ccr(double ccr, int32_t *K)
{
    clear_error();
    if (!K) return fail(COVAP_EINVAL, "covap_ratio_from_ccr: null out");
    if (!(ccr > 0.0) || !std::isfinite(ccr) || ccr >= 2147483648.0)
        return fail(COVAP_EINVAL, "covap_ratio_from_ccr: CCR must be in (0, 2^31)");
    const double up = std::ceil(ccr);
    *K = up < 1.0 ? 1 : (int32_t)up;
    return COVAP_OK;
}

covap_status_t covap_ratio_from_times(double t_comm, double t_comp, int32_t *K)
{
    clear_error();
    if (!(t_comm > 0.0) || !(t_comp > 0.0) || !std::isfinite(t_comm) || !std::isfinite(t_comp))
        return fail(COVAP_EINVAL, "covap_ratio_from_times: times must be positive and finite");
    return covap_ratio_from_ccr(t_comm / t_comp, K);
}

covap_status_t covap_ef_coeff(float init_value, uint64_t num_steps, uint64_t ascend_steps,
                              float ascend_range, float *coeff)
{
    clear_error();
    if (!coeff) return fail(COVAP_EINVAL, "covap_ef_coeff: null out");
    if (ascend_steps == 0) return fail(COVAP_EINVAL, "covap_ef_coeff: ascend_steps == 0");
    if (!std::isfinite(init_value) || !std::isfinite(ascend_range))
        return fail(COVAP_EINVAL, "covap_ef_coeff: non-finite parameter");
    const double rises = (double)(num_steps / ascend_steps);
    double v = (double)init_value + rises * (double)ascend_range;
    if (v > 1.0) v = 1.0;
    *coeff = (float)v;
    return COVAP_OK;
}

namespace {
struct knob {
    const char *key;
    int covap::tuning::*field;
    int allowed[5];  // 0-terminated unless the knob allows 0 (then -1-terminated)
};
const knob kKnobs[] = {
    {"compress_threads", &covap::tuning::compress_threads, {64, 256, -1, -1, -1}},
    {"compress_unroll", &covap::tuning::compress_unroll, {1, 2, 4, -1, -1}},
    {"decompress_threads", &covap::tuning::decompress_threads, {64, 256, -1, -1, -1}},
    {"decompress_tile", &covap::tuning::decompress_tile, {1, 2, 4, -1, -1}},
    {"decompress_unroll", &covap::tuning::decompress_unroll, {1, 2, 4, -1, -1}},
    {"nontemporal", &covap::tuning::nontemporal, {0, 1, -1, -1, -1}},
    {"decompress_lds_pad", &covap::tuning::decompress_lds_pad, {0, 6144, 8192, -1, -1}},
    {"topk_pass1_waves", &covap::tuning::topk_pass1_waves, {1, 2, 4, -1, -1}},
    {"topk_pass1_lds_pad", &covap::tuning::topk_pass1_lds_pad, {0, 6144, 8192, 24576, -1}},
};
}  // namespace

covap_status_t covap_tune_set(const char *key, int32_t value)
{
    clear_error();
    if (!key) return fail(COVAP_EINVAL, "covap_tune_set: null key");
    for (const knob &k : kKnobs) {
        if (std::strcmp(key, k.key)) continue;
        for (int a : k.allowed)
            if (a >= 0 && a == value) {
                tune().*(k.field) = value;
                return COVAP_OK;
            }
        return fail(COVAP_EINVAL, std::string("covap_tune_set: value not allowed for ") + key);
    }
    return fail(COVAP_EINVAL, "covap_tune_set: unknown key");
}

int32_t covap_tune_get(const char *key)
{
    if (!key) return -1;
    for (const knob &k : kKnobs)
        if (!std::strcmp(key, k.key)) return tune().*(k.field);
    return -1;
}

const char *covap_last_error(void) { return g_last_error; }
const char *covap_version(void) { return "0.1.0"; }

}  // extern "C"
