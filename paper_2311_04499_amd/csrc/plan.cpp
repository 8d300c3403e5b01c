// Host side of libcovap: planner (arena layout, shards, buckets, interval), the
// launch geometry of a hot-path call and its replay (covap_plan_trace), ratio policy,
// error-feedback scheduler and the launch knobs.  Pure host code: nothing here
// touches the GPU, so plans can be built, queried and traced on a machine without one.
#include "plan.h"

#include <algorithm>
#include <atomic>
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

covap_status_t fail(covap_status_t st, const char *who, const char *msg)
{
    std::snprintf(g_last_error, sizeof g_last_error, "%s: %s", who ? who : "", msg ? msg : "");
    return st;
}

void clear_error() { g_last_error[0] = '\0'; }

static int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Number of shard indices s < x with s mod K < c (0 <= c <= K).
static int64_t below_class(int64_t x, int64_t c, int64_t K) { return (x / K) * c + std::min(c, x % K); }

// The shards of class c inside [lo, hi): first and last index, or first >= hi if none.
static void class_span(int32_t lo, int32_t hi, int32_t c, int32_t K, int64_t *first, int64_t *last)
{
    const int64_t f = (int64_t)lo + (((int64_t)c - lo % K) % K + K) % K;
    *first = f;
    *last = f < hi ? f + ((int64_t)hi - 1 - f) / K * K : f;
}

// Packed layout: at any step the selected shards (one residue class mod K) are
// stored in ascending shard order, each starting at the next multiple of the
// plan's alignment unit.  A shard's packed offset therefore depends only on the
// earlier shards of its own class -- the same number at every step that sends
// it -- and the packed range of a bucket (or of the arena) at a step follows from
// the first and the last shard of the step's class inside it; no table by step or
// by class is kept.  With fixed-size shards no padding ever appears (only the
// arena's last shard can be ragged).
covap_status_t resolve(const covap_plan_s *plan, uint64_t step, int32_t bucket, call_range *out)
{
    if (!plan) return fail(COVAP_EINVAL, "plan is null");
    const int32_t nb = (int32_t)plan->buckets.size();
    if (bucket < -1 || bucket >= nb) return fail(COVAP_ERANGE, "bucket out of range");
    const int32_t K = plan->K, c = first_selected(step, K);
    out->first_sel = c;
    out->bucket = bucket;
    out->sh_lo = bucket < 0 ? 0 : plan->buckets[(size_t)bucket].sh_lo;
    out->sh_hi = bucket < 0 ? (int32_t)plan->shards.size() : plan->buckets[(size_t)bucket].sh_hi;
    int64_t first, last;
    class_span(out->sh_lo, out->sh_hi, c, K, &first, &last);
    if (first < out->sh_hi) {
        const covap_shard_rec &f = plan->shards[(size_t)first], &l = plan->shards[(size_t)last];
        out->packed_base = f.packed_off;
        out->packed_elems = l.packed_off + l.len - f.packed_off;
    } else {  // nothing of this class here: the base is where the class would continue
        const int64_t prev = first - K;
        out->packed_base = prev >= 0 ? round_up(plan->shards[(size_t)prev].packed_off + plan->shards[(size_t)prev].len,
                                                plan->align_elems)
                                     : 0;
        out->packed_elems = 0;
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

// Class-by-class list of the shards [lo, hi), appended to `list`.
static void append_units(const covap_plan_s *p, int32_t lo, int32_t hi, covap_unit_list *list)
{
    const int32_t K = p->K;
    std::vector<int32_t> order;
    order.reserve((size_t)(hi - lo));
    for (int32_t s = lo; s < hi; ++s) order.push_back(s);
    std::sort(order.begin(), order.end(), [K](int32_t a, int32_t b) {
        return a % K != b % K ? a % K < b % K : a < b;
    });
    for (int32_t s : order) {
        const covap_shard_rec &sh = p->shards[(size_t)s];
        list->off.push_back(sh.off);
        list->poff.push_back(sh.packed_off);
        list->len.push_back((uint32_t)sh.len);
        for (int j = 0; j <= kTileLog2Max - kTileLog2Min; ++j) {
            const int64_t tile = (int64_t)1 << (kTileLog2Min + j);
            list->tiles[j].push_back(list->tiles[j].back() + (uint32_t)((sh.len + tile - 1) / tile));
        }
    }
}

// Packed offsets, bucket ranges, the largest payload, and (variable-length shards)
// the unit lists the launches copy from.
static void finish_tables(covap_plan_s *p)
{
    const int32_t K = p->K;
    const int64_t al = p->align_elems;
    const size_t n = p->shards.size();
    const int32_t nb = n ? p->shards.back().bucket + 1 : 0;
    p->buckets.assign((size_t)nb, covap_bucket_rec{-1, -1});
    p->packed_max = 0;
    for (size_t s = 0; s < n; ++s) {
        covap_shard_rec &sh = p->shards[s];
        covap_bucket_rec &b = p->buckets[(size_t)sh.bucket];
        if (b.sh_lo < 0) b.sh_lo = (int32_t)s;
        b.sh_hi = (int32_t)s + 1;
        // the previous shard of the same class, if any, ends where this one may start
        sh.packed_off = 0;
        if (s >= (size_t)K) {
            const covap_shard_rec &before = p->shards[s - (size_t)K];
            sh.packed_off = round_up(before.packed_off + before.len, al);
        }
        p->packed_max = std::max(p->packed_max, sh.packed_off + sh.len);
    }
    if (p->uniform) return;
    for (covap_unit_list *list : {&p->by_arena, &p->by_bucket})
        for (auto &t : list->tiles) t.assign(1, 0u);
    append_units(p, 0, (int32_t)n, &p->by_arena);
    for (const covap_bucket_rec &b : p->buckets) append_units(p, b.sh_lo, b.sh_hi, &p->by_bucket);
}

// ---- launch geometry ---------------------------------------------------------------

fixed_geom fixed_launch(const covap_plan_s *p, const call_range &cr, uint32_t tile_elems, bool sent_only,
                        uint32_t *grid)
{
    fixed_geom g;
    g.S = p->opts.shard_elems;
    g.shard_len = (uint32_t)g.S;
    g.n_shards = (uint32_t)p->shards.size();
    g.last_len = p->shards.empty() ? 0u : (uint32_t)p->shards.back().len;
    g.K = p->K;
    g.first_sel = cr.first_sel;
    g.tiles_per_shard = (uint32_t)((g.S + tile_elems - 1) / tile_elems);
    const uint32_t K = (uint32_t)g.K, lo = (uint32_t)cr.sh_lo, n = (uint32_t)(cr.sh_hi - cr.sh_lo);
    if (sent_only) {
        const uint32_t phase = ((uint32_t)cr.first_sel + K - lo % K) % K;  // offset of the first sent shard
        g.sh_lo = lo + phase;
        g.sh_step = K;
        *grid = (phase < n ? (n - phase + K - 1) / K : 0u) * g.tiles_per_shard;
    } else {
        g.sh_lo = lo;
        g.sh_step = 1u;
        *grid = n * g.tiles_per_shard;
    }
    return g;
}

// Positions [*ua, *ub) of the call's units in its list, and [*sa, *sb) of those of
// the class sent at this step.
static const covap_unit_list &call_units(const covap_plan_s *p, const call_range &cr, bool sent_only,
                                         int64_t *ua, int64_t *ub, int64_t *sa, int64_t *sb)
{
    const int64_t K = p->K, c = cr.first_sel;
    const int64_t base = cr.bucket < 0 ? 0 : cr.sh_lo;
    *sa = base + below_class(cr.sh_hi, c, K) - below_class(cr.sh_lo, c, K);
    *sb = base + below_class(cr.sh_hi, c + 1, K) - below_class(cr.sh_lo, c + 1, K);
    *ua = sent_only ? *sa : base;
    *ub = sent_only ? *sb : base + (cr.sh_hi - cr.sh_lo);
    return cr.bucket < 0 ? p->by_arena : p->by_bucket;
}

int32_t table_launches(const covap_plan_s *p, const call_range &cr, bool sent_only)
{
    int64_t ua, ub, sa, sb;
    call_units(p, cr, sent_only, &ua, &ub, &sa, &sb);
    return (int32_t)((ub - ua + kMaxUnits - 1) / kMaxUnits);
}

void table_launch(const covap_plan_s *p, const call_range &cr, uint32_t tile_elems, bool sent_only, int32_t i,
                  table_geom *g)
{
    int64_t ua, ub, sa, sb;
    const covap_unit_list &list = call_units(p, cr, sent_only, &ua, &ub, &sa, &sb);
    int lg = 0;
    while (((uint32_t)1 << lg) < tile_elems) ++lg;
    const uint32_t *tiles = list.tiles[lg - kTileLog2Min].data();
    const int64_t pa = ua + (int64_t)i * kMaxUnits, pb = std::min<int64_t>(pa + kMaxUnits, ub);
    const size_t cnt = (size_t)(pb - pa);
    std::memcpy(g->off, list.off.data() + pa, cnt * sizeof(int64_t));
    std::memcpy(g->poff, list.poff.data() + pa, cnt * sizeof(int64_t));
    std::memcpy(g->len, list.len.data() + pa, cnt * sizeof(uint32_t));
    for (size_t u = 0; u < cnt; ++u) g->first[u] = tiles[pa + (int64_t)u] - tiles[pa];
    for (size_t u = cnt; u < (size_t)kMaxUnits; ++u) {  // never looked up: no tile index reaches kNoTile
        g->off[u] = 0;
        g->poff[u] = 0;
        g->len[u] = 0u;
        g->first[u] = kNoTile;
    }
    g->first[kMaxUnits] = kNoTile;
    const uint32_t total = tiles[pb] - tiles[pa];
    const int64_t ca = std::min(std::max(sa, pa), pb), cb = std::min(std::max(sb, pa), pb);  // sent units of this launch
    g->sent_lo = tiles[ca] - tiles[pa];
    g->n_sent = tiles[cb] - tiles[ca];
    g->n_unsent = total - g->n_sent;
    // deal sent and unsent tiles out in alternating blocks when there are enough of both; blocks of
    // 1024 tiles measured best for decompress on the VGG-19-, BERT- and GPT-2-shaped sets (78.5 / 80.3 /
    // 79.8 % of peak; 64, 256 and 4096 tiles: 1 to 1.5 points lower, 16384: 7 lower)
    const uint32_t fewer = std::min(g->n_sent, g->n_unsent);
    g->mixed = fewer > 0u ? 1u : 0u;
    g->g_shift = 10;
    while (g->g_shift > 6 && fewer < (4u << g->g_shift)) --g->g_shift;
    g->rho = 0u;
    if (g->mixed) {
        const uint64_t G = (uint64_t)1 << g->g_shift;
        const uint64_t bs = (g->n_sent + G - 1) >> g->g_shift, bu = (g->n_unsent + G - 1) >> g->g_shift;
        g->rho = (uint32_t)(((bs << 32) + (bs + bu) - 1) / (bs + bu));  // ceil(bs * 2^32 / (bs + bu)) < 2^32 as bu >= 1
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

// Largest arena: the size up to which the kernels' grids and 64-bit offsets have been
// run on the hardware (2^33 elements: 32 GiB of fp32 per buffer).
static constexpr int64_t kMaxTotalElems = (int64_t)1 << 33;

namespace {
struct knob {
    const char *key;
    int covap::tuning::*field;
    int initial;
    int allowed[6];  // -1 ends the list
};
const knob kKnobs[] = {
    {"compress_threads", &covap::tuning::compress_threads, 64, {64, 256, -1, -1}},
    {"compress_unroll", &covap::tuning::compress_unroll, 1, {1, 2, 4, -1}},
    {"decompress_threads", &covap::tuning::decompress_threads, 64, {64, 256, -1, -1}},
    {"decompress_tile", &covap::tuning::decompress_tile, 1, {1, 2, 4, -1}},
    {"decompress_unroll", &covap::tuning::decompress_unroll, 1, {1, 2, 4, -1}},
    {"nontemporal", &covap::tuning::nontemporal, 1, {0, 1, -1, -1}},
    {"decompress_lds_pad", &covap::tuning::decompress_lds_pad, 6144, {0, 6144, 8192, 24576, 32768, 49152}},
    {"topk_pass1_waves", &covap::tuning::topk_pass1_waves, 4, {1, 2, 4, -1}},
    {"topk_pass1_lds_pad", &covap::tuning::topk_pass1_lds_pad, 0, {0, 6144, 8192, 24576, -1}},
};
constexpr int kNumKnobs = (int)(sizeof kKnobs / sizeof kKnobs[0]);

// The knobs' current values; -1 = never set (the knob's initial value applies).
std::atomic<int> g_knob[kNumKnobs] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}};

int knob_value(int i)
{
    const int v = g_knob[i].load(std::memory_order_relaxed);
    return v < 0 ? kKnobs[i].initial : v;
}
}  // namespace

namespace covap {
tuning tune()
{
    tuning t;
    t.decompress_shape_unset = true;
    for (int i = 0; i < kNumKnobs; ++i) {
        const int raw = g_knob[i].load(std::memory_order_relaxed);
        t.*(kKnobs[i].field) = raw < 0 ? kKnobs[i].initial : raw;
        if (raw >= 0 && (kKnobs[i].field == &tuning::decompress_threads || kKnobs[i].field == &tuning::decompress_tile ||
                         kKnobs[i].field == &tuning::decompress_lds_pad))
            t.decompress_shape_unset = false;
    }
    return t;
}
}  // namespace covap

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
        if (total > kMaxTotalElems) return fail(COVAP_EINVAL, "covap_plan: more than 2^33 elements in all");
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
        if (p->total_elems > kMaxTotalElems) {  // alignment padding of variable-length shards counts
            delete p;
            return fail(COVAP_EINVAL, "covap_plan: more than 2^33 elements in all");
        }
        finish_tables(p);
    } catch (...) {  // bad_alloc, or length_error from a vector: nothing may cross the C boundary
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
    for (int64_t s = first_selected(step, p->K); s < ns; s += p->K) {  // 64-bit: s + K passes 2^31 for large K
        if (ids && n < cap) ids[n] = (int32_t)s;
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

covap_status_t covap_tune_set(const char *key, int32_t value)
{
    clear_error();
    if (!key) return fail(COVAP_EINVAL, "covap_tune_set: null key");
    for (int i = 0; i < kNumKnobs; ++i) {
        if (std::strcmp(key, kKnobs[i].key)) continue;
        if (value == -1) {  // back to "never set"
            g_knob[i].store(-1, std::memory_order_relaxed);
            return COVAP_OK;
        }
        for (int a : kKnobs[i].allowed) {
            if (a < 0) break;
            if (a == value) {
                g_knob[i].store(value, std::memory_order_relaxed);
                return COVAP_OK;
            }
        }
        char msg[160];
        std::snprintf(msg, sizeof msg, "covap_tune_set: value %d not allowed for %s", (int)value, kKnobs[i].key);
        return fail(COVAP_EINVAL, msg);
    }
    return fail(COVAP_EINVAL, "covap_tune_set: unknown key");
}

int32_t covap_tune_get(const char *key)
{
    if (!key) return -1;
    for (int i = 0; i < kNumKnobs; ++i)
        if (!std::strcmp(key, kKnobs[i].key)) return knob_value(i);
    return -1;
}

int64_t covap_plan_trace(const covap_plan_t *plan, uint64_t step, int32_t bucket, int32_t tile_elems,
                         int32_t sent_only, int64_t cap, int64_t *off, int64_t *poff, int32_t *n,
                         uint8_t *sel, int32_t *n_launches, int64_t *n_workgroups)
{
    clear_error();
    call_range cr;
    if (resolve(plan, step, bucket, &cr) != COVAP_OK) return -1;
    if (tile_elems < (1 << kTileLog2Min) || tile_elems > (1 << kTileLog2Max) || (tile_elems & (tile_elems - 1))) {
        fail(COVAP_EINVAL, "covap_plan_trace: tile_elems must be a power of two in 256..8192");
        return -1;
    }
    int64_t count = 0, groups = 0;
    int32_t launches = 0;
    auto replay = [&](const auto &g, uint32_t grid) {
        if (grid == 0u) return;
        ++launches;
        groups += grid;
        for (uint32_t b = 0; b < grid; ++b) {
            tile_ref t;
            if (!resolve_tile(g, b, (uint32_t)tile_elems, t)) continue;
            if (count < cap) {
                if (off) off[count] = t.off;
                if (poff) poff[count] = t.poff;
                if (n) n[count] = t.n;
                if (sel) sel[count] = t.sel ? 1 : 0;
            }
            ++count;
        }
    };
    if (cr.sh_hi > cr.sh_lo) {
        if (plan->uniform) {
            uint32_t grid = 0;
            const fixed_geom g = fixed_launch(plan, cr, (uint32_t)tile_elems, sent_only != 0, &grid);
            replay(g, grid);
        } else {
            const int32_t nl = table_launches(plan, cr, sent_only != 0);
            for (int32_t i = 0; i < nl; ++i) {
                table_geom g;
                table_launch(plan, cr, (uint32_t)tile_elems, sent_only != 0, i, &g);
                replay(g, grid_of(g));
            }
        }
    }
    if (n_launches) *n_launches = launches;
    if (n_workgroups) *n_workgroups = groups;
    return count;
}

const char *covap_last_error(void) { return g_last_error; }
const char *covap_version(void) { return "0.1.0"; }

}  // extern "C"
