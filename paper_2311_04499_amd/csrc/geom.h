// Internal: launch geometry of the compress / take / decompress kernels -- how a
// workgroup index becomes a tile of the arena.  The same functions run on the
// device (a kernel resolves its blockIdx.x) and on the host (the planner's trace
// query replays a launch block by block), so what the kernels index can be
// checked on a machine without a GPU.  Not part of the public ABI.
#pragma once

#include <cstdint>

#if defined(__HIP__)  // a HIP translation unit: the kernels' side
#define COVAP_HD __host__ __device__ inline __attribute__((always_inline))
#define COVAP_UNROLL _Pragma("unroll")
#else  // plain C++: the planner (also built on its own, under sanitizers, by the tests)
#define COVAP_HD inline
#define COVAP_UNROLL
#endif

namespace covap {

// One tile: `n` consecutive elements of one shard, all sent or all kept back.
struct tile_ref {
    int64_t off;   // arena element offset
    int64_t poff;  // packed element offset
    int32_t n;     // elements in the tile, 1..tile_elems
    bool sel;      // the tile's shard is sent at this step
};

// ---- fixed-size shards ---------------------------------------------------------
//
// Shard s covers [s*S, min((s+1)*S, D)); every shard is cut into tiles_per_shard =
// ceil(S / tile_elems) tiles.  Shard s is sent at this step iff s mod K == first_sel
// (Definition 1 rewritten for a fixed step).  The shards of one residue class all
// have S elements except possibly the last of the arena, so the packed offset of
// shard s is (s / K) * S.
//
// All per-tile decisions are taken in 32-bit scalar arithmetic (S < 2^31); only
// the two final offsets are 64-bit products.  64-bit compare-and-select chains
// are avoided here on purpose: hipcc 7.2 turned `left < TILE ? left : TILE` on
// int64 into an s_cselect that read a stale SCC, so every ragged tile ran as a
// full one.
struct fixed_geom {
    int64_t S;
    uint32_t shard_len;  // S
    uint32_t last_len;   // elements of the last shard of the arena, 1..S
    uint32_t n_shards;
    int32_t K;
    int32_t first_sel;
    uint32_t tiles_per_shard;
    uint32_t sh_lo;    // first shard this launch covers (per-bucket calls start mid-arena)
    uint32_t sh_step;  // 1: every shard from sh_lo on; K: only the sent ones
};

COVAP_HD bool resolve_tile(const fixed_geom &g, uint32_t tile, uint32_t tile_elems, tile_ref &t)
{
    const uint32_t q = tile / g.tiles_per_shard;
    const uint32_t j = tile - q * g.tiles_per_shard;
    const uint32_t s = g.sh_lo + q * g.sh_step;
    const uint32_t sh_len = (s + 1u == g.n_shards) ? g.last_len : g.shard_len;
    const uint32_t in = j * tile_elems;
    if (in >= sh_len) return false;
    const uint32_t left = sh_len - in;
    t.n = (int32_t)(left < tile_elems ? left : tile_elems);
    t.off = (int64_t)s * g.S + (int64_t)in;
    t.sel = (int32_t)(s % (uint32_t)g.K) == g.first_sel;
    t.poff = (int64_t)(s / (uint32_t)g.K) * g.S + (int64_t)in;
    return true;
}

// ---- variable-length shards (median sharding) -------------------------------------
//
// The shards of a call are listed class by class (shard index mod K, then shard
// index), so the shards sent at a step -- one class -- are neighbours in the list
// whatever the step is, and the list itself does not depend on the step.  A launch
// carries up to kMaxUnits consecutive list entries ("units") in its kernel
// arguments, so no device table is ever allocated; `first` is the running tile
// count, and the tiles [sent_lo, sent_lo + n_sent) are those of the sent class.
//
// The grid does not walk the tiles in list order.  A long run of sent tiles makes
// decompress run in lock-step "generations" of long-lived waves whose last, partly
// filled generation is pure loss, so sent and unsent tiles are dealt out in blocks
// of 2^g_shift tiles (the host picks 1024, fewer for small launches) that alternate in
// proportion (measured: 18 % on the VGG-19-shaped set against sent-first order).
// Alternating workgroup by workgroup is harmful: neighbouring workgroups would then
// write streams a power of two apart.  Block j
// of the grid is a sent block iff floor((j+1) * rho / 2^32) > floor(j * rho / 2^32)
// with rho = ceil(B_s * 2^32 / (B_s + B_u)) for B_s sent and B_u unsent blocks: the
// floor counts the sent blocks before j, rises by 0 or 1 per block and reaches
// exactly B_s at j = B_s + B_u.  The last block of either kind may be partly empty;
// its surplus workgroups return at once.
constexpr int kMaxUnits = 128;
constexpr uint32_t kNoTile = 0xffffffffu;

struct table_geom {
    int64_t off[kMaxUnits];         // arena offset of each unit (vector aligned)
    int64_t poff[kMaxUnits];        // packed offset of each unit (vector aligned)
    uint32_t len[kMaxUnits];        // elements, 1..2^31-1
    uint32_t first[kMaxUnits + 1];  // first tile of each unit; unused entries hold kNoTile
    uint32_t sent_lo;               // tiles [sent_lo, sent_lo + n_sent) belong to the sent class
    uint32_t n_sent;
    uint32_t n_unsent;
    uint32_t rho;                   // see above; meaningful when mixed != 0
    uint32_t g_shift;
    uint32_t mixed;                 // 0: workgroup b takes tile b (one kind only, or too few tiles to deal out)
};

// Number of workgroups a launch with this geometry needs.
COVAP_HD uint32_t grid_of(const table_geom &g)
{
    if (!g.mixed) return g.n_sent + g.n_unsent;
    const uint32_t G = 1u << g.g_shift;
    return (((g.n_sent + G - 1u) >> g.g_shift) + ((g.n_unsent + G - 1u) >> g.g_shift)) << g.g_shift;
}

COVAP_HD uint32_t mul_hi32(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32); }

COVAP_HD bool resolve_tile(const table_geom &g, uint32_t b, uint32_t tile_elems, tile_ref &t)
{
    uint32_t tile;
    bool sel;
    if (g.mixed != 0u) {
        const uint32_t j = b >> g.g_shift, w = b & ((1u << g.g_shift) - 1u);
        const uint32_t before = mul_hi32(j, g.rho), through = mul_hi32(j + 1u, g.rho);
        sel = through != before;
        const uint32_t v = ((sel ? before : j - before) << g.g_shift) + w;  // index among the tiles of its kind
        if (v >= (sel ? g.n_sent : g.n_unsent)) return false;
        tile = sel ? g.sent_lo + v : (v < g.sent_lo ? v : v + g.n_sent);
    } else {
        tile = b;
        sel = tile - g.sent_lo < g.n_sent;  // unsigned: false below sent_lo as well
    }
    // Two-level scalar search, three dependent kernel-argument reads in all (a plain
    // binary search needs eight, and a zero-fill workgroup lives hardly longer than
    // that): eight pivots at fixed positions, then the 16 entries of one block.
    // Unused entries hold kNoTile, which no tile index reaches.
    static_assert(kMaxUnits % 16 == 0, "blocks of 16 units");
    uint32_t blk = 0;
    COVAP_UNROLL
    for (int i = 1; i < kMaxUnits / 16; ++i) blk += g.first[16 * i] <= tile ? 1u : 0u;
    const uint32_t *f = g.first + 16 * blk;
    uint32_t u = 16 * blk;
    COVAP_UNROLL
    for (int j = 1; j < 16; ++j) u += f[j] <= tile ? 1u : 0u;
    const uint32_t sh_len = g.len[u];
    const uint32_t in = (tile - g.first[u]) * tile_elems;
    if (in >= sh_len) return false;
    const uint32_t left = sh_len - in;
    t.n = (int32_t)(left < tile_elems ? left : tile_elems);
    t.off = g.off[u] + (int64_t)in;
    t.sel = sel;
    t.poff = g.poff[u] + (int64_t)in;
    return true;
}

}  // namespace covap
