// Internal: the plan object behind covap_plan_t and helpers shared by the
// library's translation units.  Not part of the public ABI.
#pragma once

#include <atomic>
#include <cstdint>
#include <vector>

#include "covap.h"
#include "geom.h"

struct covap_shard_rec {
    int64_t off;         // arena offset of the shard's first element (vector aligned)
    int64_t len;         // elements
    int64_t packed_off;  // offset in the packed layout of any step that sends it
    int32_t bucket;
};

struct covap_bucket_rec {
    int32_t sh_lo, sh_hi;  // shard range [lo, hi)
};

// Variable-length shards only: the shards listed class by class (shard index mod K,
// then shard index), once over the whole arena and once bucket by bucket (bucket b's
// list occupies positions [sh_lo, sh_hi) of the second), as the arrays a launch
// copies into its kernel arguments.  Neither depends on the step.
struct covap_unit_list {
    std::vector<int64_t> off, poff;
    std::vector<uint32_t> len;
    // running tile count over the list for every tile size a kernel can have,
    // 2^kTileLog2Min .. 2^kTileLog2Max elements: tiles[j][i] = tiles of units [0, i)
    std::vector<uint32_t> tiles[6];
};

struct covap_plan_s {
    covap_plan_opts_t opts;
    int32_t K;
    int32_t elems_per_vec;                // 4 for fp32, 8 for bf16 (16-byte vectors)
    int32_t align_elems;                  // alignment unit of shard starts, in the arena and in the packed layout
    int64_t total_elems;                  // arena size D
    std::vector<int64_t> tensor_off;
    std::vector<covap_shard_rec> shards;
    std::vector<covap_bucket_rec> buckets;
    int64_t packed_max;                   // largest whole-arena payload over the steps
    bool uniform;                         // every shard but the last has opts.shard_elems
    covap_unit_list by_arena, by_bucket;  // filled when !uniform
};

namespace covap {

constexpr int kTileLog2Min = 8, kTileLog2Max = 13;  // 64 threads x 4 elements .. 256 threads x 8 elements x 4

// Records msg as the calling thread's last error and returns st.  Never allocates.
covap_status_t fail(covap_status_t st, const char *msg);
covap_status_t fail(covap_status_t st, const char *who, const char *msg);  // "who: msg"
void clear_error();

// Residue class sent at `step`: shards with s mod K == first_selected(step).
inline int32_t first_selected(uint64_t step, int32_t K)
{
    return (int32_t)(((uint64_t)K - step % (uint64_t)K) % (uint64_t)K);
}

// Resolves (plan, step, bucket) into a shard range and the packed range the
// call touches.  Returns COVAP_OK or records an error.  O(1).
struct call_range {
    int32_t sh_lo, sh_hi;
    int64_t packed_base, packed_elems;
    int32_t first_sel;  // residue class sent at this step
    int32_t bucket;     // -1: the whole arena
};
covap_status_t resolve(const covap_plan_s *plan, uint64_t step, int32_t bucket, call_range *out);

// Launch geometry of a call.  A call over fixed-size shards is one launch; one over
// variable-length shards needs one launch per kMaxUnits list entries.
//   tile_elems  elements per workgroup, a power of two in 2^kTileLog2Min..2^kTileLog2Max
//   sent_only   cover only the shards sent at this step
// fixed_launch: *grid = 0 means nothing to launch.  table_launches: how many launches
// the call needs; table_launch fills the i-th (grid_of(*g) may be 0: skip it).
fixed_geom fixed_launch(const covap_plan_s *plan, const call_range &cr, uint32_t tile_elems, bool sent_only,
                        uint32_t *grid);
int32_t table_launches(const covap_plan_s *plan, const call_range &cr, bool sent_only);
void table_launch(const covap_plan_s *plan, const call_range &cr, uint32_t tile_elems, bool sent_only,
                  int32_t i, table_geom *g);

// Launch-shape knobs (covap_tune_set), as one call sees them: tune() loads every knob
// once, atomically, so a sweep in another thread can neither tear a value nor change
// the shape of a call between two of its launches.
struct tuning {
    int compress_threads;     // workgroup size: 64, 256
    int compress_unroll;      // 16-byte vectors per thread per tile: 1, 2, 4
    int decompress_threads;   // workgroup size: 64, 256
    int decompress_tile;      // 16-byte vectors per thread per tile: 1, 2, 4
    int decompress_unroll;    // payload rows loaded before they are summed: 1, 2, 4
    int nontemporal;          // 0 = plain loads/stores, 1 = streaming hints
    // Unused LDS reserved per decompress workgroup, in bytes: 0, 6144, 8192, 24576, 32768 or
    // 49152.  With one-wave workgroups 6144 caps a SIMD at 7 waves instead of 8 (8192: 6); a
    // little less data in flight keeps the DRAM access pattern tighter (+1.5..3 % measured).
    // The large values are for 256-thread workgroups (32768: five per compute unit).
    int decompress_lds_pad;
    // True while decompress_threads, decompress_tile and decompress_lds_pad have never been
    // set: decompress may then pick the workgroup shape from the call (few rows: store-bound).
    bool decompress_shape_unset;
    int topk_pass1_waves;     // waves that share a 1024-element tile in top-k pass 1: 1, 2, 4
    int topk_pass1_lds_pad;   // unused LDS per pass-1 workgroup, bytes: 0, 6144, 8192, 24576
};
tuning tune();

}  // namespace covap
