// Internal: the plan object behind covap_plan_t and helpers shared by the
// library's translation units.  Not part of the public ABI.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "covap.h"

struct covap_shard_rec {
    int64_t off;         // arena offset of the shard's first element (vector aligned)
    int64_t len;         // elements
    int64_t packed_off;  // offset in the packed layout of any step that sends it
    int32_t bucket;
};

struct covap_bucket_rec {
    int32_t sh_lo, sh_hi;                 // shard range [lo, hi)
    std::vector<int64_t> packed_base;     // [K]: by residue r = step mod K
    std::vector<int64_t> packed_elems;    // [K]
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
    std::vector<int64_t> packed_total;    // [K]: by residue r = step mod K
    int64_t packed_max;
    bool uniform;                         // every shard but the last has opts.shard_elems
};

namespace covap {

// Records msg as the calling thread's last error and returns st.
covap_status_t fail(covap_status_t st, const char *msg);  // no allocation: hot-path calls use this form
covap_status_t fail(covap_status_t st, const std::string &msg);
void clear_error();

// Residue class sent at `step`: shards with s mod K == first_selected(step).
inline int32_t first_selected(uint64_t step, int32_t K)
{
    return (int32_t)(((uint64_t)K - step % (uint64_t)K) % (uint64_t)K);
}

// Resolves (plan, step, bucket) into a shard range and the packed range the
// call touches.  Returns COVAP_OK or records an error.
struct call_range {
    int32_t sh_lo, sh_hi;
    int64_t packed_base, packed_elems;
    int32_t first_sel;  // residue class sent at this step
};
covap_status_t resolve(const covap_plan_s *plan, uint64_t step, int32_t bucket, call_range *out);

struct tuning {
    int compress_threads = 64;     // workgroup size: 64, 256
    int compress_unroll = 1;       // 16-byte vectors per thread per tile: 1, 2, 4
    int decompress_threads = 64;   // workgroup size: 64, 256
    int decompress_tile = 1;       // 16-byte vectors per thread per tile: 1, 2, 4
    int decompress_unroll = 1;     // payload rows loaded before they are summed: 1, 2, 4
    int nontemporal = 1;           // 0 = plain loads/stores, 1 = streaming hints
    // Unused LDS reserved per decompress workgroup, in bytes: 0, 6144 or 8192.  With one-wave
    // workgroups 6144 caps a SIMD at 7 waves instead of 8 (8192: 6); a little less data in
    // flight keeps the DRAM access pattern tighter (+1.5..3 % measured).
    int decompress_lds_pad = 6144;
    int topk_pass1_waves = 4;      // waves that share a 1024-element tile in top-k pass 1: 1, 2, 4
    int topk_pass1_lds_pad = 0;    // unused LDS per pass-1 workgroup, bytes: 0, 6144, 8192, 24576
};
tuning &tune();

}  // namespace covap
