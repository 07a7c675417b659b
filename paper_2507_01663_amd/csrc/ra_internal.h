// Internal interface between the C-ABI layer (ra_api.cpp) and the gfx950 kernels (ra_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ra {

constexpr int kPage = 16;           // tokens per page
constexpr int kPrefixRows = 64;     // query rows (members x heads-per-kv-head) one shared-prefix work row carries
constexpr int kMinUnitsPerWave = 8; // do not cut the page stream finer than this
constexpr int kStages = 2;          // LDS ring depth of the attention kernel (stages of two pages of K and V)

// Device pointers into the caller's workspace.  All offsets are fixed by the shape alone.
struct Workspace {
    int32_t *hdr;            // [16]: 0 total units, 1 units per wave, 2 rows, 3 prefix rows, 4 error flags
    int32_t *grp_count;      // [num_groups]      members that use the shared pass
    int32_t *grp_rowbase;    // [num_groups + 1]  first prefix row of the group (relative)
    int32_t *grp_membase;    // [num_groups + 1]  first slot of the group in members[]
    int32_t *seq_rank;       // [B]   rank inside the group, -1: not a member
    int32_t *seq_pfx_row;    // [B]   prefix row (relative) or -1
    int32_t *members;        // [B]   sequences ordered by prefix row
    int32_t *row_units;      // [2B]  pages in the row
    int32_t *row_start;      // [2B + 1] exclusive scan of row_units
    int4 *row_info;          // [2B]  suffix row b: {b, pages skipped, valid tokens after the skip, 0}
                             //       prefix row:   {group, first member slot, members, 0}
    int32_t *wave_first_row; // [waves + 1]
    float *suf_o;            // [(B*Hkv + waves)][G][D]   partial outputs (normalised)
    float *suf_lse;          // [(B*Hkv + waves)][G]      partial log2-sum-exp
    float *pfx_o;            // [(prefix_rows_max*Hkv + waves)][kPrefixRows][D]
    float *pfx_lse;          // [(prefix_rows_max*Hkv + waves)][kPrefixRows]
};

struct Launch {
    int32_t B, Hq, Hkv, D, G, num_pages, max_pages, num_groups;
    int32_t kv_fp8, share, waves, members_per_row;
    const uint16_t *q;
    const uint8_t *k_pool, *v_pool;
    int64_t stride_page_b, stride_head_b; // bytes
    int32_t stride_token_b;               // bytes
    const float *k_scale, *v_scale;
    const int32_t *block_table, *seq_lens, *seq_group, *pfx_off, *pfx_pages;
    float scale_log2;                     // softmax_scale * log2(e)
    uint16_t *out;
    float *lse;
    const void *zeros;                    // >= 16 bytes of zeros
    Workspace ws;
};

// Upper bound on prefix rows for a shape.
int prefix_rows_max(int B, int G, int num_groups);
// Carves the workspace; returns the bytes needed.  base may be null (size query).
size_t carve_workspace(Workspace &ws, void *base, int B, int Hkv, int G, int D, int num_groups, int waves);

// Number of attention waves (= workgroups) that are resident at once on the current device for head dim D.
hipError_t attention_waves(int D, int kv_fp8, int num_cus, int *waves);

hipError_t launch_validate(const Launch &a, hipStream_t s);
hipError_t launch_plan(const Launch &a, hipStream_t s);
hipError_t launch_attention(const Launch &a, hipStream_t s);
hipError_t launch_merge(const Launch &a, hipStream_t s);
hipError_t launch_gather(const Launch &a, int b, int kvh, void *k_out, void *v_out, int64_t cap, hipStream_t s);

} // namespace ra
