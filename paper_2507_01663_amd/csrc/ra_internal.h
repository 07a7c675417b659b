// Internal interface between the C-ABI layer (ra_api.cpp) and the gfx950 kernels (ra_kernels.hip, ra_prefill.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ra {

constexpr int kPage = 16;           // tokens per page
constexpr int kMinUnitsPerWave = 8; // do not cut the page stream finer than this many pages
constexpr int kMaxWaves = 4096;     // attention workgroups of a launch at most (16 per compute unit)
constexpr int kCostSuffix = 4;      // scheduling weight of a page of a sequence's own KV
constexpr int kChunkSegs = 7;       // segment records per chunk of a span's work list (plus one header record)
constexpr int kSelfListBytes = 4096; // room for the list a self-planning wave keeps (its LDS work list is at most this)
constexpr int kCostPrefix = 8;      // ... of a shared-prefix page of a bf16 pool (64 query rows per byte read: more time per page)
constexpr int kCostPrefixFp8 = 5;   // ... of an e4m3 pool (32 query rows)
constexpr int kCostItem = 16;       // ... of a segment, on top of its pages
constexpr int kCostItemPrefix = 16;    // ... of a shared-prefix row's segment (bf16 pools)
constexpr int kCostItemPrefixFp8 = 48; // ... (e4m3 pools)

// Device pointers into the caller's workspace.  All offsets are fixed by the shape alone.
struct Workspace {
    int32_t *hdr;            // [16]: 0 total cost units, 2 rows, 3 prefix rows, 4 error flags, 7 spans
    int32_t *grp_count;      // [num_groups]      members that use the shared pass
    int32_t *grp_rowbase;    // [num_groups + 1]  first prefix row of the group (relative)
    int32_t *grp_membase;    // [num_groups + 1]  first slot of the group in members[]
    int32_t *seq_rank;       // [B]   rank inside the group, -1: not a member
    int32_t *seq_pfx_row;    // [B]   prefix row or -1
    int32_t *seq_rank_in_row;// [B]   position among the members of that row
    int4 *merge_desc;        // [B*Hkv][2]  {pages, first span, last span, -} of the own row and of the prefix row
    int32_t *members;        // [B]   sequences ordered by prefix row
    int32_t *row_start;      // [2B + 1] exclusive scan of the rows' cost (per kv head); prefix rows come first
    int4 *row_tab;           // [2B]  prefix row: {index of the group's first page id, first member slot, members, pages};
                             //       sequence row: {sequence, pages skipped, tokens after the skip, pages}
    int4 *seg_rec;           // [chunks][8][2]  what each span's wave does: chunk c < spans belongs to span c; record 0 of a
                             //       chunk is {segments in the chunk (<= 7), next chunk of the span or -1}, then the segments
    float *suf_o;            // [(B*Hkv + spans)][G][D]   partial outputs (normalised); slot = item + span
    float *suf_lse;          // [(B*Hkv + spans)][G]      partial log2-sum-exp
    float *pfx_o;            // [(prefix_rows_max*Hkv + spans)][prefix_rows][D]
    float *pfx_lse;          // [(prefix_rows_max*Hkv + spans)][prefix_rows]
    int32_t *self_cnt;       // [spans]  records in the list that the wave of a span made for itself and kept, or -1
    uint8_t *self_rec;       // [spans][kSelfListBytes]  those lists (for a later call that reuses the schedule)
};

struct Launch {
    int32_t B, Hq, Hkv, D, G, num_pages, max_pages, num_groups;
    int32_t kv_fp8, share, waves, stages, cost_prefix, cost_item, cost_item_pfx;
    int32_t prefix_rows;     // query rows a shared-prefix work row carries (members x heads per kv head, at most)
    int32_t members_per_row; // = prefix_rows / G
    int32_t recip_g;         // ceil(2^16 / G): (x * recip_g) >> 16 == x / G for 0 <= x <= 64
    const int32_t *wave_cum; // [waves + 1] running sum of the workgroups' shares of the page stream, 0 .. 2^20
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
    int32_t self_plan;                    // the attention waves plan their spans themselves: no schedule kernel
    int32_t reuse_lists;                  // ... and take the lists that an earlier call's waves kept in the workspace
    Workspace ws;
};

// Prompt prefill: packed prompts, their causal attention, and where their K and V rows go in the cache.
struct PrefillLaunch {
    int32_t num_prompts, max_len, Hq, Hkv, D, G;
    int32_t num_cus;             // compute units of the device
    int32_t stay;                // prefill workgroups per die that stay and take block after block (at most one per
                                 // compute unit); 0: one workgroup per block; -1: chosen by prompt length
    const uint16_t *q, *k, *v;   // bf16 [T][Hq][D], [T][Hkv][D]
    const int32_t *cu;           // [num_prompts + 1] first token of each prompt
    float scale_log2;            // softmax_scale * log2(e)
    uint16_t *out;               // bf16 [T][Hq][D]
    float *lse;                  // [T][Hq]
    const void *zeros;           // >= 16 bytes of zeros
    // cache write (launch_prefill_write)
    int32_t kv_fp8, num_pages;
    uint8_t *k_pool, *v_pool;
    int64_t stride_page_b, stride_head_b; // bytes
    int32_t stride_token_b;               // bytes
    float *k_scale, *v_scale;
    const int32_t *page_off, *pages;      // [num_prompts + 1], [page_off[num_prompts]]
};

// Query rows of a shared-prefix work row for bf16 (0) or e4m3 (1) pools.
int prefix_rows(int kv_fp8);
// Upper bound on prefix rows for a shape.
int prefix_rows_max(int B, int G, int num_groups, int prefix_rows);
// Carves the workspace; returns the bytes needed.  base may be null (size query).
size_t carve_workspace(Workspace &ws, void *base, int B, int Hkv, int G, int D, int num_groups, int waves, int prefix_rows);

// LDS ring depth of the attention kernel and the number of its waves (= workgroups = spans of the page stream) to
// launch on the current device, for head dim D: as many as are resident at once (bf16 pools: one per SIMD; e4m3 pools:
// up to two per SIMD, as many as the ring's LDS lets in).
hipError_t attention_config(int D, int kv_fp8, int num_cus, int *stages, int *waves);
// Whether a batch's schedule tables fit in the LDS of an attention wave (then no schedule kernel is needed).
bool can_self_plan(int D, int kv_fp8, int stages, int B, int num_groups, int members_per_row);

// Streams entries * 16 KB per wave from buf (a power of two of bytes) through the attention kernel's ring, in pieces of
// `granule` bytes (1024 .. 16384, a power of two), scattered over the buffer or consecutive.
hipError_t launch_stream_probe(const void *buf, size_t buf_bytes, int granule, int scattered, int entries, int waves, hipStream_t s,
                               int chunk = 0, uint32_t tickets = 0, uint32_t *counter = nullptr, long long *clocks = nullptr);
hipError_t launch_validate(const Launch &a, hipStream_t s);
hipError_t launch_plan(const Launch &a, hipStream_t s);
hipError_t launch_attention(const Launch &a, hipStream_t s);
hipError_t launch_merge(const Launch &a, hipStream_t s);
// Writes the new K and V rows (bf16 [B][Hkv][D]) at position seq_lens[b] of every sequence; see append_kernel.
hipError_t launch_append(const Launch &a, const void *k_new, const void *v_new, hipStream_t s);
// Causal attention of the packed prompts (prefill_kernel) and the write of their K/V rows into pages.
// Once per device, before the first launch_prefill: lets the prefill kernels have the LDS they ask for.
hipError_t prefill_config();
hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s);
hipError_t launch_prefill_write(const PrefillLaunch &a, hipStream_t s);
hipError_t launch_gather(const Launch &a, int b, int kvh, void *k_out, void *v_out, int64_t cap, hipStream_t s);

} // namespace ra
