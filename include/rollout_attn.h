/*
 * rollout_attn: one decode step of attention over a paged KV cache, for a
 * batch of variable-length sequences sampled in groups that share a prompt.
 *
 * Setting.  In RL post-training the actor-rollout phase generates responses
 * auto-regressively and is memory-bound (paper Sec. 2.1.1, Sec. 2.2); with
 * GRPO several responses are sampled for one prompt (Sec. 7.1) and their
 * lengths vary widely (Sec. 7.4).  The paper schedules that phase but does
 * not define its kernels; the operation below is the textbook one its
 * inference engine performs once per layer per generated token.
 *
 * Definition.  For sequence b, query head h, G = Hq / Hkv, kv = h / G,
 * L = seq_lens[b], token t < L stored at
 *     pool[block_table[b][t / page_size]][kv][t % page_size][0:D]:
 *   s_t      = softmax_scale * <q[b,h,:], k_t>
 *   out[b,h] = sum_t softmax(s)_t * v_t           (bf16)
 *   lse[b,h] = ln sum_t exp(s_t)                  (fp32, natural log)
 * L == 0 gives out = 0 and lse = -inf.  There is no causal mask inside the
 * call: the single query token of each sequence attends to all L tokens.
 *
 * Every pointer marked "dev" is device memory of the GPU the context was
 * created on; it is owned by the caller, is only read (inputs) or written
 * (out, lse, workspace) while the enqueued work runs, and is never retained
 * after that.  The library allocates device memory only in
 * rollout_attn_create() and frees it in rollout_attn_destroy().
 * rollout_attn_decode (without RA_FLAG_VALIDATE and with timing off),
 * rollout_attn_append and rollout_attn_prefill do nothing on the stream but
 * launch kernels: no allocation, no memset, no copy, no synchronisation.  A
 * caller may therefore record them into a HIP graph and replay it; the
 * replays read whatever the buffers hold then (lengths, tables, queries).
 * No function throws or aborts; every failure is a status code, and
 * rollout_attn_last_error() describes the last one on that context.
 */
#ifndef ROLLOUT_ATTN_H
#define ROLLOUT_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROLLOUT_ATTN_ABI_VERSION 1u

typedef struct ra_ctx ra_ctx; /* opaque; one per (process, device); not thread-safe */

typedef enum {
    RA_OK = 0,
    RA_ERR_INVALID_ARG = 1,         /* null pointer, bad scalar, inconsistent shape; nothing was enqueued */
    RA_ERR_UNSUPPORTED = 2,         /* valid but not implemented (see ra_problem); nothing was enqueued */
    RA_ERR_WORKSPACE_TOO_SMALL = 3, /* nothing was enqueued */
    RA_ERR_OUT_OF_RANGE = 4,        /* device data (lengths, page ids, group hint) failed RA_FLAG_VALIDATE;
                                       the attention kernels were not enqueued */
    RA_ERR_DEVICE = 5               /* a HIP runtime call failed */
} ra_status;

typedef enum { RA_KV_BF16 = 0, RA_KV_FP8_E4M3 = 1 } ra_kv_dtype;

enum {
    RA_FLAG_VALIDATE = 1u,          /* check device-side lengths / page ids / hint first (one extra kernel + a
                                       stream synchronisation) */
    RA_FLAG_NO_PREFIX_SHARING = 2u, /* ignore the prompt-group hint (for A/B comparison) */
    RA_FLAG_REUSE_SCHEDULE = 4u     /* skip the schedule (its kernels for a large batch; for a smaller one, which the
                                       attention workgroups plan for themselves, their planning pass: each takes the
                                       list it kept) and use the schedule that the previous rollout_attn_decode call
                                       without this flag on the same context left in the same workspace.
                                       For the layers of one decode step: the schedule depends only on B, the head
                                       counts, D, max_pages_per_seq, seq_lens, seq_group, prefix_page_offsets and
                                       RA_FLAG_NO_PREFIX_SHARING, which must all be what they were in that call; q,
                                       out, lse, the pools, the scales and the page ids in block_table and
                                       prefix_pages may differ.  Nothing checks this. */
};

/*
 * One decode step.  Layouts:
 *   q, out      bf16 [B][Hq][D], contiguous.
 *   k_pool,     element (page, kv head, slot, d) at
 *   v_pool        page*kv_stride_page + kv*kv_stride_head + slot*kv_stride_token + d   (in elements),
 *               bf16, or OCP E4M3 codes (bias 7, max 448, no inf) when kv_dtype == RA_KV_FP8_E4M3.
 *               D is contiguous; every (page, head, slot) row must start on a 16-byte boundary.
 *   k_scale,    fp32 [num_pages][Hkv]; value = code * scale.  NULL unless fp8.
 *   v_scale
 *   block_table int32 [B][max_pages_per_seq]; entry i of row b is the page holding tokens
 *               [i*page_size, (i+1)*page_size) of sequence b, shared prompt pages included.  Entries at or
 *               past ceil(L/page_size) are never read.  Slots at or past L in the last page are read but
 *               never used (they may hold NaN).
 *   seq_lens    int32 [B], total KV tokens, 0 <= L <= max_pages_per_seq * page_size.
 * Optional prompt-group hint (num_groups == 0 disables it).  It is a promise that changes speed, not
 * results: the first page_size * n_g tokens of every member of group g live in the n_g pages
 *   prefix_pages[prefix_page_offsets[g] .. prefix_page_offsets[g+1])
 * and the member's own block_table row starts with the same ids.  Those pages are then read once per
 * group instead of once per member.
 *   seq_group           int32 [B], group id in [0, num_groups) or -1 (no group).
 *   prefix_page_offsets int32 [num_groups + 1], non-decreasing, starts at 0.
 *   prefix_pages        int32 [prefix_page_offsets[num_groups]].
 * A member shorter than its group's prefix is handled as if it had no group.
 * Supported: page_size == 16; D in {64, 128}; Hq % Hkv == 0 and Hq / Hkv <= 16.
 */
typedef struct {
    int32_t B, Hq, Hkv, D, page_size;
    int32_t num_pages, max_pages_per_seq;
    const void *q;           /* dev */
    const void *k_pool;      /* dev */
    const void *v_pool;      /* dev */
    int64_t kv_stride_page, kv_stride_head, kv_stride_token; /* in elements */
    int32_t kv_dtype;        /* ra_kv_dtype */
    const float *k_scale;    /* dev or NULL */
    const float *v_scale;    /* dev or NULL */
    const int32_t *block_table; /* dev */
    const int32_t *seq_lens;    /* dev */
    int32_t num_groups;
    const int32_t *seq_group;           /* dev or NULL when num_groups == 0 */
    const int32_t *prefix_page_offsets; /* dev or NULL when num_groups == 0 */
    const int32_t *prefix_pages;        /* dev or NULL when num_groups == 0 */
    float softmax_scale;
    void *out;               /* dev, bf16 [B][Hq][D] */
    float *lse;              /* dev, fp32 [B][Hq] */
    uint32_t flags;
} ra_problem;

/* ROLLOUT_ATTN_ABI_VERSION of the library that was loaded. */
uint32_t rollout_attn_abi_version(void);

/* Creates a context on the given HIP device: queries the device and allocates a few hundred bytes of device
 * memory that the context keeps.  *ctx is NULL on failure.  RA_ERR_DEVICE when the device cannot be used.
 *
 * Tuning knobs, read from the environment here and nowhere else (none changes a result beyond rounding; values
 * out of range are ignored):
 *   ROLLOUT_ATTN_XCD_WEIGHTS=a,..,h the share of the work each of the eight dies' workgroups get, per mille of the
 *                                   mean (700..1400; default: a built-in table, the odd dies about a tenth less
 *                                   for bf16 pools and a twentieth less for e4m3 pools)
 *   ROLLOUT_ATTN_STAGES=2|3, ROLLOUT_ATTN_FP8_STAGES=2|3   depth of the LDS ring for bf16 / e4m3 pools
 *   ROLLOUT_ATTN_WAVES_PER_CU=1..16 attention workgroups per compute unit (default: as many as are resident)
 *   ROLLOUT_ATTN_COST_PREFIX=1..16, ROLLOUT_ATTN_COST_ITEM=0..256   scheduling weights of a shared-prefix page and
 *                                   of a segment (a page of a sequence's own weighs 4)
 *   ROLLOUT_ATTN_COST_ITEM_PREFIX=0..1024   ... of a segment of shared-prefix pages, whose partial result is
 *                                   written in mid-stream (default: 16 for bf16 pools, 48 for e4m3 pools)
 *   ROLLOUT_ATTN_SELF_PLAN=0        always launch the schedule kernels (default: batches of up to 512 sequences and
 *                                   511 groups are scheduled by the attention workgroups themselves, each for its own
 *                                   share of the work, which saves a kernel; the schedule is the same either way)
 *   ROLLOUT_ATTN_PREFILL_WGS_PER_DIE=0..64   prefill: one workgroup per block of 256 query rows (0), or that many
 *                                   per die (at most one per compute unit) that stay and take block after block,
 *                                   loading the next one's inputs under the current one's last keys; default: one
 *                                   per compute unit for prompts of up to 512 tokens, one per block for longer ones
 *   ROLLOUT_ATTN_VERBOSE            print the die weights to stderr */
ra_status rollout_attn_create(ra_ctx **ctx, int device_ordinal);

/* Frees the context's device memory.  NULL is accepted.  Work already enqueued must have finished. */
void rollout_attn_destroy(ra_ctx *ctx);

/* Text of the last failure on ctx (library-owned, valid until the next call on ctx).  With ctx == NULL,
 * the text of the last failure of a call that had no context (create, check_problem). */
const char *rollout_attn_last_error(const ra_ctx *ctx);

/* Host-only check of the scalars, strides and pointers of a problem (device data is not read).  Returns
 * what rollout_attn_decode would return for them before touching the device.  msg (may be NULL) receives
 * a NUL-terminated explanation of at most msg_len bytes. */
ra_status rollout_attn_check_problem(const ra_problem *problem, char *msg, size_t msg_len);

/* Bytes of device workspace rollout_attn_decode needs for problems of this shape (only B, Hq, Hkv, D,
 * page_size, num_groups are read).  ctx may be NULL: the size for a 256-compute-unit device is returned. */
ra_status rollout_attn_workspace_size(const ra_ctx *ctx, const ra_problem *shape_only, size_t *bytes);

/* Enqueues the whole step (schedule, attention over shared prompt pages and over each sequence's own
 * pages, log-sum-exp merge: two kernels for batches of up to 512 sequences, where the attention workgroups schedule
 * themselves, else three or four) on hip_stream (a hipStream_t, NULL = default stream) and returns without
 * waiting; out and lse are valid once the stream has reached that point.  workspace is dev memory of at
 * least rollout_attn_workspace_size() bytes, 256-byte aligned, contents irrelevant on entry and undefined
 * afterwards; calls that overlap in time need distinct workspaces.  Results are deterministic: the same
 * inputs give byte-identical outputs. */
ra_status rollout_attn_decode(ra_ctx *ctx, const ra_problem *problem, void *workspace, size_t workspace_bytes,
                              void *hip_stream);

/* rollout_attn_decode for callers that cannot allocate device memory or have none to spare for a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same step with the same
 * kernels and byte-identical results, on a workspace that is built into the library, a fixed 64 MiB array in
 * device memory that every GPU the library is loaded on holds until the process ends.  Neither this call nor
 * anything it launches allocates or frees memory.  RA_ERR_WORKSPACE_TOO_SMALL when the problem's shape needs more
 * than 64 MiB (rollout_attn_workspace_size says how much a shape needs; the 7B-shaped batch of 256 sequences needs
 * about 51 MiB); nothing is enqueued then.  All calls on one GPU share the one array, whatever their context or
 * stream: calls that overlap in time on one GPU race, so order them on one stream or with events.  RA_FLAG_REUSE_SCHEDULE
 * refers to the schedule the previous call on the GPU left in the array.  Everything else is as for
 * rollout_attn_decode. */
ra_status rollout_attn_decode_static(ra_ctx *ctx, const ra_problem *problem, void *hip_stream);

/* Copies the stored K and V elements of sequence b, KV head kv_head, in logical token order, to k_out and
 * v_out (dev, [L_b][D] raw elements: 2 bytes each for bf16, 1 for e4m3), through the same block-table
 * arithmetic as the attention kernels.  capacity_tokens is the room in k_out / v_out; a longer sequence is
 * truncated to it.  Enqueued on hip_stream. */
ra_status rollout_attn_debug_gather(ra_ctx *ctx, const ra_problem *problem, int32_t b, int32_t kv_head,
                                    void *k_out, void *v_out, int64_t capacity_tokens, void *hip_stream);

/* Where rollout_attn_debug_schedule left the schedule in the workspace (byte offsets from its start). */
typedef struct {
    int64_t header_offset;      /* int32[16]: [0] cost units of the stream, [2] work rows, [3] of which shared-prefix
                                   rows, [7] spans */
    int64_t work_list_offset;   /* chunks of 8 records of 8 int32; chunk c < spans starts span c's list; record 0 of a
                                   chunk is {segments in the chunk, next chunk or -1}; a segment record is {index of the
                                   row's first page id in its table, first page, end page, token limit, kv head |
                                   shared << 16, sequence or first member slot, query rows, partial slot} */
    int64_t merge_desc_offset;  /* per (sequence, kv head) two int32[4]: {pages, first span, last span, 0} of the
                                   sequence's own pages and of its group's shared pages (first > last: none) */
    int32_t waves;              /* resident attention waves = static spans */
    int32_t segments_per_chunk;
} ra_schedule_info;

/* Runs only the schedule kernels of rollout_attn_decode (same arguments) and reports where their results lie in
 * the workspace, for tests of the schedule's invariants: every page of every (work row, kv head) item belongs
 * to exactly one span's list, in order, and the merge descriptors name exactly the spans that hold them. */
ra_status rollout_attn_debug_schedule(ra_ctx *ctx, const ra_problem *problem, void *workspace, size_t workspace_bytes,
                                      void *hip_stream, ra_schedule_info *info);

/* KV append: writes one new token per sequence into the paged cache, the step that precedes the attention
 * of a decode iteration (auto-regressive generation: paper Sec. 2.1.1; the paper does not define the write,
 * this header does).  For every sequence b the token goes to position L = seq_lens[b], the length BEFORE the
 * append: page block_table[b][L / page_size], slot L % page_size, every kv head.  seq_lens is not modified
 * (the caller adds one afterwards).  k_new, v_new: dev, bf16 [B][Hkv][D], contiguous, 4-byte aligned.
 * `problem` must be valid as for rollout_attn_decode; of its device data only block_table and seq_lens are
 * read, and the pools (for e4m3 also k_scale and v_scale) are WRITTEN although the struct declares them
 * const.  No two sequences may append into the same page (shared prompt pages are whole pages, so a new
 * token never lands in one).  A sequence whose length is negative or not below max_pages_per_seq * page_size,
 * or whose page id is not in [0, num_pages), is skipped.
 *   bf16 pools: the 16-bit patterns are copied.
 *   e4m3 pools, per (page, kv head), K and V alike, in IEEE binary32 with round-to-nearest-even:
 *     a = max_d |x_d| of the new row;
 *     slot 0 (a fresh page): scale = a > 0 ? a / 448 : 1;
 *     slot s > 0: if a <= scale * 448 the page keeps its scale, else scale' = a / 448 and every stored
 *       slot j < s is re-quantised, code = enc((dec(code) * scale) / scale');
 *     the new row is stored as enc(x_d / scale); enc rounds to the nearest E4M3 value, ties to the even code,
 *     saturating at +-448.
 * Enqueued on hip_stream; returns without waiting. */
ra_status rollout_attn_append(ra_ctx *ctx, const ra_problem *problem, const void *k_new, const void *v_new,
                              void *hip_stream);

/*
 * Prompt prefill: the step before the first decode step.  The prompts of a batch (one per prompt group when
 * several responses are sampled per prompt: paper Sec. 7.1) are packed back to back; every prompt token attends
 * causally to its own prompt, and the prompts' K and V rows are written into the pages that the group's
 * members then share.  The paper runs this inside its inference engine and does not define it (Sec. 2.1.1);
 * this header does.  Prompt g holds tokens [cu_seqlens[g], cu_seqlens[g+1]) of the packed arrays; for its token
 * i (0-based inside the prompt), head h, kv = h / (Hq / Hkv):
 *     s_j      = softmax_scale * <q[i,h,:], k[j,kv,:]>,  j = 0 .. i
 *     out[i,h] = sum_j softmax(s)_j * v[j,kv,:]          (bf16)
 *     lse[i,h] = ln sum_j exp(s_j)                       (fp32, natural log)
 * Layouts: q, out bf16 [T][Hq][D]; k, v bf16 [T][Hkv][D]; lse fp32 [T][Hq]; all contiguous, 16-byte aligned,
 * T = total_tokens = cu_seqlens[num_prompts].  cu_seqlens: dev int32 [num_prompts + 1], starts at 0,
 * non-decreasing.  max_prompt_len is a HOST-side upper bound of every prompt's length (the launch is sized by
 * it; a prompt's tokens at or past it may be left unprocessed, in whole blocks of query rows and whole pages).
 * Cache write (k_pool != NULL): token i of prompt g goes to page pages[page_offsets[g] + i / page_size], slot
 * i % page_size, every kv head, of pools laid out as in ra_problem (same strides, kv_dtype, scales); a prompt
 * with more tokens than its pages hold has the rest left unwritten, and so has a page id outside
 * [0, num_pages).  No page may be listed twice.  bf16 pools take the bit patterns.  e4m3 pools are quantised
 * one (page, kv head) at a time in IEEE binary32: scale = (largest |x| among the rows written to the page) /
 * 448, or 1 when that is 0; code = nearest E4M3 of x / scale, ties to the even code; slots of a last, partly
 * filled page that receive no token are left as they were.
 * Supported: page_size == 16; D in {64, 128}; Hq % Hkv == 0.  total_tokens * Hq * D < 2^40.
 */
typedef struct {
    int32_t num_prompts, total_tokens, max_prompt_len;
    int32_t Hq, Hkv, D;
    const void *q;               /* dev */
    const void *k;               /* dev */
    const void *v;               /* dev */
    const int32_t *cu_seqlens;   /* dev */
    float softmax_scale;
    void *out;                   /* dev */
    float *lse;                  /* dev */
    /* cache write; k_pool == NULL: none, and the fields below are not read */
    void *k_pool;                /* dev or NULL */
    void *v_pool;                /* dev */
    int32_t page_size, num_pages;
    int64_t kv_stride_page, kv_stride_head, kv_stride_token; /* in elements */
    int32_t kv_dtype;            /* ra_kv_dtype */
    float *k_scale;              /* dev, fp32 [num_pages][Hkv]; NULL unless fp8 */
    float *v_scale;
    const int32_t *page_offsets; /* dev int32 [num_prompts + 1] */
    const int32_t *pages;        /* dev int32 [page_offsets[num_prompts]] */
} ra_prefill;

/* Host-only check of the scalars, strides and pointers of a prefill (device data is not read): what
 * rollout_attn_prefill would return for them before touching the device.  msg (may be NULL) receives a
 * NUL-terminated explanation of at most msg_len bytes. */
ra_status rollout_attn_check_prefill(const ra_prefill *prefill, char *msg, size_t msg_len);

/* Enqueues the cache write (if asked for) and the causal attention of the packed prompts on hip_stream and
 * returns without waiting.  Needs no workspace.  Deterministic.  RA_ERR_INVALID_ARG / RA_ERR_UNSUPPORTED as
 * for rollout_attn_decode; nothing is enqueued then. */
ra_status rollout_attn_prefill(ra_ctx *ctx, const ra_prefill *prefill, void *hip_stream);

/* Token-balanced dispatch, on the host (no device is touched, no context is needed): deals n items with
 * weights[i] >= 0 (say, the KV tokens of prompt group i) to k parts (data-parallel ranks, GPUs) so that the
 * parts' totals are close.  The paper balances its workers' tokens this way, as one-dimensional bin packing
 * solved with the Karmarkar-Karp algorithm, with equal sample counts for data parallelism and without that
 * constraint for pipeline stages (Sec. 4.4).  This is the k-way largest differencing method: every item
 * starts as a partial solution of k sets (itself and k-1 empty ones); the two partial solutions with the
 * largest spread (largest minus smallest set total) are merged, largest set with smallest, until one is left.
 * equal_count != 0 starts instead from groups of k consecutive items of the list sorted by decreasing weight,
 * one item per set, so that every part ends with floor(n/k) or ceil(n/k) items.  Ties are broken by item
 * index and creation order, so the result is unique: part[i] in [0, k), parts numbered by decreasing total;
 * part_sums (may be NULL) receives the k totals.  weights, part, part_sums: HOST memory, caller-owned.
 * RA_ERR_INVALID_ARG for n < 0, k < 1, a negative weight or a missing array; RA_ERR_DEVICE when host memory
 * runs out. */
ra_status rollout_attn_balance(const int64_t *weights, int64_t n, int32_t k, int32_t equal_count, int32_t *part,
                               int64_t *part_sums);

/* The attention kernel is launched as one single-wave workgroup per resident slot of the device, and workgroup c
 * streams the c-th share of the batch's pages.  The workgroups do not all stream equally fast: the accelerator dies
 * get different shares of the memory bandwidth and so do the compute units inside a die, in a pattern that repeats
 * from launch to launch.  These two calls let a caller tell the schedule: rollout_attn_wave_count says how many
 * workgroups the launch for (kv_dtype, head_dim) has, rollout_attn_set_wave_weights sets their shares (weights: HOST
 * int32 [n], per mille of the mean, clamped to 700..1400; n must equal the wave count).  Default: a fixed share per
 * die.  The weights only move work between workgroups (paper Sec. 4.4 balances tokens between workers the same way);
 * results stay within rounding of each other, and identical for identical weights.  Copies to the device
 * synchronously: call it while no work of the context is in flight. */
ra_status rollout_attn_wave_count(const ra_ctx *ctx, int32_t kv_dtype, int32_t head_dim, int32_t *waves);
ra_status rollout_attn_set_wave_weights(ra_ctx *ctx, int32_t kv_dtype, int32_t head_dim, const int32_t *weights, int32_t n);

/* Streaming probe for benchmarks: what the memory system delivers to the attention kernel's access pattern when no
 * arithmetic is done (the decode step is memory-bound, paper Sec. 2.1.1, so this is the practical ceiling its achieved
 * bandwidth is judged against, beside the published peak).  Launches the attention kernel's grid (one wave per
 * workgroup, all resident) with its LDS ring of 16 KB entries fed by direct global-to-LDS loads; every wave reads
 * entries_per_wave entries, each as 16384 / granule_bytes pieces of granule_bytes (a power of two, 1024..16384; 4096
 * is the K or V tile of one page and head at head dim 128 in bf16), each piece from a place of its own: a fixed
 * permutation of the buffer's granules when bit 0 of scattered is set, consecutive granules (the grid sweeps the
 * buffer, wrapping around) otherwise.  The loads carry the non-temporal hint, as the attention kernel's page loads do
 * (a decode step reads every page once); with bit 1 of scattered set they are ordinary loads, for comparison.
 * buf: dev, read only, 16-byte aligned, buf_bytes a power of two >= 16384.  *bytes_read (may be
 * NULL) receives the bytes the launch reads.  Enqueued on hip_stream; the caller times it. */
ra_status rollout_attn_debug_stream(ra_ctx *ctx, const void *buf, size_t buf_bytes, int32_t granule_bytes, int32_t scattered,
                                    int32_t entries_per_wave, void *hip_stream, size_t *bytes_read);

/* The same probe (4096-byte pieces, scattered) with the end of the stream handed out at run time: every wave
 * streams static_entries entries of its own, then the waves draw tickets from a counter in the context and a
 * ticket is the next chunk_entries entries of what is left of waves * entries_per_wave, until none is left.  For
 * benchmarks that ask whether evening out the waves' end times that way would buy anything over the static split of
 * the page stream that the attention kernel uses (paper Sec. 4.4 balances statically too); nothing else calls it.
 * 0 <= static_entries < entries_per_wave <= 65536, chunk_entries in 1..1024; buf as above.  Launches that use the
 * ticket counter of one context must not overlap.  Enqueued on hip_stream; the caller times it. */
ra_status rollout_attn_debug_stream_tail(ra_ctx *ctx, const void *buf, size_t buf_bytes, int32_t entries_per_wave,
                                         int32_t static_entries, int32_t chunk_entries, void *hip_stream, size_t *bytes_read);

/* Per-kernel timing for benchmarks.  While enabled, rollout_attn_decode records HIP events on its stream
 * around its three phases (schedule, attention, merge); rollout_attn_get_timing waits for the events of the
 * most recent decode call and returns the three durations in milliseconds (schedule: 0 when that call launched
 * no schedule kernel, because its attention workgroups planned their spans themselves or the schedule was
 * reused; the attention phase then starts at the call's first event).  Off by default: the events cost
 * a little time between kernels.  The numbers are measurements, not part of the result (the decode step is
 * memory-bound, paper Sec. 2.1.1, so the attention phase is the one to watch). */
ra_status rollout_attn_set_timing(ra_ctx *ctx, int enable);
ra_status rollout_attn_get_timing(ra_ctx *ctx, float phase_ms[3]);

#ifdef __cplusplus
}
#endif
#endif /* ROLLOUT_ATTN_H */
