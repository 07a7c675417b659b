// C-ABI of rollout_attn (see include/rollout_attn.h): argument checks, workspace carving, kernel sequencing.
#include "../../include/rollout_attn.h"
#include "ra_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

// Workspace of rollout_attn_decode_static: device memory that exists from the moment the library is loaded, one
// copy per GPU.  The name is a host-side handle; the device address is asked for once per context (= per device).
constexpr size_t kScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct ra_ctx {
    int device;
    void *scratch_ptr; // device address of `scratch` on this context's device
    int num_cus;
    int waves[2][2];  // resident attention waves, [e4m3 KV][D == 128]
    int stages[2][2]; // LDS ring depth, same indices
    int cost_prefix[2]; // scheduling weight of a shared-prefix page, [e4m3 KV]
    int cost_item;   // ... of a segment, on top of its pages
    int cost_item_pfx[2]; // ... of a shared-prefix row's segment (bf16, e4m3 pools)
    int xcd_w[8];              // default share of the page stream per accelerator die, per mille of the mean
    int32_t *wave_cum[2][2];   // device: running sums of the workgroups' shares, [e4m3 KV][D == 128], kMaxWaves + 1 each
    uint32_t *tickets;         // device: the streaming probe's ticket counter (cleared by every launch that uses it)
    int prefill_stay;          // -1: the prefill launch chooses by prompt length; else ROLLOUT_ATTN_PREFILL_WGS_PER_DIE
    void *zeros;  // 256 bytes of zeros on the device
    int self_plan; // attention waves may plan their spans themselves (no schedule kernel)
    int32_t *host_flags; // pinned, for RA_FLAG_VALIDATE
    int timing;          // record events around the phases
    int timed;           // a decode call has recorded them (2: with a schedule launch between the first two)
    hipEvent_t ev[4];
    char err[512];
};

namespace {

thread_local char g_err[512] = "";

void set_err(ra_ctx *ctx, const char *fmt, ...)
{
    char *dst = ctx ? ctx->err : g_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
}

ra_status check(const ra_problem *p, char *msg, size_t n)
{
    auto fail = [&](ra_status st, const char *fmt, ...) {
        if (msg && n) {
            va_list ap;
            va_start(ap, fmt);
            vsnprintf(msg, n, fmt, ap);
            va_end(ap);
        }
        return st;
    };
    if (msg && n) msg[0] = 0;
    if (!p) return fail(RA_ERR_INVALID_ARG, "problem is NULL");
    if (p->B < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->D <= 0 || p->page_size <= 0 || p->num_pages < 0 ||
        p->max_pages_per_seq < 0 || p->num_groups < 0)
        return fail(RA_ERR_INVALID_ARG, "negative or zero dimension (B=%d Hq=%d Hkv=%d D=%d page_size=%d num_pages=%d "
                                        "max_pages_per_seq=%d num_groups=%d)",
                    p->B, p->Hq, p->Hkv, p->D, p->page_size, p->num_pages, p->max_pages_per_seq, p->num_groups);
    if (p->Hq % p->Hkv) return fail(RA_ERR_INVALID_ARG, "Hq=%d is not a multiple of Hkv=%d", p->Hq, p->Hkv);
    if (p->kv_dtype != RA_KV_BF16 && p->kv_dtype != RA_KV_FP8_E4M3)
        return fail(RA_ERR_INVALID_ARG, "kv_dtype=%d is not a ra_kv_dtype", p->kv_dtype);
    if (p->flags & ~(uint32_t)(RA_FLAG_VALIDATE | RA_FLAG_NO_PREFIX_SHARING | RA_FLAG_REUSE_SCHEDULE))
        return fail(RA_ERR_INVALID_ARG, "unknown bits in flags=0x%x", p->flags);
    if (!std::isfinite(p->softmax_scale)) return fail(RA_ERR_INVALID_ARG, "softmax_scale is not finite");
    if (p->page_size != 16) return fail(RA_ERR_UNSUPPORTED, "page_size=%d (only 16 is supported)", p->page_size);
    if (p->D != 64 && p->D != 128) return fail(RA_ERR_UNSUPPORTED, "D=%d (only 64 and 128 are supported)", p->D);
    if (p->Hq / p->Hkv > 16) return fail(RA_ERR_UNSUPPORTED, "Hq/Hkv=%d (at most 16 is supported)", p->Hq / p->Hkv);
    // 32-bit indices into the block table, and a schedule whose cost stream (at most 16 units per page and kv head,
    // 256 per sequence and kv head, twice) stays below 2^31 units
    if ((int64_t)p->B * p->Hq > (int64_t)1 << 30 || (int64_t)p->B * p->max_pages_per_seq >= (int64_t)1 << 31 ||
        (int64_t)p->Hkv * p->B * (512 + 16 * (int64_t)p->max_pages_per_seq) >= (int64_t)1 << 31)
        return fail(RA_ERR_UNSUPPORTED, "batch too large");
    if (p->B == 0) return RA_OK;
    if (!p->q || !p->k_pool || !p->v_pool || !p->block_table || !p->seq_lens || !p->out || !p->lse)
        return fail(RA_ERR_INVALID_ARG, "a required pointer (q, k_pool, v_pool, block_table, seq_lens, out, lse) is NULL");
    const int es = p->kv_dtype == RA_KV_FP8_E4M3 ? 1 : 2;
    if (p->kv_stride_token < p->D || p->kv_stride_head < 0 || p->kv_stride_page < 0)
        return fail(RA_ERR_INVALID_ARG, "kv strides must be non-negative and kv_stride_token >= D");
    if ((p->kv_stride_token * es) % 16 || (p->kv_stride_head * es) % 16 || (p->kv_stride_page * es) % 16)
        return fail(RA_ERR_INVALID_ARG, "kv strides must be multiples of 16 bytes");
    if (p->kv_stride_token * es * 16 > INT32_MAX)
        return fail(RA_ERR_UNSUPPORTED, "kv_stride_token too large");
    if (((uintptr_t)p->k_pool | (uintptr_t)p->v_pool | (uintptr_t)p->q | (uintptr_t)p->out) % 16)
        return fail(RA_ERR_INVALID_ARG, "q, out, k_pool and v_pool must be 16-byte aligned");
    if (p->kv_dtype == RA_KV_FP8_E4M3 && (!p->k_scale || !p->v_scale))
        return fail(RA_ERR_INVALID_ARG, "fp8 KV needs k_scale and v_scale");
    if (p->num_groups > 0 && (!p->seq_group || !p->prefix_page_offsets || !p->prefix_pages))
        return fail(RA_ERR_INVALID_ARG, "num_groups > 0 needs seq_group, prefix_page_offsets and prefix_pages");
    return RA_OK;
}

void fill_launch(ra::Launch &a, const ra_ctx *ctx, const ra_problem *p)
{
    memset(&a, 0, sizeof a);
    const int es = p->kv_dtype == RA_KV_FP8_E4M3 ? 1 : 2;
    a.B = p->B; a.Hq = p->Hq; a.Hkv = p->Hkv; a.D = p->D; a.G = p->Hq / p->Hkv;
    a.num_pages = p->num_pages; a.max_pages = p->max_pages_per_seq; a.num_groups = p->num_groups;
    a.kv_fp8 = p->kv_dtype == RA_KV_FP8_E4M3;
    a.share = p->num_groups > 0 && !(p->flags & RA_FLAG_NO_PREFIX_SHARING);
    a.waves = ctx ? ctx->waves[a.kv_fp8][p->D == 128] : 2048;
    a.stages = ctx ? ctx->stages[a.kv_fp8][p->D == 128] : 4;
    a.prefix_rows = ra::prefix_rows(a.kv_fp8);
    a.members_per_row = a.prefix_rows / a.G;
    a.recip_g = (65536 + a.G - 1) / a.G;
    a.cost_prefix = ctx ? ctx->cost_prefix[a.kv_fp8] : (a.kv_fp8 ? ra::kCostPrefixFp8 : ra::kCostPrefix);
    a.cost_item = ctx ? ctx->cost_item : ra::kCostItem;
    a.cost_item_pfx = ctx ? ctx->cost_item_pfx[a.kv_fp8] : (a.kv_fp8 ? ra::kCostItemPrefixFp8 : ra::kCostItemPrefix);
    a.wave_cum = ctx ? ctx->wave_cum[a.kv_fp8][p->D == 128] : nullptr;
    a.q = (const uint16_t *)p->q;
    a.k_pool = (const uint8_t *)p->k_pool; a.v_pool = (const uint8_t *)p->v_pool;
    a.stride_page_b = p->kv_stride_page * es; a.stride_head_b = p->kv_stride_head * es;
    a.stride_token_b = (int32_t)(p->kv_stride_token * es);
    a.k_scale = p->k_scale; a.v_scale = p->v_scale;
    a.block_table = p->block_table; a.seq_lens = p->seq_lens;
    a.seq_group = p->seq_group; a.pfx_off = p->prefix_page_offsets; a.pfx_pages = p->prefix_pages;
    a.scale_log2 = p->softmax_scale * 1.4426950408889634f;
    a.out = (uint16_t *)p->out; a.lse = p->lse;
    a.zeros = ctx ? ctx->zeros : nullptr;
    a.self_plan = ctx && ctx->self_plan && ra::can_self_plan(a.D, a.kv_fp8, a.stages, a.B, a.share ? a.num_groups : 0, a.members_per_row);
    a.reuse_lists = a.self_plan && (p->flags & RA_FLAG_REUSE_SCHEDULE) != 0;
}

// Turns per-workgroup weights (per mille of the mean, clamped to 700..1400 so that no span is shorter than half the
// mean) into the running sums the schedule reads, and uploads them.
static hipError_t upload_wave_weights(ra_ctx *c, int f, int d, const int32_t *w, int n)
{
    std::vector<int32_t> cum((size_t)n + 1);
    double total = 0;
    for (int i = 0; i < n; i++) total += w[i] < 700 ? 700 : (w[i] > 1400 ? 1400 : w[i]);
    double run = 0;
    for (int i = 0; i < n; i++) {
        cum[i] = (int32_t)std::llround(run / total * 1048576.0);
        run += w[i] < 700 ? 700 : (w[i] > 1400 ? 1400 : w[i]);
    }
    cum[n] = 1 << 20;
    return hipMemcpy(c->wave_cum[f][d], cum.data(), ((size_t)n + 1) * 4, hipMemcpyHostToDevice);
}

} // namespace

extern "C" {

uint32_t rollout_attn_abi_version(void) { return ROLLOUT_ATTN_ABI_VERSION; }

ra_status rollout_attn_create(ra_ctx **out, int device)
{
    if (!out) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    *out = nullptr;
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess) e = hipSetDevice(device);
    if (e != hipSuccess) { set_err(nullptr, "hipSetDevice(%d): %s", device, hipGetErrorString(e)); return RA_ERR_DEVICE; }
    ra_ctx *c = new (std::nothrow) ra_ctx();
    if (!c) { set_err(nullptr, "out of host memory"); return RA_ERR_DEVICE; }
    memset(c, 0, sizeof *c);
    c->device = device;
    c->cost_prefix[0] = ra::kCostPrefix;
    c->cost_prefix[1] = ra::kCostPrefixFp8;
    c->cost_item = ra::kCostItem;
    c->cost_item_pfx[0] = ra::kCostItemPrefix;
    c->cost_item_pfx[1] = ra::kCostItemPrefixFp8;
    // Share of the page stream each accelerator die's workgroups get, per mille of the mean (workgroups are dealt to the
    // dies round-robin).  The odd dies stream about a tenth slower than the even ones on the machines measured; beyond
    // that the pattern is per workgroup and per machine: rollout_attn_set_wave_weights takes a measured one.
    static const int kXcdShare[8] = {1060, 950, 1060, 935, 1045, 930, 1055, 965};
    static const int kYoungerWaveShare = 820; // per mille of its die's share
    for (int x = 0; x < 8; x++) c->xcd_w[x] = kXcdShare[x];
    bool own_table = true;
    if (const char *ev = getenv("ROLLOUT_ATTN_XCD_WEIGHTS")) {
        int v[8];
        if (sscanf(ev, "%d,%d,%d,%d,%d,%d,%d,%d", &v[0], &v[1], &v[2], &v[3], &v[4], &v[5], &v[6], &v[7]) == 8) {
            bool ok = true;
            for (int x = 0; x < 8; x++) ok = ok && v[x] >= 700 && v[x] <= 1400; // no span under half the mean
            if (ok) {
                for (int x = 0; x < 8; x++) c->xcd_w[x] = v[x];
                own_table = false;
            }
        }
    }
    c->prefill_stay = -1;
    if (const char *ev = getenv("ROLLOUT_ATTN_PREFILL_WGS_PER_DIE")) {
        int v = atoi(ev);
        if (v >= 0 && v <= 64) c->prefill_stay = v;
    }
    c->self_plan = 1;
    if (const char *ev = getenv("ROLLOUT_ATTN_SELF_PLAN")) c->self_plan = atoi(ev) != 0;
    if (const char *ev = getenv("ROLLOUT_ATTN_COST_PREFIX")) {
        int v = atoi(ev);
        if (v >= 1 && v <= 16) c->cost_prefix[0] = c->cost_prefix[1] = v;
    }
    if (const char *ev = getenv("ROLLOUT_ATTN_COST_ITEM")) {
        int v = atoi(ev);
        if (v >= 0 && v <= 256) c->cost_item = v;
    }
    if (const char *ev = getenv("ROLLOUT_ATTN_COST_ITEM_PREFIX")) {
        int v = atoi(ev);
        if (v >= 0 && v <= 1024) c->cost_item_pfx[0] = c->cost_item_pfx[1] = v;
    }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e == hipSuccess && strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        set_err(nullptr, "device %d is %s; this library only runs on gfx950", device, prop.gcnArchName);
        delete c; (void)hipSetDevice(prev);
        return RA_ERR_UNSUPPORTED;
    }
    if (e == hipSuccess) { c->num_cus = prop.multiProcessorCount; e = hipMalloc(&c->zeros, 256); }
    if (e == hipSuccess) e = hipMemset(c->zeros, 0, 256);
    if (e == hipSuccess) e = hipMalloc((void **)&c->tickets, 256);
    if (e == hipSuccess) e = hipHostMalloc((void **)&c->host_flags, 64, hipHostMallocDefault);
    for (int i = 0; i < 4 && e == hipSuccess; i++) e = hipEventCreate(&c->ev[i]);
    for (int f = 0; f < 2; f++)
        for (int d = 0; d < 2; d++)
            if (e == hipSuccess) e = ra::attention_config(d ? 128 : 64, f, c->num_cus, &c->stages[f][d], &c->waves[f][d]);
    if (e == hipSuccess) e = ra::prefill_config();
    for (int f = 0; f < 2; f++)
        for (int d = 0; d < 2; d++) {
            if (e == hipSuccess) e = hipMalloc((void **)&c->wave_cum[f][d], ((size_t)ra::kMaxWaves + 1) * 4);
            if (e == hipSuccess && c->waves[f][d] > ra::kMaxWaves) e = hipErrorInvalidValue;
            if (e == hipSuccess) {
                std::vector<int32_t> w((size_t)c->waves[f][d]);
                for (size_t i = 0; i < w.size(); i++) {
                    w[i] = c->waves[f][d] % 8 == 0 ? c->xcd_w[i % 8] : 1000;
                    // (e4m3 pools: a wave spends more of its time on arithmetic, so the dies' memory paths matter half
                    // as much; measured with the built-in table at 0, 0.5, 0.75, 1, 1.25 and 1.5 times its spread)
                    if (f == 1 && own_table) w[i] = 1000 + (w[i] - 1000) / 2;
                    // A compute unit has four SIMDs: its fifth and later workgroups (e4m3 pools) each share one with an
                    // older wave, which the SIMD serves first; measured, they stream a sixth slower than the others.
                    if ((int)i >= 4 * c->num_cus) w[i] = w[i] * kYoungerWaveShare / 1000;
                }
                e = upload_wave_weights(c, f, d, w.data(), (int)w.size());
            }
        }
    if (e == hipSuccess) e = hipGetSymbolAddress(&c->scratch_ptr, HIP_SYMBOL(scratch)); // this device's copy
    if (getenv("ROLLOUT_ATTN_VERBOSE"))
        fprintf(stderr, "rollout_attn: die shares %d %d %d %d %d %d %d %d\n", c->xcd_w[0], c->xcd_w[1], c->xcd_w[2], c->xcd_w[3], c->xcd_w[4],
                c->xcd_w[5], c->xcd_w[6], c->xcd_w[7]);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        set_err(nullptr, "context set-up on device %d: %s", device, hipGetErrorString(e));
        rollout_attn_destroy(c);
        return RA_ERR_DEVICE;
    }
    *out = c;
    return RA_OK;
}

void rollout_attn_destroy(ra_ctx *c)
{
    if (!c) return;
    if (c->zeros) (void)hipFree(c->zeros);
    if (c->tickets) (void)hipFree(c->tickets);
    for (int f = 0; f < 2; f++)
        for (int d = 0; d < 2; d++)
            if (c->wave_cum[f][d]) (void)hipFree(c->wave_cum[f][d]);
    if (c->host_flags) (void)hipHostFree(c->host_flags);
    for (int i = 0; i < 4; i++)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    delete c;
}

const char *rollout_attn_last_error(const ra_ctx *c) { return c ? c->err : g_err; }

ra_status rollout_attn_check_problem(const ra_problem *p, char *msg, size_t n)
{
    char local[512];
    ra_status st = check(p, local, sizeof local);
    if (st != RA_OK) set_err(nullptr, "%s", local);
    if (msg && n) snprintf(msg, n, "%s", local);
    return st;
}

ra_status rollout_attn_workspace_size(const ra_ctx *c, const ra_problem *p, size_t *bytes)
{
    if (!p || !bytes) { set_err(const_cast<ra_ctx *>(c), "problem or bytes is NULL"); return RA_ERR_INVALID_ARG; }
    if (p->B < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->Hq % p->Hkv || p->num_groups < 0) {
        set_err(const_cast<ra_ctx *>(c), "bad shape for a workspace query");
        return RA_ERR_INVALID_ARG;
    }
    if ((p->D != 64 && p->D != 128) || p->Hq / p->Hkv > 16) {
        set_err(const_cast<ra_ctx *>(c), "unsupported shape for a workspace query (D in {64,128}, Hq/Hkv <= 16)");
        return RA_ERR_UNSUPPORTED;
    }
    ra::Workspace ws;
    int waves = c ? c->waves[p->kv_dtype == RA_KV_FP8_E4M3][p->D == 128] : 2048;
    *bytes = ra::carve_workspace(ws, nullptr, p->B, p->Hkv, p->Hq / p->Hkv, p->D, p->num_groups, waves,
                                     ra::prefix_rows(p->kv_dtype == RA_KV_FP8_E4M3));
    return RA_OK;
}

// The decode step on a checked problem whose workspace has been carved: validation (if asked for), schedule,
// attention, merge.
static ra_status enqueue_decode(ra_ctx *c, const ra_problem *p, const ra::Launch &a, hipStream_t s)
{
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess && (p->flags & RA_FLAG_VALIDATE)) {
        e = ra::launch_validate(a, s);
        if (e == hipSuccess) e = hipMemcpyAsync(c->host_flags, a.ws.hdr + 4, 4, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e == hipSuccess && c->host_flags[0]) {
            int f = c->host_flags[0];
            set_err(c, "device data failed validation:%s%s%s%s", f & 1 ? " sequence length out of range;" : "",
                    f & 2 ? " page id out of range;" : "", f & 4 ? " bad group id or prefix page list;" : "",
                    f & 8 ? " a member's block table does not start with its group's shared pages;" : "");
            if (prev != c->device) (void)hipSetDevice(prev);
            return RA_ERR_OUT_OF_RANGE;
        }
    }
    const bool tm = c->timing != 0;
    if (e == hipSuccess && tm) e = hipEventRecord(c->ev[0], s);
    // no schedule kernel when the batch's tables fit in the attention waves' LDS (they plan their spans themselves)
    const bool reuse = (p->flags & RA_FLAG_REUSE_SCHEDULE) != 0;
    const bool planned = !reuse && !a.self_plan;
    if (e == hipSuccess && planned) e = ra::launch_plan(a, s);
    if (e == hipSuccess && tm && planned) e = hipEventRecord(c->ev[1], s); // (no launch: no phase, no event)
    if (e == hipSuccess) e = ra::launch_attention(a, s);
    if (e == hipSuccess && tm) e = hipEventRecord(c->ev[2], s);
    if (e == hipSuccess) e = ra::launch_merge(a, s);
    if (e == hipSuccess && tm) e = hipEventRecord(c->ev[3], s);
    if (e == hipSuccess && tm) c->timed = planned ? 2 : 1;
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

ra_status rollout_attn_decode(ra_ctx *c, const ra_problem *p, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    ra_status st = check(p, c->err, sizeof c->err);
    if (st != RA_OK) return st;
    if (p->B == 0) return RA_OK;
    ra::Launch a;
    fill_launch(a, c, p);
    size_t need = ra::carve_workspace(a.ws, workspace, a.B, a.Hkv, a.G, a.D, a.num_groups, a.waves, a.prefix_rows);
    if (!workspace || ((uintptr_t)workspace & 255)) { set_err(c, "workspace is NULL or not 256-byte aligned"); return RA_ERR_INVALID_ARG; }
    if (workspace_bytes < need) {
        set_err(c, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
        return RA_ERR_WORKSPACE_TOO_SMALL;
    }
    return enqueue_decode(c, p, a, (hipStream_t)stream);
}

ra_status rollout_attn_decode_static(ra_ctx *c, const ra_problem *p, void *stream)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    ra_status st = check(p, c->err, sizeof c->err);
    if (st != RA_OK) return st;
    if (p->B == 0) return RA_OK;
    ra::Launch a;
    fill_launch(a, c, p);
    size_t need = ra::carve_workspace(a.ws, c->scratch_ptr, a.B, a.Hkv, a.G, a.D, a.num_groups, a.waves, a.prefix_rows);
    if (need > kScratchBytes) {
        set_err(c, "this problem needs a workspace of %zu bytes; the built-in one holds %zu (use rollout_attn_decode)", need,
                kScratchBytes);
        return RA_ERR_WORKSPACE_TOO_SMALL;
    }
    return enqueue_decode(c, p, a, (hipStream_t)stream);
}

ra_status rollout_attn_debug_gather(ra_ctx *c, const ra_problem *p, int32_t b, int32_t kvh, void *k_out, void *v_out,
                                    int64_t cap, void *stream)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    ra_status st = check(p, c->err, sizeof c->err);
    if (st != RA_OK) return st;
    if (b < 0 || b >= p->B || kvh < 0 || kvh >= p->Hkv || !k_out || !v_out || cap < 0) {
        set_err(c, "gather: b, kv_head, capacity or output pointer out of range");
        return RA_ERR_INVALID_ARG;
    }
    ra::Launch a;
    fill_launch(a, c, p);
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess) e = ra::launch_gather(a, b, kvh, k_out, v_out, cap, (hipStream_t)stream);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

ra_status rollout_attn_debug_schedule(ra_ctx *c, const ra_problem *p, void *workspace, size_t workspace_bytes, void *stream,
                                      ra_schedule_info *info)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    ra_status st = check(p, c->err, sizeof c->err);
    if (st != RA_OK) return st;
    if (!info) { set_err(c, "info is NULL"); return RA_ERR_INVALID_ARG; }
    ra::Launch a;
    fill_launch(a, c, p);
    size_t need = ra::carve_workspace(a.ws, workspace, a.B, a.Hkv, a.G, a.D, a.num_groups, a.waves, a.prefix_rows);
    if (!workspace || ((uintptr_t)workspace & 255)) { set_err(c, "workspace is NULL or not 256-byte aligned"); return RA_ERR_INVALID_ARG; }
    if (workspace_bytes < need) {
        set_err(c, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
        return RA_ERR_WORKSPACE_TOO_SMALL;
    }
    info->header_offset = (char *)a.ws.hdr - (char *)workspace;
    info->work_list_offset = (char *)a.ws.seg_rec - (char *)workspace;
    info->merge_desc_offset = (char *)a.ws.merge_desc - (char *)workspace;
    info->waves = a.waves;
    info->segments_per_chunk = ra::kChunkSegs;
    if (p->B == 0) return RA_OK;
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess) e = ra::launch_plan(a, (hipStream_t)stream);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

ra_status rollout_attn_append(ra_ctx *c, const ra_problem *p, const void *k_new, const void *v_new, void *stream)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    ra_status st = check(p, c->err, sizeof c->err);
    if (st != RA_OK) return st;
    if (p->B == 0) return RA_OK;
    if (!k_new || !v_new || (((uintptr_t)k_new | (uintptr_t)v_new) & 3)) {
        set_err(c, "append: k_new and v_new must be non-NULL and 4-byte aligned");
        return RA_ERR_INVALID_ARG;
    }
    ra::Launch a;
    fill_launch(a, c, p);
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess) e = ra::launch_append(a, k_new, v_new, (hipStream_t)stream);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

static ra_status check_prefill(const ra_prefill *p, char *msg, size_t n)
{
    auto fail = [&](ra_status st, const char *fmt, ...) {
        if (msg && n) {
            va_list ap;
            va_start(ap, fmt);
            vsnprintf(msg, n, fmt, ap);
            va_end(ap);
        }
        return st;
    };
    if (msg && n) msg[0] = 0;
    if (!p) return fail(RA_ERR_INVALID_ARG, "prefill is NULL");
    if (p->num_prompts < 0 || p->total_tokens < 0 || p->max_prompt_len < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->D <= 0)
        return fail(RA_ERR_INVALID_ARG, "negative or zero dimension (num_prompts=%d total_tokens=%d max_prompt_len=%d Hq=%d "
                                        "Hkv=%d D=%d)", p->num_prompts, p->total_tokens, p->max_prompt_len, p->Hq, p->Hkv, p->D);
    if (p->Hq % p->Hkv) return fail(RA_ERR_INVALID_ARG, "Hq=%d is not a multiple of Hkv=%d", p->Hq, p->Hkv);
    if (!std::isfinite(p->softmax_scale) || p->softmax_scale <= 0.f)
        return fail(RA_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
    if (p->D != 64 && p->D != 128) return fail(RA_ERR_UNSUPPORTED, "D=%d (only 64 and 128 are supported)", p->D);
    if ((int64_t)p->total_tokens * p->Hq * p->D >= (int64_t)1 << 40) return fail(RA_ERR_UNSUPPORTED, "batch too large");
    if (p->num_prompts == 0 || p->total_tokens == 0 || p->max_prompt_len == 0) return RA_OK;
    if (!p->q || !p->k || !p->v || !p->cu_seqlens || !p->out || !p->lse)
        return fail(RA_ERR_INVALID_ARG, "a required pointer (q, k, v, cu_seqlens, out, lse) is NULL");
    if (((uintptr_t)p->q | (uintptr_t)p->k | (uintptr_t)p->v | (uintptr_t)p->out) % 16 || (uintptr_t)p->lse % 4)
        return fail(RA_ERR_INVALID_ARG, "q, k, v and out must be 16-byte aligned, lse 4-byte aligned");
    if (p->k_pool) {
        if (p->kv_dtype != RA_KV_BF16 && p->kv_dtype != RA_KV_FP8_E4M3)
            return fail(RA_ERR_INVALID_ARG, "kv_dtype=%d is not a ra_kv_dtype", p->kv_dtype);
        if (p->page_size != 16) return fail(RA_ERR_UNSUPPORTED, "page_size=%d (only 16 is supported)", p->page_size);
        const int es = p->kv_dtype == RA_KV_FP8_E4M3 ? 1 : 2;
        if (!p->v_pool || !p->page_offsets || !p->pages || p->num_pages < 0)
            return fail(RA_ERR_INVALID_ARG, "the cache write needs v_pool, page_offsets, pages and num_pages >= 0");
        if (p->kv_stride_token < p->D || p->kv_stride_head < 0 || p->kv_stride_page < 0)
            return fail(RA_ERR_INVALID_ARG, "kv strides must be non-negative and kv_stride_token >= D");
        if ((p->kv_stride_token * es) % 16 || (p->kv_stride_head * es) % 16 || (p->kv_stride_page * es) % 16)
            return fail(RA_ERR_INVALID_ARG, "kv strides must be multiples of 16 bytes");
        if (p->kv_stride_token * es * 16 > INT32_MAX) return fail(RA_ERR_UNSUPPORTED, "kv_stride_token too large");
        if (((uintptr_t)p->k_pool | (uintptr_t)p->v_pool) % 16)
            return fail(RA_ERR_INVALID_ARG, "k_pool and v_pool must be 16-byte aligned");
        if (es == 1 && (!p->k_scale || !p->v_scale)) return fail(RA_ERR_INVALID_ARG, "fp8 KV needs k_scale and v_scale");
    }
    return RA_OK;
}

ra_status rollout_attn_check_prefill(const ra_prefill *p, char *msg, size_t n) { return check_prefill(p, msg, n); }

ra_status rollout_attn_prefill(ra_ctx *c, const ra_prefill *p, void *stream)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    ra_status st = check_prefill(p, c->err, sizeof c->err);
    if (st != RA_OK) return st;
    if (p->num_prompts == 0 || p->total_tokens == 0 || p->max_prompt_len == 0) return RA_OK;
    ra::PrefillLaunch a;
    memset(&a, 0, sizeof a);
    a.num_prompts = p->num_prompts; a.max_len = p->max_prompt_len; a.Hq = p->Hq; a.Hkv = p->Hkv; a.D = p->D; a.G = p->Hq / p->Hkv;
    a.q = (const uint16_t *)p->q; a.k = (const uint16_t *)p->k; a.v = (const uint16_t *)p->v;
    a.cu = p->cu_seqlens;
    a.scale_log2 = p->softmax_scale * 1.4426950408889634f;
    a.out = (uint16_t *)p->out; a.lse = p->lse; a.zeros = c->zeros;
    a.num_cus = c->num_cus;
    a.stay = c->prefill_stay;
    if (p->k_pool) {
        const int es = p->kv_dtype == RA_KV_FP8_E4M3 ? 1 : 2;
        a.kv_fp8 = es == 1; a.num_pages = p->num_pages;
        a.k_pool = (uint8_t *)p->k_pool; a.v_pool = (uint8_t *)p->v_pool;
        a.stride_page_b = p->kv_stride_page * es; a.stride_head_b = p->kv_stride_head * es;
        a.stride_token_b = (int32_t)(p->kv_stride_token * es);
        a.k_scale = p->k_scale; a.v_scale = p->v_scale;
        a.page_off = p->page_offsets; a.pages = p->pages;
    }
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess && p->k_pool) e = ra::launch_prefill_write(a, (hipStream_t)stream);
    if (e == hipSuccess) e = ra::launch_prefill(a, (hipStream_t)stream);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

ra_status rollout_attn_wave_count(const ra_ctx *c, int32_t kv_dtype, int32_t head_dim, int32_t *waves)
{
    if (!c || !waves || (kv_dtype != RA_KV_BF16 && kv_dtype != RA_KV_FP8_E4M3) || (head_dim != 64 && head_dim != 128)) {
        set_err(const_cast<ra_ctx *>(c), "wave count: bad context, kv_dtype or head_dim");
        return RA_ERR_INVALID_ARG;
    }
    *waves = c->waves[kv_dtype == RA_KV_FP8_E4M3][head_dim == 128];
    return RA_OK;
}

ra_status rollout_attn_set_wave_weights(ra_ctx *c, int32_t kv_dtype, int32_t head_dim, const int32_t *weights, int32_t n)
{
    if (!c || !weights || (kv_dtype != RA_KV_BF16 && kv_dtype != RA_KV_FP8_E4M3) || (head_dim != 64 && head_dim != 128)) {
        set_err(c, "wave weights: bad context, kv_dtype, head_dim or weights");
        return RA_ERR_INVALID_ARG;
    }
    const int f = kv_dtype == RA_KV_FP8_E4M3, d = head_dim == 128;
    if (n != c->waves[f][d]) {
        set_err(c, "wave weights: %d given, this launch shape has %d workgroups (rollout_attn_wave_count)", n, c->waves[f][d]);
        return RA_ERR_INVALID_ARG;
    }
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess) e = upload_wave_weights(c, f, d, weights, n);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

ra_status rollout_attn_debug_stream(ra_ctx *c, const void *buf, size_t buf_bytes, int32_t granule_bytes, int32_t scattered,
                                    int32_t entries_per_wave, void *stream, size_t *bytes_read)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    const bool pow2 = buf_bytes && !(buf_bytes & (buf_bytes - 1));
    if (!buf || ((uintptr_t)buf & 15) || !pow2 || buf_bytes < 16384 || buf_bytes > ((size_t)1 << 40) || entries_per_wave < 1 ||
        (granule_bytes != 1024 && granule_bytes != 2048 && granule_bytes != 4096 && granule_bytes != 8192 && granule_bytes != 16384)) {
        set_err(c, "stream probe: buf must be 16-byte aligned, buf_bytes a power of two of at least 16384, granule_bytes a power "
                   "of two in 1024..16384, entries_per_wave positive");
        return RA_ERR_INVALID_ARG;
    }
    const int waves = c->waves[0][1];
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess) e = ra::launch_stream_probe(buf, buf_bytes, granule_bytes, scattered & 3, entries_per_wave, waves, (hipStream_t)stream);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    if (bytes_read) *bytes_read = (size_t)waves * entries_per_wave * 16384;
    return RA_OK;
}

ra_status rollout_attn_debug_stream_tail(ra_ctx *c, const void *buf, size_t buf_bytes, int32_t entries_per_wave, int32_t static_entries,
                                         int32_t chunk_entries, void *stream, size_t *bytes_read)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    const bool pow2 = buf_bytes && !(buf_bytes & (buf_bytes - 1));
    if (!buf || ((uintptr_t)buf & 15) || !pow2 || buf_bytes < 16384 || buf_bytes > ((size_t)1 << 40) || entries_per_wave < 1 ||
        entries_per_wave > 65536 || static_entries < 0 || static_entries >= entries_per_wave || chunk_entries < 1 || chunk_entries > 1024) {
        set_err(c, "stream probe with a ticketed tail: buf must be 16-byte aligned, buf_bytes a power of two of at least 16384, "
                   "0 <= static_entries < entries_per_wave <= 65536, chunk_entries in 1..1024");
        return RA_ERR_INVALID_ARG;
    }
    const int waves = c->waves[0][1];
    // the tail: what the static parts leave, in whole chunks (a last partial chunk is rounded up)
    const int64_t tail = (int64_t)waves * (entries_per_wave - static_entries);
    const int64_t tickets = (tail + chunk_entries - 1) / chunk_entries;
    int prev = 0;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess && prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess)
        e = ra::launch_stream_probe(buf, buf_bytes, 4096, 1, static_entries, waves, (hipStream_t)stream, chunk_entries, (uint32_t)tickets,
                                    c->tickets);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    if (bytes_read) *bytes_read = ((size_t)waves * static_entries + (size_t)tickets * chunk_entries) * 16384;
    return RA_OK;
}

ra_status rollout_attn_set_timing(ra_ctx *c, int enable)
{
    if (!c) { set_err(nullptr, "ctx is NULL"); return RA_ERR_INVALID_ARG; }
    c->timing = enable != 0;
    c->timed = 0;
    return RA_OK;
}

ra_status rollout_attn_get_timing(ra_ctx *c, float ms[3])
{
    if (!c || !ms) { set_err(c, "ctx or phase_ms is NULL"); return RA_ERR_INVALID_ARG; }
    if (!c->timed) { set_err(c, "no decode call has been timed (rollout_attn_set_timing first)"); return RA_ERR_INVALID_ARG; }
    hipError_t e = hipEventSynchronize(c->ev[3]);
    if (c->timed == 2) {
        for (int i = 0; i < 3 && e == hipSuccess; i++) e = hipEventElapsedTime(&ms[i], c->ev[i], c->ev[i + 1]);
    } else {
        // no schedule kernel was launched in that call: the attention phase starts at the first event
        ms[0] = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms[1], c->ev[0], c->ev[2]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms[2], c->ev[2], c->ev[3]);
    }
    if (e != hipSuccess) { set_err(c, "HIP: %s", hipGetErrorString(e)); return RA_ERR_DEVICE; }
    return RA_OK;
}

} // extern "C"
