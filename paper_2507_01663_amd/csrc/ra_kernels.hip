// gfx950 kernels of rollout_attn: schedule, paged decode attention, log-sum-exp merge, gather, validation.
//
// The decode step is HBM-bound (the rollout phase is memory-bound: paper Sec. 2.1.1), so the design is a
// streaming one: every (page, kv head) tile of K and of V is fetched exactly once with 16-byte-per-lane
// direct global->LDS loads, shared prompt pages once per prompt group (GRPO groups: Sec. 7.1), and the
// ragged lengths (Sec. 7.4) are balanced by cutting the concatenated page stream of all work rows into
// equal spans, one per resident wave.  MFMA does the two tile products; softmax is fp32 on the VALU.
#include "ra_device.h"

#include <stdlib.h>

namespace ra {

// Kernel arguments live in memory that takes a microsecond or two to reach the first time, and the compiler
// fetches a field where it is first used, often in the middle of the work.  Touching every cache line of them
// up front makes those trips overlap; later reads hit the scalar cache.
__device__ __forceinline__ void touch_args(const Launch &a)
{
    const int32_t *p = reinterpret_cast<const int32_t *>(&a);
    int32_t s = 0;
#pragma unroll
    for (unsigned i = 0; i < sizeof(Launch) / 4; i += 16) s |= p[i];
    s |= p[sizeof(Launch) / 4 - 1];
    asm volatile("" ::"s"(s));
}

// ------------------------------------------------------------------------------------------------------
// workspace
// ------------------------------------------------------------------------------------------------------

int prefix_rows_max(int B, int G, int num_groups, int prefix_rows)
{
    if (num_groups <= 0) return 0;
    int mpr = prefix_rows / G;
    long v = (long)num_groups + B / mpr;
    return (int)(v < B ? v : B);
}

size_t carve_workspace(Workspace &ws, void *base, int B, int Hkv, int G, int D, int num_groups, int waves, int prefix_rows)
{
    size_t off = 0;
    char *p = (char *)base;
    auto take = [&](size_t bytes) {
        void *r = p ? (void *)(p + off) : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return r;
    };
    int ng = num_groups > 0 ? num_groups : 0;
    int prm = prefix_rows_max(B, G, num_groups, prefix_rows);
    ws.hdr = (int32_t *)take(16 * 4);
    ws.grp_count = (int32_t *)take((size_t)(ng + 1) * 4);
    ws.grp_rowbase = (int32_t *)take((size_t)(ng + 1) * 4);
    ws.grp_membase = (int32_t *)take((size_t)(ng + 1) * 4);
    ws.seq_rank = (int32_t *)take((size_t)B * 4);
    ws.seq_pfx_row = (int32_t *)take((size_t)B * 4);
    ws.seq_rank_in_row = (int32_t *)take((size_t)B * 4);
    ws.merge_desc = (int4 *)take((size_t)B * Hkv * 32);
    ws.members = (int32_t *)take((size_t)B * 4);
    ws.row_start = (int32_t *)take(((size_t)2 * B + 1) * 4);
    ws.row_tab = (int4 *)take((size_t)2 * B * 16);
    const size_t spans = (size_t)waves; // one span of the cost stream per resident wave
    // every (item, span) pair that shares pages is one segment: at most items + spans of them
    const size_t chunks = spans + ((size_t)2 * B * Hkv + spans) / kChunkSegs + 2;
    ws.seg_rec = (int4 *)take(chunks * 16 * sizeof(int4));
    size_t nsuf = (size_t)B * Hkv + spans;
    ws.suf_o = (float *)take(nsuf * G * D * 4);
    ws.suf_lse = (float *)take(nsuf * G * 4);
    size_t npfx = prm ? (size_t)prm * Hkv + spans : 0;
    ws.pfx_o = (float *)take(npfx * prefix_rows * D * 4);
    ws.pfx_lse = (float *)take(npfx * prefix_rows * 4);
    ws.self_cnt = (int32_t *)take(spans * 4);
    ws.self_rec = (uint8_t *)take(spans * kSelfListBytes);
    return off;
}

// ------------------------------------------------------------------------------------------------------
// schedule: work rows, their cost, the scan, and each span's work list
//
// Work rows: first the shared-prefix rows (one per group and block of members_per_row members), then one row
// per sequence for its own pages.  A row of n pages costs a fixed amount plus weight*n per kv head, and the
// rows, each repeated for every kv head, form one stream of cost units that is cut into spans, one per
// resident wave: the ragged lengths (paper Sec. 7.4) never leave a compute unit idle.  A page belongs to the
// wave whose span holds the page's first cost unit.  Prefix pages weigh more because a wave spends more time
// on them (more query rows per byte); the weights only balance time, they never change results.
// ------------------------------------------------------------------------------------------------------

// Pages [p_lo, p_hi) of an item (first cost unit S, weight cw per page, n pages) that belong to the span
// [lo, hi) of the cost stream: those whose first unit S + cw*p lies in the span.
__device__ __forceinline__ void span_pages(int S, int cw, int n, int lo, int hi, int &p_lo, int &p_hi)
{
    // (an integer division is dozens of instructions here; most items lie wholly inside a span and need none)
    const int last = S + cw * (n - 1); // first unit of the last page
    p_lo = lo <= S ? 0 : (lo > last ? n : (lo - S + cw - 1) / cw);
    p_hi = hi <= S ? 0 : (hi > last ? n : (hi - S + cw - 1) / cw);
}

constexpr int kPlanThreads = 256;
constexpr int kPlanCap = 2048; // sequences / groups whose intermediate arrays fit in LDS; beyond, the workspace is used

// Exclusive scans of a[0..n) and b[0..n) in place, a[n] and b[n] = totals (b may be null).  All THREADS threads of the
// workgroup call it.  A thread sums a run of consecutive elements, the threads' sums are scanned (shuffles inside a
// wave, the waves' totals through tmp), and each thread writes its run back: three barriers whatever n is.
template <int THREADS> __device__ __forceinline__ void block_scan(int32_t *a, int32_t *b, int n, int32_t *tmp /*[34], LDS*/, int tid)
{
    const int lane = tid & 63, wv = tid >> 6;
    const int per = (n + THREADS - 1) / THREADS;
    const int i0 = tid * per < n ? tid * per : n, i1 = i0 + per < n ? i0 + per : n;
    int sa = 0, sb = 0;
#pragma unroll 1
    for (int i = i0; i < i1; i++) {
        sa += a[i];
        if (b) sb += b[i];
    }
    int xa = sa, xb = sb;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int ya = __shfl_up(xa, d), yb = __shfl_up(xb, d);
        if (lane >= d) xa += ya, xb += yb;
    }
    if (lane == 63) tmp[wv] = xa, tmp[17 + wv] = xb;
    __syncthreads();
    if (wv == 0) {
        const int ta = lane < THREADS / 64 ? tmp[lane] : 0, tb = lane < THREADS / 64 ? tmp[17 + lane] : 0;
        int ua = ta, ub = tb;
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
            const int ya = __shfl_up(ua, d), yb = __shfl_up(ub, d);
            if (lane >= d) ua += ya, ub += yb;
        }
        if (lane < THREADS / 64) tmp[lane] = ua - ta, tmp[17 + lane] = ub - tb;
        if (lane == THREADS / 64 - 1) tmp[16] = ua, tmp[33] = ub;
    }
    __syncthreads();
    int ea = tmp[wv] + xa - sa, eb = tmp[17 + wv] + xb - sb; // what precedes this thread's run
#pragma unroll 1
    for (int i = i0; i < i1; i++) {
        const int va = a[i];
        a[i] = ea;
        ea += va;
        if (b) {
            const int vb = b[i];
            b[i] = eb;
            eb += vb;
        }
    }
    if (tid == 0) {
        a[n] = tmp[16];
        if (b) b[n] = tmp[33];
    }
    __syncthreads();
}

// Where the cost stream is cut: into one span per resident wave.  The workgroups do not all stream equally fast (the
// eight accelerator dies get different shares of the memory bandwidth, and so do the compute units inside a die,
// in a pattern that repeats from launch to launch), so span c gets the share cum[c+1] - cum[c] of the stream, in
// units of 2^-20; the table comes from the context (equal shares per die pair unless the context was tuned).
struct Cuts {
    int U, S0; // the stream has fewer than 2^31 units (checked on the host)
    int waves;
    long V;              // S0 * waves >= U: the length the shares refer to
    const int32_t *cum;  // [waves + 1], cum[0] = 0, cum[waves] = 2^20, increasing
    __device__ long start(int c) const { return (V * cum[c]) >> 20; }
    __device__ int at(int share) const // the cost unit at a point of the share table
    {
        const long v = (V * share) >> 20;
        return v < U ? (int)v : U;
    }
    __device__ int lo(int c) const
    {
        const long v = start(c);
        return v < U ? (int)v : U;
    }
    __device__ int span_of(int pos) const // the span that holds cost unit pos < U
    {
        int c = 0, hi = waves; // invariant: start(c) <= pos < start(hi)
        while (hi - c > 1) {
            const int mid = (c + hi) >> 1;
            if (start(mid) <= pos) c = mid;
            else hi = mid;
        }
        return c;
    }
};

// Buffers of the rows phase: the staged inputs, the groups' and sequences' intermediates, the scanned row costs and
// the row table.  They live in LDS when the batch fits (the usual case), else in the workspace.
struct RowsBuf {
    int32_t *scan_tmp;                                // [34], LDS
    int32_t *len, *grp, *poff;                        // LDS copies of the inputs to fill, or null: read the inputs in place
    int32_t *grp_count, *grp_rowbase, *grp_membase;   // [NG], [NG + 1], [NG + 1]
    int32_t *seq_rank;                                // [B]  rank in the group, later the sequence's prefix row
    int32_t *row_start;                               // [rows + 1]
    int4 *tab;                                        // [rows]
    int32_t *members;                                 // [B]  sequences ordered by prefix row, or null
    int32_t *seq_pfx_row, *seq_rank_in_row;           // [B]  for the merge kernel, or null
};

__host__ __device__ inline int rows_most(int B, int NG, int mpr) // upper bound on work rows
{
    const int pr = NG > 0 ? (NG + B / mpr < B ? NG + B / mpr : B) : 0;
    return B + pr;
}
// The rows phase: membership, the rows with their costs (scanned in place in row_start), the row table.  Returns
// the number of rows and of shared-prefix rows among them.  Everything here is a function of the inputs alone and
// comes out the same in every workgroup (of THREADS threads) that runs this.
template <int THREADS>
__device__ __forceinline__ void rows_phase(const Launch &a, const RowsBuf &R, int &nR_out, int &nPR_out, int tid /* = threadIdx.x */)
{
    const int B = a.B;
    const int NG = a.share ? a.num_groups : 0;
    const int MPR = a.members_per_row;
    const int rMPR = ((1 << 20) + MPR - 1) / MPR; // (x * rMPR) >> 20 == x / MPR for x < 2^14
    int32_t *grp_count = R.grp_count, *grp_rowbase = R.grp_rowbase, *grp_membase = R.grp_membase;
    int32_t *seq_rank = R.seq_rank, *row_start = R.row_start;
    int4 *tab = R.tab;
    const int32_t *len_src = a.seq_lens, *grp_src = a.seq_group, *poff = a.pfx_off;
    // one trip to memory for everything the schedule depends on
    if (R.len) {
#pragma unroll 1
        for (int b = tid; b < B; b += THREADS) {
            R.len[b] = a.seq_lens[b];
            R.grp[b] = NG ? a.seq_group[b] : -1;
        }
#pragma unroll 1
        for (int g = tid; g <= NG; g += THREADS) R.poff[g] = NG ? a.pfx_off[g] : 0;
        len_src = R.len, grp_src = R.grp, poff = R.poff;
    }
#pragma unroll 1
    for (int g = tid; g < NG; g += THREADS) grp_count[g] = 0;
    __syncthreads();
    auto len_of = [&](int b) { // never walk past the table row
        const int Lb = len_src[b];
        return Lb < 0 ? 0 : (Lb > a.max_pages * kPage ? a.max_pages * kPage : Lb);
    };
    auto grp_of = [&](int b) {
        const int g = NG ? grp_src[b] : -1;
        return g >= 0 && g < NG ? g : -1;
    };
    // membership: a sequence uses the shared pass when its group has shared pages and it holds all of them.  Its rank
    // in the group is the number of members before it (smaller b), a function of the inputs alone, because the rank
    // decides which shared-prefix row the member joins and with it the partials its result is merged from: sequences
    // are taken in ascending blocks, a lane finds its place among the lanes of its wave with the same group by
    // ballots, and the waves add their counts to the group's total one after the other.
#pragma unroll 1
    for (int base = 0; base < B; base += THREADS) {
        const int b = base + tid, lane = tid & 63, wv = tid >> 6;
        int g = -1;
        if (b < B) {
            const int gb = grp_of(b);
            if (gb >= 0) {
                const int np = poff[gb + 1] - poff[gb];
                if (np > 0 && len_of(b) >= np * kPage) g = gb;
            }
        }
        int pos = 0, cnt = 0;
        unsigned long long todo = __ballot(g >= 0);
#pragma unroll 1
        while (todo) {
            const int gl = __shfl(g, __ffsll((long long)todo) - 1);
            const unsigned long long same = __ballot(g == gl);
            if (g == gl) {
                pos = __popcll(same & ((1ull << lane) - 1ull));
                cnt = __popcll(same);
            }
            todo &= ~same;
        }
        int rank = -1;
#pragma unroll 1
        for (int w = 0; w < THREADS / 64; w++) {
            if (wv == w && g >= 0) {
                const int before = grp_count[g]; // the same for all lanes of the group: read by all, then written by one
                rank = before + pos;
                __builtin_amdgcn_wave_barrier();
                if (pos == 0) grp_count[g] = before + cnt;
            }
            __syncthreads();
        }
        if (b < B) seq_rank[b] = rank;
    }
    int nPR = 0;
    if (NG) {
#pragma unroll 1
        for (int g = tid; g < NG; g += THREADS) {
            grp_membase[g] = grp_count[g];
            grp_rowbase[g] = ((grp_count[g] + MPR - 1) * rMPR) >> 20;
        }
        __syncthreads();
        block_scan<THREADS>(grp_membase, grp_rowbase, NG, R.scan_tmp, tid);
        nPR = grp_rowbase[NG];
    }
    // Rows and their cost per kv head (staged in row_start, scanned in place): an item of n > 0 pages costs
    // cost_item + weight*n.  The fixed part stands for what every segment costs a wave on top of its pages
    // (query rows, a partial result, a pipeline that restarts).
#pragma unroll 1
    for (int g = tid; g < NG; g += THREADS) {
        const int cnt = grp_count[g], np = poff[g + 1] - poff[g];
        const int r0 = grp_rowbase[g];
#pragma unroll 1
        for (int k = 0; k * MPR < cnt; k++) {
            const int left = cnt - k * MPR;
            row_start[r0 + k] = a.cost_item_pfx + np * a.cost_prefix;
            tab[r0 + k] = make_int4(poff[g], grp_membase[g] + k * MPR, left < MPR ? left : MPR, np);
        }
    }
#pragma unroll 1
    for (int b = tid; b < B; b += THREADS) {
        const int Lb = len_of(b);
        const int rank = seq_rank[b];
        int skip = 0, prow = -1, in_row = -1;
        if (rank >= 0) {
            const int g = grp_of(b);
            const int k = (rank * rMPR) >> 20; // rank / MPR
            skip = poff[g + 1] - poff[g];
            prow = grp_rowbase[g] + k;
            in_row = rank - k * MPR;
            if (R.members) R.members[grp_membase[g] + rank] = b;
        }
        if (R.seq_pfx_row) {
            R.seq_pfx_row[b] = prow;
            R.seq_rank_in_row[b] = in_row;
        }
        seq_rank[b] = prow; // from here on: the sequence's prefix row
        const int pages = Lb > 0 ? (Lb + kPage - 1) / kPage - skip : 0;
        row_start[nPR + b] = pages > 0 ? a.cost_item + pages * kCostSuffix : 0;
        tab[nPR + b] = make_int4(b, skip, Lb - skip * kPage, pages);
    }
    __syncthreads();
    const int nR = B + nPR;
    block_scan<THREADS>(row_start, nullptr, nR, R.scan_tmp, tid);
    nR_out = nR;
    nPR_out = nPR;
}

// LDS of the schedule kernels' rows phase (batches of up to kPlanCap sequences and groups).
struct RowsLds {
    int32_t scan_tmp[36];
    int32_t len[kPlanCap], grp[kPlanCap], poff[kPlanCap + 1];
    int32_t grp_count[kPlanCap], grp_rowbase[kPlanCap + 1], grp_membase[kPlanCap + 1];
    int32_t seq_rank[kPlanCap], row_start[2 * kPlanCap + 1];
};
// The buffers of a schedule kernel: in LDS (L and tab) when the batch fits, else in the workspace; `publish` adds what
// the other kernels read (the members' list, each sequence's prefix row and place in it).
__device__ __forceinline__ void plan_rows_buf(RowsBuf &R, const Launch &a, RowsLds &L, bool small, int4 *tab, bool publish)
{
    const Workspace &w = a.ws;
    R.scan_tmp = L.scan_tmp;
    R.len = small ? L.len : nullptr;
    R.grp = small ? L.grp : nullptr;
    R.poff = small ? L.poff : nullptr;
    R.grp_count = small ? L.grp_count : w.grp_count;
    R.grp_rowbase = small ? L.grp_rowbase : w.grp_rowbase;
    R.grp_membase = small ? L.grp_membase : w.grp_membase;
    R.seq_rank = small ? L.seq_rank : w.seq_rank;
    R.row_start = small ? L.row_start : w.row_start;
    R.tab = tab;
    R.members = publish ? w.members : nullptr;
    R.seq_pfx_row = publish ? w.seq_pfx_row : nullptr;
    R.seq_rank_in_row = publish ? w.seq_rank_in_row : nullptr;
}

__global__ __launch_bounds__(kPlanThreads) void plan_rows_kernel(Launch a)
{
    touch_args(a);
    __shared__ RowsLds L;
    const int tid = threadIdx.x;
    const Workspace &w = a.ws;
    // inputs and intermediates live in LDS when they fit (the usual case), else in the workspace
    const bool small = a.B <= kPlanCap && (a.share ? a.num_groups : 0) <= kPlanCap;
    RowsBuf R;
    plan_rows_buf(R, a, L, small, w.row_tab, true);
    int nR, nPR;
    rows_phase<kPlanThreads>(a, R, nR, nPR, tid);

    // hand over to the second kernel: the scanned row costs and the counts
    for (int r = tid; r <= nR; r += kPlanThreads) w.row_start[r] = R.row_start[r];
    if (tid == 0) {
        w.hdr[0] = a.Hkv * R.row_start[nR];
        w.hdr[2] = nR;
        w.hdr[3] = nPR;
    }
}

// Second half of the schedule: the cuts, every span's work list, and the merge descriptors.

__device__ __forceinline__ void make_cuts(const Launch &a, int U, Cuts &cut, const int32_t *cum)
{
    cut.U = U;
    cut.waves = a.waves;
    cut.cum = cum;
    // no span is shorter than a few pages, and none is shorter than one page of either kind, so that every
    // span between the first and the last one of an item holds at least one of its pages
    int min_span = kMinUnitsPerWave * kCostSuffix;
    if (min_span < 4 * a.cost_prefix) min_span = 4 * a.cost_prefix; // (a workgroup's share is at least half the mean)
    cut.S0 = (int)(((unsigned)cut.U + a.waves - 1) / (unsigned)a.waves);
    if (cut.S0 < min_span) cut.S0 = min_span;
    cut.V = (long)cut.S0 * a.waves;
}

// The work list of spans first, first + stride, ...: one record per segment (the pages of one (row, kv head) item
// that lie in the span), so that the attention waves find their work with one load instead of walking the tables.
// A record is {index of the row's first page id in its table, first page, end page, token limit,
// kv head | prefix << 16, sequence (own pages) or first member slot (shared pages), query rows, partial slot}.
// A span with more than kChunkSegs segments chains further chunks behind the spans' own: chunk number
// nspans + (its first item) / kChunkSegs + 0, 1, ...  Items (row * Hkv + kv head) run in stream order, a span's
// segments are different items and the next span starts at or after this one's last item, so no two spans reach
// the same chunk, and there are at most (2 B Hkv) / kChunkSegs + 1 of them.
__device__ __forceinline__ void spans_phase(const Launch &a, const Cuts &cut, const int32_t *row_start, const int4 *row_tab, int nR,
                                            int nPR, int first, int stride)
{
    const Workspace &w = a.ws;
    const int nspans = cut.waves;
    for (int c = first; c < nspans; c += stride) {
        const int lo = cut.lo(c), hi = cut.lo(c + 1);
        int chunk = c, n = 0, chain = -1;
        if (lo < hi) {
            // first row of the span: the last row that starts at or before the span's first unit
            int r = 0, rhi = nR; // invariant: Hkv*row_start[r] <= lo < Hkv*row_start[rhi]
            while (rhi - r > 1) {
                const int mid = (r + rhi) >> 1;
                if ((long)a.Hkv * row_start[mid] <= lo) r = mid;
                else rhi = mid;
            }
            for (; r < nR; r++) {
                const int rs = a.Hkv * row_start[r];
                if (rs >= hi) break;
                const int ic = row_start[r + 1] - row_start[r]; // cost of one item of the row
                if (ic == 0) continue;
                const int4 info = row_tab[r];
                const bool prefix = r < nPR;
                const int cw = prefix ? a.cost_prefix : kCostSuffix;
                for (int kvh = lo > rs ? (lo - rs) / ic : 0; kvh < a.Hkv; kvh++) {
                    const int S = rs + kvh * ic;
                    if (S >= hi) break;
                    int p_lo, p_hi;
                    span_pages(S + (prefix ? a.cost_item_pfx : a.cost_item), cw, info.w, lo, hi, p_lo, p_hi);
                    if (p_lo >= p_hi) continue;
                    if (chain < 0) chain = nspans + (r * a.Hkv + kvh) / kChunkSegs; // where this span's further chunks go
                    if (n == kChunkSegs) { // chain another chunk
                        const int nc = chain++;
                        w.seg_rec[(size_t)chunk * 16] = make_int4(n, nc, 0, 0);
                        chunk = nc;
                        n = 0;
                    }
                    int4 *rec = w.seg_rec + (size_t)chunk * 16 + 2 * (1 + n);
                    if (!prefix) {
                        rec[0] = make_int4(info.x * a.max_pages + info.y, p_lo, p_hi, min(info.z, p_hi * kPage));
                        rec[1] = make_int4(kvh, info.x, a.G, info.x * a.Hkv + kvh + c);
                    } else {
                        rec[0] = make_int4(info.x, p_lo, p_hi, p_hi * kPage);
                        rec[1] = make_int4(kvh | (1 << 16), info.y, info.z * a.G, r * a.Hkv + kvh + c);
                    }
                    n++;
                }
            }
        }
        w.seg_rec[(size_t)chunk * 16] = make_int4(n, -1, 0, 0);
    }
}

// For the merge: the spans that hold pages of (sequence, kv head) item i's own row and of its prefix row prow (or -1),
// {pages, first span, last span, unused}.  Every span in that range holds at least one of the pages.
__device__ __forceinline__ void merge_desc_of(const Launch &a, const Cuts &cut, const int32_t *row_start, int nPR, int i, int prow)
{
    const int b = i / a.Hkv, kvh = i - b * a.Hkv;
    int4 own = make_int4(0, 0, -1, 0), pfx = make_int4(0, 0, -1, 0);
    {
        const int r = nPR + b;
        const int ic = row_start[r + 1] - row_start[r];
        if (ic > 0) {
            const int n = (ic - a.cost_item) / kCostSuffix;
            const int S = a.Hkv * row_start[r] + kvh * ic + a.cost_item;
            own = make_int4(n, cut.span_of(S), cut.span_of(S + kCostSuffix * (n - 1)), 0);
        }
    }
    if (prow >= 0) {
        const int ic = row_start[prow + 1] - row_start[prow];
        const int n = (ic - a.cost_item_pfx) / a.cost_prefix;
        const int S = a.Hkv * row_start[prow] + kvh * ic + a.cost_item_pfx;
        pfx = make_int4(n, cut.span_of(S), cut.span_of(S + a.cost_prefix * (n - 1)), 0);
    }
    a.ws.merge_desc[2 * i] = own;
    a.ws.merge_desc[2 * i + 1] = pfx;
}

// The second kernel of the two-kernel schedule (batches too large for the one below), spread over many compute units.
// Each workgroup first copies the scanned row costs and the row table into LDS if they fit.
constexpr int kSpanThreads = 128;

__global__ __launch_bounds__(kSpanThreads) void plan_spans_kernel(Launch a)
{
    touch_args(a);
    __shared__ int32_t l_row_start[2 * kPlanCap + 1];
    __shared__ int4 l_row_tab[2 * kPlanCap];
    __shared__ int32_t l_cum[kMaxWaves + 1];
    const int tid = threadIdx.x;
    const int gtid = blockIdx.x * kSpanThreads + tid, gstride = gridDim.x * kSpanThreads;
    for (int i = tid; i <= a.waves; i += kSpanThreads) l_cum[i] = a.wave_cum[i];
    const Workspace &w = a.ws;
    const int32_t *row_start = w.row_start;
    const int4 *row_tab = w.row_tab;
    // (there are at most 2B rows; copying that many without waiting for the count saves a trip to memory)
    const int rows_most = 2 * a.B;
    if (rows_most <= 2 * kPlanCap) {
        for (int r = tid; r <= rows_most; r += kSpanThreads) l_row_start[r] = w.row_start[r];
        for (int r = tid; r < rows_most; r += kSpanThreads) l_row_tab[r] = w.row_tab[r];
        row_start = l_row_start, row_tab = l_row_tab;
    }
    const int U = w.hdr[0], nR = w.hdr[2], nPR = w.hdr[3];
    const int my_item = gtid < a.B * a.Hkv ? gtid : 0;
    const int my_prow = w.seq_pfx_row[my_item / a.Hkv]; // for the merge descriptors below; fetched with the rest
    __syncthreads();

    Cuts cut;
    make_cuts(a, U, cut, l_cum);
    if (gtid == 0) w.hdr[7] = cut.waves;
    spans_phase(a, cut, row_start, row_tab, nR, nPR, gtid, gstride);
    for (int i = gtid; i < a.B * a.Hkv; i += gstride) merge_desc_of(a, cut, row_start, nPR, i, i == gtid ? my_prow : w.seq_pfx_row[i / a.Hkv]);
}

// The whole schedule in one launch, for batches whose tables fit in LDS (up to kPlanCap sequences and groups): every
// workgroup works the rows out for itself, which costs less than a second launch and a trip through memory.
// Workgroup 0 publishes what the other kernels read (members, prefix rows, counts) and writes the merge descriptors;
// the others write the spans' work lists.
__global__ __launch_bounds__(kPlanThreads) void plan_fused_kernel(Launch a)
{
    touch_args(a);
    __shared__ RowsLds L;
    __shared__ int4 l_row_tab[2 * kPlanCap];
    __shared__ int32_t l_cum[kMaxWaves + 1];
    const int tid = threadIdx.x;
    const Workspace &w = a.ws;
    for (int i = tid; i <= a.waves; i += kPlanThreads) l_cum[i] = a.wave_cum[i];
    RowsBuf R;
    plan_rows_buf(R, a, L, true, l_row_tab, blockIdx.x == 0);
    int nR, nPR;
    rows_phase<kPlanThreads>(a, R, nR, nPR, tid);
    const int32_t *row_start = R.row_start;
    Cuts cut;
    make_cuts(a, a.Hkv * row_start[nR], cut, l_cum);
    if (blockIdx.x == 0) {
        if (tid == 0) {
            w.hdr[0] = cut.U;
            w.hdr[2] = nR;
            w.hdr[3] = nPR;
            w.hdr[7] = cut.waves;
        }
        for (int i = tid; i < a.B * a.Hkv; i += kPlanThreads) merge_desc_of(a, cut, row_start, nPR, i, L.seq_rank[i / a.Hkv]);
    } else {
        spans_phase(a, cut, row_start, l_row_tab, nR, nPR, (blockIdx.x - 1) * kPlanThreads + tid, (gridDim.x - 1) * kPlanThreads);
    }
}

hipError_t launch_plan(const Launch &a, hipStream_t s)
{
    const int work = a.waves; // one thread per span
    if (a.B <= kPlanCap && (a.share ? a.num_groups : 0) <= kPlanCap) {
        hipLaunchKernelGGL(plan_fused_kernel, dim3(1 + (work + kPlanThreads - 1) / kPlanThreads), dim3(kPlanThreads), 0, s, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(plan_rows_kernel, dim3(1), dim3(kPlanThreads), 0, s, a);
    // ... and per (sequence, kv head)
    const int n = work > a.B * a.Hkv ? work : a.B * a.Hkv;
    hipLaunchKernelGGL(plan_spans_kernel, dim3((n + kSpanThreads - 1) / kSpanThreads), dim3(kSpanThreads), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// attention
// ------------------------------------------------------------------------------------------------------

// One unit of work of a wave: pages [pg_lo, pg_hi) of one (work row, kv head) item.  All fields but mvec are
// wave-uniform.
struct Segment {
    const int32_t *pages; // page ids of the work row (read with uniform_load)
    int pg_lo, pg_hi;
    int limit;            // tokens of the row that exist and belong to this piece: min(valid, 16*pg_hi)
    int kvh;
    int prefix;           // 1: shared prompt pages of a group, 0: a sequence's own pages
    int b;                // the sequence (own pages)
    int moff, nrows;      // shared pages: first slot in members[], query rows in use
    int64_t slot;         // partial-result slot
    uint32_t mvec;        // shared pages: lane i holds the sequence of the work row's member i
    __device__ __forceinline__ int stages() const { return (pg_hi - pg_lo + 1) >> 1; }
    // ring entries: a shared-pages segment leads with one entry that carries its query rows
    __device__ __forceinline__ int entries() const { return stages() + prefix; }
};

// The wave's LDS ring: entries (two pages each, or the query rows of a shared-pages segment) are numbered in the
// order the wave streams them, across segments; entry n lives in ring slot n % NST.
struct Ring {
    int issued; // entries whose loads have been issued
    int waited; // entries whose loads have been waited for (and consumed)
};

// 16-row query tiles that a shared-prefix work row carries: four for bf16 pools (64 rows fill a ring entry of two
// pages exactly), two for e4m3 pools, whose ring entries are half the size.
template <int KVB> struct PrefixTiles {
    static constexpr int value = KVB == 2 ? 4 : 2;
};
int prefix_rows(int kv_fp8) { return 16 * (kv_fp8 ? PrefixTiles<1>::value : PrefixTiles<2>::value); }

template <int D, int KVB, int NST> struct LdsMap {
    using G = Geo<D, KVB>;
    static constexpr int kQTile = kPage * D * 2;   // 16 query rows of bf16
    static constexpr int kQBase = NST * G::kStage;    // the query slot follows the ring
    static constexpr int kPlanBase = kQBase + kQTile; // then the work list of a wave that plans its span itself;
    static constexpr int kPlanBytes = kQTile;         // everything before it is free while the wave plans
    static constexpr int kRecCap = kPlanBytes / 32;   // records the work list holds
    static constexpr int kBytes = kPlanBase + kPlanBytes;
    static_assert(kPlanBytes <= kSelfListBytes, "a wave's list fits the room the workspace keeps for it");
    static_assert(PrefixTiles<KVB>::value * kQTile <= G::kStage, "the query rows of a shared-prefix row fill one ring entry");
    static_assert(PrefixTiles<KVB>::value * (D * 2 / 64) <= G::kDmaPerStage, "... with no more loads than two pages take");
};

// A finished partial of an own-pages segment, kept in registers.  Stores share the vector-memory counter with the
// ring's loads and take a full loaded-memory round trip to drain, so a wave keeps its partials (it rarely has
// more than three) and writes them when it has nothing left to stream.
template <int D> struct Pending {
    f32x4 o[D / 16];
    float lse2;
    int64_t slot; // wave-uniform
};
template <int D> __device__ __forceinline__ void store_pending(const Launch &a, const Pending<D> &p, int lane)
{
    const int row = lane & 15, j = lane >> 4;
    if (row < a.G) {
        float *dst = a.ws.suf_o + (p.slot * a.G + row) * D + 4 * j;
#pragma unroll
        for (int dt = 0; dt < D / 16; dt++) *(f32x4 *)(dst + 16 * dt) = p.o[dt];
        if (j == 0) a.ws.suf_lse[p.slot * a.G + row] = p.lse2;
    }
}

// The partial of a shared-prefix segment (NQT tiles of 16 query rows), held one tile to a Pending: written out.
template <int D, int NQT, int NP> __device__ __forceinline__ void store_prefix_partial(const Launch &a, const Pending<D> (&pk)[NP], int64_t slot, int nrows, int lane)
{
    const int j = lane >> 4;
#pragma unroll
    for (int t = 0; t < NQT; t++) {
        const int row = 16 * t + (lane & 15);
        if (row < nrows) {
            float *dst = a.ws.pfx_o + (slot * a.prefix_rows + row) * D + 4 * j;
#pragma unroll
            for (int dt = 0; dt < D / 16; dt++) *(f32x4 *)(dst + 16 * dt) = pk[t].o[dt];
            if (j == 0) a.ws.pfx_lse[slot * a.prefix_rows + row] = pk[t].lse2;
        }
    }
}

// Loads of one stage (two pages: K0 K1 V0 V1, and for e4m3 the four scales) of a segment into a ring slot.
template <int D, int KVB, int NST>
__device__ __forceinline__ void issue_stage(const Launch &a, const LaneConst<D, KVB> &lc, const Segment &sg, int st, int pid0,
                                            int pid1, int ring_slot, uint32_t lds_addr, int lane)
{
    using G = Geo<D, KVB>;
    const int p0 = sg.pg_lo + 2 * st;
    int nv0 = sg.limit - p0 * kPage, nv1 = nv0 - kPage;
    nv0 = nv0 > kPage ? kPage : nv0;
    nv1 = nv1 > kPage ? kPage : (nv1 < 0 ? 0 : nv1); // 0: no second page, every row reads zeros
    const uint32_t sb = lds_addr + ring_slot * G::kStage;
    const int64_t off0 = (int64_t)pid0 * a.stride_page_b + (int64_t)sg.kvh * a.stride_head_b;
    const int64_t off1 = (int64_t)pid1 * a.stride_page_b + (int64_t)sg.kvh * a.stride_head_b;
    // (a decode step reads every page once: streaming loads)
    issue_tile<D, KVB, true>(lc, a.k_pool + off0, nv0, sb, a.zeros);
    issue_tile<D, KVB, true>(lc, a.k_pool + off1, nv1, sb + G::kTile, a.zeros);
    issue_tile<D, KVB, true>(lc, a.v_pool + off0, nv0, sb + 2 * G::kTile, a.zeros);
    issue_tile<D, KVB, true>(lc, a.v_pool + off1, nv1, sb + 3 * G::kTile, a.zeros);
    if (KVB == 1) {
        // the pages' scales land behind the tiles: lanes 0..3 bring k0, v0, k1, v1
        const int64_t si = (int64_t)((lane & 2) ? pid1 : pid0) * a.Hkv + sg.kvh;
        const bool have = lane < 2 || (lane < 4 && nv1 > 0);
        const void *src = !have ? a.zeros : (lane & 1) ? (const void *)(a.v_scale + si) : (const void *)(a.k_scale + si);
        dma4(src, sb + 4 * G::kTile);
    }
}

// Query rows of an own-pages segment: the G heads of (b, kvh) are contiguous in q; rows G..15 read zeros.
template <int D, int KVB, int NST>
__device__ __forceinline__ void issue_q(const Launch &a, const uint16_t *__restrict__ q, const LaneConst<D, KVB> &lc,
                                        const Segment &sg, uint32_t lds_addr, int lane)
{
    using M = LdsMap<D, KVB, NST>;
    const uint8_t *src = (const uint8_t *)(q + ((int64_t)sg.b * a.Hq + (int64_t)sg.kvh * a.G) * D);
    const uint32_t dst = lds_addr + M::kQBase;
    // the tile in LDS: 16 rows of D bf16, 16-byte units swizzled inside the row like a bf16 K tile (worked out here,
    // once per segment, rather than kept in registers through the stream)
    constexpr int QU = D * 2 / 16, QM = QU - 1;
    asm volatile("" : "+v"(lane)); // (opaque, or the compiler works the placement out ahead of the loop after all)
#pragma unroll
    for (int n = 0; n < D * 2 / 64; n++) {
        const int slot = 64 * n + lane;
        const int r = slot / QU, cp = slot % QU;
        const void *p = r < a.G ? (const void *)(src + r * (D * 2) + (cp ^ (swz(r) & QM)) * 16) : a.zeros;
        dma16(p, dst + 1024 * n);
    }
}

// Query rows of a shared-pages segment, as a ring entry of their own: row = member * G + head of the kv head's
// group, a gather of whole rows of q (one per lane quarter), in 16-row tiles laid out like a query slot.  Rows past
// the ones in use read zeros.  Issues exactly as many loads as a stage of two pages, so that the ring's
// bookkeeping does not tell the two kinds of entry apart.
template <int D, int KVB, int NST>
__device__ __forceinline__ void issue_qrows(const Launch &a, const uint16_t *__restrict__ q, const LaneConst<D, KVB> &lc,
                                            const Segment &sg, int ring_slot, uint32_t lds_addr)
{
    using G = Geo<D, KVB>;
    using M = LdsMap<D, KVB, NST>;
    constexpr int NQT = PrefixTiles<KVB>::value, PER = D * 2 / 64, QU = D * 2 / 16;
    const uint32_t sb = lds_addr + ring_slot * G::kStage;
    // (every address below is a function of the lane alone, which the compiler would otherwise work out once and
    // keep in registers for the whole kernel, dozens of them; this happens once per segment, so recompute)
    int lane = threadIdx.x;
    asm volatile("" : "+v"(lane));
    const int r0 = lane / QU, cp = lane % QU;
#pragma unroll
    for (int t = 0; t < NQT; t++) {
#pragma unroll
        for (int n = 0; n < PER; n++) {
            const int r = (64 / QU) * n + r0, row = 16 * t + r; // row r of tile t lands where a query slot keeps it
            const int mi = (row * a.recip_g) >> 16;             // row / G (exact for rows below 64)
            const int seq = __builtin_amdgcn_ds_bpermute(4 * mi, (int)sg.mvec);
            const int head = sg.kvh * a.G + (row - mi * a.G);
            const uint8_t *src = (const uint8_t *)(q + ((int64_t)seq * a.Hq + head) * D) + (cp ^ (swz(r) & (QU - 1))) * 16;
            dma16(row < sg.nrows ? (const void *)src : a.zeros, sb + t * M::kQTile + 1024 * n);
        }
    }
#pragma unroll
    for (int k = NQT * PER; k < G::kDmaPerStage; k++) dma4(a.zeros, sb + 4 * G::kTile);
}

// Attention of NQT*16 query rows over one segment.  Two pages (32 keys) per ring stage:
//   S^T[key, row] = K_tile . Q^T      (16x16x32 MFMA over D, per page; A = K rows straight from LDS, B = Q in
//                                      registers)
//   O^T[d, row]  += V_tiles^T . P^T   (16x16x32 MFMA over the 32 keys; A = V through the transposing LDS read,
//                                      B = P: the two pages' S^T accumulators side by side, as they stand)
// The contraction index of the second product may be any permutation of the keys as long as both operands
// use the same one: slot e of lane group j is key 4j+e of the first page (e < 4) or key 4j+e-4 of the second.
// In both products a lane owns one query row (lane % 16), so the running max, the rescale factor and the
// row sum are per-lane scalars; only the row max needs a cross-lane step (lanes l, l^16, l^32, l^48).
//
// The ring does not run dry at a segment boundary: while the last entries of this segment are consumed, the
// first entries (and the query rows) of the next one are already being loaded.  On entry, the first
// min(NST-1, entries) entries of this segment are in flight; on exit the same holds for `nxt`.  Query rows of an
// own-pages segment (NQT == 1) wait in the query slot; those of a shared-pages segment are its first ring entry.
// A one-tile partial goes back in `ret` (normalised, with its log2-sum-exp); a shared-prefix partial is stored.
template <int D, int KVB, int NQT, int NST, int NP>
__device__ __forceinline__ void run_segment(const Launch &a, const uint16_t *__restrict__ q, const Segment &cur, bool has_nxt,
                                            const Segment &nxt, Ring &ring, const LaneConst<D, KVB> &lc, uint8_t *lds,
                                            uint32_t lds_addr, Pending<D> &ret, Pending<D> (&pk)[NP], bool park, int lane)
{
    static_assert(NQT == 1 || NQT <= NP, "a shared-prefix partial has a waiting register set per tile");
    using G = Geo<D, KVB>;
    using M = LdsMap<D, KVB, NST>;
    static_assert((NST - 1) * G::kDmaPerStage < 64, "the vector-memory counter holds 6 bits");
    static_assert(NQT == 1 || NQT == PrefixTiles<KVB>::value, "one tile, or a shared-prefix row");
    constexpr int QL = NQT > 1 ? 1 : 0; // this segment's first ring entry carries its query rows
    const int j = lane >> 4;
    const int niter = cur.stages() + QL;
    const int base = ring.waited; // ring number of this segment's first entry
    int nxt_pre = 0, nxt_ql = 0;
    if (has_nxt) {
        nxt_ql = nxt.prefix;
        nxt_pre = nxt.stages() + nxt_ql;
        nxt_pre = nxt_pre < NST - 1 ? nxt_pre : NST - 1;
    }
    const int total = niter + nxt_pre;
    const int ntiles = NQT > 1 ? (cur.nrows + 15) >> 4 : 1; // tiles in use (the others hold zeros and are skipped)

    // page id of page h of the entry with number base + rel (this segment's entries first, then the next one's)
    auto page_id = [&](int rel, int h) {
        int id = 0;
        if (rel < niter) {
            const int st = rel - QL, p = cur.pg_lo + 2 * st + h;
            if (st >= 0 && p < cur.pg_hi) id = uniform_load(cur.pages, p);
        } else if (rel < total) {
            const int st = rel - niter - nxt_ql, p = nxt.pg_lo + 2 * st + h;
            if (st >= 0 && p < nxt.pg_hi) id = uniform_load(nxt.pages, p);
        }
        return id;
    };
    int nid0 = page_id(ring.issued - base, 0), nid1 = page_id(ring.issued - base, 1); // one entry ahead of their use

    // Q^T operand: for k-step i, lane (row = lane%16, j) holds the eight d values that its K operand holds.
    // bf16 K: d = 32*i + 8*j .. +7.  e4m3 K: one 16-byte K read carries 16 d values and feeds two k-steps, so
    // d = 16*(4*(i/2) + j) + 8*(i%2) .. +7 (the sum over d does not care about the order).
    bf16x8 qf[NQT][G::kKSteps];

    f32x4 o[NQT][G::kDTiles];
    float m[NQT], lsum[NQT];
#pragma unroll
    for (int t = 0; t < NQT; t++) {
        m[t] = -INFINITY;
        lsum[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // keeps NST-1 entries in flight beyond entry `it` (this segment's own first entries were issued before it began)
    auto issue_ahead = [&](int it) {
        int want = it + NST;
        want = want < total ? want : total;
        while (ring.issued - base < want) {
            const int rel = ring.issued - base;
            if (rel < niter) {
                issue_stage<D, KVB, NST>(a, lc, cur, rel - QL, nid0, nid1, ring.issued % NST, lds_addr, lane);
            } else if (rel == niter && nxt_ql) {
                issue_qrows<D, KVB, NST>(a, q, lc, nxt, ring.issued % NST, lds_addr);
            } else {
                if (rel == niter) issue_q<D, KVB, NST>(a, q, lc, nxt, lds_addr, lane);
                issue_stage<D, KVB, NST>(a, lc, nxt, rel - niter - nxt_ql, nid0, nid1, ring.issued % NST, lds_addr, lane);
            }
            ring.issued++;
            nid0 = page_id(ring.issued - base, 0);
            nid1 = page_id(ring.issued - base, 1);
        }
    };
    if (!QL) {
        // The query rows were loaded into the query slot ahead of this segment's first entries; fetch them before
        // anything else is issued, because the next segment's may be (there is one slot).
        WaitTail<NST - 1, G::kDmaPerStage>::run(ring.issued - base);
#pragma unroll
        for (int i = 0; i < G::kKSteps; i++) qf[0][i] = *(const bf16x8 *)(lds + M::kQBase + lc.kq_off[i]);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    } else {
        // the first ring entry holds the query rows
        issue_ahead(0);
        WaitTail<NST - 1, G::kDmaPerStage>::run(ring.issued - base - 1);
        const uint8_t *qb = lds + (base % NST) * G::kStage;
#pragma unroll
        for (int t = 0; t < NQT; t++) {
#pragma unroll
            for (int i = 0; i < G::kKSteps; i++) qf[t][i] = *(const bf16x8 *)(qb + t * M::kQTile + lc.kq_off[i]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        ring.waited++;
    }

    for (int it = QL; it < niter; it++) {
        issue_ahead(it);
        // Loads complete in order, and every ring entry is the same number of them.  Anything else issued after
        // this entry (query rows of an own-pages segment, partial stores) only makes the wait stricter than needed.
        WaitTail<NST - 1, G::kDmaPerStage>::run(ring.issued - base - 1 - it);
        const int rslot = (base + it) % NST;
        const uint8_t *st = lds + rslot * G::kStage;
        const int pg0 = cur.pg_lo + 2 * (it - QL); // first page of this stage

        // scores of the 2 x 16 keys of this stage
        f32x4 s[NQT][2];
#pragma unroll
        for (int pg = 0; pg < 2; pg++) {
#pragma unroll
            for (int t = 0; t < NQT; t++) s[t][pg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < G::kKReads; i++) {
                if (KVB == 2) {
                    bf16x8 kf = *(const bf16x8 *)(st + pg * G::kTile + lc.k_off[i]);
#pragma unroll
                    for (int t = 0; t < NQT; t++)
                        if (t < ntiles) s[t][pg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[t][i], s[t][pg], 0, 0, 0);
                } else {
                    const int4 kc = *(const int4 *)(st + pg * G::kTile + lc.k_off[i]); // 16 codes: two k-steps
                    const bf16x8 k0 = fp8x8_to_bf16(kc.x, kc.y), k1 = fp8x8_to_bf16(kc.z, kc.w);
#pragma unroll
                    for (int t = 0; t < NQT; t++)
                        if (t < ntiles) {
                            s[t][pg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[t][2 * i], s[t][pg], 0, 0, 0);
                            s[t][pg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[t][2 * i + 1], s[t][pg], 0, 0, 0);
                        }
                }
            }
        }
        // e4m3: one scale per (page, head) for K and one for V.  The K scale folds into the fp32 score scale,
        // the V scale into P before it is rounded to bf16 (the row sum keeps the unscaled weights).
        float ks0 = a.scale_log2, ks1 = a.scale_log2, vs0 = 1.0f, vs1 = 1.0f;
        if (KVB == 1) {
            const f32x4 sc = *(const f32x4 *)(st + 4 * G::kTile);
            ks0 *= sc[0], vs0 = sc[1], ks1 *= sc[2], vs1 = sc[3];
        }
        const int tok0 = pg0 * kPage + 4 * j; // this lane's first token in the stage's first page
        const bool ragged = (pg0 + 2) * kPage > cur.limit;
        bf16x8 pf[NQT];
#pragma unroll
        for (int t = 0; t < NQT; t++) {
            if (t >= ntiles) continue;
            float v[8];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                v[e] = s[t][0][e] * ks0;
                v[4 + e] = s[t][1][e] * ks1;
            }
            if (ragged) {
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    if (tok0 + e >= cur.limit) v[e] = -INFINITY;
                    if (tok0 + kPage + e >= cur.limit) v[4 + e] = -INFINITY;
                }
            }
            const float mx = row_max(fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7]))));
            const float mn = fmaxf(m[t], mx);
            f32x8 p;
#pragma unroll
            for (int e = 0; e < 8; e++) p[e] = __builtin_amdgcn_exp2f(v[e] - mn);
            const float ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
            if (KVB == 1) {
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    p[e] *= vs0;
                    p[4 + e] *= vs1;
                }
            }
            pf[t] = __builtin_convertvector(p, bf16x8);
            // the running max rarely moves after the first pages: rescale only when some row's did
            if (__any(mn != m[t])) {
                const float alpha = __builtin_amdgcn_exp2f(m[t] - mn);
                m[t] = mn;
                lsum[t] *= alpha;
#pragma unroll
                for (int dt = 0; dt < G::kDTiles; dt++) o[t][dt] *= alpha;
            }
            lsum[t] += ps;
        }
        // O^T += V^T P^T
        typedef s16x4 __attribute__((address_space(3))) * lds_s16x4;
        typedef int __attribute__((ext_vector_type(2))) i32x2;
        typedef i32x2 __attribute__((address_space(3))) * lds_i32x2;
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const uint32_t vb = lds_addr + rslot * G::kStage + 2 * G::kTile;
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++) {
            bf16x8 vf;
            if (KVB == 2) {
                const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(vb + lc.v_off[dt]));
                const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(vb + G::kTile + lc.v_off[dt]));
                vf = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
            } else {
                // (the tile swizzle is an XOR of the unit number and the ring's slots start on multiples of 256 bytes, so
                // tile dt's address is tile 0's with 16 * dt XORed in: one lane constant instead of one per tile)
                const i32x2 vc = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2)((vb + lc.v_off[0]) ^ (uint32_t)(16 * dt)));
                vf = fp8x8_to_bf16(vc[0], vc[1]);
            }
#pragma unroll
            for (int t = 0; t < NQT; t++)
                if (t < ntiles) o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t], o[t][dt], 0, 0, 0);
        }
        // every LDS read of this stage has returned before a later load may overwrite it
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        ring.waited++;
    }

#pragma unroll
    for (int t = 0; t < NQT; t++) {
        const float l = row_sum(lsum[t]);
        const float inv = 1.0f / l;
        const float lse2 = m[t] + __builtin_amdgcn_logf(l);
        if (NQT == 1) {
#pragma unroll
            for (int dt = 0; dt < G::kDTiles; dt++) ret.o[dt] = o[t][dt] * inv;
            ret.lse2 = lse2;
        } else if (park) {
            // kept in the registers that wait for own partials (the caller has seen that they are free)
#pragma unroll
            for (int dt = 0; dt < G::kDTiles; dt++) pk[t < NP ? t : 0].o[dt] = o[t][dt] * inv;
            pk[t < NP ? t : 0].lse2 = lse2;
        } else {
            const int row = 16 * t + (lane & 15);
            if (row < cur.nrows) {
                float *dst = a.ws.pfx_o + (cur.slot * a.prefix_rows + row) * D + 4 * j;
#pragma unroll
                for (int dt = 0; dt < G::kDTiles; dt++) *(f32x4 *)(dst + 16 * dt) = o[t][dt] * inv;
                if (j == 0) a.ws.pfx_lse[cur.slot * a.prefix_rows + row] = lse2;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------------
// A wave that plans its own span (no schedule kernel).
//
// For batches whose tables fit beside the ring, the schedule kernels are not launched: every attention wave works
// the rows out for itself in the LDS it will stream through afterwards (they are a function of the lengths and the
// groups alone, so all waves get the same rows), cuts the stream, and lists the segments of its own span in the
// work-list area of its LDS.  If the list fills up, the wave streams what it has listed, drains, and plans again
// from where it stopped.  What the merge kernel needs to find an item's partials (the first and the last span that
// hold own pages of it, and the same for its prefix row, with the row and the sequence's place in it) is written by
// the waves that hold those pieces, while they plan.
// ------------------------------------------------------------------------------------------------------

struct SpanPlan {
    int nR, nPR; // work rows, of which shared-prefix rows
    int lo, hi;  // the span's cost units
    int r, kvh;  // the first item not yet listed
    bool done;
};

__device__ __forceinline__ int ufl(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Tables of a wave that plans for itself (LDS, in the ring's space while it is idle).  Leaner than the schedule
// kernels' rows phase: a wave needs the rows' costs to find its span, and the members of a prefix row only if the row
// has pages in its span, so no rank is worked out for the other groups.
struct WaveTables {
    int32_t *len;    // [B]      clamped lengths
    int32_t *grp;    // [B]      the group whose shared pass the sequence uses, or -1
    int32_t *poff;   // [NG + 1]
    int32_t *gcnt;   // [NG + 1] members per group
    int32_t *rowgrp; // [prefix rows]  group | row's number in its group << 16
    int32_t *rs;     // [rows + 1]     first cost unit of every row (per kv head)
};
constexpr int kSelfPerLane = 8; // sequences (and groups) a lane takes: batches of up to 512 sequences and 511 groups
__host__ __device__ inline size_t wave_tables_bytes(int B, int NG, int mpr)
{
    const size_t rows = (size_t)rows_most(B, NG, mpr);
    return 4 * (2 * (size_t)B + 2 * ((size_t)NG + 1) + (rows - B + 1) + rows + 1 + 8);
}
__device__ __forceinline__ void carve_wave_tables(WaveTables &T, void *base, int B, int NG, int mpr)
{
    const int rows = rows_most(B, NG, mpr);
    int32_t *p = (int32_t *)base;
    auto take = [&](int n) {
        int32_t *r = p;
        p += n;
        return r;
    };
    T.len = take(B);
    T.grp = take(B);
    T.poff = take(NG + 1);
    T.gcnt = take(NG + 1);
    T.rowgrp = take(rows - B + 1);
    T.rs = take(rows + 1);
}

// Exclusive scan of x over the 64 lanes; total: the sum.  Data-parallel-primitive moves on the VALU (no LDS trip per
// step): shifts by 1, 2, 4, 8 inside the rows of 16 lanes, then each row's last lane broadcast into the next row
// (rows 1 and 3) and lane 31 into the upper half; lanes without a source add 0.
__device__ __forceinline__ int wave_scan(int x, int lane, int &total)
{
    int v = x;
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false); // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false); // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false); // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false); // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false); // row_bcast:15
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false); // row_bcast:31
    total = __builtin_amdgcn_readlane(v, 63);
    (void)lane;
    return v - x;
}

// The rows and where they start in the cost stream, by one wave for itself (see rows_phase for what a row is and
// costs).  A lane takes runs of consecutive sequences and of consecutive groups and keeps them in registers; the
// tables in LDS are what the listing below looks up.
__device__ __forceinline__ void wave_rows(const Launch &a, const WaveTables &T, int &nR_out, int &nPR_out, int lane)
{
    constexpr int N = kSelfPerLane;
    const int B = a.B;
    const int NG = a.share ? a.num_groups : 0;
    const int MPR = a.members_per_row;
    const int rMPR = ((1 << 20) + MPR - 1) / MPR; // (x * rMPR) >> 20 == x / MPR for x < 2^14
    const int KB = (B + 63) >> 6, KG = (NG + 64) >> 6; // per lane: sequences, entries of the groups' offsets
    // one trip to memory for everything the schedule depends on
    int L[N], g[N], po[N];
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int b = lane * KB + k, gl = lane * KG + k;
        L[k] = 0, g[k] = -1, po[k] = 0;
        if (k < KB && b < B) {
            L[k] = a.seq_lens[b];
            if (NG) g[k] = a.seq_group[b];
        }
        if (NG && k < KG && gl <= NG) po[k] = a.pfx_off[gl];
    }
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int gl = lane * KG + k;
        if (k < KG && gl <= NG) {
            T.poff[gl] = po[k];
            T.gcnt[gl] = 0;
        }
    }
    __syncthreads();
    // membership: a sequence uses the shared pass when its group has shared pages and it holds all of them
    int np[N];
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int b = lane * KB + k;
        np[k] = 0;
        if (k < KB && b < B) {
            L[k] = L[k] < 0 ? 0 : (L[k] > a.max_pages * kPage ? a.max_pages * kPage : L[k]); // never walk past the table row
            if (g[k] < 0 || g[k] >= NG) g[k] = -1;
            if (g[k] >= 0) {
                np[k] = T.poff[g[k] + 1] - T.poff[g[k]];
                if (np[k] > 0 && L[k] >= np[k] * kPage) atomicAdd(&T.gcnt[g[k]], 1);
                else g[k] = -1, np[k] = 0;
            }
            T.len[b] = L[k];
            T.grp[b] = g[k];
        }
    }
    __syncthreads();
    // prefix rows: ceil(members / MPR) per group, all of a group's rows cost the same
    int rows_l = 0, cost_l = 0, rows_g[N], cost_g[N];
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int gl = lane * KG + k;
        rows_g[k] = 0, cost_g[k] = 0;
        if (k < KG && gl < NG) {
            rows_g[k] = ((T.gcnt[gl] + MPR - 1) * rMPR) >> 20;
            cost_g[k] = a.cost_item_pfx + (T.poff[gl + 1] - T.poff[gl]) * a.cost_prefix;
            rows_l += rows_g[k];
            cost_l += rows_g[k] * cost_g[k];
        }
    }
    int nPR, P;
    int row = wave_scan(rows_l, lane, nPR), at = wave_scan(cost_l, lane, P);
#pragma unroll
    for (int k = 0; k < N; k++) {
#pragma unroll 1
        for (int j = 0; j < rows_g[k]; j++) {
            T.rs[row] = at;
            T.rowgrp[row] = (lane * KG + k) | (j << 16);
            row++;
            at += cost_g[k];
        }
    }
    // sequence rows: an item of n > 0 pages costs cost_item + weight*n (see rows_phase)
    int cost[N], c_l = 0;
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int pages = L[k] > 0 ? (L[k] + kPage - 1) / kPage - np[k] : 0;
        cost[k] = pages > 0 ? a.cost_item + pages * kCostSuffix : 0;
        c_l += cost[k];
    }
    int S;
    at = P + wave_scan(c_l, lane, S);
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int b = lane * KB + k;
        if (k < KB && b < B) T.rs[nPR + b] = at;
        at += cost[k];
    }
    if (lane == 0) T.rs[nPR + B] = P + S;
    __syncthreads();
    nR_out = B + nPR;
    nPR_out = nPR;
}

// Lists the segments of span c from item (sp.r, sp.kvh) on into recs (LDS): 8 ints per segment as in the schedule
// kernels' work lists, except that a shared-pages segment carries its members' count in place of their offset and is
// followed by its members' sequence numbers, 8 to a record (the members of a group in ascending order, MPR to a row).
// Also writes, for the merge kernel, what the holder of an item's first or last piece knows: merge_desc's first and
// last span, and for the members of a prefix row the row and their place in it.  Stops when cap records would be
// exceeded (sp.done stays false).  Returns the number of records.  All lanes call it with the same arguments.
__device__ __forceinline__ int list_segments(const Launch &a, const WaveTables &T, SpanPlan &sp, int c, int32_t *recs, int cap, int lane)
{
    int n = 0;
    const int MPR = a.members_per_row;
    int32_t *md = (int32_t *)a.ws.merge_desc; // per item: {pages, first span, last span, -} of own pages, then of shared pages
#pragma unroll 1
    while (sp.r < sp.nR) {
        const int r = sp.r;
        const int rs = a.Hkv * ufl(T.rs[r]);
        if (rs >= sp.hi) break;
        const int ic = ufl(T.rs[r + 1]) - ufl(T.rs[r]); // cost of one item of the row
        if (ic == 0) {
            sp.r++;
            sp.kvh = 0;
            continue;
        }
        const bool prefix = r < sp.nPR;
        // prefix row: {index of the group's first page id, group, members, pages}; sequence row: {sequence, pages
        // skipped, tokens after the skip, pages}
        int4 info;
        int grp_k = 0;
        if (prefix) {
            const int gk = ufl(T.rowgrp[r]), g = gk & 0xffff;
            grp_k = gk >> 16;
            const int left = ufl(T.gcnt[g]) - grp_k * MPR;
            info = make_int4(ufl(T.poff[g]), g, left < MPR ? left : MPR, ufl(T.poff[g + 1]) - ufl(T.poff[g]));
        } else {
            const int b = r - sp.nPR, g = ufl(T.grp[b]), Lb = ufl(T.len[b]);
            const int skip = g >= 0 ? ufl(T.poff[g + 1]) - ufl(T.poff[g]) : 0;
            info = make_int4(b, skip, Lb - skip * kPage, (Lb + kPage - 1) / kPage - skip);
        }
        const int cw = prefix ? a.cost_prefix : kCostSuffix;
        const int need = prefix ? 1 + ((info.z + 7) >> 3) : 1;
        bool past = false;
#pragma unroll 1
        for (; sp.kvh < a.Hkv; sp.kvh++) {
            const int kvh = sp.kvh;
            const int S = rs + kvh * ic;
            if (S >= sp.hi) {
                past = true;
                break;
            }
            int p_lo, p_hi;
            span_pages(S + (prefix ? a.cost_item_pfx : a.cost_item), cw, info.w, sp.lo, sp.hi, p_lo, p_hi);
            if (p_lo >= p_hi) continue;
            if (n + need > cap) return n;
            int4 r0, r1;
            if (!prefix) {
                r0 = make_int4(info.x * a.max_pages + info.y, p_lo, p_hi, min(info.z, p_hi * kPage));
                r1 = make_int4(kvh, info.x, a.G, info.x * a.Hkv + kvh + c);
            } else {
                r0 = make_int4(info.x, p_lo, p_hi, p_hi * kPage);
                r1 = make_int4(kvh | (1 << 16), info.z, info.z * a.G, r * a.Hkv + kvh + c);
            }
            if (lane == 0) {
                *(int4 *)(recs + 8 * n) = r0;
                *(int4 *)(recs + 8 * n + 4) = r1;
            }
            if (!prefix) {
                const int i = info.x * a.Hkv + kvh;
                if (lane == 0 && p_lo == 0) {
                    md[8 * i + 1] = c;
                    if (info.y == 0) md[8 * i + 5] = 0, md[8 * i + 6] = -1; // no shared pages: says so for the merge
                }
                if (lane == 0 && p_hi == info.w) md[8 * i + 2] = c;
            } else {
                // the row's members: numbers grp_k*MPR .. of the group's members in ascending order of sequence
                int before = 0;
#pragma unroll 1
                for (int b0 = 0; b0 < a.B; b0 += 64) {
                    const int b = b0 + lane;
                    const bool is = b < a.B && T.grp[b] == info.y;
                    const unsigned long long m = __ballot(is);
                    const int place = before + __popcll(m & ((1ull << lane) - 1ull)) - grp_k * MPR;
                    if (is && place >= 0 && place < info.z) {
                        recs[8 * (n + 1) + place] = b;
                        const int i = b * a.Hkv + kvh;
                        if (p_lo == 0) {
                            md[8 * i + 5] = c;
                            a.ws.seq_pfx_row[b] = r; // (the same from every kv head)
                            a.ws.seq_rank_in_row[b] = place;
                            if (T.len[b] <= info.w * kPage) md[8 * i + 1] = 0, md[8 * i + 2] = -1; // no pages of its own
                        }
                        if (p_hi == info.w) md[8 * i + 6] = c;
                    }
                    before += __popcll(m);
                }
            }
            n += need;
        }
        if (past) break;
        sp.r++;
        sp.kvh = 0;
    }
    sp.done = true;
    return n;
}

// The read-only inputs and the schedule come in as separate restrict pointers so that the compiler can keep
// every wave-uniform lookup on the scalar unit, away from the vector-memory counter that paces the LDS ring.
#define RA_ATTN_PARAMS                                                                                                    \
    Launch a, const uint16_t *__restrict__ q, const int32_t *__restrict__ block_table, const int32_t *__restrict__ pfx_pages, \
        const int32_t *__restrict__ hdr, const uint32_t *__restrict__ seg_rec, const int32_t *__restrict__ members
#define RA_ATTN_ARGS a, q, block_table, pfx_pages, hdr, seg_rec, members

// SELF: the wave plans its own span (see above); otherwise it reads the schedule kernels' work list.
template <int D, int KVB, int NST, int NPEND, bool SELF> __device__ __forceinline__ void attention_body(RA_ATTN_PARAMS)
{
    using M = LdsMap<D, KVB, NST>;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds;
    const int lane = threadIdx.x;
    const int c = blockIdx.x;
    touch_args(a);
    if (!SELF) {
        const int nspans = uniform_load(hdr, 7);
        if (c >= nspans) return;
    }

    LaneConst<D, KVB> lc;
    if (!SELF) lane_setup<D, KVB>(lc, lane, a.stride_token_b);
    Ring ring = {0, 0};
    // Finished partials wait in registers for the end of the wave: up to NPEND of own-pages segments (and the one
    // just finished, `fresh`), or, while none of those waits, one of a shared-prefix segment, a tile to each of them.
    // Stores in mid-stream cost more than their bytes: the ring's next wait is also a wait for them, and writes among
    // the reads slow every wave's stream.
    static_assert(PrefixTiles<KVB>::value == NPEND + 1, "a shared-prefix partial fills the waiting registers exactly");
    Pending<D> pend[NPEND + 1];
    Pending<D> &fresh = pend[NPEND];
    int npend = 0;
    int parked_rows = 0; // > 0: a shared-prefix partial of that many rows waits in pend[]
    int64_t parked_slot = 0;

    // ---- the work list: segments in stream order ----
    // Schedule kernels' list: a chain of chunks of eight 8-dword records (a header and up to seven segments); a chunk
    // is one dword per lane, so it is held in one register and a field is a cross-lane read.  Own list: records in LDS.
    int32_t *recs = (int32_t *)(lds + M::kPlanBase);
    uint32_t chunk = 0;
    int wk_j = 0, wk_n = 0, wk_chain = -1;
    auto field = [&](int i) { return (int)__builtin_amdgcn_readlane(chunk, i); };
    auto load_chunk = [&](int ch) {
        chunk = seg_rec[(int64_t)ch * 64 + lane];
        wk_j = 0;
        wk_n = field(0);
        wk_chain = field(1);
    };
    auto advance = [&](Segment &out) -> bool {
        int f;
        if (SELF) {
            if (wk_j >= wk_n) return false;
            chunk = (uint32_t)recs[8 * wk_j + (lane & 7)];
            f = 0;
        } else {
            while (wk_j == wk_n) {
                if (wk_chain < 0) return false;
                load_chunk(wk_chain);
            }
            f = 8 * (1 + wk_j++);
        }
        const int where = field(f + 4);
        out.kvh = where & 0xffff;
        out.prefix = where >> 16;
        out.pages = (out.prefix ? pfx_pages : block_table) + field(f);
        out.pg_lo = field(f + 1);
        out.pg_hi = field(f + 2);
        out.limit = field(f + 3);
        out.b = out.prefix ? 0 : field(f + 5);
        out.moff = out.prefix ? field(f + 5) : 0;
        out.nrows = field(f + 6);
        out.slot = field(f + 7);
        out.mvec = 0;
        if (SELF) {
            // the members follow the segment's record, one per lane
            const int nmem = out.prefix ? out.moff : 0;
            if (lane < nmem) out.mvec = (uint32_t)recs[8 * (wk_j + 1) + lane];
            wk_j += 1 + ((nmem + 7) >> 3);
        } else if (out.prefix) {
            // the work row's members, one per lane (scalar loads four at a time: the ring's loads are not waited for)
            const int nmem = (out.nrows * a.recip_g) >> 16;
            for (int i = 0; i < nmem; i += 4) {
                int v[4];
#pragma unroll
                for (int k = 0; k < 4; k++) v[k] = i + k < nmem ? uniform_load(members, out.moff + i + k) : 0;
#pragma unroll
                for (int k = 0; k < 4; k++)
                    if (lane == i + k) out.mvec = (uint32_t)v[k];
            }
        }
        return true;
    };

    SpanPlan sp;
    sp.done = !SELF;
    bool first_pass = true;
    int keep = -2; // records of the list to keep in the workspace (-1: say that there is none), -2: nothing to do
    // the wave's two cut points of the share table: asked for now, needed when the rows are known
    const int share_lo = SELF ? uniform_load(a.wave_cum, c) : 0, share_hi = SELF ? uniform_load(a.wave_cum, c + 1) : 0;
    do {
        if (SELF) {
            // plan: the rows, the cut, this span's list (the ring is idle: its LDS holds the tables meanwhile)
            // (what is computed here is wanted here only: base and lane number are made opaque so that nothing derived
            // from them is worked out ahead of the loop and kept in registers while the wave streams)
            uint8_t *plan_base = lds;
            int plan_lane = lane;
            asm volatile("" : "+s"(plan_base), "+v"(plan_lane));
            // A call that reuses the schedule takes the list that the span's wave kept in the workspace when it planned
            // (one trip to memory in place of the planning pass), if that wave's whole span went into one list.
            const bool was_first = first_pass;
            keep = -2;
            int kept = -1;
            if (a.reuse_lists && was_first) kept = uniform_load(a.ws.self_cnt, c);
            if (kept >= 0) {
                const uint8_t *src = a.ws.self_rec + (int64_t)c * kSelfListBytes + 16 * plan_lane;
                for (int off = 0; off < 32 * kept; off += 1024) dma16(src + off, lds_addr + M::kPlanBase + off);
                wait_vmcnt<0>();
                wk_n = kept;
                sp.done = true;
                first_pass = false;
            } else {
            WaveTables T;
            carve_wave_tables(T, plan_base, a.B, a.share ? a.num_groups : 0, a.members_per_row);
            wave_rows(a, T, sp.nR, sp.nPR, plan_lane);
            if (first_pass) {
                Cuts cut;
                make_cuts(a, a.Hkv * ufl(T.rs[sp.nR]), cut, a.wave_cum);
                sp.lo = cut.at(share_lo), sp.hi = cut.at(share_hi);
                // the span's first item: the last row that starts at or before the span's first unit (starts do not decrease)
                int at_or_before = 0;
#pragma unroll 1
                for (int r0 = 0; r0 < sp.nR; r0 += 64) {
                    const int r = r0 + plan_lane;
                    at_or_before += __popcll(__ballot(r < sp.nR && (long)a.Hkv * T.rs[r] <= sp.lo));
                }
                const int r = at_or_before > 0 ? at_or_before - 1 : 0;
                const int rs = a.Hkv * ufl(T.rs[r]), ic = ufl(T.rs[r + 1]) - ufl(T.rs[r]);
                sp.r = r;
                sp.kvh = sp.lo > rs && ic > 0 ? (sp.lo - rs) / ic : 0;
                if (sp.lo >= sp.hi) sp.r = sp.nR; // nothing for this wave
                first_pass = false;
            }
            wk_n = list_segments(a, T, sp, c, (int32_t *)(plan_base + M::kPlanBase), M::kRecCap, plan_lane);
            if (was_first && !a.reuse_lists) keep = sp.done ? wk_n : -1;
            }
            wk_j = 0;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the tables have been read: the ring may overwrite them
            // (nothing is kept across a planning pass, neither the lane constants nor a partial: say so, or their
            // registers stay reserved while the wave plans)
            int stream_lane = lane;
            asm volatile("" : "+v"(stream_lane));
            lane_setup<D, KVB>(lc, stream_lane, a.stride_token_b);
#pragma unroll
            for (int k = 0; k < NPEND; k++) {
#pragma unroll
                for (int dt = 0; dt < D / 16; dt++) pend[k].o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
                pend[k].lse2 = 0.f;
                pend[k].slot = 0;
            }
        } else {
            load_chunk(c);
        }
        // (the lane number of this pass, opaque in a wave that plans, so that nothing derived from it is prepared
        // ahead of the planning pass and held in registers through it)
        int ln = lane;
        if (SELF) asm volatile("" : "+v"(ln));
        Segment cur, nxt;
        bool has_cur = advance(cur);
        if (has_cur) {
            // prime the ring with the first segment
            if (!cur.prefix) issue_q<D, KVB, NST>(a, q, lc, cur, lds_addr, ln);
            const int n = min(NST - 1, cur.entries());
            for (int k = 0; k < n; k++) {
                const int st = k - cur.prefix;
                if (st < 0) {
                    issue_qrows<D, KVB, NST>(a, q, lc, cur, ring.issued % NST, lds_addr);
                } else {
                    const int p = cur.pg_lo + 2 * st;
                    const int id0 = uniform_load(cur.pages, p), id1 = p + 1 < cur.pg_hi ? uniform_load(cur.pages, p + 1) : 0;
                    issue_stage<D, KVB, NST>(a, lc, cur, st, id0, id1, ring.issued % NST, lds_addr, ln);
                }
                ring.issued++;
            }
        }
        if (SELF && keep >= -1) {
            // Keep the list for later calls on this schedule (the layers of one decode step), now that the first loads
            // are on their way: the stores cost nothing that way.  (They are younger than those loads, so the waits
            // for the ring's first entries are only stricter for them.)
            uint8_t *dst = a.ws.self_rec + (int64_t)c * kSelfListBytes;
            for (int off = 16 * ln; off < 32 * keep; off += 1024) *(int4 *)(dst + off) = *(const int4 *)(lds + M::kPlanBase + off);
            if (ln == 0) a.ws.self_cnt[c] = keep;
            keep = -2;
        }
        while (has_cur) {
            const bool has_nxt = advance(nxt);
            if (!cur.prefix) {
                if (parked_rows) { // the registers are wanted
                    store_prefix_partial<D, PrefixTiles<KVB>::value>(a, pend, parked_slot, parked_rows, ln);
                    parked_rows = 0;
                }
                run_segment<D, KVB, 1, NST>(a, q, cur, has_nxt, nxt, ring, lc, lds, lds_addr, fresh, pend, false, ln);
                fresh.slot = cur.slot;
                if (npend == NPEND) { // full: write the oldest out
                    store_pending<D>(a, pend[0], ln);
#pragma unroll
                    for (int k = 1; k < NPEND; k++) pend[k - 1] = pend[k];
                    npend = NPEND - 1;
                }
#pragma unroll
                for (int k = 0; k < NPEND; k++)
                    if (k == npend) pend[k] = fresh;
                npend++;
            } else {
                const bool park = npend == 0 && parked_rows == 0;
                run_segment<D, KVB, PrefixTiles<KVB>::value, NST>(a, q, cur, has_nxt, nxt, ring, lc, lds, lds_addr, fresh, pend, park, ln);
                if (park) parked_rows = cur.nrows, parked_slot = cur.slot;
            }
            cur = nxt;
            has_cur = has_nxt;
        }
#pragma unroll
        for (int k = 0; k < NPEND; k++)
            if (k < npend) store_pending<D>(a, pend[k], ln);
        npend = 0;
        if (parked_rows) store_prefix_partial<D, PrefixTiles<KVB>::value>(a, pend, parked_slot, parked_rows, ln);
        parked_rows = 0;
    } while (!sp.done);
}

// Ring depths (in stages of two pages).  bf16 KV: two stages (32 KB, a 4 KB query slot and a 4 KB work list, four
// waves per compute unit) or three.  e4m3 KV: pages are half the size: three stages, or two; these kernels keep one
// finished partial in registers instead of three and are held to half the register file, so that two waves share a SIMD.
template <int D, bool SELF> __global__ __launch_bounds__(64) void attention_kernel_s3(RA_ATTN_PARAMS)
{
    attention_body<D, 2, 3, 3, SELF>(RA_ATTN_ARGS);
}
template <int D, bool SELF> __global__ __launch_bounds__(64) void attention_kernel_s2(RA_ATTN_PARAMS)
{
    attention_body<D, 2, 2, 3, SELF>(RA_ATTN_ARGS);
}
template <int D, bool SELF> __global__ __launch_bounds__(64, 2) void attention_kernel_fp8(RA_ATTN_PARAMS)
{
    attention_body<D, 1, 3, 1, SELF>(RA_ATTN_ARGS);
}
template <int D, bool SELF> __global__ __launch_bounds__(64, 2) void attention_kernel_fp8_s2(RA_ATTN_PARAMS)
{
    attention_body<D, 1, 2, 1, SELF>(RA_ATTN_ARGS);
}

// Bytes of LDS the kernel for (head dim, pool type, ring depth) asks for, and how much of it a wave that plans its
// own span has for its tables (everything before the work list).
static void attention_lds(int D, int kv_fp8, int stages, size_t *bytes, size_t *plan_bytes)
{
#define RA_LDS(DD, KVB, NST) (*bytes = LdsMap<DD, KVB, NST>::kBytes, *plan_bytes = LdsMap<DD, KVB, NST>::kPlanBase)
    if (kv_fp8) {
        if (D == 128) stages == 2 ? RA_LDS(128, 1, 2) : RA_LDS(128, 1, 3);
        else stages == 2 ? RA_LDS(64, 1, 2) : RA_LDS(64, 1, 3);
    } else {
        if (D == 128) stages == 2 ? RA_LDS(128, 2, 2) : RA_LDS(128, 2, 3);
        else stages == 2 ? RA_LDS(64, 2, 2) : RA_LDS(64, 2, 3);
    }
#undef RA_LDS
}
static size_t attention_lds_bytes(int D, int kv_fp8, int stages)
{
    size_t b, p;
    attention_lds(D, kv_fp8, stages, &b, &p);
    return b;
}

bool can_self_plan(int D, int kv_fp8, int stages, int B, int num_groups, int members_per_row)
{
    size_t b, p;
    attention_lds(D, kv_fp8, stages, &b, &p);
    return B <= 64 * kSelfPerLane && num_groups < 64 * kSelfPerLane && wave_tables_bytes(B, num_groups, members_per_row) <= p;
}

static const void *attention_fn(int D, int kv_fp8, int stages, bool self)
{
#define RA_FN(K) (self ? (D == 128 ? (const void *)K<128, true> : (const void *)K<64, true>) : (D == 128 ? (const void *)K<128, false> : (const void *)K<64, false>))
    if (kv_fp8 && stages == 2) return RA_FN(attention_kernel_fp8_s2);
    if (kv_fp8) return RA_FN(attention_kernel_fp8);
    if (stages == 2) return RA_FN(attention_kernel_s2);
    return RA_FN(attention_kernel_s3);
#undef RA_FN
}

hipError_t attention_config(int D, int kv_fp8, int num_cus, int *stages, int *waves)
{
    int st = 2, per_cu = 4;
    if (const char *ev = getenv(kv_fp8 ? "ROLLOUT_ATTN_FP8_STAGES" : "ROLLOUT_ATTN_STAGES")) {
        int v = atoi(ev);
        if (v == 2 || v == 3) st = v;
    }
    size_t lds = attention_lds_bytes(D, kv_fp8, st);
    per_cu = (int)((160u * 1024u) / lds);
    // bf16 pools: one wave per SIMD.  e4m3 pools: a wave spends a larger share of its time converting and multiplying,
    // which a second wave on the same SIMD covers; those kernels are built to fit two waves per SIMD in the register
    // file, so the ring's LDS decides how many are resident (six per compute unit for head dim 128)
    const int cap = kv_fp8 ? 8 : 4;
    if (per_cu > cap) per_cu = cap;
    if (const char *ev = getenv("ROLLOUT_ATTN_WAVES_PER_CU")) {
        int v = atoi(ev);
        if (v >= 1 && v <= 16) per_cu = v;
    }
    for (int self = 0; self < 2; self++) {
        hipError_t e = hipFuncSetAttribute(attention_fn(D, kv_fp8, st, self != 0), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    *stages = st;
    *waves = per_cu * num_cus;
    return hipSuccess;
}

hipError_t launch_attention(const Launch &a, hipStream_t s)
{
    size_t lds = attention_lds_bytes(a.D, a.kv_fp8, a.stages);
    const Workspace &w = a.ws;
#define RA_LAUNCH(K)                                                                                                      \
    hipLaunchKernelGGL(K, dim3(a.waves), dim3(64), lds, s, a, a.q, a.block_table, a.pfx_pages, w.hdr,                       \
                       (const uint32_t *)w.seg_rec, w.members)
#define RA_LAUNCH_D(K)                                                                                                    \
    do {                                                                                                                  \
        if (a.self_plan) {                                                                                                \
            if (a.D == 128) RA_LAUNCH((K<128, true>));                                                                    \
            else RA_LAUNCH((K<64, true>));                                                                                \
        } else {                                                                                                          \
            if (a.D == 128) RA_LAUNCH((K<128, false>));                                                                   \
            else RA_LAUNCH((K<64, false>));                                                                               \
        }                                                                                                                 \
    } while (0)
    if (a.kv_fp8 && a.stages == 2) RA_LAUNCH_D(attention_kernel_fp8_s2);
    else if (a.kv_fp8) RA_LAUNCH_D(attention_kernel_fp8);
    else if (a.stages == 2) RA_LAUNCH_D(attention_kernel_s2);
    else RA_LAUNCH_D(attention_kernel_s3);
#undef RA_LAUNCH_D
#undef RA_LAUNCH
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// streaming probe: what the memory system delivers to the attention kernel's access pattern with no arithmetic
//
// The attention kernel's launch shape (one wave per workgroup, the same LDS footprint, so the same waves on the
// same compute units) and its memory behaviour: a two-slot LDS ring of 16 KB entries fed by direct global->LDS
// loads.  An entry is 16 KB / granule pieces, each read from a place of its own: granule 4096 is the attention
// kernel's pattern (K0 K1 V0 V1 tiles of a 128-wide bf16 head), 16384 one contiguous block per entry.  Places are
// a fixed permutation of the buffer's granules (scattered) or consecutive (sequential: the grid sweeps the buffer).
// ------------------------------------------------------------------------------------------------------

// With chunk > 0 only the first `entries` entries of a wave are its own; after them the waves draw tickets from
// *counter (zero at launch) and ticket t streams the `chunk` entries that follow the static part at t * chunk, until
// the tickets run out: a page stream whose tail is handed out at run time, to be timed against the static split.
__global__ __launch_bounds__(64) void stream_probe_kernel(const uint8_t *__restrict__ buf, uint32_t granule_mask, int granule_shift,
                                                           int scattered, int entries, int chunk, uint32_t tickets, uint32_t *counter,
                                                           long long *clocks)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds;
    const int lane = threadIdx.x;
    const long long t0 = wall_clock64();
    const int per = 14 - granule_shift; // log2 of the pieces per entry
    // entry number e of the sweep into ring slot `slot`: its piece i is granule (e << per) + i
    auto issue = [&](uint32_t e, int slot) __attribute__((always_inline)) {
        const uint32_t first = e << per;
#pragma unroll
        for (int n = 0; n < 16; n++) {
            // load n moves 1 KB: piece (n * 1024) >> granule_shift, offset inside the piece the rest
            const uint32_t piece = (uint32_t)(n * 1024) >> granule_shift, within = (uint32_t)(n * 1024) & ((1u << granule_shift) - 1);
            uint32_t g = first + piece;
            if (scattered & 1) g = g * 2654435761u + 12345u; // odd multiplier: a permutation modulo a power of two
            const uint8_t *src = buf + ((size_t)(g & granule_mask) << granule_shift) + within;
            // streaming loads, as the attention kernel's page loads are (bit 1 of `scattered`: ordinary loads, to compare)
            if (scattered & 2) dma16_base<false>((uint32_t)(16 * lane), src, lds_addr + (slot & 1) * 16384 + 1024 * n);
            else dma16_base<true>((uint32_t)(16 * lane), src, lds_addr + (slot & 1) * 16384 + 1024 * n);
        }
    };
    // The wave's own entries (numbers w, w + waves, ...), then chunks of consecutive entries drawn from the counter,
    // through the two-slot ring without a drain in between: the ticket is asked for while the run's last entry is
    // still in flight, and its wait is that entry's wait.  Every wave leaves when the counter has passed the last ticket.
    uint32_t cur = blockIdx.x, step = gridDim.x;
    int n = entries, slot = 0;
    auto ticket = [&]() __attribute__((always_inline)) {
        uint32_t t = 0;
        if (lane == 0) t = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t = __builtin_amdgcn_readfirstlane(t);
        if (t < tickets) cur = gridDim.x * (uint32_t)entries + t * (uint32_t)chunk, step = 1u, n = chunk;
    };
    if (n <= 0 && chunk > 0) ticket();
    if (n > 0) issue(cur, slot);
    while (n > 0) {
        n--;
        cur += step;
        if (n == 0 && chunk > 0) ticket();
        if (n > 0) {
            issue(cur, slot ^ 1);
            wait_vmcnt<16>();
        } else {
            wait_vmcnt<0>();
        }
        slot ^= 1;
    }
    if (clocks && lane == 0) clocks[blockIdx.x] = wall_clock64() - t0;
}

__global__ void clear_word_kernel(uint32_t *p) { *p = 0; }

hipError_t launch_stream_probe(const void *buf, size_t buf_bytes, int granule, int scattered, int entries, int waves, hipStream_t s,
                               int chunk, uint32_t tickets, uint32_t *counter, long long *clocks)
{
    hipError_t e = hipFuncSetAttribute((const void *)stream_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 40960);
    if (e != hipSuccess) return e;
    int shift = 0;
    while ((1 << shift) < granule) shift++;
    if (chunk > 0) hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, s, counter);
    hipLaunchKernelGGL(stream_probe_kernel, dim3(waves), dim3(64), 40960, s, (const uint8_t *)buf, (uint32_t)((buf_bytes >> shift) - 1), shift,
                       scattered, entries, chunk, tickets, counter, clocks);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// merge: out[b,h] and lse[b,h] from the partials of the shared-prefix row and of the sequence's own spans.
// One workgroup per (sequence, kv head); a thread owns four output elements of one of its G heads.
// With weights w_i = 2^(lse2_i - M): out = sum w_i o_i / sum w_i, lse = (M + log2 sum w_i) ln 2, always in
// the same order (prefix spans, then own spans, by wave), so results are reproducible bit for bit.
// ------------------------------------------------------------------------------------------------------

constexpr int kMergeThreads = 256;

struct PartList {
    int c_lo, c_hi;   // spans that hold pages of the item (c_lo > c_hi: none)
    const float *o;   // partial outputs of span 0 (slot = item + span)
    const float *lse;
    int64_t ostride, lstride;
};

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(Launch a, const int4 *__restrict__ merge_desc,
                                                               const int32_t *__restrict__ seq_pfx_row,
                                                               const int32_t *__restrict__ seq_rank_in_row)
{
    touch_args(a);
    const Workspace &w = a.ws;
    const int item = blockIdx.x, b = item / a.Hkv, kvh = item - b * a.Hkv;
    const int D = a.D, tpr = D / 4; // threads per output row
    int4 own = merge_desc[2 * item], pfx = merge_desc[2 * item + 1];
    int prow = seq_pfx_row[b];
    const int row0 = seq_rank_in_row[b] * a.G;
    if (a.self_plan) {
        // The attention waves that hold an item's first own piece or first shared piece wrote both descriptors (the
        // other one as empty if the item has no such pieces); an item without tokens has no piece and no descriptor.
        if (a.seq_lens[b] <= 0 || a.max_pages <= 0) own.y = pfx.y = 0, own.z = pfx.z = -1;
        if (pfx.y > pfx.z) prow = -1;
    }
    PartList pl[2];
    {
        PartList &p = pl[1];
        p.c_lo = own.y, p.c_hi = own.z;
        p.o = w.suf_o + (int64_t)item * a.G * D;
        p.lse = w.suf_lse + (int64_t)item * a.G;
        p.ostride = (int64_t)a.G * D;
        p.lstride = a.G;
    }
    {
        PartList &p = pl[0];
        p.c_lo = pfx.y, p.c_hi = pfx.z;
        const int64_t pitem = (int64_t)(prow < 0 ? 0 : prow) * a.Hkv + kvh;
        p.o = w.pfx_o + (pitem * a.prefix_rows + row0) * D;
        p.lse = w.pfx_lse + pitem * a.prefix_rows + row0;
        p.ostride = (int64_t)a.prefix_rows * D;
        p.lstride = a.prefix_rows;
    }
    const int npfx = pl[0].c_hi - pl[0].c_lo + 1, nown = pl[1].c_hi - pl[1].c_lo + 1;
    for (int hl = threadIdx.x / tpr; hl < a.G; hl += kMergeThreads / tpr) {
        const int d4 = (threadIdx.x % tpr) * 4;
        float M = -INFINITY, wsum = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (npfx <= 2 && nown <= 4) {
            // the usual case: at most two prefix partials and four own ones; all twelve loads go out together
            constexpr int NP = 6;
            float l[NP];
            f32x4 v[NP];
#pragma unroll
            for (int i = 0; i < NP; i++) {
                const PartList &p = pl[i < 2 ? 0 : 1];
                const int c = p.c_lo + (i < 2 ? i : i - 2);
                const bool have = c <= p.c_hi;
                l[i] = have ? p.lse[c * p.lstride + hl] : -INFINITY;
                v[i] = have ? *(const f32x4 *)(p.o + c * p.ostride + (int64_t)hl * D + d4) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < NP; i++) M = fmaxf(M, l[i]);
#pragma unroll
            for (int i = 0; i < NP; i++) {
                const float wgt = l[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(l[i] - M);
                wsum += wgt;
                acc += wgt * v[i];
            }
        } else {
            for (int k = 0; k < 2; k++)
                for (int c = pl[k].c_lo; c <= pl[k].c_hi; c++) M = fmaxf(M, pl[k].lse[c * pl[k].lstride + hl]);
            for (int k = 0; k < 2; k++)
                for (int c = pl[k].c_lo; c <= pl[k].c_hi; c++) {
                    const float lv = pl[k].lse[c * pl[k].lstride + hl];
                    const float wgt = lv == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(lv - M);
                    wsum += wgt;
                    acc += wgt * *(const f32x4 *)(pl[k].o + c * pl[k].ostride + (int64_t)hl * D + d4);
                }
        }
        const bool empty = wsum == 0.f;
        const float inv = empty ? 0.f : 1.0f / wsum;
        const int64_t bh = (int64_t)b * a.Hq + kvh * a.G + hl;
        bf16x4 ob = __builtin_convertvector(acc * inv, bf16x4);
        *(bf16x4 *)(a.out + bh * D + d4) = ob;
        if (d4 == 0) a.lse[bh] = empty ? -INFINITY : (M + __builtin_amdgcn_logf(wsum)) * 0.6931471805599453f;
    }
}

hipError_t launch_merge(const Launch &a, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    const Workspace &w = a.ws;
    hipLaunchKernelGGL(merge_kernel, dim3(a.B * a.Hkv), dim3(kMergeThreads), 0, s, a, w.merge_desc, w.seq_pfx_row,
                       w.seq_rank_in_row);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// KV append: one new token per sequence into its page (the write before a decode step's attention).
// One wave per (sequence, kv head) writes the K row and the V row.  e4m3 pools quantise on write and keep
// the per-(page, head) scale: a row that fits the page's range uses the page's scale; a larger one sets a
// new scale and the page's stored rows are re-quantised to it.  All of it in binary32, every operation
// rounded once, so the codes are decided exactly as the format's definition says.
// ------------------------------------------------------------------------------------------------------

template <int EPL> // elements per lane: D / 64
__device__ __forceinline__ void append_row(const Launch &a, uint8_t *tile, float *scale_ptr, int slot, const uint16_t *row, int lane)
{
    float x[EPL];
    uint16_t bits[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) {
        bits[e] = row[EPL * lane + e];
        x[e] = __uint_as_float((uint32_t)bits[e] << 16);
    }
    if (!a.kv_fp8) {
        uint16_t *dst = (uint16_t *)(tile + (int64_t)slot * a.stride_token_b) + EPL * lane;
#pragma unroll
        for (int e = 0; e < EPL; e++) dst[e] = bits[e];
        return;
    }
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; e++) amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
    for (int d = 32; d; d >>= 1) amax = fmaxf(amax, __shfl_xor(amax, d));
    float s;
    if (slot == 0) {
        s = amax > 0.f ? amax / 448.0f : 1.0f;
    } else {
        const float old = *scale_ptr;
        if (amax <= old * 448.0f) {
            s = old;
        } else {
            s = amax / 448.0f;
            for (int j = 0; j < slot; j++) {
                uint8_t *p = tile + (int64_t)j * a.stride_token_b + EPL * lane;
#pragma unroll
                for (int e = 0; e < EPL; e++) {
                    const float y = e4m3_value(p[e]) * old;
                    p[e] = (uint8_t)e4m3_nearest(y / s);
                }
            }
        }
    }
    uint8_t *dst = tile + (int64_t)slot * a.stride_token_b + EPL * lane;
#pragma unroll
    for (int e = 0; e < EPL; e++) dst[e] = (uint8_t)e4m3_nearest(x[e] / s);
    if (lane == 0) *scale_ptr = s;
}

__global__ __launch_bounds__(64) void append_kernel(Launch a, const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new)
{
    const int item = blockIdx.x, b = item / a.Hkv, kvh = item - b * a.Hkv, lane = threadIdx.x;
    const int L = a.seq_lens[b];
    if (L < 0 || L >= a.max_pages * kPage) return; // no room in the table row: skipped
    const int pg = a.block_table[(int64_t)b * a.max_pages + L / kPage];
    if (pg < 0 || pg >= a.num_pages) return;       // never write outside the pool
    const int slot = L % kPage;
    const int64_t off = (int64_t)pg * a.stride_page_b + (int64_t)kvh * a.stride_head_b;
    const uint16_t *kr = k_new + (int64_t)item * a.D, *vr = v_new + (int64_t)item * a.D;
    float *ks = const_cast<float *>(a.k_scale) + (int64_t)pg * a.Hkv + kvh;
    float *vs = const_cast<float *>(a.v_scale) + (int64_t)pg * a.Hkv + kvh;
    uint8_t *kt = const_cast<uint8_t *>(a.k_pool) + off, *vt = const_cast<uint8_t *>(a.v_pool) + off;
    if (a.D == 128) {
        append_row<2>(a, kt, ks, slot, kr, lane);
        append_row<2>(a, vt, vs, slot, vr, lane);
    } else {
        append_row<1>(a, kt, ks, slot, kr, lane);
        append_row<1>(a, vt, vs, slot, vr, lane);
    }
}

hipError_t launch_append(const Launch &a, const void *k_new, const void *v_new, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    hipLaunchKernelGGL(append_kernel, dim3(a.B * a.Hkv), dim3(64), 0, s, a, (const uint16_t *)k_new, (const uint16_t *)v_new);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// gather (debug / parity of the page arithmetic) and validation
// ------------------------------------------------------------------------------------------------------

__global__ void gather_kernel(Launch a, int b, int kvh, uint8_t *k_out, uint8_t *v_out, int64_t cap, int row_bytes)
{
    int64_t L = a.seq_lens[b];
    if (L > cap) L = cap;
    const int upr = row_bytes / 16;
    const int64_t total = L * upr;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t t = i / upr;
        const int c = (int)(i - t * upr);
        const int pid = a.block_table[(int64_t)b * a.max_pages + t / kPage];
        const int64_t off = (int64_t)pid * a.stride_page_b + (int64_t)kvh * a.stride_head_b +
                            (int64_t)(t % kPage) * a.stride_token_b + c * 16;
        *(uint4 *)(k_out + t * row_bytes + c * 16) = *(const uint4 *)(a.k_pool + off);
        *(uint4 *)(v_out + t * row_bytes + c * 16) = *(const uint4 *)(a.v_pool + off);
    }
}

hipError_t launch_gather(const Launch &a, int b, int kvh, void *k_out, void *v_out, int64_t cap, hipStream_t s)
{
    int row_bytes = a.D * (a.kv_fp8 ? 1 : 2);
    hipLaunchKernelGGL(gather_kernel, dim3(64), dim3(256), 0, s, a, b, kvh, (uint8_t *)k_out, (uint8_t *)v_out, cap, row_bytes);
    return hipGetLastError();
}

// Flags: 1 length out of range, 2 page id out of range, 4 bad group id / prefix list, 8 member row does not
// start with its group's pages.
__global__ void validate_kernel(Launch a)
{
    const Workspace &w = a.ws;
    int bad = 0;
    const int b = blockIdx.x;
    if (b < a.B) {
        const int L = a.seq_lens[b];
        if (L < 0 || L > a.max_pages * kPage) bad |= 1;
        else {
            const int np = (L + kPage - 1) / kPage;
            for (int i = threadIdx.x; i < np; i += blockDim.x) {
                int pid = a.block_table[(int64_t)b * a.max_pages + i];
                if (pid < 0 || pid >= a.num_pages) bad |= 2;
            }
            if (a.num_groups > 0) {
                const int g = a.seq_group[b];
                if (g < -1 || g >= a.num_groups) bad |= 4;
                else if (g >= 0) {
                    const int o0 = a.pfx_off[g], o1 = a.pfx_off[g + 1];
                    if (o0 >= 0 && o1 >= o0 && (o1 - o0) * kPage <= L)
                        for (int i = threadIdx.x; i < o1 - o0; i += blockDim.x)
                            if (a.block_table[(int64_t)b * a.max_pages + i] != a.pfx_pages[o0 + i]) bad |= 8;
                }
            }
        }
    } else if (a.num_groups > 0) {
        if (threadIdx.x == 0 && a.pfx_off[0] != 0) bad |= 4;
        for (int g = threadIdx.x; g < a.num_groups; g += blockDim.x) {
            const int o0 = a.pfx_off[g], o1 = a.pfx_off[g + 1];
            if (o1 < o0 || o0 < 0) bad |= 4;
            else
                for (int i = o0; i < o1; i++) {
                    int pid = a.pfx_pages[i];
                    if (pid < 0 || pid >= a.num_pages) bad |= 2;
                }
        }
    }
    if (bad) atomicOr(&w.hdr[4], bad);
}

hipError_t launch_validate(const Launch &a, hipStream_t s)
{
    hipError_t e = hipMemsetAsync(a.ws.hdr, 0, 16 * 4, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(validate_kernel, dim3(a.B + 1), dim3(64), 0, s, a);
    return hipGetLastError();
}

} // namespace ra
