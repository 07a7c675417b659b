// gfx950 kernels of rollout_attn: schedule, paged decode attention, log-sum-exp merge, gather, validation.
//
// The decode step is HBM-bound (the rollout phase is memory-bound: paper Sec. 2.1.1), so the design is a
// streaming one: every (page, kv head) tile of K and of V is fetched exactly once with 16-byte-per-lane
// direct global->LDS loads, shared prompt pages once per prompt group (GRPO groups: Sec. 7.1), and the
// ragged lengths (Sec. 7.4) are balanced by cutting the concatenated page stream of all work rows into
// equal spans, one per resident wave.  MFMA does the two tile products; softmax is fp32 on the VALU.
#include "ra_internal.h"

namespace ra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------------------
// workspace
// ------------------------------------------------------------------------------------------------------

int prefix_rows_max(int B, int G, int num_groups)
{
    if (num_groups <= 0) return 0;
    int mpr = kPrefixRows / G;
    long v = (long)num_groups + B / mpr;
    return (int)(v < B ? v : B);
}

size_t carve_workspace(Workspace &ws, void *base, int B, int Hkv, int G, int D, int num_groups, int waves)
{
    size_t off = 0;
    char *p = (char *)base;
    auto take = [&](size_t bytes) {
        void *r = p ? (void *)(p + off) : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return r;
    };
    int ng = num_groups > 0 ? num_groups : 0;
    int prm = prefix_rows_max(B, G, num_groups);
    ws.hdr = (int32_t *)take(16 * 4);
    ws.grp_count = (int32_t *)take((size_t)(ng + 1) * 4);
    ws.grp_rowbase = (int32_t *)take((size_t)(ng + 1) * 4);
    ws.grp_membase = (int32_t *)take((size_t)(ng + 1) * 4);
    ws.seq_rank = (int32_t *)take((size_t)B * 4);
    ws.seq_pfx_row = (int32_t *)take((size_t)B * 4);
    ws.members = (int32_t *)take((size_t)B * 4);
    ws.row_units = (int32_t *)take((size_t)2 * B * 4);
    ws.row_start = (int32_t *)take(((size_t)2 * B + 1) * 4);
    ws.row_info = (int4 *)take((size_t)2 * B * 16);
    ws.wave_first_row = (int32_t *)take((size_t)(waves + 1) * 4);
    size_t nsuf = (size_t)B * Hkv + waves;
    ws.suf_o = (float *)take(nsuf * G * D * 4);
    ws.suf_lse = (float *)take(nsuf * G * 4);
    size_t npfx = prm ? (size_t)prm * Hkv + waves : 0;
    ws.pfx_o = (float *)take(npfx * kPrefixRows * D * 4);
    ws.pfx_lse = (float *)take(npfx * kPrefixRows * 4);
    return off;
}

// ------------------------------------------------------------------------------------------------------
// schedule (one workgroup): work rows, their page counts, the scan, and each wave's first row
// ------------------------------------------------------------------------------------------------------

constexpr int kPlanThreads = 1024;

// Exclusive scan of in[0..n) into out[0..n], out[n] = total.  All threads of the block call it.
__device__ void block_scan(const int32_t *in, int32_t *out, int n, int32_t *lds /*[17]*/)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int carry = 0;
    for (int base = 0; base < n; base += kPlanThreads) {
        int i = base + tid;
        int v = i < n ? in[i] : 0;
        int x = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            int y = __shfl_up(x, d);
            if (lane >= d) x += y;
        }
        if (lane == 63) lds[wv] = x;
        __syncthreads();
        if (wv == 0) {
            int t = lane < kPlanThreads / 64 ? lds[lane] : 0;
            int s = t;
#pragma unroll
            for (int d = 1; d < 16; d <<= 1) {
                int y = __shfl_up(s, d);
                if (lane >= d) s += y;
            }
            if (lane < kPlanThreads / 64) lds[lane] = s - t;
            if (lane == kPlanThreads / 64 - 1) lds[16] = s;
        }
        __syncthreads();
        if (i < n) out[i] = carry + lds[wv] + x - v;
        carry += lds[16];
        __syncthreads();
    }
    if (tid == 0) out[n] = carry;
    __syncthreads();
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(Launch a)
{
    __shared__ int32_t scan_tmp[17];
    const int tid = threadIdx.x;
    const Workspace &w = a.ws;
    const int NG = a.share ? a.num_groups : 0;
    const int MPR = a.members_per_row;

    for (int g = tid; g < NG; g += kPlanThreads) w.grp_count[g] = 0;
    __syncthreads();
    // membership: a sequence uses the shared pass when its group has shared pages and it holds all of them
    for (int b = tid; b < a.B; b += kPlanThreads) {
        int rank = -1;
        if (NG) {
            int g = a.seq_group[b];
            if (g >= 0 && g < NG) {
                int np = a.pfx_off[g + 1] - a.pfx_off[g];
                if (np > 0 && a.seq_lens[b] >= np * kPage) rank = atomicAdd(&w.grp_count[g], 1);
            }
        }
        w.seq_rank[b] = rank;
    }
    __syncthreads();
    int nPR = 0;
    if (NG) {
        block_scan(w.grp_count, w.grp_membase, NG, scan_tmp);
        // rows per group = ceil(count / MPR), scanned in place
        for (int g = tid; g < NG; g += kPlanThreads) w.grp_rowbase[g] = (w.grp_count[g] + MPR - 1) / MPR;
        __syncthreads();
        block_scan(w.grp_rowbase, w.grp_rowbase, NG, scan_tmp);
        nPR = w.grp_rowbase[NG];
    }
    __syncthreads();
    const int B = a.B;
    for (int g = tid; g < NG; g += kPlanThreads) {
        int cnt = w.grp_count[g], np = a.pfx_off[g + 1] - a.pfx_off[g];
        int r0 = w.grp_rowbase[g], m0 = w.grp_membase[g];
        for (int k = 0; k * MPR < cnt; k++) {
            int left = cnt - k * MPR;
            w.row_units[B + r0 + k] = np;
            w.row_info[B + r0 + k] = make_int4(g, m0 + k * MPR, left < MPR ? left : MPR, 0);
        }
    }
    for (int b = tid; b < B; b += kPlanThreads) {
        int L = a.seq_lens[b];
        if (L > a.max_pages * kPage) L = a.max_pages * kPage; // never walk past the table row
        int rank = w.seq_rank[b];
        int skip = 0, prow = -1;
        if (rank >= 0) {
            int g = a.seq_group[b];
            skip = a.pfx_off[g + 1] - a.pfx_off[g];
            prow = w.grp_rowbase[g] + rank / MPR;
            w.members[w.grp_membase[g] + rank] = b;
            w.seq_rank[b] = rank % MPR;
        }
        w.seq_pfx_row[b] = prow;
        int pages = L > 0 ? (L + kPage - 1) / kPage - skip : 0;
        w.row_units[b] = pages;
        w.row_info[b] = make_int4(b, skip, L - skip * kPage, 0);
    }
    __syncthreads();
    const int nR = B + nPR;
    block_scan(w.row_units, w.row_start, nR, scan_tmp);
    const long U = (long)a.Hkv * w.row_start[nR];
    long upw = (U + a.waves - 1) / a.waves;
    if (upw < kMinUnitsPerWave) upw = kMinUnitsPerWave;
    upw += upw & 1;
    if (tid == 0) {
        w.hdr[0] = (int)U;
        w.hdr[1] = (int)upw;
        w.hdr[2] = nR;
        w.hdr[3] = nPR;
    }
    // first row of every wave: the last row whose first unit is <= the wave's first unit
    for (int wv = tid; wv <= a.waves; wv += kPlanThreads) {
        long target = (long)wv * upw;
        int lo = 0, hi = nR; // invariant: Hkv*row_start[lo] <= target
        if (target >= U) lo = nR;
        else
            while (hi - lo > 1) {
                int mid = (lo + hi) >> 1;
                if ((long)a.Hkv * w.row_start[mid] <= target) lo = mid;
                else hi = mid;
            }
        w.wave_first_row[wv] = lo;
    }
}

hipError_t launch_plan(const Launch &a, hipStream_t s)
{
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// attention
// ------------------------------------------------------------------------------------------------------

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// 16 bytes per lane from global memory straight into LDS at lds_addr + lane*16 (no registers in between).
// The compiler does not see these as loads, so their completion is tracked by hand with wait_vmcnt().
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}

// LDS placement of 16-byte unit c of tile row r: rows are kept whole, units are XOR-swizzled inside the
// row so that the 16 rows of an MFMA operand read and the 4 rows of a transposed read spread over banks.
__device__ __forceinline__ int swz(int r) { return 2 * (r & 3) + ((r >> 2) & 1); }

template <int D, int KVB> struct Geo {
    static constexpr int kRowBytes = D * KVB;
    static constexpr int kUnits = kRowBytes / 16;       // 16-byte units per row
    static constexpr int kTile = kPage * kRowBytes;     // one (page, head) tile of K or of V
    static constexpr int kDmaPerTile = kTile / 1024;    // wave-wide 16-byte loads per tile
    static constexpr int kStage = 4 * kTile;            // K0 K1 V0 V1
    static constexpr int kDmaPerStage = 4 * kDmaPerTile;
    static constexpr int kKSteps = D / 32;
    static constexpr int kDTiles = D / 16;
};

template <int D, int KVB> struct LaneConst {
    int dma_row[Geo<D, KVB>::kDmaPerTile];
    int dma_off[Geo<D, KVB>::kDmaPerTile];
    int k_off[Geo<D, KVB>::kKSteps];
    int v_off[Geo<D, KVB>::kDTiles];
};

template <int D, int KVB> __device__ __forceinline__ void lane_setup(LaneConst<D, KVB> &lc, int lane, int stride_token_b)
{
    using G = Geo<D, KVB>;
    constexpr int UM = G::kUnits - 1;
#pragma unroll
    for (int n = 0; n < G::kDmaPerTile; n++) {
        int slot = 64 * n + lane;
        int r = slot / G::kUnits, cp = slot % G::kUnits;
        int c = cp ^ (swz(r) & UM);
        lc.dma_row[n] = r;
        lc.dma_off[n] = r * stride_token_b + c * 16;
    }
    const int r = lane & 15, j = lane >> 4;
#pragma unroll
    for (int i = 0; i < G::kKSteps; i++) lc.k_off[i] = 16 * (r * G::kUnits + ((4 * i + j) ^ (swz(r) & UM)));
    const int a = lane & 15;
    const int vrow = 4 * j + (a >> 2);
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; dt++) {
        int c = 2 * dt + ((a >> 1) & 1);
        lc.v_off[dt] = 16 * (vrow * G::kUnits + (c ^ (swz(vrow) & UM))) + 8 * (a & 1);
    }
}

// One tile: rows at or past nvalid come from the zero block instead (so stale or poisoned slots never reach
// the MFMA, and a page id is only dereferenced when the page exists).
template <int D, int KVB>
__device__ __forceinline__ void issue_tile(const LaneConst<D, KVB> &lc, const uint8_t *tile, int nvalid, uint32_t lds_addr,
                                           const void *zeros)
{
    using G = Geo<D, KVB>;
#pragma unroll
    for (int n = 0; n < G::kDmaPerTile; n++) {
        const void *src = lc.dma_row[n] < nvalid ? (const void *)(tile + lc.dma_off[n]) : zeros;
        dma16(src, lds_addr + 1024 * n);
    }
}

struct Segment {
    const int32_t *__restrict__ pages; // page ids of the work row (uniform)
    int pg_lo, pg_hi;     // pages of the row this wave covers
    int limit;            // tokens of the row that exist and belong to this span: min(valid, 16*pg_hi)
    int kvh;
};

// Attention of NQT*16 query rows over the pages [pg_lo, pg_hi) of one work row; writes the normalised
// partial output and its log2-sum-exp.
//   S^T[key, row] = K_tile . Q^T      (A = K rows straight from LDS, B = Q held in registers)
//   O^T[d, row]  += V_tile^T . P^T    (A = V through the transposing LDS read, B = P repacked in place)
// In both products a lane owns one query row (lane % 16), so the running max, the rescale factor and the
// row sum are per-lane scalars; only the row max needs a cross-lane step (lanes l, l^16, l^32, l^48).
template <int D, int NQT>
__device__ __forceinline__ void run_segment(const Launch &a, const uint16_t *__restrict__ q, const Segment &sg,
                                            const LaneConst<D, 2> &lc, uint8_t *lds, uint32_t lds_addr,
                                            const int (&qrow_seq)[NQT], const int (&qrow_head)[NQT], float *part_o,
                                            float *part_lse, int part_rows)
{
    using G = Geo<D, 2>;
    const int lane = threadIdx.x, j = lane >> 4;

    const int npages = sg.pg_hi - sg.pg_lo;
    const int niter = (npages + 1) >> 1;

    auto tile_ptr = [&](const uint8_t *pool, int pid) {
        return pool + (int64_t)pid * a.stride_page_b + (int64_t)sg.kvh * a.stride_head_b;
    };
    auto issue = [&](int it, int pid0, int pid1) {
        const int p0 = sg.pg_lo + 2 * it;
        int nv0 = sg.limit - p0 * kPage, nv1 = nv0 - kPage;
        nv0 = nv0 > kPage ? kPage : nv0;
        nv1 = nv1 > kPage ? kPage : (nv1 < 0 ? 0 : nv1);
        const uint32_t sb = lds_addr + (it % kStages) * G::kStage;
        issue_tile<D, 2>(lc, tile_ptr(a.k_pool, pid0), nv0, sb, a.zeros);
        issue_tile<D, 2>(lc, tile_ptr(a.k_pool, pid1), nv1, sb + G::kTile, a.zeros);
        issue_tile<D, 2>(lc, tile_ptr(a.v_pool, pid0), nv0, sb + 2 * G::kTile, a.zeros);
        issue_tile<D, 2>(lc, tile_ptr(a.v_pool, pid1), nv1, sb + 3 * G::kTile, a.zeros);
    };
    auto page_id = [&](int it, int h) {
        int p = sg.pg_lo + 2 * it + h;
        return p < sg.pg_hi ? sg.pages[p] : 0;
    };

    // page ids run one stage ahead of the loads that use them
    int nid0 = page_id(0, 0), nid1 = page_id(0, 1);
#pragma unroll
    for (int s = 0; s < kStages - 1; s++)
        if (s < niter) {
            issue(s, nid0, nid1);
            nid0 = page_id(s + 1, 0);
            nid1 = page_id(s + 1, 1);
        }

    // Q^T operand: lane (row = lane%16, j) holds d = 32*i + 8*j .. +7 of its row for k-step i
    bf16x8 qf[NQT][G::kKSteps];
#pragma unroll
    for (int t = 0; t < NQT; t++) {
#pragma unroll
        for (int i = 0; i < G::kKSteps; i++) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (qrow_seq[t] >= 0)
                v = *(const bf16x8 *)(q + ((int64_t)qrow_seq[t] * a.Hq + qrow_head[t]) * D + 32 * i + 8 * j);
            qf[t][i] = v;
        }
    }
    // Make the compiler wait for the query loads here, once, instead of at their first use inside the loop
    // (where a full vector-memory wait would drain the ring every iteration).
#pragma unroll
    for (int t = 0; t < NQT; t++) {
#pragma unroll
        for (int i = 0; i < G::kKSteps; i++) asm volatile("" ::"v"(qf[t][i]));
    }

    f32x4 o[NQT][G::kDTiles];
    float m[NQT], lsum[NQT];
#pragma unroll
    for (int t = 0; t < NQT; t++) {
        m[t] = -INFINITY;
        lsum[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int it = 0; it < niter; it++) {
        if (it + kStages - 1 < niter) {
            issue(it + kStages - 1, nid0, nid1);
            nid0 = page_id(it + kStages, 0);
            nid1 = page_id(it + kStages, 1);
            wait_vmcnt<(kStages - 1) * G::kDmaPerStage>();
        } else {
            wait_vmcnt<0>();
        }
        const uint8_t *st = lds + (it % kStages) * G::kStage;

        // scores
        f32x4 s[NQT][2];
#pragma unroll
        for (int pg = 0; pg < 2; pg++) {
#pragma unroll
            for (int t = 0; t < NQT; t++) s[t][pg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < G::kKSteps; i++) {
                bf16x8 kf = *(const bf16x8 *)(st + pg * G::kTile + lc.k_off[i]);
#pragma unroll
                for (int t = 0; t < NQT; t++)
                    s[t][pg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[t][i], s[t][pg], 0, 0, 0);
            }
        }
        const int tok0 = (sg.pg_lo + 2 * it) * kPage + 4 * j; // this lane's first token in page 0 of the stage
        const bool ragged = (sg.pg_lo + 2 * it + 2) * kPage > sg.limit;
        bf16x8 pf[NQT];
#pragma unroll
        for (int t = 0; t < NQT; t++) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                v[e] = s[t][0][e] * a.scale_log2;
                v[4 + e] = s[t][1][e] * a.scale_log2;
            }
            if (ragged) {
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    if (tok0 + e >= sg.limit) v[e] = -INFINITY;
                    if (tok0 + kPage + e >= sg.limit) v[4 + e] = -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mn = fmaxf(m[t], mx);
            const float alpha = __builtin_amdgcn_exp2f(m[t] - mn);
            m[t] = mn;
            f32x8 p;
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                p[e] = __builtin_amdgcn_exp2f(v[e] - mn);
                ps += p[e];
            }
            lsum[t] = lsum[t] * alpha + ps;
            pf[t] = __builtin_convertvector(p, bf16x8);
#pragma unroll
            for (int dt = 0; dt < G::kDTiles; dt++) o[t][dt] *= alpha;
        }
        // O^T += V^T P^T
        typedef s16x4 __attribute__((address_space(3))) * lds_s16x4;
        const uint32_t vb = lds_addr + (it % kStages) * G::kStage + 2 * G::kTile;
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++) {
            s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(vb + lc.v_off[dt]));
            s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(vb + G::kTile + lc.v_off[dt]));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
            bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
            for (int t = 0; t < NQT; t++) o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t], o[t][dt], 0, 0, 0);
        }
        // every LDS read of this stage has returned before a later load may overwrite it
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }

    // normalise and store the partial
#pragma unroll
    for (int t = 0; t < NQT; t++) {
        float l = lsum[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int row = 16 * t + (lane & 15);
        if (row < part_rows) {
            const float inv = 1.0f / l;
            float *dst = part_o + (int64_t)row * D + 4 * j;
#pragma unroll
            for (int dt = 0; dt < G::kDTiles; dt++) *(f32x4 *)(dst + 16 * dt) = o[t][dt] * inv;
            if (j == 0) part_lse[row] = m[t] + __builtin_amdgcn_logf(l);
        }
    }
}

// The read-only inputs and the schedule come in as separate restrict pointers so that the compiler can keep
// every wave-uniform lookup (page ids, row bounds) on the scalar unit, away from the vector-memory counter
// that paces the LDS ring.
template <int D>
__global__ __launch_bounds__(64) void attention_kernel(Launch a, const uint16_t *__restrict__ q,
                                                       const int32_t *__restrict__ block_table,
                                                       const int32_t *__restrict__ pfx_off,
                                                       const int32_t *__restrict__ pfx_pages, const int32_t *__restrict__ hdr,
                                                       const int32_t *__restrict__ row_start, const int4 *__restrict__ row_info,
                                                       const int32_t *__restrict__ wave_first_row,
                                                       const int32_t *__restrict__ members)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds;
    const Workspace &w = a.ws;
    const int lane = threadIdx.x;
    const int wave = blockIdx.x;
    const int U = hdr[0], upw = hdr[1];
    int u = wave * upw;
    const int u_hi = min(U, u + upw);
    if (u >= u_hi) return;

    LaneConst<D, 2> lc;
    lane_setup<D, 2>(lc, lane, a.stride_token_b);

    int r = wave_first_row[wave];
    while (u < u_hi) {
        while (a.Hkv * row_start[r + 1] <= u) r++;
        const int rs = row_start[r];
        const int units = row_start[r + 1] - rs;
        const int rel = u - a.Hkv * rs;
        Segment sg;
        sg.kvh = rel / units;
        sg.pg_lo = rel - sg.kvh * units;
        sg.pg_hi = min(units, sg.pg_lo + (u_hi - u));
        const int4 info = row_info[r];
        if (r < a.B) {
            // a sequence's own pages: the G query heads of this kv head form one 16-row tile
            const int b = info.x;
            sg.pages = block_table + (int64_t)b * a.max_pages + info.y;
            sg.limit = min(info.z, sg.pg_hi * kPage);
            const int slot = r * a.Hkv + sg.kvh + wave;
            int qs[1], qh[1];
            const int row = lane & 15;
            qs[0] = row < a.G ? b : -1;
            qh[0] = sg.kvh * a.G + row;
            run_segment<D, 1>(a, q, sg, lc, lds, lds_addr, qs, qh, w.suf_o + (int64_t)slot * a.G * D,
                              w.suf_lse + (int64_t)slot * a.G, a.G);
        } else {
            // shared prompt pages of a group: rows = members x G, packed densely into four 16-row tiles
            const int g = info.x;
            sg.pages = pfx_pages + pfx_off[g];
            sg.limit = sg.pg_hi * kPage;
            const int slot = (r - a.B) * a.Hkv + sg.kvh + wave;
            const int nrows = info.z * a.G;
            int qs[4], qh[4];
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const int row = 16 * t + (lane & 15);
                const int mi = row / a.G;
                qs[t] = row < nrows ? members[info.y + mi] : -1;
                qh[t] = sg.kvh * a.G + (row - mi * a.G);
            }
            run_segment<D, 4>(a, q, sg, lc, lds, lds_addr, qs, qh, w.pfx_o + (int64_t)slot * kPrefixRows * D,
                              w.pfx_lse + (int64_t)slot * kPrefixRows, nrows);
        }
        u += sg.pg_hi - sg.pg_lo;
    }
}

static size_t attention_lds_bytes(int D) { return (size_t)kStages * (D == 128 ? Geo<128, 2>::kStage : Geo<64, 2>::kStage); }

hipError_t attention_waves(int D, int kv_fp8, int num_cus, int *waves)
{
    (void)kv_fp8;
    const void *fn = D == 128 ? (const void *)attention_kernel<128> : (const void *)attention_kernel<64>;
    size_t lds = attention_lds_bytes(D);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    if (per_cu > 4) per_cu = 4; // one wave per SIMD; more adds nothing once HBM is saturated
    *waves = per_cu * num_cus;
    return hipSuccess;
}

hipError_t launch_attention(const Launch &a, hipStream_t s)
{
    size_t lds = attention_lds_bytes(a.D);
    const Workspace &w = a.ws;
    if (a.D == 128)
        hipLaunchKernelGGL(attention_kernel<128>, dim3(a.waves), dim3(64), lds, s, a, a.q, a.block_table, a.pfx_off, a.pfx_pages,
                           w.hdr, w.row_start, w.row_info, w.wave_first_row, w.members);
    else
        hipLaunchKernelGGL(attention_kernel<64>, dim3(a.waves), dim3(64), lds, s, a, a.q, a.block_table, a.pfx_off, a.pfx_pages,
                           w.hdr, w.row_start, w.row_info, w.wave_first_row, w.members);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// merge: out[b,h] and lse[b,h] from the partials of the shared-prefix row and of the sequence's own spans
// ------------------------------------------------------------------------------------------------------

__global__ void merge_kernel(Launch a)
{
    const Workspace &w = a.ws;
    const int bh = blockIdx.x, b = bh / a.Hq, h = bh - b * a.Hq;
    const int kvh = h / a.G, hl = h - kvh * a.G;
    const int d = threadIdx.x;
    const int upw = w.hdr[1];
    const int D = a.D;

    // two lists of partials: [0] own pages (row b), [1] shared prefix (row B + seq_pfx_row[b])
    const float *po[2], *pl[2];
    int cnt[2];
    int64_t ostride[2], lstride[2];
    {
        const int units = w.row_start[b + 1] - w.row_start[b];
        const int64_t s0 = (int64_t)a.Hkv * w.row_start[b] + (int64_t)kvh * units;
        const int w_lo = (int)(s0 / upw), w_hi = units > 0 ? (int)((s0 + units - 1) / upw) : w_lo - 1;
        const int64_t slot = (int64_t)b * a.Hkv + kvh + w_lo;
        po[0] = w.suf_o + (slot * a.G + hl) * D;
        pl[0] = w.suf_lse + slot * a.G + hl;
        ostride[0] = (int64_t)a.G * D;
        lstride[0] = a.G;
        cnt[0] = w_hi - w_lo + 1;
    }
    const int prow = w.seq_pfx_row[b];
    if (prow >= 0) {
        const int r = a.B + prow;
        const int units = w.row_start[r + 1] - w.row_start[r];
        const int64_t s0 = (int64_t)a.Hkv * w.row_start[r] + (int64_t)kvh * units;
        const int w_lo = (int)(s0 / upw), w_hi = (int)((s0 + units - 1) / upw);
        const int64_t slot = (int64_t)prow * a.Hkv + kvh + w_lo;
        const int row = w.seq_rank[b] * a.G + hl;
        po[1] = w.pfx_o + (slot * kPrefixRows + row) * D;
        pl[1] = w.pfx_lse + slot * kPrefixRows + row;
        ostride[1] = (int64_t)kPrefixRows * D;
        lstride[1] = kPrefixRows;
        cnt[1] = w_hi - w_lo + 1;
    } else {
        cnt[1] = 0;
        po[1] = po[0];
        pl[1] = pl[0];
        ostride[1] = lstride[1] = 0;
    }
    float M = -INFINITY;
    for (int k = 0; k < 2; k++)
        for (int i = 0; i < cnt[k]; i++) M = fmaxf(M, pl[k][i * lstride[k]]);
    float acc = 0.f, wsum = 0.f;
    for (int k = 1; k >= 0; k--) // fixed order: shared prefix first, then own spans in token order
        for (int i = 0; i < cnt[k]; i++) {
            const float wgt = __builtin_amdgcn_exp2f(pl[k][i * lstride[k]] - M);
            wsum += wgt;
            acc += wgt * po[k][i * ostride[k] + d];
        }
    const bool empty = cnt[0] + cnt[1] == 0;
    const float res = empty ? 0.f : acc / wsum;
    __bf16 ob = (__bf16)res;
    a.out[(int64_t)bh * D + d] = __builtin_bit_cast(uint16_t, ob);
    if (d == 0) a.lse[bh] = empty ? -INFINITY : (M + __builtin_amdgcn_logf(wsum)) * 0.6931471805599453f;
}

hipError_t launch_merge(const Launch &a, hipStream_t s)
{
    if (a.B == 0) return hipSuccess;
    hipLaunchKernelGGL(merge_kernel, dim3(a.B * a.Hq), dim3(a.D), 0, s, a);
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
