// gfx950 kernels of the prompt prefill: causal attention of packed prompts over themselves, and the write of
// their K and V rows into the pages of the cache that the decode steps then read (once per prompt group when
// several responses are sampled for one prompt: paper Sec. 7.1).
//
// Unlike the decode step this is a dense contraction, bound by the matrix cores.  A workgroup of four waves
// takes 256 consecutive query rows of one (prompt, head); the sixteen 16-row query tiles are dealt to the waves
// round-robin, so that under the causal mask every wave has the same amount of work.  K and V stream through an
// LDS ring in stages of 32 keys (K0 K1 V0 V1, one 16-key tile loaded by each wave with direct global->LDS
// loads); every wave multiplies every stage with its own four query tiles, held in registers:
//   S^T[key, row] = K_tile . Q^T,   O^T[d, row] += V_tiles^T . P^T     (16x16x32 MFMA, fp32 accumulation)
// with the softmax running per query row in fp32 (base 2), as in the decode kernel, whose tile layout in LDS
// and operand layouts this kernel shares.
#include "ra_device.h"

namespace ra {

constexpr int kPfWaves = 4;                        // waves per workgroup
constexpr int kPfTiles = 4;                        // 16-row query tiles per wave
constexpr int kPfBlock = 16 * kPfTiles * kPfWaves; // query rows per workgroup
constexpr int kPfSlots = 4;                        // ring slots of one stage (32 keys) each

// One stage of 32 keys against the query tiles TMIN..3 of a wave.  MASKED: the first of those tiles straddles
// the diagonal, so its keys beyond the row are dropped; all later tiles lie wholly below it.
// key0 = index of the stage's first key in the prompt, row0[t] = index of tile t's first row.
template <int D, int TMIN, bool MASKED>
__device__ __forceinline__ void prefill_stage(const uint8_t *st, uint32_t st_addr, const LaneConst<D, 2> &lc, float scale_log2,
                                              int key0, int row0_first, const bf16x8 (&qf)[kPfTiles][D / 32],
                                              f32x4 (&o)[kPfTiles][D / 16], float (&m)[kPfTiles], float (&lsum)[kPfTiles])
{
    using G = Geo<D, 2>;
    const int lane = threadIdx.x & 63, j = lane >> 4;
    f32x4 s[kPfTiles][2];
#pragma unroll
    for (int pg = 0; pg < 2; pg++) {
#pragma unroll
        for (int t = TMIN; t < kPfTiles; t++) s[t][pg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < G::kKReads; i++) {
            const bf16x8 kf = *(const bf16x8 *)(st + pg * G::kTile + lc.k_off[i]);
#pragma unroll
            for (int t = TMIN; t < kPfTiles; t++) s[t][pg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[t][i], s[t][pg], 0, 0, 0);
        }
    }
    bf16x8 pf[kPfTiles];
#pragma unroll
    for (int t = TMIN; t < kPfTiles; t++) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            v[e] = s[t][0][e];
            v[4 + e] = s[t][1][e];
        }
        if (MASKED && t == TMIN) {
            // this lane's row, and its keys 4j+e of the two 16-key tiles
            const int row = row0_first + (lane & 15), k = key0 + 4 * j;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                if (k + e > row) v[e] = -INFINITY;
                if (k + kPage + e > row) v[4 + e] = -INFINITY;
            }
        }
        // the scale is positive, so the maximum may be taken before it is applied
        const float mx = row_max(fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7]))));
        const float mn = fmaxf(m[t], mx * scale_log2);
        f32x8 p;
#pragma unroll
        for (int e = 0; e < 8; e++) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(v[e], scale_log2, -mn));
        const float ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        pf[t] = __builtin_convertvector(p, bf16x8);
        if (__any(mn != m[t])) {
            const float alpha = __builtin_amdgcn_exp2f(m[t] - mn);
            m[t] = mn;
            lsum[t] *= alpha;
#pragma unroll
            for (int dt = 0; dt < G::kDTiles; dt++) o[t][dt] *= alpha;
        }
        lsum[t] += ps;
    }
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4;
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const uint32_t vb = st_addr + 2 * G::kTile;
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; dt++) {
        const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(vb + lc.v_off[dt]));
        const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(vb + G::kTile + lc.v_off[dt]));
        const bf16x8 vf = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int t = TMIN; t < kPfTiles; t++) o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t], o[t][dt], 0, 0, 0);
    }
}

// Grid: (query block, prompt, head), the blocks with the most keys first.  max_len is the host's upper bound of
// a prompt's length; blocks past a prompt's real length leave at once.
template <int D> __global__ __launch_bounds__(64 * kPfWaves) void prefill_kernel(PrefillLaunch a)
{
    using G = Geo<D, 2>;
    constexpr int NST = kPfSlots;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds;
    const int lane = threadIdx.x & 63, j = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);

    const int nqb = (a.max_len + kPfBlock - 1) / kPfBlock;
    int bid = blockIdx.x;
    const int h = bid % a.Hq;
    bid /= a.Hq;
    const int g = bid % a.num_prompts;
    const int q0 = (nqb - 1 - bid / a.num_prompts) * kPfBlock;
    const int t0 = uniform_load(a.cu, g), len = uniform_load(a.cu, g + 1) - t0;
    if (q0 >= len) return; // the whole workgroup
    const int kvh = h / a.G;
    int kend = q0 + kPfBlock;
    kend = kend < len ? kend : len;
    const int nst = (kend + 31) >> 5;

    LaneConst<D, 2> lc;
    lane_setup<D, 2>(lc, lane, a.Hkv * D * 2);

    // wave w loads tile w of a stage's {K0, K1, V0, V1}
    const uint8_t *src_base = (const uint8_t *)((wave < 2 ? a.k : a.v) + ((int64_t)t0 * a.Hkv + kvh) * D);
    const int64_t tok_bytes = (int64_t)a.Hkv * D * 2;
    auto issue = [&](int s) {
        const int tok = 32 * s + kPage * (wave & 1);
        issue_tile<D, 2>(lc, src_base + tok * tok_bytes, len - tok, lds_addr + (s % NST) * G::kStage + wave * G::kTile, a.zeros);
    };
    int issued = 0;
    for (; issued < NST - 1 && issued < nst; issued++) issue(issued);

    // Q^T operand: for k-step i, lane (row = lane % 16, j) holds d = 32 i + 8 j .. + 7 of its row
    bf16x8 qf[kPfTiles][G::kKSteps];
#pragma unroll
    for (int t = 0; t < kPfTiles; t++) {
        const int row = q0 + 16 * (wave + kPfWaves * t) + (lane & 15);
#pragma unroll
        for (int i = 0; i < G::kKSteps; i++) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (row < len) v = *(const bf16x8 *)(a.q + ((int64_t)(t0 + row) * a.Hq + h) * D + 32 * i + 8 * j);
            qf[t][i] = v;
        }
    }
    f32x4 o[kPfTiles][G::kDTiles];
    float m[kPfTiles], lsum[kPfTiles];
#pragma unroll
    for (int t = 0; t < kPfTiles; t++) {
        m[t] = -INFINITY;
        lsum[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int first_diag = q0 >> 5; // stages before this one lie wholly below every row of the block
    for (int s = 0; s < nst; s++) {
        // this wave's loads of stage s have landed ...
        WaitTail<NST - 1, G::kDmaPerTile>::run(issued - 1 - s);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        // ... and so have the other waves'; and everyone is done with stage s - 1, whose slot takes stage s + NST - 1
        if (issued < nst) {
            issue(issued);
            issued++;
        }
        const uint8_t *st = lds + (s % NST) * G::kStage;
        const uint32_t st_addr = lds_addr + (s % NST) * G::kStage;
        const int key0 = 32 * s;
        if (s < first_diag) {
            prefill_stage<D, 0, false>(st, st_addr, lc, a.scale_log2, key0, 0, qf, o, m, lsum);
        } else {
            // tile T = wave + 4 t has a row at or past the stage's first key when T >= 2 (s - first_diag)
            const int need = 2 * (s - first_diag) - wave;
            const int tmin = need <= 0 ? 0 : (need + kPfWaves - 1) / kPfWaves;
            const int row0 = q0 + 16 * (wave + kPfWaves * tmin);
            switch (tmin) {
            case 0: prefill_stage<D, 0, true>(st, st_addr, lc, a.scale_log2, key0, row0, qf, o, m, lsum); break;
            case 1: prefill_stage<D, 1, true>(st, st_addr, lc, a.scale_log2, key0, row0, qf, o, m, lsum); break;
            case 2: prefill_stage<D, 2, true>(st, st_addr, lc, a.scale_log2, key0, row0, qf, o, m, lsum); break;
            case 3: prefill_stage<D, 3, true>(st, st_addr, lc, a.scale_log2, key0, row0, qf, o, m, lsum); break;
            default: break; // every row of this wave lies before the stage
            }
        }
    }

#pragma unroll
    for (int t = 0; t < kPfTiles; t++) {
        const int row = q0 + 16 * (wave + kPfWaves * t) + (lane & 15);
        const float l = row_sum(lsum[t]);
        const float inv = 1.0f / l;
        if (row < len) {
            const int64_t rh = (int64_t)(t0 + row) * a.Hq + h;
            uint16_t *dst = a.out + rh * D + 4 * j;
#pragma unroll
            for (int dt = 0; dt < G::kDTiles; dt++) *(bf16x4 *)(dst + 16 * dt) = __builtin_convertvector(o[t][dt] * inv, bf16x4);
            if (j == 0) a.lse[rh] = (m[t] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
        }
    }
}

hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s)
{
    using G128 = Geo<128, 2>;
    using G64 = Geo<64, 2>;
    const int nqb = (a.max_len + kPfBlock - 1) / kPfBlock;
    const int64_t blocks = (int64_t)nqb * a.num_prompts * a.Hq;
    if (blocks == 0) return hipSuccess;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    if (a.D == 128) {
        constexpr int lds = kPfSlots * G128::kStage;
        hipError_t e = hipFuncSetAttribute((const void *)prefill_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prefill_kernel<128>, dim3((unsigned)blocks), dim3(64 * kPfWaves), lds, s, a);
    } else {
        constexpr int lds = kPfSlots * G64::kStage;
        hipLaunchKernelGGL(prefill_kernel<64>, dim3((unsigned)blocks), dim3(64 * kPfWaves), lds, s, a);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------
// Cache write: one wave per (prompt, page of the prompt, kv head) copies the page's up to sixteen K rows and V
// rows.  bf16 pools take the bit patterns.  e4m3 pools are quantised a page at a time, in binary32: scale =
// (largest magnitude among the rows written) / 448, or 1 when that is zero; code = nearest E4M3 of x / scale.
// ------------------------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void write_tile(const PrefillLaunch &a, const uint16_t *src, int n, uint8_t *dst, float *scale, int lane)
{
    constexpr int kUnits = D * 2 / 16;       // 16-byte units per bf16 row
    constexpr int kIter = kPage * kUnits / 64;
    const int64_t row_elems = (int64_t)a.Hkv * D;
    bf16x8 x[kIter];
#pragma unroll
    for (int i = 0; i < kIter; i++) {
        const int u = lane + 64 * i, r = u / kUnits, c = u % kUnits;
        x[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (r < n) x[i] = *(const bf16x8 *)(src + r * row_elems + 8 * c);
    }
    if (!a.kv_fp8) {
#pragma unroll
        for (int i = 0; i < kIter; i++) {
            const int u = lane + 64 * i, r = u / kUnits, c = u % kUnits;
            if (r < n) *(bf16x8 *)(dst + (int64_t)r * a.stride_token_b + 16 * c) = x[i];
        }
        return;
    }
    float amax = 0.f; // a NaN input does not take part in the maximum
#pragma unroll
    for (int i = 0; i < kIter; i++) {
#pragma unroll
        for (int e = 0; e < 8; e++) amax = fmaxf(amax, fabsf((float)x[i][e]));
    }
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) amax = fmaxf(amax, __shfl_xor(amax, sh));
    const float sc = amax > 0.f ? amax / 448.0f : 1.0f;
#pragma unroll
    for (int i = 0; i < kIter; i++) {
        const int u = lane + 64 * i, r = u / kUnits, c = u % kUnits;
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            lo |= e4m3_nearest((float)x[i][e] / sc) << (8 * e);
            hi |= e4m3_nearest((float)x[i][4 + e] / sc) << (8 * e);
        }
        if (r < n) *(uint2 *)(dst + (int64_t)r * a.stride_token_b + 8 * c) = make_uint2(lo, hi);
    }
    if (lane == 0) *scale = sc;
}

template <int D> __global__ __launch_bounds__(64) void prefill_write_kernel(PrefillLaunch a)
{
    const int lane = threadIdx.x;
    const int npg = (a.max_len + kPage - 1) / kPage;
    int bid = blockIdx.x;
    const int kvh = bid % a.Hkv;
    bid /= a.Hkv;
    const int pi = bid % npg, g = bid / npg;
    const int t0 = uniform_load(a.cu, g), len = uniform_load(a.cu, g + 1) - t0;
    int n = len - kPage * pi;
    n = n < kPage ? n : kPage;
    if (n <= 0) return;
    const int p0 = uniform_load(a.page_off, g), cnt = uniform_load(a.page_off, g + 1) - p0;
    if (pi >= cnt) return; // the caller gave fewer pages than the prompt has: the rest is not cached
    const int pid = uniform_load(a.pages, (int64_t)p0 + pi);
    if (pid < 0 || pid >= a.num_pages) return;
    const int64_t off = (int64_t)pid * a.stride_page_b + (int64_t)kvh * a.stride_head_b;
    const int64_t src = ((int64_t)(t0 + kPage * pi) * a.Hkv + kvh) * D;
    const int64_t si = (int64_t)pid * a.Hkv + kvh;
    write_tile<D>(a, a.k + src, n, a.k_pool + off, a.kv_fp8 ? a.k_scale + si : nullptr, lane);
    write_tile<D>(a, a.v + src, n, a.v_pool + off, a.kv_fp8 ? a.v_scale + si : nullptr, lane);
}

hipError_t launch_prefill_write(const PrefillLaunch &a, hipStream_t s)
{
    const int npg = (a.max_len + kPage - 1) / kPage;
    const int64_t blocks = (int64_t)npg * a.num_prompts * a.Hkv;
    if (blocks == 0) return hipSuccess;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    if (a.D == 128) hipLaunchKernelGGL(prefill_write_kernel<128>, dim3((unsigned)blocks), dim3(64), 0, s, a);
    else hipLaunchKernelGGL(prefill_write_kernel<64>, dim3((unsigned)blocks), dim3(64), 0, s, a);
    return hipGetLastError();
}

} // namespace ra
