// gfx950 kernels of the prompt prefill: causal attention of packed prompts over themselves, and the write of
// their K and V rows into the pages of the cache that the decode steps then read (once per prompt group when
// several responses are sampled for one prompt: paper Sec. 7.1).
//
// Unlike the decode step this is a dense contraction, bound by the matrix cores.  A workgroup of eight waves
// (two per SIMD, so that one wave's vector work runs while the other's MFMAs do) takes 256 consecutive query
// rows of one (prompt, head), 32 rows per wave.  K and V stream through an LDS ring in chunks of two stages of 32
// keys (K0 K1 V0 V1 | K2 K3 V2 V3, one 16-key tile loaded by each wave with direct global->LDS loads); every wave
// multiplies every stage with its own query rows, held in registers:
//   S^T[key, row] = K . Q^T,   O^T[d, row] += V^T . P^T     (32x32x16 MFMA, fp32 accumulation)
// with the softmax running per query row in fp32 (base 2).  The tile layout in LDS is the decode kernel's.
#include "ra_device.h"

namespace ra {

constexpr int kPfWaves = 8;                  // waves per workgroup, two per SIMD
constexpr int kPfRows = 32;                  // query rows per wave: one 32x32 MFMA tile
constexpr int kPfBlock = kPfRows * kPfWaves; // query rows per workgroup
constexpr int kPfSlots = 4;                  // ring slots of one chunk (two stages of 32 keys) each

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Per-lane constants of the 32x32x16 products.  A lane is (n = lane % 32, hh = lane / 32).  With the tile layout
// of lane_setup() (rows of D bf16, 16-byte units XOR-swizzled inside the row) every LDS address the step needs is
// one of two per-lane bases XOR a compile-time constant, as long as stages start at multiples of their size:
//   K operand of k-step i (key n, d = 16 i + 8 hh .. + 7):          stage + (k_base ^ 32 i)
//   V operand, d-tile dt, keys 4 hh + 8 rd .. + 3 of tile V0 / V1:  stage + 2 tiles (+ 1) + (v_base ^ 64 dt ^ kVrd rd)
// the latter through the transposing read, whose 16 lanes address a 4-key x 16-d block, lane a supplying key a / 4,
// d = 4 (a % 4) .. + 3.
template <int D> struct PfLane {
    int k_base, v_base;
};

template <int D> __device__ __forceinline__ void pf_lane_setup(PfLane<D> &pl, int lane)
{
    using G = Geo<D, 2>;
    constexpr int UM = G::kUnits - 1;
    const int n = lane & 31, hh = lane >> 5;
    const int r = n & 15;
    // unit (2 i + hh) ^ swz(r) = 2 i ^ (swz(r) ^ hh)
    pl.k_base = (n >> 4) * G::kTile + G::kRowBytes * r + 16 * ((swz(r) & UM) ^ hh);
    const int a = lane & 15, dh = (lane >> 4) & 1;
    const int vrow = 4 * hh + (a >> 2);           // + 8 rd
    const int c = 2 * dh + ((a >> 1) & 1);        // + 4 dt
    pl.v_base = G::kRowBytes * vrow + 16 * (c ^ (swz(vrow) & UM)) + 8 * (a & 1);
}
template <int D> __device__ __forceinline__ int pf_k_off(const PfLane<D> &pl, int i) { return pl.k_base ^ (32 * i); }
template <int D> __device__ __forceinline__ int pf_v_off(const PfLane<D> &pl, int dt, int rd)
{
    // eight rows further on; with sixteen units per row the swizzle of those rows differs in its top bit
    constexpr int kVrd = 8 * Geo<D, 2>::kRowBytes + (Geo<D, 2>::kUnits == 16 ? 128 : 0);
    return pl.v_base ^ ((64 * dt) ^ (kVrd * rd));
}

template <int D> struct PfState {
    bf16x8 qf[D / 16]; // Q^T operand of k-step i: row n, d = 16 i + 8 hh .. + 7
    f32x16 o[D / 32];  // O^T accumulators: element e of d-tile dt is d = 32 dt + 8 (e / 4) + 4 hh + e % 4, row n
    f32x16 s;          // scores of the stage whose weights are computed next: element e is key 8 (e / 4) + 4 hh + e % 4
    float m, lsum;     // reference point of the exponent (same in both lanes of a row); this lane's part of the row sum
};

// max(a, b, c) as the instruction computes it.  (Through fmaxf the compiler first quiets possible signalling NaNs of
// every operand with an instruction of its own, which doubles the cost of the reduction.)  The compiler does not
// look inside: it pads the distance between an MFMA and a vector instruction that reads its result only for
// instructions it knows, so the first read of an MFMA's accumulator must not be one of these (see first_max).
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// The first step of a maximum over fresh MFMA results, by an instruction the compiler knows; once it has run, the
// whole accumulator (one MFMA writes all of it) is safe to read.
__device__ __forceinline__ float first_max(float a, float b) { return fmaxf(a, b); }

constexpr float kPfSlack = 8.0f;

// One step of a wave's software pipeline (see the kernel): weights of stage s and scores of stage s + 1 (NEXT; MASK:
// that stage is the wave's diagonal one), then O += P V of stage s and the row maxima of the new scores.
template <int D, bool MASK, bool NEXT>
__device__ __forceinline__ void pf_step(PfState<D> &st, const uint8_t *k_next, uint32_t v_addr, const PfLane<D> &pl,
                                        float scale_log2, int key_next, int row)
{
    using G = Geo<D, 2>;
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4;
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const int hh = (threadIdx.x & 63) >> 5;
    constexpr int KS = D / 16, DT = D / 32;
#define PF_FENCE() __builtin_amdgcn_sched_barrier(0)
    PF_FENCE();
    // K operands are read four products ahead of their use
    constexpr int KA = KS < 4 ? KS : 4;
    bf16x8 kf[KS];
    if (NEXT) {
#pragma unroll
        for (int i = 0; i < KA; i++) kf[i] = *(const bf16x8 *)(k_next + pf_k_off(pl, i));
    }
    s16x4 vr[DT][2][2];
    auto v_read = [&](int dt, int kk) {
        vr[dt][kk][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(v_addr + kk * G::kTile + pf_v_off(pl, dt, 0)));
        vr[dt][kk][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(v_addr + kk * G::kTile + pf_v_off(pl, dt, 1)));
    };
    PF_FENCE();
    // weights: item k < 16: element k (exponential, running sum, and with every second one the rounding of a pair to
    // bf16); item 16: the row sum
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    u32x4 pw[2];
    float pprev = 0.f, acc0 = 0.f, acc1 = 0.f;
    auto w_item = [&](int k) {
        if (k < 16) {
            const float pk = __builtin_amdgcn_exp2f(__builtin_fmaf(st.s[k], scale_log2, -st.m));
            if (k & 1) {
                acc1 += pk;
                pw[k >> 3][(k >> 1) & 3] = __builtin_bit_cast(unsigned, __builtin_convertvector((f32x2{pprev, pk}), bf16x2));
            } else {
                acc0 += pk;
                pprev = pk;
            }
        } else {
            st.lsum += acc0 + acc1;
        }
    };
    constexpr int NW = 17;
    f32x16 sn;
    if (NEXT) {
        // the first weights cover the latency of the K reads
#pragma unroll
        for (int k = 0; k < 3; k++) w_item(k);
        PF_FENCE();
#pragma unroll
        for (int i = 0; i < KS; i++) {
            if (i == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) sn[e] = 0.f;
            }
            sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], st.qf[i], sn, 0, 0, 0);
            if (i + KA < KS) kf[i + KA] = *(const bf16x8 *)(k_next + pf_k_off(pl, i + KA));
#pragma unroll
            for (int w = 3 + i * (NW - 3) / KS; w < 3 + (i + 1) * (NW - 3) / KS; w++) w_item(w);
            if (i >= KS - DT) v_read((i - (KS - DT)) / 2, (i - (KS - DT)) % 2);
            PF_FENCE();
        }
    } else {
#pragma unroll
        for (int n = 0; n < DT; n++) v_read(n / 2, n % 2);
#pragma unroll
        for (int w = 0; w < NW; w++) w_item(w);
        PF_FENCE();
    }
    // O^T += V^T P^T; in the MFMAs' shadow the mask and the maxima of the new scores.
    // item k: 0..3 the causal mask (MASK), 4..11 partial maxima, 12 the exchange, 13 the end
    float mx = 0.f, mn = 0.f;
    bool grew = false;
    auto m_item = [&](int k) {
        if (k < 4) {
            if (MASK) {
                // element e = 4 k + x is key 8 k + 4 hh + x of the stage
                const int kk = key_next + 8 * k + 4 * hh;
#pragma unroll
                for (int x = 0; x < 4; x++) {
                    if (kk + x > row) sn[4 * k + x] = -INFINITY;
                }
            }
        } else if (k == 4) {
            mx = max3(first_max(sn[0], sn[1]), sn[2], sn[2]);
        } else if (k < 11) {
            mx = max3(mx, sn[2 * k - 7], sn[2 * k - 6]); // k = 5..10: elements 3..14
        } else if (k == 11) {
            mx = max3(mx, sn[15], sn[15]);
        } else if (k == 12) {
            const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
            mx = max3(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[1]));
        } else {
            mn = mx * scale_log2; // the scale is positive, so the maximum may be taken before it is applied
            grew = mn > st.m + kPfSlack;
            st.s = sn;
        }
    };
    constexpr int NMI = NEXT ? 14 : 0;
    constexpr int NPV = 2 * DT;
#pragma unroll
    for (int n = 0; n < NPV; n++) {
        const int dt = n / 2, kk = n % 2;
        if (n + DT < NPV) v_read((n + DT) / 2, (n + DT) % 2); // four products ahead of its use
        const bf16x8 vf = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(vr[dt][kk][0], vr[dt][kk][1], 0, 1, 2, 3, 4, 5, 6, 7));
        st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, pw[kk]), st.o[dt], 0, 0, 0);
#pragma unroll
        for (int w = n * NMI / NPV; w < (n + 1) * NMI / NPV; w++) m_item(w);
        PF_FENCE();
    }
    if (NEXT) {
        if (__any(grew)) {
            mn = mn > st.m ? mn : st.m;
            const float alpha = __builtin_amdgcn_exp2f(st.m - mn);
            st.m = mn;
            st.lsum *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; dt++) st.o[dt] *= alpha;
        }
    }
#undef PF_FENCE
}

// Scores of a stage for the wave's rows (no vector work to overlap with: used once, for the first stage).  All K
// operands are read first and the products go to two accumulators in turn, so that neither the LDS latency nor the
// MFMA latency is paid once per k-step.
template <int D>
__device__ __forceinline__ void pf_scores(const uint8_t *k_stage, const PfLane<D> &pl, const bf16x8 (&qf)[D / 16], f32x16 &sn)
{
    bf16x8 kf[D / 16];
#pragma unroll
    for (int i = 0; i < D / 16; i++) kf[i] = *(const bf16x8 *)(k_stage + pf_k_off(pl, i));
    f32x16 s2;
#pragma unroll
    for (int e = 0; e < 16; e++) sn[e] = s2[e] = 0.f;
#pragma unroll
    for (int i = 0; i < D / 16; i += 2) {
        sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[i], sn, 0, 0, 0);
        s2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i + 1], qf[i + 1], s2, 0, 0, 0);
    }
    sn += s2;
}

// One workgroup per (prompt, head, block of 256 query rows).  max_len is the host's upper bound of a prompt's
// length; blocks past a prompt's real length leave at once.
template <int D> __global__ __launch_bounds__(64 * kPfWaves) void prefill_kernel(PrefillLaunch a)
{
    using G = Geo<D, 2>;
    constexpr int NSL = kPfSlots;           // ring slots; a stage s lives at (s % (2 NSL)) * G::kStage
    static_assert((NSL & (NSL - 1)) == 0, "slot arithmetic by masking");
    extern __shared__ __attribute__((aligned(16384))) uint8_t lds[]; // the step forms LDS addresses by XOR
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds;
    const int lane = threadIdx.x & 63, n = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);

    // Workgroups are dealt to the eight dies round-robin, and each die has its own L2.  All workgroups of a
    // (prompt, kv head) pair, which read the same K and V, therefore go to one die: die x takes the pairs x, x + 8,
    // ... one after the other, each with its query blocks from the longest down and the heads of the kv head together.
    const int nqb = (a.max_len + kPfBlock - 1) / kPfBlock;
    const int per_pair = nqb * a.G;
    const int die = blockIdx.x & 7, turn = blockIdx.x >> 3;
    const int pair = (turn / per_pair) * 8 + die, r = turn % per_pair;
    if (pair >= a.num_prompts * a.Hkv) return; // the whole workgroup
    const int g = pair / a.Hkv, kvh = pair % a.Hkv;
    const int h = kvh * a.G + r % a.G;
    const int q0 = (nqb - 1 - r / a.G) * kPfBlock;
    const int t0 = uniform_load(a.cu, g), len = uniform_load(a.cu, g + 1) - t0;
    if (q0 >= len) return; // the whole workgroup
    int kend = q0 + kPfBlock;
    kend = kend < len ? kend : len;
    const int nst = (kend + 31) >> 5;

    LaneConst<D, 2> lc;
    lane_setup<D, 2>(lc, lane, a.Hkv * D * 2);
    PfLane<D> pl;
    pf_lane_setup<D>(pl, lane);

    // waves 0..3 load the chunks {K0 K1 V0 V1 | K2 K3 V2 V3}: wave w brings tile w of both stages.  (Waves 4..7, the
    // second on each SIMD, are the ones that arrive last at the barriers; they issue no loads.)
    constexpr int DPW = 2 * G::kDmaPerTile; // loads of a loading wave per chunk
    const int nchunks = (nst + 1) >> 1;
    const int tile = wave & 3;
    const bool loader = wave < 4;
    int tok = kPage * (tile & 1); // first key of the wave's tile in the chunk to load next
    const int64_t tok_bytes = (int64_t)a.Hkv * D * 2;
    const uint8_t *src = (const uint8_t *)((tile < 2 ? a.k : a.v) + ((int64_t)(t0 + tok) * a.Hkv + kvh) * D);
    const uint32_t dst = lds_addr + tile * G::kTile;
    int issued = 0;
    auto issue = [&]() {
        if (loader) {
            const uint32_t d = dst + (issued & (NSL - 1)) * 2 * G::kStage;
            issue_tile<D, 2>(lc, src, len - tok, d, a.zeros); // keys past the end read zeros
            issue_tile<D, 2>(lc, src + 32 * tok_bytes, len - tok - 32, d + G::kStage, a.zeros);
        }
        src += 64 * tok_bytes;
        tok += 64;
        issued++;
    };
    while (issued < 2 && issued < nchunks) issue(); // the rest follows the barriers, one chunk at a time

    // The wave's 32-row tile.  Waves w and w + 4 share a SIMD; tiles w and 7 - w have the same work between them
    // under the causal mask whatever w is.
    const int T = wave < 4 ? wave : 11 - wave;
    const int row = q0 + kPfRows * T + n;
    PfState<D> st;
#pragma unroll
    for (int i = 0; i < D / 16; i++) {
        bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (row < len) v = *(const bf16x8 *)(a.q + ((int64_t)(t0 + row) * a.Hq + h) * D + 16 * i + 8 * hh);
        st.qf[i] = v;
    }
    st.lsum = 0.f;
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++) {
#pragma unroll
        for (int e = 0; e < 16; e++) st.o[dt][e] = 0.f;
    }

    // The ring.  While a wave is in step s it reads V of stage s and K of stage s + 1.  The barrier that opens chunk
    // c (before step 2 c - 1, the first to read its K) says that every wave's loads of the chunk have landed and that
    // every wave has left the last step that read chunk c - 2, whose slot then takes chunk c + 2 (chunks 0 and 1 are
    // loaded up front).
    auto open_chunk = [&](int c) {
        if (loader) WaitTail<NSL - 1, DPW>::run(issued - 1 - c);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };
    // the stage that holds the tile's diagonal is the last one the wave works on; earlier ones lie wholly below it
    int last = (q0 >> 5) + T;
    const bool diag_in_range = last < nst;
    last = diag_in_range ? last : nst - 1;

    open_chunk(0);
    pf_scores<D>(lds, pl, st.qf, st.s);
    if (last == 0) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
            if (8 * (e / 4) + 4 * hh + (e % 4) > row) st.s[e] = -INFINITY;
        }
    }
    {
        float mx = max3(first_max(st.s[0], st.s[1]), st.s[2], st.s[2]);
#pragma unroll
        for (int e = 3; e < 15; e += 2) mx = max3(mx, st.s[e], st.s[e + 1]);
        mx = max3(mx, st.s[15], st.s[15]);
        const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        st.m = max3(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[1])) * a.scale_log2;
    }
    // (only now, so that the wait for the query rows above does not also wait for these loads)
    if (issued < nchunks) issue();
    // The query rows are the one input no workgroup has touched before, so a block would start with a trip to
    // HBM.  Each block therefore touches (one dword per 64-byte line) the query rows of the block that the same die
    // starts a generation of workgroups later (32 compute units per die, one workgroup each), which then finds
    // them in the die's L2.  The dwords go to a scrap area of LDS behind the ring (a load into registers would
    // write them at a time the compiler does not know of).
    {
        const int turn2 = turn + 32;
        const int pair2 = (turn2 / per_pair) * 8 + die, r2 = turn2 % per_pair;
        bool ok = pair2 < a.num_prompts * a.Hkv;
        const int g2 = ok ? pair2 / a.Hkv : 0;
        const int t2 = uniform_load(a.cu, g2), len2 = uniform_load(a.cu, g2 + 1) - t2;
        const int h2 = (pair2 % a.Hkv) * a.G + r2 % a.G;
        const int row2 = (nqb - 1 - r2 / a.G) * kPfBlock + kPfRows * wave + (lane >> 1);
        ok = ok && row2 < len2;
        const uint16_t *p2 = ok ? a.q + ((int64_t)(t2 + row2) * a.Hq + h2) * D + 32 * (lane & 1) : a.q;
#pragma unroll
        for (int x = 0; x < D * 2 / 128; x++) dma4(p2 + 64 * x, lds_addr + NSL * 2 * G::kStage + 256 * wave);
    }
    // every wave keeps the ring going for all the stages; it computes up to its own last stage: full steps, then the
    // step whose new scores cross the diagonal, then the step without new scores
    auto ring = [&](int s) { // before step s
        if ((s & 1) && s + 1 < nst) {
            open_chunk((s + 1) >> 1);
            if (issued < nchunks) issue();
        }
    };
#define PF_STEP(MASK, NEXT)                                                                                                \
    pf_step<D, MASK, NEXT>(st, lds + ((s + 1) & (2 * NSL - 1)) * G::kStage,                                                \
                           lds_addr + (s & (2 * NSL - 1)) * G::kStage + 2 * G::kTile, pl, a.scale_log2, 32 * (s + 1), row)
    int s = 0;
    for (; s + 1 < last; s++) {
        ring(s);
        PF_STEP(false, true);
    }
    if (s + 1 == last) {
        ring(s);
        PF_STEP(true, true);
        s++;
    }
    ring(s);
    PF_STEP(false, false);
    for (s++; s < nst; s++) ring(s);
#undef PF_STEP

    wait_vmcnt<0>(); // nothing may land in LDS after the workgroup has left
    // a row's sum is spread over its two lanes
    float l;
    {
        const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(st.lsum), __float_as_uint(st.lsum), false, false);
        l = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    const float inv = 1.0f / l;
    const int64_t rh = (int64_t)(t0 + row) * a.Hq + h;
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++) {
#pragma unroll
        for (int qp = 0; qp < 2; qp++) {
            // elements 8 qp .. + 3 are d = 32 dt + 16 qp + 4 hh .. + 3, elements 8 qp + 4 .. + 7 the same 8 further on;
            // the two lanes of a row trade halves so that each holds eight consecutive d
            f32x4 lo, hi;
#pragma unroll
            for (int x = 0; x < 4; x++) {
                lo[x] = st.o[dt][8 * qp + x] * inv;
                hi[x] = st.o[dt][8 * qp + 4 + x] * inv;
            }
            const bf16x4 blo = __builtin_convertvector(lo, bf16x4), bhi = __builtin_convertvector(hi, bf16x4);
            const u32x2 wlo = __builtin_bit_cast(u32x2, blo), whi = __builtin_bit_cast(u32x2, bhi);
            const u32x2 s0 = __builtin_amdgcn_permlane32_swap(wlo[0], whi[0], false, false);
            const u32x2 s1 = __builtin_amdgcn_permlane32_swap(wlo[1], whi[1], false, false);
            // lane hh = 0 now has d = 32 dt + 16 qp + 0..7, lane hh = 1 has + 8..15
            if (row < len) *(u32x4 *)(a.out + rh * D + 32 * dt + 16 * qp + 8 * hh) = u32x4{s0[0], s1[0], s0[1], s1[1]};
        }
    }
    if (row < len && hh == 0) a.lse[rh] = (st.m + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
}

// LDS of a prefill workgroup: the ring and a scrap area
template <int D> constexpr int prefill_lds_bytes() { return kPfSlots * 2 * Geo<D, 2>::kStage + 256 * kPfWaves; }

hipError_t prefill_config()
{
    hipError_t e = hipFuncSetAttribute((const void *)prefill_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       prefill_lds_bytes<128>());
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)prefill_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, prefill_lds_bytes<64>());
}

hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s)
{
    const int nqb = (a.max_len + kPfBlock - 1) / kPfBlock;
    const int64_t pairs = (int64_t)a.num_prompts * a.Hkv; // dealt to eight dies, see the kernel
    const int64_t blocks = 8 * ((pairs + 7) / 8) * nqb * a.G;
    if (blocks == 0) return hipSuccess;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    if (a.D == 128)
        hipLaunchKernelGGL(prefill_kernel<128>, dim3((unsigned)blocks), dim3(64 * kPfWaves), prefill_lds_bytes<128>(), s, a);
    else
        hipLaunchKernelGGL(prefill_kernel<64>, dim3((unsigned)blocks), dim3(64 * kPfWaves), prefill_lds_bytes<64>(), s, a);
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
