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

constexpr int kPfStageRow = 128;                    // bytes of a row in a wave's staging area: 64 bf16
constexpr int kPfStageBytes = kPfRows * kPfStageRow; // 4 KB per wave

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

// The 16-byte pieces of a staging row are XOR-swizzled by the row, so that neither the lanes of a row group that write
// the same piece of different rows nor the eight lanes that read one row meet in a bank.
__device__ __forceinline__ int pf_stage_swz(int r) { return (r + (r >> 3)) & 7; }

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

// A block: 256 consecutive query rows of one (prompt, head), with the keys 0 .. its last row.  All fields are the same
// in every lane.
struct PfBlock {
    int h, kvh, q0, t0, len; // head, kv head, first query row; first token and length of the prompt
    int nst, nchunks;        // stages of 32 keys, chunks of two stages
};

// Workgroups are dealt to the eight dies round-robin, and each die has its own L2.  All blocks of a (prompt, kv
// head) pair, which read the same K and V, therefore go to one die: die x takes the pairs x, x + 8, ... one after
// the other, each with its query blocks from the longest down and the heads of the kv head together.  `turn` counts
// a die's blocks in that order; false past the die's last pair.  A block past its prompt's length has no stages.
__device__ __forceinline__ bool pf_block_of(const PrefillLaunch &a, int die, int turn, PfBlock &b)
{
    const int nqb = (a.max_len + kPfBlock - 1) / kPfBlock;
    const int per_pair = nqb * a.G;
    const int pair = (turn / per_pair) * 8 + die, r = turn % per_pair;
    if (pair >= a.num_prompts * a.Hkv) return false;
    const int g = pair / a.Hkv;
    b.kvh = pair % a.Hkv;
    b.h = b.kvh * a.G + r % a.G;
    b.q0 = (nqb - 1 - r / a.G) * kPfBlock;
    b.t0 = uniform_load(a.cu, g);
    b.len = uniform_load(a.cu, g + 1) - b.t0;
    int kend = b.q0 + kPfBlock;
    kend = kend < b.len ? kend : b.len;
    b.nst = b.q0 < b.len ? (kend + 31) >> 5 : 0;
    b.nchunks = (b.nst + 1) >> 1;
    return true;
}

// The first block with stages at or after `turn` among the turns turn, turn + step, ... of the die (turn comes back
// as that block's turn); false when the die has none left.
__device__ __forceinline__ bool pf_next_block(const PrefillLaunch &a, int die, int &turn, int step, PfBlock &b)
{
    while (pf_block_of(a, die, turn, b)) {
        if (b.nst > 0) return true;
        turn += step;
    }
    return false;
}

// STAY: the workgroups stay: gridDim.x / 8 of them per die, and workgroup i of a die takes the die's blocks i, i + that
// many, ...  K and V of one block after the other stream through one ring, so the first chunks of the next block
// (and its query rows, into registers) are loaded while the last stages of the current one are being multiplied: a
// block starts without a trip to memory.  Without STAY a workgroup takes the one block its number names (the launch
// has one workgroup per block then).  max_len is the host's upper bound of a prompt's length.
template <int D, bool STAY> __global__ __launch_bounds__(64 * kPfWaves) void prefill_kernel(PrefillLaunch a)
{
    using G = Geo<D, 2>;
    constexpr int NSL = kPfSlots;           // ring slots of one chunk; stage number s (counted over all the blocks of
                                            // the workgroup) lives at (s % (2 NSL)) * G::kStage
    static_assert((NSL & (NSL - 1)) == 0, "slot arithmetic by masking");
    extern __shared__ __attribute__((aligned(16384))) uint8_t lds[]; // the step forms LDS addresses by XOR
    const uint32_t lds_addr = (uint32_t)(uintptr_t)lds;
    const int lane = threadIdx.x & 63, n = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int die = blockIdx.x & 7, step = gridDim.x >> 3;

    // two cursors over the same sequence of blocks: the one being multiplied, and the one whose chunks are being loaded
    PfBlock cb, lb;
    int cturn = blockIdx.x >> 3;
    if (!pf_next_block(a, die, cturn, step, cb)) return; // the whole workgroup
    int lturn = cturn;
    lb = cb;
    bool l_ok = true;

    LaneConst<D, 2> lc;
    lane_setup<D, 2>(lc, lane, a.Hkv * D * 2);
    PfLane<D> pl;
    pf_lane_setup<D>(pl, lane);

    // waves 0..3 load the chunks {K0 K1 V0 V1 | K2 K3 V2 V3}: wave w brings tile w of both stages.  (Waves 4..7, the
    // second on each SIMD, are the ones that arrive last at the barriers; they issue no loads.)
    constexpr int DPW = 2 * G::kDmaPerTile; // loads of a loading wave per chunk
    const int tile = wave & 3;
    const bool loader = wave < 4;
    const int64_t tok_bytes = (int64_t)a.Hkv * D * 2;
    const uint32_t dst = lds_addr + tile * G::kTile;
    int issued = 0;  // chunks issued, counted over all blocks: chunk number c lives in ring slot c % NSL
    int lchunk = 0;  // chunks of the block being loaded that have been issued
    int tok = 0;     // first key of the wave's tile in the chunk to load next
    const uint8_t *src = nullptr;
    auto load_from = [&](const PfBlock &b) {
        tok = kPage * (tile & 1);
        src = (const uint8_t *)((tile < 2 ? a.k : a.v) + ((int64_t)(b.t0 + tok) * a.Hkv + b.kvh) * D);
        lchunk = 0;
    };
    load_from(lb);
    auto issue = [&]() { // the next chunk of the sequence, if there is one
        if (!l_ok) return;
        if (loader) {
            const uint32_t d = dst + (issued & (NSL - 1)) * 2 * G::kStage;
            issue_tile<D, 2>(lc, src, lb.len - tok, d, a.zeros); // keys past the end read zeros
            issue_tile<D, 2>(lc, src + 32 * tok_bytes, lb.len - tok - 32, d + G::kStage, a.zeros);
        }
        src += 64 * tok_bytes;
        tok += 64;
        issued++;
        if (++lchunk == lb.nchunks) {
            lturn += step;
            l_ok = STAY && pf_next_block(a, die, lturn, step, lb);
            if (l_ok) load_from(lb);
        }
    };
    issue();
    issue(); // the rest follows the barriers, one chunk at a time

    // The ring.  While a wave is in step s it reads V of stage s and K of stage s + 1.  The barrier that opens chunk
    // c (before the first step that reads its K) says that every wave's loads of the chunk have landed and that
    // every wave has left the last step that read chunk c - 2, whose slot then takes chunk c + 2 (the first two
    // chunks are loaded up front).  Chunks are numbered over all blocks, so the same holds across a block's end.
    auto open_chunk = [&](int c) {
        if (loader) WaitTail<NSL - 1, DPW>::run(issued - 1 - c);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        issue();
    };

    // The wave's 32-row tile.  Waves w and w + 4 share a SIMD; tiles w and 7 - w have the same work between them
    // under the causal mask whatever w is.
    const int T = wave < 4 ? wave : 11 - wave;
    // A lane's part of its query row (a row past the prompt's end reads the prompt's last row instead, and is
    // zeroed by keep_q when the registers are taken into use: nothing writes the registers but the loads themselves,
    // so the compiler has no reason to wait for older loads before them).
    auto load_q = [&](const PfBlock &b, bf16x8 (&qf)[D / 16]) {
        int row = b.q0 + kPfRows * T + n;
        row = row < b.len ? row : b.len - 1;
#pragma unroll
        for (int i = 0; i < D / 16; i++) qf[i] = *(const bf16x8 *)(a.q + ((int64_t)(b.t0 + row) * a.Hq + b.h) * D + 16 * i + 8 * hh);
    };
    auto keep_q = [&](const PfBlock &b, bf16x8 (&qf)[D / 16]) {
        const bool ok = b.q0 + kPfRows * T + n < b.len;
#pragma unroll
        for (int i = 0; i < D / 16; i++) {
            if (!ok) qf[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            asm volatile("" : "+v"(qf[i]));
        }
    };
    // the wave's staging area behind the ring (32 rows of 128 bytes)
    uint8_t *const stage = lds + NSL * 2 * G::kStage + kPfStageBytes * wave;
    const uint32_t stage_addr = lds_addr + NSL * 2 * G::kStage + kPfStageBytes * wave;
    // Query rows come straight from memory, 16 bytes per lane and row.  A workgroup that stays asks for those of the
    // block after the current one (into qn) when the current block has its first scores, and waits for them when its
    // last step is done: qn and st.qf change places there.  (The empty asm statements pin the compiler's wait for the
    // loads to these places; left to the first use it would sit inside a block and wait for younger loads as well.)
    PfState<D> st;
    bf16x8 qn[D / 16];
    load_q(cb, st.qf);
    keep_q(cb, st.qf);
    PfBlock nb;
    int nturn = cturn + step;
    bool n_ok = STAY && pf_next_block(a, die, nturn, step, nb);
    int chunk0 = 0; // number of the current block's first chunk

    for (;;) {
        const int nst = cb.nst, q0 = cb.q0, len = cb.len;
        const int stage0 = 2 * chunk0;
        const int row = q0 + kPfRows * T + n;
        st.lsum = 0.f;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++) {
#pragma unroll
            for (int e = 0; e < 16; e++) st.o[dt][e] = 0.f;
        }
        // the stage that holds the tile's diagonal is the last one the wave works on; earlier ones lie wholly below it
        int last = (q0 >> 5) + T;
        last = last < nst ? last : nst - 1;

        open_chunk(chunk0);
        pf_scores<D>(lds + (stage0 & (2 * NSL - 1)) * G::kStage, pl, st.qf, st.s);
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
        // A workgroup that has no further block of its own (one workgroup per block: long prompts) cannot ask for the
        // next block's query rows, and they are the one input no workgroup has touched before, so every block would
        // start with a trip to HBM.  Such a block therefore touches (one dword per 64-byte line) the query rows of the
        // block that the same die starts a generation of workgroups later (one per compute unit), which then finds
        // them in the die's L2.  The dwords go to the wave's staging area (a load into registers would write them at a
        // time the compiler does not know of).
        if (n_ok) load_q(nb, qn);
        const bool touched = !n_ok;
        if (touched) {
            PfBlock tb;
            const bool ok = pf_block_of(a, die, cturn + a.num_cus / 8, tb);
            const int row2 = tb.q0 + kPfRows * wave + (lane >> 1);
            const uint16_t *p2 = ok && row2 < tb.len ? a.q + ((int64_t)(tb.t0 + row2) * a.Hq + tb.h) * D + 32 * (lane & 1) : a.q;
#pragma unroll
            for (int x = 0; x < D * 2 / 128; x++) dma4(p2 + 64 * x, stage_addr);
        }
        // every wave keeps the ring going for all the stages; it computes up to its own last stage: full steps, then
        // the step whose new scores cross the diagonal, then the step without new scores
        auto ring = [&](int s) __attribute__((always_inline)) { // before step s
            if ((s & 1) && s + 1 < nst) open_chunk(chunk0 + ((s + 1) >> 1));
        };
#define PF_STEP(MASK, NEXT)                                                                                                \
    pf_step<D, MASK, NEXT>(st, lds + ((stage0 + s + 1) & (2 * NSL - 1)) * G::kStage,                                       \
                           lds_addr + ((stage0 + s) & (2 * NSL - 1)) * G::kStage + 2 * G::kTile, pl, a.scale_log2, 32 * (s + 1), row)
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

        // the next block's query rows take their place (the staging area is free for the results after that)
        const PfBlock done = cb;
        const bool more = n_ok;
        if (more) {
#pragma unroll
            for (int i = 0; i < D / 16; i++) st.qf[i] = qn[i];
            keep_q(nb, st.qf);
            chunk0 += cb.nchunks;
            cb = nb;
            cturn = nturn;
            nturn = cturn + step;
            n_ok = STAY && pf_next_block(a, die, nturn, step, nb);
        }

        // a row's sum is spread over its two lanes
        float l;
        {
            const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(st.lsum), __float_as_uint(st.lsum), false, false);
            l = __uint_as_float(r[0]) + __uint_as_float(r[1]);
        }
        const float inv = 1.0f / l;
        const int64_t rh = (int64_t)(done.t0 + row) * a.Hq + done.h;
        // A workgroup that stays sends its results through the wave's staging area, 64 d (128 bytes of every row) at a
        // time: a lane holds four consecutive d of its own row per accumulator quarter, and storing from there is 32
        // separate pieces of 16 bytes per instruction, which keeps the compute unit's one memory pipeline busy for
        // microseconds per block; read back eight lanes to a row, an instruction stores whole 128-byte lines.  (A
        // workgroup with one long block stores directly: the detour's latency would be the last thing before it ends.)
        if (STAY && touched) wait_vmcnt<0>(); // the dwords of the touch above land in this area
        int sl = lane;
        if (STAY) asm volatile("" : "+v"(sl));
        const int sn = sl & 31, sh = sl >> 5;
#pragma unroll
        for (int p = 0; p < (STAY ? D / 64 : 0); p++) {
#pragma unroll
            for (int dtl = 0; dtl < 2; dtl++) {
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    f32x4 v;
#pragma unroll
                    for (int x = 0; x < 4; x++) v[x] = st.o[2 * p + dtl][4 * j + x] * inv; // d = 64 p + 32 dtl + 8 j + 4 hh + x
                    *(bf16x4 *)(stage + kPfStageRow * sn + 16 * ((4 * dtl + j) ^ pf_stage_swz(sn)) + 8 * sh) = __builtin_convertvector(v, bf16x4);
                }
            }
#pragma unroll
            for (int m = 0; m < 4; m++) {
                const int r = 8 * m + (sl >> 3), c = sl & 7; // row of the tile, 16-byte piece of its 128 bytes
                const u32x4 v = *(const u32x4 *)(stage + kPfStageRow * r + 16 * (c ^ pf_stage_swz(r)));
                const int orow = q0 + kPfRows * T + r;
                if (orow < len) *(u32x4 *)(a.out + ((int64_t)(done.t0 + orow) * a.Hq + done.h) * D + 64 * p + 8 * c) = v;
            }
        }
#pragma unroll
        for (int dt = 0; dt < (STAY ? 0 : D / 32); dt++) {
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
        if (!more) break;
    }
    wait_vmcnt<0>(); // nothing may land in LDS after the workgroup has left
}

// LDS of a prefill workgroup: the ring and the waves' staging areas
template <int D> constexpr int prefill_lds_bytes() { return kPfSlots * 2 * Geo<D, 2>::kStage + kPfStageBytes * kPfWaves; }

hipError_t prefill_config()
{
    const void *k[4] = {(const void *)prefill_kernel<128, false>, (const void *)prefill_kernel<128, true>,
                        (const void *)prefill_kernel<64, false>, (const void *)prefill_kernel<64, true>};
    for (int i = 0; i < 4; i++) {
        hipError_t e = hipFuncSetAttribute(k[i], hipFuncAttributeMaxDynamicSharedMemorySize,
                                           i < 2 ? prefill_lds_bytes<128>() : prefill_lds_bytes<64>());
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s)
{
    const int nqb = (a.max_len + kPfBlock - 1) / kPfBlock;
    const int64_t pairs = (int64_t)a.num_prompts * a.Hkv; // dealt to eight dies, see the kernel
    const int64_t turns = ((pairs + 7) / 8) * nqb * a.G;  // blocks of a die
    if (turns == 0) return hipSuccess;
    if (turns > INT32_MAX / 16) return hipErrorInvalidValue;
    // Short prompts (one or two blocks of query rows each): the blocks are alike and a block's start-up is a third of
    // its time, so the workgroups stay, one per compute unit (the ring takes most of a unit's LDS), and each takes
    // every (units per die)-th block of its die.  Longer prompts: blocks differ by up to the prompt's length and
    // start-up is small beside them, so there is one workgroup per block and the hardware hands them out as units
    // become free (the same kernel: a workgroup that finds no further block of its own ends).
    int per_die = a.num_cus / 8;
    per_die = per_die < 1 ? 1 : per_die;
    if (a.stay > 0 && a.stay < per_die) per_die = a.stay; // fewer were asked for
    const bool stay = a.stay < 0 ? nqb <= 2 : a.stay != 0;
    const bool one_each = !stay || turns <= per_die;
    if (one_each) per_die = (int)turns;
#define RA_PF_LAUNCH(DD, ST)                                                                                                \
    hipLaunchKernelGGL((prefill_kernel<DD, ST>), dim3(8u * per_die), dim3(64 * kPfWaves), prefill_lds_bytes<DD>(), s, a)
    if (a.D == 128) {
        if (one_each) RA_PF_LAUNCH(128, false);
        else RA_PF_LAUNCH(128, true);
    } else {
        if (one_each) RA_PF_LAUNCH(64, false);
        else RA_PF_LAUNCH(64, true);
    }
#undef RA_PF_LAUNCH
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
