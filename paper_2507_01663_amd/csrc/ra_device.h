// Device-side building blocks shared by the gfx950 kernels: vector types, direct global->LDS loads and their
// hand-kept completion counter, the LDS layout of a 16-token K or V tile and the lane constants that address it,
// row reductions over the MFMA accumulator layout, and the E4M3 encoding.
#pragma once
#include "ra_internal.h"

namespace ra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Waits until at most min(stages_after, N) younger stages of DPS loads each are still in flight.
template <int N, int DPS> struct WaitTail {
    static __device__ __forceinline__ void run(int stages_after)
    {
        if (stages_after >= N) wait_vmcnt<N * DPS>();
        else WaitTail<N - 1, DPS>::run(stages_after);
    }
};
template <int DPS> struct WaitTail<0, DPS> {
    static __device__ __forceinline__ void run(int) { wait_vmcnt<0>(); }
};

// 16 bytes per lane from global memory straight into LDS at lds_addr + lane*16 (no registers in between).
// The compiler does not see these as loads, so their completion is tracked by hand with wait_vmcnt().
// Two address forms: a full 64-bit address per lane, or a wave-uniform base plus a 32-bit lane offset.
// (The LDS address and the base are wave-uniform by construction; readfirstlane says so to the compiler, which
// may have computed them on the vector unit.)
// STREAM marks data that is read once (the pages of a decode step): the loads carry the non-temporal hint, which tells
// the caches not to keep the lines.  Measured on the streaming probe, 4 KB tiles from scattered places: 6.1 TB/s
// without the hint, 6.9 TB/s with it (consecutive tiles: 6.4 and 7.1); the system-coherence bits change nothing.
template <bool STREAM = false> __device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr)
{
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
    if (STREAM) asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gptr), "s"(m0) : "memory", "m0");
    else asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(m0) : "memory", "m0");
}
template <bool STREAM = false> __device__ __forceinline__ void dma16_base(uint32_t lane_off, const void *uniform_base, uint32_t lds_addr)
{
    const uint64_t u = (uint64_t)(uintptr_t)uniform_base;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    const uint64_t sbase = ((uint64_t)hi << 32) | lo;
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
    if (STREAM)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(lane_off), "s"(sbase), "s"(m0)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(sbase), "s"(m0)
                     : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void *gptr, uint32_t lds_addr) // 4 bytes per lane, to lds_addr + lane*4
{
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(gptr), "s"(m0) : "memory", "m0");
}

// Reductions over the four lanes that own one query row (l, l^16, l^32, l^48), on the VALU (no LDS trip).
__device__ __forceinline__ float row_max(float x)
{
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float row_sum(float x)
{
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS placement of 16-byte unit c of tile row r: rows are kept whole, units are XOR-swizzled inside the
// row so that the 16 rows of an MFMA operand read and the 4 rows of a transposed read spread over banks.
__device__ __forceinline__ int swz(int r) { return 2 * (r & 3) + ((r >> 2) & 1) + (r & 8); }

// Geometry of a page in LDS for head dim D and KVB bytes per stored element (2: bf16, 1: e4m3).
template <int D, int KVB> struct Geo {
    static constexpr int kRowBytes = D * KVB;
    static constexpr int kUnits = kRowBytes / 16;       // 16-byte units per row
    static constexpr int kTile = kPage * kRowBytes;     // one (page, head) tile of K or of V
    static constexpr int kDmaPerTile = kTile / 1024;    // wave-wide 16-byte loads per tile
    static constexpr int kScaleBytes = KVB == 1 ? 256 : 0; // e4m3: the two pages' k and v scales ride along
    static constexpr int kStage = 4 * kTile + kScaleBytes; // K0 K1 V0 V1 (and scales): two pages per ring stage
    static constexpr int kDmaPerStage = 4 * kDmaPerTile + (KVB == 1 ? 1 : 0);
    static constexpr int kKSteps = D / 32;              // 16x16x32 MFMA steps over the head dim
    static constexpr int kKReads = kUnits / 4;          // 16-byte K reads per lane per page
    static constexpr int kDTiles = D / 16;
};

template <int D, int KVB> struct LaneConst {
    int dma_row[Geo<D, KVB>::kDmaPerTile];
    int dma_off[Geo<D, KVB>::kDmaPerTile];
    int kq_off[D / 32];                       // where lane (row, j) finds its Q operand of k-step i in that tile
    int k_off[Geo<D, KVB>::kKReads];
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
    {
        // query tile: 16 rows of D bf16, 16-byte units swizzled inside the row like a bf16 K tile
        constexpr int QU = D * 2 / 16, QM = QU - 1;
        const int r = lane & 15, j = lane >> 4;
#pragma unroll
        for (int i = 0; i < D / 32; i++) {
            // the eight d values of k-step i that this lane's K operand holds start at d0 (see run_segment)
            const int d0 = KVB == 2 ? 32 * i + 8 * j : 16 * (4 * (i / 2) + j) + 8 * (i % 2);
            lc.kq_off[i] = 16 * (r * QU + ((d0 / 8) ^ (swz(r) & QM)));
        }
    }
    // K operand: lane (key = lane%16, j = lane/16) reads unit 4*i + j of its key's row
    const int r = lane & 15, j = lane >> 4;
#pragma unroll
    for (int i = 0; i < G::kKReads; i++) lc.k_off[i] = 16 * (r * G::kUnits + ((4 * i + j) ^ (swz(r) & UM)));
    // V operand through the transposing read: the 16 lanes of group j address a 4-key x 16-d block
    const int a = lane & 15;
    if (KVB == 2) {
        // ds_read_b64_tr_b16: lane a supplies key 4j + a/4, d = 16*dt + 4*(a%4) .. +3 (8 bytes)
        const int vrow = 4 * j + (a >> 2);
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++) {
            int c = 2 * dt + ((a >> 1) & 1);
            lc.v_off[dt] = 16 * (vrow * G::kUnits + (c ^ (swz(vrow) & UM))) + 8 * (a & 1);
        }
    } else {
        // ds_read_b64_tr_b8: lane a supplies row a/2 of eight, d = 16*dt + 8*(a%2) .. +7 (8 bytes); rows 0-3 are
        // keys 4j .. 4j+3 of the stage's first page, rows 4-7 the same keys of its second page (the next tile)
        const int vrow = 4 * j + ((a >> 1) & 3);
#pragma unroll
        for (int dt = 0; dt < G::kDTiles; dt++)
            lc.v_off[dt] = (a >> 3) * G::kTile + 16 * (vrow * G::kUnits + (dt ^ (swz(vrow) & UM))) + 8 * (a & 1);
    }
}

// e4m3 -> bf16 is exact (3 mantissa bits into 7); four codes of one dword at a time.
__device__ __forceinline__ bf16x4 fp8x4_to_bf16(int codes)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, false);
    bf16x2 hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, true);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
}
__device__ __forceinline__ bf16x8 fp8x8_to_bf16(int c0, int c1)
{
    return __builtin_shufflevector(fp8x4_to_bf16(c0), fp8x4_to_bf16(c1), 0, 1, 2, 3, 4, 5, 6, 7);
}

// One tile.  A full page goes the cheap way (uniform base + lane offset).  In the last page of a sequence
// the rows at or past nvalid come from the zero block instead, so stale or poisoned slots never reach the
// MFMA; a page id is only dereferenced when the page exists.
template <int D, int KVB, bool STREAM = false>
__device__ __forceinline__ void issue_tile(const LaneConst<D, KVB> &lc, const uint8_t *tile, int nvalid, uint32_t lds_addr,
                                           const void *zeros)
{
    using G = Geo<D, KVB>;
    if (nvalid >= kPage) {
#pragma unroll
        for (int n = 0; n < G::kDmaPerTile; n++) dma16_base<STREAM>((uint32_t)lc.dma_off[n], tile, lds_addr + 1024 * n);
    } else {
#pragma unroll
        for (int n = 0; n < G::kDmaPerTile; n++) {
            const void *src = lc.dma_row[n] < nvalid ? (const void *)(tile + lc.dma_off[n]) : zeros;
            dma16<STREAM>(src, lds_addr + 1024 * n);
        }
    }
}

// Wave-uniform lookups in read-only tables (block table, schedule): read through the constant address space
// so that they are scalar loads, which leave the vector-memory counter that paces the ring alone.
typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
__device__ __forceinline__ int32_t uniform_load(const int32_t *p, int64_t i) { return ((const_i32_ptr)(uintptr_t)p)[i]; }

// E4M3 value of a code (exact in binary32).  S.1111.111 is NaN.
__device__ __forceinline__ float e4m3_value(uint32_t c)
{
    const int e = (c >> 3) & 15, m = c & 7;
    float v = e ? ldexpf(1.0f + 0.125f * (float)m, e - 7) : 0.001953125f * (float)m;
    if (e == 15 && m == 7) v = __uint_as_float(0x7fc00000u);
    return (c & 0x80) ? -v : v;
}

// Nearest E4M3 code of z: ties to the even code, saturating at +-448, NaN -> 0x7F.
__device__ __forceinline__ uint32_t e4m3_nearest(float z)
{
    uint32_t u = __float_as_uint(z);
    const uint32_t sign = (u >> 24) & 0x80;
    u &= 0x7fffffffu;
    if (u > 0x7f800000u) return 0x7f;
    const float a = __uint_as_float(u);
    if (a >= 448.0f) return sign | 0x7e;
    if (a < 0.015625f) return sign | (uint32_t)rintf(a * 512.0f); // steps of 2^-9 below 2^-6; 8 steps are 2^-6 itself
    u += 0x7ffffu + ((u >> 20) & 1); // keep three mantissa bits, round half to even (a carry moves to the next binade)
    const uint32_t code = ((((u >> 23) - 127 + 7) << 3) | ((u >> 20) & 7));
    return sign | (code > 0x7e ? 0x7e : code);
}

} // namespace ra
