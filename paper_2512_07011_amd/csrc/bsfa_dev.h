// Device-side building blocks shared by the forward kernels of libbsfa.so (gfx950, wave64):
// element types and MFMA wrappers, the swizzled LDS tile layout with its direct HBM -> LDS copies,
// counters and barriers that leave those copies in flight, wave-level maxima, work decomposition.
#pragma once
#include "bsfa_internal.h"

#include <math.h>

#include <type_traits>
#include <utility>

namespace bsfa {

// The 16-bit element type of Q, K, V, P and O: bf16 or fp16 (the paper's kernel is fp16
// throughout, Section 5.1).  Same storage size, same MFMA shape, same LDS layout; only the
// matrix instruction, the pack and the pair sum differ.
template <bool F16> struct Elem;
template <> struct Elem<false> {
    typedef __bf16 T;
    typedef __bf16 x8 __attribute__((ext_vector_type(8)));
    typedef __bf16 x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 x2 __attribute__((ext_vector_type(2)));
};
template <> struct Elem<true> {
    typedef _Float16 T;
    typedef _Float16 x8 __attribute__((ext_vector_type(8)));
    typedef _Float16 x4 __attribute__((ext_vector_type(4)));
    typedef _Float16 x2 __attribute__((ext_vector_type(2)));
};
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
// 32x32x16 MFMA, fp32 accumulate, and p0 + p1 + acc on a packed pair: one overload per element type
__device__ __forceinline__ f32x16 mfma16(bf16x8_t a, bf16x8_t b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ f32x16 mfma16(f16x8_t a, f16x8_t b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ float pair_sum(bf16x2_t pp, float acc)
{
    const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(pp, ones, acc, false);
}
__device__ __forceinline__ float pair_sum(f16x2_t pp, float acc)
{
    const f16x2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
    return __builtin_amdgcn_fdot2(pp, ones, acc, false);
}
// 32x32x64 MFMA on fp8 (e4m3) operands, fp32 accumulate: a lane holds 32 consecutive bytes of the
// contraction dimension of its row (A) or column (B); block scales fixed at 2^0
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x16 mfma64_fp8(i32x8 a, i32x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 127, 0, 127);
}
// eight fp32 -> two dwords of fp8 (e4m3), round to nearest even
__device__ __forceinline__ void cvt8_fp8(const float (&f)[8], int &w0, int &w1)
{
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], w1, true);
}
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(uintptr_t)(p))
#define GLB_PTR(T, p) ((const __attribute__((address_space(1))) T *)(p))

// ---- LDS tile layout --------------------------------------------------------------------
// A K or V tile is 64 rows x D bf16, stored as 16-byte chunks, row-major, the chunk index
// XOR-ed with a function of the row so that the operand gathers spread over the banks.  The
// swizzle is applied on the global side of the copy (lane -> which chunk it fetches); the LDS
// side of a direct copy is always linear (wave base + lane * 16 bytes).  Both swizzles only
// touch chunk bits that the gather loops step through with XOR-able constants, so every
// operand address is  (per-lane base) ^ (loop constant) + (immediate offset).
template <int D> __device__ __forceinline__ int swz_k(int row)
{
    return (D == 128) ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int swz_v(int row)
{
    return (D == 128) ? ((row & 7) << 1) : (((row >> 1) & 3) << 1);
}

// Byte offset (relative to the tile's first row) of the chunk thread `tid` copies in
// repetition r; rows at and beyond `rows` are fetched from row rows - 1.
template <int D, int NT, bool ISV>
__device__ __forceinline__ uint32_t chunk_src_offset(int r, int tid, int stride_n, int rows = 64)
{
    constexpr int CPR = D / 8;
    const int sigma = r * NT + tid;
    const int row = sigma / CPR, cp = sigma % CPR;
    const int c = cp ^ (ISV ? swz_v<D>(row) : swz_k<D>(row));
    return (uint32_t)(min(row, rows - 1) * stride_n + 8 * c) * 2u;
}

// Asynchronous HBM -> LDS copy of one tile in NREP repetitions of NT x 16 bytes (NREP = 64 * D * 2 /
// 16 / NT for a 64 x D tile of 16-bit elements); lds_tile is the byte address of the tile's slot.  Each lane fetches 16 bytes; the hardware writes them at M0 + lane * 16.  The tile's first
// row is addressed through a scalar base (it is the same for the whole workgroup), each lane adds
// its 32-bit byte offset (callers pass a base computed from workgroup-uniform values only; a base
// the compiler cannot prove uniform is rejected at build time, the asm operand being a scalar pair).
// Completion is tracked by vmcnt, which this kernel manages itself
// (wait_vmcnt): the instruction is emitted through inline asm so that the compiler does not
// serialise every later LDS read behind all copies in flight.
template <int NREP, int NT>
__device__ __forceinline__ void tile_copy_async(const void *gtile, const uint32_t (&off)[NREP],
                                                uint32_t lds_tile, int wave)
{
#pragma unroll
    for (int r = 0; r < NREP; ++r) {
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_tile + (uint32_t)(r * NT + wave * 64) * 16u);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(dst), "v"(off[r]), "s"(gtile)
                     : "memory", "m0");
    }
}

// The same copy for the last key block of a sequence that does not fill it: rows at and beyond
// `rows` are fetched from row rows-1, which is the repeat-last-token padding of Section 4.3
// (and keeps the copy inside the caller's buffers).  Same number of requests per lane as
// tile_copy_async, so the vmcnt bookkeeping does not change.  The offsets are computed here, at
// the one place per sequence that needs them, from the lane id (no long-lived registers).
template <int D, int NT, bool ISV>
__device__ __forceinline__ void tile_copy_async_clamped(const uint16_t *gtile, int stride_n, int rows,
                                                        uint32_t lds_tile, int wave)
{
    int tid = wave * 64 + (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(tid));       // keeps the offsets from being hoisted out of the key loop
    uint32_t off[64 * (D / 8) / NT];
#pragma unroll
    for (int r = 0; r < 64 * (D / 8) / NT; ++r) off[r] = chunk_src_offset<D, NT, ISV>(r, tid, stride_n, rows);
    tile_copy_async<64 * (D / 8) / NT, NT>(gtile, off, lds_tile, wave);
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14, no wait on the others)
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// Workgroup barrier that orders LDS traffic only: the global -> LDS copies in flight are tracked
// separately with wait_vmcnt, so the barrier must not drain them.
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// max over lanes l and l^32, result in both lanes.  v_permlane32_swap exchanges the upper half
// of its first operand with the lower half of its second: with two copies of x the first
// register ends up holding x[l & 31] and the second x[32 + (l & 31)] in every lane.  Written as
// one asm block so that the two copies are guaranteed to live in different registers.
__device__ __forceinline__ float pair_max(float x)
{
    float a = x, b;
    asm volatile("v_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1\n\tv_max_f32 %0, %0, %1"
                 : "+v"(a), "=&v"(b));
    return a;
}

// max over the wave of a value that is already equal in lanes l and l^32 (wave-uniform result):
// four DPP steps inside each row of 16 lanes, then rows 0 and 1 are combined through SGPRs.
__device__ __forceinline__ float wave_max_paired(float x)
{
    asm volatile("s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1"
                 : "+v"(x));
    const int xi = __builtin_bit_cast(int, x);
    return fmaxf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0)),
                 __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16)));
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order: a fully unrolled loop
// whose body sees its index as a constant expression
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Work decomposition: a work item is (batch b, KV head, group of HP query heads, query tile i).
// With at least 8 (batch, KV head) pairs the pair is chosen by the low three bits of the
// workgroup id, which is the XCD the hardware dispatches the group to, so that all groups
// streaming one K/V sequence share one L2.  Heavy (late) query tiles first.
template <int HP>
__device__ __forceinline__ bool decode_work(const FwdParams &p, int w, int &b, int &h0, int &i)
{
    const int pairs = p.batch * p.hkv;
    const int gsub = p.group / HP;               // head groups per KV head
    int pair, hg, idesc;
    if (pairs >= 8) {
        const int x = w & 7, r = w >> 3;
        const int npx = (pairs + 7) >> 3;
        const int per_tile = npx * gsub;
        idesc = r / per_tile;
        const int rest = r - idesc * per_tile;
        const int pl = rest / gsub;
        hg = rest - pl * gsub;
        pair = x + 8 * pl;
        if (pair >= pairs) return false;
    } else {
        const int per_tile = pairs * gsub;
        idesc = w / per_tile;
        const int rest = w - idesc * per_tile;
        pair = rest / gsub;
        hg = rest - pair * gsub;
    }
    b = pair / p.hkv;
    h0 = (pair - b * p.hkv) * p.group + hg * HP;
    i = p.mq - 1 - idesc;
    return true;
}

}  // namespace bsfa
