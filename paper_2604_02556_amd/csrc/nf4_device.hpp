// Device-side pieces shared by the gfx950 kernels: the level table, nibble
// handling and the round-to-nearest-even narrowing conversions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nf4.h"

namespace nf4 {

constexpr int kWave = 64;

// Sec. II-B: the 16 NormalFloat levels (normal quantiles scaled to [-1, 1]),
// as binary32 bit patterns so that no decimal parsing stands between the source
// and the value.
__device__ __constant__ const uint32_t kLevelBits[16] = {
    0xbf800000u, 0xbf3239b1u, 0xbf066b30u, 0xbeca32a0u, 0xbe91a24du, 0xbe3d353fu,
    0xbdba7871u, 0x00000000u, 0x3da2faffu, 0x3e24cae3u, 0x3e7c04ddu, 0x3ead033au,
    0x3ee1a4b8u, 0x3f1007abu, 0x3f3913b3u, 0x3f800000u};

// level[i] as a bit pattern selected from instruction literals: a table in LDS
// or in a register can be filled without reading memory.
__host__ __device__ __forceinline__ uint32_t level_literal(uint32_t i) {
    uint32_t v = 0xbf800000u;
    v = i == 1 ? 0xbf3239b1u : v;  v = i == 2 ? 0xbf066b30u : v;  v = i == 3 ? 0xbeca32a0u : v;
    v = i == 4 ? 0xbe91a24du : v;  v = i == 5 ? 0xbe3d353fu : v;  v = i == 6 ? 0xbdba7871u : v;
    v = i == 7 ? 0x00000000u : v;  v = i == 8 ? 0x3da2faffu : v;  v = i == 9 ? 0x3e24cae3u : v;
    v = i == 10 ? 0x3e7c04ddu : v; v = i == 11 ? 0x3ead033au : v; v = i == 12 ? 0x3ee1a4b8u : v;
    v = i == 13 ? 0x3f1007abu : v; v = i == 14 ? 0x3f3913b3u : v; v = i == 15 ? 0x3f800000u : v;
    return v;
}

// Order LDS traffic within one wave.  The hardware serves a wave's LDS
// instructions in issue order, so only the compiler must be kept from moving
// accesses across this point; no s_barrier is involved.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Two FP32 values -> one dword of two 16-bit values, `lo` in the low half.
// Both conversions round to nearest even (the wave's default rounding mode),
// keep subnormals and overflow to infinity.
template <int DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi);

template <>
__device__ __forceinline__ uint32_t pack2<NF4_FP16>(float lo, float hi) {
    float2_t v = {lo, hi};
    half2_t h = __builtin_convertvector(v, half2_t);
    return __builtin_bit_cast(uint32_t, h);
}

template <>
__device__ __forceinline__ uint32_t pack2<NF4_BF16>(float lo, float hi) {
    float2_t v = {lo, hi};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

// rne_fp16(a * s) for two values, packed (`lo` product in the low half): the exact
// product narrowed to FP16 in ONE rounding.  Written as a fused multiply-add with
// a -0 addend (a * s + (-0) keeps the product's sign of zero), which the compiler
// turns into one mixed-precision instruction per value (v_fma_mixlo_f16 /
// v_fma_mixhi_f16) instead of multiply, multiply, convert.  A multiply followed
// by a convert rounds twice (to FP32, then to FP16); the two results differ, by
// one FP16 ulp, only where the FP32-rounded product lies exactly half way between
// two FP16 values -- about one product in 10^4 to 10^5.  Kernels whose output must
// equal that two-step result bit for bit (the dequantiser) do not use this.
// `neg_zero` must come from opaque_neg_zero(): a visible constant would let the
// compiler fold the FMA back into a multiply.
__device__ __forceinline__ float opaque_neg_zero() {
    float z = -0.0f;
    asm("" : "+s"(z));
    return z;
}
__device__ __forceinline__ uint32_t scaled_pack2_f16(float lo, float hi, float s, float neg_zero) {
    half2_t h = {(_Float16)__builtin_fmaf(lo, s, neg_zero), (_Float16)__builtin_fmaf(hi, s, neg_zero)};
    return __builtin_bit_cast(uint32_t, h);
}

// One value.  The empty asm pins `v` as a finished FP32 result: without it the
// compiler folds a preceding multiply into a mixed-precision multiply-add with
// a +0 addend, which turns a product of -0 into +0.
template <int DT>
__device__ __forceinline__ uint16_t narrow1(float v) {
    asm volatile("" : "+v"(v));
    return (uint16_t)(pack2<DT>(v, 0.0f) & 0xffffu);
}

// Eight level lookups for one dword of codes.  Two masked copies of the dword
// hold code*4 (the LDS byte address) in each byte, so an address is one
// bit-field extract; the empty asm keeps the compiler from undoing that.
__device__ __forceinline__ void issue_lookups(uint32_t q, const float* lut, float (&lv)[8]) {
    uint32_t lo4 = (q << 2) & 0x3C3C3C3Cu;                         // low nibbles  = odd elements
    uint32_t hi4 = (q >> 2) & 0x3C3C3C3Cu;                         // high nibbles = even elements
    asm("" : "+v"(lo4), "+v"(hi4));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        lv[2 * j] = *(const float*)((const char*)lut + ((hi4 >> (8 * j)) & 0xFFu));
        lv[2 * j + 1] = *(const float*)((const char*)lut + ((lo4 >> (8 * j)) & 0xFFu));
    }
}

// The same eight levels from a table indexed by whole code bytes: entry [byte][replica] holds the pair
// (level[byte >> 4], level[byte & 15]), 32 replicas of 8 bytes per byte value (64 KiB).  Lane l reads replica
// l % 32, so every lane of a half-wave owns its own pair of LDS banks whatever the codes are, the address is a
// single byte permute (byte k of q into bits 15:8 above the lane's offset) and one 64-bit read brings two levels:
// 8 instructions per dword of codes instead of 18.  The table must start at LDS address 0 (the only __shared__
// object of the kernel, or the first bytes of it) so that the permuted value is the address itself.
constexpr int kPairReplicas = 32;
constexpr int kPairTableBytes = 256 * kPairReplicas * 8;
__device__ __forceinline__ uint32_t pair_lane_offset(int lane) { return (uint32_t)(lane & (kPairReplicas - 1)) * 8u; }

// Fill the table from the 16 levels in `lut` (LDS, already visible to the caller's threads), two replicas of a
// byte's pair per 128-bit write.
__device__ __forceinline__ void fill_pair_table(float2_t* table, const float* lut, int tid, int threads) {
    typedef float float4_t __attribute__((ext_vector_type(4)));
    for (int i = tid; i < 256 * kPairReplicas / 2; i += threads) {
        const int byte = i / (kPairReplicas / 2);
        const float e = lut[byte >> 4], o = lut[byte & 15];
        ((float4_t*)table)[i] = (float4_t){e, o, e, o};
    }
}

// The split table: entry [byte][replica] = (half2(hi(level[byte >> 4]), hi(level[byte & 15])),
// half2(lo(..), lo(..))) with hi = rne_fp16(level), lo = rne_fp16(level - hi) (the difference is exact in FP32):
// hi + lo is the level to about 2^-22 relative.  Same shape and addressing as the pair table.
__device__ __forceinline__ void fill_split_table(float2_t* table, const float* lut, int tid, int threads) {
    for (int i = tid; i < 256 * kPairReplicas; i += threads) {
        const int byte = i / kPairReplicas;
        const float e = lut[byte >> 4], o = lut[byte & 15];
        const _Float16 eh = (_Float16)e, oh = (_Float16)o;
        const half2_t hi = {eh, oh};
        const half2_t lo = {(_Float16)(e - (float)eh), (_Float16)(o - (float)oh)};
        table[i] = (float2_t){__builtin_bit_cast(float, hi), __builtin_bit_cast(float, lo)};
    }
}

__device__ __forceinline__ void issue_pair_lookups(uint32_t q, const uint8_t* table, uint32_t lane_off,
                                                   float (&lv)[8]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        // result bytes: [0] = lane_off, [1] = byte k of q, [2] = [3] = 0
        const uint32_t a = __builtin_amdgcn_perm(q, lane_off, 0x0c0c0000u | ((4u + k) << 8));
        const float2_t pr = *(const float2_t*)(table + a);
        lv[2 * k] = pr[0];                                         // high nibble = even element
        lv[2 * k + 1] = pr[1];
    }
}

// Wait until at most `left` LDS operations of this wave are outstanding, and keep
// the instruction scheduler from moving anything across.  The kernel is bound by
// instruction issue, and a wave spends an issue slot on every s_waitcnt: one wait
// per eight lookups instead of the one per multiply-add the compiler would emit.
template <int LEFT>
__device__ __forceinline__ void lds_wait() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F | (LEFT << 8));              // lgkmcnt(LEFT); vmcnt, expcnt untouched
    __builtin_amdgcn_sched_barrier(0);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}

// Sum over the 64 lanes; the total lands in lane 63.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
    v = dpp_add<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x114, 0xF>(v);   // row_shr:4
    v = dpp_add<0x118, 0xF>(v);   // row_shr:8   -> lane 15 of each row holds the row sum
    v = dpp_add<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

}  // namespace nf4
