// Host-side argument checks and launch bookkeeping shared by the entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nf4.h"

namespace nf4 {

// hipError_t of the last failed launch on this thread (nf4_last_hip_error).
extern thread_local int g_last_hip_error;

inline int record_hip(hipError_t e) {
    if (e == hipSuccess) return NF4_OK;
    g_last_hip_error = (int)e;
    return NF4_ERR_HIP;
}

inline bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// log2(blocksize) for a power of two in [64, 4096], else -1.
inline int log2_blocksize(int bs) {
    for (int s = 6; s <= 12; ++s)
        if (bs == (1 << s)) return s;
    return -1;
}

// log2(group) for a power of two in [1, 65536] blocks per second-level scale, else -1.
inline int log2_dq_group(int group) {
    for (int s = 0; s <= 16; ++s)
        if (group == (1 << s)) return s;
    return -1;
}

// The data type as a parameter (Sec. V-A) for the fused kernels: blocks per second-level scale as a shift, and the
// caller's 16 levels (device) or nullptr for the NF4 literals.
struct Fmt {
    int log2_group;
    const float* codebook;
};
constexpr Fmt kNf4Fmt = {8, nullptr};

// Compute units of the current device (queried once per thread; 256 on MI355X).
int compute_units();

// How the split-K GEMM divides a problem: row blocks x splits workgroups, each
// split taking `wps` windows of 256 k (nf4_gemm_splitk.hip).
struct SplitPlan {
    int tg, rg, waves;       // token groups, row groups per wave, waves per workgroup
    int64_t row_blocks;
    int wps, splits;
};
SplitPlan plan_split(int64_t N, int64_t K, int B);

// The GEMV's sum (FP32 weights: levels to 22 bits as two FP16 terms, FP32 block scales) on the matrix cores,
// B <= 16 (nf4_gemm.hip).
int launch_gemv_mfma(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                     const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                     _Float16* y, hipStream_t s);

// Split-K GEMM: `partial` holds plan.splits * B * N floats when plan.splits > 1.  gemv_weights (B <= 16): W is the
// FP32 product level * scale (levels as two FP16 terms, FP32 block scales) instead of rne_fp16(level * scale).
int launch_gemm_splitk(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                       const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                       _Float16* y, float* partial, bool gemv_weights, hipStream_t s);

// One and two tokens by column slices (nf4_gemv_slice.hip): which shapes it takes, and the launch.
bool gemv_slice_eligible(int64_t N, int64_t K, int B, const Fmt& fmt);
int launch_gemv_slice(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                      const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                      _Float16* y, hipStream_t s);

// Up to four tokens by column pieces on the 4 x 4 x 4 matrix-core instruction (nf4_gemv_quad.hip).
bool gemv_quad_eligible(int64_t N, int64_t K, int B, int log2_bs, const Fmt& fmt);
int launch_gemv_quad(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                     const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                     _Float16* y, hipStream_t s);

// nf4_dequant_gemv_ws after its argument checks: FMA kernels for one and two tokens, split-K on the matrix cores
// with `partial` (plan_split(N, K, B).splits * B * N floats, written before they are read) above that.
int launch_gemv_ws(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                   const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                   _Float16* y, float* partial, hipStream_t s);

}  // namespace nf4
