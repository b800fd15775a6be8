// Fused NF4 dequantise + decode GEMV for gfx950: y[b][r] = sum_k x[b][k] *
// W[r][k] with W kept in its 4-bit form (the paper dequantises the whole
// matrix into an FP16 temporary before a dense matmul, Sec. III-C; for a
// handful of tokens that temporary is the dominant traffic, so it is never
// written here).
//
// Not a dense contraction at these batch sizes, so no MFMA: FP32 FMAs, wave64
// reductions.  Layout of the work:
//   * a workgroup of 4 waves owns kRows consecutive rows of W; wave w takes the
//     k-slices w, w+4, ... so the four waves stream disjoint parts of the same
//     rows and their partial sums meet in LDS in a fixed order (deterministic);
//   * inside a slice lane l owns CH consecutive dwords of codes (8*CH elements,
//     always inside one quantisation block), loads them with one 128-bit (CH=4)
//     or 32-bit (CH=1) load per row, contiguous across the wave;
//   * its 8*CH activations per token are converted to FP32 once per slice and
//     reused for all kRows rows;
//   * the block scale is applied once per lane chunk (sum of level*x first,
//     then one multiply-add by the scale), not once per element.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

constexpr int kGThreads = 256;
constexpr int kGWaves = kGThreads / kWave;
constexpr int kRows = 4;

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

template <int B, int CH>
__global__ __launch_bounds__(kGThreads) void gemv_kernel(const uint8_t* __restrict__ packed,
                                                         const uint8_t* __restrict__ q8,
                                                         const float* __restrict__ scale2,
                                                         const float* __restrict__ offset_p,
                                                         const float* __restrict__ code2, int log2_bs,
                                                         int64_t N, int64_t K,
                                                         const _Float16* __restrict__ x,
                                                         _Float16* __restrict__ y) {
    constexpr int E = 8 * CH;                 // elements per lane per slice
    constexpr int kSlice = E * kWave;         // elements per wave per slice
    __shared__ float lut[16];
    __shared__ float code2_lds[256];
    __shared__ float partial[kGWaves][kRows][B];

    if (threadIdx.x < 16) lut[threadIdx.x] = __uint_as_float(kLevelBits[threadIdx.x]);
    code2_lds[threadIdx.x] = code2[threadIdx.x];
    __syncthreads();
    const float offset = offset_p[0];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r0 = (int64_t)blockIdx.x * kRows;

    float acc[kRows][B];
#pragma unroll
    for (int r = 0; r < kRows; ++r)
#pragma unroll
        for (int b = 0; b < B; ++b) acc[r][b] = 0.0f;

    for (int64_t k0 = (int64_t)wave * kSlice; k0 < K; k0 += (int64_t)kGWaves * kSlice) {
        const int64_t k = k0 + (int64_t)lane * E;
        if (k < K) {                                   // K % E == 0: a lane chunk is all in or all out
            float xf[B][E];
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const half8_t h = *(const half8_t*)(x + (int64_t)b * K + k + 8 * c);
#pragma unroll
                    for (int j = 0; j < 8; ++j) xf[b][8 * c + j] = (float)h[j];
                }
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                if (r0 + r < N) {
                    const int64_t e = (r0 + r) * K + k;            // flat element index
                    uint32_t q[CH];
                    if constexpr (CH == 4) {
                        const u32x4 v = *(const u32x4*)(packed + (e >> 1));
                        q[0] = v[0]; q[1] = v[1]; q[2] = v[2]; q[3] = v[3];
                    } else {
#pragma unroll
                        for (int c = 0; c < CH; ++c) q[c] = *(const uint32_t*)(packed + (e >> 1) + 4 * c);
                    }
                    const int64_t blk = e >> log2_bs;
                    const float prod = code2_lds[q8[blk]] * scale2[blk >> 8];
                    const float s = prod + offset;
                    float part[B];
#pragma unroll
                    for (int b = 0; b < B; ++b) part[b] = 0.0f;
#pragma unroll
                    for (int c = 0; c < CH; ++c)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float hi = lut[(q[c] >> (8 * j + 4)) & 15u];
                            const float lo = lut[(q[c] >> (8 * j)) & 15u];
#pragma unroll
                            for (int b = 0; b < B; ++b) {
                                part[b] = __builtin_fmaf(hi, xf[b][8 * c + 2 * j], part[b]);
                                part[b] = __builtin_fmaf(lo, xf[b][8 * c + 2 * j + 1], part[b]);
                            }
                        }
#pragma unroll
                    for (int b = 0; b < B; ++b) acc[r][b] = __builtin_fmaf(s, part[b], acc[r][b]);
                }
            }
        }
    }

    // wave64 butterfly, then the four waves' sums meet in LDS in wave order
#pragma unroll
    for (int r = 0; r < kRows; ++r)
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float v = acc[r][b];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
            if (lane == 0) partial[wave][r][b] = v;
        }
    __syncthreads();
    if (threadIdx.x < kRows * B) {
        const int r = threadIdx.x / B, b = threadIdx.x % B;
        if (r0 + r < N) {
            float v = partial[0][r][b];
#pragma unroll
            for (int w = 1; w < kGWaves; ++w) v += partial[w][r][b];
            y[(int64_t)b * N + r0 + r] = (_Float16)v;
        }
    }
}

template <int B, int CH>
static void launch_gemv(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                        const float* code2, int log2_bs, int64_t N, int64_t K, const void* x, void* y,
                        hipStream_t s) {
    const unsigned groups = (unsigned)((N + kRows - 1) / kRows);
    hipLaunchKernelGGL((gemv_kernel<B, CH>), dim3(groups), dim3(kGThreads), 0, s, packed, q8, scale2, offset,
                       code2, log2_bs, N, K, (const _Float16*)x, (_Float16*)y);
}

}  // namespace nf4

extern "C" int nf4_dequant_gemv(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                const float* offset, const float* code2, int blocksize, int64_t N,
                                int64_t K, const void* x, int B, void* y, void* stream) {
    using namespace nf4;
    if (N < 0 || K < 0) return NF4_ERR_SIZE;
    const int log2_bs = log2_blocksize(blocksize);
    if (log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (B < 1 || B > 16) return NF4_ERR_SHAPE;
    if (N > 0 && (K <= 0 || K % blocksize != 0)) return NF4_ERR_SHAPE;   // blocksize is a multiple of 32
    if (N > (int64_t)0x7fffffff / kRows * kRows) return NF4_ERR_SIZE;
    if (N == 0) return NF4_OK;
    if (!y) return NF4_ERR_NULL;
    if (!aligned(y, 2)) return NF4_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (!packed || !absmax_q8 || !scale2 || !offset || !code2 || !x) return NF4_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(x, 16) || !aligned(scale2, 4) || !aligned(offset, 4) ||
        !aligned(code2, 4))
        return NF4_ERR_ALIGN;

#define NF4_GEMV_CASE(b, ch) \
    case b: launch_gemv<b, ch>(packed, absmax_q8, scale2, offset, code2, log2_bs, N, K, x, y, s); break;
    switch (B) {
        NF4_GEMV_CASE(1, 4) NF4_GEMV_CASE(2, 4) NF4_GEMV_CASE(3, 1) NF4_GEMV_CASE(4, 1)
        NF4_GEMV_CASE(5, 1) NF4_GEMV_CASE(6, 1) NF4_GEMV_CASE(7, 1) NF4_GEMV_CASE(8, 1)
        NF4_GEMV_CASE(9, 1) NF4_GEMV_CASE(10, 1) NF4_GEMV_CASE(11, 1) NF4_GEMV_CASE(12, 1)
        NF4_GEMV_CASE(13, 1) NF4_GEMV_CASE(14, 1) NF4_GEMV_CASE(15, 1) NF4_GEMV_CASE(16, 1)
    }
#undef NF4_GEMV_CASE
    return record_hip(hipGetLastError());
}
