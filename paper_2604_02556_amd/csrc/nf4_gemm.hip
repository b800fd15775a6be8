// Fused NF4 dequantise + small-batch GEMM on the matrix cores of gfx950:
// y[b][r] = sum_k x[b][k] * W16[r][k],  W16 = rne_fp16(level[code] * scale).
//
// This is the paper's quantised matmul (Sec. III-A, III-C: dequantise the weight
// matrix to FP16 because the matrix units take 16-bit inputs, then multiply with
// FP32 accumulation) for its batch range of 2..64 tokens, with the FP16 copy of
// W living only in registers.  From about 4 tokens on, the FMA-based GEMV is
// bound by the vector ALU; here the multiply-adds go to MFMA and only the
// dequantisation stays on the vector ALU, so the cost is nearly flat in B.
//
// v_mfma_f32_16x16x32_f16: A is 16 rows x 32 k, B is 32 k x 16 tokens, both as 8
// halves per lane (lane l: row or token l mod 16, k = 8 (l / 16) .. + 7); C is
// 16 x 16 FP32, 4 per lane (token l mod 16, rows 4 (l / 16) .. + 3).  A sum over
// k does not care which k a lane carries as long as A and B agree.  Per step a
// wave covers a window of 256 k; MFMA step j (0..7) gives lane group g the eight
// k at 32 j + 8 g.  With that assignment
//   * the activation loads are cheap for the vector cache: the four lanes of a
//     token read 64 contiguous bytes, 16 cache lines per load instruction (the
//     obvious assignment "64 consecutive k per lane" touches 64 lines per load
//     and made the kernel bound by cache-line lookups: 86 us instead of 43 us
//     at 16 tokens);
//   * the codes are still read with two 128-bit loads per lane, 128 contiguous
//     bytes per row, and cross lanes through LDS (row stride 36 dwords: 2-way
//     bank conflicts at most) so that lane group g gets dword g of each 16-byte
//     group;
//   * a lane sees four quantisation blocks per step; lane group g rebuilds the
//     scale of block g and the four lanes of a row swap them with ds_bpermute.
//
// A workgroup of W waves owns 16 RG rows (RG row groups); wave w takes the k
// windows w, w + W, ...; the partial 16 x 16 tiles meet in LDS and are summed in
// wave order (deterministic).  Up to 64 tokens run as up to four 16-token groups
// against the same dequantised A operands, and the activation registers of a
// step are reused by the RG row groups: every workgroup re-reads all of x from
// L2, and that traffic, not the matrix cores or HBM, bounds the kernel.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

constexpr int kWindow = 256;                 // k per wave per step: 4 lane groups x 64

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowStride = 36;               // dwords per row in the exchange buffer (32 + padding)

// SPLIT = false: the weight enters the matrix cores as rne_fp16(level * scale), the GEMM's definition of W.
// SPLIT = true: the FP32 product level * scale, the GEMV's definition of W, without any arithmetic per weight: the
//   table holds every LEVEL as two FP16 terms (hi + lo = the level to about 2^-22), the lookups deliver the MFMA
//   operands as they are, an MFMA step's 32 k lie in one quantisation block, so the products of a block are summed
//   unscaled (hi and lo into the same tile) and the block's FP32 scale multiplies the tile afterwards: four FMAs
//   per lane and block instead of mixed-precision instructions per weight, and the scale is never narrowed (no
//   bound on |W|, no underflow of small scales).  Needs the pair table's space (PAIR).  nf4_dequant_gemv uses it.
// PAIR: levels come from the byte-indexed pair table (issue_pair_lookups) instead of the 16-entry table: fewer
// instructions, 64 KiB more LDS (the final reduction buffer shares that space).

template <int TG, int RG, int kMWaves, bool SPLIT, bool PAIR>
__global__ __launch_bounds__(kMWaves * kWave) void gemm_kernel(const uint8_t* __restrict__ packed,
                                                               const uint8_t* __restrict__ q8,
                                                               const float* __restrict__ scale2,
                                                               const float* __restrict__ offset_p,
                                                               const float* __restrict__ code2, int log2_bs,
                                                               Fmt fmt, int64_t N, int64_t K,
                                                               const _Float16* __restrict__ x, int B,
                                                               _Float16* __restrict__ y) {
    constexpr int kMThreads = kMWaves * kWave;
    constexpr int kTiles = RG * TG;              // 16 x 16 output tiles per wave
    // One LDS object: [pair table or nothing | reduction buffer over the same bytes] | exchange rows | code2 | levels
    constexpr int kRedBytes = kMWaves * kTiles * 4 * kWave * 4;
    constexpr int kHeadBytes = PAIR ? (kRedBytes > kPairTableBytes ? kRedBytes : kPairTableBytes) : kRedBytes;
    constexpr int kStageBytes = 16 * kRowStride * 4;
    constexpr int kOffStage = kHeadBytes, kOffCode2 = kOffStage + kMWaves * kStageBytes, kOffLut = kOffCode2 + 1024;
    __shared__ __attribute__((aligned(16))) uint8_t smem[kOffLut + 64];
    static_assert(sizeof(smem) <= 160 * 1024, "LDS of one compute unit");
    float* lut = (float*)(smem + kOffLut);
    float* code2_lds = (float*)(smem + kOffCode2);
    float (*red)[kTiles * 4][kWave] = (float (*)[kTiles * 4][kWave])smem;

    const int tid = threadIdx.x;
    const int lg = fmt.log2_group;
    if (tid < 16) lut[tid] = fmt.codebook ? fmt.codebook[tid] : __uint_as_float(level_literal(tid));
    for (int i = tid; i < 256; i += kMThreads) code2_lds[i] = code2[i];
    __syncthreads();
    static_assert(!SPLIT || PAIR, "the split levels live in the pair table's space");
    if constexpr (PAIR) {
        if constexpr (SPLIT) fill_split_table((float2_t*)smem, lut, tid, kMThreads);
        else fill_pair_table((float2_t*)smem, lut, tid, kMThreads);
        __syncthreads();
    }
    const float offset = offset_p[0];
    const float nz = opaque_neg_zero();

    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane & 15;                   // row of a tile (A) / token of a group (B, C)
    const int g = lane >> 4;                     // lane group
    const int64_t row0 = (int64_t)blockIdx.x * (16 * RG);
    uint32_t* my_row = (uint32_t*)(smem + kOffStage + wave * kStageBytes) + sub * kRowStride;
    const uint32_t lane_off = pair_lane_offset(lane);
    auto lookups = [&](uint32_t q, float (&lv)[8]) {
        if constexpr (PAIR) issue_pair_lookups(q, smem, lane_off, lv);
        else issue_lookups(q, lut, lv);
    };
    constexpr int kPerDword = PAIR ? 4 : 8;      // LDS reads per dword of codes

    f32x4 acc[RG][TG];
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
        for (int t = 0; t < TG; ++t) acc[r][t] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};

    for (int64_t kw = (int64_t)wave * kWindow; kw < K; kw += (int64_t)kMWaves * kWindow) {
        // ---- loads.  K is a multiple of 64, so each 32- or 64-wide piece of the window is all in or all out.
        u32x4 c[RG][2];
        float mine[RG];                          // scale of the window's g-th 64-element quarter, per row group
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const int64_t row = row0 + 16 * r + sub;
            const bool row_ok = row < N;
            const int64_t e0 = row * K + kw;     // flat index of the row's first element in the window
#pragma unroll
            for (int h = 0; h < 2; ++h) {        // 16-byte groups g and g + 4 of the row's 128 bytes
                c[r][h] = (u32x4){0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u};   // level 0 if not loaded
                if (row_ok && kw + 32 * (g + 4 * h) < K)
                    c[r][h] = __builtin_nontemporal_load((const u32x4*)(packed + (e0 >> 1)) + g + 4 * h);
            }
            mine[r] = 0.0f;
            if (row_ok && kw + 64 * g < K) {
                const int64_t blk = (e0 + 64 * g) >> log2_bs;
                const float prod = code2_lds[q8[blk]] * scale2[blk >> lg];   // rounded product, then rounded sum
                mine[r] = prod + offset;
            }
        }
        half8_t xb[TG][8];
#pragma unroll
        for (int t = 0; t < TG; ++t) {
            const int token = 16 * t + sub;
            const _Float16* xt = x + (int64_t)token * K + kw + 8 * g;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (token < B && kw + 32 * j < K) xb[t][j] = *(const half8_t*)(xt + 32 * j);
                else xb[t][j] = (half8_t)(_Float16)0;
            }
        }

#pragma unroll
        for (int r = 0; r < RG; ++r) {
            // ---- codes cross lanes: group j of the row goes to dwords 4 j .. 4 j + 3; lane group g reads dword g
            *(u32x4*)(my_row + 4 * g) = c[r][0];
            *(u32x4*)(my_row + 4 * (g + 4)) = c[r][1];
            if constexpr (SPLIT)                 // scale of (row sub, quarter g) -> row 4 g + sub / 4, element sub % 4
                *(float*)(my_row - sub * kRowStride + (4 * g + (sub >> 2)) * kRowStride + 32 + (sub & 3)) = mine[r];
            wave_lds_fence();
            uint32_t q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = my_row[4 * j + g];
            float s[4];                          // quarter jj of the window: k = 64 jj .. -> MFMA steps 2 jj, 2 jj + 1
            if constexpr (!SPLIT) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    s[jj] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((sub + 16 * jj) << 2,
                                                                                   __builtin_bit_cast(int, mine[r])));
            }

            if constexpr (SPLIT) {
                // The block scales in the layout of the C tile: lane (token, g) needs those of rows 4 g .. 4 g + 3.
                // They travel in the padding of the exchange rows: row 4 q + g' holds, for quarter q, the scales of
                // rows 4 g' .. 4 g' + 3 (written above, with the codes).
                f32x4 sc[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    sc[jj] = *(const f32x4*)(my_row - sub * kRowStride + (4 * jj + g) * kRowStride + 32);
                const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
                f32x4 blk[TG];
                float lv[2][8];
                lookups(q[0], lv[0]);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (j + 1 < 8) {
                        lookups(q[j + 1], lv[(j + 1) & 1]);
                        lds_wait<kPerDword>();
                    } else {
                        lds_wait<0>();
                    }
                    u32x4 a, a_lo;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        a[i] = __builtin_bit_cast(uint32_t, lv[j & 1][2 * i]);
                        a_lo[i] = __builtin_bit_cast(uint32_t, lv[j & 1][2 * i + 1]);
                    }
                    const half8_t ah = __builtin_bit_cast(half8_t, a), al = __builtin_bit_cast(half8_t, a_lo);
#pragma unroll
                    for (int t = 0; t < TG; ++t) {
                        blk[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, xb[t][j], (j & 1) ? blk[t] : zero, 0, 0, 0);
                        blk[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, xb[t][j], blk[t], 0, 0, 0);
                    }
                    if (j & 1) {                 // both halves of quarter j / 2 are in: scale the tile
#pragma unroll
                        for (int t = 0; t < TG; ++t)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                acc[r][t][i] = __builtin_fmaf(sc[j >> 1][i], blk[t][i], acc[r][t][i]);
                    }
                }
                wave_lds_fence();                // the exchange buffer is overwritten next
                continue;
            }
            // ---- dequantise to FP16 in registers and multiply: lookups pipelined two dwords deep
            float lv[2][8];
            lookups(q[0], lv[0]);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j + 1 < 8) {
                    lookups(q[j + 1], lv[(j + 1) & 1]);
                    lds_wait<kPerDword>();
                } else {
                    lds_wait<0>();
                }
                const float sj = s[j >> 1];
                u32x4 a;
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = scaled_pack2_f16(lv[j & 1][2 * i], lv[j & 1][2 * i + 1], sj, nz);
                const half8_t ah = __builtin_bit_cast(half8_t, a);
#pragma unroll
                for (int t = 0; t < TG; ++t)
                    acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, xb[t][j], acc[r][t], 0, 0, 0);
            }
            wave_lds_fence();                    // the exchange buffer is overwritten next
        }
    }

    if constexpr (PAIR) __syncthreads();         // the reduction buffer overwrites the table: every wave is done with it
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
        for (int t = 0; t < TG; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][(r * TG + t) * 4 + i][lane] = acc[r][t][i];
    __syncthreads();
    // kTiles * 256 outputs per workgroup; thread v: (row group r, token group t, C register i, C lane l)
    for (int v = tid; v < kTiles * 4 * kWave; v += kMThreads) {
        const int l = v & (kWave - 1), ti = v >> 6;
        float sum = red[0][ti][l];
#pragma unroll
        for (int w = 1; w < kMWaves; ++w) sum += red[w][ti][l];
        const int tile = ti >> 2, r = tile / TG, t = tile % TG;
        const int token = 16 * t + (l & 15);
        const int64_t out_row = row0 + 16 * r + 4 * (l >> 4) + (ti & 3);
        if (token < B && out_row < N) y[(int64_t)token * N + out_row] = (_Float16)sum;
    }
}

template <int TG, int RG, int W, bool SPLIT = false, bool PAIR = false>
static void launch_gemm(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                        const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                        _Float16* y, hipStream_t s) {
    const unsigned groups = (unsigned)((N + 16 * RG - 1) / (16 * RG));
    hipLaunchKernelGGL((gemm_kernel<TG, RG, W, SPLIT, PAIR>), dim3(groups), dim3(W * kWave), 0, s, packed, q8, scale2, offset, code2,
                       log2_bs, fmt, N, K, x, B, y);
}

// y = x W^T with W = level * scale on the matrix cores (levels as two FP16 terms, FP32 block scales), at most 16
// tokens.  One shape for all matrices: two row groups per workgroup of 16 waves (four and one row groups, and 8
// waves, all measured slower on 28672 x 8192: 77, 62-92 and more us against 54-56).
int launch_gemv_mfma(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                     const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                     _Float16* y, hipStream_t s) {
    launch_gemm<1, 2, 16, true, true>(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, y, s);
    return record_hip(hipGetLastError());
}

}  // namespace nf4

extern "C" size_t nf4_dequant_gemm_workspace_bytes(int64_t N, int64_t K, int B) {
    if (N <= 0 || K <= 0 || B < 1 || B > 64) return 0;
    const nf4::SplitPlan p = nf4::plan_split(N, K, B);
    // at least one byte, so that a caller who passes a workspace always gets the split-K path
    return p.splits > 1 ? (size_t)p.splits * (size_t)B * (size_t)N * sizeof(float) : 16;
}

namespace nf4 {
static int gemm_entry(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2, const float* offset,
                      const float* code2, int blocksize, Fmt fmt, int64_t N, int64_t K, const void* x, int B, void* y,
                      void* workspace, size_t workspace_bytes, void* stream) {
    if (N < 0 || K < 0) return NF4_ERR_SIZE;
    if (fmt.log2_group < 0) return NF4_ERR_SHAPE;
    const int log2_bs = log2_blocksize(blocksize);
    if (log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (B < 1 || B > 64) return NF4_ERR_SHAPE;
    if (N > 0 && (K <= 0 || K % blocksize != 0)) return NF4_ERR_SHAPE;
    if (N > 0x7fffffffLL) return NF4_ERR_SIZE;
    if (N == 0) return NF4_OK;
    if (!packed || !absmax_q8 || !scale2 || !offset || !code2 || !x || !y) return NF4_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(x, 16) || !aligned(y, 2) || !aligned(scale2, 4) || !aligned(offset, 4) ||
        !aligned(code2, 4) || !aligned(fmt.codebook, 4))
        return NF4_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    const _Float16* xp = (const _Float16*)x;
    _Float16* yp = (_Float16*)y;
    if (workspace) {
        if (!aligned(workspace, 16)) return NF4_ERR_ALIGN;
        if (workspace_bytes < nf4_dequant_gemm_workspace_bytes(N, K, B)) return NF4_ERR_SIZE;
        return launch_gemm_splitk(packed, absmax_q8, scale2, offset, code2, log2_bs, fmt, N, K, xp, B, yp,
                                  (float*)workspace, false, s);
    }
    // (token groups, row groups per wave, waves per workgroup = split of K), picked by sweeping on MI355X:
    // sharing the activation registers between row groups halves the L2 traffic that bounds this kernel,
    // but matrices with few rows need the smaller tile to fill the machine.
    const bool tall = N >= 16384;
#define NF4_GEMM_ARGS packed, absmax_q8, scale2, offset, code2, log2_bs, fmt, N, K, xp, B, yp, s
    switch ((B + 15) / 16) {
        case 1: if (tall) launch_gemm<1, 2, 8>(NF4_GEMM_ARGS); else launch_gemm<1, 2, 16>(NF4_GEMM_ARGS); break;
        // 17..32 tokens: the reduction buffer already takes the LDS that the pair table needs, so it is free
        case 2:
            if (tall) launch_gemm<2, 4, 8, false, true>(NF4_GEMM_ARGS);
            else launch_gemm<2, 2, 8, false, true>(NF4_GEMM_ARGS);
            break;
        case 3: launch_gemm<3, 2, 8>(NF4_GEMM_ARGS); break;
        default: launch_gemm<4, 2, 8>(NF4_GEMM_ARGS); break;
    }
#undef NF4_GEMM_ARGS
    return record_hip(hipGetLastError());
}
}  // namespace nf4

extern "C" int nf4_dequant_gemm(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                const float* offset, const float* code2, int blocksize, int64_t N,
                                int64_t K, const void* x, int B, void* y, void* workspace,
                                size_t workspace_bytes, void* stream) {
    return nf4::gemm_entry(packed, absmax_q8, scale2, offset, code2, blocksize, nf4::kNf4Fmt, N, K, x, B, y, workspace,
                           workspace_bytes, stream);
}

// the data type as a parameter (Sec. V-A): any 16 levels, any second-level group size
extern "C" int nf4_dequant_gemm_codebook(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                         const float* offset, const float* code2, int dq_group,
                                         const float* codebook, int blocksize, int64_t N, int64_t K, const void* x,
                                         int B, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    const nf4::Fmt fmt = {nf4::log2_dq_group(dq_group), codebook};
    return nf4::gemm_entry(packed, absmax_q8, scale2, offset, code2, blocksize, fmt, N, K, x, B, y, workspace,
                           workspace_bytes, stream);
}
