// Fused NF4 dequantise + decode GEMV for one token, laid out by columns: a wave owns a slice of 2048
// columns of W and streams rows through it (the kernels of nf4_gemv.hip give a wave a few rows over all of K).
//
// Why: in the row-owning layout a wave must fetch the activations of every step again for its four rows -- at one
// token as many load instructions as the codes themselves -- and every wave of the grid reads its own strided
// pieces of the scale arrays.  Here
//   * lane l of a slice keeps the 32 activations of ITS columns, 2048 s + 32 l .. + 31, in registers as FP32 for
//     the whole kernel: no activation traffic inside the loop, and plain FP32 multiply-adds (the mixed-precision
//     form that takes FP16 activations issues at half their rate);
//   * per row a wave issues one 128-bit load per lane, 1 KiB of contiguous codes, and the KS waves of a workgroup
//     that share a row read its whole K / 2 bytes side by side; four rows per wave are in flight, every load unconditional;
//   * a lane's 32 columns lie in one quantisation block, so the block scale multiplies the lane's partial sum
//     once; the scales of the workgroup's rows -- contiguous in memory, because the rows are -- are decoded once,
//     by all threads, into LDS before the loop, which then has one memory request per row and wave;
//   * levels come from the byte-indexed pair table (one permute and one 64-bit LDS read per two weights);
//   * the lane sums of four rows are reduced together (eleven DPP and select instructions for the four instead
//     of six adds each) down to one sum per 16 lanes, which go to LDS; when the workgroup has done its rows, the
//     4 KS parts of each row are added in a fixed order (deterministic) and rounded.
// A workgroup is KS x RS waves (KS = slices that cover K, RS = rows handled side by side, at most 16 waves) and
// owns a contiguous range of rows; one workgroup per compute unit, because the pair table takes 64 KiB of LDS.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

constexpr int kSliceElems = 32 * kWave;      // columns per slice
constexpr int kSliceRows = 4;                // rows a wave has in flight and reduces together
constexpr int kSliceChunk = 2;                // code dwords (8 weights each) per step of the lookup pipeline
constexpr int kSliceRedFloats = 4096;        // reduction buffer: rows per workgroup x tokens x slices x 4
constexpr int kSliceScaleFloats = 15360;     // decoded block scales of the workgroup's rows (60 KiB)
constexpr int kSliceMaxWaves = 16;

// Four per-lane values, one per row -> per-row sums over the wave, in 11 instructions instead of 4 x 6: after the
// first exchange the two lanes of a pair hold the same sums, so each keeps one row's; after the second the four
// lanes of a quad hold one row each (lane % 4 = row) and two shifts by 4 and 8 lanes leave in lanes 12..15 of
// every group of 16 lanes the group's sum for rows 0..3.  The four groups' sums are added later, from LDS.
__device__ __forceinline__ float reduce_four_rows(const float (&p)[4], int lane) {
    const float q0 = dpp_add<0xB1, 0xF>(p[0]), q1 = dpp_add<0xB1, 0xF>(p[1]);      // quad_perm [1,0,3,2]
    const float q2 = dpp_add<0xB1, 0xF>(p[2]), q3 = dpp_add<0xB1, 0xF>(p[3]);
    const bool odd = lane & 1;
    const float t0 = odd ? q1 : q0, t1 = odd ? q3 : q2;
    const float u0 = dpp_add<0x4E, 0xF>(t0), u1 = dpp_add<0x4E, 0xF>(t1);          // quad_perm [2,3,0,1]
    float v = (lane & 2) ? u1 : u0;                                                // lane % 4 = row
    v = dpp_add<0x114, 0xF>(v);                                                    // row_shr:4
    v = dpp_add<0x118, 0xF>(v);                                                    // row_shr:8
    return v;
}

// FULL: K is a multiple of 2048, every lane of every slice has columns.  Otherwise the lanes of the last slice
// past K load from the slice's first columns (an address inside the matrix) and contribute exactly zero: their
// activations and their scale are forced to 0.
template <bool FULL>
__global__ __launch_bounds__(kSliceMaxWaves * kWave) void gemv_slice_kernel(
    const uint8_t* __restrict__ packed, const uint8_t* __restrict__ q8, const float* __restrict__ scale2,
    const float* __restrict__ offset_p, const float* __restrict__ code2, int log2_bs, Fmt fmt, int64_t N, int64_t K,
    const _Float16* __restrict__ x, _Float16* __restrict__ y, int KS, int RS, int rows_per_wg) {
    // one LDS object, so that the pair table sits at address 0:
    // table | 16 levels | code2 | reduction buffer | block scales of the workgroup's rows
    constexpr int kOffLut = kPairTableBytes, kOffCode2 = kOffLut + 64, kOffRed = kOffCode2 + 1024;
    constexpr int kOffScales = kOffRed + kSliceRedFloats * 4;
    __shared__ __attribute__((aligned(16))) uint8_t smem[kOffScales + kSliceScaleFloats * 4];
    static_assert(sizeof(smem) <= 160 * 1024, "LDS of one compute unit");
    float* lut = (float*)(smem + kOffLut);
    float* code2_lds = (float*)(smem + kOffCode2);
    float* red = (float*)(smem + kOffRed);
    float* scales = (float*)(smem + kOffScales);

    const int tid = threadIdx.x;
    const int threads = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float offset = offset_p[0];
    const uint32_t lane_off = pair_lane_offset(lane);

    const int ks = wave % KS, rs = wave / KS;
    const int64_t k_slice = (int64_t)ks * kSliceElems;
    const bool live = FULL || k_slice + (uint32_t)lane * 32u < K;  // K is a multiple of 64: 32 columns all in or all out
    const uint32_t le = live ? (uint32_t)lane * 32u : 0u;          // the lane's first column inside the slice
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t r_last = r_begin + rows_per_wg < N ? r_begin + rows_per_wg : N;   // one past the last row; > r_begin

    // The codes of one row of the slice: one load, never predicated (a conditional load would make the compiler
    // wait for everything in flight instead of for the load it needs).  Rows past the workgroup's last are replaced
    // by that last row and their results dropped.
    // Addresses are a wave-uniform row pointer plus the lane's 32-bit offset, so the clamp is scalar arithmetic.
    const uint32_t lane_bytes = le >> 1;
    const uint8_t* last_row_codes = packed + (((r_last - 1) * K + k_slice) >> 1);
    const int n_rows = (int)(r_last - r_begin);                    // rows of this workgroup; rows are counted from r_begin
    auto load_codes = [&](int row, const uint8_t* p) {
        const uint8_t* base = row < n_rows ? p : last_row_codes;   // wave-uniform
        return __builtin_nontemporal_load((const u32x4*)(base + lane_bytes));
    };
    // first thing, so that memory is busy while the tables are built: the first rows' codes
    const int stride = RS;
    const int64_t stride_bytes = ((int64_t)stride * K) >> 1;
    int row = rs;
    const uint8_t* next = packed + (((r_begin + row) * K + k_slice) >> 1);   // codes of the next row to request (wave-uniform)
    u32x4 ring[kSliceRows];
#pragma unroll
    for (int i = 0; i < kSliceRows; ++i) {
        ring[i] = load_codes(row + i * stride, next);
        next += stride_bytes;
    }

    // the lane's activations, converted to FP32 once
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    float xf[32];
    {
        const u32x4* xb = (const u32x4*)(x + k_slice + le);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const u32x4 h = xb[v];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t pair = h[j];                        // (a bit_cast straight from the vector element reads element 0)
                const half2v p = __builtin_bit_cast(half2v, pair);
                xf[8 * v + 2 * j] = live ? (float)p[0] : 0.0f;
                xf[8 * v + 2 * j + 1] = live ? (float)p[1] : 0.0f;
            }
        }
    }

    const int lg = fmt.log2_group;
    if (tid < 16) lut[tid] = fmt.codebook ? fmt.codebook[tid] : __uint_as_float(level_literal(tid));
    for (int i = tid; i < 256; i += threads) code2_lds[i] = code2[i];
    __syncthreads();
    fill_pair_table((float2_t*)smem, lut, tid, threads);
    // Block scales of all the workgroup's rows, decoded once: they are contiguous in memory (rows are), so the
    // workgroup reads them in whole lines, and the loop below takes each lane's scale from LDS.
    const int64_t b_begin = (r_begin * K) >> log2_bs;              // K is a multiple of the block size
    const int nblk = (int)(((r_last - r_begin) * K) >> log2_bs);
    const uint8_t* q8w = q8 + b_begin;
    const bool q8_aligned = ((uintptr_t)q8w & 3) == 0;             // wave-uniform
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int kTurns = 4;                                      // dwords of scale codes per thread and pass
    for (int i0 = 4 * tid; i0 < nblk; i0 += 4 * kTurns * threads) {
        // Thread t takes the four blocks 4 t .. 4 t + 3 of each turn: neighbouring threads read neighbouring
        // dwords and write neighbouring 16-byte pieces of LDS.  Every load first, then the arithmetic: one
        // memory latency per pass, not one per block.
        uint32_t c[kTurns];
        float s2a[kTurns], s2b[kTurns];
#pragma unroll
        for (int t = 0; t < kTurns; ++t) {
            const int i = i0 + 4 * t * threads;
            c[t] = 0;
            s2a[t] = s2b[t] = 0.0f;
            if (i < nblk) {
                if (q8_aligned && i + 4 <= nblk) {
                    c[t] = *(const uint32_t*)(q8w + i);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) c[t] |= (uint32_t)q8w[i + j < nblk ? i + j : nblk - 1] << (8 * j);
                }
                // (four or more blocks per second-level scale -- gemv_slice_eligible -- so that four consecutive blocks
                // touch at most two groups)
                s2a[t] = scale2[(b_begin + i) >> lg];
                s2b[t] = scale2[(b_begin + (i + 3 < nblk ? i + 3 : nblk - 1)) >> lg];
            }
        }
#pragma unroll
        for (int t = 0; t < kTurns; ++t) {
            const int i = i0 + 4 * t * threads;
            if (i >= nblk) continue;
            const int64_t g_first = (b_begin + i) >> lg;
            f32x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float s2 = ((b_begin + i + j) >> lg) == g_first ? s2a[t] : s2b[t];
                const float prod = code2_lds[(c[t] >> (8 * j)) & 0xffu] * s2;      // rounded product, then rounded sum
                v[j] = prod + offset;
            }
            if (i + 4 <= nblk) {
                *(f32x4*)&scales[i] = v;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (i + j < nblk) scales[i + j] = v[j];
            }
        }
    }
    __syncthreads();                                               // tables and scales are complete

    const int blocks_per_row = (int)(K >> log2_bs);
    const int my_block = (int)((k_slice + le) >> log2_bs);         // the lane's block inside a row
    const int group_lane = lane >> 4;                              // which 16 lanes
    constexpr int kChunksPerRow = 4 / kSliceChunk, kLookups = 4 * kSliceChunk, kChunks = kSliceRows * kChunksPerRow;
    for (; row < n_rows; row += kSliceRows * stride) {
        // The four rows as chunks of kSliceChunk code dwords: the lookups of chunk h + 1 are in flight while chunk h
        // is multiplied, so that the LDS latency hides behind the multiply-adds of a chunk.
        float sc[kSliceRows];
#pragma unroll
        for (int i = 0; i < kSliceRows; ++i) {
            const int r = row + i * stride;
            sc[i] = scales[(r < n_rows ? r : n_rows - 1) * blocks_per_row + my_block];
        }
        float2_t lv[2][kLookups];
        auto issue = [&](int h, float2_t (&dst)[kLookups]) {
            const int i = h / kChunksPerRow, c0 = kSliceChunk * (h % kChunksPerRow);
#pragma unroll
            for (int c = 0; c < kSliceChunk; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t a = __builtin_amdgcn_perm(ring[i][c0 + c], lane_off, 0x0c0c0000u | ((4u + k) << 8));
                    dst[4 * c + k] = *(const float2_t*)(smem + a);
                }
        };
        float sums[kSliceRows];
        float pa = 0.0f, pb = 0.0f;
        issue(0, lv[0]);
#pragma unroll
        for (int h = 0; h < kChunks; ++h) {
            const int i = h / kChunksPerRow, x0 = 8 * kSliceChunk * (h % kChunksPerRow);
            if (h + 1 < kChunks) {
                issue(h + 1, lv[(h + 1) & 1]);
                lds_wait<(kLookups < 15 ? kLookups : 15)>();       // everything before the lookups just issued has landed
            } else {
                lds_wait<0>();
            }
            if (h % kChunksPerRow == 0) pa = pb = 0.0f;
#pragma unroll
            for (int k = 0; k < kLookups; ++k) {
                pa = __builtin_fmaf(lv[h & 1][k][0], xf[x0 + 2 * k], pa);          // high nibble: even column
                pb = __builtin_fmaf(lv[h & 1][k][1], xf[x0 + 2 * k + 1], pb);      // low nibble: odd column
            }
            if (h % kChunksPerRow == kChunksPerRow - 1) {          // the row is complete
                float s = sc[i];
                if constexpr (!FULL) s = live ? s : 0.0f;
                sums[i] = s * (pa + pb);
                ring[i] = load_codes(row + (i + kSliceRows) * stride, next);
                next += stride_bytes;
            }
        }
#pragma unroll
        for (int q = 0; q < kSliceRows / 4; ++q) {
            const float four[4] = {sums[4 * q], sums[4 * q + 1], sums[4 * q + 2], sums[4 * q + 3]};
            const float v = reduce_four_rows(four, lane);
            // lane 12 + i of each group of 16 holds that group's sum for row 4 q + i
            const int r = row + (4 * q + (lane & 3)) * stride;
            if ((lane & 12) == 12 && r < n_rows) red[((r * KS + ks) << 2) + group_lane] = v;
        }
    }

    __syncthreads();
    // y[b][r] = the four 16-lane sums of each of the KS slices of row r, in slice order
    for (int r = tid; r < n_rows; r += threads) {
        const float* pr = red + (size_t)r * KS * 4;
        float sum = 0.0f;
        for (int s = 0; s < KS; ++s) sum += (pr[4 * s] + pr[4 * s + 1]) + (pr[4 * s + 2] + pr[4 * s + 3]);
        y[r_begin + r] = (_Float16)sum;
    }
}

// Shapes the column-slice kernel takes: one token (for two, the 64 activations of a lane do not fit the registers of
// a 16-wave workgroup beside the lookup pipeline: the kernel spills and is slower than the row-owning one), rows
// long enough to fill a few slices and short enough for one workgroup to cover K, second-level groups of at least
// four blocks (the decoder of the scales fetches two second-level scales per four blocks; a per-block fetch behind
// a test of the group size put the decoder's registers into scratch memory, and a kernel that uses any scratch
// memory at all measured 5 us slower).
bool gemv_slice_eligible(int64_t N, int64_t K, int B, const Fmt& fmt) {
    return B == 1 && N >= 1 && K >= 4096 && K <= (int64_t)kSliceMaxWaves * kSliceElems && fmt.log2_group >= 2;
}

int launch_gemv_slice(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                      const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                      _Float16* y, hipStream_t s) {
    const int KS = (int)((K + kSliceElems - 1) / kSliceElems);
    const int RS = kSliceMaxWaves / KS;
    const int64_t G = compute_units();
    int64_t rows = (N + G - 1) / G;                                // rows per workgroup: a multiple of RS ...
    rows = (rows + RS - 1) / RS * RS;
    int64_t cap = kSliceRedFloats / (4 * KS);                  // ... whose partial sums and block scales fit LDS
    const int64_t cap_scales = kSliceScaleFloats / (K >> log2_bs);
    if (cap_scales < cap) cap = cap_scales;
    cap = cap / RS * RS;
    if (rows > cap) rows = cap;
    const unsigned groups = (unsigned)((N + rows - 1) / rows);
    const dim3 grid(groups), block(KS * RS * kWave);
    const bool full = K % kSliceElems == 0;
#define NF4_SLICE_LAUNCH(FULL_)                                                                            \
    hipLaunchKernelGGL((gemv_slice_kernel<FULL_>), grid, block, 0, s, packed, q8, scale2, offset, code2, log2_bs, \
                       fmt, N, K, x, y, KS, RS, (int)rows)
    if (B != 1) return NF4_ERR_SHAPE;                              // gemv_slice_eligible
    if (full) NF4_SLICE_LAUNCH(true);
    else NF4_SLICE_LAUNCH(false);
#undef NF4_SLICE_LAUNCH
    return record_hip(hipGetLastError());
}

}  // namespace nf4
