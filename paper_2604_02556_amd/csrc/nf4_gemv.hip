// Fused NF4 dequantise + decode GEMV for gfx950: y[b][r] = sum_k x[b][k] *
// W[r][k] with W kept in its 4-bit form (the paper dequantises the whole
// matrix into an FP16 temporary before a dense matmul, Sec. III-C; for a
// handful of tokens that temporary is the dominant traffic, so it is never
// written here).
//
// For one or two tokens (up to four on matrices of 16384 rows and more) this is
// not a dense contraction, so no MFMA: FP32 FMAs and wave64 DPP reductions, the
// kernels of this file.  For more tokens the entry point hands the same sum to
// the matrix-core kernel of nf4_gemm.hip with every level carried as two FP16
// terms and the block scale applied in FP32.  Layout of the work here:
//   * one wave owns R consecutive rows of W over the whole of K, so no partial
//     sums ever leave the wave and the summation order is fixed (deterministic
//     results); the grid is one-shot.  Short rows: single-wave workgroups
//     (gemv_kernel).  Long rows (K >= 16384): eight waves per workgroup, which
//     share one table (gemv_pair_kernel);
//   * per step lane l owns CH consecutive dwords of codes of each row (8*CH
//     elements, always inside one quantisation block): one 128-bit (CH=4) or
//     64-bit (CH=2) load per row, contiguous across the wave.  The loads of
//     step i+1 are issued before the arithmetic of step i;
//   * its 8*CH activations per token stay FP16 in registers and enter the FP32
//     multiply-add directly (mixed-precision FMA), reused for all R rows;
//   * levels come from a 16-entry LDS table written from literals (no bank
//     conflicts, see nf4_dequant.hip) or, in the eight-wave form, from the
//     byte-indexed pair table (issue_pair_lookups: one permute and one 64-bit
//     read per two weights); the double-quantisation map code2 sits in 1 KiB
//     of LDS;
//   * the block scale is applied once per lane chunk (sum of level*x first,
//     then one multiply-add by the scale), not once per element.  Each lane
//     loads the scale code and second-level scale of its own chunk; the
//     long-row kernel, where whole steps allow it, fetches the codes of all four
//     rows with one 16-bit load per lane and shares the decoded scales through
//     LDS (two memory requests per step instead of eight: 6 % faster);
//   * addresses of the level table are taken four at a time: two masked copies
//     of a code dword hold code*4 in each byte, one bit-field extract each;
//   * each accumulator is reduced across the wave with six DPP adds.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

// One step's worth of operands for one lane.
template <int B, int CH, int R>
struct StepRegs {
    uint32_t q[R][CH];      // codes
    half8_t xh[B][CH];      // activations, still FP16
    uint32_t q8[R];         // 8-bit scale codes
    float s2[R];            // second-level scales
};

// Wave-uniform row bases, computed once: codes and scale codes of the rows'
// first elements.  K is a multiple of the blocksize, so a row starts a block.
template <int R>
struct RowBases {
    const uint8_t* codes[R];   // packed + row_start / 2
    const uint8_t* q8[R];      // q8 + row_start / blocksize
    uint32_t blk_lo[R];        // (row_start / blocksize) mod group (blocks per second-level scale)
    const float* s2[R];        // scale2 + (row_start / blocksize) / group
};

// Loads of one step.  `k0` (first element of the step) is wave-uniform, so every
// address is a scalar base plus a 32-bit per-lane offset.
// FULL: every lane chunk is inside K and all R rows exist, so nothing is predicated.
template <int B, int CH, int R, bool FULL>
__device__ __forceinline__ void load_step(StepRegs<B, CH, R>& g, const RowBases<R>& rb,
                                          const _Float16* __restrict__ x, int log2_bs, int lg, int64_t K, int rows,
                                          int64_t k0, int lane) {
    constexpr int E = 8 * CH;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const uint32_t le = (uint32_t)lane * E;                        // element offset of this lane in the step
    const bool live = FULL || k0 + le < K;
    if (live) {
        // block index inside the row = (k0 + le) >> log2_bs: uniform part + small per-lane part
        const int64_t kb = k0 >> log2_bs;
        const uint32_t vb = ((uint32_t)(k0 & ((1 << log2_bs) - 1)) + le) >> log2_bs;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (FULL || r < rows) {                                // wave-uniform
                const uint8_t* codes = rb.codes[r] + (k0 >> 1);
                if constexpr (CH == 4) {
                    const u32x4 v = __builtin_nontemporal_load((const u32x4*)codes + lane);
                    g.q[r][0] = v[0]; g.q[r][1] = v[1]; g.q[r][2] = v[2]; g.q[r][3] = v[3];
                } else if constexpr (CH == 2) {
                    const u32x2 v = __builtin_nontemporal_load((const u32x2*)codes + lane);
                    g.q[r][0] = v[0]; g.q[r][1] = v[1];
                } else {
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        g.q[r][c] = __builtin_nontemporal_load((const uint32_t*)codes + lane * CH + c);
                }
                g.q8[r] = (rb.q8[r] + kb)[vb];
                const int64_t gb = (int64_t)rb.blk_lo[r] + kb;     // block index relative to the row's group base
                const uint32_t vg = ((uint32_t)(gb & ((int64_t(1) << lg) - 1)) + vb) >> lg;
                g.s2[r] = (rb.s2[r] + (gb >> lg))[vg];
            } else {                                               // rows past N: level 0, scale code 0
#pragma unroll
                for (int c = 0; c < CH; ++c) g.q[r][c] = 0x77777777u;
                g.q8[r] = 0;
                g.s2[r] = 0.0f;
            }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const half8_t* xb = (const half8_t*)(x + (int64_t)b * K + k0);
#pragma unroll
            for (int c = 0; c < CH; ++c) g.xh[b][c] = xb[lane * CH + c];
        }
    } else {                                                       // lanes past K in the last step
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int c = 0; c < CH; ++c) g.q[r][c] = 0x77777777u;
            g.q8[r] = 0;
            g.s2[r] = 0.0f;
        }
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
            for (int c = 0; c < CH; ++c) g.xh[b][c] = (half8_t)(_Float16)0;
    }
}

template <int B, int CH, int R>
__device__ __forceinline__ void compute_step(const StepRegs<B, CH, R>& g, const float* lut, const float* code2_lds,
                                             float offset, float (&acc)[R][B]) {
    constexpr int U = R * CH;                                      // dwords of codes in this step
    float c2[R];
#pragma unroll
    for (int r = 0; r < R; ++r) c2[r] = code2_lds[g.q8[r]];
    float lv[2][8];
    issue_lookups(g.q[0][0], lut, lv[0]);
    float part[B];
#pragma unroll
    for (int u = 0; u < U; ++u) {                                  // software pipeline, depth 2
        const int r = u / CH, c = u % CH;
        if (u + 1 < U) {
            issue_lookups(g.q[(u + 1) / CH][(u + 1) % CH], lut, lv[(u + 1) & 1]);
            lds_wait<8>();                                         // everything but the 8 just issued has landed
        } else {
            lds_wait<0>();
        }
        if (c == 0) {
#pragma unroll
            for (int b = 0; b < B; ++b) part[b] = 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int b = 0; b < B; ++b) part[b] = __builtin_fmaf(lv[u & 1][j], (float)g.xh[b][c][j], part[b]);
        if (c == CH - 1) {
            const float prod = c2[r] * g.s2[r];                    // rounded product, then rounded sum
            const float s = prod + offset;
#pragma unroll
            for (int b = 0; b < B; ++b) acc[r][b] = __builtin_fmaf(s, part[b], acc[r][b]);
        }
    }
}

// The block scales of a step through two loads instead of eight (block size 64, whole steps, R = 4 rows of CH
// dwords per lane: 8 CH blocks per row and step).  Sixteen lanes serve a row: lane l fetches the 8-bit codes of
// CH / 2 consecutive blocks of row l / 16 -- one 16-bit load for CH = 4, one byte for CH = 2; the wave reads the
// four rows' 32 or 16 bytes each in one request -- and their second-level scale (two blocks fetched together share
// a group: a group starts at an even block), decodes them and leaves them in this wave's LDS slice, where every
// lane picks up the scale of its own block of each row.  Same arithmetic per scale as the per-lane form (table
// value times second-level scale, rounded, plus offset).
template <int B, int CH>
__device__ __forceinline__ void load_step_merged(StepRegs<B, CH, 4>& g, const RowBases<4>& rb, uint32_t blocks_per_row,
                                                 const _Float16* __restrict__ x, int64_t K, int64_t k0, int lane) {
    static_assert(CH == 2 || CH == 4, "one or two blocks per lane");
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    constexpr uint32_t kPer = CH / 2;                              // blocks per fetching lane
    const int64_t kb = k0 >> 6;
    const uint32_t v = (uint32_t)(lane >> 4) * blocks_per_row + kPer * (uint32_t)(lane & 15);   // blocks past (row 0, kb)
    if constexpr (CH == 4) g.q8[0] = *(const uint16_t*)(rb.q8[0] + kb + v);
    else g.q8[0] = (rb.q8[0] + kb)[v];
    const int64_t gb = (int64_t)rb.blk_lo[0] + kb;
    g.s2[0] = (rb.s2[0] + (gb >> 8))[((uint32_t)(gb & 255) + v) >> 8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint8_t* codes = rb.codes[r] + (k0 >> 1);
        if constexpr (CH == 4) {
            const u32x4 c = __builtin_nontemporal_load((const u32x4*)codes + lane);
            g.q[r][0] = c[0]; g.q[r][1] = c[1]; g.q[r][2] = c[2]; g.q[r][3] = c[3];
        } else {
            const u32x2 c = __builtin_nontemporal_load((const u32x2*)codes + lane);
            g.q[r][0] = c[0]; g.q[r][1] = c[1];
        }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const half8_t* xb = (const half8_t*)(x + (int64_t)b * K + k0);
#pragma unroll
        for (int c = 0; c < CH; ++c) g.xh[b][c] = xb[lane * CH + c];
    }
}

// Decode the scales this lane fetched, hand them round through the wave's LDS slice (4 rows x 8 CH floats) and
// pick up the scale of this lane's own block of each row.
template <int CH>
__device__ __forceinline__ void merged_scales(uint32_t q8_codes, float s2, const float* code2_lds, float offset,
                                              float* wave_scales, int lane, float (&sc)[4]) {
    const float pa = code2_lds[q8_codes & 255u] * s2;              // rounded product, then rounded sum
    if constexpr (CH == 4) {
        const float pb = code2_lds[q8_codes >> 8] * s2;
        *(float2_t*)&wave_scales[2 * lane] = (float2_t){pa + offset, pb + offset};   // [row l / 16][block 2 (l % 16)]
    } else {
        wave_scales[lane] = pa + offset;                           // [row l / 16][block l % 16]
    }
    wave_lds_fence();
    // the lane's 8 CH elements lie in block 8 CH lane / 64 of the step
#pragma unroll
    for (int r = 0; r < 4; ++r) sc[r] = wave_scales[8 * CH * r + (lane >> (CH == 4 ? 1 : 2))];
}

// One step of the long-row kernel with the scales fetched that way.
template <int B, int CH>
__device__ __forceinline__ void compute_step_merged(const StepRegs<B, CH, 4>& g, const uint8_t* table, uint32_t lane_off,
                                                    const float* code2_lds, float offset, float* wave_scales,
                                                    int lane, float (&acc)[4][B]) {
    constexpr int R = 4, U = R * CH;
    float sc[R];
    merged_scales<CH>(g.q8[0], g.s2[0], code2_lds, offset, wave_scales, lane, sc);
    float lv[2][8];
    issue_pair_lookups(g.q[0][0], table, lane_off, lv[0]);
    float part[B];
#pragma unroll
    for (int u = 0; u < U; ++u) {                                  // software pipeline, depth 2
        const int r = u / CH, c = u % CH;
        if (u + 1 < U) {
            issue_pair_lookups(g.q[(u + 1) / CH][(u + 1) % CH], table, lane_off, lv[(u + 1) & 1]);
            lds_wait<4>();                                         // everything but the 4 just issued has landed
        } else {
            lds_wait<0>();
        }
        if (c == 0) {
#pragma unroll
            for (int b = 0; b < B; ++b) part[b] = 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int b = 0; b < B; ++b) part[b] = __builtin_fmaf(lv[u & 1][j], (float)g.xh[b][c][j], part[b]);
        if (c == CH - 1) {
#pragma unroll
            for (int b = 0; b < B; ++b) acc[r][b] = __builtin_fmaf(sc[r], part[b], acc[r][b]);
        }
    }
    wave_lds_fence();                                              // the slice is rewritten by the next step
}

template <int B, int CH, int R, bool FULL>
__global__ __launch_bounds__(kWave, 2) void gemv_kernel(const uint8_t* __restrict__ packed,
                                                     const uint8_t* __restrict__ q8,
                                                     const float* __restrict__ scale2,
                                                     const float* __restrict__ offset_p,
                                                     const float* __restrict__ code2, int log2_bs, Fmt fmt,
                                                     int64_t N, int64_t K, const _Float16* __restrict__ x,
                                                     _Float16* __restrict__ y) {
    constexpr int E = 8 * CH;                 // elements per lane per step
    constexpr int kSlice = E * kWave;         // elements per wave per step
    __shared__ float lut[16];
    __shared__ float code2_lds[256];

    const int lane = threadIdx.x;
    const int lg = fmt.log2_group;
    if (lane < 16) lut[lane] = fmt.codebook ? fmt.codebook[lane] : __uint_as_float(level_literal(lane));
#pragma unroll
    for (int i = 0; i < 4; ++i) code2_lds[lane + 64 * i] = code2[lane + 64 * i];
    wave_lds_fence();
    const float offset = offset_p[0];

    const int64_t r0 = (int64_t)blockIdx.x * R;
    const int rows = (N - r0) < R ? (int)(N - r0) : R;

    float acc[R][B];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < B; ++b) acc[r][b] = 0.0f;

    // K % (8*CH) == 0, so a lane chunk is entirely inside or outside the row
    const int64_t steps = (K + kSlice - 1) / kSlice;
    // two register sets used alternately: the loads of one step are in flight
    // while the other step is being consumed, and nothing is ever copied
    RowBases<R> rb;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t row_start = (r0 + (r < rows ? r : 0)) * K;   // rows past N alias row r0 and are never read
        const int64_t row_blk = row_start >> log2_bs;
        rb.codes[r] = packed + (row_start >> 1);
        rb.q8[r] = q8 + row_blk;
        rb.blk_lo[r] = (uint32_t)(row_blk & ((int64_t(1) << lg) - 1));
        rb.s2[r] = scale2 + (row_blk >> lg);
    }
    StepRegs<B, CH, R> ping, pong;
    load_step<B, CH, R, FULL>(ping, rb, x, log2_bs, lg, K, rows, 0, lane);
    for (int64_t it = 0;;) {
        if (it + 1 < steps) load_step<B, CH, R, FULL>(pong, rb, x, log2_bs, lg, K, rows, (it + 1) * kSlice, lane);
        compute_step<B, CH, R>(ping, lut, code2_lds, offset, acc);
        if (++it >= steps) break;
        if (it + 1 < steps) load_step<B, CH, R, FULL>(ping, rb, x, log2_bs, lg, K, rows, (it + 1) * kSlice, lane);
        compute_step<B, CH, R>(pong, lut, code2_lds, offset, acc);
        if (++it >= steps) break;
    }

#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float total = wave_sum_to_lane63(acc[r][b]);
            if (lane == kWave - 1 && r < rows) y[(int64_t)b * N + r0 + r] = (_Float16)total;
        }
}

// ---- the same kernel for long rows: eight waves per workgroup share the 64 KiB byte-pair table, which cuts a
// third of the instructions per weight.  Building the table once per workgroup pays when a wave has many steps
// (measured on MI355X, 1 to 6 tokens: K = 28672 -> 7-18 % faster, K = 8192 -> 9-17 % slower).  The two kernels
// are kept apart on purpose: the single-wave one is bound by instruction issue and loses 6 % to a few more
// instructions in front of its loop.
constexpr int kPairWaves = 8;
constexpr int64_t kPairMinK = 16384;

template <int B, int CH, int R>
__device__ __forceinline__ void compute_step_pair(const StepRegs<B, CH, R>& g, const uint8_t* table,
                                                  uint32_t lane_off, const float* code2_lds, float offset,
                                                  float (&acc)[R][B]) {
    constexpr int U = R * CH;
    float c2[R];
#pragma unroll
    for (int r = 0; r < R; ++r) c2[r] = code2_lds[g.q8[r]];
    float lv[2][8];
    issue_pair_lookups(g.q[0][0], table, lane_off, lv[0]);
    float part[B];
#pragma unroll
    for (int u = 0; u < U; ++u) {                                  // software pipeline, depth 2
        const int r = u / CH, c = u % CH;
        if (u + 1 < U) {
            issue_pair_lookups(g.q[(u + 1) / CH][(u + 1) % CH], table, lane_off, lv[(u + 1) & 1]);
            lds_wait<4>();                                         // everything but the 4 just issued has landed
        } else {
            lds_wait<0>();
        }
        if (c == 0) {
#pragma unroll
            for (int b = 0; b < B; ++b) part[b] = 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int b = 0; b < B; ++b) part[b] = __builtin_fmaf(lv[u & 1][j], (float)g.xh[b][c][j], part[b]);
        if (c == CH - 1) {
            const float prod = c2[r] * g.s2[r];                    // rounded product, then rounded sum
            const float s = prod + offset;
#pragma unroll
            for (int b = 0; b < B; ++b) acc[r][b] = __builtin_fmaf(s, part[b], acc[r][b]);
        }
    }
}

template <int B, int CH, int R, bool FULL, bool MERGED = false>
__global__ __launch_bounds__(kPairWaves * kWave) void gemv_pair_kernel(const uint8_t* __restrict__ packed,
                                                                       const uint8_t* __restrict__ q8,
                                                                       const float* __restrict__ scale2,
                                                                       const float* __restrict__ offset_p,
                                                                       const float* __restrict__ code2, int log2_bs,
                                                                       Fmt fmt, int64_t N, int64_t K,
                                                                       const _Float16* __restrict__ x,
                                                                       _Float16* __restrict__ y) {
    constexpr int E = 8 * CH;
    constexpr int kSlice = E * kWave;
    constexpr int kThreads = kPairWaves * kWave;
    // one LDS object, so that the pair table sits at address 0: table | 16 levels | code2
    static_assert(!MERGED || (FULL && (CH == 4 || CH == 2) && R == 4), "the two-load scale fetch is for whole steps of four rows");
    constexpr int kScaleBytes = MERGED ? kPairWaves * R * 8 * CH * 4 : 0;   // per wave: R rows x 8 CH block scales
    __shared__ __attribute__((aligned(16))) uint8_t smem[kPairTableBytes + 64 + 1024 + kScaleBytes];
    float* lut = (float*)(smem + kPairTableBytes);
    float* code2_lds = (float*)(smem + kPairTableBytes + 64);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lg = fmt.log2_group;
    if (tid < 16) lut[tid] = fmt.codebook ? fmt.codebook[tid] : __uint_as_float(level_literal(tid));
    for (int i = tid; i < 256; i += kThreads) code2_lds[i] = code2[i];
    __syncthreads();
    fill_pair_table((float2_t*)smem, lut, tid, kThreads);
    __syncthreads();
    const float offset = offset_p[0];
    const uint32_t lane_off = pair_lane_offset(lane);

    const int64_t r0 = ((int64_t)blockIdx.x * kPairWaves + wave) * R;
    if (r0 >= N) return;                      // a whole wave past the last row; no barrier follows
    const int rows = (N - r0) < R ? (int)(N - r0) : R;

    float acc[R][B];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < B; ++b) acc[r][b] = 0.0f;

    const int64_t steps = (K + kSlice - 1) / kSlice;
    RowBases<R> rb;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t row_start = (r0 + (r < rows ? r : 0)) * K;   // rows past N alias row r0 and are never read
        const int64_t row_blk = row_start >> log2_bs;
        rb.codes[r] = packed + (row_start >> 1);
        rb.q8[r] = q8 + row_blk;
        rb.blk_lo[r] = (uint32_t)(row_blk & ((int64_t(1) << lg) - 1));
        rb.s2[r] = scale2 + (row_blk >> lg);
    }
    StepRegs<B, CH, R> ping, pong;
    if constexpr (MERGED) {
        float* wave_scales = (float*)(smem + kPairTableBytes + 64 + 1024) + wave * (R * 8 * CH);
        const uint32_t blocks_per_row = (uint32_t)(K >> 6);
        load_step_merged<B, CH>(ping, rb, blocks_per_row, x, K, 0, lane);
        for (int64_t it = 0;;) {
            if (it + 1 < steps) load_step_merged<B, CH>(pong, rb, blocks_per_row, x, K, (it + 1) * kSlice, lane);
            compute_step_merged<B, CH>(ping, smem, lane_off, code2_lds, offset, wave_scales, lane, acc);
            if (++it >= steps) break;
            if (it + 1 < steps) load_step_merged<B, CH>(ping, rb, blocks_per_row, x, K, (it + 1) * kSlice, lane);
            compute_step_merged<B, CH>(pong, smem, lane_off, code2_lds, offset, wave_scales, lane, acc);
            if (++it >= steps) break;
        }
    } else {
        load_step<B, CH, R, FULL>(ping, rb, x, log2_bs, lg, K, rows, 0, lane);
        for (int64_t it = 0;;) {
            if (it + 1 < steps) load_step<B, CH, R, FULL>(pong, rb, x, log2_bs, lg, K, rows, (it + 1) * kSlice, lane);
            compute_step_pair<B, CH, R>(ping, smem, lane_off, code2_lds, offset, acc);
            if (++it >= steps) break;
            if (it + 1 < steps) load_step<B, CH, R, FULL>(ping, rb, x, log2_bs, lg, K, rows, (it + 1) * kSlice, lane);
            compute_step_pair<B, CH, R>(pong, smem, lane_off, code2_lds, offset, acc);
            if (++it >= steps) break;
        }
    }

#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float total = wave_sum_to_lane63(acc[r][b]);
            if (lane == kWave - 1 && r < rows) y[(int64_t)b * N + r0 + r] = (_Float16)total;
        }
}

template <int B, int CH, int R>
static void launch_gemv(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                        const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const void* x, void* y,
                        hipStream_t s) {
    if (K >= kPairMinK) {
        const unsigned pair_groups = (unsigned)((N + R * kPairWaves - 1) / (R * kPairWaves));
        if constexpr ((CH == 4 || CH == 2) && R == 4) {
            // whole steps, block size 64, the scale codes loadable in pairs: the two-load scale fetch
            // (two neighbouring blocks share a second-level scale: groups of at least two blocks; taken for 256)
            if (K % (8 * CH * kWave) == 0 && N % R == 0 && log2_bs == 6 && aligned(q8, 2) && K % 128 == 0 &&
                K < (int64_t(1) << 31) && fmt.log2_group == 8) {
                hipLaunchKernelGGL((gemv_pair_kernel<B, CH, R, true, true>), dim3(pair_groups),
                                   dim3(kPairWaves * kWave), 0, s, packed, q8, scale2, offset, code2, log2_bs, fmt,
                                   N, K, (const _Float16*)x, (_Float16*)y);
                return;
            }
        }
        if (K % (8 * CH * kWave) == 0 && N % R == 0)
            hipLaunchKernelGGL((gemv_pair_kernel<B, CH, R, true>), dim3(pair_groups), dim3(kPairWaves * kWave), 0, s,
                               packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, (const _Float16*)x,
                               (_Float16*)y);
        else
            hipLaunchKernelGGL((gemv_pair_kernel<B, CH, R, false>), dim3(pair_groups), dim3(kPairWaves * kWave), 0,
                               s, packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, (const _Float16*)x,
                               (_Float16*)y);
        return;
    }
    const unsigned groups = (unsigned)((N + R - 1) / R);
    if (K % (8 * CH * kWave) == 0 && N % R == 0)
        hipLaunchKernelGGL((gemv_kernel<B, CH, R, true>), dim3(groups), dim3(kWave), 0, s, packed, q8, scale2,
                           offset, code2, log2_bs, fmt, N, K, (const _Float16*)x, (_Float16*)y);
    else
        hipLaunchKernelGGL((gemv_kernel<B, CH, R, false>), dim3(groups), dim3(kWave), 0, s, packed, q8, scale2,
                           offset, code2, log2_bs, fmt, N, K, (const _Float16*)x, (_Float16*)y);
}

// Three and four tokens of a shape the 4 x 4 x 4 matrix-core kernel takes.  (One token is faster on the vector ALU;
// two are within a tenth of it there, 37-40 us against 34, and keep the FP32 weight.)
static bool gemv_quad_tokens(int64_t N, int64_t K, int B, int log2_bs, const Fmt& fmt) {
    return B >= 3 && B <= 4 && gemv_quad_eligible(N, K, B, log2_bs, fmt);
}

static int gemv_tokens(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                       const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                       _Float16* y, hipStream_t s) {
    // Column layouts first (rows of 4096 columns and more): one token on the vector ALU, three and four on the small
    // matrix-core instruction (on the 70B MLP shapes 35-39 us, against 44-60 us for the row-owning kernels below
    // and 42-45 us for the split-K kernel).
    if (gemv_slice_eligible(N, K, B, fmt))
        return launch_gemv_slice(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, y, s);
    if (gemv_quad_tokens(N, K, B, log2_bs, fmt))
        return launch_gemv_quad(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, y, s);
#define NF4_GEMV_CASE(b, ch, r) \
    case b: launch_gemv<b, ch, r>(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, y, s); break;
    switch (B) {
        // (tokens, code dwords per lane per row, rows per wave): picked by sweeping on MI355X
        NF4_GEMV_CASE(1, 4, 4) NF4_GEMV_CASE(2, 4, 4) NF4_GEMV_CASE(3, 2, 4) NF4_GEMV_CASE(4, 2, 4)
        default: return NF4_ERR_SHAPE;           // more tokens go to the matrix cores (mfma_min_tokens)
    }
#undef NF4_GEMV_CASE
    return record_hip(hipGetLastError());
}

}  // namespace nf4

namespace nf4 {
// Where the matrix-core kernel takes over, measured on MI355X (us per call, FMA kernels / matrix cores):
//   8192 x 28672:  2 tokens 38.9 / 42.7,  3 tokens 46.1 / 43.2,  4 tokens 54.3 / 43.2,  6 tokens 65.7 / 43.9
//   28672 x 8192:  3 tokens 44.8 / 54.9,  4 tokens 54.0 / 55.4,  5 tokens 62.3 / 55.4,  6 tokens 76.3 / 56.2
// (matrices of 16384 rows and more run it with more workgroups than stay resident, which costs it 12 us).
static int mfma_min_tokens(int64_t N) { return N < 16384 ? 3 : 5; }
// With a workspace (nf4_dequant_gemv_ws) the matrix-core sum is split along K across workgroups that share the
// activations through LDS: 38-41 us for 2 to 16 tokens on both 70B MLP shapes, against 36-37 us for the FMA kernels
// at 2 tokens and 41-44 at 3.
constexpr int kSplitMinTokens = 3;

int launch_gemv_ws(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                   const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                   _Float16* y, float* partial, hipStream_t s) {
    if (B < kSplitMinTokens || gemv_quad_tokens(N, K, B, log2_bs, fmt))
        return gemv_tokens(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, y, s);
    return launch_gemm_splitk(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, y, partial, true, s);
}

// Argument checks shared by the GEMV entry points (everything but the workspace).
static int check_gemv_args(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                           const float* code2, int blocksize, int64_t N, int64_t K, const void* x, int B,
                           const void* y, const Fmt& fmt, int* log2_bs) {
    if (N < 0 || K < 0) return NF4_ERR_SIZE;
    *log2_bs = log2_blocksize(blocksize);
    if (*log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (B < 1 || B > 16) return NF4_ERR_SHAPE;
    if (fmt.log2_group < 0) return NF4_ERR_SHAPE;
    if (N > 0 && (K <= 0 || K % blocksize != 0)) return NF4_ERR_SHAPE;   // blocksize is a multiple of 32
    if (N > 0x7fffffffLL) return NF4_ERR_SIZE;
    if (N == 0) return NF4_OK;
    if (!packed || !q8 || !scale2 || !offset || !code2 || !x || !y) return NF4_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(x, 16) || !aligned(y, 2) || !aligned(scale2, 4) || !aligned(offset, 4) ||
        !aligned(code2, 4) || !aligned(fmt.codebook, 4))
        return NF4_ERR_ALIGN;
    return NF4_OK;
}

// nf4_dequant_gemv / nf4_dequant_gemv_ws (workspace != nullptr) for any format.
static int gemv_entry(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                      const float* code2, int blocksize, Fmt fmt, int64_t N, int64_t K, const void* x, int B,
                      void* y, bool with_workspace, void* workspace, size_t workspace_bytes, void* stream) {
    int log2_bs = 0;
    const int rc = check_gemv_args(packed, q8, scale2, offset, code2, blocksize, N, K, x, B, y, fmt, &log2_bs);
    if (rc != NF4_OK || N == 0) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (with_workspace) {
        if (!workspace) return NF4_ERR_NULL;
        if (!aligned(workspace, 16)) return NF4_ERR_ALIGN;
        if (workspace_bytes < nf4_dequant_gemv_workspace_bytes(N, K, B)) return NF4_ERR_SIZE;
        return launch_gemv_ws(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, (const _Float16*)x, B,
                              (_Float16*)y, (float*)workspace, s);
    }
    // From mfma_min_tokens tokens on the sum goes to the matrix cores: the levels enter them as two FP16 terms
    // (22 significant bits), the activations as they are, the block scale multiplies each block's partial sums in
    // FP32, accumulation in FP32.  Below that, FMAs on the vector ALU with the FP32 weight never narrowed.
    if (B >= mfma_min_tokens(N) && !gemv_quad_tokens(N, K, B, log2_bs, fmt))
        return launch_gemv_mfma(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, (const _Float16*)x, B,
                                (_Float16*)y, s);
    return gemv_tokens(packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, (const _Float16*)x, B, (_Float16*)y, s);
}
}

extern "C" int nf4_dequant_gemv(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                const float* offset, const float* code2, int blocksize, int64_t N,
                                int64_t K, const void* x, int B, void* y, void* stream) {
    return nf4::gemv_entry(packed, absmax_q8, scale2, offset, code2, blocksize, nf4::kNf4Fmt, N, K, x, B, y, false,
                           nullptr, 0, stream);
}

// ---- the same sum with a caller workspace: from kSplitMinTokens tokens on K is split across workgroups (the
// split-K kernel of nf4_gemm_splitk.hip with the GEMV's weights: levels as two FP16 terms, FP32 block scales).
extern "C" size_t nf4_dequant_gemv_workspace_bytes(int64_t N, int64_t K, int B) {
    if (N <= 0 || K <= 0 || B < 1 || B > 16) return 0;
    const nf4::SplitPlan p = nf4::plan_split(N, K, B);
    return p.splits > 1 ? (size_t)p.splits * (size_t)B * (size_t)N * sizeof(float) : 16;
}

extern "C" int nf4_dequant_gemv_ws(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                   const float* offset, const float* code2, int blocksize, int64_t N, int64_t K,
                                   const void* x, int B, void* y, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    return nf4::gemv_entry(packed, absmax_q8, scale2, offset, code2, blocksize, nf4::kNf4Fmt, N, K, x, B, y, true,
                           workspace, workspace_bytes, stream);
}

// ---- the data type as a parameter (Sec. V-A): the same two calls for any 16 levels and second-level group size
extern "C" int nf4_dequant_gemv_codebook(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                         const float* offset, const float* code2, int dq_group,
                                         const float* codebook, int blocksize, int64_t N, int64_t K, const void* x,
                                         int B, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    const nf4::Fmt fmt = {nf4::log2_dq_group(dq_group), codebook};
    return nf4::gemv_entry(packed, absmax_q8, scale2, offset, code2, blocksize, fmt, N, K, x, B, y,
                           workspace != nullptr, workspace, workspace_bytes, stream);
}
