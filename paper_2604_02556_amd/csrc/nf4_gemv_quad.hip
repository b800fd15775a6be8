// Fused NF4 dequantise + decode GEMV for up to four tokens on the small matrix-core instruction
// (v_mfma_f32_4x4x4_16B_f16: sixteen independent 4 x 4 x 4 products per wave), laid out by columns like the one-token
// kernel of nf4_gemv_slice.hip.
//
// Why this instruction: its lane layout is the one a coalesced read of W wants.  Lane l belongs to block l / 4 and
// supplies, as the B operand, four consecutive k of ONE weight row (row l % 4 of a group of four rows) and, as the A
// operand, four consecutive k of ONE token (token l % 4); the result D[token][row] of a block lands in the lane of that
// row, four tokens in four registers.  So
//   * lane (c = l / 4, i = l % 4) loads the 16 bytes of codes of row i of the group at columns 32 c .. 32 c + 31 of
//     the wave's 512 columns: a wave-load is 4 rows x 256 contiguous bytes, and the waves of a workgroup that share
//     the rows read them side by side (the 16-row tiles of the big MFMA shapes would be 64 bytes per row, and at
//     block size 64 could not keep the 32 k of a step in one quantisation block without moving codes between lanes);
//   * the lane's 32 activations (token i, its own columns) stay in 32 registers, each pair twice, for the whole pass over
//     the rows: no activation traffic in the loop, nothing goes through LDS except the lookups;
//   * a lane's 32 columns lie in one quantisation block and its results are those of its own row, so the block scale
//     is applied by the lane that owns it, in FP32, to the four sums of eight 4-wide steps;
//   * every level enters as two FP16 terms (the split table of nf4_device.hpp: hi + lo = the level to about 2^-22),
//     two MFMAs per step, as on the other matrix-core paths of the GEMV; accumulation in FP32;
//   * the cost does not depend on the number of tokens (1 to 4): 16 lookups, 16 permutes, 16 small MFMAs (8 cycles
//     each) and about 33 other vector instructions per 2048 weights and wave, against 32 B multiply-adds, 16 permutes
//     and about 11 others on the vector ALU: slower than the one-token kernel, level with two tokens, ahead from three.
// A workgroup is KSW column waves x RS row streams (at most 16 waves) and owns a contiguous range of rows; when K is
// wider than its waves it passes over the rows once per group of columns, reloading the 32 activation registers, and
// adds into the same LDS slots; the ring of four loads per wave keeps running from one pass into the next.  Per
// (row, token) the sums of the sixteen 32-column pieces of a wave meet by two DPP adds down to one per 16 lanes;
// those go to LDS and are added in a fixed order at the end (deterministic).  Block scales are decoded once per
// workgroup into LDS as in the one-token kernel.
// Measured on the 70B MLP shapes (8192 x 28672 / 28672 x 8192, eight weight copies cycled): 32-34 / 34-36 us at three
// tokens, 33.5-36.5 / 36-37.4 us at four; with the code loads alone 25.5-28.6 us, with everything but them 27-28 us:
// the kernel is bound by instruction issue (a SIMD's vector pipe is taken for 11-12 k of the 14-18 k issue slots a
// wave lives, a fifth of the instructions being MFMAs that hold it for two).
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kQuadCols = 512;               // columns per wave: 16 blocks of the MFMA x 32
constexpr int kQuadRing = 4;                 // row groups whose codes a wave has in flight
constexpr int kQuadMaxWaves = 16;
constexpr int kQuadRedBytes = 32 * 1024;     // per row and slot (column wave x 16 lanes) one f32x4 of token sums
constexpr int kQuadScaleFloats = 15360;      // decoded block scales of the workgroup's rows (60 KiB)

// FULL: K is a multiple of 512 and the column groups divide it evenly: every lane of every wave has columns in every
// pass.  Otherwise lanes past K load from the row's first columns and contribute exactly zero (their activations and
// scale are forced to 0).
// CGN: passes over the rows, one per group of KSW x 512 columns; a template parameter, the loop over it unrolled.
template <bool FULL, int CGN>
__global__ __launch_bounds__(kQuadMaxWaves * kWave) void gemv_quad_kernel(
    const uint8_t* __restrict__ packed, const uint8_t* __restrict__ q8, const float* __restrict__ scale2,
    const float* __restrict__ offset_p, const float* __restrict__ code2, int log2_bs, Fmt fmt, int64_t N, int64_t K,
    const _Float16* __restrict__ x, int B, _Float16* __restrict__ y, int KSW, int RS, int rows_per_wg) {
    // one LDS object, so that the split table sits at address 0:
    // table | 16 levels | code2 | token sums per row and slot | block scales of the workgroup's rows
    constexpr int kOffLut = kPairTableBytes, kOffCode2 = kOffLut + 64, kOffRed = kOffCode2 + 1024;
    constexpr int kOffScales = kOffRed + kQuadRedBytes;
    __shared__ __attribute__((aligned(16))) uint8_t smem[kOffScales + kQuadScaleFloats * 4];
    static_assert(sizeof(smem) <= 160 * 1024, "LDS of one compute unit");
    float* lut = (float*)(smem + kOffLut);
    float* code2_lds = (float*)(smem + kOffCode2);
    f32x4* red = (f32x4*)(smem + kOffRed);
    float* scales = (float*)(smem + kOffScales);

    const int tid = threadIdx.x;
    const int threads = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lg = fmt.log2_group;
    const float offset = offset_p[0];
    const uint32_t lane_off = pair_lane_offset(lane);
    const int ksw = wave % KSW, rs = wave / KSW;
    const int c = lane >> 2, i = lane & 3;       // block of the MFMA = 32-column piece; row of the group = token
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t r_last = r_begin + rows_per_wg < N ? r_begin + rows_per_wg : N;   // one past the last row; > r_begin
    const int n_rows = (int)(r_last - r_begin);
    const int n_groups = (n_rows + 3) >> 2;      // groups of four rows

    // ---- tables and block scales (as in nf4_gemv_slice.hip)
    if (tid < 16) lut[tid] = fmt.codebook ? fmt.codebook[tid] : __uint_as_float(level_literal(tid));
    for (int t = tid; t < 256; t += threads) code2_lds[t] = code2[t];
    __syncthreads();
    fill_split_table((float2_t*)smem, lut, tid, threads);
    const int blocks_per_row = (int)(K >> log2_bs);
    {
        const int64_t b_begin = (r_begin * K) >> log2_bs;          // K is a multiple of the block size
        const int nblk = n_rows * blocks_per_row;
        const uint8_t* q8w = q8 + b_begin;
        const bool q8_aligned = ((uintptr_t)q8w & 3) == 0;         // wave-uniform
        constexpr int kTurns = 4;                                  // dwords of scale codes per thread and pass
        for (int i0 = 4 * tid; i0 < nblk; i0 += 4 * kTurns * threads) {
            uint32_t cq[kTurns];
            float s2a[kTurns], s2b[kTurns];
#pragma unroll
            for (int t = 0; t < kTurns; ++t) {
                const int b = i0 + 4 * t * threads;
                cq[t] = 0;
                s2a[t] = s2b[t] = 0.0f;
                if (b < nblk) {
                    if (q8_aligned && b + 4 <= nblk) {
                        cq[t] = *(const uint32_t*)(q8w + b);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) cq[t] |= (uint32_t)q8w[b + j < nblk ? b + j : nblk - 1] << (8 * j);
                    }
                    // (four or more blocks per second-level scale -- gemv_quad_eligible -- so that four consecutive
                    // blocks touch at most two groups)
                    s2a[t] = scale2[(b_begin + b) >> lg];
                    s2b[t] = scale2[(b_begin + (b + 3 < nblk ? b + 3 : nblk - 1)) >> lg];
                }
            }
#pragma unroll
            for (int t = 0; t < kTurns; ++t) {
                const int b = i0 + 4 * t * threads;
                if (b >= nblk) continue;
                const int64_t g_first = (b_begin + b) >> lg;
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float s2 = ((b_begin + b + j) >> lg) == g_first ? s2a[t] : s2b[t];
                    const float prod = code2_lds[(cq[t] >> (8 * j)) & 0xffu] * s2;   // rounded product, then rounded sum
                    v[j] = prod + offset;
                }
                if (b + 4 <= nblk) {
                    *(f32x4*)&scales[b] = v;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (b + j < nblk) scales[b + j] = v[j];
                }
            }
        }
    }
    __syncthreads();                                               // tables and scales are complete

    const int slots = 4 * KSW;                                     // per row: column wave x 16 lanes
    const int my_slot = 4 * ksw + (lane >> 4);
    const int stride = RS;                                         // in groups of four rows

    // The wave's columns in pass cg: lane piece c of column wave cg * KSW + ksw.  A lane past K reads the rows' first
    // columns instead (and contributes zero).
    auto pass_columns = [&](int cg, bool& live, int64_t& first) {
        const int64_t col0 = ((int64_t)cg * KSW + ksw) * kQuadCols;
        live = FULL || col0 + 32 * c < K;                          // K is a multiple of 64: 32 columns all in or all out
        first = live ? col0 + 32 * c : 0;                          // the lane's first column
    };
    // Codes of one group of four rows: one load per lane, never predicated; rows past the workgroup's last are
    // replaced by that last row and their results dropped.  A wave-uniform pointer plus a 32-bit lane offset
    // (rows per workgroup x K / 2 stays far below 2^31).
    const uint8_t* rows0 = packed + ((r_begin * K) >> 1);
    const uint32_t row_bytes = (uint32_t)(K >> 1);
    uint32_t col_bytes[CGN];
#pragma unroll
    for (int cg = 0; cg < CGN; ++cg) {
        bool live;
        int64_t first;
        pass_columns(cg, live, first);
        col_bytes[cg] = (uint32_t)(first >> 1);
    }
    auto load_codes = [&](int g, uint32_t cb) {
        const int row = 4 * g + i;
        const uint32_t rc = (uint32_t)(row < n_rows ? row : n_rows - 1);
        const uint32_t off = __umul24(rc, row_bytes) + cb;         // both factors below 2^24: one full-rate multiply-add
        return __builtin_nontemporal_load((const u32x4*)(rows0 + off));
    };
    // Four groups in flight per wave, and the ring does not drain between passes: in the last round of a pass the
    // reloads fetch the first groups of the next pass (with 8 to 28 groups per wave and pass, stopping and
    // restarting the stream at every pass cost 2 to 3 us each).
    u32x4 ring[kQuadRing];
#pragma unroll
    for (int r = 0; r < kQuadRing; ++r) ring[r] = load_codes(rs + r * stride, col_bytes[0]);

    // The 16 lookups of a group in two halves (two dwords of codes, eight lookups, four MFMA steps each), one half
    // ahead of the MFMAs: while the matrix core works on one half the LDS serves the other -- across groups and
    // passes too, the first half of the next group is requested before the second half of this one is multiplied.
    float2_t lva[8], lvb[8];
    auto issue = [&](const u32x4& codes, int h, float2_t (&dst)[8]) {
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t a = __builtin_amdgcn_perm(codes[2 * h + d], lane_off, 0x0c0c0000u | ((4u + k) << 8));
                dst[4 * d + k] = *(const float2_t*)(smem + a);
            }
    };
    issue(ring[0], 0, lva);

#pragma unroll
    for (int cg = 0; cg < CGN; ++cg) {
        bool live;
        int64_t first;
        pass_columns(cg, live, first);
        // The lane's activations for this pass: token i, columns first .. first + 31.  One MFMA handles one byte of
        // codes, i.e. two columns: its B operand is what the lookup returns -- (hi, hi) of the two weights, then
        // (lo, lo) -- and its A operand the two activations twice, (x_even, x_odd, x_even, x_odd), so that the four
        // products of the step are hi * x + lo * x of both columns.  16 such operands, 2 registers each.
        u32x2 xa[16];
        {
            const u32x4* xb = (const u32x4*)(x + (int64_t)(i < B ? i : 0) * K + first);
            const bool on = live && i < B;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const u32x4 h = xb[v];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t pair = on ? h[j] : 0u;
                    xa[4 * v + j] = (u32x2){pair, pair};
                }
            }
        }
        const int my_block = (int)(first >> log2_bs);              // the lane's block inside a row
        auto multiply = [&](const float2_t (&lv)[8], int h, f32x4& acc0, f32x4& acc1) {
#pragma unroll
            for (int b = 0; b < 8; b += 2) {                       // byte 8 h + b of the lane's 16: columns 16 h + 2 b, + 1
                const half4_t w0 = __builtin_bit_cast(half4_t, lv[b]), w1 = __builtin_bit_cast(half4_t, lv[b + 1]);
                acc0 = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, xa[8 * h + b]), w0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, xa[8 * h + b + 1]), w1, acc1, 0, 0, 0);
            }
        };
        for (int g = rs; g < n_groups; g += kQuadRing * stride) {
            const bool last_round = g + kQuadRing * stride >= n_groups;   // wave-uniform
#pragma unroll
            for (int r = 0; r < kQuadRing; ++r) {
                const int gg = g + r * stride;                     // this group (may be past the end: dropped below)
                const int row = 4 * gg + i;
                const int rc = row < n_rows ? row : n_rows - 1;
                float sc = scales[__umul24((uint32_t)rc, (uint32_t)blocks_per_row) + (uint32_t)my_block];
                if constexpr (!FULL) sc = live ? sc : 0.0f;
                issue(ring[r], 1, lvb);
                // its codes are all turned into addresses: the slot's next group, in this pass or the next one
                if (cg + 1 < CGN)
                    ring[r] = load_codes(last_round ? rs + r * stride : gg + kQuadRing * stride,
                                         last_round ? col_bytes[cg + 1] : col_bytes[cg]);
                else
                    ring[r] = load_codes(gg + kQuadRing * stride, col_bytes[cg]);
                f32x4 acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};   // two chains: MFMA latency
                lds_wait<8>();
                multiply(lva, 0, acc0, acc1);
                issue(ring[(r + 1) % kQuadRing], 0, lva);          // the next group's first half (after the last group: unused)
                lds_wait<8>();
                multiply(lvb, 1, acc0, acc1);
                const f32x4 acc = acc0 + acc1;
                // acc[m] = token m, this lane's row, this lane's 32 columns: scale, then add the 4 pieces of a DPP row
                // (the four tokens step by step: a lane shift must wait two instructions for its operand)
                f32x4 v;
#pragma unroll
                for (int m = 0; m < 4; ++m) v[m] = sc * acc[m];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int m = 0; m < 4; ++m) v[m] = dpp_add<0x114, 0xF>(v[m]);      // row_shr:4
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int m = 0; m < 4; ++m) v[m] = dpp_add<0x118, 0xF>(v[m]);      // row_shr:8 -> lanes 12..15 hold the sums for rows 0..3
                // (used here, before the branch: otherwise the compiler moves the last adds into the branch, where
                // they cannot merge with the lane shifts, and pays a move, the add and a cleared register instead)
                asm volatile("" : "+v"(v));
                if ((lane & 12) == 12 && row < n_rows) {
                    f32x4* slot = red + my_slot * rows_per_wg + row;   // the four rows of a group side by side: no bank conflict
                    if (cg == 0) *slot = v;
                    else *slot = *slot + v;
                }
            }
        }
    }
    lds_wait<0>();                                                 // the lookups requested last are not used

    __syncthreads();
    // y[b][r] = the sums of row r's slots, in slot order
    for (int o = tid; o < n_rows * B; o += threads) {
        const int r = o / B, b = o % B;
        const f32x4* pr = red + r;
        float sum = 0.0f;
        for (int s = 0; s < slots; ++s) sum += pr[s * rows_per_wg][b];
        y[(int64_t)b * N + r_begin + r] = (_Float16)sum;
    }
}

// Shapes it takes: up to four tokens; K from 4096 up; second-level groups of at least four blocks (the scale decoder).
// The split of a shape: rows per workgroup, column waves, passes, row streams.
struct QuadPlan {
    int64_t rows;
    int ksw, cgn, rs;
};
static bool plan_quad(int64_t N, int64_t K, int log2_bs, QuadPlan& p) {
    const int nsl = (int)((K + kQuadCols - 1) / kQuadCols);        // 512-column slices of a row
    const int64_t G = compute_units();
    int64_t rows = (N + G - 1) / G;
    rows = (rows + 3) / 4 * 4;
    const int64_t cap_scales = kQuadScaleFloats / (K >> log2_bs) / 4 * 4;   // rows whose block scales fit LDS
    if (cap_scales < 4) return false;
    if (rows > cap_scales) rows = cap_scales;
    // column waves: as many as keep rows x 4 KSW slots of 16 bytes inside the reduction buffer, at most 16 and nsl
    int ksw = (int)(kQuadRedBytes / 16 / 4 / rows);
    if (ksw > kQuadMaxWaves) ksw = kQuadMaxWaves;
    if (ksw > nsl) ksw = nsl;
    if (ksw < 1) return false;
    const int cgn = (nsl + ksw - 1) / ksw;
    if (cgn > 4) return false;
    ksw = (nsl + cgn - 1) / cgn;                                   // even the passes out
    int rs = kQuadMaxWaves / ksw;
    if (rs > (int)(rows / 4)) rs = (int)(rows / 4);
    p = {rows, ksw, cgn, rs};
    return true;
}

// Shapes it takes: up to four tokens; rows of 4096 columns and more that four passes of a workgroup cover; second-level
// groups of at least four blocks (the scale decoder).
bool gemv_quad_eligible(int64_t N, int64_t K, int B, int log2_bs, const Fmt& fmt) {
    QuadPlan p;
    return B >= 1 && B <= 4 && N >= 1 && K >= 4096 && fmt.log2_group >= 2 && plan_quad(N, K, log2_bs, p);
}

int launch_gemv_quad(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                     const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                     _Float16* y, hipStream_t s) {
    QuadPlan p;
    if (!plan_quad(N, K, log2_bs, p)) return NF4_ERR_SHAPE;       // gemv_quad_eligible keeps such shapes away
    const int64_t rows = p.rows;
    const int ksw = p.ksw, cgn = p.cgn, rs = p.rs;
    const int nsl = (int)((K + kQuadCols - 1) / kQuadCols);
    const unsigned grid = (unsigned)((N + rows - 1) / rows);
    const bool full = K % kQuadCols == 0 && nsl == cgn * ksw;
#define NF4_QUAD_LAUNCH(FULL_, CGN_)                                                                             \
    hipLaunchKernelGGL((gemv_quad_kernel<FULL_, CGN_>), dim3(grid), dim3(ksw * rs * kWave), 0, s, packed, q8, scale2, \
                       offset, code2, log2_bs, fmt, N, K, x, B, y, ksw, rs, (int)rows)
    switch (cgn) {
        case 1: if (full) NF4_QUAD_LAUNCH(true, 1); else NF4_QUAD_LAUNCH(false, 1); break;
        case 2: if (full) NF4_QUAD_LAUNCH(true, 2); else NF4_QUAD_LAUNCH(false, 2); break;
        case 3: if (full) NF4_QUAD_LAUNCH(true, 3); else NF4_QUAD_LAUNCH(false, 3); break;
        default: if (full) NF4_QUAD_LAUNCH(true, 4); else NF4_QUAD_LAUNCH(false, 4); break;
    }
#undef NF4_QUAD_LAUNCH
    return record_hip(hipGetLastError());
}

}  // namespace nf4
