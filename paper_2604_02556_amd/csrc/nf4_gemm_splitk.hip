// Fused NF4 dequantise + small-batch GEMM, split along K across workgroups, with
// the activations staged through LDS (same arithmetic as nf4_gemm.hip: the
// paper's quantised matmul of Sec. III-A / III-C with the FP16 copy of W kept in
// registers; y[b][r] = sum_k x[b][k] * rne_fp16(level[code] * scale)).
//
// The single-launch kernel lets every wave fetch its own activation operands
// from L2, and that traffic -- every workgroup re-reads all of x -- bounds it.
// Here the W waves of a workgroup work on the SAME window of 256 or 512 k for W
// different groups of 16 RG rows, so one copy of the window's activations
// (16 TG tokens x 2 WIN bytes) in LDS serves them all: the workgroup loads it
// once, coalesced, one window ahead, into the other half of a double buffer, and
// the waves read their MFMA B operands from it with ds_read_b128.  Token rows are
// 2 WIN + 32 (SPLIT) or + 16 bytes apart: timed on MI355X, the SPLIT form's reads
// (lane (token, g) at 16 g inside the row) run at the LDS's full rate with + 32
// only (4.2 cycles per wave instruction, 8.0 with + 16, + 48, + 64); the other
// form's (64 g inside the row) take 8.0 whatever the padding.
//
// Because x comes from LDS, a lane is free to take whichever k it likes: lane
// (row, group g) expands k = 128 h + 32 g .. + 31 of the window as its piece h,
// i.e. whole 16-byte pieces as they lie in memory.  The loads use another lane
// numbering than the arithmetic (row = lane / 4, piece = lane % 4 + 4 h, so
// that a quad of lanes reads 64 contiguous bytes); the pieces change lanes
// through a per-wave LDS buffer, one 128-bit write and read each, and the block
// scales come from the lane that loaded them with ds_bpermute.
// Two register sets alternate, the next window's codes in flight while this
// one's are expanded.  The levels come from the byte-indexed pair table
// (issue_pair_lookups, 64 KiB at LDS address 0), the weight is narrowed to FP16 by
// one mixed-precision instruction (scaled_pack2_f16).
//
// Where the time goes (8192 x 28672, 16 tokens, 39-42 us for the kernel): the
// loads alone take about 20 us (a plain read of the same bytes 19), the
// arithmetic alone about 17 us, and the two add up rather than overlap: when the
// memory queues are full a wave blocks in the issue of its next load instead of
// computing, and with one barrier per window all 16 waves are in that state
// together.  Without the scale loads the kernel would be 3 us faster.  Requesting
// two windows ahead, loads spread over the arithmetic steps, waves of a SIMD in
// opposite phases and dedicated loader waves that bring the data straight into
// LDS were each built and measured: no gain.  Nor is the barrier what keeps
// loads and arithmetic apart: with the activations of four windows resident in
// LDS (up to 16 tokens: 64.5 KiB) and the waves meeting once per four windows
// instead of once per window, the kernel takes the same time to 0.5 us
// (40.7 / 41.6 us against 40.3 / 41.3 us at 5 and 16 tokens).
//
// SPLIT = true carries the GEMV's weights through the same kernel (nf4_dequant_gemv_ws): the table holds every
// level as two FP16 terms, lane group g takes dword g of each 16-byte piece instead of whole pieces -- so that the
// 32 k of an MFMA step, 128 h + 32 p + 8 g .., lie in one quantisation block --, the products of a block go
// unscaled into one tile (hi and lo terms, two steps) and the block's FP32 scales, handed from the loading lanes
// to the layout of the C tile through a small per-wave LDS buffer, multiply the tile into the accumulator.  No
// arithmetic per weight, the scale never narrowed.  38-41 us for 3 to 16 tokens on the 70B MLP shapes.
//
// Since all waves of a workgroup share k, K is split across workgroups instead:
// blockIdx.y = split s takes `wps` consecutive windows and writes its partial
// 16 x 16 tiles to partial[s][token][row] (FP32) in the caller's workspace; a
// second kernel adds the S partials in order of s (deterministic) and rounds to
// FP16.  With S = 1 the first kernel writes y itself.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// k per step: 512 for up to 16 tokens (256 bytes of codes per row and step: HBM likes that better than 128,
// and half as many barriers), 256 above that: with two token groups the 512-wide window spilled six registers, and
// a kernel that touches scratch memory at all costs about 4 us per launch (32 tokens: 54 -> 50 us with the narrower
// window and no spill); the activation tiles of 64 tokens would not fit twice in LDS anyway.
constexpr int window_of(int token_groups) { return token_groups <= 1 ? 512 : 256; }

template <int TG, int RG, int W, int WIN, bool SPLIT>
__global__ __launch_bounds__(W * kWave) void gemm_splitk_kernel(const uint8_t* __restrict__ packed,
                                                                const uint8_t* __restrict__ q8,
                                                                const float* __restrict__ scale2,
                                                                const float* __restrict__ offset_p,
                                                                const float* __restrict__ code2, int log2_bs,
                                                                Fmt fmt, int64_t N, int64_t K,
                                                                const _Float16* __restrict__ x, int B, int wps,
                                                                float* __restrict__ partial,
                                                                _Float16* __restrict__ y) {
    constexpr int kThreads = W * kWave;
    constexpr int kTokens = 16 * TG;
    constexpr int kH = WIN / 128;                // 128-bit pieces of codes per lane and row: k = 128 h + 32 g ..
    // Token row of the activation tile.  The 128-bit reads of the MFMA B operands, lane (token, g) at token * row +
    // 16 g (SPLIT) or + 64 g, were timed on MI355X for rows of 2 WIN + 16, + 32, + 48 and + 64 bytes: the first
    // form runs at the LDS's full rate (4.2 cycles per wave instruction) only with + 32, at half of it otherwise.
    constexpr int kXRowBytes = 2 * WIN + (SPLIT ? 32 : 16);
    constexpr int kPiecesPerToken = WIN / 8;     // 16-byte pieces of one token's window
    constexpr int kChunks = kTokens * kPiecesPerToken;
    // Transpose buffer: 64 bytes per row, the four 16-byte pieces of row r at positions piece ^ (r / 4).  Written by
    // lane (row l / 4, piece l % 4) that is the wave's 1 KiB in order, 16 lanes per 256 bytes: full rate (rows of 80
    // bytes took three times as long); read by lane (row l % 16, group l / 16).
    constexpr int kTurnRow = 64;
    constexpr int kU = (kChunks + kThreads - 1) / kThreads;
    constexpr int kXTileBytes = kTokens * kXRowBytes;
    constexpr int kTurnBytes = 16 * kTurnRow;    // one 16-byte piece of each of 16 rows
    // One LDS object, so that the level-pair table sits at address 0 (see issue_pair_lookups):
    // table | two activation tiles | per wave and row group one lane-transpose buffer | code2 | levels
    constexpr int kOffX = kPairTableBytes, kOffTurn = kOffX + 2 * kXTileBytes;
    // SPLIT (the GEMV's weights, see gemm_kernel in nf4_gemm.hip): per wave and row group the window's block scales
    // as [quarter][row] floats, read back in the layout of the C tile
    constexpr int kScaleBytes = SPLIT ? 2 * kH * 16 * 4 : 0;
    constexpr int kOffScale = kOffTurn + W * RG * kTurnBytes;
    constexpr int kOffCode2 = kOffScale + W * RG * kScaleBytes, kOffLut = kOffCode2 + 1024;
    __shared__ __attribute__((aligned(16))) uint8_t smem[kOffLut + 64];
    static_assert(sizeof(smem) <= 160 * 1024, "LDS of one compute unit");
    const uint8_t* table = smem;
    uint8_t* xtile0 = smem + kOffX;
    float* code2_lds = (float*)(smem + kOffCode2);
    float* lut = (float*)(smem + kOffLut);

    const int tid = threadIdx.x;
    const int lg = fmt.log2_group;
    if (tid < 16) lut[tid] = fmt.codebook ? fmt.codebook[tid] : __uint_as_float(level_literal(tid));
    for (int i = tid; i < 256; i += kThreads) code2_lds[i] = code2[i];
    __syncthreads();
    // visible after the barrier that follows the first tile
    if constexpr (SPLIT) fill_split_table((float2_t*)smem, lut, tid, kThreads);
    else fill_pair_table((float2_t*)smem, lut, tid, kThreads);
    const float offset = offset_p[0];
    const float nz = opaque_neg_zero();

    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane & 15;                   // row of a tile (A) / token of a group (B, C)
    const int g = lane >> 4;                     // lane group
    // Loads use another numbering of the lanes than the arithmetic: lane l fetches for row l / 4 its piece l % 4,
    // so that the four lanes of a quad read 64 contiguous bytes.  The address unit of a CU takes about 16 cycles for
    // a 128-bit load whose quads are contiguous and about 64 (one lane per cycle) when neighbouring lanes are in
    // different rows, as they are in the MFMA numbering (row = l % 16) -- measured with cache-resident data.
    const int lrow = lane >> 2;                  // load numbering: row of the tile
    const int lpc = lane & 3;                    //   and 16-byte piece (codes) / 64-element quarter (scales)
    const uint32_t lane_off = pair_lane_offset(lane);
    uint8_t* turn = smem + kOffTurn + wave * (RG * kTurnBytes);   // this wave's transpose buffers
    float* wave_scales = (float*)(smem + kOffScale + wave * (RG * kScaleBytes));
    const int64_t row0 = ((int64_t)blockIdx.x * W + wave) * (16 * RG);
    const int64_t k_begin = (int64_t)blockIdx.y * wps * WIN;
    const int64_t k_stop = k_begin + (int64_t)wps * WIN;
    const int64_t k_end = k_stop < K ? k_stop : K;       // multiple of 64

    // ---- loaders.  K and k_end are multiples of 64, so each 8-, 32- or 64-wide piece is all in or all out.
    // One window of this wave's weights as it arrives from memory; two sets alternate, so that the next
    // window's are in flight while this one's are expanded.
    struct CodeRegs {
        u32x4 c[RG][kH];                         // codes of row lrow: 16-byte groups lpc + 4 h of its WIN / 2 bytes
        uint32_t qb[RG][kH / 2];                 // 8-bit scale code and second-level scale of the window's
        float s2[RG][kH / 2];                    //   64-element quarters lpc and (WIN = 512) lpc + 4
    };
    u32x4 xr[kU];                                // this thread's pieces of the next activation tile
    // A window that lies inside the split with all its rows inside the matrix -- all but the edges -- is loaded
    // without predicates from wave-uniform bases plus 32-bit lane offsets (no register pre-sets, no exec-mask
    // branches, no 64-bit address arithmetic per lane); `small_k` keeps those offsets inside 32 bits.
    const bool small_k = K <= (int64_t(1) << 26);
    const bool rows_inside = row0 + 16 * RG <= N;
    auto load_codes = [&](int64_t kw, CodeRegs& cr) {
        if (small_k && rows_inside && kw + WIN <= k_end) {   // wave-uniform
            const int64_t u = row0 * K + kw;     // flat index of the wave's first element in the window
            const uint8_t* cbase = packed + (u >> 1);
            const int64_t ub = u >> log2_bs;
            const uint32_t ulow = (uint32_t)(u & ((int64_t(1) << log2_bs) - 1));
            const uint8_t* qbase = q8 + ub;
            const float* sbase = scale2 + (ub >> lg);
            const uint32_t ub_low = (uint32_t)(ub & ((int64_t(1) << lg) - 1));
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const uint32_t v = (uint32_t)(16 * r + lrow) * (uint32_t)K;       // elements past u
#pragma unroll
                for (int h = 0; h < kH; ++h)
                    cr.c[r][h] = __builtin_nontemporal_load((const u32x4*)(cbase + ((v >> 1) + 16u * (lpc + 4 * h))));
#pragma unroll
                for (int m = 0; m < kH / 2; ++m) {
                    const uint32_t lb = (ulow + v + 64u * (lpc + 4 * m)) >> log2_bs;   // blocks past ub
                    cr.qb[r][m] = qbase[lb];
                    cr.s2[r][m] = sbase[(ub_low + lb) >> lg];
                }
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const int64_t row = row0 + 16 * r + lrow;
            const bool row_ok = row < N;
            const int64_t e0 = row * K + kw;     // flat index of the row's first element in the window
#pragma unroll
            for (int h = 0; h < kH; ++h) {
                cr.c[r][h] = (u32x4){0x77777777u, 0x77777777u, 0x77777777u, 0x77777777u};   // level 0 if not loaded
                if (row_ok && kw + 32 * (lpc + 4 * h) < k_end)
                    cr.c[r][h] = __builtin_nontemporal_load((const u32x4*)(packed + (e0 >> 1)) + lpc + 4 * h);
            }
#pragma unroll
            for (int m = 0; m < kH / 2; ++m) {
                cr.qb[r][m] = 0;
                cr.s2[r][m] = 0.0f;
                if (row_ok && kw + 64 * (lpc + 4 * m) < k_end) {
                    const int64_t blk = (e0 + 64 * (lpc + 4 * m)) >> log2_bs;
                    cr.qb[r][m] = q8[blk];
                    cr.s2[r][m] = scale2[blk >> lg];
                }
            }
        }
    };
    auto load_x = [&](int64_t kw) {
        if constexpr (kChunks % kThreads == 0) {
            if (kw + WIN <= k_end) {             // uniform: tokens past B read token B - 1 (their columns are never stored)
                const _Float16* xbase = x + kw;
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    const int piece = tid + u * kThreads;
                    int token = piece / kPiecesPerToken;
                    token = token < B ? token : B - 1;
                    xr[u] = *(const u32x4*)(xbase + (int64_t)token * K + 8 * (piece % kPiecesPerToken));
                }
                return;
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int piece = tid + u * kThreads;
            const int token = piece / kPiecesPerToken, kc = piece % kPiecesPerToken;
            xr[u] = (u32x4){0u, 0u, 0u, 0u};
            if (piece < kChunks && token < B && kw + 8 * kc < k_end)
                xr[u] = *(const u32x4*)(x + (int64_t)token * K + kw + 8 * kc);
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int piece = tid + u * kThreads;
            const int token = piece / kPiecesPerToken, kc = piece % kPiecesPerToken;
            if (piece < kChunks) *(u32x4*)(xtile0 + buf * kXTileBytes + token * kXRowBytes + kc * 16) = xr[u];
        }
    };

    f32x4 acc[RG][TG];
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
        for (int t = 0; t < TG; ++t) acc[r][t] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};

    // One window: `cr` holds its codes, `nx` receives those of the next window, xtile[buf] its activations.
    // For the arithmetic lane (row sub, group g) takes piece g + 4 h of its row, k = 128 h + 32 g .. + 31, so MFMA
    // step j takes k = 128 (j / 4) + 32 g + 8 (j % 4) .. + 7.  The pieces change lanes (4 row + piece -> row +
    // 16 piece) through the wave's own LDS buffer.
    auto window = [&](int64_t kw, int buf, const CodeRegs& cr, CodeRegs& nx) {
        float s[RG][kH];
        u32x4 c[RG][kH];
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            // the loading lane holds the scales of quarters lpc and lpc + 4 of row lrow: rounded product, rounded sum
            float mine[kH / 2];
#pragma unroll
            for (int m = 0; m < kH / 2; ++m) {
                const float prod = code2_lds[cr.qb[r][m]] * cr.s2[r][m];
                mine[m] = (row0 + 16 * r + lrow < N && kw + 64 * (lpc + 4 * m) < k_end) ? prod + offset : 0.0f;
            }
            if constexpr (SPLIT) {
                // into the wave's scale buffer, [quarter][row]; read back per block in the main loop
#pragma unroll
                for (int m = 0; m < kH / 2; ++m) wave_scales[r * (kScaleBytes / 4) + (lpc + 4 * m) * 16 + lrow] = mine[m];
            } else {
                // piece h of the arithmetic lane lies in quarter 2 h + g / 2 of row sub: lane 4 sub + quarter % 4, entry h / 2
#pragma unroll
                for (int h = 0; h < kH; ++h)
                    s[r][h] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(
                                                            (4 * sub + ((2 * h + (g >> 1)) & 3)) << 2,
                                                            __builtin_bit_cast(int, mine[h >> 1])));
            }
        }
        // the pieces change lanes one h at a time through the wave's buffer (one per row group)
#pragma unroll
        for (int h = 0; h < kH; ++h) {
#pragma unroll
            for (int r = 0; r < RG; ++r)
                *(u32x4*)(turn + r * kTurnBytes + lrow * kTurnRow + 16 * (lpc ^ (lrow >> 2))) = cr.c[r][h];
            wave_lds_fence();
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                if constexpr (SPLIT) {           // dword g of each of the four pieces: an MFMA step stays in one block
                    const uint32_t* tp = (const uint32_t*)(turn + r * kTurnBytes + sub * kTurnRow + 4 * g);
                    const int sw = sub >> 2;
                    c[r][h] = (u32x4){tp[4 * sw], tp[4 * (1 ^ sw)], tp[4 * (2 ^ sw)], tp[4 * (3 ^ sw)]};
                } else {
                    c[r][h] = *(const u32x4*)(turn + r * kTurnBytes + sub * kTurnRow + 16 * (g ^ (sub >> 2)));
                }
            }
            wave_lds_fence();                    // read before the next h overwrites the buffer
        }

        // ---- the next window's codes and activations start their way from memory now
        load_codes(kw + WIN, nx);
        load_x(kw + WIN);

        constexpr int kSteps = 4 * kH;
        if constexpr (SPLIT) {
            // Lane group g holds dword g of every piece: MFMA step j = (h, p) takes k = 128 h + 32 p + 8 g .. + 7, all
            // inside quarter 2 h + p / 2.  The two steps x two terms (hi, lo) of a quarter go unscaled into one tile,
            // which the quarter's FP32 scales (rows 4 g .. 4 g + 3 of the C layout) multiply into the accumulator.
            const uint8_t* xt = xtile0 + buf * kXTileBytes + sub * kXRowBytes + 16 * g;
            const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
            f32x4 blk[RG][TG];
            f32x4 sc[RG];
            float lv[2][8];
            issue_pair_lookups(c[0][0][0], table, lane_off, lv[0]);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                half8_t xb[TG];
#pragma unroll
                for (int t = 0; t < TG; ++t)
                    xb[t] = *(const half8_t*)(xt + t * 16 * kXRowBytes + 256 * (j >> 2) + 64 * (j & 3));
                if ((j & 1) == 0) {
#pragma unroll
                    for (int r = 0; r < RG; ++r)
                        sc[r] = *(const f32x4*)(wave_scales + r * (kScaleBytes / 4) + (j >> 1) * 16 + 4 * g);
                }
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const int p = j * RG + r;
                    if (p + 1 < kSteps * RG) {
                        const int pj = (p + 1) / RG, pr = (p + 1) % RG;
                        issue_pair_lookups(c[pr][pj >> 2][pj & 3], table, lane_off, lv[(p + 1) & 1]);
                        lds_wait<4>();
                    } else {
                        lds_wait<0>();
                    }
                    u32x4 a, a_lo;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        a[i] = __builtin_bit_cast(uint32_t, lv[p & 1][2 * i]);
                        a_lo[i] = __builtin_bit_cast(uint32_t, lv[p & 1][2 * i + 1]);
                    }
                    const half8_t ah = __builtin_bit_cast(half8_t, a), al = __builtin_bit_cast(half8_t, a_lo);
#pragma unroll
                    for (int t = 0; t < TG; ++t) {
                        blk[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, xb[t], (j & 1) ? blk[r][t] : zero, 0, 0, 0);
                        blk[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, xb[t], blk[r][t], 0, 0, 0);
                    }
                    if (j & 1) {
#pragma unroll
                        for (int t = 0; t < TG; ++t)
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                acc[r][t][i] = __builtin_fmaf(sc[r][i], blk[r][t][i], acc[r][t][i]);
                    }
                }
            }
            store_x(buf ^ 1);
            __syncthreads();
            return;
        }
        // ---- dequantise to FP16 in registers and multiply: lookups pipelined two dwords deep
        const uint8_t* xt = xtile0 + buf * kXTileBytes + sub * kXRowBytes + 64 * g;
        float lv[2][8];
        issue_pair_lookups(c[0][0][0], table, lane_off, lv[0]);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            half8_t xb[TG];
#pragma unroll
            for (int t = 0; t < TG; ++t)
                xb[t] = *(const half8_t*)(xt + t * 16 * kXRowBytes + 256 * (j >> 2) + 16 * (j & 3));
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int p = j * RG + r;
                if (p + 1 < kSteps * RG) {
                    const int pj = (p + 1) / RG, pr = (p + 1) % RG;
                    issue_pair_lookups(c[pr][pj >> 2][pj & 3], table, lane_off, lv[(p + 1) & 1]);
                    lds_wait<4>();
                } else {
                    lds_wait<0>();
                }
                const float sj = s[r][j >> 2];
                u32x4 a;
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = scaled_pack2_f16(lv[p & 1][2 * i], lv[p & 1][2 * i + 1], sj, nz);
                const half8_t ah = __builtin_bit_cast(half8_t, a);
#pragma unroll
                for (int t = 0; t < TG; ++t)
                    acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, xb[t], acc[r][t], 0, 0, 0);
            }
        }

        store_x(buf ^ 1);                        // nobody reads that half before the barrier
        __syncthreads();                         // ... and nobody is still reading it: all passed the previous one
    };

    CodeRegs even, odd;
    load_codes(k_begin, even);
    load_x(k_begin);
    store_x(0);
    __syncthreads();                             // lut, code2_lds and the first tile are in place

    for (int64_t kw = k_begin; kw < k_end; kw += 2 * WIN) {
        window(kw, 0, even, odd);
        if (kw + WIN >= k_end) break;            // uniform over the workgroup
        window(kw + WIN, 1, odd, even);
    }

    // ---- C tile: lane holds token 16 t + sub, rows 4 g .. 4 g + 3 of the row group
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
        for (int t = 0; t < TG; ++t) {
            const int token = 16 * t + sub;
            const int64_t rr = row0 + 16 * r + 4 * g;
            if (token >= B || rr >= N) continue;
            if (partial) {
                float* p = partial + ((int64_t)blockIdx.y * B + token) * N + rr;
                if ((N & 3) == 0) {
                    *(f32x4*)p = acc[r][t];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (rr + i < N) p[i] = acc[r][t][i];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (rr + i < N) y[(int64_t)token * N + rr + i] = (_Float16)acc[r][t][i];
            }
        }
}

// y[i] = rne_fp16(partial[0][i] + partial[1][i] + ... ), summed in that order.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float* __restrict__ partial, int S, int64_t BN,
                                                          _Float16* __restrict__ y) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= BN) return;
    float sum = partial[i];
    for (int s = 1; s < S; ++s) sum += partial[(int64_t)s * BN + i];
    y[i] = (_Float16)sum;
}

// The split: (token groups, row groups per wave, waves per workgroup) by batch,
// then as many splits of K as fill the compute units once.
SplitPlan plan_split(int64_t N, int64_t K, int B) {
    SplitPlan p;
    p.tg = (B + 15) / 16;
    p.rg = 1;
    p.waves = 16;
    const int64_t rows_per_group = 16 * p.rg * p.waves;
    p.row_blocks = (N + rows_per_group - 1) / rows_per_group;
    const int win = window_of(p.tg);
    const int64_t windows = (K + win - 1) / win;
    int64_t S = compute_units() / (p.row_blocks > 0 ? p.row_blocks : 1);
    if (S < 1) S = 1;
    if (S > windows) S = windows;
    p.wps = (int)((windows + S - 1) / S);
    p.splits = (int)((windows + p.wps - 1) / p.wps);
    return p;
}

template <int TG, int RG, int W, bool SPLIT = false>
static void launch_splitk(const SplitPlan& p, const uint8_t* packed, const uint8_t* q8, const float* scale2,
                          const float* offset, const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K,
                          const _Float16* x, int B, float* partial, _Float16* y, hipStream_t s) {
    hipLaunchKernelGGL((gemm_splitk_kernel<TG, RG, W, window_of(TG), SPLIT>), dim3((unsigned)p.row_blocks, (unsigned)p.splits),
                       dim3(W * kWave), 0, s, packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, p.wps,
                       p.splits > 1 ? partial : nullptr, y);
}

int launch_gemm_splitk(const uint8_t* packed, const uint8_t* q8, const float* scale2, const float* offset,
                       const float* code2, int log2_bs, Fmt fmt, int64_t N, int64_t K, const _Float16* x, int B,
                       _Float16* y, float* partial, bool gemv_weights, hipStream_t s) {
    const SplitPlan p = plan_split(N, K, B);
#define NF4_SK_ARGS p, packed, q8, scale2, offset, code2, log2_bs, fmt, N, K, x, B, partial, y, s
    switch (p.tg) {
        case 1:
            if (gemv_weights) launch_splitk<1, 1, 16, true>(NF4_SK_ARGS);     // at most 16 tokens
            else launch_splitk<1, 1, 16>(NF4_SK_ARGS);
            break;
        case 2: launch_splitk<2, 1, 16>(NF4_SK_ARGS); break;
        case 3: launch_splitk<3, 1, 16>(NF4_SK_ARGS); break;
        default: launch_splitk<4, 1, 16>(NF4_SK_ARGS); break;
    }
#undef NF4_SK_ARGS
    int rc = record_hip(hipGetLastError());
    if (rc != NF4_OK || p.splits == 1) return rc;
    const int64_t BN = (int64_t)B * N;
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3((unsigned)((BN + 255) / 256)), dim3(256), 0, s, partial, p.splits,
                       BN, y);
    return record_hip(hipGetLastError());
}

}  // namespace nf4
