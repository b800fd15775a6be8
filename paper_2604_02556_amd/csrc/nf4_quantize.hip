// Tuned NF4 quantiser for gfx950 (every block size, 64 to 4096; any n): the forward direction of
// Sec. II-B, bit-identical to the reference quantiser (and so to the CPU
// definition), at HBM speed.
//
// Per block: absmax = max |x|; per element: x / absmax (IEEE division) mapped
// to the nearest of the 16 levels, nearest meaning smallest |x/absmax - level|
// evaluated in FP32, ties to the lower index.
//
// How the 16-way search is avoided without changing a single result.  For
// adjacent levels k, k+1 the predicate "level k+1 is strictly nearer (in
// rounded FP32 distance) than level k" is monotone in x, so it is equivalent to
// x >= theta_k for one FP32 threshold theta_k, and the code of x is the number
// of thresholds it reaches.  The 15 thresholds are found on the host at first
// use by bisection over the FP32 number line with exactly that predicate
// (plain FP32 subtract / abs / compare), not taken as midpoints: rounding moves
// several of them by up to one ulp.  The thresholds are at least 0.08 apart, so
// each of 64 bins of width 1/32 over [-1, 1] holds at most one; a bin stores
// the count of thresholds below it and the one inside it (or +inf), and a code
// costs one table read, one compare and one add.
//
// Data movement: one wave per 2048 elements; eight 128-bit loads per lane, each
// contiguous across the wave; a block of 64 is then spread over the 16 lanes of
// one DPP row (4 elements each), so its absmax is 3 in-lane and 4 DPP max
// operations and needs no LDS; larger blocks add one or two cross-row exchanges
// (ds_bpermute) and, from 512 on, a maximum over 2, 4 or 8 of the lane's own
// loads, and for 4096 a maximum over the two waves of a workgroup; codes leave as
// eight 2-byte stores per lane, each instruction writing one full 128-byte line.
#include <math.h>
#include <string.h>

#include <mutex>

#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

constexpr int kQTileElems = 2048;
constexpr int kBins = 65;             // x / absmax = +1 lands in a bin of its own

struct QuantBins {
    float theta[kBins];      // the threshold inside the bin, +inf if none
    uint32_t base[kBins];    // thresholds below the bin
};

// ---- host: thresholds and bins -------------------------------------------------

static float host_level(int k) {
    const uint32_t bits = level_literal((uint32_t)k);
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

// Monotone map between FP32 values and integers (for bisection over the number line).
static int64_t float_key(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    return (u >> 31) ? -(int64_t)(u & 0x7fffffffu) : (int64_t)u;
}
static float key_float(int64_t k) {
    uint32_t u = k < 0 ? (0x80000000u | (uint32_t)(-k)) : (uint32_t)k;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint32_t bin_of(float xn) {                       // same arithmetic as the kernel; xn in [-1, 1]
    const float pos = fmaf(xn, 32.0f, 32.0f);            // in [0, 64]
    return pos <= 0.0f ? 0u : (uint32_t)pos;
}

static bool build_bins(QuantBins& qb) {
    float theta[15];
    for (int k = 0; k < 15; ++k) {
        const float lo_level = host_level(k), hi_level = host_level(k + 1);
        int64_t lo = float_key(lo_level), hi = float_key(hi_level);   // predicate false at lo, true at hi
        while (hi - lo > 1) {
            const int64_t mid = lo + (hi - lo) / 2;
            const float x = key_float(mid);
            const volatile float d_lo = fabsf(x - lo_level);
            const volatile float d_hi = fabsf(x - hi_level);
            if (d_hi < d_lo) hi = mid; else lo = mid;
        }
        theta[k] = key_float(hi);
    }
    for (int b = 0; b < kBins; ++b) { qb.theta[b] = INFINITY; qb.base[b] = 0; }
    for (int k = 0; k < 15; ++k) {
        const uint32_t b = bin_of(theta[k]);
        if (qb.theta[b] != INFINITY) return false;       // two thresholds in one bin: never for NF4
        qb.theta[b] = theta[k];
        for (uint32_t later = b + 1; later < kBins; ++later) qb.base[later] += 1;
    }
    return true;
}

static const QuantBins* quant_bins() {
    static QuantBins qb;
    static bool ok = false;
    static std::once_flag once;
    std::call_once(once, [] { ok = build_bins(qb); });
    return ok ? &qb : nullptr;
}

// ---- device --------------------------------------------------------------------

typedef float f32x4 __attribute__((ext_vector_type(4)));

// The bins of a caller's codebook, built on the device (the levels live in device memory and the call must not wait
// for the GPU): what build_bins does on the host, by the same bisection with the same FP32 predicate, one threshold
// per lane -- for levels in any order, with repeats (FP4-style tables are in sign-magnitude order and hold +0 and -0):
//   * the distinct values are ranked; a value's code is the lowest index that holds it (the 16-way search keeps the
//     first of equal distances);
//   * between neighbouring values u < u' the search moves to u' where u' is strictly nearer -- or just as near, when
//     the code of u' is the lower of the two --, a predicate that is monotone in x: one threshold per pair;
//   * a bin stores the threshold inside it and the codes on both sides of it (below: the code of the number of
//     thresholds under the bin), so a level index costs the same two table reads as for NF4.
// `usable` = 0 sends the call to the reference kernel: a level that is not finite, neighbouring values closer than
// 2^-10 or than 2^-12 of their magnitude (rounded distances must order like exact ones), a threshold within 2^-30
// of zero (where the tuned kernel's division is not the IEEE one), or two thresholds in one bin of 1/32.
struct DeviceBins {
    QuantBins bins;          // base[b] = code below the bin's threshold | code at and above it << 16
    int usable;
};

__global__ __launch_bounds__(128) void quant_bins_kernel(const float* __restrict__ codebook, DeviceBins* __restrict__ out) {
    __shared__ float level[16];
    __shared__ float uval[16];       // distinct values, ascending
    __shared__ int ucode[17];        // their codes (one more: read, never used, beside the last threshold)
    __shared__ float theta[15];
    __shared__ int bin[15];
    __shared__ int bad, count;
    const int tid = threadIdx.x;
    if (tid < 16) level[tid] = codebook[tid];
    if (tid == 0) bad = 0;
    if (tid < 17) ucode[tid] = 0;
    __syncthreads();
    if (tid < 16) {
        float lv[16];                // the table in registers: the loops below unroll
#pragma unroll
        for (int j = 0; j < 16; ++j) lv[j] = level[j];
        uint32_t first_mask = 0;     // bit j: no lower index holds the value of level j
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            bool first_j = true;
#pragma unroll
            for (int i = 0; i < j; ++i) first_j = first_j && !(lv[i] == lv[j]);
            first_mask |= (first_j ? 1u : 0u) << j;
        }
        const float v = level[tid];
        if (!(__builtin_fabsf(v) < __builtin_inff())) bad = 1;     // (any writer writes the same value)
        int rank = 0;                // distinct values below v
#pragma unroll
        for (int j = 0; j < 16; ++j) rank += ((first_mask >> j) & 1u) && lv[j] < v ? 1 : 0;
        if ((first_mask >> tid) & 1u) {
            uval[rank] = v;
            ucode[rank] = tid;
        }
        if (tid == 0) count = __builtin_popcount(first_mask);
    }
    __syncthreads();
    if (tid < 15) {
        theta[tid] = __builtin_inff();
        bin[tid] = kBins;                                          // in no bin, below none
        if (bad == 0 && tid + 1 < count) {
            const float lo_level = uval[tid], hi_level = uval[tid + 1];
            const float gap = hi_level - lo_level;
            const float mag = __builtin_fmaxf(__builtin_fabsf(lo_level), __builtin_fabsf(hi_level));
            if (!(gap >= 0x1p-10f) || !(gap >= 0x1p-12f * mag)) {
                bad = 1;
            } else {
                const bool ties_go_up = ucode[tid + 1] < ucode[tid];
                // monotone map between FP32 values and integers; the predicate is false at lo, true at hi
                auto key_of = [](float f) {
                    const uint32_t u = __float_as_uint(f);
                    return (u >> 31) ? -(int64_t)(u & 0x7fffffffu) : (int64_t)u;
                };
                auto float_of = [](int64_t k) { return __uint_as_float(k < 0 ? (0x80000000u | (uint32_t)(-k)) : (uint32_t)k); };
                int64_t lo = key_of(lo_level), hi = key_of(hi_level);
                while (hi - lo > 1) {
                    const int64_t mid = lo + (hi - lo) / 2;
                    const float x = float_of(mid);
                    const float d_lo = __builtin_fabsf(x - lo_level);
                    const float d_hi = __builtin_fabsf(x - hi_level);
                    if (ties_go_up ? d_hi <= d_lo : d_hi < d_lo) hi = mid; else lo = mid;
                }
                const float th = float_of(hi);
                theta[tid] = th;
                // (div_by_block_scale is the correctly rounded quotient only down to about 2^-38: no threshold there)
                if (__builtin_fabsf(th) < 0x1p-30f) bad = 1;
                if (th <= -1.0f) {
                    bin[tid] = -1;                                 // reached by every x / absmax: below every bin
                } else if (th <= 1.0f) {
                    const float pos = __builtin_fmaf(th, 32.0f, 32.0f);
                    bin[tid] = pos <= 0.0f ? 0 : (int)(uint32_t)pos;
                }                                                  // else never reached
            }
        }
    }
    __syncthreads();
    if (tid < kBins) {
        int below = 0, inside = 0;
        float th = __builtin_inff();
        for (int k = 0; k < 15; ++k) {
            if (bin[k] < tid) ++below;
            if (bin[k] == tid) { th = theta[k]; ++inside; }
        }
        if (inside > 1) bad = 1;
        out->bins.theta[tid] = th;
        out->bins.base[tid] = (uint32_t)ucode[below] | ((uint32_t)ucode[below + 1] << 16);
    }
    __syncthreads();
    if (tid == 0) out->usable = bad ? 0 : 1;
}

template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
    // every lane has a valid source for these permutations; full masks + bound_ctrl let the
    // compiler fold the move into the max (v_max_f32_dpp)
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true);
    return __builtin_fmaxf(v, __builtin_bit_cast(float, moved));
}

// x / a, correctly rounded, for a block scale a in [2^-64, 2^64] and |x| <= a.
// `r` is the reciprocal of a refined once (shared by the block).  The sequence
// is the textbook one -- quotient estimate, two residual corrections -- i.e.
// the generic IEEE division without its range scaling, which is the identity
// in this range.  Quotients so small that a residual underflows are far below
// the smallest decision threshold (0.0398) and become code 7 either way.
__device__ __forceinline__ float div_by_block_scale(float x, float a, float r) {
    const float q0 = x * r;
    const float e1 = __builtin_fmaf(-a, q0, x);
    const float q1 = __builtin_fmaf(e1, r, q0);
    const float e2 = __builtin_fmaf(-a, q1, x);
    return __builtin_fmaf(e2, r, q1);
}

// Maximum over the lanes that differ in bit 4 (and bit 5) of the lane number: the rows of a wave.
__device__ __forceinline__ float max_across_rows(float a, int lane, bool all_four) {
    const float o = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 16) << 2, __builtin_bit_cast(int, a)));
    a = __builtin_fmaxf(a, o);
    if (all_four) {
        const float p = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, a)));
        a = __builtin_fmaxf(a, p);
    }
    return a;
}

// LOG2BS = log2(blocksize), 6..12: a block is one DPP row of one load (64), two or four rows of one load
// (128, 256), the whole wave over 2, 4 or 8 consecutive loads (512, 1024, 2048), or the two waves of a workgroup
// (4096: each wave reduces its tile, the two maxima meet in LDS).
// A wave whose tile lies wholly inside the tensor takes the unpredicated path; the one tile that does not (Sec. V-A:
// sizes that do not fill a tile) loads element by element with zeros past n -- which neither raise a block's
// maximum nor, as x / absmax = 0, give anything but the zero level's code to the unused nibble of an odd n -- and
// stores only the bytes and scales that exist.
// MEM: the bins come from device memory (quant_bins_kernel built them from the caller's levels) instead of the kernel
// arguments, and the kernel does nothing when that table is marked unusable (the reference kernel then does the work).
template <int LOG2BS, bool MEM>
__global__ __launch_bounds__((LOG2BS == 12 ? 2 : 1) * kWave) void quantize_tiles_kernel(
    const float* __restrict__ src, QuantBins qb, const DeviceBins* __restrict__ dbins, int64_t n,
    uint8_t* __restrict__ packed, float* __restrict__ absmax) {
    constexpr int kWaves = LOG2BS == 12 ? 2 : 1;
    constexpr int kLoadsPerBlock = LOG2BS >= 11 ? 8 : (1 << (LOG2BS > 8 ? LOG2BS - 8 : 0));
    __shared__ float theta_lds[kBins];
    __shared__ uint32_t base_lds[kBins];
    __shared__ float wave_max[2];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if constexpr (MEM) {
        if (dbins->usable == 0) return;                  // the same for every thread of the grid
        theta_lds[lane] = dbins->bins.theta[lane];
        base_lds[lane] = dbins->bins.base[lane];
        if (lane == 0) {
            theta_lds[kBins - 1] = dbins->bins.theta[kBins - 1];
            base_lds[kBins - 1] = dbins->bins.base[kBins - 1];
        }
    } else {
        theta_lds[lane] = qb.theta[lane];                // (both waves of a 4096-block workgroup write the same values)
        base_lds[lane] = qb.base[lane];
        if (lane == 0) {
            theta_lds[kBins - 1] = qb.theta[kBins - 1];
            base_lds[kBins - 1] = qb.base[kBins - 1];
        }
    }
    wave_lds_fence();

    const int64_t t = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t e0 = t * kQTileElems;
    const bool full = e0 + kQTileElems <= n;             // wave-uniform
    f32x4 v[8];
    if (full) {
        const f32x4* in = (const f32x4*)(src + e0);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(in + j * kWave + lane);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t i = e0 + 256 * j + 4 * lane + e;
                v[j][e] = i < n ? src[i] : 0.0f;
            }
    }

    // ---- block maxima.  Lane holds elements 256 j + 4 lane .. + 3 of the tile.
    float a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float m = __builtin_fmaxf(__builtin_fmaxf(fabsf(v[j][0]), fabsf(v[j][1])),
                                  __builtin_fmaxf(fabsf(v[j][2]), fabsf(v[j][3])));
        m = dpp_max<0xB1>(m);      // quad_perm [1,0,3,2]
        m = dpp_max<0x4E>(m);      // quad_perm [2,3,0,1]
        m = dpp_max<0x141>(m);     // row_half_mirror
        m = dpp_max<0x140>(m);     // row_mirror: all 16 lanes of the row hold the maximum of its 64 elements
        a[j] = m;
    }
    if constexpr (LOG2BS > 8) {
#pragma unroll
        for (int j0 = 0; j0 < 8; j0 += kLoadsPerBlock) {
            float m = a[j0];
#pragma unroll
            for (int i = 1; i < kLoadsPerBlock; ++i) m = __builtin_fmaxf(m, a[j0 + i]);
#pragma unroll
            for (int i = 0; i < kLoadsPerBlock; ++i) a[j0 + i] = m;
        }
    }
    if constexpr (LOG2BS >= 7) {
#pragma unroll
        for (int j = 0; j < 8; j += kLoadsPerBlock) {
            const float m = max_across_rows(a[j], lane, LOG2BS >= 8);
#pragma unroll
            for (int i = 0; i < kLoadsPerBlock; ++i) a[j + i] = m;
        }
    }
    if constexpr (LOG2BS == 12) {                        // the block is the workgroup's two tiles
        if (lane == 0) wave_max[wave] = a[0];
        __syncthreads();                                 // both waves always get here: there is no early exit
        const float m = __builtin_fmaxf(wave_max[0], wave_max[1]);
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = m;
    }
#pragma unroll
    for (int j = 0; j < 8; j += kLoadsPerBlock) {
        // first lane of each block writes its scale; block of element e0 + 256 j + 4 lane
        const int first_lane_mask = LOG2BS >= 8 ? 63 : ((1 << (LOG2BS - 2)) - 1);
        const int64_t first = e0 + 256 * j + 4 * lane;
        const bool writer = (lane & first_lane_mask) == 0 && (LOG2BS < 12 || wave == 0);
        if (writer && (full || first < n)) absmax[first >> LOG2BS] = a[j];
    }

    uint16_t* out16 = (uint16_t*)(packed + (e0 >> 1));
    const int64_t nbytes = (n + 1) >> 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float aj = a[j];
        float xn[4];
        if (aj >= 0x1p-64f && aj <= 0x1p+64f) {           // same for all lanes of the block
            const float r0 = __builtin_amdgcn_rcpf(aj);
            const float r = __builtin_fmaf(__builtin_fmaf(-aj, r0, 1.0f), r0, r0);
#pragma unroll
            for (int e = 0; e < 4; ++e) xn[e] = div_by_block_scale(v[j][e], aj, r);
        } else {
            const float div = aj == 0.0f ? 1.0f : aj;     // all-zero block: 0 / 1 = 0 -> code 7
#pragma unroll
            for (int e = 0; e < 4; ++e) xn[e] = v[j][e] / div;   // generic IEEE division
        }
        uint32_t code[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t b = (uint32_t)__builtin_fmaf(xn[e], 32.0f, 32.0f);   // 0..64; NaN -> 0
            if constexpr (MEM) {
                const uint32_t both = base_lds[b];                 // the codes below and from the bin's threshold on
                const uint32_t c = xn[e] >= theta_lds[b] ? both >> 16 : both & 0xffffu;
                code[e] = xn[e] == xn[e] ? c : 0u;                 // NaN: every distance is NaN, the search keeps code 0
            } else {
                code[e] = base_lds[b] + (xn[e] >= theta_lds[b] ? 1u : 0u);
            }
        }
        // element 2i in the high nibble of byte i; two bytes per lane, little-endian
        const uint32_t two_bytes = (code[0] << 4) | code[1] | (code[2] << 12) | (code[3] << 8);
        if (full) {
            __builtin_nontemporal_store((uint16_t)two_bytes, out16 + j * 64 + lane);   // bytes 128 j + 2 lane
        } else {
            const int64_t byte0 = (e0 >> 1) + 128 * j + 2 * lane;
            if (byte0 + 1 < nbytes) out16[j * 64 + lane] = (uint16_t)two_bytes;
            else if (byte0 < nbytes) packed[byte0] = (uint8_t)two_bytes;
        }
    }
}

// `dbins` = nullptr: the NF4 bins in `qb` (kernel arguments); otherwise the bins in device memory.
template <int LOG2BS>
static int launch_tiles(const float* src, const QuantBins& qb, const DeviceBins* dbins, int64_t n, uint8_t* packed,
                        float* absmax, hipStream_t s) {
    constexpr int kWaves = LOG2BS == 12 ? 2 : 1;
    const int64_t per_group = (int64_t)kWaves * kQTileElems;
    const int64_t groups = (n + per_group - 1) / per_group;
    if (groups > 0x7fffffffLL) return NF4_ERR_SIZE;
    if (dbins)
        hipLaunchKernelGGL((quantize_tiles_kernel<LOG2BS, true>), dim3((unsigned)groups), dim3(kWaves * kWave), 0, s, src,
                           qb, dbins, n, packed, absmax);
    else
        hipLaunchKernelGGL((quantize_tiles_kernel<LOG2BS, false>), dim3((unsigned)groups), dim3(kWaves * kWave), 0, s, src,
                           qb, dbins, n, packed, absmax);
    return record_hip(hipGetLastError());
}

static int launch_tiles_any(int log2_bs, const float* src, const QuantBins& qb, const DeviceBins* dbins, int64_t n,
                            uint8_t* packed, float* absmax, hipStream_t s) {
    switch (log2_bs) {
        case 6: return launch_tiles<6>(src, qb, dbins, n, packed, absmax, s);
        case 7: return launch_tiles<7>(src, qb, dbins, n, packed, absmax, s);
        case 8: return launch_tiles<8>(src, qb, dbins, n, packed, absmax, s);
        case 9: return launch_tiles<9>(src, qb, dbins, n, packed, absmax, s);
        case 10: return launch_tiles<10>(src, qb, dbins, n, packed, absmax, s);
        case 11: return launch_tiles<11>(src, qb, dbins, n, packed, absmax, s);
        default: return launch_tiles<12>(src, qb, dbins, n, packed, absmax, s);
    }
}

// the reference kernel (nf4_quantize_ref.hip) finishes what does not fill a tile
// (`skip_if` != nullptr: the kernel does nothing when *skip_if is not 0)
int launch_quantize_ref_range(const float* src, int64_t n, int blocksize, const float* codebook, const int* skip_if,
                              uint8_t* packed, float* absmax, hipStream_t s);

}  // namespace nf4

extern "C" int nf4_quantize(const float* src, int64_t n, int blocksize, uint8_t* packed, float* absmax,
                            void* stream) {
    using namespace nf4;
    if (n < 0) return NF4_ERR_SIZE;
    if (log2_blocksize(blocksize) < 0) return NF4_ERR_BLOCKSIZE;
    if (n == 0) return NF4_OK;
    if (!src || !packed || !absmax) return NF4_ERR_NULL;
    if (!aligned(src, 16) || !aligned(absmax, 4) || !aligned(packed, 2)) return NF4_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    const QuantBins* qb = quant_bins();
    const int log2_bs = log2_blocksize(blocksize);
    if (qb == nullptr) return launch_quantize_ref_range(src, n, blocksize, nullptr, nullptr, packed, absmax, s);
    return launch_tiles_any(log2_bs, src, *qb, nullptr, n, packed, absmax, s);
}

extern "C" int nf4_quantize_codebook(const float* src, int64_t n, int blocksize, const float* codebook, uint8_t* packed,
                                     float* absmax, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace nf4;
    static_assert(sizeof(DeviceBins) <= NF4_QUANTIZE_CODEBOOK_WORKSPACE_BYTES, "workspace of nf4_quantize_codebook");
    if (codebook == nullptr) return nf4_quantize(src, n, blocksize, packed, absmax, stream);
    if (n < 0) return NF4_ERR_SIZE;
    const int log2_bs = log2_blocksize(blocksize);
    if (log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (n == 0) return NF4_OK;
    if (!src || !packed || !absmax || !workspace) return NF4_ERR_NULL;
    if (!aligned(src, 16) || !aligned(absmax, 4) || !aligned(packed, 2) || !aligned(codebook, 4) || !aligned(workspace, 8))
        return NF4_ERR_ALIGN;
    if (workspace_bytes < NF4_QUANTIZE_CODEBOOK_WORKSPACE_BYTES) return NF4_ERR_SIZE;
    hipStream_t s = (hipStream_t)stream;
    DeviceBins* dbins = (DeviceBins*)workspace;
    hipLaunchKernelGGL(quant_bins_kernel, dim3(1), dim3(128), 0, s, codebook, dbins);
    int rc = record_hip(hipGetLastError());
    if (rc != NF4_OK) return rc;
    // one of the two does the work: the tiles kernel when the table is usable, the reference kernel when it is not
    static const QuantBins unused = {};
    rc = launch_tiles_any(log2_bs, src, unused, dbins, n, packed, absmax, s);
    if (rc != NF4_OK) return rc;
    return launch_quantize_ref_range(src, n, blocksize, codebook, &dbins->usable, packed, absmax, s);
}
