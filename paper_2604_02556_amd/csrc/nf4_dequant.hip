// Blockwise NF4 -> FP16/BF16 dequantisation for gfx950 (Algorithm 1 of the
// paper, re-designed for CDNA4).
//
// What the paper's kernel does on Ampere -- 64 threads x 8 elements, thread 0
// staging the 16 levels into shared memory (Sec. IV-B, IV-F) -- is not kept.
// Here the path is bound by HBM, 78 % of the traffic is the 16-bit output, and
// the design follows from that:
//   * a wave reads 1 KiB of codes with one 128-bit load per lane (2048
//     elements), contiguous across the wave;
//   * the codes cross lanes through 1 KiB of LDS so that every store
//     instruction of the wave writes 1 KiB of contiguous output (lane l writes
//     16 bytes at 16*l): four such stores per tile, each covering whole cache
//     lines, instead of 64-byte-strided fragments;
//   * the 16 levels sit in LDS; 16 consecutive dwords occupy 16 distinct banks
//     and lanes that pick the same level are served by broadcast, so the lookup
//     is conflict-free by construction;
//   * nibble split is a shift and a mask (Sec. IV-D), the product is one FP32
//     multiply, two products are narrowed and packed per dword, eight per
//     128-bit store;
//   * whatever does not fill a 2048-element wave tile (Sec. V-A: ragged sizes)
//     goes through a predicated byte-at-a-time tail in the last workgroup, so
//     the bulk loop carries no bounds checks.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kTileBytes = kWave * 16;     // codes per wave tile
constexpr int kTileElems = kTileBytes * 2; // 2048

struct ScaleArgs {
    const float* absmax;     // single level
    const uint8_t* q8;       // double quantisation
    const float* scale2;
    const float* offset;
    const float* code2;
};

// Order LDS traffic within one wave: the hardware serves a wave's LDS
// instructions in issue order, so only the compiler must be kept from moving
// accesses across this point.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool DQ>
__device__ __forceinline__ float block_scale(const ScaleArgs& a, const float* code2_lds, float offset,
                                             int64_t blk) {
    if constexpr (DQ) {
        float prod = code2_lds[a.q8[blk]] * a.scale2[blk >> 8];   // rounded product ...
        return prod + offset;                                     // ... then rounded sum (never an FMA)
    } else {
        return a.absmax[blk];
    }
}

// Eight codes of one dword -> eight scaled 16-bit values.  Byte j of the dword
// holds element 2j in its high nibble and element 2j+1 in its low nibble.
template <int DT>
__device__ __forceinline__ u32x4 expand8(uint32_t q, float s, const float* lut) {
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float hi = lut[(q >> (8 * j + 4)) & 15u] * s;
        float lo = lut[(q >> (8 * j)) & 15u] * s;
        r[j] = pack2<DT>(hi, lo);
    }
    return r;
}

template <int DT, bool DQ>
__global__ __launch_bounds__(kThreads) void dequant_kernel(const uint8_t* __restrict__ packed,
                                                           ScaleArgs sa, int log2_bs, int64_t n,
                                                           int64_t wave_tiles,
                                                           uint16_t* __restrict__ out) {
    __shared__ float lut[16];
    __shared__ float code2_lds[DQ ? 256 : 1];
    __shared__ uint32_t stage[kWaves][kTileBytes / 4];

    if (threadIdx.x < 16) lut[threadIdx.x] = __uint_as_float(kLevelBits[threadIdx.x]);
    if constexpr (DQ) code2_lds[threadIdx.x] = sa.code2[threadIdx.x];
    __syncthreads();
    const float offset = DQ ? sa.offset[0] : 0.0f;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t stride = (int64_t)gridDim.x * kWaves;
    int64_t t = (int64_t)blockIdx.x * kWaves + wave;

    u32x4 cur = {0, 0, 0, 0};
    if (t < wave_tiles) cur = *(const u32x4*)(packed + t * kTileBytes + lane * 16);
    while (t < wave_tiles) {
        const int64_t t_next = t + stride;
        u32x4 nxt = {0, 0, 0, 0};
        if (t_next < wave_tiles) nxt = *(const u32x4*)(packed + t_next * kTileBytes + lane * 16);

        *(u32x4*)&stage[wave][lane * 4] = cur;
        wave_lds_fence();
        const int64_t e0 = t * kTileElems;
        uint16_t* out_tile = out + e0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t q = stage[wave][64 * k + lane];
            const int e = 512 * k + 8 * lane;               // element offset inside the tile
            const float s = block_scale<DQ>(sa, code2_lds, offset, (e0 + e) >> log2_bs);
            const u32x4 v = expand8<DT>(q, s, lut);
            *(u32x4*)(out_tile + e) = v;
        }
        wave_lds_fence();
        cur = nxt;
        t = t_next;
    }

    // Ragged end: everything after the last full wave tile, one byte (two
    // elements of the same block) per thread, every access predicated on n.
    if (blockIdx.x == gridDim.x - 1) {
        const int64_t nbytes = (n + 1) >> 1;
        for (int64_t b = wave_tiles * kTileBytes + threadIdx.x; b < nbytes; b += kThreads) {
            const uint32_t q = packed[b];
            const int64_t i = 2 * b;
            const float s = block_scale<DQ>(sa, code2_lds, offset, i >> log2_bs);
            out[i] = narrow1<DT>(lut[q >> 4] * s);
            if (i + 1 < n) out[i + 1] = narrow1<DT>(lut[q & 15u] * s);
        }
    }
}

template <bool DQ>
static int launch(const uint8_t* packed, const ScaleArgs& sa, int blocksize, int64_t n, void* out,
                  int out_dtype, void* stream) {
    if (n < 0) return NF4_ERR_SIZE;
    const int log2_bs = log2_blocksize(blocksize);
    if (log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (out_dtype != NF4_FP16 && out_dtype != NF4_BF16) return NF4_ERR_DTYPE;
    if (n == 0) return NF4_OK;
    if (!packed || !out) return NF4_ERR_NULL;
    if constexpr (DQ) {
        if (!sa.q8 || !sa.scale2 || !sa.offset || !sa.code2) return NF4_ERR_NULL;
        if (!aligned(sa.scale2, 4) || !aligned(sa.offset, 4) || !aligned(sa.code2, 4)) return NF4_ERR_ALIGN;
    } else {
        if (!sa.absmax) return NF4_ERR_NULL;
        if (!aligned(sa.absmax, 4)) return NF4_ERR_ALIGN;
    }
    if (!aligned(packed, 16) || !aligned(out, 16)) return NF4_ERR_ALIGN;

    const int64_t wave_tiles = n / kTileElems;
    const int64_t group_tiles = (wave_tiles + kWaves - 1) / kWaves;
    const int64_t cap = (int64_t)compute_units() * 8;
    int64_t groups = group_tiles < cap ? group_tiles : cap;
    if (groups < 1) groups = 1;

    hipStream_t s = (hipStream_t)stream;
    uint16_t* o = (uint16_t*)out;
    dim3 grid((unsigned)groups), block(kThreads);
    if (out_dtype == NF4_FP16)
        hipLaunchKernelGGL((dequant_kernel<NF4_FP16, DQ>), grid, block, 0, s, packed, sa, log2_bs, n, wave_tiles, o);
    else
        hipLaunchKernelGGL((dequant_kernel<NF4_BF16, DQ>), grid, block, 0, s, packed, sa, log2_bs, n, wave_tiles, o);
    return record_hip(hipGetLastError());
}

}  // namespace nf4

extern "C" int nf4_dequantize(const uint8_t* packed, const float* absmax, int blocksize, int64_t n,
                              void* out, int out_dtype, void* stream) {
    nf4::ScaleArgs sa = {absmax, nullptr, nullptr, nullptr, nullptr};
    return nf4::launch<false>(packed, sa, blocksize, n, out, out_dtype, stream);
}

extern "C" int nf4_dequantize_dq(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                 const float* offset, const float* code2, int blocksize, int64_t n,
                                 void* out, int out_dtype, void* stream) {
    nf4::ScaleArgs sa = {nullptr, absmax_q8, scale2, offset, code2};
    return nf4::launch<true>(packed, sa, blocksize, n, out, out_dtype, stream);
}
