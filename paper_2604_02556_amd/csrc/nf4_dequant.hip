// Blockwise NF4 -> FP16/BF16 dequantisation for gfx950 (Algorithm 1 of the
// paper, re-designed for CDNA4).
//
// What the paper's kernel does on Ampere -- 64 threads x 8 elements, thread 0
// staging the 16 levels into shared memory behind a barrier (Sec. IV-B, IV-F)
// -- is not kept.  On MI355X the path is bound by HBM, 78 % of the traffic is
// the 16-bit output, and the design follows from measurements of that:
//   * one wave = one tile of 2048 elements: 1 KiB of codes read with a single
//     128-bit load per lane, contiguous across the wave;
//   * the codes cross lanes through 1 KiB of LDS so that every store
//     instruction of the wave writes 1 KiB of contiguous output (lane l writes
//     the 16 bytes at 16*l): four such stores per tile, each covering whole
//     cache lines.  Letting each lane store the 64 bytes it decoded itself
//     (16-byte pieces at a 64-byte stride) ran at under half the speed;
//   * the tile's block scales are fetched with one contiguous load by the
//     first 32 lanes (block size 64) and handed to the other lanes with
//     ds_bpermute.  Loading them where they are used -- four loads per lane in
//     which eight lanes share an address -- moves the same bytes with four
//     times the requests and cost 2.4 % of the stream's throughput;
//   * stores carry the non-temporal hint (+6 % measured): the output is
//     written once and not re-read by this kernel;
//   * the grid is one-shot -- one single-wave workgroup per tile, dispatched in
//     address order -- rather than a persistent grid-stride loop: in-order
//     dispatch keeps the write frontier compact and measured 15-20 % faster
//     than 2048 resident workgroups striding through the tensor;
//   * the 16 levels sit in 64 bytes of LDS, written once per wave by lanes
//     0..15 from instruction literals (no memory read, and with single-wave
//     workgroups no barrier).  16 consecutive dwords fall in 16 distinct banks
//     and lanes that pick the same level are served by broadcast, so the
//     lookup cannot conflict (SQ_LDS_BANK_CONFLICT = 0).  Measured against a
//     VGPR table read with ds_bpermute_b32, a 256-entry byte-pair LDS table, a
//     table re-read from memory and a pure select chain: the LDS tables are
//     equal within 0.5 % (the path is HBM-bound), ds_bpermute is 3 % slower
//     (it keeps the LDS pipe busy for almost twice as many cycles), the
//     byte-pair table conflicts, and the last two halve the throughput.  The
//     table is written before the wave issues its loads: the other order
//     measured 1.2 % slower;
//   * nibble split is a shift and a mask (Sec. IV-D), the product is one FP32
//     multiply, two products are narrowed and packed per dword by the packed
//     round-to-nearest-even converts, eight values per 128-bit store;
//   * whatever does not fill a tile (Sec. V-A: ragged sizes) is handled by one
//     extra workgroup, a byte (two elements) per lane, every access predicated
//     on n, so the bulk path carries no bounds checks.
//   * the size of the output picks the cache policy of the stores and the order
//     of the two loads (OutClass below), measured on the 70B-shaped stream, in which
//     every tensor is written into the same reused buffer:
//       - up to 40 MB of output (it fits the eight 4 MB L2s with room to spare):
//         non-temporal stores, codes requested before the scales;
//       - up to 240 MB (it fits the 256 MB memory-side cache): stores at agent
//         scope without the non-temporal hint (`sc1`).  The output then stays in
//         that cache, where the next tensor overwrites it and a consumer would find
//         it: 26.1 instead of 28.4 us for 8192 x 8192;
//       - above that: `sc1 nt`, and the wave asks for its codes only once its
//         scales have arrived.  One vector load in flight per wave instead of two
//         is worth 2.4 % there (91.2 instead of 93.4 us for 8192 x 28672), but only
//         together with that store policy; with plain non-temporal stores it is
//         worth nothing, and on the smaller classes it costs 1-2 %;
//   * the kernel's arguments are plain scalars with the ones a wave needs first in
//     front, so that they arrive in the wave's initial scalar registers (kernel-
//     argument preloading, -amdgpu-kernarg-preload-count) instead of through a
//     scalar load that every wave of a launch waits for: 0.25 us per launch.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

constexpr int kTileBytes = kWave * 16;     // codes per wave tile
constexpr int kTileElems = kTileBytes * 2; // 2048

struct ScaleArgs {
    const float* absmax;     // single level
    const uint8_t* q8;       // double quantisation
    const float* scale2;
    const float* offset;
    const float* code2;
    int log2_group;          // blocks per second-level scale (8 = the format's 256)
    const float* codebook;   // 16 levels in memory, or nullptr for the NF4 literals
};

// Memory policy by size of the output (see the head of this file).
enum OutClass { kOutSmall = 0, kOutCached = 1, kOutStream = 2 };
constexpr int64_t kCachedMinBytes = int64_t(40) << 20;    // beyond the L2s
constexpr int64_t kCachedMaxBytes = int64_t(240) << 20;   // inside the 256 MB memory-side cache
inline OutClass out_class(int64_t n) {
    const int64_t bytes = 2 * n;
    return bytes < kCachedMinBytes ? kOutSmall : bytes <= kCachedMaxBytes ? kOutCached : kOutStream;
}

// 16 bytes to p with the class's cache policy.  The agent-scope forms have no C spelling; the s_nop covers the
// one wait state a store of more than 8 bytes needs before its data registers may be overwritten, which the
// compiler cannot see to insert after an asm statement.
template <int CLS>
__device__ __forceinline__ void store16(u32x4 v, u32x4* p) {
    if constexpr (CLS == kOutSmall) __builtin_nontemporal_store(v, p);
    else if constexpr (CLS == kOutCached)
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 0" ::"v"(p), "v"(v) : "memory");
    else
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 0" ::"v"(p), "v"(v) : "memory");
}

// Eight codes of one dword -> eight scaled 16-bit values.  Byte j of the dword
// holds element 2j in its high nibble and element 2j+1 in its low nibble.
template <int DT>
__device__ __forceinline__ u32x4 expand8(uint32_t q, float s, const float* lut) {
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float hi = lut[(q >> (8 * j + 4)) & 15u] * s;
        const float lo = lut[(q >> (8 * j)) & 15u] * s;
        r[j] = pack2<DT>(hi, lo);
    }
    return r;
}

// Double-quantised scale of block `blk`: a rounded product, then a rounded sum
// (never an FMA).
__device__ __forceinline__ float dq_scale(const ScaleArgs& a, float offset, int64_t blk) {
    const float prod = a.code2[a.q8[blk]] * a.scale2[blk >> a.log2_group];
    return prod + offset;
}

// The work of one single-wave workgroup: tile `t` of a tensor with `tiles` full tiles, or (t == tiles) its
// ragged end.  stage (1 KiB) and lut (16 levels) are the workgroup's LDS.
template <int DT, bool DQ, int CLS>
__device__ __forceinline__ void dequant_group(const uint8_t* __restrict__ packed, const ScaleArgs& sa, int log2_bs,
                                              int64_t n, int64_t tiles, uint16_t* __restrict__ out, int64_t t,
                                              uint32_t* stage, float* lut) {
    const int lane = threadIdx.x;
    const float offset = DQ ? sa.offset[0] : 0.0f;
    // the table: instruction literals for NF4, 64 bytes from memory for a caller's codebook (Sec. V-A: the
    // data type is a parameter); either way ordered by the fence below
    if (lane < 16) lut[lane] = sa.codebook ? sa.codebook[lane] : __uint_as_float(level_literal(lane));

    if (t < tiles) {
        const int64_t e0 = t * kTileElems;
        const uint8_t* tile_codes = packed + t * kTileBytes;
        uint32_t code_off = (uint32_t)lane * 16u;
        u32x4 codes;
        // Scales.  Lane l's k-th store covers elements e0 + 512 k + 8 l .. + 7,
        // all inside one quantisation block (blocksize >= 64).
        float s[4];
        {
            // lanes 0..(blocks per tile - 1) each fetch (FP32 absmax) or rebuild (double quantisation) one block
            // scale with a single contiguous load; the others take it across lanes afterwards
            const int per_tile = log2_bs >= 11 ? 1 : (kTileElems >> log2_bs);
            const int64_t b0 = e0 >> log2_bs;
            float mine = 0.0f;
            if constexpr (DQ) {
                // One round trip to memory: the 8-bit code, the second-level scale, the whole 1 KiB code2 map (one
                // coalesced load, always a cache hit) and the codes are requested together; the map goes through
                // the exchange buffer, which is free until the codes arrive, and the dependent lookup is an LDS read.
                // (Reading code2[q] from memory once q had arrived made it two round trips: Gemma-27B leg 158 -> 155.5 us
                // per layer; the straightforward order, three: 161.)  For the largest tensors the codes wait for the
                // scale codes, as in the FP32-scale form.  Lanes past the tile's blocks repeat its first block: no
                // predicated loads, whose results the compiler would have to wait for at the end of the predicated region.
                const int64_t blk = b0 + (lane < per_tile ? lane : 0);
                const uint32_t q = sa.q8[blk];
                const float s2 = sa.scale2[blk >> sa.log2_group];
                const u32x4 map = *(const u32x4*)(sa.code2 + 4 * lane);
                if constexpr (CLS == kOutStream) asm volatile("" : "+v"(code_off) : "v"(q), "v"(s2));
                codes = *(const u32x4*)(tile_codes + code_off);
                *(u32x4*)&stage[4 * lane] = map;
                wave_lds_fence();
                const float prod = ((const float*)stage)[q] * s2;  // a rounded product, then a rounded sum (never an FMA)
                wave_lds_fence();                                  // read before the codes overwrite the buffer
                mine = prod + offset;
            } else {
                if constexpr (CLS == kOutSmall) codes = *(const u32x4*)(tile_codes + code_off);
                if (lane < per_tile) mine = sa.absmax[b0 + lane];
                // the largest tensors: the address of the codes is made to depend on the scale, so that the wave
                // requests its codes only when its scales are there
                if constexpr (CLS == kOutStream) asm volatile("" : "+v"(code_off) : "v"(mine));
                if constexpr (CLS != kOutSmall) codes = *(const u32x4*)(tile_codes + code_off);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int src = log2_bs >= 11 ? 0 : ((512 * k + 8 * lane) >> log2_bs);
                s[k] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, mine)));
            }
        }

        *(u32x4*)&stage[lane * 4] = codes;
        wave_lds_fence();
        uint16_t* out_tile = out + e0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t q = stage[64 * k + lane];
            const u32x4 v = expand8<DT>(q, s[k], lut);
            store16<CLS>(v, (u32x4*)(out_tile + 512 * k + 8 * lane));
        }
    } else {
        // Ragged end: everything after the last full tile, one byte (two
        // elements of the same block) per lane, every access predicated on n.
        wave_lds_fence();
        const int64_t nbytes = (n + 1) >> 1;
        for (int64_t base = tiles * kTileBytes; base < nbytes; base += kWave) {
            const int64_t b = base + lane;
            const int64_t i = 2 * b;
            const bool live = b < nbytes;
            uint32_t q = 0;
            float sc = 0.0f;
            if (live) {
                q = packed[b];
                sc = DQ ? dq_scale(sa, offset, i >> log2_bs) : sa.absmax[i >> log2_bs];
            }
            const float hi = lut[q >> 4] * sc;
            const float lo = lut[q & 15u] * sc;
            if (live) {
                out[i] = narrow1<DT>(hi);
                if (i + 1 < n) out[i + 1] = narrow1<DT>(lo);
            }
        }
    }
}

// The arguments are plain scalars, the ones a wave needs first in front, so that they travel in the wave's
// initial scalar registers (kernel-argument preloading) instead of being fetched from memory by every wave before
// it can issue its first load: packed, the scale pointers, out, tiles and the shifts are 13 or 14 dwords.  `n`
// (only the ragged end reads it) and the caller's codebook (only read when `shifts` says there is one) come last.
// shifts = log2(blocksize) | log2(blocks per second-level scale) << 8 | (codebook != nullptr) << 16.
template <int DT, int CLS>
__global__ __launch_bounds__(kWave) void dequant_kernel(const uint8_t* __restrict__ packed,
                                                        const float* __restrict__ absmax,
                                                        uint16_t* __restrict__ out, int tiles, int shifts, int64_t n,
                                                        const float* __restrict__ codebook) {
    __shared__ uint32_t stage[kTileBytes / 4];
    __shared__ float lut[16];
    const ScaleArgs sa = {absmax, nullptr, nullptr, nullptr, nullptr, 8, (shifts >> 16) ? codebook : nullptr};
    dequant_group<DT, false, CLS>(packed, sa, shifts & 0xff, n, tiles, out, blockIdx.x, stage, lut);
}

template <int DT, int CLS>
__global__ __launch_bounds__(kWave) void dequant_dq_kernel(const uint8_t* __restrict__ packed,
                                                           const uint8_t* __restrict__ q8,
                                                           const float* __restrict__ scale2,
                                                           const float* __restrict__ code2,
                                                           const float* __restrict__ offset,
                                                           uint16_t* __restrict__ out, int tiles, int shifts,
                                                           int64_t n, const float* __restrict__ codebook) {
    __shared__ uint32_t stage[kTileBytes / 4];
    __shared__ float lut[16];
    const ScaleArgs sa = {nullptr, q8, scale2, offset, code2, (shifts >> 8) & 0xff, (shifts >> 16) ? codebook : nullptr};
    dequant_group<DT, true, CLS>(packed, sa, shifts & 0xff, n, tiles, out, blockIdx.x, stage, lut);
}

// Several tensors in one launch: workgroup g belongs to the tensor i with first_group[i] <= g <
// first_group[i + 1], in the order given, so the write frontier still moves through one tensor after the other.
// One launch pays the fill and drain of the load -> store pipeline once instead of once per tensor, which matters
// for tensors of a few MB (a kernel that lasts a single generation of waves) and not for large ones.
struct BatchArgs {
    const uint8_t* packed[NF4_BATCH_MAX];
    const float* absmax[NF4_BATCH_MAX];
    const uint8_t* q8[NF4_BATCH_MAX];
    const float* scale2[NF4_BATCH_MAX];
    const float* offset[NF4_BATCH_MAX];
    const float* code2[NF4_BATCH_MAX];
    uint16_t* out[NF4_BATCH_MAX];
    int64_t n[NF4_BATCH_MAX];
    int64_t tiles[NF4_BATCH_MAX];
    int64_t first_group[NF4_BATCH_MAX + 1];
    int count;
};

// The memory policy goes by the output of the whole launch (the tensors of a call are written side by side).
template <int DT, bool DQ, int CLS>
__global__ __launch_bounds__(kWave) void dequant_batch_kernel(BatchArgs ba, int log2_bs) {
    const int64_t g = blockIdx.x;
    int i = 0;
#pragma unroll
    for (int k = 1; k < NF4_BATCH_MAX; ++k)
        if (k < ba.count && g >= ba.first_group[k]) i = k;             // wave-uniform
    // select by comparison rather than by indexing, so that the argument arrays stay in scalar registers
    const uint8_t* packed = ba.packed[0];
    ScaleArgs sa = {ba.absmax[0], ba.q8[0], ba.scale2[0], ba.offset[0], ba.code2[0], 8, nullptr};
    uint16_t* out = ba.out[0];
    int64_t n = ba.n[0], tiles = ba.tiles[0], first = ba.first_group[0];
#pragma unroll
    for (int k = 1; k < NF4_BATCH_MAX; ++k)
        if (i == k) {
            packed = ba.packed[k];
            sa.absmax = ba.absmax[k]; sa.q8 = ba.q8[k]; sa.scale2 = ba.scale2[k]; sa.offset = ba.offset[k];
            sa.code2 = ba.code2[k];
            out = ba.out[k];
            n = ba.n[k]; tiles = ba.tiles[k]; first = ba.first_group[k];
        }
    __shared__ uint32_t stage[kTileBytes / 4];
    __shared__ float lut[16];
    dequant_group<DT, DQ, CLS>(packed, sa, log2_bs, n, tiles, out, g - first, stage, lut);
}

template <bool DQ>
static int launch(const uint8_t* packed, const ScaleArgs& sa, int blocksize, int64_t n, void* out,
                  int out_dtype, void* stream) {
    if (n < 0) return NF4_ERR_SIZE;
    if (sa.codebook && !aligned(sa.codebook, 4)) return NF4_ERR_ALIGN;
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

    const int64_t tiles = n / kTileElems;
    const int64_t groups = tiles + (n % kTileElems != 0 ? 1 : 0);
    if (groups > 0x7fffffffLL) return NF4_ERR_SIZE;              // 4.4e12 elements

    hipStream_t s = (hipStream_t)stream;
    uint16_t* o = (uint16_t*)out;
    dim3 grid((unsigned)groups), block(kWave);
    const int shifts = log2_bs | (sa.log2_group << 8) | (sa.codebook ? 1 << 16 : 0);
    const int t32 = (int)tiles;                                  // tiles <= groups < 2^31
#define NF4_LAUNCH_DEQUANT(DT, CLS)                                                                              \
    do {                                                                                                        \
        if constexpr (DQ)                                                                                       \
            hipLaunchKernelGGL((dequant_dq_kernel<DT, CLS>), grid, block, 0, s, packed, sa.q8, sa.scale2,       \
                               sa.code2, sa.offset, o, t32, shifts, n, sa.codebook);                            \
        else                                                                                                    \
            hipLaunchKernelGGL((dequant_kernel<DT, CLS>), grid, block, 0, s, packed, sa.absmax, o, t32, shifts, \
                               n, sa.codebook);                                                                 \
    } while (0)
    const OutClass cls = out_class(n);
    if (out_dtype == NF4_FP16) {
        if (cls == kOutSmall) NF4_LAUNCH_DEQUANT(NF4_FP16, kOutSmall);
        else if (cls == kOutCached) NF4_LAUNCH_DEQUANT(NF4_FP16, kOutCached);
        else NF4_LAUNCH_DEQUANT(NF4_FP16, kOutStream);
    } else {
        if (cls == kOutSmall) NF4_LAUNCH_DEQUANT(NF4_BF16, kOutSmall);
        else if (cls == kOutCached) NF4_LAUNCH_DEQUANT(NF4_BF16, kOutCached);
        else NF4_LAUNCH_DEQUANT(NF4_BF16, kOutStream);
    }
#undef NF4_LAUNCH_DEQUANT
    return record_hip(hipGetLastError());
}

}  // namespace nf4

extern "C" int nf4_dequantize(const uint8_t* packed, const float* absmax, int blocksize, int64_t n,
                              void* out, int out_dtype, void* stream) {
    nf4::ScaleArgs sa = {absmax, nullptr, nullptr, nullptr, nullptr, 8, nullptr};
    return nf4::launch<false>(packed, sa, blocksize, n, out, out_dtype, stream);
}

extern "C" int nf4_dequantize_codebook(const uint8_t* packed, const float* absmax, const float* codebook,
                                       int blocksize, int64_t n, void* out, int out_dtype, void* stream) {
    nf4::ScaleArgs sa = {absmax, nullptr, nullptr, nullptr, nullptr, 8, codebook};
    return nf4::launch<false>(packed, sa, blocksize, n, out, out_dtype, stream);
}

extern "C" int nf4_dequantize_dq(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                 const float* offset, const float* code2, int blocksize, int64_t n,
                                 void* out, int out_dtype, void* stream) {
    nf4::ScaleArgs sa = {nullptr, absmax_q8, scale2, offset, code2, 8, nullptr};
    return nf4::launch<true>(packed, sa, blocksize, n, out, out_dtype, stream);
}

extern "C" int nf4_dequantize_dq_codebook(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                          const float* offset, const float* code2, int dq_group,
                                          const float* codebook, int blocksize, int64_t n, void* out,
                                          int out_dtype, void* stream) {
    const int log2_group = nf4::log2_dq_group(dq_group);
    if (log2_group < 0) return NF4_ERR_SHAPE;
    nf4::ScaleArgs sa = {nullptr, absmax_q8, scale2, offset, code2, log2_group, codebook};
    return nf4::launch<true>(packed, sa, blocksize, n, out, out_dtype, stream);
}

extern "C" int nf4_dequantize_batch(const nf4_tensor* tensors, int count, int blocksize, int out_dtype,
                                    void* stream) {
    using namespace nf4;
    if (count < 0 || count > NF4_BATCH_MAX) return NF4_ERR_SIZE;
    const int log2_bs = log2_blocksize(blocksize);
    if (log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (out_dtype != NF4_FP16 && out_dtype != NF4_BF16) return NF4_ERR_DTYPE;
    if (count == 0) return NF4_OK;
    if (!tensors) return NF4_ERR_NULL;
    BatchArgs ba = {};
    int64_t groups = 0;
    bool dq = false, kind_known = false;
    for (int i = 0; i < count; ++i) {
        const nf4_tensor& t = tensors[i];
        if (t.n < 0) return NF4_ERR_SIZE;
        if (t.n == 0) continue;                              // an empty tensor takes no part
        if (!t.packed || !t.out) return NF4_ERR_NULL;
        const bool this_dq = t.absmax == nullptr;
        if (this_dq) {
            if (!t.absmax_q8 || !t.scale2 || !t.offset || !t.code2) return NF4_ERR_NULL;
            if (!aligned(t.scale2, 4) || !aligned(t.offset, 4) || !aligned(t.code2, 4)) return NF4_ERR_ALIGN;
        } else if (!aligned(t.absmax, 4)) {
            return NF4_ERR_ALIGN;
        }
        if (!aligned(t.packed, 16) || !aligned(t.out, 16)) return NF4_ERR_ALIGN;
        if (kind_known && this_dq != dq) return NF4_ERR_SHAPE;       // one kind of scales per call
        dq = this_dq;
        kind_known = true;
        const int k = ba.count++;
        ba.packed[k] = t.packed; ba.absmax[k] = t.absmax; ba.q8[k] = t.absmax_q8; ba.scale2[k] = t.scale2;
        ba.offset[k] = t.offset; ba.code2[k] = t.code2; ba.out[k] = (uint16_t*)t.out;
        ba.n[k] = t.n;
        ba.tiles[k] = t.n / kTileElems;
        ba.first_group[k] = groups;
        groups += ba.tiles[k] + (t.n % kTileElems != 0 ? 1 : 0);
        ba.first_group[k + 1] = groups;
    }
    if (ba.count == 0) return NF4_OK;
    if (groups > 0x7fffffffLL) return NF4_ERR_SIZE;
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid((unsigned)groups), block(kWave);
    int64_t total = 0;
    for (int k = 0; k < ba.count; ++k) total += ba.n[k];
#define NF4_LAUNCH_BATCH(CLS)                                                                                     \
    do {                                                                                                         \
        if (out_dtype == NF4_FP16) {                                                                             \
            if (dq) hipLaunchKernelGGL((dequant_batch_kernel<NF4_FP16, true, CLS>), grid, block, 0, s, ba, log2_bs);  \
            else hipLaunchKernelGGL((dequant_batch_kernel<NF4_FP16, false, CLS>), grid, block, 0, s, ba, log2_bs);    \
        } else {                                                                                                 \
            if (dq) hipLaunchKernelGGL((dequant_batch_kernel<NF4_BF16, true, CLS>), grid, block, 0, s, ba, log2_bs);  \
            else hipLaunchKernelGGL((dequant_batch_kernel<NF4_BF16, false, CLS>), grid, block, 0, s, ba, log2_bs);    \
        }                                                                                                        \
    } while (0)
    const OutClass cls = out_class(total);
    if (cls == kOutSmall) NF4_LAUNCH_BATCH(kOutSmall);
    else if (cls == kOutCached) NF4_LAUNCH_BATCH(kOutCached);
    else NF4_LAUNCH_BATCH(kOutStream);
#undef NF4_LAUNCH_BATCH
    return record_hip(hipGetLastError());
}
