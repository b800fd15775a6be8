// Codebook-placement study for the NF4 dequantisation kernel on gfx950.
//
// The paper's contribution on Ampere is WHERE the 16-entry level table lives
// (Sec. IV-B: staged from constant memory into shared memory by thread 0;
// Sec. III-B: the baseline re-reads it from global memory).  On CDNA4 that is
// an open question, answered here by measurement.  Every variant below is the
// library's dequantisation kernel in its first form -- same tile, same 128-bit
// loads, same LDS lane exchange, non-temporal 128-bit stores for every tensor
// size (the library has since picked the stores' cache policy by output size,
// which is independent of the table's placement) -- and differs ONLY in how a
// 4-bit code becomes an FP32 level:
//
//   bpermute     level[lane mod 16] in a VGPR built from literals, read with
//                ds_bpermute_b32
//   lds16        16 floats in LDS written from literals by the first 16 lanes
//                of a workgroup, read with ds_read_b32 (the library's choice)
//   lds16_const  the paper's design transplanted: table in constant memory,
//                one lane copies it to LDS, barrier, ds_read_b32
//   lds256       256-entry byte -> (level[hi], level[lo]) table in LDS (2 KiB),
//                one ds_read_b64 per byte: half the lookups, random 8-byte reads
//   global       every lookup reads the table from memory through the vector
//                cache (the access pattern the paper's baseline has)
//   select       no memory at all: a chain of 15 v_cndmask per lookup
//
// Usage: codebook_study [--variant NAME|all] [--threads 64|256] [--iters N]
//                       [--elements N]
// Prints one line per variant with the mean kernel time (HIP events) and
// checks that every variant's output is bit-identical to the first one run.
// A plain copy kernel of known size ("copy_256MiB") runs as well, so that the
// same process can calibrate FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "../csrc/nf4_device.hpp"

using nf4::kLevelBits;
using nf4::pack2;
using nf4::u32x4;
using nf4::level_literal;
using nf4::wave_lds_fence;

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                                   \
        }                                                                              \
    } while (0)

enum Placement { BPERMUTE = 0, LDS16 = 1, LDS16_CONST = 2, LDS256 = 3, GLOBAL = 4, SELECT = 5 };
static const char* kNames[] = {"bpermute", "lds16", "lds16_const", "lds256", "global", "select"};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct Tables {
    const float* lut;        // LDS, 16 entries
    const f32x2* lut2;       // LDS, 256 entries
    const float* gtable;     // global, 16 entries
    int table_reg;           // VGPR, level[lane mod 16]
};

template <int P>
__device__ __forceinline__ float level_of(const Tables& t, uint32_t code) {
    if constexpr (P == BPERMUTE) return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)(code << 2), t.table_reg));
    else if constexpr (P == LDS16 || P == LDS16_CONST) return t.lut[code];
    else if constexpr (P == GLOBAL) return t.gtable[code];
    else return __uint_as_float(level_literal(code));
}

template <int P>
__device__ __forceinline__ u32x4 expand8(const Tables& t, uint32_t q, float s) {
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float hi, lo;
        if constexpr (P == LDS256) {
            const f32x2 p = t.lut2[(q >> (8 * j)) & 255u];
            hi = p[0];
            lo = p[1];
        } else {
            hi = level_of<P>(t, (q >> (8 * j + 4)) & 15u);
            lo = level_of<P>(t, (q >> (8 * j)) & 15u);
        }
        r[j] = pack2<NF4_FP16>(hi * s, lo * s);
    }
    return r;
}

template <int P, int THREADS>
__global__ __launch_bounds__(THREADS) void study_kernel(const uint8_t* __restrict__ packed,
                                                        const float* __restrict__ absmax,
                                                        const float* __restrict__ gtable, int64_t tiles,
                                                        uint16_t* __restrict__ out) {
    constexpr int WAVES = THREADS / 64;
    __shared__ __attribute__((aligned(16))) float lut[16];
    __shared__ f32x2 lut2[P == LDS256 ? 256 : 1];
    __shared__ uint32_t stage[WAVES][256];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t = (int64_t)blockIdx.x * WAVES + wave;
    const bool live = t < tiles;
    const int64_t e0 = t * 2048;

    Tables tb = {lut, lut2, gtable, 0};
    if constexpr (P == BPERMUTE) tb.table_reg = (int)level_literal(lane & 15);
    if constexpr (P == LDS16) {
        if (threadIdx.x < 16) lut[threadIdx.x] = __uint_as_float(level_literal(threadIdx.x));
        __syncthreads();
    }
    if constexpr (P == LDS16_CONST) {
        if (threadIdx.x == 0)
            for (int i = 0; i < 16; ++i) lut[i] = __uint_as_float(kLevelBits[i]);
        __syncthreads();
    }
    if constexpr (P == LDS256) {
        for (int i = threadIdx.x; i < 256; i += THREADS) {
            f32x2 p = {__uint_as_float(level_literal(i >> 4)), __uint_as_float(level_literal(i & 15))};
            lut2[i] = p;
        }
        __syncthreads();
    }
    // the loads come after the table is written, as in the library's kernel (the other order measured 1.2 % slower)
    u32x4 codes = {0, 0, 0, 0};
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        codes = *(const u32x4*)(packed + t * 1024 + lane * 16);
        // the tile's 32 block scales: one contiguous load by lanes 0..31, then shared across lanes
        float mine = 0.0f;
        if (lane < 32) mine = absmax[(e0 >> 6) + lane];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            s[k] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((8 * k + (lane >> 3)) << 2,
                                                                            __builtin_bit_cast(int, mine)));
    }
    if (!live) return;

    *(u32x4*)&stage[wave][lane * 4] = codes;
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t q = stage[wave][64 * k + lane];
        const u32x4 v = expand8<P>(tb, q, s[k]);
        __builtin_nontemporal_store(v, (u32x4*)(out + e0 + 512 * k + 8 * lane));
    }
}

// Calibration for the HBM byte counters: reads n16*16 bytes, writes n16*16 bytes.
__global__ __launch_bounds__(256) void copy_known_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out,
                                                         int64_t n16) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) out[i] = in[i];
}

__global__ void init_gtable_kernel(float* gtable) { gtable[threadIdx.x] = __uint_as_float(kLevelBits[threadIdx.x]); }

template <int P, int THREADS>
static void launch_variant(const uint8_t* packed, const float* absmax, const float* gtable, int64_t tiles,
                           uint16_t* out, hipStream_t st) {
    constexpr int WAVES = THREADS / 64;
    const unsigned grid = (unsigned)((tiles + WAVES - 1) / WAVES);
    hipLaunchKernelGGL((study_kernel<P, THREADS>), dim3(grid), dim3(THREADS), 0, st, packed, absmax, gtable, tiles, out);
}

typedef void (*LaunchFn)(const uint8_t*, const float*, const float*, int64_t, uint16_t*, hipStream_t);

template <int THREADS>
static LaunchFn pick(int p) {
    switch (p) {
        case BPERMUTE: return launch_variant<BPERMUTE, THREADS>;
        case LDS16: return launch_variant<LDS16, THREADS>;
        case LDS16_CONST: return launch_variant<LDS16_CONST, THREADS>;
        case LDS256: return launch_variant<LDS256, THREADS>;
        case GLOBAL: return launch_variant<GLOBAL, THREADS>;
        default: return launch_variant<SELECT, THREADS>;
    }
}

int main(int argc, char** argv) {
    std::string want = "all";
    int threads = 64, iters = 20;
    int64_t n = 234881024;                        // one 8192 x 28672 projection
    for (int i = 1; i < argc; ++i) {
        if (!strcmp(argv[i], "--variant") && i + 1 < argc) want = argv[++i];
        else if (!strcmp(argv[i], "--threads") && i + 1 < argc) threads = atoi(argv[++i]);
        else if (!strcmp(argv[i], "--iters") && i + 1 < argc) iters = atoi(argv[++i]);
        else if (!strcmp(argv[i], "--elements") && i + 1 < argc) n = atoll(argv[++i]);
        else { fprintf(stderr, "unknown argument %s\n", argv[i]); return 2; }
    }
    if (threads != 64 && threads != 256) { fprintf(stderr, "--threads must be 64 or 256\n"); return 2; }
    if (n < 2048 || n % 2048 != 0 || iters < 1) { fprintf(stderr, "--elements must be a positive multiple of 2048\n"); return 2; }
    const int64_t tiles = n / 2048;

    // synthetic codes (every byte value equally likely) and scales, 4 distinct inputs
    const int NIN = 4;
    std::vector<uint8_t> h(n / 2);
    std::vector<float> ha(n / 64);
    uint8_t* packed[NIN];
    float* absmax[NIN];
    for (int i = 0; i < NIN; ++i) {
        uint64_t x = 88172645463325252ull + i;
        for (size_t j = 0; j < h.size(); j += 8) { x ^= x << 13; x ^= x >> 7; x ^= x << 17; memcpy(&h[j], &x, 8); }
        for (size_t j = 0; j < ha.size(); ++j) { x ^= x << 13; x ^= x >> 7; x ^= x << 17; ha[j] = 0.01f + (x & 0xffff) * 1e-6f; }
        CK(hipMalloc(&packed[i], n / 2));
        CK(hipMalloc(&absmax[i], n / 64 * 4));
        CK(hipMemcpy(packed[i], h.data(), n / 2, hipMemcpyHostToDevice));
        CK(hipMemcpy(absmax[i], ha.data(), n / 64 * 4, hipMemcpyHostToDevice));
    }
    uint16_t *out, *ref;
    CK(hipMalloc(&out, n * 2));
    CK(hipMalloc(&ref, n * 2));
    float* gtable;
    CK(hipMalloc(&gtable, 64));
    hipStream_t st;
    CK(hipStreamCreate(&st));
    hipLaunchKernelGGL(init_gtable_kernel, dim3(1), dim3(16), 0, st, gtable);
    CK(hipStreamSynchronize(st));
    hipEvent_t ea, eb;
    CK(hipEventCreate(&ea));
    CK(hipEventCreate(&eb));

    const double bytes = n * 2.5625;
    std::vector<uint16_t> first, cur(1 << 20);
    printf("# elements=%lld threads=%d iters=%d algorithmic bytes per launch=%.0f\n", (long long)n, threads, iters, bytes);
    for (int p = 0; p < 6; ++p) {
        if (want != "all" && want != kNames[p]) continue;
        LaunchFn f = threads == 64 ? pick<64>(p) : pick<256>(p);
        for (int i = 0; i < 3; ++i) f(packed[i % NIN], absmax[i % NIN], gtable, tiles, out, st);
        CK(hipStreamSynchronize(st));
        CK(hipEventRecord(ea, st));
        for (int i = 0; i < iters; ++i) f(packed[i % NIN], absmax[i % NIN], gtable, tiles, out, st);
        CK(hipEventRecord(eb, st));
        CK(hipStreamSynchronize(st));
        CK(hipGetLastError());
        float ms;
        CK(hipEventElapsedTime(&ms, ea, eb));
        const double us = ms * 1e3 / iters;
        // output check on input 0: first and last MiB of elements against the first variant run
        f(packed[0], absmax[0], gtable, tiles, out, st);
        CK(hipStreamSynchronize(st));
        const size_t chunk = cur.size() < (size_t)n ? cur.size() : (size_t)n;
        bool same = true;
        for (int part = 0; part < 2; ++part) {
            const size_t off = part == 0 ? 0 : (size_t)n - chunk;
            CK(hipMemcpy(cur.data(), out + off, chunk * 2, hipMemcpyDeviceToHost));
            if (first.size() < 2 * chunk) first.insert(first.end(), cur.begin(), cur.begin() + chunk);
            else same = same && memcmp(first.data() + part * chunk, cur.data(), chunk * 2) == 0;
        }
        printf("%-12s %9.2f us  %8.1f GB/s  %5.1f%% of 8 TB/s  output %s\n", kNames[p], us, bytes / us * 1e-3,
               bytes / us * 1e-3 / 80.0, same ? "identical" : "DIFFERS");
        fflush(stdout);
        if (!same) return 1;
    }
    // calibration copy: 256 MiB read + 256 MiB written
    const int64_t n16 = (256ll << 20) / 16;
    if ((int64_t)n * 2 >= (256ll << 20)) {
        hipLaunchKernelGGL(copy_known_kernel, dim3((unsigned)(n16 / 256)), dim3(256), 0, st, (const u32x4*)out, (u32x4*)ref, n16);
        CK(hipStreamSynchronize(st));
        CK(hipGetLastError());
        printf("copy_256MiB  done (268435456 bytes read, 268435456 bytes written)\n");
    }
    return 0;
}
