// Reference-quality NF4 quantiser for gfx950: the forward direction of
// Sec. II-B (block absmax, nearest of the 16 levels), plus this library's
// second-level quantisation of the absmax array.  Written for exactness, not
// speed: every FP32 step is the one the definition names, in the same order,
// so codes and scales are reproducible bit for bit.
#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

constexpr int kQThreads = 256;
constexpr int kQWaves = kQThreads / kWave;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        float o = __shfl_xor(v, m, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// Nearest of the 16 levels: smallest |xn - level| in FP32, codes scanned upward, strict comparison (a tie
// keeps the lower code).
__device__ __forceinline__ unsigned nearest_code(const float* lut, float xn) {
    float best_d = fabsf(xn - lut[0]);
    unsigned best = 0;
#pragma unroll
    for (unsigned k = 1; k < 16; ++k) {
        float d = fabsf(xn - lut[k]);
        if (d < best_d) { best_d = d; best = k; }
    }
    return best;
}

// One wave per quantisation block.  Pass 1: absmax.  Pass 2: for every pair of
// elements the even lane gathers its neighbour's code and writes the byte
// (element 2j in the high nibble).  `codebook` is the caller's 16 levels, or
// nullptr for NF4; an all-zero block and the unused nibble of an odd n take the
// code nearest to zero (7 for NF4).
__global__ __launch_bounds__(kQThreads) void quantize_kernel(const float* __restrict__ src, int64_t n,
                                                             int blocksize, int64_t nb,
                                                             const float* __restrict__ codebook,
                                                             const int* __restrict__ skip_if,
                                                             uint8_t* __restrict__ packed,
                                                             float* __restrict__ absmax) {
    if (skip_if && *skip_if != 0) return;                  // the tuned kernel has done the work (nf4_quantize_codebook)
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = codebook ? codebook[threadIdx.x] : __uint_as_float(kLevelBits[threadIdx.x]);
    __syncthreads();
    const unsigned zero_code = nearest_code(lut, 0.0f);
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t stride = (int64_t)gridDim.x * kQWaves;
    for (int64_t b = (int64_t)blockIdx.x * kQWaves + (threadIdx.x >> 6); b < nb; b += stride) {
        const int64_t lo = b * blocksize;
        const int64_t hi = lo + blocksize < n ? lo + blocksize : n;
        float a = 0.0f;
        for (int64_t i = lo + lane; i < hi; i += kWave) {
            float m = fabsf(src[i]);
            a = m > a ? m : a;
        }
        a = wave_max(a);
        if (lane == 0) absmax[b] = a;
        for (int64_t i0 = lo; i0 < hi; i0 += kWave) {      // uniform trip count: shuffles stay converged
            const int64_t i = i0 + lane;
            unsigned best = zero_code;
            if (i < hi && a != 0.0f) best = nearest_code(lut, src[i] / a);   // IEEE division
            const unsigned next = __shfl_down(best, 1, kWave); // code of element i + 1
            if ((lane & 1) == 0 && i < hi) packed[i >> 1] = (uint8_t)((best << 4) | (i + 1 < hi ? next : zero_code));
        }
    }
}

// offset = float(sum(absmax) / nb) with the sum as a sequential double-precision sum in index order would give
// it, bit for bit.  Taken literally that is one lane adding 3.7 million values (56 ms for a 8192 x 28672
// tensor).  But a double holds 53 bits: when every partial sum -- of any subset, in any order -- is exactly
// representable, all summation orders give the same, exact, result.  With non-negative terms that is the case
// if the total is below 2^53 units in the last place of the smallest non-zero term, i.e. total < 2^(e_min + 30)
// for a smallest term 1.m x 2^e_min (FP32 subnormals: e_min = -126).  So 1024 threads add strided slices,
// a tree combines them, and only if the test fails (scales spread over more than about 2^29, or a non-finite
// or negative value) does one lane redo the sum in index order.
// Large arrays are first summed slice by slice by many workgroups (dq_partial_kernel) into a scratch area -- the
// head of the absmax_q8 output, which is written only afterwards -- and dq_offset_kernel then combines the slices.
constexpr int kOffsetThreads = 1024;
constexpr int kPartialThreads = 256;
constexpr int kMaxPartials = 1024;                         // slices at most (16 bytes of scratch each)
constexpr int kNoTerm = 1 << 20;                           // "no non-zero term seen"

struct SlicePartial {
    double sum;
    int emin;                                              // smallest biased exponent; kNoTerm; or -1: not clean
    int pad;
};

// Running state of one thread: sum, smallest exponent of a non-zero term, and whether all terms were finite and
// non-negative.
struct OffsetAcc {
    double acc = 0.0;
    int emin = kNoTerm;
    bool clean = true;
    __device__ __forceinline__ void take(float v) {
        const uint32_t bits = __float_as_uint(v);
        const int e = (int)((bits >> 23) & 0xFF);
        clean = clean && (bits >> 31) == 0 && e != 0xFF;
        if ((bits & 0x7FFFFFFFu) != 0) {
            const int eff = e == 0 ? 1 : e;                // subnormals share the exponent of the smallest normals
            emin = eff < emin ? eff : emin;
        }
        acc += (double)v;
    }
    // elements first + tid, first + tid + stride, ... below `end`, eight loads in flight (the order of an exact
    // sum is free)
    __device__ __forceinline__ void take_strided(const float* __restrict__ a, int64_t first, int64_t end, int tid,
                                                 int stride) {
        constexpr int kAhead = 8;
        int64_t i = first + tid;
        for (; i + (int64_t)(kAhead - 1) * stride < end; i += (int64_t)kAhead * stride) {
            float v[kAhead];
#pragma unroll
            for (int j = 0; j < kAhead; ++j) v[j] = a[i + (int64_t)j * stride];
#pragma unroll
            for (int j = 0; j < kAhead; ++j) take(v[j]);
        }
        for (; i < end; i += stride) take(a[i]);
    }
};

__global__ __launch_bounds__(kPartialThreads) void dq_partial_kernel(const float* __restrict__ absmax, int64_t nb,
                                                                      int64_t per_slice,
                                                                      SlicePartial* __restrict__ partials) {
    __shared__ double part[kPartialThreads];
    __shared__ int emin_part[kPartialThreads];
    const int tid = threadIdx.x;
    const int64_t first = (int64_t)blockIdx.x * per_slice;
    const int64_t end = first + per_slice < nb ? first + per_slice : nb;
    OffsetAcc st;
    st.take_strided(absmax, first, end, tid, kPartialThreads);
    part[tid] = st.acc;
    emin_part[tid] = st.clean ? st.emin : -1;
    __syncthreads();
    for (int half = kPartialThreads / 2; half >= 1; half >>= 1) {
        if (tid < half) {
            part[tid] += part[tid + half];
            const int o = emin_part[tid + half];
            emin_part[tid] = o < emin_part[tid] ? o : emin_part[tid];
        }
        __syncthreads();
    }
    if (tid == 0) partials[blockIdx.x] = SlicePartial{part[0], emin_part[0], 0};
}

__global__ __launch_bounds__(kOffsetThreads) void dq_offset_kernel(const float* __restrict__ absmax, int64_t nb,
                                                                   const SlicePartial* __restrict__ partials,
                                                                   int slices, float* __restrict__ offset,
                                                                   float* __restrict__ code2) {
    __shared__ double part[kOffsetThreads];
    __shared__ int emin_part[kOffsetThreads];
    __shared__ float buf[1024];
    __shared__ int exact;
    const int tid = threadIdx.x;
    for (int u = tid; u < 256; u += kOffsetThreads) code2[u] = (float)(u - 127) / 127.0f;

    OffsetAcc st;
    if (slices > 0) {                                      // the slices' sums are the terms (slices <= kOffsetThreads)
        if (tid < slices) {
            st.acc = partials[tid].sum;
            st.emin = partials[tid].emin;
            st.clean = st.emin >= 0;
        }
    } else {
        st.take_strided(absmax, 0, nb, tid, kOffsetThreads);
    }
    double acc = st.acc;
    int emin = st.emin;
    bool clean = st.clean;
    part[tid] = acc;
    emin_part[tid] = clean ? emin : -1;                    // -1 poisons the minimum
    __syncthreads();
    for (int half = kOffsetThreads / 2; half >= 1; half >>= 1) {
        if (tid < half) {
            part[tid] += part[tid + half];
            const int o = emin_part[tid + half];
            emin_part[tid] = o < emin_part[tid] ? o : emin_part[tid];
        }
        __syncthreads();
    }
    if (tid == 0) {
        const double total = part[0];
        const int e = emin_part[0];
        bool ok = e >= 0;                                  // no negative or non-finite term
        if (ok && e != kNoTerm) {                        // some non-zero term: total < 2^(e_min + 30)
            const double limit = __builtin_ldexp(1.0, (e - 127) + 30);
            ok = total < limit;
        }
        exact = ok ? 1 : 0;
        if (ok) offset[0] = (float)(total / (double)nb);
    }
    __syncthreads();
    if (exact) return;

    // the literal definition: index order, one lane; the block only stages 1024 values at a time in LDS
    double sum = 0.0;
    for (int64_t base = 0; base < nb; base += 1024) {
        const int64_t left = nb - base;
        const int cnt = left < 1024 ? (int)left : 1024;
        __syncthreads();
        if (tid < cnt) buf[tid] = absmax[base + tid];
        __syncthreads();
        if (tid == 0)
            for (int j = 0; j < cnt; ++j) sum += (double)buf[j];
    }
    if (tid == 0) offset[0] = (float)(sum / (double)nb);
}

// One wave per group of `group` first-level scales (256 in the format's default).
__global__ __launch_bounds__(kQThreads) void dq_encode_kernel(const float* __restrict__ absmax, int64_t nb,
                                                              int64_t ng, int64_t group,
                                                              const float* __restrict__ offset,
                                                              uint8_t* __restrict__ q8,
                                                              float* __restrict__ scale2) {
    const int lane = threadIdx.x & (kWave - 1);
    const float off = offset[0];
    const int64_t stride = (int64_t)gridDim.x * kQWaves;
    for (int64_t g = (int64_t)blockIdx.x * kQWaves + (threadIdx.x >> 6); g < ng; g += stride) {
        const int64_t lo = g * group;
        const int64_t hi = lo + group < nb ? lo + group : nb;
        float s = 0.0f;
        for (int64_t b = lo + lane; b < hi; b += kWave) {
            float d = fabsf(absmax[b] - off);
            s = d > s ? d : s;
        }
        s = wave_max(s);
        if (lane == 0) scale2[g] = s;
        for (int64_t b = lo + lane; b < hi; b += kWave) {
            int q = 127;
            if (s != 0.0f) {
                const float centred = absmax[b] - off;
                const float scaled = 127.0f * centred;
                float r = rintf(scaled / s);               // ties to even
                r = r < -127.0f ? -127.0f : r;
                r = r > 127.0f ? 127.0f : r;
                q = 127 + (int)r;
            }
            q8[b] = (uint8_t)q;
        }
    }
}

// First level only (codes and absmax) of a range that starts on a block boundary;
// also used by the tuned quantiser for other block sizes and for ragged ends.
int launch_quantize_ref_range(const float* src, int64_t n, int blocksize, const float* codebook, const int* skip_if,
                              uint8_t* packed, float* absmax, hipStream_t s) {
    const int64_t nb = (n + blocksize - 1) / blocksize;
    const int64_t cap = (int64_t)compute_units() * 16;
    int64_t groups = (nb + kQWaves - 1) / kQWaves;
    groups = groups < cap ? groups : cap;
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)groups), dim3(kQThreads), 0, s, src, n, blocksize, nb,
                       codebook, skip_if, packed, absmax);
    return record_hip(hipGetLastError());
}

}  // namespace nf4

extern "C" int nf4_quantize_ref_codebook(const float* src, int64_t n, int blocksize, const float* codebook,
                                         int dq_group, uint8_t* packed, float* absmax, uint8_t* absmax_q8,
                                         float* scale2, float* offset, float* code2, void* stream) {
    using namespace nf4;
    if (n < 0) return NF4_ERR_SIZE;
    if (log2_blocksize(blocksize) < 0) return NF4_ERR_BLOCKSIZE;
    const bool dq = absmax_q8 != nullptr;
    if (dq && log2_dq_group(dq_group) < 0) return NF4_ERR_SHAPE;
    if (n == 0) return NF4_OK;
    if (!src || !packed || !absmax) return NF4_ERR_NULL;
    if (dq && (!scale2 || !offset || !code2)) return NF4_ERR_NULL;
    if (!aligned(src, 4) || !aligned(absmax, 4) || (codebook && !aligned(codebook, 4))) return NF4_ERR_ALIGN;
    if (dq && (!aligned(scale2, 4) || !aligned(offset, 4) || !aligned(code2, 4))) return NF4_ERR_ALIGN;

    hipStream_t s = (hipStream_t)stream;
    const int64_t nb = (n + blocksize - 1) / blocksize;
    int rc = launch_quantize_ref_range(src, n, blocksize, codebook, nullptr, packed, absmax, s);
    if (rc != NF4_OK || !dq) return rc;

    return nf4_dq_encode(absmax, nb, dq_group, absmax_q8, scale2, offset, code2, stream);
}

extern "C" int nf4_dq_encode(const float* absmax, int64_t nb, int dq_group, uint8_t* absmax_q8, float* scale2,
                             float* offset, float* code2, void* stream) {
    using namespace nf4;
    if (nb < 0) return NF4_ERR_SIZE;
    if (log2_dq_group(dq_group) < 0) return NF4_ERR_SHAPE;
    if (nb == 0) return NF4_OK;
    if (!absmax || !absmax_q8 || !scale2 || !offset || !code2) return NF4_ERR_NULL;
    if (!aligned(absmax, 4) || !aligned(scale2, 4) || !aligned(offset, 4) || !aligned(code2, 4)) return NF4_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    const int64_t cap = (int64_t)compute_units() * 16;
    const int64_t ng = (nb + dq_group - 1) / dq_group;
    // slices of at least 16384 scales, as many as fit the scratch area at the (8-byte aligned) head of absmax_q8
    const uintptr_t q8_addr = (uintptr_t)absmax_q8;
    SlicePartial* partials = (SlicePartial*)((q8_addr + 7) & ~(uintptr_t)7);
    const int64_t room = (nb - (int64_t)((uintptr_t)partials - q8_addr)) / (int64_t)sizeof(SlicePartial);
    int64_t slices = nb / 16384;
    slices = slices < room ? slices : room;
    slices = slices < kMaxPartials ? slices : kMaxPartials;
    int rc;
    if (slices >= 2) {
        const int64_t per_slice = (nb + slices - 1) / slices;
        slices = (nb + per_slice - 1) / per_slice;
        hipLaunchKernelGGL(dq_partial_kernel, dim3((unsigned)slices), dim3(kPartialThreads), 0, s, absmax, nb, per_slice,
                           partials);
        rc = record_hip(hipGetLastError());
        if (rc != NF4_OK) return rc;
    } else {
        slices = 0;
    }
    hipLaunchKernelGGL(dq_offset_kernel, dim3(1), dim3(kOffsetThreads), 0, s, absmax, nb,
                       (const SlicePartial*)partials, (int)slices, offset, code2);
    rc = record_hip(hipGetLastError());
    if (rc != NF4_OK) return rc;
    int64_t g2 = (ng + kQWaves - 1) / kQWaves;
    g2 = g2 < cap ? g2 : cap;
    hipLaunchKernelGGL(dq_encode_kernel, dim3((unsigned)g2), dim3(kQThreads), 0, s, absmax, nb, ng,
                       (int64_t)dq_group, (const float*)offset, absmax_q8, scale2);
    return record_hip(hipGetLastError());
}

extern "C" int nf4_quantize_ref(const float* src, int64_t n, int blocksize, uint8_t* packed, float* absmax,
                                uint8_t* absmax_q8, float* scale2, float* offset, float* code2,
                                void* stream) {
    return nf4_quantize_ref_codebook(src, n, blocksize, nullptr, 256, packed, absmax, absmax_q8, scale2, offset,
                                     code2, stream);
}
