/*
 * nf4_oracle.c -- plain, slow, scalar CPU statement of blockwise NF4
 * (4-bit NormalFloat) quantization and dequantization.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the HIP kernels are
 * compared against.  It shares no code, header, table or helper with the GPU
 * library; nothing in the product path may call it.  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg load it.
 *
 * What it follows (paper = "Fast NF4 Dequantization Kernels for Large
 * Language Model Inference"):
 *   - Sec. II-B "NF4 Quantization Fundamentals": 16 levels that are quantiles
 *     of a normal distribution normalised to [-1, 1]; one scaling factor
 *     (absmax) per block of 64 elements.
 *   - Algorithm 1: out[2j] = table[q >> 4] * scale, out[2j+1] = table[q & 15]
 *     * scale; the table is FP32, the result is FP16.
 *   - Sec. V-A "Kernel Architecture": sizes that do not fill a tile are legal.
 * The paper never prints the 16 levels; they are the FP32 constants published
 * for NF4 by the QLoRA paper it cites in Sec. II-B, and tests pin them to the
 * normal-quantile construction.
 *
 * Points on which the paper is silent and the reading taken here:
 *   - "absmax[blockIdx]" in Algorithm 1 is the quantisation-block index
 *     floor(i / blocksize) of element i (Sec. II-B: one scale per 64 elements).
 *   - One FP32 multiply, then one round-to-nearest-even conversion to the
 *     16-bit output type; IEEE semantics throughout (subnormals kept,
 *     overflow to infinity, 0 * inf = NaN).
 *   - BF16 output, the double-quantised absmax and the fused GEMV are not in
 *     the paper; their definitions below are this build's statement of them.
 *     Parity unpinned (no external reference exists): nf4o_dq_encode and its
 *     group-size form nf4o_dq_encode_group.  Their decoder formula and
 *     invariants are pinned by tests.
 *   - Sec. V-A names the data type as a parameter of the kernel; the *_codebook
 *     functions at the end state the same format for any table of 16 FP32
 *     levels and any number of blocks per second-level group.
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fPIC -shared (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* Sec. II-B: the 16 NF4 levels, index 0..15, ascending, level 7 is zero. */
static const float NF4_LEVEL[16] = {
    -1.0f,
    -0.6961928009986877f,
    -0.5250730514526367f,
    -0.39491748809814453f,
    -0.28444138169288635f,
    -0.18477343022823334f,
    -0.09105003625154495f,
    0.0f,
    0.07958029955625534f,
    0.16093020141124725f,
    0.24611230194568634f,
    0.33791524171829224f,
    0.44070982933044434f,
    0.5626170039176941f,
    0.7229568362236023f,
    1.0f,
};

enum { NF4O_FP16 = 0, NF4O_BF16 = 1, NF4O_FP32 = 2 };

void nf4o_table(float *dst16) {
    for (int k = 0; k < 16; ++k) dst16[k] = NF4_LEVEL[k];
}

static uint32_t bits_of(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/* IEEE-754 binary32 -> binary16, round to nearest, ties to even. */
uint16_t nf4o_f32_to_f16(float f) {
    uint32_t u = bits_of(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t bexp = (u >> 23) & 0xFFu;
    uint32_t frac = u & 0x7FFFFFu;

    if (bexp == 0xFFu) {
        if (frac == 0) return (uint16_t)(sign | 0x7C00u);              /* inf */
        return (uint16_t)(sign | 0x7E00u | (frac >> 13));              /* quiet NaN */
    }
    if (bexp == 0) return sign;          /* |f| < 2^-126: far below half of 2^-24 */

    int e = (int)bexp - 127;             /* f = 1.frac * 2^e */
    if (e > 15) return (uint16_t)(sign | 0x7C00u);
    if (e >= -14) {
        /* normal half: keep 10 fraction bits, 13 are dropped */
        uint32_t h = ((uint32_t)(e + 15) << 10) | (frac >> 13);
        uint32_t dropped = frac & 0x1FFFu;
        if (dropped > 0x1000u || (dropped == 0x1000u && (h & 1u))) h += 1; /* carry may reach inf */
        return (uint16_t)(sign | h);
    }
    /* subnormal half: units of 2^-24.  f = sig * 2^(e-23), sig has 24 bits. */
    uint32_t sig = 0x800000u | frac;
    int shift = -(e + 1);                /* f / 2^-24 = sig / 2^shift, shift >= 14 */
    if (shift > 24) return sign;         /* below half a unit */
    uint32_t q = sig >> shift;
    uint32_t dropped = sig & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (dropped > half || (dropped == half && (q & 1u))) q += 1;
    return (uint16_t)(sign | q);
}

/* IEEE-754 binary32 -> bfloat16, round to nearest, ties to even. */
uint16_t nf4o_f32_to_bf16(float f) {
    uint32_t u = bits_of(f);
    if (((u >> 23) & 0xFFu) == 0xFFu && (u & 0x7FFFFFu) != 0)
        return (uint16_t)((u >> 16) | 0x0040u);                        /* quiet NaN */
    uint32_t kept = u >> 16;
    uint32_t dropped = u & 0xFFFFu;
    if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) kept += 1;
    return (uint16_t)kept;
}

/* Algorithm 1, nibble split: element i lives in byte i/2; the even element
 * is the high nibble. */
static unsigned code_of(const uint8_t *packed, int64_t i) {
    uint8_t q = packed[i >> 1];
    return (i & 1) == 0 ? (unsigned)(q >> 4) : (unsigned)(q & 0x0Fu);
}

static void store_out(void *out, int64_t i, float v, int out_dtype) {
    if (out_dtype == NF4O_FP16) ((uint16_t *)out)[i] = nf4o_f32_to_f16(v);
    else if (out_dtype == NF4O_BF16) ((uint16_t *)out)[i] = nf4o_f32_to_bf16(v);
    else ((float *)out)[i] = v;
}

/* Algorithm 1 with the scale of Sec. II-B: out[i] = round(table[code_i] *
 * absmax[i / blocksize]).  Elements [first, first + count) only, so a caller
 * may split the range over threads; indices are global. */
void nf4o_dequantize_range(const uint8_t *packed, const float *absmax, int blocksize,
                           int64_t first, int64_t count, void *out, int out_dtype) {
    for (int64_t i = first; i < first + count; ++i) {
        float level = NF4_LEVEL[code_of(packed, i)];
        float scale = absmax[i / blocksize];
        float v = level * scale;
        store_out(out, i, v, out_dtype);
    }
}

void nf4o_dequantize(const uint8_t *packed, const float *absmax, int blocksize, int64_t n,
                     void *out, int out_dtype) {
    nf4o_dequantize_range(packed, absmax, blocksize, 0, n, out, out_dtype);
}

/* Double-quantised scale of block b: an 8-bit code looked up in a 256-entry
 * map, times the second-level scale of its group of 256 blocks, plus one
 * global offset.  Multiply and add are two separately rounded FP32 operations. */
static float dq_scale(const uint8_t *absmax_q8, const float *scale2, float offset,
                      const float *code2, int64_t b) {
    float prod = code2[absmax_q8[b]] * scale2[b / 256];
    return prod + offset;
}

void nf4o_dq_decode(const uint8_t *absmax_q8, const float *scale2, const float *offset,
                    const float *code2, int64_t nb, float *absmax) {
    for (int64_t b = 0; b < nb; ++b) absmax[b] = dq_scale(absmax_q8, scale2, offset[0], code2, b);
}

void nf4o_dequantize_dq(const uint8_t *packed, const uint8_t *absmax_q8, const float *scale2,
                        const float *offset, const float *code2, int blocksize, int64_t n,
                        void *out, int out_dtype) {
    for (int64_t i = 0; i < n; ++i) {
        float level = NF4_LEVEL[code_of(packed, i)];
        float scale = dq_scale(absmax_q8, scale2, offset[0], code2, i / blocksize);
        float v = level * scale;
        store_out(out, i, v, out_dtype);
    }
}

/* Sec. II-B, forward direction.  Per block: absmax = max |x|; each element is
 * divided by it and mapped to the nearest level.  Nearest = smallest
 * |x/absmax - level| in FP32, levels scanned in ascending order with a strict
 * comparison, so an exact tie keeps the lower index.  An all-zero block stores
 * absmax 0 and code 7.  A partial last block uses the elements it has; with an
 * odd n the unused low nibble of the last byte is code 7. */
void nf4o_quantize(const float *src, int64_t n, int blocksize, uint8_t *packed, float *absmax) {
    int64_t nb = (n + blocksize - 1) / blocksize;
    for (int64_t b = 0; b < nb; ++b) {
        int64_t lo = b * blocksize;
        int64_t hi = lo + blocksize < n ? lo + blocksize : n;
        float a = 0.0f;
        for (int64_t i = lo; i < hi; ++i) {
            float m = fabsf(src[i]);
            if (m > a) a = m;
        }
        absmax[b] = a;
        for (int64_t i = lo; i < hi; ++i) {
            unsigned best = 7;
            if (a != 0.0f) {
                float xn = src[i] / a;
                float best_d = fabsf(xn - NF4_LEVEL[0]);
                best = 0;
                for (unsigned k = 1; k < 16; ++k) {
                    float d = fabsf(xn - NF4_LEVEL[k]);
                    if (d < best_d) { best_d = d; best = k; }
                }
            }
            uint8_t *byte = &packed[i >> 1];
            if ((i & 1) == 0) *byte = (uint8_t)((best << 4) | 7u);   /* low nibble until filled */
            else *byte = (uint8_t)((*byte & 0xF0u) | best);
        }
    }
}

/* Second-level quantisation of the absmax array (this build's encoder; the
 * decoder formula above is the contract).  code2[u] = (u - 127) / 127;
 * offset = mean(absmax) summed in double in index order; per group of 256
 * blocks scale2 = max |absmax - offset|; q8 = 127 + clamp(rint(127 * (absmax -
 * offset) / scale2), -127, 127), rint = ties to even; a group whose scale2 is
 * zero stores q8 = 127 everywhere. */
void nf4o_dq_encode(const float *absmax, int64_t nb, uint8_t *absmax_q8, float *scale2,
                    float *offset, float *code2) {
    for (int u = 0; u < 256; ++u) code2[u] = (float)(u - 127) / 127.0f;
    double sum = 0.0;
    for (int64_t b = 0; b < nb; ++b) sum += (double)absmax[b];
    float off = nb > 0 ? (float)(sum / (double)nb) : 0.0f;
    offset[0] = off;
    int64_t ng = (nb + 255) / 256;
    for (int64_t g = 0; g < ng; ++g) {
        int64_t lo = g * 256;
        int64_t hi = lo + 256 < nb ? lo + 256 : nb;
        float s = 0.0f;
        for (int64_t b = lo; b < hi; ++b) {
            float d = fabsf(absmax[b] - off);
            if (d > s) s = d;
        }
        scale2[g] = s;
        for (int64_t b = lo; b < hi; ++b) {
            int q = 127;
            if (s != 0.0f) {
                float centred = absmax[b] - off;
                float scaled = 127.0f * centred;
                float r = rintf(scaled / s);
                if (r < -127.0f) r = -127.0f;
                if (r > 127.0f) r = 127.0f;
                q = 127 + (int)r;
            }
            absmax_q8[b] = (uint8_t)q;
        }
    }
}

/* Fused dequantise + matrix-vector product, stated in double precision:
 * y[b][r] = round_fp16( sum_k x[b][k] * W[r][k] ), W[r][k] = FP32 product
 * table[code] * scale of element r*K + k (W is [N][K] row-major, quantisation
 * blocks run along the flat index), no rounding of W to 16 bits, the sum taken
 * in index order.  x and y are FP16 bit patterns; y_f64 (optional) receives the
 * unrounded sums. */
static double f16_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

/* Rows [r_first, r_first + r_count) only; y and y_f64 are [B][r_count]. */
void nf4o_dequant_gemv_rows(const uint8_t *packed, const uint8_t *absmax_q8, const float *scale2,
                            const float *offset, const float *code2, int blocksize, int64_t K,
                            const uint16_t *x, int B, int64_t r_first, int64_t r_count,
                            uint16_t *y, double *y_f64) {
    for (int b = 0; b < B; ++b) {
        for (int64_t r = r_first; r < r_first + r_count; ++r) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t i = r * K + k;
                float scale = dq_scale(absmax_q8, scale2, offset[0], code2, i / blocksize);
                float w = NF4_LEVEL[code_of(packed, i)] * scale;
                acc += f16_bits_to_double(x[(int64_t)b * K + k]) * (double)w;
            }
            int64_t o = (int64_t)b * r_count + (r - r_first);
            if (y_f64) y_f64[o] = acc;
            if (y) y[o] = nf4o_f32_to_f16((float)acc);
        }
    }
}

void nf4o_dequant_gemv(const uint8_t *packed, const uint8_t *absmax_q8, const float *scale2,
                       const float *offset, const float *code2, int blocksize, int64_t N,
                       int64_t K, const uint16_t *x, int B, uint16_t *y, double *y_f64) {
    nf4o_dequant_gemv_rows(packed, absmax_q8, scale2, offset, code2, blocksize, K, x, B, 0, N, y, y_f64);
}

/* Fused dequantise + small-batch GEMM as the paper's flow defines it (Sec. III-A:
 * the weights are dequantised to FP16 because the matrix units take 16-bit
 * inputs, then multiplied with FP32 accumulation): the same sum as
 * nf4o_dequant_gemv_rows, but every weight is first rounded to FP16,
 * W16 = round_fp16(table[code] * scale).  Rows [r_first, r_first + r_count). */
void nf4o_dequant_gemm_rows(const uint8_t *packed, const uint8_t *absmax_q8, const float *scale2,
                            const float *offset, const float *code2, int blocksize, int64_t K,
                            const uint16_t *x, int B, int64_t r_first, int64_t r_count,
                            uint16_t *y, double *y_f64) {
    for (int b = 0; b < B; ++b) {
        for (int64_t r = r_first; r < r_first + r_count; ++r) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t i = r * K + k;
                float scale = dq_scale(absmax_q8, scale2, offset[0], code2, i / blocksize);
                float w = NF4_LEVEL[code_of(packed, i)] * scale;
                double w16 = f16_bits_to_double(nf4o_f32_to_f16(w));
                acc += f16_bits_to_double(x[(int64_t)b * K + k]) * w16;
            }
            int64_t o = (int64_t)b * r_count + (r - r_first);
            if (y_f64) y_f64[o] = acc;
            if (y) y[o] = nf4o_f32_to_f16((float)acc);
        }
    }
}

/* ---- the same format with the data type as a parameter (Sec. V-A) -------------
 *
 * `table` is any 16 FP32 levels, indexed by the 4-bit code; `group` is the number
 * of quantisation blocks that share one second-level scale.  With the NF4 table
 * and group = 256 these compute what the functions above compute. */

void nf4o_dequantize_codebook(const uint8_t *packed, const float *absmax, const float *table,
                              int blocksize, int64_t n, void *out, int out_dtype) {
    for (int64_t i = 0; i < n; ++i) {
        float level = table[code_of(packed, i)];
        float scale = absmax[i / blocksize];
        float v = level * scale;
        store_out(out, i, v, out_dtype);
    }
}

void nf4o_dequantize_dq_codebook(const uint8_t *packed, const uint8_t *absmax_q8,
                                 const float *scale2, const float *offset, const float *code2,
                                 int group, const float *table, int blocksize, int64_t n,
                                 void *out, int out_dtype) {
    for (int64_t i = 0; i < n; ++i) {
        int64_t b = i / blocksize;
        float prod = code2[absmax_q8[b]] * scale2[b / group];
        float scale = prod + offset[0];
        float level = table[code_of(packed, i)];
        float v = level * scale;
        store_out(out, i, v, out_dtype);
    }
}

/* Nearest level of `table` to xn: smallest |xn - table[k]| in FP32, codes scanned
 * from 0 upward with a strict comparison (a tie keeps the lower code). */
static unsigned nearest_code(const float *table, float xn) {
    unsigned best = 0;
    float best_d = fabsf(xn - table[0]);
    for (unsigned k = 1; k < 16; ++k) {
        float d = fabsf(xn - table[k]);
        if (d < best_d) { best_d = d; best = k; }
    }
    return best;
}

/* Forward direction for any table.  As nf4o_quantize, except that an all-zero
 * block and the unused nibble of an odd n take the code nearest to 0 (for NF4
 * that is code 7, the zero level). */
void nf4o_quantize_codebook(const float *src, int64_t n, int blocksize, const float *table,
                            uint8_t *packed, float *absmax) {
    unsigned zero_code = nearest_code(table, 0.0f);
    int64_t nb = (n + blocksize - 1) / blocksize;
    for (int64_t b = 0; b < nb; ++b) {
        int64_t lo = b * blocksize;
        int64_t hi = lo + blocksize < n ? lo + blocksize : n;
        float a = 0.0f;
        for (int64_t i = lo; i < hi; ++i) {
            float m = fabsf(src[i]);
            if (m > a) a = m;
        }
        absmax[b] = a;
        for (int64_t i = lo; i < hi; ++i) {
            unsigned best = a != 0.0f ? nearest_code(table, src[i] / a) : zero_code;
            uint8_t *byte = &packed[i >> 1];
            if ((i & 1) == 0) *byte = (uint8_t)((best << 4) | zero_code);
            else *byte = (uint8_t)((*byte & 0xF0u) | best);
        }
    }
}

/* nf4o_dq_encode with `group` blocks per second-level scale instead of 256. */
void nf4o_dq_encode_group(const float *absmax, int64_t nb, int group, uint8_t *absmax_q8,
                          float *scale2, float *offset, float *code2) {
    for (int u = 0; u < 256; ++u) code2[u] = (float)(u - 127) / 127.0f;
    double sum = 0.0;
    for (int64_t b = 0; b < nb; ++b) sum += (double)absmax[b];
    float off = nb > 0 ? (float)(sum / (double)nb) : 0.0f;
    offset[0] = off;
    int64_t ng = (nb + group - 1) / group;
    for (int64_t g = 0; g < ng; ++g) {
        int64_t lo = g * group;
        int64_t hi = lo + group < nb ? lo + group : nb;
        float s = 0.0f;
        for (int64_t b = lo; b < hi; ++b) {
            float d = fabsf(absmax[b] - off);
            if (d > s) s = d;
        }
        scale2[g] = s;
        for (int64_t b = lo; b < hi; ++b) {
            int q = 127;
            if (s != 0.0f) {
                float centred = absmax[b] - off;
                float scaled = 127.0f * centred;
                float r = rintf(scaled / s);
                if (r < -127.0f) r = -127.0f;
                if (r > 127.0f) r = 127.0f;
                q = 127 + (int)r;
            }
            absmax_q8[b] = (uint8_t)q;
        }
    }
}

/* The fused products for any table and group size: the same sums as
 * nf4o_dequant_gemv_rows (weight = the FP32 product table[code] * scale, never
 * rounded to 16 bits) and nf4o_dequant_gemm_rows (weight rounded to FP16 first,
 * Sec. III-A), with the scale of nf4o_dequantize_dq_codebook.  Accumulated in
 * double in index order.  Rows [r_first, r_first + r_count). */
void nf4o_dequant_gemv_rows_codebook(const uint8_t *packed, const uint8_t *absmax_q8,
                                     const float *scale2, const float *offset, const float *code2,
                                     int group, const float *table, int blocksize, int64_t K,
                                     const uint16_t *x, int B, int64_t r_first, int64_t r_count,
                                     int round_weights_to_fp16, uint16_t *y, double *y_f64) {
    for (int b = 0; b < B; ++b) {
        for (int64_t r = r_first; r < r_first + r_count; ++r) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t i = r * K + k;
                int64_t blk = i / blocksize;
                float prod = code2[absmax_q8[blk]] * scale2[blk / group];
                float scale = prod + offset[0];
                float w = table[code_of(packed, i)] * scale;
                double wd = round_weights_to_fp16 ? f16_bits_to_double(nf4o_f32_to_f16(w)) : (double)w;
                acc += f16_bits_to_double(x[(int64_t)b * K + k]) * wd;
            }
            int64_t o = (int64_t)b * r_count + (r - r_first);
            if (y_f64) y_f64[o] = acc;
            if (y) y[o] = nf4o_f32_to_f16((float)acc);
        }
    }
}
