/*
 * nf4.h -- C-ABI of libnf4: blockwise NF4 (4-bit NormalFloat) dequantisation
 * for AMD MI355X (gfx950).
 *
 * Paper: "Fast NF4 Dequantization Kernels for Large Language Model Inference".
 *
 * Format (Sec. II-B; Algorithm 1):
 *   - 16 FP32 levels in [-1, 1] (normal quantiles; level 7 is 0, level 0 is -1,
 *     level 15 is +1).
 *   - Two 4-bit codes per byte; byte j holds element 2j in its HIGH nibble and
 *     element 2j+1 in its LOW nibble.
 *   - One scale ("absmax") per block of `blocksize` consecutive elements of the
 *     flat tensor (the paper uses 64).
 *   - value(i) = level[code(i)] * scale(i / blocksize), one FP32 multiply, then
 *     one round-to-nearest-even conversion to FP16 (the paper's output type) or
 *     BF16.
 *   - Double-quantised scales (not in the paper; this library's definition):
 *     scale(b) = code2[absmax_q8[b]] * scale2[b / 256] + offset[0], an FP32
 *     multiply and an FP32 add, each rounded once (never fused).
 *
 * Conventions for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or synchronises; it only enqueues kernels on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     returns at once.  Inputs must stay valid and unchanged until that work
 *     has run; inputs and outputs must not overlap.
 *   - The return value is an nf4_status.  Nothing aborts or throws.  Arguments
 *     are checked on the host before anything is launched: a call that returns
 *     an error other than NF4_ERR_HIP has launched nothing.
 *   - n == 0 (or N == 0) returns NF4_OK without launching.
 *   - `blocksize` must be a power of two in [64, 4096] (tuned for 64).
 *   - `packed` and the 16-bit outputs must be 16-byte aligned; FP32 arrays
 *     4-byte aligned (else NF4_ERR_ALIGN).
 *   - A tensor with n elements has ceil(n/2) packed bytes, nb = ceil(n /
 *     blocksize) scales and ceil(nb / 256) second-level scales.  Nothing is read
 *     past those sizes or written past out[n-1]; with an odd n the low nibble of
 *     the last byte is ignored (Sec. V-A: sizes that do not fill a tile are
 *     handled by predication).
 */
#ifndef NF4_H
#define NF4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NF4_OK = 0,
    NF4_ERR_NULL = 1,      /* a required pointer is NULL */
    NF4_ERR_SIZE = 2,      /* negative element count, or a size beyond the supported range */
    NF4_ERR_BLOCKSIZE = 3, /* blocksize not a power of two in [64, 4096] */
    NF4_ERR_DTYPE = 4,     /* out_dtype is neither NF4_FP16 nor NF4_BF16 */
    NF4_ERR_ALIGN = 5,     /* a pointer is not aligned as stated above */
    NF4_ERR_SHAPE = 6,     /* GEMV: K not a multiple of blocksize, or B outside [1, 16] */
    NF4_ERR_HIP = 7        /* the HIP runtime refused the launch; see nf4_last_hip_error */
} nf4_status;

typedef enum { NF4_FP16 = 0, NF4_BF16 = 1 } nf4_dtype;

/*
 * Algorithm 1 (with the per-64-element scale of Sec. II-B):
 *   out[i] = rne16( level[code(i)] * absmax[i / blocksize] ),  0 <= i < n.
 * packed : uint8[ceil(n/2)], absmax : float[ceil(n/blocksize)],
 * out    : uint16[n] holding FP16 or BF16 bit patterns per out_dtype.
 */
int nf4_dequantize(const uint8_t* packed, const float* absmax, int blocksize, int64_t n,
                   void* out, int out_dtype, void* stream);

/*
 * Same as nf4_dequantize with double-quantised scales:
 *   scale(b) = code2[absmax_q8[b]] * scale2[b / 256] + offset[0].
 * absmax_q8 : uint8[nb], scale2 : float[ceil(nb/256)], offset : float[1],
 * code2 : float[256] (the caller's map of the 8-bit code).
 */
int nf4_dequantize_dq(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                      const float* offset, const float* code2, int blocksize, int64_t n,
                      void* out, int out_dtype, void* stream);

/*
 * Several tensors dequantised by ONE launch (Algorithm 1 per tensor, exactly as
 * nf4_dequantize / nf4_dequantize_dq compute it): e.g. the projections of a
 * decoder layer.  One launch fills and drains the load -> store pipeline once:
 * on MI355X tensors of a few MB take about 1 us less each this way (3.5 us
 * instead of 4.4 us for 8192 x 1024); tensors of hundreds of MB gain nothing.
 * tensors : HOST array of `count` descriptors (read during the call; the device
 *           pointers in it follow the conventions above), 0 <= count <=
 *           NF4_BATCH_MAX (else NF4_ERR_SIZE).  A descriptor with absmax != NULL
 *           is a tensor with FP32 scales (the other scale pointers are ignored);
 *           with absmax == NULL it has double-quantised scales and needs
 *           absmax_q8, scale2, offset and code2.  All tensors of a call must be of
 *           the same kind (else NF4_ERR_SHAPE) and share blocksize and out_dtype.
 *           A descriptor with n == 0 is skipped.  Outputs must not overlap.
 */
#define NF4_BATCH_MAX 8
typedef struct {
    const uint8_t* packed;     /* uint8[ceil(n/2)] */
    const float* absmax;       /* float[nb], or NULL for double-quantised scales */
    const uint8_t* absmax_q8;  /* uint8[nb] */
    const float* scale2;       /* float[ceil(nb/256)] */
    const float* offset;       /* float[1] */
    const float* code2;        /* float[256] */
    void* out;                 /* uint16[n] */
    int64_t n;
} nf4_tensor;
int nf4_dequantize_batch(const nf4_tensor* tensors, int count, int blocksize, int out_dtype,
                         void* stream);

/*
 * Fused dequantise + decode GEMV (not in the paper, which dequantises into a
 * temporary before a dense matmul, Sec. III-C; here W is never materialised):
 *   y[b][r] = rne_fp16( sum_k x[b][k] * W[r][k] ),
 *   W[r][k] = level[code(r*K + k)] * scale((r*K + k) / blocksize)   (FP32),
 * FP32 accumulation, W is [N][K] row-major with double-quantised scales as in
 * nf4_dequantize_dq.  x : FP16 [B][K], y : FP16 [B][N], 1 <= B <= 16, K > 0
 * and K % blocksize == 0 (else NF4_ERR_SHAPE).  packed and x must be 16-byte
 * aligned.  For one and two tokens W stays the FP32 product (vector-ALU FMAs);
 * so it does for three and four when N >= 16384 and K < 4096.  Otherwise the
 * sum runs on the matrix cores (three and four tokens with K >= 4096: the
 * 4 x 4 x 4 instruction, one column piece per lane; else 16-row tiles): every
 * level enters them as two FP16 terms (the level to about 2^-22 relative), the
 * products of a quantisation block are summed unscaled in FP32 and the block's
 * FP32 scale multiplies that sum, so W is carried to about 22 significant bits
 * whatever its magnitude.
 */
int nf4_dequant_gemv(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                     const float* offset, const float* code2, int blocksize, int64_t N,
                     int64_t K, const void* x, int B, void* y, void* stream);

/*
 * nf4_dequant_gemv with a workspace (device, 16-byte aligned, owned by the
 * caller, contents undefined before and after; at least
 * nf4_dequant_gemv_workspace_bytes(N, K, B) bytes, else NF4_ERR_SIZE; NULL is
 * NF4_ERR_NULL).  Same definition of y, same arguments, layouts and limits.
 * One and two tokens run as in nf4_dequant_gemv, and so do three and four
 * when K >= 4096 (the workspace is not touched).  From 5 tokens on (from 3
 * when K < 4096), K is split across
 * workgroups that share the activations through LDS; FP32 partial sums go to
 * the workspace and a second kernel adds them in a fixed order
 * (deterministic).  W is carried as on the matrix-core path above (levels as
 * two FP16 terms, FP32 block scales).  About 42 us for 5 to 16 tokens on the
 * 70B MLP shapes, where nf4_dequant_gemv takes 55 to 70.
 * Calls that share a workspace must not overlap.
 */
int nf4_dequant_gemv_ws(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                        const float* offset, const float* code2, int blocksize, int64_t N,
                        int64_t K, const void* x, int B, void* y, void* workspace,
                        size_t workspace_bytes, void* stream);

/* Bytes of workspace nf4_dequant_gemv_ws needs for this shape on the current
 * device (0 for shapes it rejects). */
size_t nf4_dequant_gemv_workspace_bytes(int64_t N, int64_t K, int B);

/*
 * nf4_dequant_gemv_ws for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * definition of y, same arguments, layouts, limits and results as
 * nf4_dequant_gemv_ws (bit for bit), without the workspace: the FP32 partial
 * sums go to a device array of NF4_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (every GPU the library runs on holds its own copy until
 * the process ends).  The call allocates and frees nothing.  A shape whose
 * partial sums do not fit (nf4_dequant_gemv_workspace_bytes(N, K, B) >
 * NF4_STATIC_SCRATCH_BYTES) returns NF4_ERR_SIZE and launches nothing; K is
 * split at most as many ways as fill the compute units once, so on a GPU with up
 * to 256 of them (MI355X) every shape the call accepts needs at most 256 * 256
 * rows x 16 tokens x 4 bytes = 4 MiB and fits.  All
 * calls on one GPU share that GPU's array: calls that may overlap on one GPU
 * (different streams, different threads) race and must be serialised by the
 * caller.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that call outside a graph capture.
 */
#define NF4_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
int nf4_dequant_gemv_static(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                            const float* offset, const float* code2, int blocksize, int64_t N,
                            int64_t K, const void* x, int B, void* y, void* stream);

/*
 * Fused dequantise + small-batch GEMM on the matrix cores, for the paper's batch
 * range (Sec. VI-A: 2 to 64).  It is the paper's quantised matmul (Sec. III-A,
 * III-C: dequantise W to FP16, then an FP16 matmul with FP32 accumulation)
 * without the FP16 copy of W in memory:
 *   y[b][r] = rne_fp16( sum_k x[b][k] * W16[r][k] ),
 *   W16[r][k] = rne_fp16( level[code(r*K + k)] * scale((r*K + k) / blocksize) ),
 * the exact product narrowed in one rounding.  (nf4_dequantize_dq rounds the
 * product to FP32 first; its FP16 result differs from W16 by one FP16 ulp where
 * that FP32 value lies exactly between two FP16 values, about 1 weight in 10^4
 * to 10^5.)
 * Same arguments and layouts as nf4_dequant_gemv; 1 <= B <= 64, K > 0 and
 * K % blocksize == 0 (else NF4_ERR_SHAPE).  packed and x 16-byte aligned.
 *
 * workspace (device, 16-byte aligned, owned by the caller, contents undefined
 * before and after) selects the algorithm:
 *   NULL     : one kernel; every workgroup sums over all of K and re-reads x
 *              from L2 (workspace_bytes is ignored);
 *   non-NULL : K is split across workgroups that share x through LDS; FP32
 *              partial sums go to the workspace and a second kernel adds them in
 *              a fixed order.  Faster from about 16 tokens on.  workspace_bytes
 *              must be at least nf4_dequant_gemm_workspace_bytes(N, K, B), else
 *              NF4_ERR_SIZE.  Calls that share a workspace must not overlap.
 * Both give the sum above with FP32 accumulation; the order of the additions
 * differs, each is deterministic.
 */
int nf4_dequant_gemm(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                     const float* offset, const float* code2, int blocksize, int64_t N,
                     int64_t K, const void* x, int B, void* y, void* workspace,
                     size_t workspace_bytes, void* stream);

/* Bytes of workspace the split-K path of nf4_dequant_gemm needs for this shape
 * on the current device (0 for shapes nf4_dequant_gemm rejects). */
size_t nf4_dequant_gemm_workspace_bytes(int64_t N, int64_t K, int B);

/*
 * The same format with the data type as a parameter (Sec. V-A names it as one of
 * the kernel's parameters): `codebook` is any 16 FP32 levels indexed by the 4-bit
 * code (device, 4-byte aligned; NULL = the NF4 levels), `dq_group` the number of
 * quantisation blocks per second-level scale (a power of two in [1, 65536], else
 * NF4_ERR_SHAPE; scale2 then holds ceil(nb / dq_group) floats).  Everything else
 * as in nf4_dequantize / nf4_dequantize_dq, which are these calls with NULL and
 * 256.  out[i] = rne16(codebook[code_i] * scale(i / blocksize)).
 */
int nf4_dequantize_codebook(const uint8_t* packed, const float* absmax, const float* codebook,
                            int blocksize, int64_t n, void* out, int out_dtype, void* stream);
int nf4_dequantize_dq_codebook(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                               const float* offset, const float* code2, int dq_group,
                               const float* codebook, int blocksize, int64_t n, void* out,
                               int out_dtype, void* stream);

/*
 * The fused products with the data type as a parameter (Sec. V-A), for tensors
 * made by nf4_quantize_ref_codebook / nf4_dq_encode with another table or group
 * size: nf4_dequant_gemv / nf4_dequant_gemv_ws and nf4_dequant_gemm with
 * `codebook` (16 FP32 levels, device, 4-byte aligned; NULL = the NF4 levels) and
 * `dq_group` (blocks per second-level scale, a power of two in [1, 65536], else
 * NF4_ERR_SHAPE) as in nf4_dequantize_dq_codebook.  Everything else -- the
 * definition of y, layouts, limits, the kernels chosen -- is that of the calls
 * without these two arguments, which are these calls with NULL and 256 and
 * accept no other format.  workspace == NULL selects the form without a
 * workspace (nf4_dequant_gemv; the single kernel of nf4_dequant_gemm), a
 * workspace of nf4_dequant_gemv_workspace_bytes / nf4_dequant_gemm_workspace_bytes
 * the form with one.
 */
int nf4_dequant_gemv_codebook(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                              const float* offset, const float* code2, int dq_group,
                              const float* codebook, int blocksize, int64_t N, int64_t K,
                              const void* x, int B, void* y, void* workspace, size_t workspace_bytes,
                              void* stream);
int nf4_dequant_gemm_codebook(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                              const float* offset, const float* code2, int dq_group,
                              const float* codebook, int blocksize, int64_t N, int64_t K,
                              const void* x, int B, void* y, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Reference-quality (untuned) quantiser, the forward direction of Sec. II-B:
 * per block absmax = max |src|, code = nearest level to src / absmax (FP32
 * distance, ties to the lower index, all-zero block -> absmax 0 and code 7,
 * unused last low nibble -> 7).  Writes packed[ceil(n/2)] and absmax[nb].
 * If absmax_q8 != NULL it also double-quantises the scales: code2[u] = (u -
 * 127)/127, offset = mean(absmax), scale2[g] = max |absmax - offset| over the
 * group, absmax_q8 = 127 + clamp(rint(127 * (absmax - offset) / scale2), -127,
 * 127); then scale2, offset and code2 must be non-NULL too.  absmax is always
 * required (it is the first-level result the second level encodes).
 */
int nf4_quantize_ref(const float* src, int64_t n, int blocksize, uint8_t* packed, float* absmax,
                     uint8_t* absmax_q8, float* scale2, float* offset, float* code2,
                     void* stream);

/*
 * nf4_quantize_ref for any codebook and second-level group size (see
 * nf4_dequantize_codebook for both arguments).  Nearest level = smallest
 * |x / absmax - codebook[k]| in FP32, codes scanned from 0 upward, a tie keeps the
 * lower code; an all-zero block and the unused nibble of an odd n take the code
 * nearest to 0.  dq_group is only read when absmax_q8 != NULL.
 */
int nf4_quantize_ref_codebook(const float* src, int64_t n, int blocksize, const float* codebook,
                              int dq_group, uint8_t* packed, float* absmax, uint8_t* absmax_q8,
                              float* scale2, float* offset, float* code2, void* stream);

/*
 * Tuned quantiser, first level only (Sec. II-B, forward direction): writes
 * exactly the packed[] and absmax[] that nf4_quantize_ref writes, bit for bit,
 * at HBM speed for every block size and any n (the tile that n does not fill is
 * handled by predication inside the same kernel).  src must be 16-byte aligned,
 * packed 2-byte aligned.  The first call on a process builds a 512-byte table
 * on the host (no device allocation).
 */
int nf4_quantize(const float* src, int64_t n, int blocksize, uint8_t* packed, float* absmax,
                 void* stream);

/*
 * nf4_quantize for any 16 levels (Sec. V-A: the data type as a parameter):
 * writes exactly the packed[] and absmax[] that nf4_quantize_ref_codebook
 * writes for `codebook` (float[16], device; NULL = NF4, then nf4_quantize), bit
 * for bit.  The decision thresholds of the levels are found on the device by
 * a one-workgroup kernel ahead of the quantiser, into `workspace` (device,
 * 8-byte aligned, at least NF4_QUANTIZE_CODEBOOK_WORKSPACE_BYTES, else
 * NF4_ERR_SIZE; owned by the caller, contents undefined before and after;
 * calls that share it must not overlap).  The levels may be in any order and
 * repeat (FP4-style tables in sign-magnitude order with +0 and -0).  Tables
 * whose levels are finite, whose distinct values are at least 2^-10 and 2^-12
 * of their magnitude apart, and of whose decision thresholds none lies within
 * 2^-30 of zero and no two fall into one interval of 1/32 (NF4, E2M1, evenly
 * spaced levels, any sensible 4-bit type) run at the speed
 * of nf4_quantize; any other table is quantised by the
 * reference kernel inside the same call, with the same results.  The call
 * never waits for the GPU.
 */
#define NF4_QUANTIZE_CODEBOOK_WORKSPACE_BYTES ((size_t)1024)
int nf4_quantize_codebook(const float* src, int64_t n, int blocksize, const float* codebook,
                          uint8_t* packed, float* absmax, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * The second level alone: double-quantises an existing array of nb block scales
 * (e.g. nf4_quantize's absmax) exactly as nf4_quantize_ref_codebook does, bit for
 * bit: code2[u] = (u - 127)/127, offset = mean(absmax) (the double-precision sum
 * in index order), scale2[g] = max |absmax - offset| over each group of dq_group
 * blocks (a power of two in [1, 65536], else NF4_ERR_SHAPE), absmax_q8 = 127 +
 * clamp(rint(127 * (absmax - offset) / scale2), -127, 127).  Writes
 * absmax_q8[nb], scale2[ceil(nb / dq_group)], offset[1], code2[256]; absmax is
 * only read.
 */
int nf4_dq_encode(const float* absmax, int64_t nb, int dq_group, uint8_t* absmax_q8, float* scale2,
                  float* offset, float* code2, void* stream);

/* hipError_t (as int) behind the most recent NF4_ERR_HIP on the calling thread; 0 if none. */
int nf4_last_hip_error(void);

/* Static, NUL-terminated name of a status code ("NF4_OK", ...); "NF4_ERR_UNKNOWN" otherwise. */
const char* nf4_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* NF4_H */
