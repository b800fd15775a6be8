// nf4_dequant_gemv_static: nf4_dequant_gemv_ws for callers that cannot allocate (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc).  The FP32 partial sums of the split-K kernel go to a
// file-scope device array instead of a caller workspace.  Nothing here calls hipMalloc, hipFree or any
// allocating routine; the array is part of the library's code object and each GPU the library runs on holds
// its own copy until the process ends.
//
// In host code the array's name is only a handle for the symbol, never a device address: the address is asked
// for once per device (with that device current) through hipGetSymbolAddress and only that pointer is handed
// to the kernels.
#include <atomic>
#include <mutex>

#include "nf4_device.hpp"
#include "nf4_host.hpp"

namespace nf4 {

// 4 MiB.  plan_split cuts K into at most (compute units / blocks of 256 rows) pieces, so splits * N <= 256 *
// compute units and 16 tokens of FP32 partial sums need at most 4 MiB on a 256-CU part (8192 x 28672, 16 tokens:
// 8 splits, exactly 4 MiB; 28672 x 8192: 2 splits, 3.5 MiB).  A device with more compute units can ask for more
// and is then refused by the size check below.
constexpr size_t kStaticScratchBytes = NF4_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<float*> g_scratch_ptr[kMaxDevices];   // per device: address of that device's copy of `scratch`
static std::mutex g_scratch_mutex;

// Address of the current device's scratch array (nullptr and an nf4_status in *rc on failure).
static float* scratch_of_current_device(int* rc) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { *rc = record_hip(e); return nullptr; }
    if (dev < 0 || dev >= kMaxDevices) { *rc = NF4_ERR_SIZE; return nullptr; }
    float* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void* addr = nullptr;
    e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || addr == nullptr) { *rc = record_hip(e != hipSuccess ? e : hipErrorInvalidSymbol); return nullptr; }
    p = (float*)addr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

}  // namespace nf4

extern "C" int nf4_dequant_gemv_static(const uint8_t* packed, const uint8_t* absmax_q8, const float* scale2,
                                       const float* offset, const float* code2, int blocksize, int64_t N, int64_t K,
                                       const void* x, int B, void* y, void* stream) {
    using namespace nf4;
    if (N < 0 || K < 0) return NF4_ERR_SIZE;
    const int log2_bs = log2_blocksize(blocksize);
    if (log2_bs < 0) return NF4_ERR_BLOCKSIZE;
    if (B < 1 || B > 16) return NF4_ERR_SHAPE;
    if (N > 0 && (K <= 0 || K % blocksize != 0)) return NF4_ERR_SHAPE;
    if (N > 0x7fffffffLL) return NF4_ERR_SIZE;
    if (N == 0) return NF4_OK;
    if (!packed || !absmax_q8 || !scale2 || !offset || !code2 || !x || !y) return NF4_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(x, 16) || !aligned(y, 2) || !aligned(scale2, 4) || !aligned(offset, 4) ||
        !aligned(code2, 4))
        return NF4_ERR_ALIGN;
    // the partial sums of this shape must fit the array: splits * B * N floats
    if (nf4_dequant_gemv_workspace_bytes(N, K, B) > kStaticScratchBytes) return NF4_ERR_SIZE;
    int rc = NF4_OK;
    float* partial = scratch_of_current_device(&rc);
    if (!partial) return rc;
    // Every partial sum that the second kernel reads is written by the first one in the same call, so what the
    // previous call left in the array does not matter and nothing has to be cleared.
    return launch_gemv_ws(packed, absmax_q8, scale2, offset, code2, log2_bs, kNf4Fmt, N, K, (const _Float16*)x, B,
                          (_Float16*)y, partial, (hipStream_t)stream);
}
