// The device workspace of star_group_update_noalloc: a fixed array in the library's device code
// instead of memory from hipMalloc, for callers that cannot allocate (code under HIP graph capture,
// tight serving loops, harnesses that forbid it), and the two small kernels that fill it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>

#include "star_kernels.h"

namespace star {

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels get the
// resolved address as an argument.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 16;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Host data travels in the kernel arguments, kUploadBytes at a time (the argument block of a launch
// holds 4 KB).
constexpr int kUploadBytes = 3584;
struct UploadBlock {
    uint32_t w[kUploadBytes / 4];
};

__global__ __launch_bounds__(kBlock) void upload_kernel(const UploadBlock blk, uint32_t* __restrict__ dst,
                                                        const int nwords) {
    for (int i = threadIdx.x; i < nwords; i += kBlock) dst[i] = blk.w[i];
}

__global__ void queue_clear_kernel(TileQueue* __restrict__ q) {
    if (threadIdx.x == 0) {
        q->next = 0ull;
        q->done = 0u;
        q->pad = 0u;
    }
}

}  // namespace

hipError_t scratch_address(void** out) {
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // the current device's copy
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

hipError_t launch_upload(void* dst_dev, const void* src_host, size_t bytes, hipStream_t s) {
    const unsigned char* src = static_cast<const unsigned char*>(src_host);
    unsigned char* dst = static_cast<unsigned char*>(dst_dev);
    for (size_t off = 0; off < bytes; off += kUploadBytes) {
        const size_t n = std::min<size_t>(kUploadBytes, bytes - off);
        UploadBlock blk;
        std::memset(&blk, 0, sizeof blk);
        std::memcpy(blk.w, src + off, n);
        hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(kBlock), 0, s, blk, reinterpret_cast<uint32_t*>(dst + off),
                           (int)((n + 3) / 4));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_queue_clear(TileQueue* q, hipStream_t s) {
    hipLaunchKernelGGL(queue_clear_kernel, dim3(1), dim3(64), 0, s, q);
    return hipGetLastError();
}

}  // namespace star
