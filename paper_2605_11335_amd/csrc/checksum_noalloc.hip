// Streamed-bytes checksum for callers that may not allocate (code under graph capture, serving
// loops, harnesses that forbid hipMalloc): same definition as cf_op_checksum, but the only device
// memory beyond the caller's input and output is a fixed array that lives in this library's image.
//
// Two kernels: every workgroup reduces its CS_WG_WORDS 64-bit words to one partial sum in the
// array, then one workgroup adds the partial sums and stores the result.  Sums are modulo 2^64, so
// the order of additions does not matter and the result equals cf_op_checksum's bit for bit.
#include <mutex>

#include "context.h"

namespace {

constexpr int CS_WG_WORDS = 4096;          // words per workgroup: 256 lanes x 16
constexpr int CS_MAX_PARTIALS = 32768;     // one partial sum per workgroup: 256 KiB of device memory
constexpr uint64_t CS_MAX_BYTES = (uint64_t)CS_MAX_PARTIALS * CS_WG_WORDS * 8;   // 1 GiB per call

// Partial sums.  Each GPU the library runs on holds its own copy until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device (scratch_of_current_device) and kernels receive that pointer as an argument.
static __device__ __align__(256) unsigned long long scratch[CS_MAX_PARTIALS];

constexpr int CS_MAX_DEVICES = 64;
std::mutex g_mu;
unsigned long long* g_scratch_ptr[CS_MAX_DEVICES] = {};

hipError_t scratch_of_current_device(unsigned long long** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= CS_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = (unsigned long long*)p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t acc) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)acc, o), hi = __shfl_xor((uint32_t)(acc >> 32), o);
        acc += ((uint64_t)hi << 32) | lo;
    }
    return acc;
}

// workgroup sum of the four waves' totals; valid in thread 0
__device__ __forceinline__ uint64_t block_sum_u64(uint64_t acc) {
    __shared__ unsigned long long part[4];
    acc = wave_sum_u64(acc);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    return part[0] + part[1] + part[2] + part[3];
}

// workgroup b: words [b * CS_WG_WORDS, min(n_words, (b + 1) * CS_WG_WORDS)) -> partials[b]
__global__ __launch_bounds__(256) void checksum_partial_kernel(const uint64_t* __restrict__ w, uint64_t n_words,
                                                               uint64_t first_word, unsigned long long* __restrict__ partials) {
    const uint64_t base = (uint64_t)blockIdx.x * CS_WG_WORDS;
    uint64_t acc = 0;
#pragma unroll 4
    for (int j = 0; j < CS_WG_WORDS / 256; ++j) {
        const uint64_t i = base + (uint64_t)j * 256 + threadIdx.x;
        if (i < n_words) acc += cf_mix64(w[i] ^ ((first_word + i + 1) * CF_GOLDEN64));
    }
    const uint64_t total = block_sum_u64(acc);
    if (threadIdx.x == 0) partials[blockIdx.x] = total;
}

// one workgroup: out = sum of partials[0 .. n) (0 for n = 0); reads nothing beyond n, so what an
// earlier, larger call left further up in the array is never seen
__global__ __launch_bounds__(256) void checksum_finish_kernel(const unsigned long long* __restrict__ partials, int n,
                                                              unsigned long long* __restrict__ out) {
    uint64_t acc = 0;
    for (int i = threadIdx.x; i < n; i += 256) acc += partials[i];
    const uint64_t total = block_sum_u64(acc);
    if (threadIdx.x == 0) *out = total;
}

}  // namespace

extern "C" int cf_op_checksum_noalloc(const void* data, uint64_t bytes, uint64_t first_word, uint64_t* dev_out, void* stream) {
    if (!dev_out || (!data && bytes)) return cf_fail(nullptr, CF_ERR_ARG, "checksum_noalloc: null operand");
    if (bytes % 8 || ((uintptr_t)data % 8) || ((uintptr_t)dev_out % 8))
        return cf_fail(nullptr, CF_ERR_ARG, "checksum_noalloc: data, dev_out and the byte count must be 8-byte aligned");
    if (bytes > CS_MAX_BYTES)
        return cf_fail(nullptr, CF_ERR_ARG, "checksum_noalloc: %llu bytes exceed the %llu a call can cover (fixed partial-sum array)",
                       (unsigned long long)bytes, (unsigned long long)CS_MAX_BYTES);
    unsigned long long* partials = nullptr;
    hipError_t e = scratch_of_current_device(&partials);
    if (e != hipSuccess) return cf_fail(nullptr, CF_ERR_HIP, "checksum_noalloc: scratch lookup failed: %s", hipGetErrorString(e));
    const uint64_t n_words = bytes / 8;
    const int n_wg = (int)((n_words + CS_WG_WORDS - 1) / CS_WG_WORDS);        // <= CS_MAX_PARTIALS by the check above
    hipStream_t s = (hipStream_t)stream;
    if (n_wg)
        hipLaunchKernelGGL(checksum_partial_kernel, dim3(n_wg), dim3(256), 0, s, (const uint64_t*)data, n_words, first_word, partials);
    hipLaunchKernelGGL(checksum_finish_kernel, dim3(1), dim3(256), 0, s, partials, n_wg, (unsigned long long*)dev_out);
    e = hipGetLastError();
    return e == hipSuccess ? CF_OK : cf_fail(nullptr, CF_ERR_HIP, "checksum_noalloc launch: %s", hipGetErrorString(e));
}
