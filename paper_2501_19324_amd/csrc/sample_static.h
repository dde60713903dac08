// rsd_sample_static: the sampler of sample.h behind an entry point that allocates nothing.
// Included by rsd.hip (one translation unit: the kernels of sample.h are defined there).
#pragma once
#include <mutex>
#include "rsd.h"
#include "sample.h"

// The sampler for callers that cannot allocate: its workspace is a file-scope device array instead of
// the context's buffers.  Every device holds its own copy of the array at its own address; host code
// never uses the array's name as a pointer, only the address looked up once per device.
namespace {

constexpr size_t kSmpHist = (size_t)RSD_SAMPLE_STATIC_MAX_ROWS * 3 * SMP_BINS;      // u64 each
constexpr size_t kSmpPsum = (size_t)RSD_SAMPLE_STATIC_MAX_ROWS * SMP_NB;            // u64
constexpr size_t kSmpSel = (size_t)RSD_SAMPLE_STATIC_MAX_ROWS * 8;                  // u64
constexpr size_t kSmpPmax = (size_t)RSD_SAMPLE_STATIC_MAX_ROWS * SMP_NB;            // float
constexpr size_t kSmpPidx = (size_t)RSD_SAMPLE_STATIC_MAX_ROWS * SMP_NB;            // int
constexpr size_t kSmpScratchBytes = (kSmpHist + kSmpPsum + kSmpSel) * sizeof(u64_t) + kSmpPmax * sizeof(float) + kSmpPidx * sizeof(int);

static __device__ __align__(256) unsigned char scratch[kSmpScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void* scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each device, looked up on first use

// the device address of the array on the current device (nullptr + error code on failure)
hipError_t scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int rsd_sample_static(const float* logits_dev, const float* u_dev, int32_t n, int32_t vocab, float temperature,
                                 float top_p, int32_t* out_dev, void* hip_stream) {
    if (!logits_dev || !out_dev || n < 1 || vocab < 1) return RSD_EINVAL;
    if (n > RSD_SAMPLE_STATIC_MAX_ROWS) return RSD_EINVAL;                 // beyond the static workspace
    if (temperature > 0.f && !u_dev) return RSD_EINVAL;
    if (temperature < 0.f || top_p < 0.f || top_p > 1.f) return RSD_EINVAL;
    void* base = nullptr;
    if (scratch_address(&base) != hipSuccess) return RSD_EHIP;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    u64_t* hist = static_cast<u64_t*>(base);
    u64_t* psum = hist + kSmpHist;
    u64_t* sel = psum + kSmpPsum;
    float* pmax = reinterpret_cast<float*>(sel + kSmpSel);
    int* pidx = reinterpret_cast<int*>(pmax + kSmpPmax);
    // the array keeps what the last call left: histograms and selections of the rows in use start at zero
    // (a fill kernel, not a memset node: the caller may be recording a graph)
    const size_t nh = (size_t)n * 3 * SMP_BINS * 2, ns = (size_t)n * 8 * 2;       // as ints
    hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((nh + 255) / 256)), dim3(256), 0, st, reinterpret_cast<int*>(hist), 0, nh);
    hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((ns + 255) / 256)), dim3(256), 0, st, reinterpret_cast<int*>(sel), 0, ns);
    SampleArgs a{logits_dev, vocab, vocab, u_dev, nullptr, 1, temperature, top_p, -1, 0.f, nullptr, out_dev,
                 pmax, pidx, hist, psum, sel};
    sample_launch(st, a, AppendArgs{}, n);
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_EHIP;
}
