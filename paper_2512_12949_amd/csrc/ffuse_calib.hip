// Calibration probes: what this device sustains on the two resources the fused chain is priced
// against -- the matrix cores and the memory system's read path.  The traffic model (Sec. 4.4:
// every level priced with its bandwidth) holds calibrated rates; these probes re-measure them on the
// device at hand, so that a benchmark can state its result against the published peak and against
// what an ideal loop reaches under the same power limit.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "../../include/ffuse.h"
#include "ffuse_dev.h"

namespace ffuse {

// Every wave issues `iters` rounds of four independent 32x32x16 products (no memory access at all):
// the upper bound of any kernel's matrix rate.  Operands are pseudo-random values of magnitude
// 0.5..1 so that the data paths toggle as they do on real data (a loop over zeros draws less power
// and clocks higher than anything useful).
template <typename T> __global__ __launch_bounds__(256) void mfma_issue_kernel(float* out, int iters, int zeros) {
    typedef typename Mma<T>::vec8 vec8;
    union { vec8 v; uint16_t h[8]; } a, b;
    uint32_t s = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    for (int i = 0; i < 8; ++i) {
        s = s * 1664525u + 1013904223u;
        // sign and mantissa random, exponent of 0.5..1 in either 16-bit format
        const uint16_t top = sizeof(T) == 2 && __is_same(T, __bf16) ? 0x3F00 : 0x3800;
        const uint16_t mant = __is_same(T, __bf16) ? 0x007F : 0x03FF;
        a.h[i] = (uint16_t)(top | ((s >> 8) & mant) | ((s >> 16) & 0x8000));
        b.h[i] = (uint16_t)(top | ((s >> 3) & mant) | ((s >> 11) & 0x8000));
        if (zeros) a.h[i] = b.h[i] = 0;     // nothing toggles: what the issue logic alone allows
    }
    f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
        c0 = Mma<T>::mma(a.v, b.v, c0);
        c1 = Mma<T>::mma(b.v, a.v, c1);
        c2 = Mma<T>::mma(a.v, a.v, c2);
        c3 = Mma<T>::mma(b.v, b.v, c3);
    }
    float sum = 0.f;
    for (int i = 0; i < 16; ++i) sum += c0[i] + c1[i] + c2[i] + c3[i];
    if (sum == 0.123456789f) out[threadIdx.x] = sum;   // never true in practice: keeps the loop alive
}

// A plain streaming read: every workgroup walks a contiguous share of the buffer, 32 KB per step
// (eight 16-byte loads in flight per lane), as the library's weight-streaming loops do.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, uint64_t n16, uint32_t* out) {
    const uint64_t share = ((n16 + gridDim.x - 1) / gridDim.x + 2047) / 2048 * 2048;   // whole steps of 256 lanes x 8
    const uint64_t lo = (uint64_t)blockIdx.x * share;
    const uint64_t hi = lo + share < n16 ? lo + share : n16;
    u32x4 acc = {0, 0, 0, 0};
    for (uint64_t base = lo; base < hi; base += 2048) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint64_t i = base + (uint64_t)j * 256 + threadIdx.x;
            v[j] = i < hi ? src[i] : acc;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) out[threadIdx.x] = acc[0];   // keeps the loads alive
}

}  // namespace ffuse

extern "C" int ffuse_calibrate(int what, int dtype, const void* buf, int64_t bytes, int64_t iters, void* scratch16k,
                               double* result, void* stream) {
    if (!result || !scratch16k) return FFUSE_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return FFUSE_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return FFUSE_ERR_LAUNCH;
    const int cus = prop.multiProcessorCount;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FFUSE_ERR_LAUNCH;
    int rc = FFUSE_OK;
    double work = 0.0;   // flop or bytes of the timed launch
    (void)hipGetLastError();
    if (what == FFUSE_CAL_MFMA || what == FFUSE_CAL_MFMA_IDLE) {
        if (dtype != FFUSE_DT_BF16 && dtype != FFUSE_DT_F16) rc = FFUSE_ERR_ACT;
        const int grid = cus * 2;   // two workgroups of four waves per CU: two waves per SIMD
        for (int rep = 0; rep < 2 && rc == FFUSE_OK; ++rep) {   // the first launch warms up, the second is timed
            if (rep) (void)hipEventRecord(e0, st);
            if (dtype == FFUSE_DT_BF16)
                ffuse::mfma_issue_kernel<__bf16><<<grid, 256, 0, st>>>(static_cast<float*>(scratch16k), (int)iters, what == FFUSE_CAL_MFMA_IDLE);
            else
                ffuse::mfma_issue_kernel<_Float16><<<grid, 256, 0, st>>>(static_cast<float*>(scratch16k), (int)iters, what == FFUSE_CAL_MFMA_IDLE);
            if (rep) (void)hipEventRecord(e1, st);
        }
        work = (double)grid * 4 /*waves*/ * (double)iters * 4 /*products*/ * (2.0 * 32 * 32 * 16);
    } else if (what == FFUSE_CAL_READ) {
        if (!buf) rc = FFUSE_ERR_NULL;
        else if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0) rc = FFUSE_ERR_ALIGN;
        else if (bytes < 16 || (bytes & 15) != 0) rc = FFUSE_ERR_SHAPE;
        const int grid = cus * 8;
        for (int64_t rep = 0; rep <= iters && rc == FFUSE_OK; ++rep) {   // one warm-up pass, `iters` timed passes
            if (rep == 1) (void)hipEventRecord(e0, st);
            ffuse::stream_read_kernel<<<grid, 256, 0, st>>>(static_cast<const ffuse::u32x4*>(buf), (uint64_t)bytes / 16,
                                                           static_cast<uint32_t*>(scratch16k));
        }
        if (rc == FFUSE_OK) (void)hipEventRecord(e1, st);
        work = (double)bytes * (double)iters;
    } else {
        rc = FFUSE_ERR_ACT;
    }
    if (rc == FFUSE_OK) {
        float ms = 0.f;
        if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
            rc = FFUSE_ERR_LAUNCH;
        else
            *result = work / (ms * 1e-3);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
