// fp32 debug path: the same chain on plain FMA (no matrix cores), for checking the schedule
// and the boundary at full precision.  Same "reduce" structure as the 16-bit fused kernel:
// one workgroup per (16-row block, 64-wide hidden slice), complete K sums before the
// activation (paper Sec. 4.3, Rule 3), partial second products added atomically into Y.
#include "ffuse_dev.h"
#include "ffuse_launch.h"
#include <mutex>
#include <unordered_map>

#include <cstdlib>

namespace ffuse {

static __device__ __forceinline__ float act_f32(int act, float x) {
    switch (act) {
        case ACT_RELU: return fmaxf(x, 0.0f);
        case ACT_GELU_TANH: {
            const float z = 0.7978845608028654f * (x + 0.044715f * x * x * x);
            return 0.5f * x * (1.0f + tanhf(z));
        }
        case ACT_SILU: return x / (1.0f + expf(-x));
        default: return x;
    }
}

constexpr int F_BM = 16, F_BH = 64, F_BK = 32;

// H block [16][64] of act(X W1) [.* X W3] for rows m0.., hidden n0.. into hs (LDS).
static __device__ __forceinline__ void first_product_f32(const float* X, const float* W1, const float* W3,
                                                         int64_t M, int K, int N1, int act, int64_t m0, int n0,
                                                         float (*xs)[F_BK + 1], float (*ws)[F_BH], float (*w3s)[F_BH],
                                                         float (*hs)[F_BH + 1]) {
    const int tid = threadIdx.x;
    const int c = tid & 63, r0 = tid >> 6;  // column, first of 4 rows (r0, r0+4, r0+8, r0+12)
    float g[4] = {0, 0, 0, 0}, u[4] = {0, 0, 0, 0};
    for (int k0 = 0; k0 < K; k0 += F_BK) {
        for (int i = tid; i < F_BM * F_BK; i += 256) {
            const int r = i / F_BK, k = i % F_BK;
            xs[r][k] = (m0 + r < M && k0 + k < K) ? X[(m0 + r) * K + k0 + k] : 0.0f;
        }
        for (int i = tid; i < F_BK * F_BH; i += 256) {
            const int k = i / F_BH, n = i % F_BH;
            const bool ok = (k0 + k < K) && (n0 + n < N1);
            ws[k][n] = ok ? W1[(int64_t)(k0 + k) * N1 + n0 + n] : 0.0f;
            if (W3) w3s[k][n] = ok ? W3[(int64_t)(k0 + k) * N1 + n0 + n] : 0.0f;
        }
        __syncthreads();
        for (int k = 0; k < F_BK; ++k) {
            const float w = ws[k][c];
            const float w3 = W3 ? w3s[k][c] : 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float xv = xs[r0 + 4 * q][k];
                g[q] = fmaf(xv, w, g[q]);
                u[q] = fmaf(xv, w3, u[q]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float v = act_f32(act, g[q]);
        if (W3) v *= u[q];
        hs[r0 + 4 * q][c] = v;
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void fused_f32_kernel(FusedArgs a, float* Y) {
    __shared__ float xs[F_BM][F_BK + 1];
    __shared__ float ws[F_BK][F_BH];
    __shared__ float w3s[F_BK][F_BH];
    __shared__ float hs[F_BM][F_BH + 1];
    const float* X = (const float*)a.X;
    const float* W1 = (const float*)a.W1;
    const float* W3 = (const float*)a.W3;
    const float* W2 = (const float*)a.W2;
    const int64_t m0 = (int64_t)blockIdx.x * F_BM;
    const int n0 = blockIdx.y * F_BH;
    first_product_f32(X, W1, W3, a.M, a.K, a.N1, a.act, m0, n0, xs, ws, w3s, hs);
    const int nvalid = min(F_BH, a.N1 - n0);
    for (int j = threadIdx.x; j < a.N2; j += 256) {
        float acc[F_BM];
#pragma unroll
        for (int r = 0; r < F_BM; ++r) acc[r] = 0.0f;
        for (int n = 0; n < nvalid; ++n) {
            const float w = W2[(int64_t)(n0 + n) * a.N2 + j];
#pragma unroll
            for (int r = 0; r < F_BM; ++r) acc[r] = fmaf(hs[r][n], w, acc[r]);
        }
#pragma unroll
        for (int r = 0; r < F_BM; ++r)
            if (m0 + r < a.M)
                __hip_atomic_fetch_add(Y + (m0 + r) * a.N2 + j, acc[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// C = act(A B) [.* A B3], fp32, 16 x 64 tile per workgroup
__global__ __launch_bounds__(256) void gemm_act_f32_kernel(GemmArgs a) {
    __shared__ float xs[F_BM][F_BK + 1];
    __shared__ float ws[F_BK][F_BH];
    __shared__ float w3s[F_BK][F_BH];
    __shared__ float hs[F_BM][F_BH + 1];
    const int64_t m0 = (int64_t)blockIdx.x * F_BM;
    const int n0 = blockIdx.y * F_BH;
    first_product_f32((const float*)a.A, (const float*)a.B, (const float*)a.B3, a.M, a.K, a.N, a.act, m0, n0, xs, ws,
                      w3s, hs);
    float* C = (float*)a.C;
    for (int i = threadIdx.x; i < F_BM * F_BH; i += 256) {
        const int r = i / F_BH, c = i % F_BH;
        if (m0 + r < a.M && n0 + c < a.N) C[(m0 + r) * a.N + n0 + c] = hs[r][c];
    }
}

__global__ __launch_bounds__(256) void zero_kernel(u32x4* p, size_t n16) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = z;
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t want = (n16 + 255) / 256;
    const int blocks = (int)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(zero_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<u32x4*>(p), n16);
    return hipGetLastError();
}

hipError_t launch_resident(const void* fn, int grid, void** params, hipStream_t st) {
    static const bool cooperative = getenv("FFUSE_COOPERATIVE_LAUNCH") != nullptr;
    if (cooperative) return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(256), params, 0, st);
    // how many workgroups of this kernel the device holds at once: asked once per kernel
    static std::mutex mu;
    static std::unordered_map<const void*, int> capacity;
    int cap = 0;
    {
        std::lock_guard<std::mutex> lock(mu);
        auto it = capacity.find(fn);
        if (it != capacity.end()) cap = it->second;
    }
    if (cap == 0) {
        int per_cu = 0, dev = 0, cus = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 256, 0);
        if (e != hipSuccess) return e;
        if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        cap = per_cu * cus;
        if (cap <= 0) return hipErrorCooperativeLaunchTooLarge;
        std::lock_guard<std::mutex> lock(mu);
        capacity[fn] = cap;
    }
    if (grid > cap) return hipErrorCooperativeLaunchTooLarge;
    return hipLaunchKernel(fn, dim3(grid), dim3(256), params, 0, st);
}

hipError_t launch_fused_f32(const FusedArgs& a, float* Y, hipStream_t st) {
    // N2 is a multiple of 8, so the output is a whole number of 16-byte units
    hipError_t e = launch_zero(Y, sizeof(float) * (size_t)a.M * a.N2, st);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((a.M + F_BM - 1) / F_BM), (unsigned)((a.N1 + F_BH - 1) / F_BH));
    hipLaunchKernelGGL(fused_f32_kernel, grid, dim3(256), 0, st, a, Y);
    return hipGetLastError();
}

hipError_t launch_gemm_act_f32(const GemmArgs& a, hipStream_t st) {
    dim3 grid((unsigned)((a.M + F_BM - 1) / F_BM), (unsigned)((a.N + F_BH - 1) / F_BH));
    hipLaunchKernelGGL(gemm_act_f32_kernel, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ffuse
