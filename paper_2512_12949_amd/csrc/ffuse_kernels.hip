// gfx950 kernels of the 16-bit paths:
//   * fused_reduce_kernel  -- the whole chain for one (row block, hidden slice) unit; the
//     activated slice never leaves registers; partial second products are summed across
//     hidden slices with fp32 atomics (paper Sec. 4.1: "reduce" strategy, with the hidden
//     split taking the place of the cluster's n dimension).
//   * finalize_kernel      -- fp32 sums -> Y in the operand type, workspace back to zero.
//   * gemm_act_kernel      -- plain GEMM with the activation/gate epilogue: the two launches of
//     the unfused comparison path.
#include "ffuse_gemm0.h"
#include "ffuse_launch.h"

namespace ffuse {

// blockIdx -> work unit, XCD aware.  Workgroups are dealt round-robin to the 8 XCDs, so
// blockIdx % 8 is the XCD and blockIdx / 8 the arrival order on it.  Each XCD gets one
// contiguous range of units ordered so that the ~32 units in flight on it form a patch of
// `raster` row blocks x consecutive hidden slices: the patch shares X row blocks and weight
// slices through that XCD's L2.
__device__ __forceinline__ bool map_unit(int MB, int S, int raster, int& i, int& s) {
    const int total = MB * S;
    const int per = (total + 7) / 8;
    const int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
    const int v = xcd * per + loc;
    if (loc >= per || v >= total) return false;
    const int panel = v / (raster * S);
    const int rem = v - panel * raster * S;
    const int rows = min(raster, MB - panel * raster);
    i = panel * raster + rem % rows;
    s = rem / rows;
    return true;
}

template <typename T> __device__ __forceinline__ float act_rt(int act, float x) {
    switch (act) {
        case ACT_RELU: return activate<ACT_RELU>(x);
        case ACT_GELU_TANH: return activate<ACT_GELU_TANH>(x);
        case ACT_SILU: return activate<ACT_SILU>(x);
        default: return x;
    }
}

// ---------------------------------------------------------------------------------------
// Fused chain, "reduce" family.
// ---------------------------------------------------------------------------------------
template <typename T, bool GATED, int BM, int BH>
__global__ __launch_bounds__(256) void fused_reduce_kernel(FusedArgs a) {
    typedef FirstGemm<T, GATED, BM, BH, 4, 1> G0;
    typedef typename Mma<T>::vec8 vec8;
    constexpr int MT = G0::MT, HT = G0::HT;
    constexpr int BN2 = 128, JT = BN2 / 32;
    constexpr int SUBS = (BH >= 128) ? 2 : 1;        // 64-deep W2 sub-tiles per stage
    constexpr int NST = BH / (64 * SUBS);            // stages per block of output columns
    constexpr int SUB_BYTES = BN2 * 128;
    constexpr int STAGE2 = SUBS * SUB_BYTES;
    constexpr int LDS_BYTES = (G0::LDS_BYTES > 2 * STAGE2) ? G0::LDS_BYTES : 2 * STAGE2;
    __shared__ __attribute__((aligned(16))) char smem[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int MB = (int)((a.M + BM - 1) / BM), S = (a.N1 + BH - 1) / BH;
    int ui, us;
    if (!map_unit(MB, S, a.raster, ui, us)) return;
    const int m0 = ui * BM, n0 = us * BH;

    // ---- first product, K complete ------------------------------------------------------
    f32x16 acc[HT][MT];
    f32x16 acc3[GATED ? HT : 1][GATED ? MT : 1];
    {
        typename G0::Ctx c;
        G0::init(c, a.X, a.W1, a.W3, a.M, a.K, a.N1, m0, n0, tid);
        G0::run(smem, c, acc, acc3, tid);
    }

    // ---- activation (and gate) on complete sums; round to the operand type.  Registers
    //      8b..8b+7 of a tile are the 8 k-slots this lane feeds to the second product for
    //      hidden block 16*(2*ht + b): slot e <-> hidden 32*ht + 16*b + 8*(e/4) + 4*(lane/32) + e%4.
    vec8 hreg[HT][MT][2];
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                u32x4 pk;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    float v0 = act_rt<T>(a.act, acc[ht][mt][8 * b + 2 * d]);
                    float v1 = act_rt<T>(a.act, acc[ht][mt][8 * b + 2 * d + 1]);
                    if (GATED) {
                        v0 *= acc3[ht][mt][8 * b + 2 * d];
                        v1 *= acc3[ht][mt][8 * b + 2 * d + 1];
                    }
                    pk[d] = pack2<T>(v0, v1);
                }
                hreg[ht][mt][b] = __builtin_bit_cast(vec8, pk);
            }

    // ---- second product: for every block of BN2 output columns, H (registers) times the
    //      W2 rows of this hidden slice, then fp32 atomic adds into the sums -------------
    const __amdgpu_buffer_rsrc_t rw2 = make_rsrc(a.W2, (uint32_t)((uint64_t)a.N1 * a.N2 * 2));
    const uint32_t w2row = (uint32_t)a.N2 * 2u;
    const int u = (SUBS == 2) ? (tid >> 7) : 0;      // sub-tile this thread loads
    const int tt = tid & 127;
    const bool loader = (SUBS == 2) || tid < 128;
    const int jg = tt & 15, ch = tt >> 4;            // 8 columns jg, k-chunk ch (0..7)
    // rows of the hidden slice this thread gathers: chunk ch = (tile parity, b, lane half)
    const uint32_t nl_base = 32u * (ch >> 2) + 16u * ((ch >> 1) & 1) + 4u * (ch & 1);

    const int NJ = (a.N2 + BN2 - 1) / BN2;
    u32x4 w2r[8];
    auto gload2 = [&](int jc, int st) {
        const uint32_t col = (uint32_t)jc * BN2 + 8u * jg;
        const uint32_t nl0 = 64u * (uint32_t)(st * SUBS + u) + nl_base;
        const bool ok = loader && col < (uint32_t)a.N2;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t row = (uint32_t)n0 + nl0 + (e & 3) + 8u * (e >> 2);
            w2r[e] = buf_load16(rw2, ok ? row * w2row + col * 2u : kOob);
        }
    };
    auto store2 = [&](char* dst) {
        if (loader) {
            u32x4 t[8];
            transpose8x8_b16(w2r, t);
            char* base = dst + u * SUB_BYTES;
#pragma unroll
            for (int i = 0; i < 8; ++i) lds_write16(base, lds_col_off<BN2>(8 * jg + i, ch), t[i]);
        }
    };

    const uint32_t x = lane & 31, h = lane >> 5;
    gload2(0, 0);
    store2(smem);
    __syncthreads();
    int cur = 0;
    for (int jc = 0; jc < NJ; ++jc) {
        f32x16 acc2[MT][JT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc2[mt][jt][r] = 0.0f;
#pragma unroll
        for (int st = 0; st < NST; ++st) {
            const bool last = (st == NST - 1);
            const bool more = !last || (jc + 1 < NJ);
            if (more) gload2(last ? jc + 1 : jc, last ? 0 : st + 1);
            const char* buf = smem + cur * STAGE2;
#pragma unroll
            for (int su = 0; su < SUBS; ++su)
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    vec8 bw[JT];
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt)
                        bw[jt] = lds_read16<vec8>(buf + su * SUB_BYTES,
                                                  lds_col_off<BN2>(32 * jt + x, 2 * kb + h));
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int jt = 0; jt < JT; ++jt)
                            acc2[mt][jt] = Mma<T>::mma(hreg[2 * (st * SUBS + su) + (kb >> 1)][mt][kb & 1],
                                                       bw[jt], acc2[mt][jt]);
                }
            if (more) store2(smem + (cur ^ 1) * STAGE2);
            __syncthreads();
            cur ^= 1;
        }
        // acc2[mt][jt][r]: row m0 + wave*(BM/4) + 32*mt + 8*(r/4) + 4*h + r%4, column 128*jc + 32*jt + x
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                const int col = jc * BN2 + 32 * jt + (int)x;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = (int64_t)m0 + wave * (BM / 4) + 32 * mt + 8 * (r >> 2) + 4 * (int)h + (r & 3);
                    if (row < a.M && col < a.N2)
                        __hip_atomic_fetch_add(a.Ysum + row * a.N2 + col, acc2[mt][jt][r], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                }
            }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 sums -> Y (operand type, RNE); the sums are set back to zero for the next call.
// One thread per 8 consecutive outputs (N2 is a multiple of 8).
// ---------------------------------------------------------------------------------------
template <typename T> __global__ __launch_bounds__(256) void finalize_kernel(float* __restrict__ sums, void* __restrict__ Y, int64_t n8) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    f32x4* p = reinterpret_cast<f32x4*>(sums) + 2 * i;
    const f32x4 v0 = p[0], v1 = p[1];
    u32x4 o;
    o[0] = pack2<T>(v0[0], v0[1]);
    o[1] = pack2<T>(v0[2], v0[3]);
    o[2] = pack2<T>(v1[0], v1[1]);
    o[3] = pack2<T>(v1[2], v1[3]);
    reinterpret_cast<u32x4*>(Y)[i] = o;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    p[0] = z;
    p[1] = z;
}

// ---------------------------------------------------------------------------------------
// C[M][N] = act(A * B) [.* (A * B3)], operands and C in type T, fp32 accumulation.
// 256 x BH tile per workgroup (BH = 256, or 128 when gated), waves 2 x 2.
// ---------------------------------------------------------------------------------------
template <typename T, bool GATED, int BM, int BH>
__global__ __launch_bounds__(256) void gemm_act_kernel(GemmArgs a) {
    typedef FirstGemm<T, GATED, BM, BH, 2, 2> G0;
    constexpr int MT = G0::MT, HT = G0::HT;
    __shared__ __attribute__((aligned(16))) char smem[G0::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int MB = (int)((a.M + BM - 1) / BM), S = (a.N + BH - 1) / BH;
    int ui, us;
    if (!map_unit(MB, S, a.raster, ui, us)) return;
    const int m0 = ui * BM, n0 = us * BH;
    f32x16 acc[HT][MT];
    f32x16 acc3[GATED ? HT : 1][GATED ? MT : 1];
    {
        typename G0::Ctx c;
        G0::init(c, a.A, a.B, a.B3, a.M, a.K, a.N, m0, n0, tid);
        G0::run(smem, c, acc, acc3, tid);
    }
    const int wm = wave % 2, wn = wave / 2;
    const int x = lane & 31, h = lane >> 5;
    char* C = reinterpret_cast<char*>(a.C);
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int64_t row = (int64_t)m0 + wm * G0::WMR + 32 * mt + x;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + wn * G0::WHR + 32 * ht + 8 * q + 4 * h;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = act_rt<T>(a.act, acc[ht][mt][4 * q + e]);
                    if (GATED) v[e] *= acc3[ht][mt][4 * q + e];
                }
                if (row < a.M && col < a.N) {
                    uint2 o;
                    o.x = pack2<T>(v[0], v[1]);
                    o.y = pack2<T>(v[2], v[3]);
                    *reinterpret_cast<uint2*>(C + (row * a.N + col) * 2) = o;
                }
            }
        }
}

// ---------------------------------------------------------------------------------------
// host-side launchers
// ---------------------------------------------------------------------------------------
static inline int grid_for(int64_t M, int N, int BM, int BH) {
    const int64_t total = ((M + BM - 1) / BM) * ((N + BH - 1) / BH);
    return (int)(((total + 7) / 8) * 8);
}

template <typename T, bool GATED, int BM, int BH>
static hipError_t launch_fused_t(const FusedArgs& a, hipStream_t st) {
    hipLaunchKernelGGL((fused_reduce_kernel<T, GATED, BM, BH>), dim3(grid_for(a.M, a.N1, BM, BH)), dim3(256), 0, st, a);
    return hipGetLastError();
}

template <typename T> static hipError_t launch_fused_dt(const FusedArgs& a, int bm, int bh, hipStream_t st) {
    const bool g = a.W3 != nullptr;
    if (!g && bm == 256 && bh == 256) return launch_fused_t<T, false, 256, 256>(a, st);
    if (!g && bm == 128 && bh == 256) return launch_fused_t<T, false, 128, 256>(a, st);
    if (!g && bm == 128 && bh == 128) return launch_fused_t<T, false, 128, 128>(a, st);
    if (!g && bm == 128 && bh == 64) return launch_fused_t<T, false, 128, 64>(a, st);
    if (g && bm == 256 && bh == 128) return launch_fused_t<T, true, 256, 128>(a, st);
    if (g && bm == 128 && bh == 128) return launch_fused_t<T, true, 128, 128>(a, st);
    if (g && bm == 128 && bh == 64) return launch_fused_t<T, true, 128, 64>(a, st);
    return hipErrorInvalidValue;
}

hipError_t launch_fused_reduce(int dtype, const FusedArgs& a, int bm, int bh, hipStream_t st) {
    return dtype == 0 ? launch_fused_dt<__bf16>(a, bm, bh, st) : launch_fused_dt<_Float16>(a, bm, bh, st);
}

bool fused_reduce_supported(int gated, int bm, int bh) {
    if (!gated) return (bm == 256 && bh == 256) || (bm == 128 && (bh == 256 || bh == 128 || bh == 64));
    return (bm == 256 && bh == 128) || (bm == 128 && (bh == 128 || bh == 64));
}

hipError_t launch_finalize(int dtype, float* sums, void* Y, int64_t count, hipStream_t st) {
    const int64_t n8 = count / 8;
    const int blocks = (int)((n8 + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL(finalize_kernel<__bf16>, dim3(blocks), dim3(256), 0, st, sums, Y, n8);
    else
        hipLaunchKernelGGL(finalize_kernel<_Float16>, dim3(blocks), dim3(256), 0, st, sums, Y, n8);
    return hipGetLastError();
}

template <typename T> static hipError_t launch_gemm_dt(const GemmArgs& a, hipStream_t st) {
    if (a.B3) {
        hipLaunchKernelGGL((gemm_act_kernel<T, true, 256, 128>), dim3(grid_for(a.M, a.N, 256, 128)), dim3(256), 0, st, a);
    } else {
        hipLaunchKernelGGL((gemm_act_kernel<T, false, 256, 256>), dim3(grid_for(a.M, a.N, 256, 256)), dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_gemm_act(int dtype, const GemmArgs& a, hipStream_t st) {
    return dtype == 0 ? launch_gemm_dt<__bf16>(a, st) : launch_gemm_dt<_Float16>(a, st);
}

}  // namespace ffuse
