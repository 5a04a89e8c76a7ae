// First product of the chain on the matrix cores: a BH x BM block of (X * W1)^T (and of
// (X * W3)^T for the gated chain) with K innermost and complete, as the activation requires
// (paper Sec. 4.3, Rule 3).  Shared by the fused kernels and by the plain GEMM kernel of the
// unfused path.
//
// The product is computed transposed -- weights are the MFMA "A" operand, X the "B" operand --
// so that every lane ends up holding 4 consecutive hidden indices of one row of X: exactly
// the operand layout the second product needs for H, with no shuffle in between.
//
// 256 threads = 4 waves arranged WM (over rows of X) x WN (over hidden columns).
// Per K step of 64: X tile [BM][64] and W tile [64][BH] go global -> registers -> LDS
// (weights through the 8x8 register transpose), double buffered in LDS, one barrier per step.
#pragma once
#include "ffuse_dev.h"

namespace ffuse {

template <typename T, bool GATED, int BM, int BH, int WM, int WN>
struct FirstGemm {
    static_assert(WM * WN == 4, "four waves");
    typedef typename Mma<T>::vec8 vec8;
    static constexpr int G = GATED ? 2 : 1;
    static constexpr int WMR = BM / WM, WHR = BH / WN;  // rows / hidden columns per wave
    static constexpr int MT = WMR / 32, HT = WHR / 32;  // 32x32 tiles per wave
    static_assert(MT >= 1 && HT >= 1 && BM % 32 == 0 && BH % 64 == 0, "tile shape");
    static constexpr int XB = BM * 128;       // bytes of one X stage
    static constexpr int WB = BH * 128;       // bytes of one weight stage
    static constexpr int STAGE = XB + G * WB;
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int XCH = BM / 32;       // 16-byte X chunks per thread per stage
    static constexpr int NBLK1 = BH;          // 8x8 weight blocks per matrix per stage
    static constexpr int NBLK = NBLK1 * G;
    static constexpr int WPT = (NBLK + 255) / 256;

    struct Stage {
        u32x4 x[XCH];
        u32x4 w[WPT][8];
    };

    struct Ctx {
        __amdgpu_buffer_rsrc_t rx;
        __amdgpu_buffer_rsrc_t rw[WPT];  // W1 or W3, uniform per wave
        uint32_t xoff[XCH];   // byte offset of this thread's X chunks at k0 = 0
        uint32_t woff[WPT];   // byte offset of row 0 of this thread's weight block(s)
        uint32_t wrow;        // bytes per weight row
        uint32_t xc;          // this thread's chunk (0..7) within an X row
        int K;
    };

    // m0: first row of X; n0: first hidden column; N1: row length of the weights.
    static __device__ __forceinline__ void init(Ctx& c, const void* X, const void* W1, const void* W3,
                                                int64_t M, int K, int N1, int m0, int n0, int tid) {
        c.rx = make_rsrc(X, (uint32_t)((uint64_t)M * K * 2));
        c.K = K;
        c.wrow = (uint32_t)N1 * 2u;
        c.xc = tid & 7;
#pragma unroll
        for (int p = 0; p < XCH; ++p) {
            const uint32_t row = (uint32_t)m0 + (tid >> 3) + 32u * p;
            c.xoff[p] = (row * (uint32_t)K + 8u * c.xc) * 2u;
        }
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int blk = tid + 256 * q;
            // which matrix this thread's block belongs to: constant per wave by construction
            int which = 0;
            if (GATED)
                which = (NBLK1 >= 256) ? (256 * q) / NBLK1
                                       : (__builtin_amdgcn_readfirstlane(tid / NBLK1) & 1);
            c.rw[q] = make_rsrc(which ? W3 : W1, (uint32_t)((uint64_t)K * N1 * 2));
            const int b = blk % NBLK1;
            const int ng = b % (BH / 8), kg = b / (BH / 8);
            const uint32_t col = (uint32_t)n0 + 8u * ng;
            c.woff[q] = (blk < NBLK && col < (uint32_t)N1)
                            ? ((uint32_t)(8 * kg) * (uint32_t)N1 + col) * 2u
                            : kOob;
        }
    }

    static __device__ __forceinline__ void gload(const Ctx& c, Stage& s, int k0) {
        const bool xok = (k0 + 8 * (int)c.xc) < c.K;
#pragma unroll
        for (int p = 0; p < XCH; ++p)
            s.x[p] = buf_load16(c.rx, xok ? c.xoff[p] + (uint32_t)k0 * 2u : kOob);
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const uint32_t base = c.woff[q];
            const uint32_t kb = (uint32_t)k0 * c.wrow;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint32_t off = (base == kOob) ? kOob : base + kb + (uint32_t)r * c.wrow;
                s.w[q][r] = buf_load16(c.rw[q], off);
            }
        }
    }

    static __device__ __forceinline__ void lds_store(char* smem, const Stage& s, int tid) {
#pragma unroll
        for (int p = 0; p < XCH; ++p)
            lds_write16(smem, lds_row_off((tid >> 3) + 32u * p, tid & 7), s.x[p]);
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int blk = tid + 256 * q;
            if (blk < NBLK) {
                const int which = blk / NBLK1, b = blk % NBLK1;
                const int ng = b % (BH / 8), kg = b / (BH / 8);
                u32x4 t[8];
                transpose8x8_b16(s.w[q], t);
                char* base = smem + XB + which * WB;
#pragma unroll
                for (int i = 0; i < 8; ++i) lds_write16(base, lds_col_off<BH>(8 * ng + i, kg), t[i]);
            }
        }
    }

    // One K step of 64 from the LDS stage at `smem`.
    static __device__ __forceinline__ void compute(const char* smem, f32x16 (&acc)[HT][MT],
                                                   f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                   int wm, int wn, int lane) {
        const uint32_t x = lane & 31, h = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint32_t chunk = 2 * ks + h;
            vec8 b[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                b[mt] = lds_read16<vec8>(smem, lds_row_off(wm * WMR + 32 * mt + x, chunk));
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) {
                const uint32_t off = lds_col_off<BH>(wn * WHR + 32 * ht + x, chunk);
                const vec8 a = lds_read16<vec8>(smem + XB, off);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[ht][mt] = Mma<T>::mma(a, b[mt], acc[ht][mt]);
                if (GATED) {
                    const vec8 a3 = lds_read16<vec8>(smem + XB + WB, off);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc3[ht][mt] = Mma<T>::mma(a3, b[mt], acc3[ht][mt]);
                }
            }
        }
    }

    // Whole K loop.  On return acc[ht][mt][r] holds (X*W1)[m][n] with
    //   m = m0 + wm*WMR + 32*mt + lane%32,
    //   n = n0 + wn*WHR + 32*ht + 8*(r/4) + 4*(lane/32) + r%4,
    // acc3 the same for W3.  Ends with a barrier: LDS may be reused by the caller.
    static __device__ __forceinline__ void run(char* smem, const Ctx& c, f32x16 (&acc)[HT][MT],
                                               f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                               int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        const int wm = wave % WM, wn = wave / WM;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[ht][mt][r] = 0.0f;
                if (GATED) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc3[ht][mt][r] = 0.0f;
                }
            }
        const int KT = (c.K + 63) / 64;
        Stage st;
        gload(c, st, 0);
        lds_store(smem, st, tid);
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            char* cur = smem + (kt & 1) * STAGE;
            char* nxt = smem + ((kt + 1) & 1) * STAGE;
            const bool more = kt + 1 < KT;
            if (more) gload(c, st, (kt + 1) * 64);
            compute(cur, acc, acc3, wm, wn, lane);
            if (more) lds_store(nxt, st, tid);
            __syncthreads();
        }
    }
};

}  // namespace ffuse
