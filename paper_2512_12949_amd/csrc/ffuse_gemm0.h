// Block GEMM on the matrix cores, shared by every 16-bit kernel of the library:
//   D^T[BH x BM] += B^T[BH x K] * A^T[K x BM]
// i.e. a BM x BH block of A*B (and of A*B3 for the gated chain) computed TRANSPOSED: the
// weight matrix B[K][N] is the MFMA "A" operand, the row operand A[M][K] the MFMA "B"
// operand, so that every lane ends up holding 4 consecutive columns n of one row m -- the
// layout the second product of the chain wants for its own row operand, and the layout
// that turns the output tile into 8-byte stores.
//
// K is innermost and complete before anything downstream sees the sums, as the activation
// between the two products requires (paper Sec. 4.3, Rule 3).
//
// 256 threads = 4 waves arranged WM (over rows) x WN (over columns).  Per K step of 64:
//   A tile [BM][64] and B tile [64][BH]: global -> registers -> LDS (B through an 8x8
//   register transpose), LDS double buffered, one barrier per step, prefetch distance two
//   steps: the registers loaded during step i are written to LDS during step i+1 (between
//   its MFMAs) and multiplied in step i+2.
#pragma once
#include <utility>

#include "ffuse_dev.h"


namespace ffuse {

// CONV: the row operand is the implicit im2col matrix of a 3x3, stride-1, zero-padded
// convolution over a channels-last image (row m = pixel m, column k = tap * IC + channel):
// the loader adds the tap's pixel shift to the row's address and masks the taps that fall
// outside the image.  IC must be a multiple of 64, so that a K step of 64 stays in one tap.
// NT: the weight tiles are loaded with the non-temporal hint (for weights that are streamed once
// and too large for the memory-side cache to keep; the caller picks the instantiation)
template <typename T, bool GATED, int BM, int BH, int WM, int WN, bool CONV = false, bool NT = false>
struct FirstGemm {
    static_assert(WM * WN == 4, "four waves");
    typedef typename Mma<T>::vec8 vec8;
    static constexpr int G = GATED ? 2 : 1;
    static constexpr int WMR = BM / WM, WHR = BH / WN;  // rows / columns per wave
    static constexpr int MT = WMR / 32, HT = WHR / 32;  // 32x32 tiles per wave
    // (a gated tile needs BH >= 64: which of the two weight matrices a lane loads must be uniform per wave)
    static_assert(MT >= 1 && HT >= 1 && BM % 32 == 0 && BH % 32 == 0 && (BH % 64 == 0 || !GATED), "tile shape");
    static constexpr int XB = BM * 128;       // bytes of one A stage
    static constexpr int WB = BH * 128;       // bytes of one B stage
    static constexpr int STAGE = XB + G * WB;
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int XCH = BM / 32;       // 16-byte A chunks per thread per stage
    static constexpr int NBLK1 = BH;          // 8x8 B blocks per matrix per stage
    static constexpr int NBLK = NBLK1 * G;
    static constexpr int WPT = (NBLK + 255) / 256;
    static constexpr bool ALL_LOAD_B = (NBLK % 256) == 0;  // every thread owns a B block

    struct Stage {
        u32x4 x[XCH];
        u32x4 w[WPT][8];
    };

    struct Ctx {
        __amdgpu_buffer_rsrc_t rx;
        __amdgpu_buffer_rsrc_t rw[WPT];  // B or B3, uniform per wave
        uint32_t xoff[XCH];   // byte offset of this thread's A chunks at k = 0
        uint32_t abase;       // uniform byte offset added to every A offset (kOob: reads as zero)
        uint32_t woff[WPT];   // byte offset of row 0 of this thread's B block(s)
        uint32_t wrow;        // bytes per B row
        uint32_t xc;          // this thread's chunk (0..7) within an A row
        int KX;               // extent of the A operand along k (chunks at or past it read as 0)
        // LDS read offsets of this lane's fragments at sub-step 0, stage 0
        uint32_t rdx[MT], rdw[HT];
        // CONV only: channels and width of the image; per row, bit t set = tap t is inside the image
        int conv_ic, conv_w;
        uint32_t vmask[CONV ? XCH : 1];
    };

    // A operand: `rows x lda` elements at `A` (+ base_bytes), first row row0; rows past the
    // end of the buffer read as zero.
    static __device__ __forceinline__ void init_a(Ctx& c, const void* A, uint32_t a_bytes, uint32_t base_bytes,
                                                  uint32_t row0, uint32_t lda, int kx, int tid) {
        c.rx = make_rsrc(A, a_bytes);
        c.KX = kx;
        c.abase = base_bytes;
        c.xc = tid & 7;
#pragma unroll
        for (int p = 0; p < XCH; ++p) {
            const uint32_t row = row0 + (tid >> 3) + 32u * p;
            c.xoff[p] = (row * lda + 8u * c.xc) * 2u;
        }
    }
    // CONV: A = im2col of the image X[npix][IC] (npix = B*H*W pixels, channels last) for a 3x3
    // kernel; rows are pixels, K = 9 * IC.
    static __device__ __forceinline__ void init_a_conv(Ctx& c, const void* X, uint32_t x_bytes, uint32_t row0, int64_t npix,
                                                       int H, int W, int IC, int tid) {
        c.rx = make_rsrc(X, x_bytes);
        c.KX = 9 * IC;
        c.abase = 0u;
        c.xc = tid & 7;
        c.conv_ic = IC;
        c.conv_w = W;
#pragma unroll
        for (int p = 0; p < XCH; ++p) {
            const uint32_t row = row0 + (tid >> 3) + 32u * p;
            c.xoff[p] = (row * (uint32_t)IC + 8u * c.xc) * 2u;
            const int h = (int)((row / (uint32_t)W) % (uint32_t)H), w = (int)(row % (uint32_t)W);
            uint32_t m = 0;
            if ((int64_t)row < npix)
                for (int t = 0; t < 9; ++t) {
                    const int hh = h + t / 3 - 1, ww = w + t % 3 - 1;
                    if (hh >= 0 && hh < H && ww >= 0 && ww < W) m |= 1u << t;
                }
            c.vmask[CONV ? p : 0] = m;
        }
    }
    // per K step: the uniform part of the A addresses
    struct AStep {
        bool ok;
        uint32_t add;
        int tap;
    };
    static __device__ __forceinline__ AStep a_step(const Ctx& c, int kx) {
        AStep s;
        if (CONV) {
            const int tap = kx / c.conv_ic, ic0 = kx - tap * c.conv_ic;
            const int dh = tap / 3 - 1, dw = tap - 3 * (tap / 3) - 1;
            s.add = (uint32_t)(((dh * c.conv_w + dw) * c.conv_ic + ic0) * 2);   // may be "negative": offsets add modulo 2^32
            s.tap = tap;
            s.ok = kx < c.KX;
        } else {
            s.add = (uint32_t)kx * 2u;
            s.tap = 0;
            s.ok = (kx + 8 * (int)c.xc) < c.KX && c.abase != kOob;
        }
        return s;
    }
    static __device__ __forceinline__ uint32_t a_offset(const Ctx& c, const AStep& s, int p) {
        const bool ok = s.ok && (!CONV || ((c.vmask[CONV ? p : 0] >> s.tap) & 1u));
        return ok ? c.xoff[p] + c.abase + s.add : kOob;
    }

    // B operands: [K][ldb] matrices, first column n0 (columns at or past ncols read as zero).
    static __device__ __forceinline__ void init_b(Ctx& c, const void* B, const void* B3, uint32_t b_bytes,
                                                  uint32_t ldb, uint32_t ncols, uint32_t n0, int tid) {
        c.wrow = ldb * 2u;
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int blk = tid + 256 * q;
            // which matrix this thread's block belongs to: constant per wave by construction
            int which = 0;
            if (GATED)
                which = (NBLK1 >= 256) ? (256 * q) / NBLK1 : (__builtin_amdgcn_readfirstlane(tid / NBLK1) & 1);
            c.rw[q] = make_rsrc(which ? B3 : B, b_bytes);
            const int b = blk % NBLK1;
            const int ng = b % (BH / 8), kg = b / (BH / 8);
            const uint32_t col = n0 + 8u * ng;
            c.woff[q] = (blk < NBLK && col < ncols) ? ((uint32_t)(8 * kg) * ldb + col) * 2u : kOob;
        }
    }
    static __device__ __forceinline__ void init_lds(Ctx& c, int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        const int wm = wave % WM, wn = wave / WM;
        const uint32_t x = lane & 31, h = lane >> 5;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) c.rdx[mt] = lds_row_off(wm * WMR + 32 * mt + x, h);
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) c.rdw[ht] = XB + lds_col_off<BH>(wn * WHR + 32 * ht + x, h);
    }

    // global -> registers for the K step whose A columns start at kx / B rows at kw
    static __device__ __forceinline__ void gload_a(const Ctx& c, Stage& s, int kx) {
        const AStep as = a_step(c, kx);
#pragma unroll
        for (int p = 0; p < XCH; ++p) s.x[p] = buf_load16(c.rx, a_offset(c, as, p));
    }
    static __device__ __forceinline__ void gload_b(const Ctx& c, Stage& s, int kw) {
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const uint32_t base = c.woff[q];
            const uint32_t kb = (uint32_t)kw * c.wrow;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const uint32_t off = (base == kOob) ? kOob : base + kb + (uint32_t)r * c.wrow;
                s.w[q][r] = NT ? buf_load16_nt(c.rw[q], off) : buf_load16(c.rw[q], off);
            }
        }
    }
    static __device__ __forceinline__ void gload(const Ctx& c, Stage& s, int kx, int kw) {
        gload_a(c, s, kx);
        gload_b(c, s, kw);
    }

    static __device__ __forceinline__ void store_a(char* smem, const Stage& s, int tid) {
#pragma unroll
        for (int p = 0; p < XCH; ++p) lds_write16(smem, lds_row_off((tid >> 3) + 32u * p, tid & 7), s.x[p]);
    }
    static __device__ __forceinline__ void store_b(char* smem, const Stage& s, int tid) {
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int blk = tid + 256 * q;
            if (ALL_LOAD_B || blk < NBLK) {
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

    struct Frags {
        vec8 b[MT];
        vec8 a[HT];
        vec8 a3[GATED ? HT : 1];
    };
    // fragments of sub-step ks (k = 16*ks .. +15 of the stage at `smem`)
    static __device__ __forceinline__ void load_frags(const char* smem, const Ctx& c, int ks, Frags& f) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) f.b[mt] = lds_read16<vec8>(smem, c.rdx[mt] ^ (uint32_t)(ks << 5));
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            f.a[ht] = lds_read16<vec8>(smem, c.rdw[ht] ^ (uint32_t)(ks << 5));
            if (GATED) f.a3[ht] = lds_read16<vec8>(smem + WB, c.rdw[ht] ^ (uint32_t)(ks << 5));
        }
    }
    static __device__ __forceinline__ void mma_frags(const Frags& f, f32x16 (&acc)[HT][MT],
                                                     f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[ht][mt] = Mma<T>::mma(f.a[ht], f.b[mt], acc[ht][mt]);
            if (GATED) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc3[ht][mt] = Mma<T>::mma(f.a3[ht], f.b[mt], acc3[ht][mt]);
            }
        }
    }

    // fragment read number i of a sub-step, in the order the MFMAs need them:
    // b[0], a[0] (, a3[0]), b[1..MT-1], a[1] (, a3[1]), ...
    static __device__ __forceinline__ void read_one(const char* smem, const Ctx& c, int ks, int i, Frags& f) {
        const uint32_t kx = (uint32_t)(ks << 5);
        if (i == 0) { f.b[0] = lds_read16<vec8>(smem, c.rdx[0] ^ kx); return; }
        if (i == 1) { f.a[0] = lds_read16<vec8>(smem, c.rdw[0] ^ kx); return; }
        int j = i - 2;
        if (GATED) {
            if (j == 0) { f.a3[0] = lds_read16<vec8>(smem + WB, c.rdw[0] ^ kx); return; }
            j -= 1;
        }
        if (j < MT - 1) { f.b[j + 1] = lds_read16<vec8>(smem, c.rdx[j + 1] ^ kx); return; }
        j -= MT - 1;
        const int ht = 1 + j / G;
        if (!GATED || (j % G) == 0) f.a[ht] = lds_read16<vec8>(smem, c.rdw[ht] ^ kx);
        else f.a3[ht] = lds_read16<vec8>(smem + WB, c.rdw[ht] ^ kx);
    }
    // MFMA number i of a sub-step: ht-major, then (gate,) mt
    static __device__ __forceinline__ void mma_one(const Frags& f, int i, f32x16 (&acc)[HT][MT],
                                                   f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
        const int ht = i / (MT * G), r = i % (MT * G);
        if (!GATED || r < MT) acc[ht][r % MT] = Mma<T>::mma(f.a[ht], f.b[r % MT], acc[ht][r % MT]);
        else acc3[GATED ? ht : 0][GATED ? r - MT : 0] = Mma<T>::mma(f.a3[GATED ? ht : 0], f.b[r - MT], acc3[GATED ? ht : 0][GATED ? r - MT : 0]);
    }

    // One K step of 64 out of the stage at `cur`.  Meanwhile the registers in `st` (loaded
    // one step earlier) are written to the stage at `nxt` and re-filled from global memory
    // for the step after that (A columns from kx, B rows from kw).  With one wave per SIMD
    // nothing but the issue order hides latency, so the step is written as micro-chunks of
    // one MFMA plus a little other work, fenced so the compiler keeps the interleaving:
    //   sub-steps 0-2: the fragment reads of the next sub-step ride under the MFMAs,
    //   sub-step 2   : + A stores to LDS, each followed by the A load that refills its register,
    //   sub-step 3   : + B transpose, B stores and B loads.
    static __device__ __forceinline__ void step(const char* cur, char* nxt, const Ctx& c, Stage& st, int kx, int kw,
                                                f32x16 (&acc)[HT][MT],
                                                f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1], int tid) {
        constexpr int NM = HT * MT * G;   // MFMAs per sub-step
        constexpr int NR = MT + HT * G;   // LDS fragment reads per sub-step
        Frags f[2];
#pragma unroll
        for (int i = 0; i < NR; ++i) read_one(cur, c, 0, i, f[0]);
        __builtin_amdgcn_sched_barrier(0);
        const AStep as = a_step(c, kx);
        const uint32_t kb = (uint32_t)kw * c.wrow;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                mma_one(f[ks & 1], i, acc, acc3);
                if (ks < 3) {
#pragma unroll
                    for (int e = (i * NR) / NM; e < ((i + 1) * NR) / NM; ++e) read_one(cur, c, ks + 1, e, f[(ks + 1) & 1]);
                }
                if (ks == 2) {
#pragma unroll
                    for (int e = (i * XCH) / NM; e < ((i + 1) * XCH) / NM; ++e) {
                        lds_write16(nxt, lds_row_off((tid >> 3) + 32u * e, tid & 7), st.x[e]);
                        st.x[e] = buf_load16(c.rx, a_offset(c, as, e));
                    }
                }
                if (ks == 3) {
                    // first half of the MFMAs: transpose + store the 8*WPT columns of the old
                    // B block(s); second half: refill the same registers (every column needs
                    // all 8 old rows, so no row may be overwritten before the last store)
                    constexpr int H1 = (NM + 1) / 2, H2 = NM - H1;   // H2 == 0 only when NM == 1
                    if (i < H1) {
#pragma unroll
                        for (int e = (i * 8 * WPT) / H1; e < ((i + 1) * 8 * WPT) / H1; ++e) {
                            const int q = e / 8, r = e % 8;
                            const int blk = tid + 256 * q;
                            if (ALL_LOAD_B || blk < NBLK) {
                                const int which = blk / NBLK1, b = blk % NBLK1;
                                const int ng = b % (BH / 8), kg = b / (BH / 8);
                                lds_write16(nxt + XB + which * WB, lds_col_off<BH>(8 * ng + r, kg),
                                            transpose8x8_col(st.w[q], r));
                            }
                        }
                    } else {
                        const int i2 = i - H1;
#pragma unroll
                        for (int e = (i2 * 8 * WPT) / (H2 > 0 ? H2 : 1); e < ((i2 + 1) * 8 * WPT) / (H2 > 0 ? H2 : 1); ++e) {
                            const int q = e / 8, r = e % 8;
                            const uint32_t base = c.woff[q];
                            st.w[q][r] = NT ? buf_load16_nt(c.rw[q], (base == kOob) ? kOob : base + kb + (uint32_t)r * c.wrow) : buf_load16(c.rw[q], (base == kOob) ? kOob : base + kb + (uint32_t)r * c.wrow);
                        }
                    }
                    if (H2 == 0 && i == NM - 1) {   // a single MFMA per sub-step: refill right after the stores
#pragma unroll
                        for (int e = 0; e < 8 * WPT; ++e) {
                            const int q = e / 8, r = e % 8;
                            const uint32_t base = c.woff[q];
                            st.w[q][r] = NT ? buf_load16_nt(c.rw[q], (base == kOob) ? kOob : base + kb + (uint32_t)r * c.wrow) : buf_load16(c.rw[q], (base == kOob) ? kOob : base + kb + (uint32_t)r * c.wrow);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    static __device__ __forceinline__ void zero(f32x16 (&acc)[HT][MT], f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
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
    }

    // K loop over k = kbegin .. kend-1 (A columns and B rows advance together; kend - kbegin is
    // rounded up to whole steps of 64, so a range that is not the tail of the operands must
    // be a multiple of 64).  On return acc[ht][mt][r] holds the partial (A*B)[m][n] with
    //   m = row0 + wm*WMR + 32*mt + lane%32,
    //   n = n0 + wn*WHR + 32*ht + 8*(r/4) + 4*(lane/32) + r%4,
    // acc3 the same for B3.  Loads past the operands return zeros (buffer range check), so
    // the prefetch needs no tail branch.  Ends with a barrier: LDS may be reused by the caller.
    static __device__ __forceinline__ void run(char* smem, const Ctx& c, int kbegin, int kend, f32x16 (&acc)[HT][MT],
                                               f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1], int tid,
                                               uint64_t* t_loop = nullptr) {
        zero(acc, acc3);
        const int KT = (kend - kbegin + 63) / 64;
        Stage st;
        gload(c, st, kbegin, kbegin);
        store_a(smem, st, tid);
        store_b(smem, st, tid);
        gload(c, st, kbegin + 64, kbegin + 64);
        __syncthreads();
        if (t_loop) *t_loop = wall_clock64();
        for (int kt = 0; kt < KT; ++kt) {
            char* cur = smem + (kt & 1) * STAGE;
            char* nxt = smem + ((kt + 1) & 1) * STAGE;
            const int k2 = kbegin + (kt + 2) * 64;
            step(cur, nxt, c, st, k2, k2, acc, acc3, tid);
            __syncthreads();
        }
    }

    // Same K loop with TWO register stages, i.e. prefetch distance three steps: every global
    // load has two whole steps to land before it is written to LDS, which doubles the bytes in
    // flight per CU.  For the bandwidth-bound small-M kernels, whose accumulators are small.
    static __device__ __forceinline__ void run_deep(char* smem, const Ctx& c, int kbegin, int kend, f32x16 (&acc)[HT][MT],
                                                    f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1], int tid) {
        zero(acc, acc3);
        const int KT = (kend - kbegin + 63) / 64;
        Stage sa, sb;
        gload(c, sa, kbegin, kbegin);
        store_a(smem, sa, tid);
        store_b(smem, sa, tid);
        gload(c, sa, kbegin + 64, kbegin + 64);
        gload(c, sb, kbegin + 128, kbegin + 128);
        __syncthreads();
        for (int kt = 0; kt < KT; kt += 2) {
            const int k3 = kbegin + (kt + 3) * 64;
            step(smem, smem + STAGE, c, sa, k3, k3, acc, acc3, tid);          // multiplies step kt, stores kt+1, loads kt+3
            __syncthreads();
            if (kt + 1 < KT) {
                step(smem + STAGE, smem, c, sb, k3 + 64, k3 + 64, acc, acc3, tid);  // step kt+1, stores kt+2, loads kt+4
                __syncthreads();
            }
        }
    }

    // acc (and the gate) -> activation -> type T -> C[row][col] (leading dimension ldc),
    // rows < row_lim and columns < col_lim only.  8-byte stores: 4 consecutive columns.
    template <int ACT>
    static __device__ __forceinline__ void store_tile(const f32x16 (&acc)[HT][MT],
                                                      const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                      char* C, int64_t ldc, int64_t row0, int col0,
                                                      int64_t row_lim, int col_lim, int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        const int wm = wave % WM, wn = wave / WM;
        const int x = lane & 31, h = lane >> 5;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int64_t row = row0 + wm * WMR + 32 * mt + x;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = col0 + wn * WHR + 32 * ht + 8 * q + 4 * h;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = activate<ACT>(acc[ht][mt][4 * q + e]);
                        if (GATED) v[e] *= acc3[ht][mt][4 * q + e];
                    }
                    if (row < row_lim && col < col_lim) {
                        uint2 o;
                        o.x = pack2<T>(v[0], v[1]);
                        o.y = pack2<T>(v[2], v[3]);
                        *reinterpret_cast<uint2*>(C + (row * ldc + col) * 2) = o;
                    }
                }
            }
    }
    static __device__ __forceinline__ void store_tile_rt(int act, const f32x16 (&acc)[HT][MT],
                                                         const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                         char* C, int64_t ldc, int64_t row0, int col0,
                                                         int64_t row_lim, int col_lim, int tid) {
        switch (act) {
            case ACT_RELU: store_tile<ACT_RELU>(acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
            case ACT_GELU_TANH: store_tile<ACT_GELU_TANH>(acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
            case ACT_SILU: store_tile<ACT_SILU>(acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
            default: store_tile<ACT_IDENTITY>(acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
        }
    }

    // Same result as store_tile, but through LDS so that the global stores are coalesced: in
    // the accumulator layout a lane owns 4 consecutive columns of ONE row and the 64 lanes of a
    // store instruction touch 64 different rows (64 cache lines, 8 bytes each); after the
    // detour each lane stores 16 bytes and 16 lanes cover 256 contiguous bytes of a row.
    // Every wave stages its own WMR x WHR block in its own region of `smem` (BM*BH*2 bytes in
    // all, never more than LDS_BYTES), so no workgroup barrier is needed -- but the caller
    // must make sure that no wave still reads the stages and that no load is still in flight
    // to them.  8-byte slots of a row are XOR-swizzled with the row so that both the 8-byte
    // writes (32 rows per instruction) and the 16-byte reads are free of bank conflicts.
    // Requires ldc, col0 and col_lim to be multiples of 8 (16-byte aligned chunks).
    // THROUGH: the global stores are written through the L2 (device scope) as they are issued,
    // so that workgroups on other XCDs can read the tile after a flag without anybody having
    // to write back a whole L2 first; C must then be smaller than 2 GiB.
    static constexpr int EPI_RB = WHR * 2;                    // bytes per staged row
    static constexpr int EPI_SLOTS = EPI_RB / 8;
    static constexpr int EPI_SHIFT = EPI_RB >= 256 ? 0 : (EPI_RB == 128 ? 1 : 2);
    static constexpr int EPI_LPR = EPI_RB / 16;               // lanes per row on the way out
    static constexpr int EPI_RPI = 64 / EPI_LPR;              // rows per store instruction
    static_assert(EPI_RB == 64 || EPI_RB == 128 || EPI_RB == 256 || EPI_RB == 512, "staged row size");
    static __device__ __forceinline__ uint32_t epi_key(uint32_t row) {
        return (row >> EPI_SHIFT) & (uint32_t)((EPI_SLOTS < 32 ? EPI_SLOTS : 32) - 1);
    }
    template <int ACT, bool THROUGH = false>
    static __device__ __forceinline__ void store_tile_lds(char* smem, const f32x16 (&acc)[HT][MT],
                                                          const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                          char* C, int64_t ldc, int64_t row0, int col0,
                                                          int64_t row_lim, int col_lim, int tid) {
        const int wave = tid >> 6;
        int lane = tid & 63;
        // opaque to the optimiser: otherwise the per-row LDS addresses below are hoisted out of
        // the caller's tile loop and live (spilled) across its main loop
        asm volatile("" : "+v"(lane));
        const int wm = wave % WM, wn = wave / WM;
        const uint32_t x = lane & 31, h = lane >> 5;
        char* mine = smem + wave * (WMR * EPI_RB);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint32_t row = 32 * mt + x;
            const uint32_t key = epi_key(row);
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = activate<ACT>(acc[ht][mt][4 * q + e]);
                        if (GATED) v[e] *= acc3[ht][mt][4 * q + e];
                    }
                    uint2 o;
                    o.x = pack2<T>(v[0], v[1]);
                    o.y = pack2<T>(v[2], v[3]);
                    const uint32_t slot = (uint32_t)(8 * ht + 2 * q) + h;
                    *reinterpret_cast<uint2*>(mine + row * EPI_RB + ((slot ^ key) << 3)) = o;
                }
        }
        // wave-private region: LDS operations of one wave complete in order
        const uint32_t rin = lane / EPI_LPR, ch = lane % EPI_LPR;
        const int col = col0 + wn * WHR + 8 * (int)ch;
        // in batches of 8 rows-per-lane, fenced: left alone the compiler hoists all the LDS
        // reads above the stores and runs out of registers
        constexpr int NOUT = WMR / EPI_RPI, BATCH = NOUT < 8 ? NOUT : 8;
        __amdgpu_buffer_rsrc_t rc;
        if constexpr (THROUGH) rc = make_rsrc(C, (uint32_t)(row_lim * ldc * 2));
#pragma unroll
        for (int i0 = 0; i0 < NOUT; i0 += BATCH) {
            u32x4 v[BATCH];
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const uint32_t row = (uint32_t)((i0 + i) * EPI_RPI) + rin;
                const uint32_t key = epi_key(row);
                v[i] = *reinterpret_cast<const u32x4*>(mine + row * EPI_RB + ((ch ^ (key >> 1)) << 4));
                if (key & 1u) { u32x4 w = {v[i][2], v[i][3], v[i][0], v[i][1]}; v[i] = w; }
            }
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const int64_t grow = row0 + wm * WMR + (i0 + i) * EPI_RPI + rin;
                if constexpr (THROUGH) {
                    // out-of-range chunks get an offset beyond the buffer: the hardware drops the store
                    const uint32_t off = (grow < row_lim && col < col_lim) ? (uint32_t)((grow * ldc + col) * 2) : kOob;
                    buf_store16_through(v[i], rc, off);
                } else {
                    if (grow < row_lim && col < col_lim) *reinterpret_cast<u32x4*>(C + (grow * ldc + col) * 2) = v[i];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // store_tile_lds in slabs of 32 rows per wave: the same values and the same coalesced stores, but only
    // 4 * 32 * EPI_RB bytes of staging (32 KB at most) at `staging`, reused slab after slab -- a wave's LDS
    // operations complete in order and the region is its own, so a slab's reads are done before the next
    // slab's writes land.  For callers that have loads in flight to the rest of LDS meanwhile (the next
    // item's ring fill, DeepGemm::prefill).  `wave`: the wave's number in the workgroup, uniform (a scalar).
    template <int ACT, bool THROUGH = false>
    static __device__ __forceinline__ void store_tile_slabs(char* staging, const f32x16 (&acc)[HT][MT],
                                                            const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                            char* C, int64_t ldc, int64_t row0, int col0,
                                                            int64_t row_lim, int col_lim, int wave) {
        // the lane number from the hardware, not from the thread index: that one lives in scratch memory by now, and
        // a reload here would wait for every load the caller has in flight
        const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        const int wm = wave % WM, wn = wave / WM;
        const uint32_t x = lane & 31, h = lane >> 5;
        char* mine = staging + wave * (32 * EPI_RB);
        const uint32_t wkey = epi_key(x);               // epi_key(32 mt + x) = epi_key(x)
        const uint32_t rin = lane / EPI_LPR, ch = lane % EPI_LPR;
        const int col = col0 + wn * WHR + 8 * (int)ch;
        constexpr int NOUT = 32 / EPI_RPI;              // store instructions per slab: 8, 4 or 2
        __amdgpu_buffer_rsrc_t rc;
        if constexpr (THROUGH) rc = make_rsrc(C, (uint32_t)(row_lim * ldc * 2));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = activate<ACT>(acc[ht][mt][4 * q + e]);
                        if (GATED) v[e] *= acc3[ht][mt][4 * q + e];
                    }
                    uint2 o;
                    o.x = pack2<T>(v[0], v[1]);
                    o.y = pack2<T>(v[2], v[3]);
                    const uint32_t slot = (uint32_t)(8 * ht + 2 * q) + h;
                    *reinterpret_cast<uint2*>(mine + x * EPI_RB + ((slot ^ wkey) << 3)) = o;
                }
            u32x4 v[NOUT];
#pragma unroll
            for (int i = 0; i < NOUT; ++i) {
                const uint32_t row = (uint32_t)(i * EPI_RPI) + rin;
                const uint32_t key = epi_key(row);
                v[i] = *reinterpret_cast<const u32x4*>(mine + row * EPI_RB + ((ch ^ (key >> 1)) << 4));
                if (key & 1u) { u32x4 w = {v[i][2], v[i][3], v[i][0], v[i][1]}; v[i] = w; }
            }
#pragma unroll
            for (int i = 0; i < NOUT; ++i) {
                const int64_t grow = row0 + wm * WMR + 32 * mt + i * EPI_RPI + rin;
                if constexpr (THROUGH) {
                    const uint32_t off = (grow < row_lim && col < col_lim) ? (uint32_t)((grow * ldc + col) * 2) : kOob;
                    buf_store16_through(v[i], rc, off);
                } else {
                    if (grow < row_lim && col < col_lim) *reinterpret_cast<u32x4*>(C + (grow * ldc + col) * 2) = v[i];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    template <bool THROUGH = false>
    static __device__ __forceinline__ void store_tile_slabs_rt(char* staging, int act, const f32x16 (&acc)[HT][MT],
                                                               const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                               char* C, int64_t ldc, int64_t row0, int col0,
                                                               int64_t row_lim, int col_lim, int wave) {
        switch (act) {
            case ACT_RELU: store_tile_slabs<ACT_RELU, THROUGH>(staging, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, wave); break;
            case ACT_GELU_TANH: store_tile_slabs<ACT_GELU_TANH, THROUGH>(staging, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, wave); break;
            case ACT_SILU: store_tile_slabs<ACT_SILU, THROUGH>(staging, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, wave); break;
            default: store_tile_slabs<ACT_IDENTITY, THROUGH>(staging, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, wave); break;
        }
    }
    template <bool THROUGH = false>
    static __device__ __forceinline__ void store_tile_lds_rt(char* smem, int act, const f32x16 (&acc)[HT][MT],
                                                             const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                                             char* C, int64_t ldc, int64_t row0, int col0,
                                                             int64_t row_lim, int col_lim, int tid) {
        switch (act) {
            case ACT_RELU: store_tile_lds<ACT_RELU, THROUGH>(smem, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
            case ACT_GELU_TANH: store_tile_lds<ACT_GELU_TANH, THROUGH>(smem, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
            case ACT_SILU: store_tile_lds<ACT_SILU, THROUGH>(smem, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
            default: store_tile_lds<ACT_IDENTITY, THROUGH>(smem, acc, acc3, C, ldc, row0, col0, row_lim, col_lim, tid); break;
        }
    }
};

}  // namespace ffuse
