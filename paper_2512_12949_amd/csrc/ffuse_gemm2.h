// DeepGemm (ffuse_gemm1.h) with the row operand loaded in WHOLE 128-byte cache lines.
//
// DeepGemm's A stage is [BM][32 k]: 64 bytes per row, half a cache line, and the other half is
// fetched one step later by another instruction.  Measured on the m = 128 shapes, where every
// workgroup re-reads the whole row operand from L2: each line then crosses the L2 -> CU path
// twice, and that path is what bounds the first phase (same loads, same bytes, whole lines:
// 47 -> 37 us for the first phase of 128 x 4096 x 16384).
//
// Here the A operand lives in "super-stages" of 64 k -- [BM][64 k], rows of 128 bytes -- in a
// ring of their own (NS / 2 + 1 of them), while the B operand keeps DeepGemm's ring of NS stages
// of 32 k.  Every step still issues the same number of loads: its B stage and HALF of an A
// super-stage (the upper rows on even steps, the lower rows on odd steps), each A instruction
// covering 8 rows x 128 bytes.  Super-stage v is multiplied in steps 2v and 2v + 1 and loaded
// in steps 2v - 2 NSA + 2 and 2v - 2 NSA + 3, into the slot freed after step 2v - 2 NSA + 1;
// with NSA = NS / 2 + 1 its last load is issued NS - 2 steps of loads before the barrier that
// needs it, which is exactly DeepGemm's distance for B, so one vmcnt value serves both.
//
//   A super-stage [BM][64 k]: 16-byte slot c of row r sits at position c ^ ((r >> 1) & 7): the 16
//                             rows a quarter-wave reads cover all 16 bank groups of 16 bytes.
//   B stage, fragment reads, the step's structure (MFMAs, fragment prefetch, ONE barrier between
//   the two 16-k sub-steps), the epilogue: as in DeepGemm.
#pragma once
#include "ffuse_gemm1.h"

namespace ffuse {

template <typename T, bool GATED, int BM, int BH, int WM, int WN, int NS_ = 4, bool NT_ = false>
struct WideGemm : FirstGemm<T, GATED, BM, BH, WM, WN> {
    typedef FirstGemm<T, GATED, BM, BH, WM, WN> Base;
    typedef typename Base::vec8 vec8;
    using Base::G; using Base::HT; using Base::MT; using Base::WHR; using Base::WMR;
    static_assert(BH == 64 || BH == 128 || BH == 256, "unit swizzle is defined for rows of 4, 8 or 16 units of 32 bytes");
    static __device__ __forceinline__ uint32_t bkey(uint32_t k) { return BH == 64 ? (k & 2u) : ((k & 3u) << 1); }
    static_assert(BM == 32 || BM == 64 || BM == 128 || BM == 256, "rows");
    static constexpr int NS = NS_;                     // B stages in flight (ring)
    static constexpr int NSA = NS / 2 + 1;             // A super-stages (ring)
    static constexpr int XBW = BM * 128;               // bytes of one A super-stage
    static constexpr int WB = BH * 64;                 // bytes of one B stage (one matrix)
    static constexpr int BST = G * WB;
    static constexpr int A_RING = NSA * XBW;
    static constexpr int LDS_BYTES = A_RING + NS * BST;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    // BM = 32: a super-stage is 4 instructions, one per wave, all issued on even steps; odd steps
    // issue no A load (any NS - 2 consecutive steps still issue the same number of loads per wave)
    static constexpr bool SMALL_A = BM == 32;
    static constexpr int XI = SMALL_A ? 1 : BM / 64;   // A load instructions per wave per step
    static constexpr int QH = SMALL_A ? 0 : BM / 16;   // A instructions per step, whole workgroup
    static constexpr int ROWB = BH * 2;
    static constexpr int RPI = 1024 / ROWB;
    static constexpr int BI = 32 / RPI / 4;
    static constexpr int NLOAD = XI + G * BI;
    static constexpr int NM = HT * MT * G;
    static constexpr int NR = MT + HT * G;
    // loads a wave issues in NS - 2 consecutive steps: what may still be in flight at a step's barrier
    static constexpr int WAITN = SMALL_A ? (NS - 2) * G * BI + (NS - 2) / 2 : (NS - 2) * NLOAD;
    static_assert((NS == 4 || NS == 8) && WAITN <= 63, "ring depth: the vmcnt field holds 6 bits");

    struct Ctx {
        __amdgpu_buffer_rsrc_t rx, rw[G];
        // this lane's A chunk in the wave's first instruction of an EVEN step: global byte offset at k = 0
        // and k within the super-stage.  Instruction j is 8 j rows further down, and its rows' swizzle
        // key differs by 4 when j is odd: chunk ^ 4, i.e. k ^ 32 and the offset +- 64 bytes (xflip).
        uint32_t xoff, xk;
        int32_t xflip;
        uint32_t xstep;         // bytes between the rows of consecutive instructions (8 rows)
        uint32_t xhalf;         // added on odd steps: BM / 2 rows further down
        uint32_t boff[BI];
        uint32_t abase, brow;
        int KX;
        uint32_t lds_a, lds_b;  // LDS offsets (within a super-stage / a B stage) of this wave's first instruction
        uint32_t rdx[MT], rdw[HT];
    };

    static __device__ __forceinline__ void init_a(Ctx& c, const void* A, uint32_t a_bytes, uint32_t base_bytes,
                                                  uint32_t row0, uint32_t lda, int kx, int tid) {
        const uint32_t wave = tid >> 6, lane = tid & 63;
        c.rx = make_rsrc(A, a_bytes);
        c.KX = kx;
        c.abase = base_bytes;
        c.xhalf = (uint32_t)(BM / 2) * lda * 2u;
        c.xstep = 8u * lda * 2u;
        // instruction q of a super-stage fills rows 8q .. 8q + 7: lane i -> row 8q + (i >> 3), slot i & 7,
        // which holds chunk slot ^ ((row >> 1) & 7).  (Rows BM / 2 further down have the same key.)
        const uint32_t q = wave * XI;
        const uint32_t row = 8u * q + (lane >> 3);
        const uint32_t chunk = (lane & 7u) ^ ((row >> 1) & 7u);
        c.xk = 8u * chunk;
        c.xoff = ((row0 + row) * lda + 8u * chunk) * 2u;
        c.xflip = (chunk & 4u) ? -64 : 64;
    }
    static __device__ __forceinline__ void init_b(Ctx& c, const void* B, const void* B3, uint32_t b_bytes,
                                                  uint32_t ldb, uint32_t ncols, uint32_t n0, int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        c.rw[0] = make_rsrc(B, b_bytes);
        if (GATED) c.rw[G - 1] = make_rsrc(B3, b_bytes);
        c.brow = ldb * 2u;
#pragma unroll
        for (int j = 0; j < BI; ++j) {
            const uint32_t byte = (uint32_t)(wave * BI + j) * 1024u + 16u * lane;
            const uint32_t k = byte / ROWB, pp = (byte % ROWB) / 16u;
            const uint32_t p = ((((pp >> 1) ^ bkey(k)) << 1) | (pp & 1u));
            const uint32_t col = n0 + 8u * p;
            c.boff[j] = col < ncols ? (k * ldb + col) * 2u : kOob;
        }
    }
    static __device__ __forceinline__ void init_lds(Ctx& c, int tid) {
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
        const int wm = wave % WM, wn = wave / WM;
        const uint32_t x = lane & 31, h = lane >> 5;
        c.lds_a = (uint32_t)(wave * XI) * 1024u;
        c.lds_b = (uint32_t)(wave * BI) * 1024u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint32_t row = wm * WMR + 32 * mt + x;
            c.rdx[mt] = row * 128u + ((h ^ ((row >> 1) & 7u)) << 4);
        }
        const uint32_t gidx = lane >> 4, jj = (lane >> 2) & 3u, q = lane & 3u;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            const uint32_t u = (uint32_t)(wn * WHR + 32 * ht) / 16u + (gidx & 1u);
            c.rdw[ht] = (8u * (gidx >> 1) + jj) * ROWB + ((u ^ bkey(jj)) * 32u) + 8u * q;
        }
    }

    static __device__ __forceinline__ void lds_dma16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t lds) {
        asm volatile("s_mov_b32 m0, %1\n\tbuffer_load_dwordx4 %0, %2, 0 offen lds"
                     :: "v"(voff), "s"(lds), "s"(r) : "memory", "m0");
    }
    static __device__ __forceinline__ void lds_dma16_nt(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t lds) {
        asm volatile("s_mov_b32 m0, %1\n\tbuffer_load_dwordx4 %0, %2, 0 offen nt lds"
                     :: "v"(voff), "s"(lds), "s"(r) : "memory", "m0");
    }

    // What a step loads: half `par` (0: upper rows, 1: lower rows) of the A super-stage that starts at
    // column kx into super-stage slot `sa`, and the B stage of rows kw.. into stage slot `sb`.
    struct Load {
        uint32_t sa, sb;   // LDS byte addresses of the A slot / B slot
        int kx, kw, par;
        bool bvalid;
    };
    // load instruction i of the step
    static __device__ __forceinline__ void issue_one(const Ctx& c, const Load& l, int xlim, int i) {
        if (i < XI) {
            if (SMALL_A && l.par != 0) return;
            const uint32_t xk = (i & 1) ? (c.xk ^ 32u) : c.xk;
            const bool ok = (l.kx + (int)xk) < xlim && c.abase != kOob;
            const uint32_t half = SMALL_A ? 0u : (uint32_t)l.par;
            const uint32_t xo = c.xoff + (uint32_t)i * c.xstep + ((i & 1) ? (uint32_t)c.xflip : 0u);
            lds_dma16(c.rx, ok ? xo + half * c.xhalf + c.abase + (uint32_t)l.kx * 2u : kOob,
                      l.sa + c.lds_a + half * (uint32_t)(QH * 1024) + (uint32_t)i * 1024u);
        } else {
            const int which = (i - XI) / BI, j = (i - XI) % BI;
            const uint32_t off = c.boff[j];
            const uint32_t vo = (off == kOob || !l.bvalid) ? kOob : off + (uint32_t)l.kw * c.brow;
            const uint32_t la = l.sb + c.lds_b + (uint32_t)which * WB + (uint32_t)j * 1024u;
            if (NT_) lds_dma16_nt(c.rw[which], vo, la);
            else lds_dma16(c.rw[which], vo, la);
        }
    }
    template <int N> static __device__ __forceinline__ void loads_in_flight_at_most() {
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
    }

    struct Frags {
        vec8 b[MT];
        vec8 a[HT];
        vec8 a3[GATED ? HT : 1];
    };
    static __device__ __forceinline__ vec8 read_b_frag(const char* smem, uint32_t off) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(smem + off));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(smem + off + 4 * ROWB));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(vec8, v);
    }
    // fragment read number i of the 16-k sub-step that starts at k = 16 * q16 (q16 = 0..3) of the A
    // super-stage `pa`, and at k = 16 * (q16 & 1) of the B stage `pb`
    static __device__ __forceinline__ void read_one(const char* pa, const char* pb, const Ctx& c, int q16, int i, Frags& f) {
        const uint32_t kxor = (uint32_t)(q16 << 5), kadd = (uint32_t)(16 * (q16 & 1)) * ROWB;
        if (i == 0) { f.b[0] = lds_read16<vec8>(pa, c.rdx[0] ^ kxor); return; }
        if (i == 1) { f.a[0] = read_b_frag(pb, c.rdw[0] + kadd); return; }
        int j = i - 2;
        if (GATED) {
            if (j == 0) { f.a3[0] = read_b_frag(pb + WB, c.rdw[0] + kadd); return; }
            j -= 1;
        }
        if (j < MT - 1) { f.b[j + 1] = lds_read16<vec8>(pa, c.rdx[j + 1] ^ kxor); return; }
        j -= MT - 1;
        const int ht = 1 + j / G;
        if (!GATED || (j % G) == 0) f.a[ht] = read_b_frag(pb, c.rdw[ht] + kadd);
        else f.a3[ht] = read_b_frag(pb + WB, c.rdw[ht] + kadd);
    }
    static __device__ __forceinline__ void mma_one(const Frags& f, int i, f32x16 (&acc)[HT][MT],
                                                   f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
        const int ht = i / (MT * G), r = i % (MT * G);
        if (!GATED || r < MT) acc[ht][r % MT] = Mma<T>::mma(f.a[ht], f.b[r % MT], acc[ht][r % MT]);
        else acc3[GATED ? ht : 0][GATED ? r - MT : 0] = Mma<T>::mma(f.a3[GATED ? ht : 0], f.b[r - MT], acc3[GATED ? ht : 0][GATED ? r - MT : 0]);
    }

    // One step of 32 k.  (pa, qa): the A super-stage being multiplied and which half of it (0 / 2: the
    // 16-k quarter the step starts at); pb: its B stage; (na, nqa, nb): the same for the next step.
    static __device__ __forceinline__ void step(const char* pa, int qa, const char* pb, const char* na, int nqa, const char* nb,
                                                const Ctx& c, const Load& l, int xlim, Frags (&f)[2],
                                                f32x16 (&acc)[HT][MT], f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            mma_one(f[0], i, acc, acc3);
#pragma unroll
            for (int e = (i * NR) / NM; e < ((i + 1) * NR) / NM; ++e) read_one(pa, pb, c, qa + 1, e, f[1]);
#pragma unroll
            for (int e = (i * NLOAD) / NM; e < ((i + 1) * NLOAD) / NM; ++e) issue_one(c, l, xlim, e);
            __builtin_amdgcn_sched_barrier(0);
        }
        loads_in_flight_at_most<WAITN>();
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            mma_one(f[1], i, acc, acc3);
#pragma unroll
            for (int e = (i * NR) / NM; e < ((i + 1) * NR) / NM; ++e) read_one(na, nb, c, nqa, e, f[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // Issues, ahead of time, this wave's B loads of the first NS - 1 stages of the stream [kbegin, kend): the
    // data lands where a later run() over the same stream loads it again, which then finds the lines in L2
    // instead of in DRAM.  The caller must own the LDS (nobody reads or loads it meanwhile).
    static __device__ __forceinline__ void prefetch_b(char* smem, const Ctx& c, int kbegin, int kend) {
        const int KT = (kend - kbegin + 31) / 32;
        const uint32_t b_lds = (uint32_t)(uintptr_t)smem + (uint32_t)A_RING;
#pragma unroll
        for (int sb = 0; sb < NS - 1; ++sb) {
            const Load l{0u, b_lds + (uint32_t)(sb * BST), 0, kbegin + 32 * sb, 0, sb < KT};
#pragma unroll
            for (int i = XI; i < NLOAD; ++i) issue_one(c, l, 0, i);
        }
    }

    static __device__ __forceinline__ void run(char* smem, const Ctx& c, int kbegin, int kend, f32x16 (&acc)[HT][MT],
                                               f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1], int tid) {
        (void)tid;
        Base::zero(acc, acc3);
        const int KT = (kend - kbegin + 31) / 32;
        const int xlim = kend < c.KX ? kend : c.KX;
        const uint32_t a_lds = (uint32_t)(uintptr_t)smem, b_lds = a_lds + (uint32_t)A_RING;
        char* bring = smem + A_RING;
        Frags f[2];
        // fill: super-stages 0 .. NSA - 2 (both halves) and B stages 0 .. NS - 2, interleaved in the order
        // the steady state would have issued them, so that the one vmcnt value holds from the first step on
#pragma unroll
        for (int u = 0; u < NSA - 1; ++u) {
#pragma unroll
            for (int par = 0; par < 2; ++par) {
                const Load l{a_lds + (uint32_t)(u * XBW), 0u, kbegin + 64 * u, 0, par, false};
#pragma unroll
                for (int i = 0; i < XI; ++i) issue_one(c, l, xlim, i);
            }
#pragma unroll
            for (int d = 0; d < 2; ++d) {
                const int sb = 2 * u + d;
                if (sb <= NS - 2) {
                    const Load l{0u, b_lds + (uint32_t)(sb * BST), 0, kbegin + 32 * sb, 0, sb < KT};
#pragma unroll
                    for (int i = XI; i < NLOAD; ++i) issue_one(c, l, xlim, i);
                }
            }
        }
        loads_in_flight_at_most<WAITN>();
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NR; ++i) read_one(smem, bring, c, 0, i, f[0]);
        int sa = 0;          // slot of the super-stage being multiplied
        for (int s = 0; s < KT; s += 2) {
            const int sa_ld = sa == 0 ? NSA - 1 : sa - 1;          // slot of super-stage (s >> 1) + NSA - 1
            const int sa_nx = sa == NSA - 1 ? 0 : sa + 1;
            const char* pa = smem + sa * XBW;
            const char* pan = smem + sa_nx * XBW;
            const int kld = kbegin + 64 * ((s >> 1) + NSA - 1);
            {   // even step s: first half of the super-stage, B stage s
                const Load l{a_lds + (uint32_t)(sa_ld * XBW), b_lds + (uint32_t)(((s + NS - 1) & (NS - 1)) * BST), kld,
                             kbegin + 32 * (s + NS - 1), 0, s + NS - 1 < KT};
                step(pa, 0, bring + (s & (NS - 1)) * BST, pa, 2, bring + ((s + 1) & (NS - 1)) * BST, c, l, xlim, f, acc, acc3);
            }
            if (s + 1 < KT) {   // odd step s + 1: second half, B stage s + 1; next: super-stage sa_nx, first half
                const Load l{a_lds + (uint32_t)(sa_ld * XBW), b_lds + (uint32_t)(((s + NS) & (NS - 1)) * BST), kld,
                             kbegin + 32 * (s + NS), 1, s + NS < KT};
                step(pa, 2, bring + ((s + 1) & (NS - 1)) * BST, pan, 0, bring + ((s + 2) & (NS - 1)) * BST, c, l, xlim, f, acc, acc3);
            }
            sa = sa_nx;
        }
        loads_in_flight_at_most<0>();
        __syncthreads();
    }
};

}  // namespace ffuse
