// Block GEMM with LDS-direct loads: same contract and accumulator layout as FirstGemm
// (ffuse_gemm0.h), but operand tiles go from global memory STRAIGHT into LDS
// (buffer_load_dwordx4 ... lds, 16 bytes per lane, no staging registers, no LDS store
// instructions), the weight operand is transposed on the way OUT of LDS by
// ds_read_b64_tr_b16 instead of by a register transpose on the way in, and the stages form
// a ring of FOUR stages of 32 k each, so that loads are issued three stages (1.5 K steps of
// 64) before their data is multiplied.
//
// Why so deep: measured on this chip the L2 delivers about 30 bytes per clock per CU, which
// for a 256 x 256 tile is the same time as the tile's MFMAs.  With both units near saturation
// the L2 queues are long (over 1500 clocks) and only a deep ring keeps the matrix cores fed.
//
//   A stage [BM][32 k] : rows of 64 bytes; 16-byte slot c of row r sits at position
//                        c ^ ((r >> 2) & 3) (rows r, r+4, r+8, r+12 share banks).  The swizzle
//                        is realised by WHICH global chunk each lane fetches, because an
//                        LDS-direct load writes lane i's 16 bytes at base + 16*i.
//   B stage [32 k][BH] : kept in its global orientation, rows of BH*2 bytes; 32-byte units
//                        within a row are XOR-swizzled with a key of k so that the four
//                        k-rows one transposing read touches fall into different banks.
//   ds_read_b64_tr_b16 : in every group of 16 lanes, lanes 4j..4j+3 supply the address of 16
//                        consecutive n of row k0 + j; lane L receives (k0..k0+3, n0 + L).
//                        Two of them give the 8 consecutive k an MFMA operand register holds.
//
// Step s multiplies stage s & 3 in two sub-steps of 16 k:
//   sub-step 0: MFMAs on f[0]; reads the fragments of sub-step 1 into f[1]; issues the
//               loads of step s + 3 into stage (s + 3) & 3 (last read in step s - 1);
//   then      : waits until this wave's loads of step s + 1 have landed and its LDS reads are
//               complete; ONE barrier;
//   sub-step 1: MFMAs on f[1]; reads the fragments of step s + 1, sub-step 0, into f[0].
// After the barrier of step s every wave is done reading stage s & 3 and every wave's part
// of stage (s + 1) & 3 is in LDS; the stage written after it, (s + 4) & 3 = s & 3, is
// written by loads issued in step s + 1, i.e. after the barrier.
#pragma once
#include "ffuse_gemm0.h"

namespace ffuse {

typedef __attribute__((ext_vector_type(4))) short s16x4;

// NS_: stages in the ring (a power of two): loads run NS_ - 1 stages ahead.  Four keeps a 256 x 256
// tile fed.  (Row blocks below 256 rows use WideGemm, ffuse_gemm2.h, which loads the row operand
// in whole cache lines.)
template <typename T, bool GATED, int BM, int BH, int WM, int WN, int NS_ = 4>
struct DeepGemm : FirstGemm<T, GATED, BM, BH, WM, WN> {
    typedef FirstGemm<T, GATED, BM, BH, WM, WN> Base;
    typedef typename Base::vec8 vec8;
    using Base::G; using Base::HT; using Base::MT; using Base::WHR; using Base::WMR;
    static_assert(BH == 64 || BH == 128 || BH == 256, "unit swizzle is defined for rows of 4, 8 or 16 units of 32 bytes");
    // XOR key of the 32-byte units of B row k: the four k-rows one transposing read touches
    // must land in four different 32-byte bank groups.  Rows of 256 or 512 bytes all start in
    // the same bank, so each of the four gets its own key; rows of 128 bytes alternate
    // between two banks already, so rows k and k + 2 need different keys.
    static __device__ __forceinline__ uint32_t bkey(uint32_t k) { return BH == 64 ? (k & 2u) : ((k & 3u) << 1); }
    static_assert(BM % 64 == 0, "every wave issues the same number of whole load instructions");
    static constexpr int NS = NS_;                     // stages in the ring
    static constexpr int XB = BM * 64;                 // bytes of one A stage
    static constexpr int WB = BH * 64;                 // bytes of one B stage (one matrix)
    static constexpr int STAGE = XB + G * WB;
    static constexpr int LDS_BYTES = NS * STAGE;
    static constexpr int XI = BM / 64;                 // A load instructions per wave per stage
    static constexpr int ROWB = BH * 2;                // bytes of one B row in LDS
    static constexpr int RPI = 1024 / ROWB;            // B rows per load instruction
    static constexpr int BI = 32 / RPI / 4;            // B load instructions per wave per matrix
    static constexpr int NLOAD = XI + G * BI;          // load instructions per wave per stage
    static constexpr int NM = HT * MT * G;             // MFMAs per wave per sub-step
    static constexpr int NR = MT + HT * G;             // fragment reads per wave per sub-step
    static_assert((NS == 4 || NS == 8 || NS == 16) && (NS - 2) * NLOAD <= 63, "ring depth: the vmcnt field holds 6 bits");

    struct Ctx {
        __amdgpu_buffer_rsrc_t rx, rw[G];
        uint32_t xoff[XI];      // global byte offset of this lane's A chunk, per instruction, at k = 0
        uint32_t xk;            // k of this lane's A chunk within the step
        uint32_t boff[BI];      // global byte offset of this lane's B chunk, per instruction, at k = 0
        uint32_t abase;         // uniform byte offset added to A offsets (kOob: reads as zero)
        uint32_t brow;          // bytes per global B row
        int KX;                 // extent of A along k
        uint32_t lds_a, lds_b;  // uniform LDS byte offsets of this wave's first A / B instruction
        uint32_t rdx[MT];       // LDS read offsets: A fragments (sub-step 0)
        uint32_t rdw[HT];       //                   B fragments (sub-step 0, first half)
    };

    static __device__ __forceinline__ void init_a(Ctx& c, const void* A, uint32_t a_bytes, uint32_t base_bytes,
                                                  uint32_t row0, uint32_t lda, int kx, int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        c.rx = make_rsrc(A, a_bytes);
        c.KX = kx;
        c.abase = base_bytes;
        // lane i of an instruction fills slot i & 3 of the row (i >> 2) rows below the
        // instruction's first: the chunk that lives there is slot ^ ((row >> 2) & 3), which is
        // the same for every instruction of a wave (their first rows are 16 apart)
        const uint32_t first = (uint32_t)(wave * XI) * 16u;
        const uint32_t chunk = (lane & 3) ^ (((first + (lane >> 2)) >> 2) & 3u);
        c.xk = 8u * chunk;
#pragma unroll
        for (int j = 0; j < XI; ++j) {
            const uint32_t row = first + (uint32_t)j * 16u + (lane >> 2);
            c.xoff[j] = ((row0 + row) * lda + 8u * chunk) * 2u;
        }
    }
    static __device__ __forceinline__ void init_b(Ctx& c, const void* B, const void* B3, uint32_t b_bytes,
                                                  uint32_t ldb, uint32_t ncols, uint32_t n0, int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        c.rw[0] = make_rsrc(B, b_bytes);
        if (GATED) c.rw[G - 1] = make_rsrc(B3, b_bytes);
        c.brow = ldb * 2u;
#pragma unroll
        for (int j = 0; j < BI; ++j) {
            const uint32_t byte = (uint32_t)(wave * BI + j) * 1024u + 16u * lane;   // within the B stage
            const uint32_t k = byte / ROWB, pp = (byte % ROWB) / 16u;             // row, 16-byte position
            const uint32_t p = ((((pp >> 1) ^ bkey(k)) << 1) | (pp & 1u));   // global chunk stored there
            const uint32_t col = n0 + 8u * p;
            c.boff[j] = col < ncols ? (k * ldb + col) * 2u : kOob;
        }
    }
    static __device__ __forceinline__ void init_lds(Ctx& c, int tid) {
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // uniform: feeds M0
        const int wm = wave % WM, wn = wave / WM;
        const uint32_t x = lane & 31, h = lane >> 5;
        c.lds_a = (uint32_t)(wave * XI) * 1024u;
        c.lds_b = XB + (uint32_t)(wave * BI) * 1024u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint32_t row = wm * WMR + 32 * mt + x;
            c.rdx[mt] = row * 64u + ((h ^ ((row >> 2) & 3u)) << 4);
        }
        const uint32_t gidx = lane >> 4, jj = (lane >> 2) & 3u, q = lane & 3u;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            const uint32_t u = (uint32_t)(wn * WHR + 32 * ht) / 16u + (gidx & 1u);
            c.rdw[ht] = XB + (8u * (gidx >> 1) + jj) * ROWB + ((u ^ bkey(jj)) * 32u) + 8u * q;   // bkey(k) = bkey(jj): k = jj mod 4
        }
    }

    // One LDS-direct load: 16 bytes per lane from buffer `r` at byte offset `voff` to LDS bytes
    // [lds, lds + 1024).  Inline assembly on purpose: with the compiler's builtin every
    // transposing LDS read is preceded by a conservative s_waitcnt vmcnt(0).  The kernel
    // counts and waits for these loads itself.
    static __device__ __forceinline__ void lds_dma16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t lds) {
        asm volatile("s_mov_b32 m0, %1\n\tbuffer_load_dwordx4 %0, %2, 0 offen lds"
                     :: "v"(voff), "s"(lds), "s"(r) : "memory", "m0");
    }
    // load instruction i of the step whose A columns start at kx and whose B rows start at kw.
    // A chunks at or past column xlim, and everything when `valid` is false, load nothing from
    // memory (out-of-range offsets: LDS receives zeros) -- the instruction is issued all the
    // same so that every step puts the same number of loads in flight.
    static __device__ __forceinline__ void issue_one(char* stage, const Ctx& c, int kx, int kw, int xlim, bool valid, int i) {
        if (i < XI) {
            const bool ok = valid && (kx + (int)c.xk) < xlim && c.abase != kOob;
            lds_dma16(c.rx, ok ? c.xoff[i] + c.abase + (uint32_t)kx * 2u : kOob,
                          (uint32_t)(uintptr_t)stage + c.lds_a + (uint32_t)i * 1024u);
        } else {
            const int which = (i - XI) / BI, j = (i - XI) % BI;
            const uint32_t off = c.boff[j];
            const uint32_t vo = (off == kOob || !valid) ? kOob : off + (uint32_t)kw * c.brow;
            const uint32_t la = (uint32_t)(uintptr_t)stage + c.lds_b + (uint32_t)which * WB + (uint32_t)j * 1024u;
            lds_dma16(c.rw[which], vo, la);
        }
    }
    static __device__ __forceinline__ void issue(char* stage, const Ctx& c, int kx, int kw, int xlim, bool valid) {
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) issue_one(stage, c, kx, kw, xlim, valid, i);
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
    // fragment read number i of sub-step ks (0 or 1), in the order the MFMAs need them
    static __device__ __forceinline__ void read_one(const char* smem, const Ctx& c, int ks, int i, Frags& f) {
        const uint32_t kxor = (uint32_t)(ks << 5), kadd = (uint32_t)(16 * ks) * ROWB;
        if (i == 0) { f.b[0] = lds_read16<vec8>(smem, c.rdx[0] ^ kxor); return; }
        if (i == 1) { f.a[0] = read_b_frag(smem, c.rdw[0] + kadd); return; }
        int j = i - 2;
        if (GATED) {
            if (j == 0) { f.a3[0] = read_b_frag(smem + WB, c.rdw[0] + kadd); return; }
            j -= 1;
        }
        if (j < MT - 1) { f.b[j + 1] = lds_read16<vec8>(smem, c.rdx[j + 1] ^ kxor); return; }
        j -= MT - 1;
        const int ht = 1 + j / G;
        if (!GATED || (j % G) == 0) f.a[ht] = read_b_frag(smem, c.rdw[ht] + kadd);
        else f.a3[ht] = read_b_frag(smem + WB, c.rdw[ht] + kadd);
    }
    static __device__ __forceinline__ void mma_one(const Frags& f, int i, f32x16 (&acc)[HT][MT],
                                                   f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
        const int ht = i / (MT * G), r = i % (MT * G);
        if (!GATED || r < MT) acc[ht][r % MT] = Mma<T>::mma(f.a[ht], f.b[r % MT], acc[ht][r % MT]);
        else acc3[GATED ? ht : 0][GATED ? r - MT : 0] = Mma<T>::mma(f.a3[GATED ? ht : 0], f.b[r - MT], acc3[GATED ? ht : 0][GATED ? r - MT : 0]);
    }

    // One step of 32 k (see the struct comment): multiplies `cur`, leaves the first fragments
    // of `nxt` in f[0], issues the loads of a later step (A columns from kx, B rows from kw)
    // into `ld`.
    static __device__ __forceinline__ void step(const char* cur, const char* nxt, char* ld, const Ctx& c,
                                                int kx, int kw, int xlim, bool valid,
                                                Frags (&f)[2], f32x16 (&acc)[HT][MT],
                                                f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1]) {
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            mma_one(f[0], i, acc, acc3);
#pragma unroll
            for (int e = (i * NR) / NM; e < ((i + 1) * NR) / NM; ++e) read_one(cur, c, 1, e, f[1]);
#pragma unroll
            for (int e = (i * NLOAD) / NM; e < ((i + 1) * NLOAD) / NM; ++e) issue_one(ld, c, kx, kw, xlim, valid, e);
            __builtin_amdgcn_sched_barrier(0);
        }
        loads_in_flight_at_most<(NS - 2) * NLOAD>();   // all but the oldest of the stages in flight may still be on their way
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            mma_one(f[1], i, acc, acc3);
#pragma unroll
            for (int e = (i * NR) / NM; e < ((i + 1) * NR) / NM; ++e) read_one(nxt, c, 0, e, f[0]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // The loads that fill the ring for a stream of steps over [kbegin, kend): stages 0..NS-2 <- steps 0..NS-2.
    // Nothing is waited for.  May be called while slot NS - 1 of the ring is still in use as the staging
    // area of the previous tile's epilogue (store_tile_lds with SLAB): the fill of a workgroup's next item
    // then travels under that epilogue, and run(..., prefilled = true) picks it up.
    static __device__ __forceinline__ void prefill(char* smem, const Ctx& c, int kbegin, int kend) {
        const int KT = (kend - kbegin + 31) / 32;
        const int xlim = kend < c.KX ? kend : c.KX;
#pragma unroll
        for (int j = 0; j < NS - 1; ++j) issue(smem + j * STAGE, c, kbegin + 32 * j, kbegin + 32 * j, xlim, KT > j);
    }
    static constexpr int STAGING_SLOT = (NS - 1) * STAGE;   // where such an epilogue may stage (STAGE bytes)
    // Waits for the first stage of a filled ring and leaves the fragments of step 0 in f[0].  after_stores:
    // the fill was issued before a slab epilogue, whose WMR / EPI_RPI global stores per wave are younger
    // than every load of the fill and count in the same counter, which is decremented in issue order: once
    // no more than that many operations are outstanding, the whole fill has landed.
    static __device__ __forceinline__ void await_fill(char* smem, const Ctx& c, bool after_stores, Frags (&f)[2]) {
        if (after_stores) loads_in_flight_at_most<WMR / Base::EPI_RPI>();
        else loads_in_flight_at_most<(NS - 2) * NLOAD>();
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NR; ++i) read_one(smem, c, 0, i, f[0]);
    }
    // Fills the ring for a stream of steps that starts at (kx, kw): stages 0..NS-2 <- steps
    // 0..NS-2, and leaves the fragments of step 0 in f[0].  `nvalid` says how many of them exist.
    static __device__ __forceinline__ void prime(char* smem, const Ctx& c, int kx, int kw, int xlim, int nvalid, Frags (&f)[2]) {
#pragma unroll
        for (int j = 0; j < NS - 1; ++j) issue(smem + j * STAGE, c, kx + 32 * j, kw + 32 * j, xlim, nvalid > j);
        await_fill(smem, c, false, f);
    }
    // After the last step: the loads still in flight target stages nobody reads any more, but
    // LDS must be quiet, and every wave done with it, before anybody reuses it.
    static __device__ __forceinline__ void drain() {
        loads_in_flight_at_most<0>();
        __syncthreads();
    }

    static __device__ __forceinline__ void run(char* smem, const Ctx& c, int kbegin, int kend, f32x16 (&acc)[HT][MT],
                                               f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1], int tid,
                                               bool prefilled = false, uint64_t* t_loop = nullptr) {
        (void)tid;
        Base::zero(acc, acc3);
        const int KT = (kend - kbegin + 31) / 32;
        const int xlim = kend < c.KX ? kend : c.KX;
        Frags f[2];
        if (!prefilled) prefill(smem, c, kbegin, kend);
        await_fill(smem, c, prefilled, f);
        if (t_loop) *t_loop = wall_clock64();
        for (int s = 0; s < KT; ++s) {
            const char* cur = smem + (s & (NS - 1)) * STAGE;
            const char* nxt = smem + ((s + 1) & (NS - 1)) * STAGE;
            char* ld = smem + ((s + NS - 1) & (NS - 1)) * STAGE;
            const int kl = kbegin + (s + NS - 1) * 32;
            step(cur, nxt, ld, c, kl, kl, xlim, s + NS - 1 < KT, f, acc, acc3);
        }
        drain();
    }
};

}  // namespace ffuse
