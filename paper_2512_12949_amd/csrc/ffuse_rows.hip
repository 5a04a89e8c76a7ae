// Fused chain, "rows" family (row-stationary): a workgroup owns 64 rows of X and ALL N2 output
// columns of those rows, walks through the hidden dimension in chunks of 64 columns, and keeps
//   * its rows of X in REGISTERS for the whole walk (each of the four waves holds a quarter of K),
//   * the running output block Y[64][N2] in fp32 accumulator registers (N2 <= 1024: 256 per lane),
//   * the activated chunk H[64][64] in LDS,
// so the M x N1 intermediate never exists outside the compute unit: nothing is exchanged between
// workgroups, nothing but Y is ever stored.  This is the paper's MLNK-style order (Sec. 4.2, LoopSchedule:
// the output block stays resident while the hidden dimension is walked) with the Resource Mapping of
// Sec. 4.2 ending at the second level (registers -> shared memory) because the per-chunk slice is small.
//
// Per chunk c (64 hidden columns) and wave w:
//   first product, K split over the waves (Sec. 4.1: a split reduction dimension needs an Add exchange
//   before the activation; Sec. 4.3 Rule 3): P_w[64][64] = X[:, Kq(w)] * W1[Kq(w), chunk] with X from
//   registers and W1 from the wave's PRIVATE LDS ring; the four partial tiles are exchanged through
//   LDS so that wave t ends up with the complete 32 x 32 tile t, applies the activation to complete
//   sums, rounds to the operand type and writes its tile of H;
//   second product: Y[:, cols(w)] += H * W2[chunk, cols(w)], wave w owning N2/4 output columns, H
//   from LDS and W2 from the same private ring.
// Every weight element is used by exactly one wave, so the weight stream needs no workgroup barrier:
// each wave issues LDS-direct loads (buffer_load ... lds) into its own ring of 4 KB slots, two to three
// slots ahead, and waits on its own vmcnt.  The only barriers are the two around the partial-tile exchange.
//
// What bounds it (measured, 32768 x 1024 x 8192 x 1024: matrix pipelines about half occupied): with 64 rows per
// workgroup a weight byte feeds 64 rows only, so per chunk a compute unit pulls 256 KB through its L2 -> LDS
// path -- at that path's 64 bytes per clock as long as the chunk's matrix instructions take -- and the eight
// L2s deliver 17 GB per call, 2.0 TB/s each, close to what an L2 delivers on hits.  The family trades that for
// memory traffic: the weights are filled into an XCD's L2 once per round of row blocks, X and Y cross the
// fabric once, nothing else does.  (Tried and dropped: the exchange of chunk c + 1 riding inside the second
// product of chunk c, with two H buffers -- no faster; and one plain
// 16-byte read per fragment in place of the two transposing reads -- no faster either: the LDS is not the limit.)
//
// Why X sits in registers: measured on this chip, 32 workgroups per XCD that each re-read a private
// 128 KB row block once per chunk evict each other from the 4 MB L2 completely (2 GiB of refills per
// call at M = 32768), while the weight chunks, which all 32 walk through together, are filled once.
#include <utility>

#include "ffuse_dev.h"
#include "ffuse_launch.h"

namespace ffuse {

typedef __attribute__((ext_vector_type(4))) short rows_s16x4;

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop whose index is a constant expression in
// every iteration.  (The step loop below indexes register arrays with it; a pragma-unrolled loop of that size
// is not always unrolled, and then those arrays move to scratch memory.)
template <class F, int... I> __device__ __forceinline__ void rows_static_for(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}

// A wave-private 4 KB slot [KR k][COLS n] of 16-bit weights in their global orientation (n contiguous).
// 32-byte units of a row are XOR-swizzled with a key of k so that the four k-rows one transposing read
// touches fall into different bank groups.
template <int COLS> struct RowsSlot {
    static_assert(COLS == 64 || COLS == 128, "rows of 128 or 256 bytes");
    static constexpr int ROWB = COLS * 2;
    static __device__ __forceinline__ uint32_t bkey(uint32_t k) { return COLS == 64 ? (k & 2u) : ((k & 3u) << 1); }
    // load instruction j (1 KB: lane i writes 16 bytes at 1024 j + 16 i) covers rows 1024 j / ROWB ...;
    // this lane's row within the instruction and the global 16-byte chunk of the row it must fetch
    static __device__ __forceinline__ uint32_t lane_row(int lane) { return (uint32_t)(16 * lane) / ROWB; }
    static __device__ __forceinline__ uint32_t lane_chunk(int lane) {
        const uint32_t k = lane_row(lane), pp = ((uint32_t)(16 * lane) % ROWB) / 16u;
        return (((pp >> 1) ^ bkey(k)) << 1) | (pp & 1u);
    }
    // byte offset, within a slot, of the first transposing read of the fragment "32 columns from 32 ht,
    // 16 k from row 0" for this lane (the second read is 4 rows further down)
    static __device__ __forceinline__ uint32_t frag_off(int ht, int lane) {
        const uint32_t gidx = lane >> 4, jj = (lane >> 2) & 3u, q = lane & 3u;
        const uint32_t u = 2u * ht + (gidx & 1u);
        return (8u * (gidx >> 1) + jj) * ROWB + ((u ^ bkey(jj)) * 32u) + 8u * q;
    }
    template <typename V> static __device__ __forceinline__ V read_frag(const char* p) {
        const rows_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) rows_s16x4*)(p));
        const rows_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) rows_s16x4*)(p + 4 * ROWB));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(V, v);
    }
};

__device__ __forceinline__ void rows_dma16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %1\n\tbuffer_load_dwordx4 %0, %2, 0 offen lds"
                 :: "v"(voff), "s"(lds), "s"(r) : "memory", "m0");
}
template <int N> __device__ __forceinline__ void rows_loads_in_flight_at_most() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// Every LDS read this wave has issued has delivered.  REQUIRED before an LDS-direct load is aimed at a slot
// the wave has read from: measured on this chip, the load's data can land before reads that were issued
// ahead of it have been served (the reads queue up when the LDS is saturated, the load's write does not).
__device__ __forceinline__ void rows_lds_reads_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// the same for all but the N LDS instructions issued last (LDS instructions of a wave complete in order; there
// must BE at least N younger ones, or the wait says nothing about the older)
template <int N> __device__ __forceinline__ void rows_lds_reads_older_done() { asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(N) : "memory"); }

// The first product's MFMA with its accumulator in ARCHITECTURAL registers.  The compiler gives all
// matrix instructions of a kernel one register form; this kernel's running output block fills all 256
// accumulation registers, so the small accumulator of the first product has to live in the other file, which
// only inline assembly can say.  Consequences handled here by hand (the compiler does not look inside): an
// accumulator is re-used every fourth instruction at the earliest (four tiles in rotation), far beyond the
// dependent-issue window, and rows_mfma_settle() separates the last of them from the first ordinary
// instruction that reads or writes the tiles.
template <typename T> struct RowsMmaV;
template <> struct RowsMmaV<__bf16> {
    static __device__ __forceinline__ void mma(bf16x8 a, bf16x8 b, f32x16& c) {
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
    }
};
template <> struct RowsMmaV<_Float16> {
    static __device__ __forceinline__ void mma(f16x8 a, f16x8 b, f32x16& c) {
        asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
    }
};
// 32 idle issue slots around the architectural-register MFMAs: the longest wait the ISA asks for between a
// matrix instruction and an ordinary read or overwrite of its registers is below that
__device__ __forceinline__ void rows_mfma_settle(f32x16 (&p)[2][2]) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(p[0][0]), "+v"(p[0][1]), "+v"(p[1][0]), "+v"(p[1][1]));
}

// complete sums of one 32 x 32 tile -> activation -> operand type -> H (rows of 128 bytes, 16-byte chunks
// swizzled with the row): register 4 q + e of lane (x, h) is row `hrow`, hidden column 32 ht + 8 q + 4 h + e
// of the chunk; groups of four columns at or past `nlim` (counted from this lane's first column) lie beyond
// N1 and are stored as zeros, so that whatever the weight slots held for them cannot reach the output
template <typename T, int ACT>
__device__ __forceinline__ void rows_write_h(const f32x16& s, char* hbuf, uint32_t hrow, uint32_t ht, uint32_t h, int nlim) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint2 o;
        o.x = pack2<T>(activate<ACT>(s[4 * q]), activate<ACT>(s[4 * q + 1]));
        o.y = pack2<T>(activate<ACT>(s[4 * q + 2]), activate<ACT>(s[4 * q + 3]));
        if (8 * q >= nlim) o.x = o.y = 0u;
        *reinterpret_cast<uint2*>(hbuf + lds_row_off(hrow, 4u * ht + q) + 8u * h) = o;
    }
}

// NKS: 16-k steps of the first product per wave (K <= 64 NKS); NT2: 32-column tiles of the output per
// wave (N2 <= 128 NT2), a multiple of 4.
//
// The weight stream of a wave is one endless sequence of 4 KB slots -- per chunk NKS / 2 slots of W1
// ([32 k][64 hidden columns]) and then 4 NT2 / 4 slots of W2 ([16 hidden][128 output columns]), chunk after
// chunk, row block after row block (the weights do not depend on the row block) -- through a ring of
// kRowsRing positions.  A slot is multiplied in two STEPS of four MFMAs; a step takes its two weight fragments
// from registers (set t % 3), and before its MFMAs are issued the two fragments of step t + 2 are read from LDS
// into the set that step t - 1 has just finished with: one step of 128 matrix cycles is less than the LDS latency
// under load, two cover it.  In the middle of a slot's first step every read of the slot has delivered
// (rows_lds_reads_older_done), and only then are the loads of the slot kRowsRing further down the stream aimed
// at its position, two in each of the slot's two steps.  The wait for a slot to have landed sits at the top of the step that first
// reads it.
template <typename T, int NKS, int NT2, bool RAGGED>
__global__ __launch_bounds__(256) void fused_rows_kernel(RowsArgs a) {
    typedef typename Mma<T>::vec8 vec8;
    typedef RowsSlot<64> S1;     // W1 slot: [32 k][64 hidden columns]
    typedef RowsSlot<128> S2;    // W2 slot: [16 hidden][128 output columns]
    constexpr int RING = kRowsRing, SLOT = 4096;
    constexpr int NH2 = NT2 / 4;            // 128-column halves of a wave's output range
    constexpr int NST1 = NKS;               // steps of the first product per chunk: one per 16 k
    constexpr int NST2 = 8 * NH2;           // steps of the second: (hidden step, half, pair of 32-column tiles)
    constexpr int NST = NST1 + NST2;        // steps per chunk; a slot is two steps
    constexpr int SPC = NST / 2;            // slots per chunk and wave
    constexpr int NS1 = NST1 / 2;
    constexpr int NW = 32 * NT2;            // output columns per wave
    constexpr int KQ = 16 * NKS;            // k range per wave
    static_assert(NKS % 2 == 0 && NT2 % 4 == 0 && SPC > RING, "slot arithmetic");
    // The first product's accumulator: with the output block in all 256 accumulation registers (NT2 = 8) it has to
    // live in ordinary registers, which only hand-written matrix instructions can say (RowsMmaV).  The compiler
    // does not know that their results arrive late: it must never copy those registers between two of them, which
    // holds only as long as it has no reason to -- no spare accumulation registers to park values in (seen once,
    // with NT2 = 4 and a few registers too many in flight: the tiles were parked in the idle half of the accumulation
    // file between two instructions, and a few hundred output elements per call came out wrong).  With half the
    // output block (NT2 = 4) there is room for the accumulator beside it, and the compiler's own instructions, whose
    // timing it knows, are used; so they are with half of X (NKS = 8), where the compiler finds room without
    // spilling inside the chunk loop.  Only the largest instantiation issues them by hand.
    constexpr bool P_BY_HAND = NT2 > 4 && NKS > 8;
    static_assert((RING - 1) * 4 <= 63, "vmcnt holds 6 bits");
    __shared__ __attribute__((aligned(16))) char smem[kRowsLdsBytes];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    char* const ring = smem + wave * (RING * SLOT);
    char* const part = smem + 4 * RING * SLOT;          // 12 partial tiles of 4 KB
    char* const hbuf = part + 12 * SLOT;                // H chunk [64][64], rows of 128 bytes
    const uint32_t ring_lds = (uint32_t)(uintptr_t)ring;

    const int K = a.K, N1 = a.N1, N2 = a.N2;
    const int NC = (N1 + 63) / 64;
    const int MB = (int)((a.M + 63) / 64);
    const __amdgpu_buffer_rsrc_t r1 = make_rsrc(a.W1, (uint32_t)((uint64_t)K * N1 * 2));
    const __amdgpu_buffer_rsrc_t r2 = make_rsrc(a.W2, (uint32_t)((uint64_t)N1 * N2 * 2));
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.X, (uint32_t)((uint64_t)a.M * K * 2));
    const int nrb = (MB > (int)blockIdx.x) ? (MB - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    if (nrb == 0) return;
    uint64_t t_wall = 0, t_core = 0;
    if (a.stats) { t_wall = wall_clock64(); t_core = clock64(); }

    // ---- lane constants of the weight stream -------------------------------------------------------
    // Every address of the stream is INSIDE its matrix: rows past the end are clamped to the last row and
    // columns past the end to column 0 (their products are multiplied by zeros of X, by the zeros rows_write_h
    // stores, or land in output columns that are never stored).  Loads that fetch nothing are avoided on
    // purpose: the ring's waits count on loads completing in the order they were issued.
    // W1 slot i of chunk c: rows wave KQ + 32 i + 8 j + lane/8, columns 64 c + 8 chunk1
    const int lrow1 = wave * KQ + (int)S1::lane_row(lane);
    const uint32_t colb1 = 16u * S1::lane_chunk(lane);
    const uint32_t base1 = (uint32_t)lrow1 * (uint32_t)N1 * 2u + colb1;
    const int klimb1 = (K - 1 - lrow1) * N1 * 2;      // byte offset of the last row, from this lane's first (may be negative)
    // W2 slot (ks2, half) of chunk c: rows 64 c + 16 ks2 + 4 j + lane/16, columns wave NW + 128 half + 8 chunk2
    const int lrow2 = (int)S2::lane_row(lane);
    const uint32_t colb2 = (uint32_t)(wave * NW) * 2u + 16u * S2::lane_chunk(lane);
    const uint32_t base2 = (uint32_t)lrow2 * (uint32_t)N2 * 2u + colb2;
    const int klimb2 = (N1 - 1 - lrow2) * N2 * 2;
    // read offsets of the fragments: the one for 32-column tile ht differs from tile 0's in bits 6.. of the
    // byte offset only (the unit index is 2 ht + (lane bit), XOR-ed with a key: the XOR commutes)
    const uint32_t rd1 = S1::frag_off(0, lane), rd2 = S2::frag_off(0, lane);
    // H fragment of hidden step ks2, rows 32 mt + x: lds_row_off(32 mt + x, 2 ks2 + h) = (hrd ^ (ks2 << 5)) + 4096 mt
    const uint32_t hrd = lds_row_off(lane & 31, lane >> 5);

    // Load j (0 .. 3) of slot `idx` (0 .. SPC-1) of chunk `c` into ring position `pos`.  The lane's constants are
    // made opaque per load: left alone, the compiler precomputes the addresses of all slots of a chunk and keeps
    // them in registers that this kernel does not have.  RAGGED says that some address of the stream can fall
    // outside its matrix and has to be clamped (K != 64 NKS, N1 % 64 != 0 or N2 != 128 NT2); for whole tiles the
    // address is one add.
    auto issue_one = [&](int idx, int c, int pos, int j) {
        const uint32_t lds = ring_lds + (uint32_t)pos * SLOT + 1024u * j;
        if (idx < NS1) {
            uint32_t b = base1;
            asm volatile("" : "+v"(b));
            const int rowb = (32 * idx + 8 * j) * N1 * 2;
            if constexpr (!RAGGED) {
                rows_dma16(r1, b + (uint32_t)(rowb + c * 128), lds);
            } else {
                uint32_t cb = colb1;
                int kl = klimb1;
                asm volatile("" : "+v"(kl), "+v"(cb));
                b += (128 * c + (int)cb < 2 * N1) ? (uint32_t)c * 128u : 0u - cb;
                rows_dma16(r1, b + (uint32_t)min(rowb, kl), lds);
            }
        } else {
            const int ks2 = (idx - NS1) / NH2, half = (idx - NS1) % NH2;
            uint32_t b = base2;
            asm volatile("" : "+v"(b));
            const int rowb = (64 * c + 16 * ks2 + 4 * j) * N2 * 2;
            if constexpr (!RAGGED) {
                rows_dma16(r2, b + (uint32_t)(rowb + 256 * half), lds);
            } else {
                uint32_t cb = colb2;
                int kl = klimb2;
                asm volatile("" : "+v"(kl), "+v"(cb));
                b += (256 * half + (int)cb < 2 * N2) ? 256u * half : 0u - cb;
                rows_dma16(r2, b + (uint32_t)min(rowb, kl), lds);
            }
        }
    };
    auto issue = [&](int idx, int c, int pos) {
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_one(idx, c, pos, j);
    };
    // fragment e (0 / 1) of step t (0 .. NST-1) from the slot at `sb`
    auto read_frag = [&](int t, const char* sb, int e) -> vec8 {
        if (t < NST1) return S1::template read_frag<vec8>(sb + (rd1 ^ (uint32_t)(e << 6)) + (t & 1) * 16 * S1::ROWB);
        return S2::template read_frag<vec8>(sb + (rd2 ^ (uint32_t)((2 * ((t - NST1) & 1) + e) << 6)));
    };

    // ---- prime: slots 0 .. RING-1 of chunk 0, then the fragments of steps 0 and 1
#pragma unroll
    for (int s = 0; s < RING; ++s) issue(s, 0, s);
    vec8 fr[3][2];
    rows_loads_in_flight_at_most<(RING - 1) * 4>();
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int e = 0; e < 2; ++e) fr[tt][e] = read_frag(tt, ring, e);
    int pos = 0;                                         // ring position of the slot being multiplied

    for (int rbi = 0; rbi < nrb; ++rbi) {
        const int64_t row0 = ((int64_t)blockIdx.x + (int64_t)rbi * gridDim.x) * 64;
        // ---- this wave's quarter of the row block, as MFMA operand fragments, into registers -------
        // (lane coordinates made opaque per row block: the address arithmetic below and in the output stores
        //  is loop invariant in part, and hoisted out of the row-block loop it would occupy registers that the
        //  main loop needs)
        uint32_t xo, ho;
        {
            uint32_t l = (uint32_t)lane;
            asm volatile("" : "+v"(l));
            xo = l & 31u; ho = l >> 5;
        }
        const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.Y, (uint32_t)((uint64_t)a.M * N2 * 2));
        vec8 xf[NKS][2];
        {
            const int kl = wave * KQ + 8 * (int)ho;      // this lane's k at ks = 0
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                // rows at or past M lie behind the end of the buffer: zeros
                const uint32_t rowoff = (uint32_t)(((uint64_t)row0 + 32 * mt + xo) * (uint64_t)K * 2u) + (uint32_t)kl * 2u;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    xf[ks][mt] = __builtin_bit_cast(vec8, buf_load16(rx, (kl + 16 * ks < K) ? rowoff + 32u * ks : kOob));
            }
        }
        // everything this wave has in flight lands here: the output stores of the previous row block complete in
        // no fixed order relative to loads, and the ring's waits below count loads only
        rows_loads_in_flight_at_most<0>();
        // (the compiler cannot see that wait; handing the fragments through an empty statement makes it place its
        //  own here, once, instead of a stricter one in front of every first use inside the chunk loop, where it
        //  would drain the weight ring)
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) asm volatile("" : "+v"(xf[ks][mt]));
        f32x16 yacc[NT2][2];
#pragma unroll
        for (int t = 0; t < NT2; ++t)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) yacc[t][mt][r] = 0.0f;

        for (int c = 0; c < NC; ++c) {
            const int cn = (c + 1 == NC) ? 0 : c + 1;   // (past the last chunk of the last row block the stream just goes on: a few slots nobody reads)
            f32x16 p[2][2];
#pragma unroll
            for (int ht = 0; ht < 2; ++ht)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) p[ht][mt][r] = 0.0f;
            if constexpr (P_BY_HAND) rows_mfma_settle(p);
            vec8 hb[2][2];                              // H fragments of hidden step ks2, set ks2 & 1
            rows_static_for([&](auto tc) {
                constexpr int t = decltype(tc)::value;
                constexpr int cur = t % 3, rds = (t + 2) % 3;       // fragment sets: multiplied now / read now (for step t + 2)
                constexpr int t2 = (t + 2) % NST;                   // the step whose fragments are read now
                constexpr bool first = (t & 1) == 0;                // first step of its slot
                const int pn = pos + 1 == RING ? 0 : pos + 1;       // position of the next slot: steps t + 1 (t odd) and t + 2 belong to it
                // ---- the next slot has landed (all but the youngest RING - 2 slots have)
                if (first) rows_loads_in_flight_at_most<(RING - 2) * 4>();
                // ---- four micro-chunks of one MFMA plus a little other work each (one wave per SIMD: nothing but
                //      the issue order keeps the matrix pipeline fed): a fragment of step t + 2 under the first and the
                //      third, one of the four loads of the slot RING further down the stream under the second and the
                //      fourth (evenly spaced: the load path of the compute unit is as busy as its matrix pipelines).
                //      That slot takes the position of the slot this step belongs to, whose fragments were read in steps
                //      t - 2 and t - 1 (t even): before its first load is issued, all LDS reads but the two of this
                //      step's first fragment have delivered.
                constexpr int fi = t / 2 + RING;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int e = m >> 1, mt = m & 1;
                    if constexpr (t < NST1) {
                        if constexpr (P_BY_HAND) RowsMmaV<T>::mma(fr[cur][e], xf[t][mt], p[e][mt]);
                        else p[e][mt] = Mma<T>::mma(fr[cur][e], xf[t][mt], p[e][mt]);
                    } else {
                        constexpr int u = t - NST1, ks2 = u / (2 * NH2), half = (u / 2) % NH2;
                        const int ht = 2 * (u & 1) + e;
                        yacc[4 * half + ht][mt] = Mma<T>::mma(fr[cur][e], hb[ks2 & 1][mt], yacc[4 * half + ht][mt]);
                    }
                    if ((m & 1) == 0) {
                        fr[rds][m >> 1] = read_frag(t2, ring + pn * SLOT, m >> 1);
                    } else {
                        if (first && m == 1) rows_lds_reads_older_done<2>();
                        const int j = 2 * (t & 1) + (m >> 1);
                        if (fi < SPC) issue_one(fi, c, pos, j);
                        else issue_one(fi - SPC, cn, pos, j);
                        if (t >= NST1) {
                            // H fragments of the next hidden step, during the last step of this one (an odd step)
                            constexpr int u = t >= NST1 ? t - NST1 : 0, ks2 = u / (2 * NH2);
                            if (u % (2 * NH2) == 2 * NH2 - 1 && ks2 + 1 < 4)
                                hb[(ks2 + 1) & 1][m >> 1] = lds_read16<vec8>(hbuf, (hrd ^ (uint32_t)((ks2 + 1) << 5)) + 4096u * (m >> 1));
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (!first) pos = pn;
                if (t == NST1 - 1) {
                    // ---- Add exchange of the partial tiles: wave t collects tile t = 2 ht + mt ------------
                    if constexpr (P_BY_HAND) rows_mfma_settle(p);
                    f32x16 s;
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        if (tt == wave) {            // (the own tile stays in registers; no dynamic register indexing)
                            s = p[tt >> 1][tt & 1];
                            continue;
                        }
                        const int src = (wave - tt + 4) % 4 - 1;     // 0..2: which of tile tt's three foreign parts
                        // (lane made opaque: these addresses do not depend on the chunk, and hoisted out of the chunk
                        //  loop they would live in registers this kernel does not have -- spilled, and every reload
                        //  of a spilled register makes the compiler wait for ALL outstanding loads, the ring's included)
                        uint32_t l = (uint32_t)lane;
                        asm volatile("" : "+v"(l));
                        char* dst = part + (tt * 3 + src) * SLOT + l * 16;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const f32x16& v = p[tt >> 1][tt & 1];
                            f32x4 o = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
                            *reinterpret_cast<f32x4*>(dst + q * 1024) = o;
                        }
                    }
                    asm volatile("" : "+v"(s));      // (the four tiles are dead from here on)
                    __syncthreads();
                    {
#pragma unroll
                        for (int src = 0; src < 3; ++src) {
                            uint32_t l = (uint32_t)lane;
                            asm volatile("" : "+v"(l));
                            const char* from = part + (wave * 3 + src) * SLOT + l * 16;
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const f32x4 v = *reinterpret_cast<const f32x4*>(from + q * 1024);
                                s[4 * q] += v[0]; s[4 * q + 1] += v[1]; s[4 * q + 2] += v[2]; s[4 * q + 3] += v[3];
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        // activation on complete sums, round to the operand type, into H: tile (ht, mt) = (wave / 2, wave % 2)
                        uint32_t l = (uint32_t)lane;
                        asm volatile("" : "+v"(l));
                        const uint32_t x = l & 31, h = l >> 5;
                        const uint32_t hrow = 32u * (wave & 1) + x, ht = (uint32_t)(wave >> 1);
                        const int nlim = N1 - 64 * c - 32 * (int)ht - 4 * (int)h;
                        switch (a.act) {
                            case ACT_RELU: rows_write_h<T, ACT_RELU>(s, hbuf, hrow, ht, h, nlim); break;
                            case ACT_GELU_TANH: rows_write_h<T, ACT_GELU_TANH>(s, hbuf, hrow, ht, h, nlim); break;
                            case ACT_SILU: rows_write_h<T, ACT_SILU>(s, hbuf, hrow, ht, h, nlim); break;
                            default: rows_write_h<T, ACT_IDENTITY>(s, hbuf, hrow, ht, h, nlim); break;
                        }
                    }
                    __syncthreads();
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) hb[0][mt] = lds_read16<vec8>(hbuf, hrd + 4096u * mt);
                }
            }, std::make_integer_sequence<int, NST>{});
            // the next chunk's steps 0 and 1 were read into sets NST % 3 and (NST + 1) % 3: rotate them to 0 and 1
            if constexpr (NST % 3 == 1) {
                const vec8 a0 = fr[1][0], a1 = fr[1][1];
                fr[1][0] = fr[2][0]; fr[1][1] = fr[2][1];
                fr[0][0] = a0; fr[0][1] = a1;
            } else if constexpr (NST % 3 == 2) {
                const vec8 a0 = fr[0][0], a1 = fr[0][1];
                fr[0][0] = fr[2][0]; fr[0][1] = fr[2][1];
                fr[1][0] = a0; fr[1][1] = a1;
            }
            // (no barrier at the end of a chunk: the next chunk writes its partial tiles after this chunk's second
            //  barrier, which a wave passes only when all four have summed theirs, and it writes H after its own
            //  first barrier, which a wave reaches only when it has finished reading this chunk's H)
        }
        // ---- store the output block: lane (x, h) holds, per tile, row 32 mt + x and 4 consecutive
        //      columns wave NW + 32 t + 8 q + 4 h + (0..3).  Rows at or past M lie behind the end of the
        //      buffer: the hardware drops those stores.  N2 is a multiple of 8: a group of 8 columns is
        //      inside or outside as a whole, for both values of h.
        {
            uint32_t l = (uint32_t)lane;
            asm volatile("" : "+v"(l));
            xo = l & 31u; ho = l >> 5;
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const uint32_t yoff = (uint32_t)((((uint64_t)row0 + 32 * mt + xo) * (uint64_t)N2 + (uint64_t)(wave * NW) + 4u * ho) * 2u);
#pragma unroll
            for (int t = 0; t < NT2; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (wave * NW + 32 * t + 8 * q < N2) {
                        typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                        u32x2 o;
                        o[0] = pack2<T>(yacc[t][mt][4 * q], yacc[t][mt][4 * q + 1]);
                        o[1] = pack2<T>(yacc[t][mt][4 * q + 2], yacc[t][mt][4 * q + 3]);
                        __builtin_amdgcn_raw_buffer_store_b64(o, ry, yoff + (uint32_t)(32 * t + 8 * q) * 2u, 0, 0);
                    }
                }
        }
    }
    rows_loads_in_flight_at_most<0>();   // the tail of the stream has landed before LDS is given back
    if (a.stats && tid == 0) {
        a.stats[2 * blockIdx.x] = wall_clock64() - t_wall;       // 100 MHz ticks
        a.stats[2 * blockIdx.x + 1] = clock64() - t_core;        // core clocks
    }
}

template <typename T, bool RAGGED> static const void* rows_fn(int nks, int nt2) {
    if (nks == 16 && nt2 == 8) return (const void*)fused_rows_kernel<T, 16, 8, RAGGED>;
    if (nks == 8 && nt2 == 8) return (const void*)fused_rows_kernel<T, 8, 8, RAGGED>;
    if (nks == 16 && nt2 == 4) return (const void*)fused_rows_kernel<T, 16, 4, RAGGED>;
    if (nks == 8 && nt2 == 4) return (const void*)fused_rows_kernel<T, 8, 4, RAGGED>;
    return nullptr;
}

hipError_t launch_fused_rows(int dtype, const RowsArgs& a, int nks, int nt2, int grid, hipStream_t st) {
    if (a.W3 != nullptr) return hipErrorInvalidValue;   // the gated chain is not built in this family
    // what the kernel assumes about its operands
    if (a.K > 64 * nks || a.N2 > 128 * nt2 || grid < 1 || a.M < 1) return hipErrorInvalidValue;
    const bool ragged = a.K != 64 * nks || (a.N1 & 63) != 0 || a.N2 != 128 * nt2;
    const void* fn = dtype == 0 ? (ragged ? rows_fn<__bf16, true>(nks, nt2) : rows_fn<__bf16, false>(nks, nt2))
                                : (ragged ? rows_fn<_Float16, true>(nks, nt2) : rows_fn<_Float16, false>(nks, nt2));
    if (!fn) return hipErrorInvalidValue;
    RowsArgs copy = a;
    void* params[] = {&copy};
    return hipLaunchKernel(fn, dim3(grid), dim3(256), params, 0, st);
}

}  // namespace ffuse
