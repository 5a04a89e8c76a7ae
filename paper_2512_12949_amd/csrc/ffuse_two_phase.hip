// Fused chain, "two-phase" family: ONE persistent kernel, two phases separated by ONE
// device-wide barrier; the intermediate is exchanged through the shared cache levels (the
// per-XCD L2s and the 256 MB Infinity Cache behind them) in the operand type.
//
//   phase 1: work items (row block of BM rows, hidden slice of BH1 columns); each computes,
//            with K complete, H[rows, slice] = act(X W1[:, slice]) [.* X W3[:, slice]];
//   barrier : every workgroup has published its tiles (write-through stores, counted arrivals;
//            no cache invalidate is needed: nobody has read H in this launch yet).  A gated chain
//            whose branches are separate first-phase items (TwoPhaseArgs::U) meets twice, with the
//            Mul pass that joins the two intermediates in between;
//   phase 2: work items (row block, 256 output columns, one of `splits` ranges of the hidden
//            dimension); each multiplies its part of H with its W2 block.  With splits == 1
//            the tile goes straight to Y; otherwise every range stores its partial tile into
//            its own fp32 plane and `finalize_planes_kernel` sums the planes in a fixed order
//            and converts to Y (deterministic, nothing has to be zeroed).
//
// In the paper's terms (Sec. 4.1) this is the "shuffle" strategy with the whole device as
// the cluster, followed (for splits > 1) by a small "reduce" with cls_reduce = splits whose
// volume, 4 M N2 splits bytes, is negligible next to the weights when M is small.  Splitting
// the hidden dimension all the way (the reduce family) would cost 4 M N2 (N1/128) bytes of
// atomics: more than the weights themselves at M = 64.
//
// Rows are blocked by BM = 32, 64, 128 (the weight-streaming and mid-M regime: the LDS-direct
// block GEMM with whole-line row-operand loads, WideGemm, or the register-staged FirstGemm with
// two stages in flight) or 256 (2 x 2 waves, DeepGemm: the compute-bound regime).
//
// Work items are dealt to workgroups XCD by XCD (blockIdx % 8 is the XCD): the items in
// flight on one XCD form a patch of `raster` row blocks x consecutive slices, so that a
// weight slice is fetched into that XCD's L2 once for all the row blocks of the patch.
#include "ffuse_gemm2.h"
#include "ffuse_launch.h"
#include <cstdlib>

namespace ffuse {


// item `idx` of XCD `xcd` -> (row block i, slice s); false past the XCD's share
__device__ __forceinline__ bool map_item(int MB, int S, int raster, int xcd, int idx, int& i, int& s) {
    const int total = MB * S;
    const int per = (total + 7) / 8;
    const int v = xcd * per + idx;
    if (idx >= per || v >= total) return false;
    const int panel = v / (raster * S);
    const int rem = v - panel * raster * S;
    const int rows = min(raster, MB - panel * raster);
    i = panel * raster + rem % rows;
    s = rem / rows;
    return true;
}

// BH1: hidden slice of a phase-1 work item.  With few rows the first phase is a weight stream
// that a single workgroup can only pull at 20-40 GB/s, so it wants at least as many items as
// there are CUs: 128-column slices (four waves along the columns), 64 (2 x 2 waves) or 32
// (four waves along the rows) give N1/128, N1/64 or N1/32 of them.
template <typename T, bool GATED, int BM, bool CONV, int BH1_, bool DEEP_> struct TwoPhaseGemms {
    static constexpr int BH1 = BH1_;
    static constexpr int WM1 = BH1 == 128 ? 1 : (BH1 == 64 ? 2 : 4);
    template <bool NT> using G1 = FirstGemm<T, GATED, BM, BH1, WM1, 4 / WM1, CONV, NT>;   // phase 1: X * W1 (, X * W3); CONV: im2col(X) * W1
    template <bool NT> using G2 = FirstGemm<T, false, BM, 256, 1, 4, false, NT>;   // phase 2: H * W2
    static constexpr bool HAS_NT = true;
    static constexpr bool DEEP = false;
    static constexpr bool PREFETCH = false;
};
template <typename T, bool GATED, int BH1_, bool DEEP_> struct TwoPhaseGemms<T, GATED, 256, false, BH1_, DEEP_> {
    static constexpr int BH1 = GATED ? 128 : 256;
    template <bool NT> using G1 = DeepGemm<T, GATED, 256, BH1, 2, 2>;
    template <bool NT> using G2 = DeepGemm<T, false, 256, 256, 2, 2>;
    static constexpr bool HAS_NT = false;   // 256-row blocks re-use their weight tiles through L2
    static constexpr bool DEEP = true;
    static constexpr bool PREFETCH = false;
};
// 32 / 64 / 128 rows with the LDS-direct block GEMM and a deeper ring in the first phase: more
// bytes in flight per workgroup than the register-staged loop can hold, the row operand in
// whole cache lines
template <typename T, bool GATED> struct TwoPhaseGemms<T, GATED, 128, false, 128, true> {
    static constexpr int BH1 = 128;
    template <bool NT> using G1 = WideGemm<T, GATED, 128, 128, 2, 2, GATED ? 4 : 8, NT>;
    template <bool NT> using G2 = WideGemm<T, false, 128, 256, 2, 2, 4, NT>;
    static constexpr bool HAS_NT = true;
    static constexpr bool DEEP = true;
    static constexpr bool PREFETCH = true;
};
template <typename T, bool GATED> struct TwoPhaseGemms<T, GATED, 128, false, 64, true> {
    static constexpr int BH1 = 64;
    template <bool NT> using G1 = WideGemm<T, GATED, 128, 64, 2, 2, 8, NT>;
    template <bool NT> using G2 = WideGemm<T, false, 128, 256, 2, 2, 4, NT>;
    static constexpr bool HAS_NT = true;
    static constexpr bool DEEP = true;
    static constexpr bool PREFETCH = true;
};
template <typename T, bool GATED> struct TwoPhaseGemms<T, GATED, 64, false, 64, true> {
    static constexpr int BH1 = 64;
    template <bool NT> using G1 = WideGemm<T, GATED, 64, 64, 2, 2, 8, NT>;
    template <bool NT> using G2 = WideGemm<T, false, 64, 256, 2, 2, 4, NT>;
    static constexpr bool HAS_NT = true;
    static constexpr bool DEEP = true;
    static constexpr bool PREFETCH = true;
};
template <typename T, bool GATED> struct TwoPhaseGemms<T, GATED, 32, false, 128, true> {
    static constexpr int BH1 = 128;
    template <bool NT> using G1 = WideGemm<T, GATED, 32, 128, 1, 4, 8, NT>;   // (a sixteen-stage ring measured no faster)
    template <bool NT> using G2 = WideGemm<T, false, 32, 256, 1, 4, 8, NT>;
    static constexpr bool HAS_NT = true;
    static constexpr bool DEEP = true;
    static constexpr bool PREFETCH = true;
};
template <typename T, bool GATED> struct TwoPhaseGemms<T, GATED, 64, false, 128, true> {
    static constexpr int BH1 = 128;
    template <bool NT> using G1 = WideGemm<T, GATED, 64, 128, 2, 2, GATED ? 4 : 8, NT>;
    template <bool NT> using G2 = WideGemm<T, false, 64, 256, 2, 2, 4, NT>;
    static constexpr bool HAS_NT = true;
    static constexpr bool DEEP = true;
    static constexpr bool PREFETCH = true;
};

// Phase 1 for one workgroup: its share of the (row block, hidden slice) items.  G1 is the block
// GEMM (with or without the non-temporal hint on its weight loads).
template <typename G1, bool CONV, bool DEEP, int BM, int BH1>
__device__ __forceinline__ void two_phase_first(const TwoPhaseArgs& a, char* smem, int tid, int xcd, int loc, int GX, int MB) {
    f32x16 acc[G1::HT][G1::MT];
    f32x16 acc3[G1::G == 2 ? G1::HT : 1][G1::G == 2 ? G1::MT : 1];
    typename G1::Ctx c;
    G1::init_lds(c, tid);
    const int NS = (a.N1 + BH1 - 1) / BH1;
    // a.U: the gated chain's branches as separate items (Sec. 4.1, gated FFN, first realisation): slice
    // index 2 s is the activated branch of hidden slice s (X W1, into H), 2 s + 1 the multiplying one
    // (X W3, unactivated, into U) -- neighbours in the item order, so they run side by side
    const bool split = G1::G == 1 && !CONV && a.U != nullptr;
    // 256-row tiles (DeepGemm): the ring fill of a workgroup's NEXT item is issued before the epilogue of the
    // present one and travels under it -- the epilogue stages through the one ring slot the fill leaves alone
    constexpr bool EARLY = DEEP && BM == 256 && !CONV;
    const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NI = split ? 2 * NS : NS;
    int rb, s, idx = loc;
    bool have = map_item(MB, NI, a.raster, xcd, idx, rb, s), filled = false;
    auto aim = [&](int rb_, int s_) {   // points the loader at item (rb_, s_)
        const bool up_ = split && (s_ & 1);
        const int sl_ = split ? s_ >> 1 : s_;
        if constexpr (CONV)
            G1::init_a_conv(c, a.X, (uint32_t)((uint64_t)a.M * a.conv_ic * 2), (uint32_t)rb_ * BM, a.M, a.conv_h, a.conv_w, a.conv_ic, tid);
        else
            G1::init_a(c, a.X, (uint32_t)((uint64_t)a.M * a.K * 2), 0u, (uint32_t)rb_ * BM, (uint32_t)a.K, a.K, tid);
        G1::init_b(c, up_ ? a.W3 : a.W1, split ? nullptr : a.W3, (uint32_t)((uint64_t)a.K * a.N1 * 2), (uint32_t)a.N1, (uint32_t)a.N1, (uint32_t)sl_ * BH1, tid);
    };
    while (have) {
        const bool up = split && (s & 1);
        const int sl = split ? s >> 1 : s;
        if (!filled) aim(rb, s);
        if constexpr (EARLY) G1::run(smem, c, 0, a.K, acc, acc3, tid, filled);
        else if constexpr (DEEP) G1::run(smem, c, 0, a.K, acc, acc3, tid);
        else G1::run_deep(smem, c, 0, a.K, acc, acc3, tid);
        int rbn, sn;
        idx += GX;
        have = map_item(MB, NI, a.raster, xcd, idx, rbn, sn);
        char* C = reinterpret_cast<char*>(up ? a.U : a.H);
        const int act = up ? (int)ACT_IDENTITY : a.act;
        if constexpr (EARLY) {
            filled = have && a.early_fill;
            if (filled) { aim(rbn, sn); G1::prefill(smem, c, 0, a.K); }
            G1::template store_tile_slabs_rt<true>(smem + G1::STAGING_SLOT, act, acc, acc3, C, a.N1, (int64_t)rb * BM, sl * BH1, a.M, a.N1, wave_u);
            // (no barrier: the next run() has one between this epilogue and the first load aimed at its slot)
        } else {
            G1::template store_tile_lds_rt<true>(smem, act, acc, acc3, C, a.N1, (int64_t)rb * BM, sl * BH1, a.M, a.N1, tid);
            __syncthreads();   // LDS is free again before the next item's loads
        }
        rb = rbn; s = sn;
    }
    if constexpr (EARLY) __syncthreads();   // every wave is done with the staging slot
}

// The Mul exchange of the split gated chain: H <- H .* U, tile by tile, in place.  Every workgroup joins
// the tiles of the activated branch that it computed itself: those lines are its own XCD's (written
// through, still valid in that L2), the U lines it reads for the first time in this launch, and no
// other XCD has touched either -- so, as at the rendezvous, nothing stale can be read and nothing
// needs invalidating.  The products are rounded once more to the operand type.
template <typename T, int BM, int BH1>
__device__ __forceinline__ void two_phase_join(const TwoPhaseArgs& a, int tid, int xcd, int loc, int GX, int MB) {
    const int NS = (a.N1 + BH1 - 1) / BH1;
    const uint32_t bytes = (uint32_t)((uint64_t)a.M * a.N1 * 2);
    const __amdgpu_buffer_rsrc_t rh = make_rsrc(a.H, bytes), ru = make_rsrc(a.U, bytes);
    constexpr int UPR = BH1 / 8;    // 16-byte units per tile row
    int rb, s;
    for (int idx = loc; map_item(MB, 2 * NS, a.raster, xcd, idx, rb, s); idx += GX) {
        if (s & 1) continue;
        s >>= 1;
        for (int u = tid; u < BM * UPR; u += 256) {
            const int64_t row = (int64_t)rb * BM + u / UPR;
            const int col = s * BH1 + 8 * (u % UPR);
            if (row >= a.M || col >= a.N1) continue;
            const uint32_t off = (uint32_t)((row * a.N1 + col) * 2);
            const u32x4 h = buf_load16(rh, off), g = buf_load16(ru, off);
            u32x4 o;
            float h0, h1, g0, g1;
            unpack2<T>(h[0], h0, h1); unpack2<T>(g[0], g0, g1); o[0] = pack2<T>(h0 * g0, h1 * g1);
            unpack2<T>(h[1], h0, h1); unpack2<T>(g[1], g0, g1); o[1] = pack2<T>(h0 * g0, h1 * g1);
            unpack2<T>(h[2], h0, h1); unpack2<T>(g[2], g0, g1); o[2] = pack2<T>(h0 * g0, h1 * g1);
            unpack2<T>(h[3], h0, h1); unpack2<T>(g[3], g0, g1); o[3] = pack2<T>(h0 * g0, h1 * g1);
            buf_store16_through(o, rh, off);
        }
    }
}

// Phase 2 for one workgroup: its share of the (row block, 256 output columns, hidden range) items.
template <typename G2, bool DEEP, int BM>
__device__ __forceinline__ void two_phase_second(const TwoPhaseArgs& a, char* smem, int tid, int xcd, int loc, int GX, int MB) {
    constexpr int BH2 = 256;
    f32x16 acc[G2::HT][G2::MT];
    f32x16 acc3[1][1];
    typename G2::Ctx c;
    G2::init_lds(c, tid);
    const int NCB = (a.N2 + BH2 - 1) / BH2;
    const int wave = tid >> 6, lane = tid & 63, x = lane & 31, h = lane >> 5;
    constexpr int WM2 = G2::WMR == BM ? 1 : 2;   // waves along the rows of a phase-2 tile
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave % WM2, wn = wave / WM2;
    int rb, u;
    // slices of this phase: u = range * NCB + column block, so that neighbours share their part of H
    for (int idx = loc; map_item(MB, NCB * a.splits, a.raster, xcd, idx, rb, u); idx += GX) {
        const int cb = u % NCB, sp = u / NCB;
        const int k0 = sp * a.ksplit, k1 = min(a.N1, k0 + a.ksplit);
        G2::init_a(c, a.H, (uint32_t)((uint64_t)a.M * a.N1 * 2), 0u, (uint32_t)rb * BM, (uint32_t)a.N1, a.N1, tid);
        G2::init_b(c, a.W2, nullptr, (uint32_t)((uint64_t)a.N1 * a.N2 * 2), (uint32_t)a.N2, (uint32_t)a.N2, (uint32_t)cb * BH2, tid);
        if constexpr (DEEP) G2::run(smem, c, k0, k1, acc, acc3, tid);
        else G2::run_deep(smem, c, k0, k1, acc, acc3, tid);
        if (a.splits == 1) {
            if constexpr (DEEP && BM == 256)   // (the slab epilogue keeps everything in registers: no reloads that wait for stores)
                G2::template store_tile_slabs<ACT_IDENTITY>(smem, acc, acc3, reinterpret_cast<char*>(a.Y), a.N2, (int64_t)rb * BM,
                                                            cb * BH2, a.M, a.N2, wave_u);
            else
                G2::template store_tile_lds<ACT_IDENTITY>(smem, acc, acc3, reinterpret_cast<char*>(a.Y), a.N2, (int64_t)rb * BM,
                                                          cb * BH2, a.M, a.N2, tid);
            __syncthreads();
            continue;
        }
        // acc[ht][mt][4q..4q+3]: row wm*WMR + 32*mt + x, columns wn*WHR + 32*ht + 8*q + 4*h + 0..3 of the tile
        // -> one 16-byte store into this range's own partial-sum plane (no atomics: the
        //    planes are summed in a fixed order by the finalize pass)
        // (ordinary write-back stores: writing the planes or Y through as well measured 3-7 % slower)
        float* plane = a.part + (size_t)sp * (size_t)a.M * a.N2;
#pragma unroll
        for (int ht = 0; ht < G2::HT; ++ht)
#pragma unroll
            for (int mt = 0; mt < G2::MT; ++mt) {
                const int64_t row = (int64_t)rb * BM + wm * G2::WMR + 32 * mt + x;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = cb * BH2 + wn * G2::WHR + 32 * ht + 8 * q + 4 * h;
                    if (row < a.M && col < a.N2) {
                        f32x4 v = {acc[ht][mt][4 * q], acc[ht][mt][4 * q + 1], acc[ht][mt][4 * q + 2], acc[ht][mt][4 * q + 3]};
                        *reinterpret_cast<f32x4*>(plane + row * a.N2 + col) = v;
                    }
                }
            }
    }
}

// While a workgroup waits at the barrier, the weight tile of its first phase-2 item can already be on
// its way: the first stages' loads are issued early (by the waves that do not poll), into the place
// where phase 2 will load them again -- then from L2, not from DRAM.  Only for the block GEMM that has
// the hook (row blocks below 256 in the LDS-direct loop).
template <typename G2, int BM>
__device__ __forceinline__ void two_phase_prefetch(const TwoPhaseArgs& a, char* smem, int tid, int xcd, int loc, int MB) {
    constexpr int BH2 = 256;
    const int NCB = (a.N2 + BH2 - 1) / BH2;
    int rb, u;
    if ((tid >> 6) == 0 || !map_item(MB, NCB * a.splits, a.raster, xcd, loc, rb, u)) return;
    const int cb = u % NCB, sp = u / NCB;
    const int k0 = sp * a.ksplit, k1 = min(a.N1, k0 + a.ksplit);
    typename G2::Ctx c;
    G2::init_lds(c, tid);
    G2::init_b(c, a.W2, nullptr, (uint32_t)((uint64_t)a.N1 * a.N2 * 2), (uint32_t)a.N2, (uint32_t)a.N2, (uint32_t)cb * BH2, tid);
    G2::prefetch_b(smem, c, k0, k1);
}

// One device-wide rendezvous of a launch's workgroups; `round` counts them from 1 (the group counters keep
// counting up: round r is complete for a group when its counter has reached r times the group's size).
// The tiles stored before it were stored write-through, so once this workgroup's stores have completed
// they are visible device-wide and arriving takes no L2 write-back (which costs 5+ us when
// the L2 holds a few MB of dirty lines).  A workgroup arrives with ONE atomic add whose
// result it does not wait for, on the counter of its group of G/8 workgroups (eight counters
// a cache line apart: 256 adds on one word take three times as long as 32 on each of 8), and
// then polls, together, the counters of the groups in `wait`: those whose tiles its own group reads next
// (a.wait_masks, enumerated on the host from the two item maps: often its own group alone, and
// then a group that is done starts phase 2 while others still stream their weights).  Measured in
// isolation, waiting for all eight: 1.8-3.9 us, against 3.8-6.5
// with a returning add plus a second, group-to-global add, and 7-12.5 with a releasing add.
// Bounded: on expiry the error word is set and every workgroup leaves (returns false).
// `between` runs after the arrival and before the wait (loads that may be issued early).
template <class Between>
__device__ __forceinline__ bool two_phase_rendezvous(const TwoPhaseArgs& a, volatile uint32_t& verdict, int tid, int xcd, int GX,
                                                     uint32_t wait, uint32_t round, Between&& between) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0)
        __hip_atomic_fetch_add(a.flags + kTwoPhaseGroupWord * (1 + xcd), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    between();
    if (tid == 0) {
        uint32_t ok = 1;
        uint32_t spins = 0;
        const uint32_t target = round * (uint32_t)GX + (uint32_t)a.extra_arrivals;
        for (;;) {
            uint32_t fewest = ~0u;
#pragma unroll
            for (int g = 0; g < 8; ++g)
                if ((wait >> g) & 1u) {
                    const uint32_t n = __hip_atomic_load(a.flags + kTwoPhaseGroupWord * (1 + g), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    fewest = n < fewest ? n : fewest;
                }
            if (fewest >= target) break;
            __builtin_amdgcn_s_sleep(1);
            // gives up after spin_limit polls, or (looked at every 1024 polls) when another workgroup has
            if (++spins >= a.spin_limit ||
                ((spins & 1023u) == 0 && __hip_atomic_load(a.flags + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                __hip_atomic_fetch_or(a.flags + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
        }
        verdict = ok;
    }
    __syncthreads();
    // No cache invalidate here.  An agent-scope acquire would drop this XCD's whole L2 (measured: 4-5 us
    // with the L2 full of weight lines), and there is nothing stale to drop: the caches were emptied of
    // other agents' data when the kernel started, nobody has read a byte of H since (phase 1 only writes
    // it), and the lines this XCD wrote itself hold what it wrote.  (Probed on the device: two XCDs
    // writing halves of the same lines, then reading each other's halves after this barrier, launch
    // after launch, see fresh data without an invalidate; they see stale data only if they had READ the
    // lines earlier in the same kernel.)
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const bool ok = verdict != 0;
    __syncthreads();   // everybody has read the word before the next loads reuse its place
    return ok;
}

// CONV: the first product is a 3x3 convolution (rows = pixels of a channels-last image,
// a.K = 9 * a.conv_ic); everything after the first product's loads is unchanged.
// a.nt selects, per launch, the instantiations of the block GEMMs that stream the weights with
// the non-temporal hint (row blocks below 256 only): the loops themselves stay branch-free.
template <typename T, bool GATED, int BM, bool CONV = false, int BH1_ = 128, bool DEEP_ = false>
__global__ __launch_bounds__(256) void fused_two_phase_kernel(TwoPhaseArgs a) {
    typedef TwoPhaseGemms<T, GATED, BM, CONV, BH1_, DEEP_> TG;
    typedef typename TG::template G1<false> G1;
    typedef typename TG::template G2<false> G2;
    constexpr int BH1 = TG::BH1;
    constexpr int LDS_BYTES = G1::LDS_BYTES > G2::LDS_BYTES ? G1::LDS_BYTES : G2::LDS_BYTES;
    __shared__ __attribute__((aligned(16))) char smem[LDS_BYTES];
    // the barrier's verdict word lives in the stage memory, which is idle between the phases
    // (the deepest ring takes all 160 KB)
    volatile uint32_t& verdict = *reinterpret_cast<volatile uint32_t*>(smem);
    const int tid = threadIdx.x;
    const int G = gridDim.x, GX = G >> 3;             // workgroups, workgroups per XCD
    const int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
    const int MB = (int)((a.M + BM - 1) / BM);
    uint64_t t0 = 0, t1 = 0, t2 = 0, c0 = 0, c1 = 0;
    if (a.stats) { t0 = wall_clock64(); c0 = clock64(); }
    const bool both = a.phases == 3;

    // ---------------------------------------------------------------- phase 1
    if (a.phases & 1) {
        if (TG::HAS_NT && a.nt) two_phase_first<typename TG::template G1<true>, CONV, TG::DEEP, BM, BH1>(a, smem, tid, xcd, loc, GX, MB);
        else two_phase_first<G1, CONV, TG::DEEP, BM, BH1>(a, smem, tid, xcd, loc, GX, MB);
    }

    if (a.stats) { t1 = wall_clock64(); c1 = clock64(); }
    // ---------------------------------------------------------------- rendezvous between the phases
    // (only when both phases run in this launch: launched one phase at a time, the kernel
    // boundary is the barrier -- the unfused comparison path).  See two_phase_rendezvous.
    bool ok = true;
    if (both) {
        if (a.U) {
            // split gated chain: every branch tile is out, then the workgroups join their own, then H is complete
            ok = two_phase_rendezvous(a, verdict, tid, xcd, GX, 0xffu, 1u, [] {});
            if (ok) two_phase_join<T, BM, BH1>(a, tid, xcd, loc, GX, MB);
        }
        if (ok)
            ok = two_phase_rendezvous(a, verdict, tid, xcd, GX, a.U ? 0xffu : (uint32_t)(a.wait_masks >> (8 * xcd)) & 0xffu, a.U ? 2u : 1u, [&] {
                if constexpr (TG::PREFETCH) {
                    if (TG::HAS_NT && a.nt) two_phase_prefetch<typename TG::template G2<true>, BM>(a, smem, tid, xcd, loc, MB);
                    else two_phase_prefetch<G2, BM>(a, smem, tid, xcd, loc, MB);
                }
            });
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    if (a.stats) t2 = wall_clock64();

    // ---------------------------------------------------------------- phase 2
    if (ok && (a.phases & 2)) {
        if (TG::HAS_NT && a.nt) two_phase_second<typename TG::template G2<true>, TG::DEEP, BM>(a, smem, tid, xcd, loc, GX, MB);
        else two_phase_second<G2, TG::DEEP, BM>(a, smem, tid, xcd, loc, GX, MB);
    }

    if constexpr (TG::PREFETCH) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (early loads of a phase 2 that did not run)
    if (a.stats && tid == 0) {
        uint64_t* p = a.stats + 4 * blockIdx.x;
        p[0] = t1 - t0; p[1] = t2 - t1; p[2] = wall_clock64() - t2; p[3] = c1 - c0;   // p[3]: core clocks of phase 1
    }
    // ---------------------------------------------------------------- leave the flags clean
    // the last workgroup to get here resets the counters for the next launch, and moves this launch's
    // error word to where the host reads it: a wait that expired once must not make the next launch give up
    __syncthreads();
    if (tid == 0 && both) {
        const uint32_t prev = __hip_atomic_fetch_add(a.flags + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev == (uint32_t)G - 1u) {
            __hip_atomic_store(a.flags + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int i = 0; i < 8; ++i)
                __hip_atomic_store(a.flags + kTwoPhaseGroupWord * (1 + i), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t verdict_word = __hip_atomic_load(a.flags + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.flags + 3, verdict_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.flags + 2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Y = sum over planes (fixed order: plane 0 first) of fp32 partial sums, rounded once to the operand type.
// The loads of eight planes are issued together and only then summed: the pass is latency-bound on small
// outputs (the planes were written by other XCDs and come from behind the L2), and one round trip per plane
// instead of one per eight made every call on the small shapes 1.2-1.5 us longer.
template <typename T> __global__ __launch_bounds__(256) void finalize_planes_kernel(const float* __restrict__ part, void* __restrict__ Y,
                                                                                 int64_t n8, int64_t plane_elems, int planes) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
    const f32x4 zero = s0;
    for (int p0 = 0; p0 < planes; p0 += 8) {
        f32x4 v0[8], v1[8];
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const bool live = p0 + p < planes;
            const f32x4* q = reinterpret_cast<const f32x4*>(part + (size_t)(live ? p0 + p : 0) * plane_elems) + 2 * i;
            v0[p] = live ? q[0] : zero;
            v1[p] = live ? q[1] : zero;
        }
#pragma unroll
        for (int p = 0; p < 8; ++p)
            if (p0 + p < planes) {   // (x + 0 is x, but -0 + 0 is +0: dead planes are skipped, not added)
                s0 += v0[p];
                s1 += v1[p];
            }
    }
    u32x4 o;
    o[0] = pack2<T>(s0[0], s0[1]);
    o[1] = pack2<T>(s0[2], s0[3]);
    o[2] = pack2<T>(s1[0], s1[1]);
    o[3] = pack2<T>(s1[2], s1[3]);
    reinterpret_cast<u32x4*>(Y)[i] = o;
}

hipError_t launch_finalize_planes(int dtype, const float* part, void* Y, int64_t count, int planes, hipStream_t st) {
    const int64_t n8 = count / 8;
    const int blocks = (int)((n8 + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL(finalize_planes_kernel<__bf16>, dim3(blocks), dim3(256), 0, st, part, Y, n8, count, planes);
    else
        hipLaunchKernelGGL(finalize_planes_kernel<_Float16>, dim3(blocks), dim3(256), 0, st, part, Y, n8, count, planes);
    return hipGetLastError();
}

template <typename T, bool GATED> static const void* two_phase_fn(int bm, int bh1, int bk) {
    if (bk == 32 && bh1 == 128) {   // the LDS-direct block GEMM for small row blocks
        if (bm == 32) return (const void*)fused_two_phase_kernel<T, GATED, 32, false, 128, true>;
        if (bm == 64) return (const void*)fused_two_phase_kernel<T, GATED, 64, false, 128, true>;
        if (bm == 128) return (const void*)fused_two_phase_kernel<T, GATED, 128, false, 128, true>;
    }
    if (bk == 32 && bh1 == 64) {
        if (bm == 64) return (const void*)fused_two_phase_kernel<T, GATED, 64, false, 64, true>;
        if (bm == 128) return (const void*)fused_two_phase_kernel<T, GATED, 128, false, 64, true>;
    }
    if (bk == 32 && bm != 256) return nullptr;
    if (bm == 32 && bh1 == 128) return (const void*)fused_two_phase_kernel<T, GATED, 32>;
    if (bm == 64 && bh1 == 128) return (const void*)fused_two_phase_kernel<T, GATED, 64>;
    if (bm == 64 && bh1 == 64) return (const void*)fused_two_phase_kernel<T, GATED, 64, false, 64>;
    if (bm == 128 && bh1 == 128) return (const void*)fused_two_phase_kernel<T, GATED, 128>;
    if (bm == 128 && bh1 == 64) return (const void*)fused_two_phase_kernel<T, GATED, 128, false, 64>;
    if constexpr (!GATED)
        if (bm == 128 && bh1 == 32) return (const void*)fused_two_phase_kernel<T, GATED, 128, false, 32>;
    if (bm == 256) return (const void*)fused_two_phase_kernel<T, GATED, 256>;
    return nullptr;
}

template <typename T> static const void* two_phase_conv_fn(int bm, int bh1) {
    if (bh1 == 128) {
        if (bm == 32) return (const void*)fused_two_phase_kernel<T, false, 32, true>;
        if (bm == 64) return (const void*)fused_two_phase_kernel<T, false, 64, true>;
        if (bm == 128) return (const void*)fused_two_phase_kernel<T, false, 128, true>;
    }
    // narrow slices: the table's deepest layers have 256 / 512 hidden channels, two or four 128-column items
    if (bh1 == 64) {
        if (bm == 64) return (const void*)fused_two_phase_kernel<T, false, 64, true, 64>;
        if (bm == 128) return (const void*)fused_two_phase_kernel<T, false, 128, true, 64>;
    }
    if (bh1 == 32 && bm == 128) return (const void*)fused_two_phase_kernel<T, false, 128, true, 32>;
    return nullptr;
}

hipError_t launch_fused_two_phase(int dtype, const TwoPhaseArgs& a, int bm, int bh1, int bk, int grid, hipStream_t st) {
    const bool g = a.W3 != nullptr && a.U == nullptr;   // (a.U: the branches are separate single-branch items)
    if (a.U && (a.W3 == nullptr || a.phases != 3 || a.conv_ic > 0 || (a.N1 & 63))) return hipErrorInvalidValue;
    const void* fn;
    if (a.conv_ic > 0) {
        // 3x3 first product: one tap per K step of 64, and the shifted addresses must fit 32 bits
        if (g || bk == 32 || a.conv_ic % 64 || a.K != 9 * a.conv_ic || a.conv_h < 1 || a.conv_w < 1) return hipErrorInvalidValue;
        fn = dtype == 0 ? two_phase_conv_fn<__bf16>(bm, bh1) : two_phase_conv_fn<_Float16>(bm, bh1);
    } else {
        fn = dtype == 0 ? (g ? two_phase_fn<__bf16, true>(bm, bh1, bk) : two_phase_fn<__bf16, false>(bm, bh1, bk))
                        : (g ? two_phase_fn<_Float16, true>(bm, bh1, bk) : two_phase_fn<_Float16, false>(bm, bh1, bk));
    }
    if (!fn || grid < 8 || (grid & 7) || a.raster < 1 || a.splits < 1 || a.phases < 1 || a.phases > 3) return hipErrorInvalidValue;
    TwoPhaseArgs copy = a;
    void* params[] = {&copy};
    return launch_resident(fn, grid, params, st);
}

}  // namespace ffuse
