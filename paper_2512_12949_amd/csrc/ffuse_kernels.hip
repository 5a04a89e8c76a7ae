// gfx950 kernels of the 16-bit paths:
//   * fused_reduce_kernel   -- the whole chain for one (row block, hidden slice) unit; the
//     activated slice never leaves registers; partial second products are summed across
//     hidden slices with fp32 atomics (paper Sec. 4.1 "reduce" strategy, with the hidden
//     split taking the place of the cluster's n dimension).
//   * fused_exchange_kernel -- persistent kernel, one workgroup per CU; on every XCD some
//     workgroups produce activated tiles into a ring buffer read through that XCD's L2, the
//     others consume them into register-resident output tiles (Sec. 4.1 "shuffle" strategy
//     with the XCD as the cluster and its L2 as the shared on-chip pool).
//   (the two-phase family, the default, lives in ffuse_two_phase.hip)
//   * finalize_kernel       -- fp32 sums -> Y in the operand type, workspace back to zero.
//   (the 16-bit unfused comparison path is the two-phase kernel launched one phase at a time)
#include "ffuse_gemm1.h"
#include "ffuse_launch.h"

namespace ffuse {

// blockIdx -> work unit, XCD aware.  Workgroups are dealt round-robin to the 8 XCDs, so
// blockIdx % 8 is the XCD and blockIdx / 8 the arrival order on it.  Each XCD gets one
// contiguous range of units ordered so that the ~32 units in flight on it form a patch of
// `raster` row blocks x consecutive column slices: the patch shares row blocks and weight
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

// ---------------------------------------------------------------------------------------
// Fused chain, "reduce" family.
// ---------------------------------------------------------------------------------------
template <typename T, bool GATED, int HT, int MT, int ACT>
__device__ __forceinline__ void make_h(const f32x16 (&acc)[HT][MT], const f32x16 (&acc3)[GATED ? HT : 1][GATED ? MT : 1],
                                       typename Mma<T>::vec8 (&hreg)[HT][MT][2]) {
#pragma unroll
    for (int ht = 0; ht < HT; ++ht)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                u32x4 pk;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    float v0 = activate<ACT>(acc[ht][mt][8 * b + 2 * d]);
                    float v1 = activate<ACT>(acc[ht][mt][8 * b + 2 * d + 1]);
                    if (GATED) {
                        v0 *= acc3[ht][mt][8 * b + 2 * d];
                        v1 *= acc3[ht][mt][8 * b + 2 * d + 1];
                    }
                    pk[d] = pack2<T>(v0, v1);
                }
                hreg[ht][mt][b] = __builtin_bit_cast(typename Mma<T>::vec8, pk);
            }
}

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
        G0::init_a(c, a.X, (uint32_t)((uint64_t)a.M * a.K * 2), 0u, (uint32_t)m0, (uint32_t)a.K, a.K, tid);
        G0::init_b(c, a.W1, a.W3, (uint32_t)((uint64_t)a.K * a.N1 * 2), (uint32_t)a.N1, (uint32_t)a.N1, (uint32_t)n0, tid);
        G0::init_lds(c, tid);
        G0::run(smem, c, 0, a.K, acc, acc3, tid);
    }

    // ---- activation (and gate) on complete sums; round to the operand type.  Registers
    //      8b..8b+7 of a tile are the 8 k-slots this lane feeds to the second product for
    //      hidden block 16*(2*ht + b): slot e <-> hidden 32*ht + 16*b + 8*(e/4) + 4*(lane/32) + e%4.
    vec8 hreg[HT][MT][2];
    switch (a.act) {
        case ACT_RELU: make_h<T, GATED, HT, MT, ACT_RELU>(acc, acc3, hreg); break;
        case ACT_GELU_TANH: make_h<T, GATED, HT, MT, ACT_GELU_TANH>(acc, acc3, hreg); break;
        case ACT_SILU: make_h<T, GATED, HT, MT, ACT_SILU>(acc, acc3, hreg); break;
        default: make_h<T, GATED, HT, MT, ACT_IDENTITY>(acc, acc3, hreg); break;
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
// Fused chain, "exchange" family.  One persistent workgroup per CU, all resident.  The
// workgroups that run on XCD x form group x (numbered by order of arrival; under round-robin
// dispatch every XCD gets the same number); within a group the first P are producers, the
// next PG*NCT are consumers:
//   producer q  : H tile (256 rows x BHP hidden) = act(X W1)[.* X W3] for item o = q, q+P, ...
//                 written to ring slot o % R in the operand type, then ready[slot] = o + 1
//   consumer c  : owns output tile (panel pi = c / NCT, 256 columns ct = c % NCT) of the group
//                 of PG panels in flight; for every hidden tile h it waits for item
//                 o = (g*NH + h)*PG + pi, multiplies it with W2[h*BHP.., ct*256..] into its
//                 register accumulators, then done[slot] += 1; after the last h it stores Y.
// Items are ordered (group of panels g, hidden tile h, panel in group pi); a producer may
// overwrite slot s only when the NCT consumers of the item that used it R items earlier are
// done.  How ring and flags are kept coherent is described below (XCD-local by default,
// agent-scope release/acquire on request).
// All waits are bounded: on expiry the error word is set and every workgroup leaves.
// ---------------------------------------------------------------------------------------
static constexpr uint32_t kSpinLimit = 1u << 23;

// Coherence of the ring.  All workgroups of a group run on one XCD and therefore share one
// L2: a producer's stores are visible to its group as soon as they have completed
// (s_waitcnt vmcnt(0)), and a consumer only has to drop its CU's own vector L1, which may
// still hold lines of the slot's previous use (buffer_inv sc0).  Flags are relaxed
// agent-scope atomics.  No L2 write-back or invalidate is involved: an agent-scope
// acquire would invalidate the whole L2 of the XCD on every wait.  `coherent` != 0 selects
// full agent-scope release/acquire instead (correct for any placement, much slower).
__device__ __forceinline__ void drop_l1() { asm volatile("buffer_inv sc0" ::: "memory"); }
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Flag polling.  Flags are read with SCALAR loads that bypass the scalar cache (glc): scalar
// loads are counted by lgkmcnt, so waiting for one does not wait for the LDS-direct vector
// loads the wave has in flight (vector loads return in order: a vector-load poll would drain
// the whole prefetch pipeline every time).  Every wave polls for itself -- the address is
// uniform, there is no broadcast and no barrier.
__device__ __forceinline__ uint32_t peek(const uint32_t* flag) {
    // the address is uniform by construction; say so, or it may sit in vector registers
    const uint64_t p = (uint64_t)flag;
    const uint64_t u = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(p >> 32)) << 32) |
                       (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    uint32_t v;
    asm volatile("s_load_dword %0, %1, 0x0 glc\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(u) : "memory");
    return v;
}
// Waits until *flag >= want; bounded: on expiry (or when another workgroup has given up) the
// error word is set and the wave returns false.  Then drops the CU's vector L1 (or, with
// `coherent`, does a full agent-scope acquire).
__device__ __forceinline__ bool wait_at_least(const uint32_t* flag, uint32_t want, uint32_t* err, int coherent) {
    uint32_t spins = 0;
    while (peek(flag) < want) {
        __builtin_amdgcn_s_sleep(2);
        if ((++spins & 1023u) == 0 && (spins > kSpinLimit || peek(err) != 0)) {
            if ((threadIdx.x & 63) == 0) __hip_atomic_fetch_or(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
    }
    if (coherent) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    else drop_l1();
    return true;
}

// optional per-workgroup timing (args.stats != nullptr): 100 MHz wall-clock ticks
struct ExchStats {
    uint64_t t0 = 0, wait = 0, tw = 0, gemm = 0, epi = 0, tg = 0;
    __device__ __forceinline__ void begin_wait(const void* on) { if (on) tw = wall_clock64(); }
    __device__ __forceinline__ void end_wait(const void* on) { if (on) wait += wall_clock64() - tw; }
};

template <typename T, bool GATED>
__global__ __launch_bounds__(256) void fused_exchange_kernel(ExchangeArgs a) {
    constexpr int BHP = GATED ? 128 : 256;
    typedef DeepGemm<T, GATED, 256, BHP, 2, 2> GP;    // producer: X * W1 (, X * W3)
    typedef DeepGemm<T, false, 256, 256, 2, 2> GC;    // consumer: H * W2
    constexpr int LDS_BYTES = GP::LDS_BYTES > GC::LDS_BYTES ? GP::LDS_BYTES : GC::LDS_BYTES;
    constexpr uint32_t SLOT_BYTES = 256u * BHP * 2u;
    constexpr int SPI = BHP / 32;                     // steps of 32 k per item on the consumer side
    static_assert(GC::NS == 4 && SPI % GC::NS == 0 && SPI > 3, "an item is a whole number of turns of the four-stage ring");
    __shared__ __attribute__((aligned(16))) char smem[LDS_BYTES];
    const int tid = threadIdx.x;
    const int coherent = a.coherent;
    const int R = a.R;
    uint32_t* err = a.flags + 16 * R;
    // Which group, and which member of it, is this workgroup?  XCD-local protocol: the group
    // is the XCD the workgroup really runs on (read from the hardware) and the member number
    // is the order of arrival on that XCD, counted in rank[xcd] -- dispatch is round robin
    // over the XCDs, but where it starts is not ours to assume.  An XCD that receives more
    // than its share reports FFUSE_ERR_PLACEMENT; one that receives fewer runs into the
    // bounded waits.  Coherent protocol: any placement works, groups follow blockIdx.
    int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
    if (!coherent) {
        uint32_t xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(xcc));
        uint32_t* rank = err + 1;
        uint32_t* slot0 = reinterpret_cast<uint32_t*>(smem);
        if (tid == 0) *slot0 = __hip_atomic_fetch_add(rank + (xcc & 7u), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        xcd = (int)(xcc & 7u);
        loc = (int)*slot0;
        __syncthreads();
        if (loc >= (int)(gridDim.x >> 3)) {
            if (tid == 0) __hip_atomic_fetch_or(err, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
    }
    const int P = a.P, NCT = a.NCT, PG = a.PG, NH = a.NH;
    const int NP = (int)((a.M + 255) / 256);
    const int NG = (NP + PG - 1) / PG;                       // groups of panels
    const int ngx = (NG > xcd) ? (NG - xcd + 7) / 8 : 0;      // groups handled by this XCD
    const int items = ngx * NH * PG;
    uint32_t* ready = a.flags + xcd * 2 * R;
    uint32_t* done = ready + R;
    char* ring = a.ring + (size_t)xcd * R * SLOT_BYTES;
    ExchStats es;
    if (a.stats) es.t0 = wall_clock64();
    auto finish = [&](int role, int n) {
        if (a.stats && tid == 0) {
            uint64_t* p = a.stats + 4 * blockIdx.x;
            p[0] = (uint64_t)role | (es.gemm << 8); p[1] = wall_clock64() - es.t0; p[2] = es.wait; p[3] = (uint64_t)n | (es.epi << 32);
        }
    };

    {
        // ------------------------------------------------------------------ producer
        // Pass 0: the first E = min(workgroups, ring slots) items are produced by ALL
        // workgroups of the group (consumers have nothing to multiply yet, and no slot is
        // being reused, so nobody waits).  After that producer q makes items E + q, E + q + P, ...
        f32x16 acc[GP::HT][GP::MT];
        f32x16 acc3[GATED ? GP::HT : 1][GATED ? GP::MT : 1];
        typename GP::Ctx c;
        GP::init_lds(c, tid);
        const int wpx = (int)(gridDim.x >> 3);
        const int E = min(min(wpx, R), items);
        int o = (loc < E) ? loc : (loc < P ? E + loc : items);
        bool first = true;
        while (o < items) {
            const int pi = o % PG, t = o / PG, hh = t % NH, gseq = t / NH;
            const int panel = (xcd + 8 * gseq) * PG + pi;
            const int slot = o % R;
            es.begin_wait(a.stats);
            if (!wait_at_least(done + slot, (uint32_t)(o / R) * NCT, err, coherent)) return;
            es.end_wait(a.stats);
            if (panel < NP) {
                GP::init_a(c, a.X, (uint32_t)((uint64_t)a.M * a.K * 2), 0u, (uint32_t)panel * 256u, (uint32_t)a.K, a.K, tid);
                GP::init_b(c, a.W1, a.W3, (uint32_t)((uint64_t)a.K * a.N1 * 2), (uint32_t)a.N1, (uint32_t)a.N1,
                           (uint32_t)hh * BHP, tid);
                if (a.stats) es.tg = wall_clock64();
                GP::run(smem, c, 0, a.K, acc, acc3, tid);
                if (a.stats) { const uint64_t t = wall_clock64(); es.gemm += t - es.tg; es.tg = t; }
                GP::store_tile_lds_rt(smem, a.act, acc, acc3, ring + (size_t)slot * SLOT_BYTES, BHP, 0, 0, 256, BHP, tid);
            }
            stores_done();     // this thread's tile stores have reached L2
            __syncthreads();   // ... and so have everybody else's (and LDS is free again)
            if (a.stats && panel < NP) es.epi += wall_clock64() - es.tg;
            if (tid == 0) {
                if (coherent) __hip_atomic_store(ready + slot, (uint32_t)o + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                else __hip_atomic_store(ready + slot, (uint32_t)o + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (loc >= P) break;   // consumers and spare workgroups produce one item at most
            o = (first && loc < E) ? E + loc : o + P;
            first = false;
        }
        if (loc < P) {
            finish(1, items);
            return;
        }
    }
    const int cidx = loc - P;
    if (cidx >= PG * NCT) return;
    // ---------------------------------------------------------------------- consumer
    const int pi = cidx / NCT, ct = cidx % NCT;
    f32x16 acc[GC::HT][GC::MT];
    f32x16 acc3[1][1];
    typename GC::Ctx c;
    GC::init_lds(c, tid);
    GC::init_b(c, a.W2, nullptr, (uint32_t)((uint64_t)a.N1 * a.N2 * 2), (uint32_t)a.N2, (uint32_t)a.N2, (uint32_t)ct * 256u, tid);
    typename GC::Frags f[2];
    for (int gseq = 0; gseq < ngx; ++gseq) {
        // a panel past the end (ragged last group) is processed like any other: its producers
        // publish nothing, its consumers multiply whatever the slot holds and store nothing
        const int panel = (xcd + 8 * gseq) * PG + pi;
        GC::zero(acc, acc3);
        const int o0 = gseq * NH * PG + pi;   // item of hidden tile 0; tile h is o0 + h*PG
        // A operand = ring slot of the item (256 x BHP, leading dimension BHP); B rows h*BHP + k.
        // The items of a panel form ONE stream of steps of 32 k through the stage ring.  Loads
        // run three steps ahead, i.e. at most into the next item: item h+1 must be ready
        // before the steps of item h are issued.
        es.begin_wait(a.stats);
        if (!wait_at_least(ready + o0 % R, (uint32_t)o0 + 1u, err, coherent)) return;
        es.end_wait(a.stats);
        GC::init_a(c, ring, (uint32_t)R * SLOT_BYTES, (uint32_t)(o0 % R) * SLOT_BYTES, 0u, BHP, BHP, tid);
        GC::prime(smem, c, 0, 0, BHP, GC::NS - 1, f);
        for (int hh = 0; hh < NH; ++hh) {
            const int o = o0 + hh * PG, on = o + PG;
            const bool more = hh + 1 < NH;
            if (more) {
                es.begin_wait(a.stats);
                if (!wait_at_least(ready + on % R, (uint32_t)on + 1u, err, coherent)) return;
                es.end_wait(a.stats);
            }
            const uint32_t base_cur = (uint32_t)(o % R) * SLOT_BYTES;
            const uint32_t base_nxt = more ? (uint32_t)(on % R) * SLOT_BYTES : kOob;
#pragma unroll 1
            for (int ks = 0; ks < SPI; ++ks) {
                // step hh*SPI + ks multiplies; its loads fetch the step three later
                const int k3 = (ks + 3) % SPI * 32;
                const bool wrap = ks + 3 >= SPI;
                c.abase = wrap ? base_nxt : base_cur;
                const int kw3 = (wrap ? hh + 1 : hh) * BHP + k3;
                const char* cur = smem + (ks & 3) * GC::STAGE;
                const char* nxt = smem + ((ks + 1) & 3) * GC::STAGE;
                char* ld = smem + ((ks + 3) & 3) * GC::STAGE;
                GC::step(cur, nxt, ld, c, k3, kw3, BHP, !wrap || more, f, acc, acc3);
            }
            // past the barrier of the item's last step every wave's loads from the slot have
            // landed in LDS: release the slot
            if (tid == 0) __hip_atomic_fetch_add(done + o % R, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        GC::drain();
        GC::template store_tile_lds<ACT_IDENTITY>(smem, acc, acc3, reinterpret_cast<char*>(a.Y), a.N2, (int64_t)panel * 256,
                                                  ct * 256, a.M, a.N2, tid);
        __syncthreads();   // LDS is free again before the next panel's loads
    }
    finish(2, ngx * NH);
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

hipError_t launch_finalize(int dtype, float* sums, void* Y, int64_t count, hipStream_t st) {
    const int64_t n8 = count / 8;
    const int blocks = (int)((n8 + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL(finalize_kernel<__bf16>, dim3(blocks), dim3(256), 0, st, sums, Y, n8);
    else
        hipLaunchKernelGGL(finalize_kernel<_Float16>, dim3(blocks), dim3(256), 0, st, sums, Y, n8);
    return hipGetLastError();
}

hipError_t launch_fused_exchange(int dtype, const ExchangeArgs& a, int wgs_per_group, hipStream_t st) {
    const void* fn = nullptr;
    const bool g = a.W3 != nullptr;
    if (dtype == 0) fn = g ? (const void*)fused_exchange_kernel<__bf16, true> : (const void*)fused_exchange_kernel<__bf16, false>;
    else fn = g ? (const void*)fused_exchange_kernel<_Float16, true> : (const void*)fused_exchange_kernel<_Float16, false>;
    ExchangeArgs copy = a;
    void* params[] = {&copy};
    return launch_resident(fn, 8 * wgs_per_group, params, st);
}

}  // namespace ffuse
