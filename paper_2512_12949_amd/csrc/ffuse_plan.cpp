// Host-side schedule chooser and data-movement model.  No device code.
//
// Re-derivation, for a device WITHOUT distributed shared memory, of the paper's Dataflow
// Analyzer (Sec. 4.2, Algorithm 1: per-level data-movement volume of one plan, inputs and
// outputs multiplied by the trip counts of the loops that re-access them, the intermediate
// placed greedily in the fastest level that holds it) and of its cost model (Sec. 4.3,
// Eq. 1-3: cost of level l = V_l / B_l, minimise the maximum subject to capacity), with a
// matrix-core time term added because several of the workloads are compute bound.
//
// Memory levels on gfx950: registers (512 KB per CU) -> LDS (160 KB per CU) -> L2 (4 MB per
// XCD, 32 CUs) -> Infinity Cache (256 MB) -> HBM.  Cross-workgroup sums go through fp32
// atomics that execute in L2.
#include "ffuse_plan.h"

#include <algorithm>
#include <cmath>
#include <vector>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <unordered_map>

namespace ffuse {

// Calibrated on an MI355X (standalone probes: MFMA issue loop, streaming read, LDS b128
// read, coalesced fp32 atomic adds).  Datasheet peaks are 2516 TFLOP/s and 8 TB/s.
Device kDevice = {
    /*cus*/ 256, /*xcds*/ 8,
    /*mfma_flops*/ 2.40e15,     // 32x32x16 issue loop
    /*hbm_bw*/ 5.6e12,          // streaming read of 2 GiB
    /*fabric_bw*/ 9.0e12,       // re-read of an Infinity-Cache-resident 32 MiB buffer
    /*l2_bw*/ 256 * 64.0 * 2.4e9,
    /*lds_bw*/ 256 * 128.0 * 2.4e9,
    /*atomic_bw*/ 1.36e12,      // fp32 atomic add, one dword per L2 channel per clock
    /*lds_bytes*/ 160 * 1024, /*acc_regs*/ 256, /*l2_bytes*/ 4.0 * 1024 * 1024,
    /*mall_bytes*/ 256.0 * 1024 * 1024,
    /*mfma_eff*/ 0.45,          // measured: the register-staged 256x256x64 main loop
    /*launch_s*/ 4e-6};

void set_device_units(int cus) {
    if (cus <= 0 || cus == kDevice.cus) return;
    const double f = (double)cus / kDevice.cus;
    kDevice.mfma_flops *= f;
    kDevice.l2_bw *= f;
    kDevice.lds_bw *= f;
    kDevice.cus = cus;
}

static double cdiv(double a, double b) { return std::ceil(a / b); }
static constexpr double kRowsEff = 0.45;   // rows family: fraction of the MFMA peak its chunk loop sustains at K = N2 = 1024 (bound by the L2 -> LDS load path)
static constexpr double kRowsLdsModel = 4 * 4 * 4096 + 12 * 4096 + 64 * 128;   // rows family: rings, partial tiles, H chunk

bool plan_valid(const ffuse_plan_t& p, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2) {
    (void)M; (void)K; (void)N1; (void)N2;
    if (p.gate_split && p.family != FFUSE_FAMILY_TWOPHASE) return false;
    switch (p.family) {
        case FFUSE_FAMILY_SCALAR: return dtype == FFUSE_DT_F32;
        case FFUSE_FAMILY_UNFUSED: return true;
        case FFUSE_FAMILY_REDUCE:
            if (dtype == FFUSE_DT_F32) return false;
            return fused_reduce_tile_ok(gated, p.bm, p.bh) && p.raster >= 1;
        case FFUSE_FAMILY_TWOPHASE: {
            if (dtype == FFUSE_DT_F32) return false;
            TwoPhaseGeometry sg;
            return two_phase_geometry(p, gated, M, N1, N2, &sg);
        }
        case FFUSE_FAMILY_ROWS: {
            if (dtype == FFUSE_DT_F32) return false;
            RowsGeometry rg;
            return rows_geometry(p, gated, M, K, N1, N2, &rg);
        }
        case FFUSE_FAMILY_EXCHANGE: {
            if (dtype == FFUSE_DT_F32) return false;
            ExchangeGeometry e;
            return exchange_geometry(p, gated, M, N1, N2, kDevice.cus, &e);
        }
        default: return false;
    }
}

// Producers P and consumers share the CUs/8 workgroups of a group.  Every panel of 256 rows
// needs NCT = ceil(N2/256) consumers; PG panels are in flight per group.
bool exchange_geometry(const ffuse_plan_t& p, int gated, int64_t M, int64_t N1, int64_t N2, int cus, ExchangeGeometry* e) {
    (void)M;
    const int bhp = gated ? 128 : 256;
    e->wgs_per_group = cus / 8;
    e->NCT = (int)((N2 + 255) / 256);
    e->NH = (int)((N1 + bhp - 1) / bhp);
    e->P = p.producers > 0 ? p.producers : e->wgs_per_group / 2;
    e->R = p.ring > 0 ? p.ring : kExchangeMaxRing;
    if (e->wgs_per_group < 2 || e->P < 1 || e->P >= e->wgs_per_group || p.coherent < 0 || p.coherent > 1) return false;
    e->PG = (e->wgs_per_group - e->P) / e->NCT;
    if (e->PG < 1) return false;
    if (e->R < 2 * e->PG + 2 || e->R > kExchangeMaxRing || 16 * e->R + 4 > (int)(kExchangeFlagBytes / 4)) return false;
    e->ws_bytes = kExchangeFlagBytes + (size_t)8 * e->R * 256 * bhp * 2;
    return true;
}

// Rows family: 64 rows per workgroup, the whole output width in accumulators (256 registers per lane hold
// 64 x 1024 fp32), the workgroup's rows of X in registers (128 per lane hold 64 x 1024 16-bit values, a
// quarter of K per wave).  Two accumulator sets of the first product would not fit beside them: not gated.
bool rows_geometry(const ffuse_plan_t& p, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, RowsGeometry* g) {
    if (gated || M < 1 || K < 8 || N1 < 8 || N2 < 8 || K > 1024 || N2 > 1024) return false;
    if ((p.bm != 0 && p.bm != 64) || (p.bh != 0 && p.bh != 64)) return false;
    g->nks = K <= 512 ? 8 : 16;
    g->nt2 = N2 <= 512 ? 4 : 8;
    return true;
}

bool weights_streamed(int dtype, int gated, int64_t K, int64_t N1, int64_t N2) {
    const double e = dtype == FFUSE_DT_F32 ? 4.0 : 2.0;
    return e * ((gated ? 2.0 : 1.0) * (double)K * (double)N1 + (double)N1 * (double)N2) > 512.0 * 1024 * 1024;
}

int two_phase_max_splits(int64_t M, int64_t N2) {
    // as many partial-sum planes as fit in 64 MiB
    int sp = 32;
    while (sp > 1 && (double)sp * 4.0 * (double)M * (double)N2 > 64.0 * 1024 * 1024) sp >>= 1;
    return sp;
}

bool two_phase_geometry(const ffuse_plan_t& p, int gated, int64_t M, int64_t N1, int64_t N2, TwoPhaseGeometry* g) {
    // rows per block: the plan's, or the smallest block that holds all rows, or 128 / 256
    // branches on different workgroups: tiles of the two intermediates must not share cache lines (the Mul pass
    // rewrites a tile in place while its neighbours may still hold the old values): rows of whole 128-byte lines
    if (p.gate_split < 0 || p.gate_split > 1 || (p.gate_split && (!gated || (N1 & 63)))) return false;
    g->gate_split = p.gate_split;
    if (p.gate_split) gated = 0;    // the items of the first phase are single-branch tiles
    int bm = p.bm;
    if (bm <= 0) bm = M <= 32 ? 32 : (M <= 64 ? 64 : (M <= 512 ? 128 : 256));
    if (bm != 32 && bm != 64 && bm != 128 && bm != 256) return false;
    if (bm < 128 && M > 4 * bm) return false;   // the small blocks are for a few row blocks at most
    g->bm = bm;
    // hidden slice of a phase-1 item: the plan's bh where the kernels implement it
    if (bm == 256) {
        g->bh1 = gated ? 128 : 256;
    } else {
        g->bh1 = p.bh > 0 ? p.bh : 128;
        const bool ok = g->bh1 == 128 || (g->bh1 == 64 && bm >= 64) || (g->bh1 == 32 && bm == 128 && !gated);
        if (!ok) {
            if (p.bh == 256) g->bh1 = 128;   // plans written before narrow slices existed
            else return false;
        }
    }
    g->bk = bm == 256 ? 32 : (p.bk == 32 ? 32 : 64);
    if (g->bk == 32 && bm != 256 && !(g->bh1 == 128 || (g->bh1 == 64 && bm >= 64))) return false;
    const int64_t mb = (M + bm - 1) / bm;
    g->raster = p.raster > 0 ? p.raster : 1;
    if (g->raster > mb) g->raster = (int)mb;
    int splits = p.splits > 0 ? p.splits : (M <= 128 ? 8 : 1);
    if (splits > 32) return false;
    g->ksplit = (int)(((N1 + splits - 1) / splits + 63) / 64 * 64);
    g->splits = (int)((N1 + g->ksplit - 1) / g->ksplit);
    // the kernel addresses H through 32-bit buffer offsets and masks lanes with an offset of 2^31
    if ((M + 256) * N1 * 2 >= ((int64_t)1 << 31)) return false;
    g->ysum_bytes = g->splits > 1 ? (((size_t)4 * M * N2 * g->splits + 255) & ~(size_t)255) : 0;
    g->h_bytes = ((size_t)2 * M * N1 + 255) & ~(size_t)255;
    g->u_bytes = g->gate_split ? g->h_bytes : 0;
    g->ws_bytes = g->ysum_bytes + g->h_bytes + g->u_bytes + kTwoPhaseFlagBytes;
    return true;
}

namespace {
// the kernel's item map (fused_two_phase_kernel: map_item): item `idx` of group `grp` -> (row block, slice)
bool two_phase_item(int MB, int S, int raster, int grp, int idx, int* i, int* s) {
    const int total = MB * S;
    const int per = (total + 7) / 8;
    const int v = grp * per + idx;
    if (idx >= per || v >= total) return false;
    const int panel = v / (raster * S);
    const int rem = v - panel * raster * S;
    const int rows = std::min(raster, MB - panel * raster);
    *i = panel * raster + rem % rows;
    *s = rem / rows;
    return true;
}
}  // namespace

uint64_t two_phase_wait_masks(const TwoPhaseGeometry& g, int64_t M, int64_t N1, int64_t N2) {
    const int MB = (int)((M + g.bm - 1) / g.bm);
    const int NS1 = (int)((N1 + g.bh1 - 1) / g.bh1);
    const int NCB = (int)((N2 + 255) / 256);
    if (g.gate_split) return ~(uint64_t)0;   // (two device-wide rendezvous: branch tiles are joined across groups)
    if ((int64_t)MB * NS1 > 65536 || (int64_t)MB * NCB * g.splits > 65536) return ~(uint64_t)0;   // (not worth the host time)
    // producer group of every H tile (row block, phase-1 slice)
    std::vector<signed char> owner((size_t)MB * NS1, (signed char)-1);
    for (int grp = 0; grp < 8; ++grp) {
        int i, s;
        for (int idx = 0; two_phase_item(MB, NS1, g.raster, grp, idx, &i, &s); ++idx) owner[(size_t)i * NS1 + s] = (signed char)grp;
    }
    uint64_t masks = 0;
    for (int grp = 0; grp < 8; ++grp) {
        uint64_t m = (uint64_t)1 << grp;   // (a group always waits for its own stores)
        int i, u;
        for (int idx = 0; two_phase_item(MB, NCB * g.splits, g.raster, grp, idx, &i, &u); ++idx) {
            const int sp = u / NCB;
            const int64_t k0 = (int64_t)sp * g.ksplit, k1 = std::min<int64_t>(N1, k0 + g.ksplit);
            for (int64_t s = k0 / g.bh1; s * g.bh1 < k1; ++s) {
                const int o = owner[(size_t)i * NS1 + s];
                if (o < 0) return ~(uint64_t)0;   // (cannot happen: every tile has a producer)
                m |= (uint64_t)1 << o;
            }
        }
        masks |= m << (8 * grp);
    }
    return masks;
}

bool two_phase_groups_independent(const TwoPhaseGeometry& g, int64_t M, int64_t N1, int64_t N2) {
    return two_phase_wait_masks(g, M, N1, N2) == 0x8040201008040201ull;
}

bool fused_reduce_tile_ok(int gated, int bm, int bh) {
    if (!gated) return (bm == 256 && bh == 256) || (bm == 128 && (bh == 256 || bh == 128 || bh == 64));
    return (bm == 256 && bh == 128) || (bm == 128 && (bh == 128 || bh == 64));
}

// Fraction of the MFMA peak a block GEMM sustains on a compute-bound problem, by tile shape
// (measured on the two-phase kernel's first phase, 4096 x 4096 x 16384 and 2048 x 4096 x
// 2 * 11008).  Four waves share a rows x cols tile 2 x 2; per MFMA a wave reads
// r ~ 1 / wave rows + 1 / wave cols operand fragments from LDS, and the smaller the tile the
// more of the loop is LDS reads rather than matrix instructions.  The 256 x 256 tile runs at
// the chip's power limit; smaller tiles run at a higher clock but stay LDS-bound.
//     wave tile    r     LDS-direct loop   register-staged loop
//     128 x 128    1     0.51              --
//      64 x 128    1.5   0.46              0.40
//      64 x 64     2     0.36              0.275
//      64 x 32     3     0.27              0.156
// (LDS-direct below 256 rows: the loop that loads the row operand in whole cache lines; with
// half lines it measured 0.40 / 0.31 / 0.20)
// 1 / efficiency is interpolated linearly in r (and extrapolated beyond 3).
static double block_gemm_efficiency(double rows, double cols, bool lds_direct) {
    const double wr = rows >= 128.0 ? rows / 2.0 : rows, wc = rows >= 128.0 ? cols / 2.0 : cols / 4.0;
    const double r = 64.0 * (1.0 / wr + 1.0 / wc);
    static const double rs[4] = {1.0, 1.5, 2.0, 3.0};
    static const double inv_direct[4] = {1.0 / 0.51, 1.0 / 0.46, 1.0 / 0.36, 1.0 / 0.27};
    static const double inv_staged[4] = {1.0 / 0.51, 1.0 / 0.40, 1.0 / 0.275, 1.0 / 0.156};
    const double* inv = lds_direct ? inv_direct : inv_staged;
    if (r <= rs[0]) return 1.0 / inv[0];
    int i = 0;
    while (i < 2 && r > rs[i + 1]) ++i;
    const double v = inv[i] + (inv[i + 1] - inv[i]) * (r - rs[i]) / (rs[i + 1] - rs[i]);
    return 1.0 / v;
}

void traffic_model(const ffuse_plan_t& p, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                   ffuse_traffic_t* t) {
    const Device& d = kDevice;
    if (p.family == FFUSE_FAMILY_TWOPHASE && p.gate_split) {
        // Branches on different workgroups (Sec. 4.1, gated FFN): per flop the single-branch tiles load what the
        // two-accumulator tiles of the same plan load (the row-operand tile is shared there), so the plan is
        // priced as its one-workgroup twin plus the Mul pass -- both intermediates read, one rewritten, through
        // the shared cache -- and that pass's rendezvous; measured on 2048 x 4096 x 11008 x 4096 and on the
        // m = 128 gated shapes it costs 15 % and 20-47 % more than the twin (twice as many first-phase items,
        // each re-reading the row operand; the pass and its rendezvous are 8-15 us on their own).
        TwoPhaseGeometry sg;
        std::memset(t, 0, sizeof(*t));
        if (!gated || !two_phase_geometry(p, gated, M, N1, N2, &sg)) return;
        ffuse_plan_t q = p;
        q.gate_split = 0;
        if (q.bm == 256) q.bh = 128;
        traffic_model(q, dtype, gated, M, K, N1, N2, t);
        const double join = 3.0 * 2.0 * (double)M * (double)N1;
        t->exchange_bytes += join;
        t->fabric_bytes += join;
        t->t_pred = 1.10 * t->t_pred + join / d.fabric_bw + 8e-6;
        return;
    }
    std::memset(t, 0, sizeof(*t));
    const double e = dtype == FFUSE_DT_F32 ? 4.0 : 2.0, g = gated ? 2.0 : 1.0;
    const double m = (double)M, k = (double)K, n1 = (double)N1, n2 = (double)N2;
    t->flops = 2.0 * m * n1 * (g * k + n2);
    t->q_min = e * (m * k + g * k * n1 + n1 * n2 + m * n2);
    t->q_unfused = t->q_min + 2.0 * e * m * n1;
    double mfma_flops = d.mfma_flops;
    double padded = t->flops, waves = 1.0;
    t->feasible = 1;

    if (p.family == FFUSE_FAMILY_REDUCE) {
        const double bm = p.bm, bh = p.bh, R = std::max(1, p.raster);
        const double MB = cdiv(m, bm), S = cdiv(n1, bh), units = MB * S;
        t->workgroups = (int)units;
        padded = units * 2.0 * bm * bh * (g * k + n2);
        waves = cdiv(units, d.cus) * d.cus / units;
        // every unit streams its X row block, its weight slices: L2 -> CU
        t->l2_bytes = units * e * (bm * k + g * k * bh + bh * n2);
        // an XCD patch of R row blocks x (32/R) slices fills each tile once into its L2
        const double P = std::max(1.0, 32.0 / R);
        t->fabric_bytes = units / 32.0 * e * (R * bm * k + P * (g * k * bh + bh * n2));
        // matrix pipeline LDS reads: per k=16 step a wave reads (g*HT + MT) KB in the first
        // product (4 waves split rows), JT KB in the second (H comes from registers)
        const double ht = bh / 32.0, mt = bm / 128.0, jt = 4.0;
        t->lds_bytes = units * 4.0 * 1024.0 * ((k / 16.0) * (g * ht + mt) + (n2 / 128.0) * (bh / 16.0) * jt);
        t->reduce_bytes = 4.0 * m * n2 * S;
        t->exchange_bytes = 0.0;
        // fp32 sums: read + zero-write by the finalise pass; HBM only if they overflow the
        // Infinity Cache
        const double sums = 4.0 * m * n2;
        t->hbm_bytes = t->q_min + (sums > 0.5 * d.mall_bytes ? 2.0 * sums : 0.0);
        t->lds_used = std::max(2.0 * (bm * 128.0 + g * bh * 128.0), 2.0 * (bh >= 128 ? 2.0 : 1.0) * 128.0 * 128.0);
        t->acc_regs = g * (bh / 32.0) * (bm / 128.0) * 16.0;
        t->feasible = t->lds_used <= d.lds_bytes && t->acc_regs <= d.acc_regs;
    } else if (p.family == FFUSE_FAMILY_TWOPHASE) {
        TwoPhaseGeometry sg;
        t->feasible = two_phase_geometry(p, gated, M, N1, N2, &sg) ? 1 : 0;
        if (t->feasible) {
            const double bh1 = gated ? 128.0 : 256.0;
            const double bm = sg.bm, ns = cdiv(n1, bh1), items = cdiv(n2, 256) * sg.splits;
            t->workgroups = d.cus;
            // small tiles keep the matrix cores mostly idle: a few MFMAs per 64-deep step
            padded = (ns * 2.0 * bm * bh1 * g * k + items * 2.0 * bm * 256 * sg.ksplit) / 0.25;
            waves = std::max(cdiv(ns, d.cus) * d.cus / ns, cdiv(items, d.cus) * d.cus / items);
            t->l2_bytes = ns * e * (bm * k + g * k * bh1) + items * e * (bm * sg.ksplit + sg.ksplit * 256.0);
            t->fabric_bytes = t->q_min + 8.0 * e * (m * k + m * n1);   // X and H fill each XCD's L2 once
            t->lds_bytes = t->l2_bytes * 2.0;
            t->exchange_bytes = 2.0 * e * m * n1;
            t->reduce_bytes = 4.0 * m * n2 * sg.splits;
            // H is written through and read back: from the memory-side cache while it fits beside the
            // operands, else from HBM (the same rule as for the unfused path below)
            const double hb = e * m * n1;
            t->hbm_bytes = t->q_min + (hb > 0.5 * d.mall_bytes ? 2.0 * hb : 0.0);
            t->lds_used = 2.0 * (bm * 128.0 + 256 * 128.0);
            t->acc_regs = 2.0 * (bm / 32.0) * 16.0;
        }
    } else if (p.family == FFUSE_FAMILY_EXCHANGE) {
        ExchangeGeometry x;
        t->feasible = exchange_geometry(p, gated, M, N1, N2, d.cus, &x) ? 1 : 0;
        if (t->feasible) {
            const double bhp = gated ? 128.0 : 256.0;
            const double NP = cdiv(m, 256), NG = cdiv(NP, x.PG), gx = cdiv(NG, 8);
            const double f_cu = d.mfma_flops / d.cus;
            // a producer tile also pays ~12 us of epilogue, publication and pipeline refill
            // (measured; expressed here at the full matrix rate like the rest of `padded`)
            const double tp = 2.0 * 256 * bhp * g * k / f_cu + 12e-6 * d.mfma_eff, tc = 2.0 * 256 * 256 * bhp / f_cu;
            // per group: producers share gx*NH*PG tiles; every consumer multiplies gx*NH items;
            // the consumers start one producer tile late
            const double Tp = cdiv(gx * x.NH * x.PG, x.P) * tp, Tc = gx * x.NH * tc;
            padded = (std::max(Tp, Tc) + tp) * d.mfma_flops;   // expressed as chip-time x chip-rate
            t->workgroups = 8 * x.wgs_per_group;
            t->l2_bytes = NP * x.NH * e * (256 * k + g * k * bhp) + NP * x.NCT * e * (256 * n1 + n1 * 256);
            // every group streams all weights once per set of PG panels; X and Y once
            t->fabric_bytes = NG * e * (g * k * n1 + n1 * n2) + e * m * k + e * m * n2;
            t->lds_bytes = NP * x.NH * 4.0 * 1024.0 * (k / 16.0) * (g * bhp / 64.0 + 4.0) +
                           NP * x.NCT * 4.0 * 1024.0 * (n1 / 16.0) * 8.0;
            t->exchange_bytes = e * m * n1 * (1.0 + x.NCT);   // written once, read by NCT consumers (L2)
            t->hbm_bytes = t->q_min;
            t->lds_used = 2.0 * (256 * 128.0 + 256 * 128.0);
            t->acc_regs = 256;
        }
    } else if (p.family == FFUSE_FAMILY_ROWS) {
        RowsGeometry rg;
        t->feasible = rows_geometry(p, gated, M, K, N1, N2, &rg) ? 1 : 0;
        if (t->feasible) {
            const double mb = cdiv(m, 64.0), kq = 16.0 * rg.nks * 4.0, nw = 128.0 * rg.nt2;
            t->workgroups = (int)std::min(mb, (double)d.cus);
            // every row block walks the whole hidden dimension at the kernel's padded K and N2
            padded = mb * 2.0 * 64.0 * cdiv(n1, 64.0) * 64.0 * (kq + nw);
            waves = cdiv(mb, d.cus) * d.cus / mb;
            // L2 -> CU: every row block streams all weights; X once
            t->l2_bytes = mb * e * (k * n1 + n1 * n2) + e * m * k;
            // the workgroups of an XCD walk the chunks together: one fill per XCD and round of row blocks
            t->fabric_bytes = std::min(8.0, mb) * cdiv(mb, d.cus) * e * (k * n1 + n1 * n2) + e * m * k + e * m * n2;
            // LDS: every weight byte is written once and read once; partial tiles 2 x 48 KB + H per chunk
            t->lds_bytes = t->l2_bytes + mb * cdiv(n1, 64.0) * (2.0 * 49152.0 + 4.0 * 8192.0 + 8192.0);
            t->exchange_bytes = 0.0;
            t->reduce_bytes = 0.0;
            t->hbm_bytes = t->q_min;
            t->lds_used = kRowsLdsModel;
            t->acc_regs = 16.0 * 2.0 * rg.nt2;
        }
    } else if (p.family == FFUSE_FAMILY_UNFUSED) {
        const double bm = 256.0, bh0 = gated ? 128.0 : 256.0, bh1 = 256.0;
        const double u0 = cdiv(m, bm) * cdiv(n1, bh0), u1 = cdiv(m, bm) * cdiv(n2, bh1);
        t->workgroups = (int)std::max(u0, u1);
        padded = u0 * 2.0 * bm * bh0 * g * k + u1 * 2.0 * bm * bh1 * n1;
        waves = (cdiv(u0, d.cus) * d.cus * g * k + cdiv(u1, d.cus) * d.cus * n1) / (u0 * g * k + u1 * n1);
        t->l2_bytes = u0 * e * (bm * k + g * k * bh0) + u1 * e * (bm * n1 + n1 * bh1) + e * m * n1;
        t->fabric_bytes = u0 / 32.0 * e * (4 * bm * k + 8 * g * k * bh0) + u1 / 32.0 * e * (4 * bm * n1 + 8 * n1 * bh1) + e * m * n1;
        t->lds_bytes = u0 * 4.0 * 1024.0 * (k / 16.0) * (g * bh0 / 64.0 + 4.0) + u1 * 4.0 * 1024.0 * (n1 / 16.0) * 8.0;
        const double h = e * m * n1;
        t->hbm_bytes = t->q_min + (h > 0.5 * d.mall_bytes ? 2.0 * h : 0.0);
        t->exchange_bytes = 2.0 * h;
        t->lds_used = 2.0 * (bm * 128.0 + g * bh0 * 128.0);
        t->acc_regs = 256;
    } else {  // scalar fp32 debug path
        const double units = cdiv(m, 16) * cdiv(n1, 64);
        t->workgroups = (int)units;
        mfma_flops = 256 * 128.0 * 2.4e9;  // fp32 FMA rate, not matrix cores
        t->l2_bytes = units * e * (16 * k + g * k * 64 + 64 * n2);
        t->fabric_bytes = t->l2_bytes / 8.0;
        t->reduce_bytes = 4.0 * m * n2 * cdiv(n1, 64);
        t->hbm_bytes = t->q_min;
        t->lds_bytes = t->flops * 2.0;
    }
    // the reduce family's 4x1 wave layout and 128-row tiles run the matrix cores at ~2/3 of the
    // 256x256 main loop's efficiency (measured on the m = 128 shapes)
    const double eff = p.family == FFUSE_FAMILY_SCALAR ? 1.0 : (p.family == FFUSE_FAMILY_REDUCE ? 0.67 * d.mfma_eff : d.mfma_eff);
    t->t_mfma = padded * waves / (mfma_flops * eff);
    // the reduce family's kernel streams weights at well under half the HBM rate (measured at M <= 16)
    t->t_hbm = t->hbm_bytes / (p.family == FFUSE_FAMILY_REDUCE ? 0.45 * d.hbm_bw : d.hbm_bw);
    t->t_fabric = t->fabric_bytes / d.fabric_bw;
    t->t_l2 = t->l2_bytes / d.l2_bw;
    t->t_lds = t->lds_bytes / d.lds_bw;
    t->t_reduce = t->reduce_bytes / d.atomic_bw;
    double worst = std::max({t->t_mfma, t->t_hbm, t->t_fabric, t->t_l2, t->t_lds});
    // atomics of one unit are issued after its matrix work: with a single round of units
    // nothing overlaps them; with several rounds about half does
    const double overlap = (t->workgroups <= d.cus) ? 0.0 : 0.5;
    worst = std::max(worst, t->t_reduce) + (1.0 - overlap) * std::min(worst, t->t_reduce);
    const double launches = 2.0;  // main kernel + finalise / second GEMM / zero fill
    t->t_pred = worst + launches * d.launch_s;
    // the reduce family's units run their two products and their atomics one after the other, which this
    // bandwidth model does not see: measured on the smallest m = 128 shapes it is 5-35 % optimistic
    if (p.family == FFUSE_FAMILY_REDUCE) t->t_pred *= 1.25;
    if (p.family == FFUSE_FAMILY_ROWS && t->feasible) {
        // The kernel is a weight stream through LDS at 64 flop per weight byte: per chunk a CU pulls the chunk's
        // weights through its load path, as long as the chunk's matrix instructions take.  Fitted on the device
        // (row-block rounds x (chunks x chunk time + a fixed part per row block)): the fraction of the matrix peak
        // a chunk sustains grows with its size -- 0.36 for K = N2 = 512 (8.4 Mflop per chunk: 32768 x 512 x 4096 x 512
        // in 368 us), kRowsEff for K = N2 = 1024 (16.8 Mflop: 32768 x 1024 x 8192 x 1024 in 1056 us, x 1024 x 1024 in
        // 170) -- and every row block pays about 20 us on top (X into registers, the ring primed again after the
        // output stores, the output block stored; the first one also the kernel's start: 120 KB of LDS, a long
        // unrolled loop to fetch), which is why the family loses to every other on problems of a few row blocks.
        RowsGeometry rg;
        rows_geometry(p, gated, M, K, N1, N2, &rg);
        const double chunk_flops = 2.0 * 64.0 * 64.0 * (64.0 * rg.nks + 128.0 * rg.nt2);
        const double small = 2.0 * 64.0 * 64.0 * 1024.0, big = 2.0 * small;
        const double eff = std::min(kRowsEff, std::max(0.30, 0.36 + (kRowsEff - 0.36) * (chunk_flops - small) / (big - small)));
        const double t_chunk = chunk_flops / (d.mfma_flops / d.cus * eff);
        t->t_mfma = cdiv(cdiv(m, 64.0), d.cus) * (cdiv(n1, 64.0) * t_chunk + 20e-6);
        t->t_pred = std::max({t->t_mfma, t->t_l2, t->t_fabric, t->t_hbm}) + d.launch_s;
    }
    if (p.family == FFUSE_FAMILY_TWOPHASE && t->feasible) {
        // two phases back to back, each the longer of its streaming time and its matrix time.
        // Streaming: a workgroup of this kernel keeps ~64 KB in flight and sustains ~25 GB/s on
        // its own (measured), so a phase with few work items is bounded by items x 25 GB/s
        // rather than by HBM; every item also pays ~3 us of pipeline fill and epilogue.  A
        // weight slice is fetched once per XCD patch of `raster` row blocks: the first fetch
        // comes from HBM, repeats (and the rows, once per slice group) from the Infinity Cache.
        // Fixed: launch, one device-wide barrier, finalize (~13 us).
        TwoPhaseGeometry sg;
        two_phase_geometry(p, gated, M, N1, N2, &sg);
        const double bh1 = sg.bh1;
        // a workgroup keeps a fixed number of bytes in flight, split between its row tile and its
        // weight tile in proportion to their widths: ~50 GB/s in all, of which the weights' share
        // (and never more than ~30 GB/s: three K steps of loads against a loaded memory latency)
        // the LDS-direct loop's eight-stage ring holds about a third more
        const bool deep = sg.bk == 32 && sg.bm < 256;
        // (the second phase's ring has eight stages only for 32-row blocks)
        const bool deep2 = deep && sg.bm == 32;
        const double wg_all = deep ? 65e9 : 50e9, wg_cap = deep ? 40e9 : 30e9;
        const double wg_all2 = deep2 ? 65e9 : 50e9, wg_cap2 = deep2 ? 40e9 : 30e9;
        const double per_wg1 = std::min(wg_cap, wg_all * (g * bh1) / (sg.bm + g * bh1)), per_wg2 = std::min(wg_cap2, wg_all2 * 256.0 / (sg.bm + 256.0));
        const double mb = cdiv(m, sg.bm), patches = cdiv(mb, sg.raster);
        const double n_s = cdiv(n1, bh1), ncb = cdiv(n2, 256);
        const double items1 = mb * n_s, items = mb * ncb * sg.splits;
        const double b1 = e * g * k * n1, b2 = e * n1 * n2;
        const double cols_per_patch = std::max(1.0, 32.0 / std::min(mb, (double)sg.raster));
        const double re1 = b1 * (patches - 1.0) + e * m * k * std::max(0.0, n_s / cols_per_patch / 8.0 - 1.0);
        const double re2 = b2 * (patches - 1.0) + e * m * n1 * std::max(0.0, ncb / cols_per_patch / 8.0 - 1.0) + e * m * n1;
        // pipeline fill and epilogue per item: the LDS-direct loop primes its ring faster (measured on the m = 128 tables)
        const double per_item = (sg.bk == 32 && sg.bm < 256) ? 1.5e-6 : 3e-6;
        // weights streamed with the non-temporal hint are not kept for the next row block: each streams its own copy
        const double copies = (weights_streamed(dtype, gated, K, N1, N2) && sg.bm < 256) ? mb : 1.0;
        const double t1 = copies * b1 / std::min(d.hbm_bw, std::min(items1, (double)d.cus) * per_wg1) + re1 / d.fabric_bw + per_item * cdiv(items1, d.cus);
        const double t2 = copies * b2 / std::min(d.hbm_bw, std::min(items, (double)d.cus) * per_wg2) + re2 / d.fabric_bw + per_item * cdiv(items, d.cus);
        // planes are written and read once; small transfers reach about half the cache rate
        const double planes = sg.splits > 1 ? 2.0 * 4.0 * m * n2 * sg.splits / (0.5 * d.fabric_bw) : 0.0;
        // matrix-core time of each phase: items run one per CU, at the block GEMM's efficiency
        // for the item's tile shape
        const double f1 = d.mfma_flops * block_gemm_efficiency(sg.bm, g * bh1, sg.bk == 32 || sg.bm == 256) / d.cus;
        const double f2 = d.mfma_flops * block_gemm_efficiency(sg.bm, 256.0, sg.bk == 32 || sg.bm == 256) / d.cus;
        // items are dealt statically, one per CU and round; a last, partly filled round is cheaper than a
        // full one (fewer CUs share the power budget and the L2: its items run faster) -- fitted exponent
        const auto rounds = [&](double n) {
            const double full = std::floor(n / d.cus), frac = n / d.cus - full;
            return full + (frac > 0.0 ? std::pow(frac, 0.6) : 0.0);
        };
        // the efficiencies above were measured on items whose inner loop runs over 4096: they contain those items'
        // ring fill and epilogue (about 10 us of a 256-row item, a tenth of it).  An item with a shorter loop
        // pays the same fixed part on less work: the part the calibration does not already contain is added.
        // (128-row items: 3.5 us, fitted on 32768 x 512 x 4096 x 512 and 65536 x 256 x 2048 x 256, where the model was 25-40 % optimistic)
        const double item_fixed = sg.bm == 256 ? 10e-6 : (sg.bm == 128 ? 3.5e-6 : 0.0);
        const auto short_loop = [&](double loop) { return item_fixed * std::max(0.0, 1.0 - loop / 4096.0); };
        const double m1 = (2.0 * sg.bm * bh1 * g * k / f1 + short_loop(k)) * rounds(items1);
        const double m2 = (2.0 * sg.bm * 256.0 * sg.ksplit / f2 + short_loop(sg.ksplit)) * rounds(items);
        t->workgroups = d.cus;
        // weights (and their repeats per patch), X once and its repeats, the intermediate written through and read
        // back, the output (through fp32 planes, written and read, when the hidden dimension is split)
        t->fabric_bytes = b1 + b2 + re1 + re2 + e * m * k + e * m * n1 + e * m * n2 +
                          (sg.splits > 1 ? 2.0 * 4.0 * m * n2 * sg.splits : 0.0);
        t->t_hbm = t1 + t2;
        t->t_mfma = m1 + m2;
        // launch, barrier, pipeline fills: 13 us.  (Where the barrier is per group the kernel is 2-3 us faster, but
        // crediting that moved the boundary to the reduce family the wrong way on the smallest shapes -- 196 x 256 x
        // 1024 x 256: reduce 13 us, two-phase 20 us, predicted 16.7 and 16.6 -- so the constant stays as fitted.)
        t->t_pred = std::max(t1, m1) + std::max(t2, m2) + planes + 13e-6;
    }
}

// Enumerates the plans the kernels implement, discards infeasible ones and ranks the rest by
// predicted time (Sec. 4.3, Algorithm 2 up to the top-k list; the on-device profiling of that
// list is ffuse_tune in the API layer).
void rank_plans(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, std::vector<RankedPlan>* out) {
    (void)act;
    out->clear();
    ffuse_plan_t best;
    std::memset(&best, 0, sizeof(best));
    if (dtype == FFUSE_DT_F32) {
        best.family = FFUSE_FAMILY_SCALAR;
        best.bm = 16; best.bh = 64; best.bn2 = 256; best.bk = 32; best.h_level = 1; best.raster = 1;
        best.splits = (int)((N1 + 63) / 64);
        out->push_back({0.0, best});
        return;
    }
    static const int tiles[][2] = {{256, 256}, {128, 256}, {256, 128}, {128, 128}, {128, 64}};
    static const int rasters[] = {1, 2, 4, 8, 16};
    for (auto& tl : tiles) {
        if (!fused_reduce_tile_ok(gated, tl[0], tl[1])) continue;
        for (int r : rasters) {
            ffuse_plan_t p;
            std::memset(&p, 0, sizeof(p));
            p.family = FFUSE_FAMILY_REDUCE;
            p.bm = tl[0]; p.bh = tl[1]; p.bn2 = 128; p.bk = 64; p.h_level = 0; p.raster = r;
            p.splits = (int)((N1 + p.bh - 1) / p.bh);
            if (r > 1 && r > (M + p.bm - 1) / p.bm) continue;
            ffuse_traffic_t t;
            traffic_model(p, dtype, gated, M, K, N1, N2, &t);
            if (!t.feasible) continue;
            out->push_back({t.t_pred, p});
        }
    }
    {
        static const int splits[] = {1, 2, 4, 8, 16, 32};
        static const int bms[] = {32, 64, 128, 256};
        static const int rasters2[] = {4, 2, 8, 1};   // the model does not tell these apart: measured order of preference
        for (int bm : bms) {
            // measured: two 64-row blocks beat one of 128 on the m = 128 shapes (half the row-operand
            // bytes per item, half the planes); more, or smaller, blocks lose
            if (bm < 128 && M > (bm == 64 ? 128 : bm)) continue;
            if (bm > 32 && M <= bm / 2) continue;             // more than half a block of padding
            // 128 / 64 / 32: register-staged loop with that slice width; -128 / -64: LDS-direct loop
            static const int slices[] = {128, 64, 32, -128, -64};
            for (int sl : slices) {
                const int bh1 = sl < 0 ? -sl : sl;
                if (bm == 256 && sl != 128) continue;                         // the 256-row kernel has one variant
                if ((bh1 == 64 && bm < 64) || (bh1 == 32 && (bm != 128 || gated))) continue;
                for (int sp : splits) {
                    if (sp > two_phase_max_splits(M, N2)) continue;
                    for (int r : rasters2) {
                        if (r > 1 && r > (M + bm - 1) / bm) continue;   // a patch cannot have more row blocks than there are
                        ffuse_plan_t p;
                        std::memset(&p, 0, sizeof(p));
                        p.family = FFUSE_FAMILY_TWOPHASE;
                        p.bm = bm; p.bh = bm == 256 ? (gated ? 128 : 256) : bh1; p.bn2 = 256; p.bk = (bm == 256 || sl < 0) ? 32 : 64; p.h_level = 2; p.raster = r;
                        p.splits = sp;
                        ffuse_traffic_t t;
                        traffic_model(p, dtype, gated, M, K, N1, N2, &t);
                        if (!t.feasible) continue;
                        out->push_back({t.t_pred, p});
                    }
                }
            }
        }
    }
    if (gated) {
        // the best two-phase plan with its branches on different workgroups (never predicted faster: it is there to be measured)
        const RankedPlan* b = nullptr;
        for (const RankedPlan& c : *out)
            if (c.plan.family == FFUSE_FAMILY_TWOPHASE && (!b || c.t_pred < b->t_pred)) b = &c;
        if (b) {
            ffuse_plan_t p = b->plan;
            p.gate_split = 1;
            if (p.bm == 256) p.bh = 256;
            ffuse_traffic_t t;
            traffic_model(p, dtype, gated, M, K, N1, N2, &t);
            if (t.feasible) out->push_back({t.t_pred, p});
        }
    }
    {
        ffuse_plan_t p;
        std::memset(&p, 0, sizeof(p));
        p.family = FFUSE_FAMILY_ROWS;
        p.bm = 64; p.bh = 64; p.bn2 = (int)std::min<int64_t>(N2, 1024); p.bk = 16; p.h_level = 1; p.raster = 1; p.splits = 1;
        ffuse_traffic_t t;
        traffic_model(p, dtype, gated, M, K, N1, N2, &t);
        if (t.feasible) out->push_back({t.t_pred, p});
    }
    static const int producers[] = {8, 12, 16, 20, 24};
    for (int pr : producers) {
        ffuse_plan_t p;
        std::memset(&p, 0, sizeof(p));
        p.family = FFUSE_FAMILY_EXCHANGE;
        p.bm = 256; p.bh = gated ? 128 : 256; p.bn2 = 256; p.bk = 64; p.h_level = 2; p.raster = 1; p.splits = 1;
        p.producers = pr; p.ring = kExchangeMaxRing;
        ffuse_traffic_t t;
        traffic_model(p, dtype, gated, M, K, N1, N2, &t);
        if (!t.feasible) continue;
        out->push_back({t.t_pred, p});
    }
    // stable: among equal predictions the enumeration order (the measured preference) decides
    std::stable_sort(out->begin(), out->end(), [](const RankedPlan& x, const RankedPlan& y) { return x.t_pred < y.t_pred; });
}

void choose_plan(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, ffuse_plan_t* out, int objective) {
    std::vector<RankedPlan> r;
    rank_plans(dtype, act, gated, M, K, N1, N2, &r);
    if (r.empty()) {
        std::memset(out, 0, sizeof(*out));
        return;
    }
    *out = r.front().plan;
    if (objective != FFUSE_OBJECTIVE_BYTES) {
        // time objective: a near-tie goes to the schedule that keeps the traffic on the chip -- a plan predicted
        // within 6 % of the fastest whose bytes between the L2s and the fabric are at most half of its
        ffuse_traffic_t tb;
        traffic_model(*out, dtype, gated, M, K, N1, N2, &tb);
        for (const RankedPlan& c : r) {
            if (c.t_pred > 1.06 * r.front().t_pred) break;
            ffuse_traffic_t t;
            traffic_model(c.plan, dtype, gated, M, K, N1, N2, &t);
            if (t.feasible && t.fabric_bytes <= 0.5 * tb.fabric_bytes) { *out = c.plan; tb = t; }
        }
        return;
    }
    // fewest bytes between the L2s and the rest of the memory system among the plans predicted within
    // kBytesObjectiveSlack of the fastest (the ranking is sorted: stop at the first plan beyond the slack)
    double best_bytes = 0.0;
    bool have = false;
    for (const RankedPlan& c : r) {
        if (c.t_pred > kBytesObjectiveSlack * r.front().t_pred) break;
        ffuse_traffic_t t;
        traffic_model(c.plan, dtype, gated, M, K, N1, N2, &t);
        if (!t.feasible) continue;
        if (!have || t.fabric_bytes < best_bytes) { best_bytes = t.fabric_bytes; *out = c.plan; have = true; }
    }
}

size_t plan_workspace_bytes(const ffuse_plan_t& p, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2) {
    (void)K;
    switch (p.family) {
        case FFUSE_FAMILY_REDUCE: return sizeof(float) * (size_t)M * (size_t)N2;
        case FFUSE_FAMILY_EXCHANGE: {
            ExchangeGeometry e;
            return exchange_geometry(p, gated, M, N1, N2, kDevice.cus, &e) ? e.ws_bytes : 0;
        }
        case FFUSE_FAMILY_TWOPHASE: {
            TwoPhaseGeometry t;
            return two_phase_geometry(p, gated, M, N1, N2, &t) ? t.ws_bytes : 0;
        }
        case FFUSE_FAMILY_UNFUSED: return (dtype == FFUSE_DT_F32 ? 4 : 2) * (size_t)M * (size_t)N1;
        case FFUSE_FAMILY_ROWS: return 0;
        default: return 0;
    }
}

// Sec. 4.2 (LoopSchedule) and the table of spatial / temporal partitions in Sec. 4.3: a schedule picks which
// of the four loop dimensions (m, n, k, l) are spatial -- at least one -- and orders the temporal rest.
int loop_schedule_count(int spatial_dims) {
    const auto fact = [](int n) { int f = 1; for (int i = 2; i <= n; ++i) f *= i; return f; };
    const auto choose = [&](int n, int r) { return fact(n) / (fact(r) * fact(n - r)); };
    if (spatial_dims < 0 || spatial_dims > 4) return 0;
    if (spatial_dims > 0) return choose(4, spatial_dims) * fact(4 - spatial_dims);
    int total = 0;
    for (int sdim = 1; sdim <= 4; ++sdim) total += choose(4, sdim) * fact(4 - sdim);
    return total;
}

// Sec. 4.1: blocks of a shuffle group exchange their slices of the intermediate; the groups that hold
// partial sums of the same output block are reduced.  cls_shuffle = cls_l / cls_k, cls_reduce = cls_n cls_k / cls_l.
bool cluster_exchange(int cls_n, int cls_k, int cls_l, int* cls_shuffle, int* cls_reduce) {
    if (cls_n < 1 || cls_k < 1 || cls_l < 1 || cls_l % cls_k || (cls_n * cls_k) % cls_l) return false;
    *cls_shuffle = cls_l / cls_k;
    *cls_reduce = cls_n * cls_k / cls_l;
    return true;
}

int m_bin(int64_t M) {
    int b = 0;
    for (int64_t edge = 16; edge < M; edge <<= 1) ++b;
    return b;
}

}  // namespace ffuse
