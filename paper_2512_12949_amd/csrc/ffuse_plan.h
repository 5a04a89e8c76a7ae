// Host-side plan chooser / traffic model interface (no device code, no torch types).
#pragma once
#include <vector>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ffuse.h"

namespace ffuse {

struct Device {
    int cus, xcds;
    double mfma_flops;   // sustained dense 16-bit MFMA rate, flop/s
    double hbm_bw;       // achievable HBM read bandwidth, B/s
    double fabric_bw;    // Infinity Cache -> L2 fill bandwidth, B/s
    double l2_bw;        // L2 -> CU, all CUs, B/s
    double lds_bw;       // LDS read, all CUs, B/s
    double atomic_bw;    // fp32 atomic-add bytes per second, whole chip
    double lds_bytes;    // per workgroup
    double acc_regs;     // accumulator registers per lane at one wave per SIMD
    double l2_bytes, mall_bytes;
    double mfma_eff;     // fraction of mfma_flops the library's main loop sustains
    double launch_s;     // fixed cost of one kernel launch
};
extern Device kDevice;              // starts as a whole MI355X (256 CUs in 8 XCDs)
// Unit counts of the device the library runs on (a partitioned or harvested part has fewer): the
// per-unit rates stay, everything that scales with the unit count is rescaled.
void set_device_units(int cus);

// Exchange family: derived launch geometry of a plan for one problem.
constexpr size_t kExchangeFlagBytes = 8192;
constexpr size_t kTwoPhaseFlagBytes = 1024;   // barrier counters of the two-phase family, behind its H
constexpr int kExchangeMaxRing = 64;
struct ExchangeGeometry {
    int wgs_per_group;  // workgroups per XCD group = CUs / 8
    int P, NCT, PG, R, NH;
    size_t ws_bytes;    // flags + ring
};
bool exchange_geometry(const ffuse_plan_t& p, int gated, int64_t M, int64_t N1, int64_t N2, int cus, ExchangeGeometry* out);

// Two-phase family: derived geometry.
struct TwoPhaseGeometry {
    int bm;             // rows per block: 32, 64, 128 or 256
    int bk;             // 32: LDS-direct block GEMM (always for bm = 256; optional for bm = 64 / 128 with bh1 = 128); 64: register-staged
    int bh1;            // hidden slice of a phase-1 item: 128 / 64 / 32 (bm <= 128), 256 or 128 gated (bm = 256)
    int splits, ksplit; // phase-2 ranges of the hidden dimension (splits == 1: no partial planes)
    int raster;         // row blocks per XCD patch
    int gate_split;     // gated chain with its branches on different workgroups (phase-1 items are not gated then)
    size_t ysum_bytes, h_bytes, u_bytes, ws_bytes;   // workspace layout: partial-sum planes | H | U (gate_split) | flags (kTwoPhaseFlagBytes)
};
// most hidden-dimension ranges the chooser considers for an M x N2 output (bounds the workspace)
int two_phase_max_splits(int64_t M, int64_t N2);
// Weights far larger than the 256 MB memory-side cache (above 512 MB): the two-phase kernel streams
// them with the non-temporal hint (row blocks below 256)
bool weights_streamed(int dtype, int gated, int64_t K, int64_t N1, int64_t N2);
bool two_phase_geometry(const ffuse_plan_t& p, int gated, int64_t M, int64_t N1, int64_t N2, TwoPhaseGeometry* out);
// Which groups of workgroups (blockIdx % 8; the kernel deals its work items group by group) a group has to
// wait for between the phases: byte g of the result has bit h set when some phase-2 item of group g reads a
// tile of H that a phase-1 item of group h writes.  All ones when the item counts are too large to enumerate.
uint64_t two_phase_wait_masks(const TwoPhaseGeometry& g, int64_t M, int64_t N1, int64_t N2);
// every group waits for itself alone
bool two_phase_groups_independent(const TwoPhaseGeometry& g, int64_t M, int64_t N1, int64_t N2);

// Rows family (row-stationary): which kernel instantiation runs a plan.
struct RowsGeometry {
    int nks;   // 16-k steps of the first product per wave: 8 (K <= 512) or 16 (K <= 1024)
    int nt2;   // 32-column output tiles per wave: 4 (N2 <= 512) or 8 (N2 <= 1024)
};
bool rows_geometry(const ffuse_plan_t& p, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, RowsGeometry* out);

bool fused_reduce_tile_ok(int gated, int bm, int bh);
bool plan_valid(const ffuse_plan_t& p, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2);
void traffic_model(const ffuse_plan_t& p, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                   ffuse_traffic_t* out);
// All plans the kernels implement for this problem that pass the capacity constraints,
// in order of increasing predicted time (Sec. 4.3, Algorithm 2: the analytical ranking that
// precedes the on-device profiling of the top-k list).
struct RankedPlan {
    double t_pred;
    ffuse_plan_t plan;
};
void rank_plans(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, std::vector<RankedPlan>* out);
// objective: FFUSE_OBJECTIVE_TIME -- the plan with the smallest predicted time; FFUSE_OBJECTIVE_BYTES -- among the
// plans predicted within kBytesObjectiveSlack of that time, the one that moves the fewest bytes between the L2s
// and the rest of the memory system
constexpr double kBytesObjectiveSlack = 1.35;
void choose_plan(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, ffuse_plan_t* out,
                 int objective = FFUSE_OBJECTIVE_TIME);
// Bytes of workspace a plan needs for this problem.
size_t plan_workspace_bytes(const ffuse_plan_t& p, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2);
// The paper's bookkeeping of the search space (host arithmetic only; the chooser above enumerates the few
// schedules that survive its pruning rules on this device, these two functions restate the full space)
int loop_schedule_count(int spatial_dims);   // schedules with that many spatial dimensions (0: all of them)
bool cluster_exchange(int cls_n, int cls_k, int cls_l, int* cls_shuffle, int* cls_reduce);
// Bin of the row count for the plan table (Sec. 4.3: plans are chosen offline per range of
// the dynamic dimension M and looked up at run time): 0 for M <= 16, then one per power of two.
int m_bin(int64_t M);

}  // namespace ffuse
