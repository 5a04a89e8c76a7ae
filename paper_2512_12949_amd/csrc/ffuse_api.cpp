// C-ABI layer of libffuse.so: argument validation, plan selection, workspace bookkeeping
// and kernel launches.  See include/ffuse.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <array>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include "../../include/ffuse.h"
#include "ffuse_launch.h"
#include "ffuse_plan.h"

namespace {

// What the library remembers about a caller-owned workspace between calls: how much of its start is
// known to be zero (the reduce family keeps its sums there) and where the two-phase family last left
// clean barrier flags.  A workspace the library has not seen (or whose size changed) counts as dirty.
struct Workspace {
    void* ptr = nullptr;
    size_t bytes = 0;
    size_t zero = 0;                  // bytes at the start known to be zero
    uint32_t* small_flags = nullptr;  // where the two-phase family last left clean barrier flags
    uint64_t used = 0;                // age, for replacement
    bool in_graph = false;            // a call on this workspace was recorded into a graph: replays the library does
                                      // not see may dirty it at any time, so nothing above is trusted any more
};

// geometry of a 3x3 first convolution (ic == 0: the first product is a plain GEMM)
struct ConvGeom {
    int ic = 0, h = 0, w = 0;
};

struct State {
    std::mutex mu;
    Workspace reg;           // the workspace registered with ffuse_set_workspace
    Workspace seen[8];       // workspaces passed per call (ffuse_ffn_ws ...), most recently used kept
    uint64_t clock = 0;
    uint32_t spin_limit = 1u << 24;   // bounded waits of the two-phase barrier (ffuse_debug_barrier)
    int extra_arrivals = 0;
    int objective = FFUSE_OBJECTIVE_TIME;
    bool no_alloc_call = false;   // inside ffuse_ffn_static: nothing that could allocate (no profiling events)
    bool forced = false;
    ffuse_plan_t forced_plan{};
    ffuse_plan_t last_plan{};
    bool env_checked = false;
    bool profiling = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
    int arch_ok = -1;        // -1 unknown, 0 no, 1 yes
    int cus = 0;             // compute units of the current device
    uint32_t* exch_err = nullptr;  // device address of the error word of the last exchange launch
    bool log = std::getenv("FFUSE_LOG") != nullptr;  // diagnostics on stderr
    uint64_t* exch_stats = nullptr;
    bool small_split = false;
    uint64_t* small_stats = nullptr;
    uint64_t* rows_stats = nullptr;
    int rows_wgs = 0;
    int exch_wgs = 0;
    // plan table (Sec. 4.3: plans are fixed ahead of time per range of the dynamic dimension M
    // and looked up at run time).  Key: dtype, gated, K, N1, N2 and either the M bin (plans
    // measured by ffuse_tune) or, negated, the exact M (plans chosen by the model).
    struct TableEntry {
        ffuse_plan_t plan;
        double ms;        // measured time of a tuned plan; 0 for a modelled one
    };
    std::map<std::array<int64_t, 6>, TableEntry> table;
};
State g;

// the record of a per-call workspace; the caller holds the lock
Workspace& workspace_record(void* ptr, size_t bytes) {
    Workspace* oldest = &g.seen[0];
    for (Workspace& w : g.seen) {
        if (w.ptr == ptr && w.bytes == bytes) { w.used = ++g.clock; return w; }
        if (w.used < oldest->used) oldest = &w;
    }
    *oldest = Workspace{ptr, bytes, 0, nullptr, ++g.clock, false};
    return *oldest;
}
// forget what is known about any record that overlaps [ptr, ptr + bytes): its memory is about to change hands
void forget_overlapping(const void* ptr, size_t bytes) {
    const char* a = static_cast<const char*>(ptr);
    for (Workspace& w : g.seen) {
        const char* b = static_cast<const char*>(w.ptr);
        if (w.ptr && a < b + w.bytes && b < a + bytes) w = Workspace{};
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_arch() {
    if (g.arch_ok < 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return FFUSE_ERR_LAUNCH;
        g.arch_ok = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 0;
        g.cus = prop.multiProcessorCount;
        ffuse::set_device_units(g.cus);
    }
    return g.arch_ok == 1 ? FFUSE_OK : FFUSE_ERR_ARCH;
}

int validate(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
             int64_t N1, int64_t N2, const void* Y, int elem) {
    if (!X || !W1 || !W2 || !Y) return FFUSE_ERR_NULL;
    if (act < FFUSE_ACT_IDENTITY || act > FFUSE_ACT_SILU) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8 || (K % 8) || (N1 % 8) || (N2 % 8)) return FFUSE_ERR_SHAPE;
    const int64_t lim = (int64_t)1 << 31;
    // (the M x N1 intermediate counts as a tensor: the kernels that keep it in the workspace address it, like
    // the operands, through 32-bit buffer offsets, and mask lanes with an offset of 2^31)
    if ((M + 256) * K * elem >= lim || (K + 128) * N1 * elem >= lim || (N1 + 512) * N2 * elem >= lim ||
        M * N2 * 4 >= ((int64_t)1 << 40) || M * N2 * elem >= lim || (M + 256) * N1 * elem >= lim)
        return FFUSE_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(W1) || !aligned16(W2) || !aligned16(Y) || (W3 && !aligned16(W3)))
        return FFUSE_ERR_ALIGN;
    return FFUSE_OK;
}

void read_env_plan() {
    if (g.env_checked) return;
    g.env_checked = true;
    const char* s = std::getenv("FFUSE_FORCE_PLAN");
    if (!s || !*s) return;
    int v[12] = {0, 0, 0, 128, 64, 0, 0, 4, 0, 0, 0, 0};
    const int n = std::sscanf(s, "%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", &v[0], &v[1], &v[2], &v[3], &v[4], &v[5], &v[6], &v[7],
                              &v[8], &v[9], &v[10], &v[11]);
    if (n >= 3) {
        std::memset(&g.forced_plan, 0, sizeof(g.forced_plan));
        g.forced_plan.family = v[0]; g.forced_plan.bm = v[1]; g.forced_plan.bh = v[2]; g.forced_plan.bn2 = v[3];
        g.forced_plan.bk = v[4]; g.forced_plan.splits = v[5]; g.forced_plan.h_level = v[6]; g.forced_plan.raster = v[7];
        g.forced_plan.producers = v[8]; g.forced_plan.ring = v[9]; g.forced_plan.coherent = v[10];
        g.forced_plan.gate_split = v[11];
        g.forced = true;
    }
}

// makes the first `need` bytes of the workspace zero (they usually already are)
bool ensure_zero(Workspace& w, size_t need, hipStream_t st) {
    if (w.zero >= need) return true;
    if (ffuse::launch_zero(w.ptr, (need + 15) & ~(size_t)15, st) != hipSuccess) return false;
    w.zero = need;
    return true;
}

// A launch recorded into a graph runs later, any number of times, between other calls: what the library
// knows about the workspace now says nothing about its state then, so a captured call always records its
// own clearing -- and from then on every call on that workspace, recorded or not, clears what it needs: a
// replay may have run since the last call the library saw.
bool stream_is_capturing(hipStream_t st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone;
}

struct Timer {  // brackets the dominant kernel with events when profiling is on
    hipStream_t st;
    hipEvent_t a = nullptr, b = nullptr;
    explicit Timer(hipStream_t s) : st(s) {
        if (g.profiling && !g.no_alloc_call && hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) (void)hipEventRecord(a, st);
    }
    void stop() {
        if (a && b) {
            (void)hipEventRecord(b, st);
            g.events.emplace_back(a, b);
            a = b = nullptr;
        }
    }
};

std::array<int64_t, 6> table_key(int dtype, int gated, int64_t K, int64_t N1, int64_t N2, int64_t m_or_bin) {
    return {dtype, gated, K, N1, N2, m_or_bin};
}

// a0: the plan for this call -- a tuned plan of M's bin if there is one that fits, else the
// model's choice for exactly this M (computed once, then looked up).  ws_bytes: the workspace the
// call will run in (0: none yet, nothing to fit).
ffuse_plan_t lookup_plan(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, size_t ws_bytes) {
    auto it = g.table.find(table_key(dtype, gated, K, N1, N2, ffuse::m_bin(M)));
    if (it != g.table.end() && ffuse::plan_valid(it->second.plan, dtype, gated, M, K, N1, N2) &&
        (!ws_bytes || ffuse::plan_workspace_bytes(it->second.plan, dtype, gated, M, K, N1, N2) <= ws_bytes))
        return it->second.plan;
    const auto key = table_key(dtype + 64 * g.objective, gated, K, N1, N2, -M);   // (modelled plans: one slot per objective)
    it = g.table.find(key);
    if (it != g.table.end()) return it->second.plan;
    ffuse_plan_t plan;
    ffuse::choose_plan(dtype, act, gated, M, K, N1, N2, &plan, g.objective);
    if (g.table.size() > 4096) g.table.clear();
    g.table[key] = {plan, 0.0};
    return plan;
}

int run_plan(const ffuse_plan_t& plan, int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act,
             int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, Workspace& w, void* stream, bool two_launches = false,
             const ConvGeom& conv = ConvGeom{});

// `ws`: the workspace of this call (nullptr: the registered one); the caller holds the lock
int run_fused_locked(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                     int64_t N1, int64_t N2, void* Y, Workspace& w, void* stream) {
    int rc = check_arch();
    if (rc != FFUSE_OK) return rc;
    read_env_plan();
    const int gated = W3 != nullptr;
    ffuse_plan_t plan;
    if (g.forced && g.forced_plan.family != FFUSE_FAMILY_AUTO) {
        plan = g.forced_plan;
        if (!ffuse::plan_valid(plan, dtype, gated, M, K, N1, N2) || plan.family == FFUSE_FAMILY_UNFUSED) return FFUSE_ERR_PLAN;
    } else {
        plan = lookup_plan(dtype, act, gated, M, K, N1, N2, w.ptr ? w.bytes : 0);
    }
    return run_plan(plan, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, w, stream);
}

int run_fused(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
              int64_t N1, int64_t N2, void* Y, void* stream) {
    const int elem = dtype == FFUSE_DT_F32 ? 4 : 2;
    int rc = validate(X, W1, W3, W2, act, M, K, N1, N2, Y, elem);
    if (rc != FFUSE_OK) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    return run_fused_locked(dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, g.reg, stream);
}

// Weights far larger than the 256 MB memory-side cache are streamed with the non-temporal
// hint (measured on the 1.4 GB decode shapes: 9 % faster, 5.8 instead of 5.3 TB/s); weights the
// cache can keep between calls are not (the hint cost 10-40 % on the 64-270 MB shapes when the
// same weights are used call after call).
int stream_weights(int dtype, int gated, int64_t K, int64_t N1, int64_t N2) {
    if (const char* env = std::getenv("FFUSE_NT")) return std::atoi(env) != 0;   // read per call: a test can switch it
    return ffuse::weights_streamed(dtype, gated, K, N1, N2) ? 1 : 0;
}

// The barrier's wait masks are an enumeration of the kernel's item maps (thousands of items at the large
// shapes): remembered for the last few (geometry, shape) pairs, so that a serving loop pays for them once.
// The caller holds the lock.
uint64_t wait_masks(const ffuse::TwoPhaseGeometry& sg, int64_t M, int64_t N1, int64_t N2) {
    struct Entry { int bm, bh1, splits, ksplit, raster; int64_t M, N1, N2; uint64_t masks; bool used; };
    static Entry cache[8] = {};
    static int next = 0;
    for (const Entry& e : cache)
        if (e.used && e.bm == sg.bm && e.bh1 == sg.bh1 && e.splits == sg.splits && e.ksplit == sg.ksplit && e.raster == sg.raster &&
            e.M == M && e.N1 == N1 && e.N2 == N2)
            return e.masks;
    const uint64_t m = ffuse::two_phase_wait_masks(sg, M, N1, N2);
    cache[next] = Entry{sg.bm, sg.bh1, sg.splits, sg.ksplit, sg.raster, M, N1, N2, m, true};
    next = (next + 1) % 8;
    return m;
}

// FFUSE_GROUP_BARRIER=0: the barrier between the phases always waits for every workgroup; read per call
bool group_barrier() {
    const char* env = std::getenv("FFUSE_GROUP_BARRIER");
    return !env || std::atoi(env) != 0;
}

// FFUSE_EARLY_FILL=0: 256-row tiles start a workgroup's next first-phase ring fill after the epilogue instead of
// under it (for A/B timing; same bits); read per call
int early_fill() {
    const char* env = std::getenv("FFUSE_EARLY_FILL");
    return (!env || std::atoi(env) != 0) ? 1 : 0;
}

// launches one validated plan in workspace `w`; the caller holds the lock.  two_launches (two-phase
// family only): each phase is a launch of its own and the kernel boundary replaces the barrier.
int run_plan(const ffuse_plan_t& plan, int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act,
             int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, Workspace& w, void* stream, bool two_launches,
             const ConvGeom& conv) {
    const int gated = W3 != nullptr;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (stream_is_capturing(st)) w.in_graph = true;
    if (w.in_graph) { w.zero = 0; w.small_flags = nullptr; }
    // (and whatever this call leaves behind, a replay may find something else)
    struct Forget {
        Workspace& w;
        ~Forget() { if (w.in_graph) { w.zero = 0; w.small_flags = nullptr; } }
    } forget{w};
    ffuse::FusedArgs a{X, W1, W3, W2, nullptr, M, (int)K, (int)N1, (int)N2, act, plan.raster > 0 ? plan.raster : 1};
    if (plan.family == FFUSE_FAMILY_SCALAR) {
        Timer t(st);
        if (ffuse::launch_fused_f32(a, reinterpret_cast<float*>(Y), st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        t.stop();
        g.last_plan = plan;
        g.exch_err = nullptr;
        return FFUSE_OK;
    }
    if (plan.family == FFUSE_FAMILY_ROWS) {
        ffuse::RowsGeometry rg;
        if (!ffuse::rows_geometry(plan, gated, M, K, N1, N2, &rg)) return FFUSE_ERR_PLAN;
        ffuse::RowsArgs r{X, W1, W3, W2, Y, M, (int)K, (int)N1, (int)N2, act, nullptr};
        g.rows_stats = nullptr;
        if (g.log && w.ptr && w.bytes >= 16 * 1024) {   // diagnostics only: the family itself needs no workspace
            r.stats = reinterpret_cast<uint64_t*>(w.ptr);
            g.rows_stats = r.stats;
            g.rows_wgs = (int)std::min<int64_t>((M + 63) / 64, g.cus);
            w.zero = 0; w.small_flags = nullptr;
        }
        Timer t(st);
        const int64_t mb = (M + 63) / 64;
        if (ffuse::launch_fused_rows(dtype, r, rg.nks, rg.nt2, (int)std::min<int64_t>(mb, g.cus), st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        t.stop();
        g.last_plan = plan;
        g.exch_err = nullptr;
        return FFUSE_OK;
    }
    if (plan.family == FFUSE_FAMILY_EXCHANGE) {
        ffuse::ExchangeGeometry e;
        if (!ffuse::exchange_geometry(plan, gated, M, N1, N2, g.cus, &e)) return FFUSE_ERR_PLAN;
        if (!w.ptr || w.bytes < e.ws_bytes) return FFUSE_ERR_WORKSPACE;
        char* base = reinterpret_cast<char*>(w.ptr);
        if (ffuse::launch_zero(base, ffuse::kExchangeFlagBytes, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        w.zero = 0;      // the ring overwrites the region the other families keep at zero
        w.small_flags = nullptr;
        ffuse::ExchangeArgs x{X, W1, W3, W2, Y, base + ffuse::kExchangeFlagBytes, reinterpret_cast<uint32_t*>(base),
                              M, (int)K, (int)N1, (int)N2, act, e.P, e.NCT, e.PG, e.R, e.NH, plan.coherent, nullptr};
        if (g.log && w.bytes >= e.ws_bytes + 8192 * 4) {
            x.stats = reinterpret_cast<uint64_t*>(base + e.ws_bytes);
            g.exch_stats = x.stats;
            g.exch_wgs = 8 * e.wgs_per_group;
            if (ffuse::launch_zero(x.stats, 8192 * 4, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        }
        g.exch_err = reinterpret_cast<uint32_t*>(base) + 16 * e.R;
        Timer t(st);
        if (ffuse::launch_fused_exchange(dtype, x, e.wgs_per_group, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        t.stop();
        g.last_plan = plan;
        return FFUSE_OK;
    }
    if (plan.family == FFUSE_FAMILY_TWOPHASE) {
        ffuse::TwoPhaseGeometry sg;
        if (!ffuse::two_phase_geometry(plan, gated, M, N1, N2, &sg)) return FFUSE_ERR_PLAN;
        if (!w.ptr || w.bytes < sg.ws_bytes) return FFUSE_ERR_WORKSPACE;
        char* base = reinterpret_cast<char*>(w.ptr);
        uint32_t* flags = reinterpret_cast<uint32_t*>(base + sg.ysum_bytes + sg.h_bytes + sg.u_bytes);
        if (sg.gate_split && two_launches) return FFUSE_ERR_PLAN;   // (the Mul pass sits between two rendezvous of one launch)
        if (w.small_flags != flags) {
            if (ffuse::launch_zero(flags, ffuse::kTwoPhaseFlagBytes, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
            w.small_flags = flags;
        }
        w.zero = 0;      // planes and H overwrite the region the reduce family keeps at zero
        ffuse::TwoPhaseArgs s{X, W1, W3, W2, base + sg.ysum_bytes, Y, reinterpret_cast<float*>(base), flags,
                              M, (int)K, (int)N1, (int)N2, act, sg.splits, sg.ksplit, sg.raster, nullptr,
                              conv.ic, conv.h, conv.w, stream_weights(dtype, gated, K, N1, N2),
                              group_barrier() ? wait_masks(sg, M, N1, N2) : ~(uint64_t)0, 3,
                              g.spin_limit, g.extra_arrivals, early_fill(), sg.gate_split ? base + sg.ysum_bytes + sg.h_bytes : nullptr};
        if (g.log && w.bytes >= sg.ws_bytes + 65536) {
            s.stats = reinterpret_cast<uint64_t*>(base + sg.ws_bytes);
            g.small_stats = s.stats;
            g.small_split = two_launches;
        }
        // (launched one phase at a time there is no barrier and no verdict)
        g.exch_err = two_launches ? nullptr : flags + 3;
        {
            Timer t(st);
            if (two_launches) {
                s.phases = 1;
                if (ffuse::launch_fused_two_phase(dtype, s, sg.bm, sg.bh1, sg.bk, g.cus, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
                s.phases = 2;
                if (s.stats) s.stats += 4 * 1024;
            }
            if (ffuse::launch_fused_two_phase(dtype, s, sg.bm, sg.bh1, sg.bk, g.cus, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
            if (sg.splits > 1 && ffuse::launch_finalize_planes(dtype, s.part, Y, M * N2, sg.splits, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
            t.stop();
        }
        g.last_plan = plan;
        return FFUSE_OK;
    }
    if (plan.family != FFUSE_FAMILY_REDUCE) return FFUSE_ERR_PLAN;
    const size_t need = sizeof(float) * (size_t)M * (size_t)N2;
    if (!w.ptr || w.bytes < need) return FFUSE_ERR_WORKSPACE;
    if (!ensure_zero(w, need, st)) return FFUSE_ERR_LAUNCH;
    w.small_flags = nullptr;   // (the sums may lie over the two-phase family's flags)
    a.Ysum = reinterpret_cast<float*>(w.ptr);
    g.exch_err = nullptr;
    {
        Timer t(st);
        if (ffuse::launch_fused_reduce(dtype, a, plan.bm, plan.bh, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        if (ffuse::launch_finalize(dtype, a.Ysum, Y, M * N2, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
        t.stop();
    }
    g.last_plan = plan;
    return FFUSE_OK;
}

// The comparison path: the same two GEMMs with the intermediate written and re-read between
// two launches.  16-bit types run the two-phase family's kernel one phase per launch, in
// the tile plan the model ranks best for this shape, so that the only differences from the
// fused call are the second launch and the kernel boundary in place of the barrier.
int run_unfused_locked(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M,
                       int64_t K, int64_t N1, int64_t N2, void* Y, Workspace& w, void* stream) {
    const int elem = dtype == FFUSE_DT_F32 ? 4 : 2;
    int rc = check_arch();
    if (rc != FFUSE_OK) return rc;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (dtype != FFUSE_DT_F32) {
        const int gated = W3 != nullptr;
        const auto key = table_key(dtype + 16, gated, K, N1, N2, -M);   // its own slot beside the fused plans
        auto it = g.table.find(key);
        if (it == g.table.end()) {
            std::vector<ffuse::RankedPlan> ranked;
            ffuse::rank_plans(dtype, act, gated, M, K, N1, N2, &ranked);
            ffuse_plan_t best{};
            for (const auto& r : ranked)
                if (r.plan.family == FFUSE_FAMILY_TWOPHASE) { best = r.plan; break; }
            if (best.family != FFUSE_FAMILY_TWOPHASE) return FFUSE_ERR_PLAN;
            if (g.table.size() > 4096) g.table.clear();
            g.table[key] = {best, 0.0};
            it = g.table.find(key);
        }
        const ffuse_plan_t keep = g.last_plan;
        rc = run_plan(it->second.plan, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, w, stream, true);
        g.last_plan = keep;   // ffuse_last_plan reports fused calls only
        return rc;
    }
    const size_t need = (size_t)elem * (size_t)M * (size_t)N1;
    if (!w.ptr || w.bytes < need) return FFUSE_ERR_WORKSPACE;
    w.zero = 0;      // H overwrites whatever the fused path kept at zero
    w.small_flags = nullptr;
    g.exch_err = nullptr;
    ffuse::GemmArgs g0{X, W1, W3, w.ptr, M, (int)K, (int)N1, act};
    ffuse::GemmArgs g1{w.ptr, W2, nullptr, Y, M, (int)N1, (int)N2, FFUSE_ACT_IDENTITY};
    Timer t(st);
    if (ffuse::launch_gemm_act_f32(g0, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
    if (ffuse::launch_gemm_act_f32(g1, st) != hipSuccess) return FFUSE_ERR_LAUNCH;
    t.stop();
    return FFUSE_OK;
}

int run_unfused(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M,
                int64_t K, int64_t N1, int64_t N2, void* Y, void* stream) {
    const int elem = dtype == FFUSE_DT_F32 ? 4 : 2;
    int rc = validate(X, W1, W3, W2, act, M, K, N1, N2, Y, elem);
    if (rc != FFUSE_OK) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    return run_unfused_locked(dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, g.reg, stream);
}

// the workspace argument of a per-call entry point: nullptr / 0 is allowed (families that need none)
int check_ws_arg(const void* ws, size_t bytes) {
    if (!ws) return bytes == 0 ? FFUSE_OK : FFUSE_ERR_NULL;
    if (!aligned16(ws)) return FFUSE_ERR_ALIGN;
    if (bytes % 16) return FFUSE_ERR_SHAPE;
    return FFUSE_OK;
}

}  // namespace

extern "C" {

int ffuse_ffn(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K, int64_t N1,
              int64_t N2, void* Y, void* stream) {
    return run_fused(FFUSE_DT_BF16, X, W1, W3, W2, act, M, K, N1, N2, Y, stream);
}
int ffuse_ffn_f16(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                  int64_t N1, int64_t N2, void* Y, void* stream) {
    return run_fused(FFUSE_DT_F16, X, W1, W3, W2, act, M, K, N1, N2, Y, stream);
}
int ffuse_ffn_f32(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                  int64_t N1, int64_t N2, void* Y, void* stream) {
    return run_fused(FFUSE_DT_F32, X, W1, W3, W2, act, M, K, N1, N2, Y, stream);
}
int ffuse_ffn_unfused(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                      int64_t N1, int64_t N2, void* Y, void* stream) {
    return run_unfused(FFUSE_DT_BF16, X, W1, W3, W2, act, M, K, N1, N2, Y, stream);
}
int ffuse_ffn_unfused_f16(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                          int64_t N1, int64_t N2, void* Y, void* stream) {
    return run_unfused(FFUSE_DT_F16, X, W1, W3, W2, act, M, K, N1, N2, Y, stream);
}
int ffuse_ffn_unfused_f32(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                          int64_t N1, int64_t N2, void* Y, void* stream) {
    return run_unfused(FFUSE_DT_F32, X, W1, W3, W2, act, M, K, N1, N2, Y, stream);
}

int ffuse_ffn_ws(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                 int64_t N1, int64_t N2, void* Y, void* workspace, size_t workspace_bytes, void* stream) {
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    int rc = validate(X, W1, W3, W2, act, M, K, N1, N2, Y, dtype == FFUSE_DT_F32 ? 4 : 2);
    if (rc != FFUSE_OK) return rc;
    if ((rc = check_ws_arg(workspace, workspace_bytes)) != FFUSE_OK) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    Workspace none;
    return run_fused_locked(dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, workspace ? workspace_record(workspace, workspace_bytes) : none, stream);
}
int ffuse_ffn_unfused_ws(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                         int64_t N1, int64_t N2, void* Y, void* workspace, size_t workspace_bytes, void* stream) {
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    int rc = validate(X, W1, W3, W2, act, M, K, N1, N2, Y, dtype == FFUSE_DT_F32 ? 4 : 2);
    if (rc != FFUSE_OK) return rc;
    if ((rc = check_ws_arg(workspace, workspace_bytes)) != FFUSE_OK) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    Workspace none;
    return run_unfused_locked(dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, workspace ? workspace_record(workspace, workspace_bytes) : none, stream);
}

}  // extern "C"

// ---- the entry point that allocates nothing ---------------------------------------------------------
// Its workspace is this array: device memory that exists from the moment the library is loaded on a
// device until the process ends (every device the library runs on holds its own copy, at its own
// address).  In host code the name `scratch` is a stand-in, not a device address: the address is asked
// for once per device and only that pointer is ever used.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
Workspace static_ws[kMaxDevices];   // per device: address of its copy of `scratch`, and what the library left there

// the record of the current device's scratch array (address resolved on first use); the caller holds the lock
int static_workspace(Workspace** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FFUSE_ERR_LAUNCH;
    Workspace& w = static_ws[dev];
    if (!w.ptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return FFUSE_ERR_LAUNCH;
        w = Workspace{ptr, kStaticScratchBytes, 0, nullptr, 0, false};   // (nothing assumed about its contents)
    }
    *out = &w;
    return FFUSE_OK;
}
}  // namespace

extern "C" {

int ffuse_ffn_static(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
                     int64_t N1, int64_t N2, void* Y, void* stream) {
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    int rc = validate(X, W1, W3, W2, act, M, K, N1, N2, Y, dtype == FFUSE_DT_F32 ? 4 : 2);
    if (rc != FFUSE_OK) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    if ((rc = check_arch()) != FFUSE_OK) return rc;
    Workspace* w = nullptr;
    if ((rc = static_workspace(&w)) != FFUSE_OK) return rc;
    // the best-ranked plan whose workspace fits the array (looked up after the first call for a shape)
    const int gated = W3 != nullptr;
    const auto key = table_key(dtype + 128, gated, K, N1, N2, -M);
    auto it = g.table.find(key);
    if (it == g.table.end()) {
        std::vector<ffuse::RankedPlan> ranked;
        ffuse::rank_plans(dtype, act, gated, M, K, N1, N2, &ranked);
        const ffuse::RankedPlan* fit = nullptr;
        for (const auto& r : ranked)
            if (ffuse::plan_workspace_bytes(r.plan, dtype, gated, M, K, N1, N2) <= kStaticScratchBytes) { fit = &r; break; }
        if (!fit) return FFUSE_ERR_WORKSPACE;     // the problem is too large for the built-in scratch memory
        if (g.table.size() > 4096) g.table.clear();
        it = g.table.insert({key, {fit->plan, 0.0}}).first;
    }
    g.no_alloc_call = true;
    rc = run_plan(it->second.plan, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, *w, stream);
    g.no_alloc_call = false;
    return rc;
}

int ffuse_debug_barrier(int extra_arrivals, unsigned int spin_limit) {
    if (extra_arrivals < 0 || extra_arrivals > 1024 || spin_limit < 1) return FFUSE_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g.mu);
    g.extra_arrivals = extra_arrivals;
    g.spin_limit = spin_limit;
    return FFUSE_OK;
}

size_t ffuse_workspace_bytes(int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, int unfused) {
    (void)K;
    if (M < 1 || N1 < 1 || N2 < 1) return 0;
    const size_t elem = dtype == FFUSE_DT_F32 ? 4 : 2;
    size_t b = unfused ? elem * (size_t)M * (size_t)N1 : (dtype == FFUSE_DT_F32 ? 0 : sizeof(float) * (size_t)M * (size_t)N2);
    if (dtype != FFUSE_DT_F32) {   // (the 16-bit unfused path runs the two-phase family's kernel)
        // room for the exchange family's flags + ring at its largest ring setting
        const size_t ex = ffuse::kExchangeFlagBytes + (size_t)8 * ffuse::kExchangeMaxRing * 256 * (gated ? 128 : 256) * 2;
        if (!unfused && ex > b) b = ex;
        // two-phase family: partial-sum planes (at the most splits the chooser uses for this M) | H | flags
        const int sp = ffuse::two_phase_max_splits(M, N2);
        const size_t planes = sp > 1 ? (((size_t)4 * M * N2 * sp + 255) & ~(size_t)255) : 0;
        // (gated: twice the intermediate, for plans that keep the two branches apart)
        const size_t tp = planes + (gated ? 2 : 1) * (((size_t)2 * M * N1 + 255) & ~(size_t)255) + ffuse::kTwoPhaseFlagBytes;
        if (tp > b) b = tp;
    }
    return (b + 255) & ~(size_t)255;
}

int ffuse_set_workspace(void* dev_ptr, size_t bytes, void* stream) {
    std::lock_guard<std::mutex> lock(g.mu);
    if (!dev_ptr) {
        g.reg = Workspace{};
        g.exch_err = nullptr;
        return FFUSE_OK;
    }
    if (!aligned16(dev_ptr)) return FFUSE_ERR_ALIGN;
    if (bytes % 16) return FFUSE_ERR_SHAPE;
    if (ffuse::launch_zero(dev_ptr, bytes, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return FFUSE_ERR_LAUNCH;
    forget_overlapping(dev_ptr, bytes);
    g.reg = Workspace{dev_ptr, bytes, bytes, nullptr, 0, false};
    g.exch_err = nullptr;
    return FFUSE_OK;
}

int ffuse_choose_plan(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, ffuse_plan_t* out) {
    if (!out) return FFUSE_ERR_NULL;
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32 || act < FFUSE_ACT_IDENTITY || act > FFUSE_ACT_SILU) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8 || (K % 8) || (N1 % 8) || (N2 % 8)) return FFUSE_ERR_SHAPE;
    int objective;
    {
        std::lock_guard<std::mutex> lock(g.mu);
        objective = g.objective;
    }
    ffuse::choose_plan(dtype, act, gated ? 1 : 0, M, K, N1, N2, out, objective);
    return FFUSE_OK;
}

int ffuse_traffic_model(const ffuse_plan_t* plan, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                        ffuse_traffic_t* out) {
    if (!plan || !out) return FFUSE_ERR_NULL;
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8) return FFUSE_ERR_SHAPE;
    if (!ffuse::plan_valid(*plan, dtype, gated ? 1 : 0, M, K, N1, N2)) return FFUSE_ERR_PLAN;
    ffuse::traffic_model(*plan, dtype, gated ? 1 : 0, M, K, N1, N2, out);
    return FFUSE_OK;
}

int ffuse_plan_group_local(const ffuse_plan_t* plan, int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2) {
    if (!plan) return FFUSE_ERR_NULL;
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F16) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8) return FFUSE_ERR_SHAPE;
    ffuse::TwoPhaseGeometry sg;
    if (plan->family != FFUSE_FAMILY_TWOPHASE || !ffuse::plan_valid(*plan, dtype, gated ? 1 : 0, M, K, N1, N2) ||
        !ffuse::two_phase_geometry(*plan, gated ? 1 : 0, M, N1, N2, &sg))
        return FFUSE_ERR_PLAN;
    return ffuse::two_phase_groups_independent(sg, M, N1, N2) ? 1 : 0;
}

int ffuse_loop_schedule_count(int spatial_dims) { return ffuse::loop_schedule_count(spatial_dims); }

int ffuse_cluster_exchange(int cls_n, int cls_k, int cls_l, int* cls_shuffle, int* cls_reduce) {
    if (!cls_shuffle || !cls_reduce) return FFUSE_ERR_NULL;
    return ffuse::cluster_exchange(cls_n, cls_k, cls_l, cls_shuffle, cls_reduce) ? FFUSE_OK : FFUSE_ERR_SHAPE;
}

int ffuse_set_objective(int objective) {
    if (objective != FFUSE_OBJECTIVE_TIME && objective != FFUSE_OBJECTIVE_BYTES) return FFUSE_ERR_ACT;
    std::lock_guard<std::mutex> lock(g.mu);
    g.objective = objective;
    return FFUSE_OK;
}

int ffuse_force_plan(const ffuse_plan_t* plan) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.env_checked = true;  // an explicit call overrides the environment
    if (!plan) { g.forced = false; return FFUSE_OK; }
    g.forced_plan = *plan;
    g.forced = true;
    return FFUSE_OK;
}

int ffuse_last_plan(ffuse_plan_t* out) {
    if (!out) return FFUSE_ERR_NULL;
    std::lock_guard<std::mutex> lock(g.mu);
    *out = g.last_plan;
    return FFUSE_OK;
}

int ffuse_sync_status(void* stream) {
    if (hipStreamSynchronize(reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return FFUSE_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g.mu);
    if (g.log && g.small_stats) {
        std::vector<uint64_t> h(8 * 1024);
        if (hipMemcpy(h.data(), g.small_stats, h.size() * 8, hipMemcpyDeviceToHost) == hipSuccess) {
            // launched one phase at a time, the second launch's record follows the first's
            const uint64_t* h2 = h.data() + (g.small_split ? 4 * 1024 : 0);
            double p1 = 0, b = 0, p2 = 0, m1 = 0, m2 = 0, clk = 0; int n = 0;
            for (int i = 0; i < g.cus && i < 1024; ++i) {
                p1 += h[4 * i]; clk += h[4 * i + 3]; b += h[4 * i + 1]; p2 += h2[4 * i + 2]; ++n;
                m1 = std::max(m1, (double)h[4 * i]); m2 = std::max(m2, (double)h2[4 * i + 2]);
            }
            std::fprintf(stderr, "[ffuse] two-phase%s: phase 1 avg %.1f us (max %.1f) at %.0f MHz, barrier wait avg %.1f us, phase 2 avg %.1f us (max %.1f)\n",
                         g.small_split ? " (one launch per phase)" : "", p1 / n * 0.01, m1 * 0.01, p1 > 0 ? clk / p1 * 100.0 : 0.0,
                         b / n * 0.01, p2 / n * 0.01, m2 * 0.01);
        }
        g.small_stats = nullptr;
    }
    if (g.log && g.rows_stats) {
        std::vector<uint64_t> h(2 * (size_t)g.rows_wgs);
        if (hipMemcpy(h.data(), g.rows_stats, h.size() * 8, hipMemcpyDeviceToHost) == hipSuccess) {
            double wall = 0, core = 0, mx = 0;
            for (int i = 0; i < g.rows_wgs; ++i) { wall += h[2 * i]; core += h[2 * i + 1]; mx = std::max(mx, (double)h[2 * i]); }
            std::fprintf(stderr, "[ffuse] rows: workgroup busy avg %.1f us (max %.1f) at %.0f MHz\n", wall / g.rows_wgs * 0.01, mx * 0.01,
                         wall > 0 ? core / wall * 100.0 : 0.0);
        }
        g.rows_stats = nullptr;
    }
    if (!g.exch_err) return FFUSE_OK;
    uint32_t word = 0;
    if (hipMemcpy(&word, g.exch_err, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess) return FFUSE_ERR_LAUNCH;
    if (g.log && g.exch_stats) {
        std::vector<uint64_t> h(4 * (size_t)g.exch_wgs);
        if (hipMemcpy(h.data(), g.exch_stats, h.size() * 8, hipMemcpyDeviceToHost) == hipSuccess) {
            for (int role = 1; role <= 2; ++role) {
                double tot = 0, wt = 0, mx = 0, mxw = 0, gm = 0, ep = 0; int n = 0;
                for (int i = 0; i < g.exch_wgs; ++i)
                    if ((int)(h[4 * i] & 255u) == role) {
                        tot += h[4 * i + 1]; wt += h[4 * i + 2]; mx = std::max(mx, (double)h[4 * i + 1]); mxw = std::max(mxw, (double)h[4 * i + 2]);
                        gm += (double)(h[4 * i] >> 8); ep += (double)(h[4 * i + 3] >> 32); ++n;
                    }
                if (n) std::fprintf(stderr, "[ffuse] exchange %s: %d wgs, busy+wait avg %.1f us (max %.1f), waiting avg %.1f us (max %.1f), producing: GEMM avg %.1f us, epilogue+publish avg %.1f us\n",
                                    role == 1 ? "producers" : "consumers", n, tot / n * 0.01, mx * 0.01, wt / n * 0.01, mxw * 0.01, gm / n * 0.01, ep / n * 0.01);
            }
        }
    }
    if (word & 2u) return FFUSE_ERR_PLACEMENT;
    return word ? FFUSE_ERR_TIMEOUT : FFUSE_OK;
}

// Convolution chain (Evaluation, table of conv-chain configurations): conv k1 x k1 ->
// activation -> conv 1 x 1 over a channels-last image.  A 1x1 first convolution is the GEMM
// chain on the pixel rows; a 3x3 one runs the two-phase kernel with implicit-im2col loads.
int run_conv_chain(int dtype, const void* X, const void* W1, const void* W2, int act, int64_t B, int64_t H, int64_t W,
                   int64_t IC, int64_t OC1, int64_t OC2, int k1, int k2, void* Y, void* stream) {
    Workspace& ws = g.reg;
    if (B < 1 || H < 1 || W < 1 || IC < 8 || H > 32768 || W > 32768) return FFUSE_ERR_SHAPE;
    if (k2 != 1 || (k1 != 1 && k1 != 3)) return FFUSE_ERR_SHAPE;
    const int64_t M = B * H * W, K = (int64_t)k1 * k1 * IC;
    if (k1 == 1) return run_fused(dtype, X, W1, nullptr, W2, act, M, K, OC1, OC2, Y, stream);
    if (IC % 64) return FFUSE_ERR_SHAPE;   // one tap per K step of 64
    int rc = validate(X, W1, nullptr, W2, act, M, K, OC1, OC2, Y, 2);
    if (rc != FFUSE_OK) return rc;
    std::lock_guard<std::mutex> lock(g.mu);
    rc = check_arch();
    if (rc != FFUSE_OK) return rc;
    read_env_plan();
    ffuse_plan_t plan{};
    bool found = false;
    if (g.forced && g.forced_plan.family == FFUSE_FAMILY_TWOPHASE) {
        plan = g.forced_plan;
        if (plan.bm == 0) plan.bm = M <= 32 ? 32 : (M <= 64 ? 64 : 128);
        plan.bk = 64;                  // the 3x3 loader exists for the register-staged loop only
        if (plan.bh != 64 && plan.bh != 32) plan.bh = 128;
        found = plan.bm <= 128 && ffuse::plan_valid(plan, dtype, 0, M, K, OC1, OC2);
        if (!found) return FFUSE_ERR_PLAN;
    } else {
        // the model's best plan among those the 3x3 loader's kernels implement: ranked once per shape, then
        // looked up (its own key space in the plan table: dtype + 32)
        const auto key = table_key(dtype + 32, 0, K, OC1, OC2, -M);
        auto it = g.table.find(key);
        if (it != g.table.end() && ffuse::plan_workspace_bytes(it->second.plan, dtype, 0, M, K, OC1, OC2) <= ws.bytes) {
            plan = it->second.plan;
            found = true;
        } else {
            std::vector<ffuse::RankedPlan> ranked;
            ffuse::rank_plans(dtype, act, 0, M, K, OC1, OC2, &ranked);
            for (const auto& r : ranked)
                if (r.plan.family == FFUSE_FAMILY_TWOPHASE && r.plan.bm <= 128 && r.plan.bk != 32 &&
                    ffuse::plan_workspace_bytes(r.plan, dtype, 0, M, K, OC1, OC2) <= ws.bytes) {
                    plan = r.plan;
                    found = true;
                    break;
                }
            if (found) {
                if (g.table.size() > 4096) g.table.clear();
                g.table[key] = {plan, 0.0};
            }
        }
    }
    if (!found) return FFUSE_ERR_WORKSPACE;
    return run_plan(plan, dtype, X, W1, nullptr, W2, act, M, K, OC1, OC2, Y, ws, stream, false, ConvGeom{(int)IC, (int)H, (int)W});
}

// Sec. 4.3, Algorithm 2, second half: time the analytically best `top_k` plans on the device
// and keep the fastest in the plan table for M's bin.
int ffuse_tune(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M, int64_t K,
               int64_t N1, int64_t N2, void* Y, int top_k, int reps, void* stream, ffuse_plan_t* best_plan, double* best_ms) {
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    const int elem = dtype == FFUSE_DT_F32 ? 4 : 2;
    int rc = validate(X, W1, W3, W2, act, M, K, N1, N2, Y, elem);
    if (rc != FFUSE_OK) return rc;
    if (top_k < 1 || reps < 1 || top_k > 64 || reps > 1000) return FFUSE_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g.mu);
    rc = check_arch();
    if (rc != FFUSE_OK) return rc;
    const int gated = W3 != nullptr;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    std::vector<ffuse::RankedPlan> ranked;
    ffuse::rank_plans(dtype, act, gated, M, K, N1, N2, &ranked);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FFUSE_ERR_LAUNCH;
    const bool was_profiling = g.profiling;
    g.profiling = false;
    double best = 1e30;
    ffuse_plan_t bestp{};
    int last_rc = FFUSE_ERR_WORKSPACE;
    // the candidates: the model's first top_k plans that are valid and fit the workspace, each run
    // once, untimed and checked
    struct Cand { ffuse_plan_t plan; double t_pred, ms; };
    std::vector<Cand> cands;
    bool stop = false;
    for (const auto& cand : ranked) {
        if ((int)cands.size() >= top_k) break;
        const ffuse_plan_t& p = cand.plan;
        if (!ffuse::plan_valid(p, dtype, gated, M, K, N1, N2)) continue;
        if (ffuse::plan_workspace_bytes(p, dtype, gated, M, K, N1, N2) > g.reg.bytes) continue;
        last_rc = run_plan(p, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, g.reg, stream);
        if (last_rc != FFUSE_OK) continue;
        if (hipStreamSynchronize(st) != hipSuccess) { last_rc = FFUSE_ERR_LAUNCH; stop = true; break; }
        if (g.exch_err) {
            uint32_t word = 0;
            if (hipMemcpy(&word, g.exch_err, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess) { last_rc = FFUSE_ERR_LAUNCH; stop = true; break; }
            if (word) { last_rc = (word & 2u) ? FFUSE_ERR_PLACEMENT : FFUSE_ERR_TIMEOUT; stop = true; break; }   // device state is suspect: stop
        }
        cands.push_back({p, cand.t_pred, 1e30});
    }
    if (!stop && !cands.empty()) {
        // bring clocks and caches to their steady state before anything is timed, or the first
        // candidate is measured on a different chip than the last
        for (int r = 0; r < 2 * reps && last_rc == FFUSE_OK; ++r)
            last_rc = run_plan(cands[0].plan, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, g.reg, stream);
        // two timed passes, the second in reverse order (drift of the clocks cancels); a candidate's
        // time is the better of its two
        for (int pass = 0; pass < 2 && !stop; ++pass)
            for (size_t n = 0; n < cands.size(); ++n) {
                Cand& c = cands[pass == 0 ? n : cands.size() - 1 - n];
                last_rc = run_plan(c.plan, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, g.reg, stream);   // (its own warm-up: LDS size, L2 contents)
                (void)hipEventRecord(e0, st);
                for (int r = 0; r < reps && last_rc == FFUSE_OK; ++r) last_rc = run_plan(c.plan, dtype, X, W1, W3, W2, act, M, K, N1, N2, Y, g.reg, stream);
                (void)hipEventRecord(e1, st);
                if (hipEventSynchronize(e1) != hipSuccess) { last_rc = FFUSE_ERR_LAUNCH; stop = true; break; }
                if (last_rc != FFUSE_OK) continue;
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, e0, e1);
                const double per = (double)ms / reps;
                if (per < c.ms) c.ms = per;
            }
        // the model's order breaks near-ties: a later candidate has to win by more than 1 %
        for (const Cand& c : cands) {
            if (g.log) std::fprintf(stderr, "[ffuse] tune: family %d bm %d bh %d splits %d raster %d producers %d: model %.1f us, measured %.1f us\n",
                                    c.plan.family, c.plan.bm, c.plan.bh, c.plan.splits, c.plan.raster, c.plan.producers, c.t_pred * 1e6, c.ms * 1e3);
            if (c.ms < 1e30 && c.ms < best * 0.99) { best = c.ms; bestp = c.plan; }
        }
        // ... and a near-tie in time goes to the schedule that keeps far more of the traffic on the chip: a candidate
        // measured within 8 % of the fastest in these short runs (the rows family reaches its steady clock more
        // slowly than the others: at steady state the gap is 1-2 %) whose modelled bytes between the L2s and the fabric are at most half
        // of the fastest plan's takes its place (the rows family on 32768 x 1024 x 8192 x 1024: equal time within
        // the noise of the measurement, 0.3 of the bytes)
        if (best < 1e30) {
            ffuse_traffic_t tb;
            ffuse::traffic_model(bestp, dtype, gated, M, K, N1, N2, &tb);
            const double fastest = best;
            for (const Cand& c : cands) {
                if (c.ms >= 1e30 || c.ms > fastest * 1.08) continue;
                ffuse_traffic_t tc;
                ffuse::traffic_model(c.plan, dtype, gated, M, K, N1, N2, &tc);
                if (tc.feasible && tc.fabric_bytes <= 0.5 * tb.fabric_bytes) { best = c.ms; bestp = c.plan; tb = tc; }
            }
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    g.profiling = was_profiling;
    if (best >= 1e30) return last_rc != FFUSE_OK ? last_rc : FFUSE_ERR_PLAN;
    g.table[table_key(dtype, gated, K, N1, N2, ffuse::m_bin(M))] = {bestp, best};
    if (best_plan) *best_plan = bestp;
    if (best_ms) *best_ms = best;
    return FFUSE_OK;
}

int ffuse_conv_chain(const void* X, const void* W1, const void* W2, int act, int64_t B, int64_t H, int64_t W, int64_t IC,
                     int64_t OC1, int64_t OC2, int k1, int k2, void* Y, void* stream) {
    if (!X || !W1 || !W2 || !Y) return FFUSE_ERR_NULL;
    return run_conv_chain(FFUSE_DT_BF16, X, W1, W2, act, B, H, W, IC, OC1, OC2, k1, k2, Y, stream);
}
int ffuse_conv_chain_f16(const void* X, const void* W1, const void* W2, int act, int64_t B, int64_t H, int64_t W, int64_t IC,
                         int64_t OC1, int64_t OC2, int k1, int k2, void* Y, void* stream) {
    if (!X || !W1 || !W2 || !Y) return FFUSE_ERR_NULL;
    return run_conv_chain(FFUSE_DT_F16, X, W1, W2, act, B, H, W, IC, OC1, OC2, k1, k2, Y, stream);
}

int ffuse_rank_plans(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, ffuse_plan_t* plans,
                     double* t_pred_s, int capacity) {
    if (!plans || capacity < 1) return FFUSE_ERR_NULL;
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8) return FFUSE_ERR_SHAPE;
    std::vector<ffuse::RankedPlan> ranked;
    ffuse::rank_plans(dtype, act, gated ? 1 : 0, M, K, N1, N2, &ranked);
    int n = 0;
    for (const auto& r : ranked) {
        if (n >= capacity) break;
        plans[n] = r.plan;
        if (t_pred_s) t_pred_s[n] = r.t_pred;
        ++n;
    }
    return n;
}

int ffuse_plan_table_set(int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, const ffuse_plan_t* plan, double ms) {
    if (!plan) return FFUSE_ERR_NULL;
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8) return FFUSE_ERR_SHAPE;
    if (!ffuse::plan_valid(*plan, dtype, gated ? 1 : 0, M, K, N1, N2)) return FFUSE_ERR_PLAN;
    std::lock_guard<std::mutex> lock(g.mu);
    g.table[table_key(dtype, gated ? 1 : 0, K, N1, N2, ffuse::m_bin(M))] = {*plan, ms > 0.0 ? ms : 1e-9};
    return FFUSE_OK;
}

// Text format, one tuned entry per line:
//   ffuse-plan 1 <dtype> <gated> <K> <N1> <N2> <bin> <ms> <family> <bm> <bh> <bn2> <bk> <splits> <h_level> <raster> <producers> <ring> <coherent> [<gate_split>]
int ffuse_plan_table_save(const char* path) {
    if (!path) return FFUSE_ERR_NULL;
    std::lock_guard<std::mutex> lock(g.mu);
    std::FILE* f = std::fopen(path, "w");
    if (!f) return FFUSE_ERR_LAUNCH;
    int n = 0;
    for (const auto& kv : g.table) {
        if (kv.first[5] < 0) continue;   // modelled entries are recomputed, not stored
        const ffuse_plan_t& p = kv.second.plan;
        std::fprintf(f, "ffuse-plan 1 %lld %lld %lld %lld %lld %lld %.9g %d %d %d %d %d %d %d %d %d %d %d %d\n", (long long)kv.first[0],
                     (long long)kv.first[1], (long long)kv.first[2], (long long)kv.first[3], (long long)kv.first[4],
                     (long long)kv.first[5], kv.second.ms, p.family, p.bm, p.bh, p.bn2, p.bk, p.splits, p.h_level, p.raster,
                     p.producers, p.ring, p.coherent, p.gate_split);
        ++n;
    }
    std::fclose(f);
    return n;
}

int ffuse_plan_table_load(const char* path) {
    if (!path) return FFUSE_ERR_NULL;
    std::FILE* f = std::fopen(path, "r");
    if (!f) return FFUSE_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g.mu);
    int n = 0;
    char line[512];
    while (std::fgets(line, sizeof(line), f)) {
        long long k[6];
        double ms;
        int v[12] = {0}, ver;
        if (std::sscanf(line, "ffuse-plan %d %lld %lld %lld %lld %lld %lld %lf %d %d %d %d %d %d %d %d %d %d %d %d", &ver, &k[0], &k[1], &k[2],
                        &k[3], &k[4], &k[5], &ms, &v[0], &v[1], &v[2], &v[3], &v[4], &v[5], &v[6], &v[7], &v[8], &v[9], &v[10], &v[11]) < 19)
            continue;
        if (ver != 1 || k[0] < FFUSE_DT_BF16 || k[0] > FFUSE_DT_F32 || k[5] < 0 || k[5] > 62) continue;
        ffuse_plan_t p{};
        p.family = v[0]; p.bm = v[1]; p.bh = v[2]; p.bn2 = v[3]; p.bk = v[4]; p.splits = v[5]; p.h_level = v[6]; p.raster = v[7];
        p.producers = v[8]; p.ring = v[9]; p.coherent = v[10]; p.gate_split = v[11];
        if (p.family <= FFUSE_FAMILY_AUTO || p.family > FFUSE_FAMILY_ROWS) continue;
        // validity for a concrete M is checked again at lookup time
        g.table[table_key((int)k[0], (int)k[1], k[2], k[3], k[4], k[5])] = {p, ms > 0.0 ? ms : 1e-9};
        ++n;
    }
    std::fclose(f);
    return n;
}

int ffuse_plan_table_clear(void) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.table.clear();
    return FFUSE_OK;
}

int ffuse_plan_lookup(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2, ffuse_plan_t* out, double* tuned_ms) {
    if (!out) return FFUSE_ERR_NULL;
    if (dtype < FFUSE_DT_BF16 || dtype > FFUSE_DT_F32) return FFUSE_ERR_ACT;
    if (M < 1 || K < 8 || N1 < 8 || N2 < 8) return FFUSE_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g.mu);
    *out = lookup_plan(dtype, act, gated ? 1 : 0, M, K, N1, N2, g.reg.ptr ? g.reg.bytes : 0);
    if (tuned_ms) {
        auto it = g.table.find(table_key(dtype, gated ? 1 : 0, K, N1, N2, ffuse::m_bin(M)));
        *tuned_ms = (it != g.table.end() && std::memcmp(&it->second.plan, out, sizeof(*out)) == 0) ? it->second.ms : 0.0;
    }
    return FFUSE_OK;
}

int ffuse_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.profiling = on != 0;
    return FFUSE_OK;
}

int ffuse_profile_read(double* kernel_ms_total, int64_t* launches) {
    if (!kernel_ms_total || !launches) return FFUSE_ERR_NULL;
    std::lock_guard<std::mutex> lock(g.mu);
    double total = 0.0;
    int64_t n = 0;
    for (auto& ev : g.events) {
        float ms = 0.0f;
        if (hipEventSynchronize(ev.second) == hipSuccess && hipEventElapsedTime(&ms, ev.first, ev.second) == hipSuccess) {
            total += ms;
            ++n;
        }
        (void)hipEventDestroy(ev.first);
        (void)hipEventDestroy(ev.second);
    }
    g.events.clear();
    *kernel_ms_total = total;
    *launches = n;
    return FFUSE_OK;
}

const char* ffuse_status_string(int status) {
    switch (status) {
        case FFUSE_OK: return "ok";
        case FFUSE_ERR_NULL: return "a required pointer is NULL";
        case FFUSE_ERR_SHAPE: return "shape violates the rules (M>=1; K,N1,N2 multiples of 8; tensors < 2 GiB)";
        case FFUSE_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case FFUSE_ERR_ACT: return "unknown activation or dtype code";
        case FFUSE_ERR_WORKSPACE: return "workspace missing or too small";
        case FFUSE_ERR_LAUNCH: return "HIP runtime error";
        case FFUSE_ERR_ARCH: return "device is not gfx950";
        case FFUSE_ERR_PLAN: return "plan not valid for this problem";
        case FFUSE_ERR_TIMEOUT: return "a cooperative kernel timed out waiting for a peer workgroup";
        case FFUSE_ERR_PLACEMENT: return "exchange group not placed on one XCD (force coherent = 1)";
        default: return "unknown status";
    }
}

int ffuse_version(void) { return 1; }

}  // extern "C"
