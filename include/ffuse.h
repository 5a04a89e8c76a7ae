/*
 * ffuse.h -- C ABI of libffuse.so: fused feed-forward chains for AMD MI355X (gfx950).
 *
 * The library evaluates the two-GEMM operator chain that the FlashFuser paper fuses
 * (Background, Fig. "three common GEMM chains" (b) standard FFN and (c) gated FFN;
 * Sec. 4.1, description of the tile graph):
 *
 *     standard:  Y = act(X * W1) * W2
 *     gated   :  Y = (act(X * W1) .* (X * W3)) * W2          (SwiGLU when act = SiLU)
 *
 * in ONE kernel that exchanges the M x N1 intermediate through the on-chip cache levels
 * (or, in the reduce family, never lets it leave the register file), and, for comparison, as
 * a plain unfused two-GEMM path of two launches.
 *
 * Conventions (all entry points)
 *   - Every tensor is row-major and contiguous:  X[M][K], W1[K][N1], W3[K][N1], W2[N1][N2],
 *     Y[M][N2].  Paper notation (m, k, n, l) = ours (M, K, N1, N2).
 *   - X, W1, W3, W2, Y and the workspace are DEVICE pointers, 16-byte aligned.  The library
 *     never allocates, frees or retains device memory; the caller owns all of it.
 *   - Inputs are read-only; Y is fully overwritten.  Calls are asynchronous and ordered on
 *     `stream` (a hipStream_t passed as void*, NULL = the null stream).
 *   - Gated  <=>  W3 != NULL; `act` is then applied to the X*W1 branch (Sec. 4.1: one branch
 *     passes through the activation, the other multiplies it element-wise).
 *   - The activation sees complete sums over K only (Sec. 4.3, pruning Rule 3), accumulation
 *     is fp32, the intermediate is rounded to the operand type (round-to-nearest-even) before
 *     the second product, and Y is rounded once from fp32 to the operand type.
 *   - Shape rules: M >= 1 (any value, row tails are masked); K, N1, N2 >= 8 and multiples
 *     of 8; every tensor smaller than 2 GiB, and the M x N1 intermediate counts as one
 *     ((M + 256) N1 elements of the operand type: rows are independent, a taller problem is two
 *     calls).  Anything else returns FFUSE_ERR_SHAPE.
 *   - Errors are returned as negative status codes; nothing is written on a validation error.
 *   - The fused and unfused paths need a caller-owned workspace of ffuse_workspace_bytes: either
 *     ONE registered with ffuse_set_workspace and used by every call that does not name another,
 *     or one passed per call (ffuse_ffn_ws, ffuse_ffn_unfused_ws).  A call leaves its workspace
 *     ready for the next call on the same stream.  Calls that overlap in time (different
 *     streams) need different workspaces: give each stream its own through the _ws calls.
 *     Between calls the library remembers, per workspace address, what it left there (which
 *     part is zero, where clean barrier flags lie); a caller that writes into a workspace
 *     itself must hand it over again (ffuse_set_workspace, or any other size in a _ws call).
 *   - Graph capture: a call recorded while `stream` is capturing records its own clearing of
 *     the flags or sums it needs, whatever the library believes about the workspace, and from
 *     then on every call on that workspace clears what it needs too (until the workspace is
 *     registered or named anew), so the graph may be replayed between any other calls on the
 *     same workspace (not concurrently with them).
 */
#ifndef FFUSE_H
#define FFUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FFUSE_ACT_IDENTITY = 0,  /* x                                                         */
    FFUSE_ACT_RELU = 1,      /* max(x, 0)                                                 */
    FFUSE_ACT_GELU_TANH = 2, /* 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) ))         */
    FFUSE_ACT_SILU = 3       /* x / (1 + exp(-x))   (the activation Sec. 4.1 names)       */
} ffuse_act_t;

typedef enum { FFUSE_DT_BF16 = 0, FFUSE_DT_F16 = 1, FFUSE_DT_F32 = 2 } ffuse_dtype_t;

typedef enum {
    FFUSE_OK = 0,
    FFUSE_ERR_NULL = -1,      /* a required pointer is NULL                                */
    FFUSE_ERR_SHAPE = -2,     /* a dimension violates the shape rules above                */
    FFUSE_ERR_ALIGN = -3,     /* a pointer is not 16-byte aligned                          */
    FFUSE_ERR_ACT = -4,       /* unknown activation / dtype code                           */
    FFUSE_ERR_WORKSPACE = -5, /* no workspace set, or it is too small for this call        */
    FFUSE_ERR_LAUNCH = -6,    /* the HIP runtime refused a launch or a copy                */
    FFUSE_ERR_ARCH = -7,      /* the current device is not gfx950                          */
    FFUSE_ERR_PLAN = -8,      /* a forced plan is not valid for this problem               */
    FFUSE_ERR_TIMEOUT = -9,   /* a cooperative kernel gave up waiting for a peer workgroup  */
    FFUSE_ERR_PLACEMENT = -10 /* an XCD received more workgroups of an exchange launch than
                                 its share (dispatch was not round robin over the XCDs)     */
} ffuse_status_t;

/*
 * Execution plan = loop schedule + tile sizes + placement of the intermediate (Sec. 4.2:
 * LoopSchedule, Tile Selection, Resource Mapping), reduced to the schedules that survive
 * the pruning rules of Sec. 4.3 on a device without distributed shared memory.
 */
typedef enum {
    FFUSE_FAMILY_AUTO = 0,
    FFUSE_FAMILY_REDUCE = 1,  /* hidden dimension split across workgroups; each keeps its
                                 activated slice on chip and the partial second products are
                                 summed with fp32 atomics (Sec. 4.1 "reduce" strategy)      */
    FFUSE_FAMILY_EXCHANGE = 2,/* cooperating workgroups publish activated tiles to an
                                 L2-resident buffer and consume each other's tiles
                                 (Sec. 4.1 "shuffle" strategy, exchange through L2)         */
    FFUSE_FAMILY_UNFUSED = 3, /* traffic model only: two GEMM launches of 256-row tiles       */
    FFUSE_FAMILY_SCALAR = 4,  /* fp32 debug kernels (plain FMA, no matrix cores)            */
    FFUSE_FAMILY_ROWS = 6,    /* row-stationary: a workgroup owns bm = 64 rows and ALL N2 output columns
                                 (N2 <= 1024), keeps its rows of X in registers (K <= 1024), the output
                                 block in accumulators and one activated chunk of bh = 64 hidden columns in
                                 LDS while it walks the hidden dimension; nothing is exchanged between
                                 workgroups, no workspace, Y is the only thing stored (Sec. 4.2: the
                                 MLNK-style loop order with the intermediate mapped to registers -> shared
                                 memory).  Not gated.  For large M.                                   */
    FFUSE_FAMILY_TWOPHASE = 5 /* any M: one persistent kernel; every CU computes tiles of the
                                 intermediate into an L2 / Infinity-Cache resident buffer, one
                                 device-wide barrier, then every CU multiplies a row block of it
                                 with a block of W2 (Sec. 4.1 "shuffle" with the device as the
                                 cluster).  bm = 32 / 64 / 128 (M <= bm for the first two) or
                                 256; `splits` ranges of the hidden dimension: 1 = the tile is
                                 stored straight to Y, > 1 = per-range fp32 planes summed in a
                                 fixed order by a finalize pass (Sec. 4.1 "reduce")          */
} ffuse_family_t;

typedef struct {
    int32_t family;   /* ffuse_family_t                                                     */
    int32_t bm;       /* rows of X per workgroup                                            */
    int32_t bh;       /* hidden columns (of N1) per workgroup step                          */
    int32_t bn2;      /* output columns (of N2) per inner step of the second product        */
    int32_t bk;       /* K step of the first product                                        */
    int32_t splits;   /* number of partial second products summed per output element        */
    int32_t h_level;  /* where the activated slice lives: 0 registers, 1 LDS, 2 L2 buffer   */
    int32_t raster;   /* row blocks that share one XCD's L2 at a time                       */
    int32_t producers;/* exchange family: producer workgroups per XCD group (0 = default)  */
    int32_t ring;     /* exchange family: ring slots per XCD group (0 = default)           */
    int32_t coherent; /* exchange family: 0 = ring kept coherent through the XCD's shared L2
                         (groups form by the XCD a workgroup runs on; needs an even spread of the
                         launch over the XCDs, checked on the device); 1 = agent-scope
                         release/acquire, valid for any placement, much slower            */
    int32_t gate_split;/* two-phase family, gated chains (Sec. 4.1, gated FFN): 0 = both branches in one
                         workgroup, two accumulator sets, Mul in registers; 1 = the branches are separate
                         work items on different workgroups (full-width tiles each) and a Mul pass
                         through the shared cache joins them before the second product          */
} ffuse_plan_t;

/* Analytical data-movement volumes (Sec. 4.2, Algorithm 1) and per-level costs
 * (Sec. 4.3, Eq. 1-3: cost of a level = volume / bandwidth, objective = the maximum). */
typedef struct {
    double flops;        /* useful flops 2*M*N1*(g*K + N2)                                  */
    double hbm_bytes;    /* predicted HBM traffic                                           */
    double fabric_bytes; /* bytes filled into the per-XCD L2s from Infinity Cache / HBM     */
    double l2_bytes;     /* bytes delivered from L2 to the compute units                    */
    double lds_bytes;    /* bytes read from LDS by the matrix pipelines                     */
    double reduce_bytes; /* fp32 bytes combined across workgroups (atomics)                 */
    double exchange_bytes;/* intermediate bytes written to + read from the L2 buffer        */
    double q_min;        /* compulsory bytes: X + weights + Y once                          */
    double q_unfused;    /* q_min + one write and one read of the intermediate              */
    double t_mfma, t_hbm, t_fabric, t_l2, t_lds, t_reduce; /* seconds per level             */
    double t_pred;       /* max of the above plus fixed launch/sync terms                   */
    double lds_used;     /* bytes of LDS per workgroup                                      */
    double acc_regs;     /* accumulator registers per lane                                  */
    int32_t feasible;    /* capacity constraints (Eq. 3) hold                               */
    int32_t workgroups;
} ffuse_traffic_t;

/* ---- the fused chain.  bf16 operands and output; _f16 / _f32 twins take the same
 *      arguments (fp32 is a debug mode on plain FMA).  Returns a ffuse_status_t. ---------- */
int ffuse_ffn(const void* X, const void* W1, const void* W3 /* NULL = not gated */, const void* W2,
              int act, int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);
int ffuse_ffn_f16(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M,
                  int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);
int ffuse_ffn_f32(const void* X, const void* W1, const void* W3, const void* W2, int act, int64_t M,
                  int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);

/* The same two paths with the workspace named per call (dtype: ffuse_dtype_t).  `workspace` is a
 * device pointer, 16-byte aligned, of `workspace_bytes` bytes (a multiple of 16); NULL / 0 is
 * accepted and runs the plans that need none (FFUSE_ERR_WORKSPACE otherwise).  Nothing about
 * the workspace has to be prepared by the caller: a workspace the library has not seen before
 * (or sees with another size) is treated as dirty, and the call clears what it needs on `stream`.
 * Two streams with two workspaces may overlap in time. */
int ffuse_ffn_ws(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act,
                 int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, void* workspace,
                 size_t workspace_bytes, void* stream);
int ffuse_ffn_unfused_ws(int dtype, const void* X, const void* W1, const void* W3, const void* W2,
                         int act, int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ---- for callers that cannot allocate device memory and have no workspace to hand over (code under
 *      HIP graph capture, tight serving loops, harnesses that forbid allocation): ffuse_ffn_ws with the
 *      workspace built into the library -- 32 MiB of device memory per GPU that the library's code object
 *      brings with it and that stays until the process ends.  The call allocates and frees nothing, on the
 *      host side of the device or on the device.  It runs the best-ranked plan whose workspace fits those
 *      32 MiB (all the m = 128 shapes of the paper's tables, the decode shapes, and every shape the rows
 *      family runs, which needs none) and returns FFUSE_ERR_WORKSPACE when no plan for the problem fits.
 *      All calls on one GPU share that GPU's memory, which keeps what the last call left in it (each call
 *      clears what it needs to start from zero, on `stream`): calls that overlap in time on one GPU
 *      race.  The first call on a device resolves the address of the memory and must not be made
 *      while a stream of that device is capturing; later calls may be captured. ------------------- */
int ffuse_ffn_static(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act,
                     int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);

/* ---- the unfused comparison path (Evaluation, "Performance Analysis": the baseline writes
 *      the intermediate to global memory and reads it back): GEMM + activation/gate into a
 *      workspace-resident H[M][N1] in the operand type, then H * W2, as two kernel launches
 *      (plus the plane sum when the second GEMM splits the hidden dimension).  The 16-bit
 *      types run the two-phase family's kernel one phase per launch in the tile plan the
 *      model ranks best for the shape: same block GEMMs and tiles as the fused call, so a
 *      timing difference is the fusion's.  Forced plans do not apply; ffuse_last_plan is
 *      left unchanged. ---------------------------------------------------------------- */
int ffuse_ffn_unfused(const void* X, const void* W1, const void* W3, const void* W2, int act,
                      int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);
int ffuse_ffn_unfused_f16(const void* X, const void* W1, const void* W3, const void* W2, int act,
                          int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);
int ffuse_ffn_unfused_f32(const void* X, const void* W1, const void* W3, const void* W2, int act,
                          int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, void* stream);

/* ---- convolution chains (Evaluation, table "The configuration of conv chain": IC, H, W,
 *      OC1, OC2, k1, k2): Y = conv_k2(act(conv_k1(X, W1)), W2), both convolutions stride 1
 *      with zero padding k/2 (H x W is preserved), cross-correlation, no bias.  Layouts:
 *      X[B][H][W][IC] and Y[B][H][W][OC2] channels-last, W1[k1][k1][IC][OC1],
 *      W2[k2][k2][OC1][OC2]; bf16 (or fp16 for the _f16 twin), device pointers as above.
 *      Built: k2 = 1 with k1 = 1 (the standard chain on the B*H*W pixel rows, any plan) or
 *      k1 = 3 (two-phase kernel whose first product gathers the 3x3 neighbourhood while
 *      loading; needs IC % 64 == 0).  Other kernel sizes return FFUSE_ERR_SHAPE.  IC, OC1, OC2
 *      multiples of 8.  Workspace: ffuse_workspace_bytes(dtype, 0, B*H*W, k1*k1*IC, OC1, OC2, 0). */
int ffuse_conv_chain(const void* X, const void* W1, const void* W2, int act, int64_t B, int64_t H,
                     int64_t W, int64_t IC, int64_t OC1, int64_t OC2, int k1, int k2, void* Y, void* stream);
int ffuse_conv_chain_f16(const void* X, const void* W1, const void* W2, int act, int64_t B, int64_t H,
                         int64_t W, int64_t IC, int64_t OC1, int64_t OC2, int k1, int k2, void* Y, void* stream);

/* ---- workspace.  ffuse_workspace_bytes: bytes the given problem needs (fused path when
 *      unfused == 0; with unfused != 0 the two-launch path's intermediate, partial-sum planes
 *      and flags).  ffuse_set_workspace: registers a caller-owned device buffer with the
 *      library (it is zero-filled once on `stream`); passing NULL unregisters it. --------- */
size_t ffuse_workspace_bytes(int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                             int unfused);
int ffuse_set_workspace(void* dev_ptr, size_t bytes, void* stream);

/* ---- host-side schedule chooser and traffic model (Sec. 4.2 / 4.3); no device work.
 *      ffuse_choose_plan: the model's choice under the objective in force (ffuse_set_objective). ---- */
int ffuse_choose_plan(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                      ffuse_plan_t* out);
int ffuse_traffic_model(const ffuse_plan_t* plan, int dtype, int gated, int64_t M, int64_t K,
                        int64_t N1, int64_t N2, ffuse_traffic_t* out);
/* Two-phase family, host logic only: 1 when, under *plan, every second-phase work item of each of the
 * kernel's eight workgroup groups reads only tiles of the intermediate written by first-phase items of
 * the same group -- the barrier between the phases then waits for the group's own workgroups only
 * (Sec. 4.1: the synchronisation scope follows the data dependence) -- 0 when not, or a negative status
 * (FFUSE_ERR_NULL, FFUSE_ERR_SHAPE, FFUSE_ERR_PLAN: not a valid two-phase plan for this problem). */
int ffuse_plan_group_local(const ffuse_plan_t* plan, int dtype, int gated, int64_t M, int64_t K,
                           int64_t N1, int64_t N2);
/* What the chooser minimises for later fused calls that are not forced and not tuned (Sec. 4.3, Eq. 1-3 put
 * every level's cost into one objective; this exposes the two ends): FFUSE_OBJECTIVE_TIME (default) -- the
 * predicted time; FFUSE_OBJECTIVE_BYTES -- among the plans predicted within 35 % of the fastest, the one
 * that moves the fewest bytes between the L2s and the rest of the memory system (for a chain that shares
 * the memory system with bandwidth-bound work running beside it). */
typedef enum { FFUSE_OBJECTIVE_TIME = 0, FFUSE_OBJECTIVE_BYTES = 1 } ffuse_objective_t;
int ffuse_set_objective(int objective);
/* Forces every later fused call onto *plan (NULL: back to the chooser).  Also settable with
 * the environment variable FFUSE_FORCE_PLAN="family,bm,bh,bn2,bk,splits,h_level,raster,producers,ring,coherent". */
int ffuse_force_plan(const ffuse_plan_t* plan);
/* Other environment variables, read by the fused and unfused calls:
 *   FFUSE_NT=0|1   two-phase family, row blocks below 256: never / always stream the weights with the
 *                  non-temporal load hint.  Default: only when the weights exceed 512 MB -- far more than
 *                  the 256 MB memory-side cache can keep from one call to the next.  A caller that cycles
 *                  through many layers' weights may want 1 for smaller layers too.
 *   FFUSE_GROUP_BARRIER=0  the two-phase kernel's barrier always waits for every workgroup (default: a group
 *                  of workgroups waits for the groups whose tiles of the intermediate its second-phase
 *                  items read -- for itself alone where ffuse_plan_group_local says 1).
 *   FFUSE_EARLY_FILL=0  256-row tiles of the two-phase kernel start the loads of a workgroup's next first-phase
 *                  item after the epilogue of the present one (default: before it, so that they travel under
 *                  it).  Same bits either way; for A/B timing.
 *   FFUSE_LOG=1    (read once) per-launch diagnostics on stderr from ffuse_sync_status.
 *   FFUSE_COOPERATIVE_LAUNCH=1  launch the persistent kernels with the runtime's cooperative launch. */
/* Plan used by the most recent fused call of this process. */
int ffuse_last_plan(ffuse_plan_t* out);
/* Blocks until `stream` is idle, then reports whether the most recent two-phase or
 * exchange-family launch ran to completion: FFUSE_OK, or FFUSE_ERR_TIMEOUT if a workgroup's
 * bounded wait for a peer expired, or FFUSE_ERR_PLACEMENT if the exchange family's XCD-local
 * protocol found a workgroup on the wrong XCD (the output of that call is then undefined;
 * force coherent = 1).  Other families always report OK. */
int ffuse_sync_status(void* stream);

/* ---- plan table and on-device tuning (Sec. 4.3: the dynamic dimension M is covered by plans
 *      fixed ahead of time per range of M and looked up at run time; Algorithm 2: the
 *      analytical ranking is followed by profiling the top-k candidates on the device).
 *      ffuse_tune runs the `top_k` analytically best plans for this problem on `stream` with
 *      the caller's operands (one checked run each, then two passes of `reps` timed runs each,
 *      the second pass in reverse order, a plan's time being the better of its two; Y is
 *      overwritten with a valid result every time), records the fastest for M's bin (M <= 16,
 *      then one bin per power of two) and returns it; near-ties go to the analytical order: a
 *      plan ranked later has to be more than 1 % faster to win -- except that a plan measured within
 *      8 % of the fastest takes its place when the model gives it at most half the bytes between the
 *      L2s and the rest of the memory system (equal time, far less traffic).  Later fused calls with the same dtype, gate, K, N1,
 *      N2 and an M of that bin use it when it is valid for their M and fits their workspace;
 *      otherwise, and for bins never tuned, the model's choice for the exact M is used (and
 *      remembered).  The registered workspace bounds which candidates can run.
 *      ffuse_plan_lookup: the plan a fused call would use now; *tuned_ms (may be NULL) is
 *      the measured milliseconds if that plan came from ffuse_tune, else 0. ---------------- */
int ffuse_tune(int dtype, const void* X, const void* W1, const void* W3, const void* W2, int act,
               int64_t M, int64_t K, int64_t N1, int64_t N2, void* Y, int top_k, int reps, void* stream,
               ffuse_plan_t* best_plan /* may be NULL */, double* best_ms /* may be NULL */);
int ffuse_plan_lookup(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                      ffuse_plan_t* out, double* tuned_ms);
int ffuse_plan_table_clear(void);
/* The offline side of the table: enter a plan for M's bin by hand (ms: its measured time, any
 * positive number), write the measured entries to a text file, read them back (entries are
 * checked against the concrete M when they are used).  save / load return the number of
 * entries written / read, or a negative status (FFUSE_ERR_LAUNCH: the file cannot be opened). */
int ffuse_plan_table_set(int dtype, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                         const ffuse_plan_t* plan, double ms);
int ffuse_plan_table_save(const char* path);
int ffuse_plan_table_load(const char* path);
/* The model's ranking itself (host only): writes up to `capacity` plans in order of increasing
 * predicted time (seconds in t_pred_s, which may be NULL) and returns how many, or a negative
 * status. */
int ffuse_rank_plans(int dtype, int act, int gated, int64_t M, int64_t K, int64_t N1, int64_t N2,
                     ffuse_plan_t* plans, double* t_pred_s, int capacity);

/* ---- the paper's bookkeeping of its search space, restated (host arithmetic only).
 *      ffuse_loop_schedule_count: Sec. 4.2 LoopSchedule / Sec. 4.3 table of spatial and temporal partitions --
 *      the number of schedules of the four loop dimensions (m, n, k, l) with `spatial_dims` of them spatial and
 *      the rest ordered temporally; 0 asks for the total over 1..4 spatial dimensions.
 *      ffuse_cluster_exchange: Sec. 4.1 -- for a cluster that splits n, k and l over cls_n, cls_k, cls_l blocks,
 *      the number of blocks in a shuffle group (cls_l / cls_k) and the number of shuffle groups whose partial
 *      outputs are reduced (cls_n cls_k / cls_l); FFUSE_ERR_SHAPE when the sizes do not divide.  In these terms
 *      the two-phase family is a shuffle over the whole device followed by a reduce over `splits` groups, the
 *      reduce family has cls_shuffle = 1, and the rows family splits k over its four waves (an Add exchange in
 *      LDS) with nothing left to shuffle or reduce between workgroups. ------------------------------------ */
int ffuse_loop_schedule_count(int spatial_dims);
int ffuse_cluster_exchange(int cls_n, int cls_k, int cls_l, int* cls_shuffle, int* cls_reduce);

/* ---- test hook for the failure path of the two-phase family's barrier: later launches wait for
 *      `extra_arrivals` workgroups more than exist (0 = normal) and give up after `spin_limit`
 *      polls (default 2^24).  With extra_arrivals > 0 and a small limit every workgroup's bounded
 *      wait expires, every workgroup leaves normally without running the second phase, and
 *      ffuse_sync_status reports FFUSE_ERR_TIMEOUT; the next normal launch is unaffected. ------ */
int ffuse_debug_barrier(int extra_arrivals, unsigned int spin_limit);

/* ---- measurement aid: when enabled, the library brackets the dominant kernel of every
 *      fused / unfused call with HIP events on the call's stream.  ffuse_profile_read
 *      synchronises those events and returns the summed milliseconds and launch count
 *      since the last read. ---------------------------------------------------------------- */
int ffuse_profile_enable(int on);
int ffuse_profile_read(double* kernel_ms_total, int64_t* launches);

const char* ffuse_status_string(int status);
/* ---- calibration probes (Sec. 4.4: the cost model prices every level with a bandwidth; these measure
 *      the two ends on the device at hand).  FFUSE_CAL_MFMA: every SIMD of the device issues `iters`
 *      rounds of four independent 32x32x16 products of `dtype` (bf16 or fp16) on pseudo-random operands and
 *      nothing else -- the matrix rate no kernel can exceed at the clock the power limit allows; *result is
 *      flop/s (buf and bytes are ignored).  FFUSE_CAL_MFMA_IDLE: the same loop on all-zero operands, which
 *      toggle nothing and draw the least power -- the rate the issue logic alone allows; the distance between the
 *      two is the power limit's doing.  FFUSE_CAL_READ: `buf` (device, 16-byte aligned, `bytes` a
 *      multiple of 16) is streamed through the device once as a warm-up and `iters` more times, timed;
 *      *result is bytes/s.  `scratch16k` is 16 KiB of device memory the probes may write (they do not in
 *      practice); `result` is a host pointer.  The call times its own launches with events on `stream` and
 *      waits for them.  Status as elsewhere (FFUSE_ERR_ACT: unknown probe or dtype). --------------------- */
enum { FFUSE_CAL_MFMA = 0, FFUSE_CAL_READ = 1, FFUSE_CAL_MFMA_IDLE = 2 };
int ffuse_calibrate(int what, int dtype, const void* buf, int64_t bytes, int64_t iters, void* scratch16k,
                    double* result, void* stream);

int ffuse_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FFUSE_H */
