// Argument blocks and launcher prototypes shared by the kernel translation units and the
// C-ABI layer.  Host and device side; no torch types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ffuse {

struct FusedArgs {
    const void* X;
    const void* W1;
    const void* W3;  // nullptr: not gated
    const void* W2;
    float* Ysum;     // fp32 sums [M][N2], zero on entry
    int64_t M;
    int K, N1, N2;
    int act;
    int raster;      // row blocks per XCD patch
};

struct GemmArgs {
    const void* A;   // [M][K]
    const void* B;   // [K][N]
    const void* B3;  // nullptr, or [K][N] second weight of the gated epilogue
    void* C;         // [M][N]
    int64_t M;
    int K, N;
    int act;
};

struct ExchangeArgs {
    const void* X;
    const void* W1;
    const void* W3;  // nullptr: not gated
    const void* W2;
    void* Y;
    char* ring;       // 8 * R slots of 256 x BHP elements (BHP = 256, or 128 when gated)
    uint32_t* flags;  // per group: ready[R], done[R]; then one error word.  Zero on entry.
    int64_t M;
    int K, N1, N2;
    int act;
    int P;            // producers per group
    int NCT;          // 256-wide output column tiles = consumers per panel
    int PG;           // panels in flight per group
    int R;            // ring slots per group
    int NH;           // hidden tiles per panel
    int coherent;     // 0: XCD-local ring protocol; 1: agent-scope release/acquire
    uint64_t* stats;  // nullptr, or 4 words per workgroup: role, total ticks, waiting ticks, items
};

// two-phase family's flag words (kTwoPhaseFlagBytes in all): 1 = workgroups that have left, 2 = error word of
// the launch in flight (cleared by the last workgroup to leave), 3 = error word of the most recent finished
// launch (what the host reads); kTwoPhaseGroupWord * (1 + g) = arrivals at the barrier of group g (a cache
// line apart)
static constexpr int kTwoPhaseGroupWord = 16;

struct TwoPhaseArgs {
    const void* X;
    const void* W1;
    const void* W3;   // nullptr: not gated
    const void* W2;
    void* H;          // [M][N1] intermediate in the operand type (L2 / Infinity Cache resident)
    void* Y;          // [M][N2] output, written by the kernel itself when splits == 1
    float* part;      // splits > 1: fp32 partial sums [splits][M][N2], fully overwritten
    uint32_t* flags;  // [1] exits, [2] error (both zero on entry and on exit), [3] verdict of the last finished launch
    int64_t M;
    int K, N1, N2;
    int act;
    int splits;       // ranges of the hidden dimension summed per output element (>= 1)
    int ksplit;       // hidden columns per range (multiple of 64)
    int raster;       // row blocks per XCD patch (>= 1)
    uint64_t* stats;  // nullptr, or 4 words per workgroup: ticks of phase 1, barrier, phase 2
    // 3x3 first product (conv_ic > 0): X is a channels-last image of M pixels (conv_h x conv_w
    // per image) with conv_ic channels, W1 is [3][3][conv_ic][N1], K = 9 * conv_ic
    int conv_ic, conv_h, conv_w;
    int nt;           // != 0: the weights are streamed with the non-temporal hint (row blocks below 256 only)
    uint64_t wait_masks;  // byte g, bit h: between the phases, workgroups of group g (blockIdx % 8) wait for the
                          // arrivals of group h -- the groups whose phase-1 tiles of H group g's phase-2 items read
    int phases;       // 3: both phases with the device-wide barrier between them (the fused chain);
                      // 1 / 2: only the first / second phase (two launches = the unfused comparison path)
    uint32_t spin_limit;   // polls after which a workgroup gives up waiting at the barrier (error word, FFUSE_ERR_TIMEOUT)
    int extra_arrivals;    // 0; a test may ask the barrier to wait for arrivals that never come, to see the wait expire
    int early_fill;        // != 0: 256-row tiles issue the ring fill of a workgroup's next first-phase item before the
                           // epilogue of the present one (FFUSE_EARLY_FILL=0 switches it off: the fill then follows the epilogue)
    void* U;               // nullptr, or (gated chain with the branches on different workgroups) [M][N1]: X W3 in the
                           // operand type; H then first holds act(X W1) and a Mul pass joins the two in place
};

// rows family (row-stationary): no workspace, no flags
struct RowsArgs {
    const void* X;
    const void* W1;
    const void* W3;   // must be nullptr (the gated chain is not built in this family)
    const void* W2;
    void* Y;
    int64_t M;
    int K, N1, N2;
    int act;
    uint64_t* stats;  // nullptr, or 2 words per workgroup: 100 MHz ticks and core clocks from start to end
};
static constexpr int kRowsRing = 4;    // 4 KB weight slots per wave (measured on 32768 x 1024 x 8192 x 1024: 3 slots 1182 us, 4 1056, 5 1079, 6 1077)
static constexpr int kRowsLdsBytes = 4 * kRowsRing * 4096 + 12 * 4096 + 64 * 128;   // rings | partial tiles | H chunk

// 16-bit paths (dtype 0 = bf16, 1 = fp16)
// nks: 16-k steps of the first product per wave (K <= 64 nks); nt2: 32-column output tiles per wave (N2 <= 128 nt2)
hipError_t launch_fused_rows(int dtype, const RowsArgs& a, int nks, int nt2, int grid, hipStream_t st);
hipError_t launch_fused_two_phase(int dtype, const TwoPhaseArgs& a, int bm, int bh1, int bk, int grid, hipStream_t st);
hipError_t launch_finalize_planes(int dtype, const float* part, void* Y, int64_t count, int planes, hipStream_t st);
hipError_t launch_fused_exchange(int dtype, const ExchangeArgs& a, int wgs_per_group, hipStream_t st);
hipError_t launch_fused_reduce(int dtype, const FusedArgs& a, int bm, int bh, hipStream_t st);
hipError_t launch_finalize(int dtype, float* sums, void* Y, int64_t count, hipStream_t st);

// Launch of a persistent kernel whose workgroups wait for each other: every workgroup must
// be resident at once.  The grid is checked against the occupancy the runtime reports
// (hipErrorCooperativeLaunchTooLarge otherwise) and then launched as an ordinary kernel,
// which costs ~17 us less per call than hipLaunchCooperativeKernel; all in-kernel waits are
// bounded, so foreign work occupying compute units surfaces as FFUSE_ERR_TIMEOUT, not as a
// hang.  FFUSE_COOPERATIVE_LAUNCH=1 selects the runtime's cooperative launch instead.
hipError_t launch_resident(const void* fn, int grid, void** params, hipStream_t st);

// zero fill with a kernel (safe to record into a captured graph, unlike a memset node);
// bytes must be a multiple of 16
hipError_t launch_zero(void* p, size_t bytes, hipStream_t st);

// fp32 debug path
hipError_t launch_fused_f32(const FusedArgs& a, float* Y, hipStream_t st);
hipError_t launch_gemm_act_f32(const GemmArgs& a, hipStream_t st);

}  // namespace ffuse
