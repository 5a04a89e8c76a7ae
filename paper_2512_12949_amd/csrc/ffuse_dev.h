// Device-side building blocks shared by the gfx950 kernels: vector types, MFMA wrappers,
// bounds-checked buffer loads, the 8x8 16-bit register transpose, LDS tile addressing and
// the activations.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ffuse {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_GELU_TANH = 2, ACT_SILU = 3 };

// ---------------------------------------------------------------------------------------
// Matrix-core wrappers.  v_mfma_f32_32x32x16_{bf16,f16}: D[32x32] += A[32x16] * B[16x32].
// Lane l holds, of A, row (l % 32) and the 8 consecutive k = 8*(l/32)..+7; of B, column
// (l % 32) and the same 8 k; of D, column (l % 32) and rows 8*(r/4) + 4*(l/32) + r%4 for
// accumulator register r = 0..15.
// ---------------------------------------------------------------------------------------
template <typename T> struct Mma;
template <> struct Mma<__bf16> {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<_Float16> {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x16 mma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------------------------------
// Buffer loads with hardware range checking: an offset at or beyond `bytes` returns zeros,
// which is how row tails (rows past the end of the tensor) are masked.  Column tails are
// masked by replacing the offset with kOob.
// ---------------------------------------------------------------------------------------
static constexpr uint32_t kOob = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
}
// the same load with the non-temporal hint: for operands that are streamed once (weights in the
// small-M regime).  Measured: with the hint on the weight loads, the row operand's lines survive
// in the CU's L1 between the two 32-k stages that share a 128-byte line (without it every line
// is fetched from L2 twice), and a pure weight stream reaches 6.0 TB/s instead of 5.4.
__device__ __forceinline__ u32x4 buf_load16_nt(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 2);
}
// 16-byte store written through to memory at device scope (cache policy sc1): complete, as
// counted by vmcnt, means visible to every XCD
__device__ __forceinline__ void buf_store16_through(u32x4 v, __amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, 16);
}

// ---------------------------------------------------------------------------------------
// 8x8 transpose of 16-bit elements held in registers.  in[r] = row r (8 elements, element c
// in bits 16*(c%2) of dword c/2); out[c] = column c as 8 elements ordered by row.
// ---------------------------------------------------------------------------------------
// column c of the 8x8 block alone
__device__ __forceinline__ u32x4 transpose8x8_col(const u32x4 (&in)[8], int c) {
    u32x4 out;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = in[2 * d][c >> 1], hi = in[2 * d + 1][c >> 1];
        out[d] = (c & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    }
    return out;
}
__device__ __forceinline__ void transpose8x8_b16(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t lo = in[2 * d][c >> 1];      // row 2d
            const uint32_t hi = in[2 * d + 1][c >> 1];  // row 2d+1
            // v_perm_b32: selector bytes 0-3 address the second operand, 4-7 the first
            out[c][d] = (c & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                                : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
    }
}

// ---------------------------------------------------------------------------------------
// LDS operand tiles.  A tile is R rows of 64 k-values (128 bytes = 8 chunks of 16 bytes);
// MFMA lanes read one chunk per instruction (ds_read_b128), 16 lanes per LDS pass, so the
// 16 lanes of a pass must fall into 16 different 16-byte bank groups (address/16 mod 16).
//
// "Row" tiles hold operands whose k is contiguous in global memory (X, H): written a row at
// a time, read with consecutive lanes on consecutive rows.
// "Col" tiles hold the weight operands, whose k is strided in global memory and which reach
// LDS through the register transpose: written with consecutive lanes 8 rows apart, read
// with consecutive lanes on consecutive rows.  Row r of a Col tile is stored at position
// (r % 8) * (R / 8) + r / 8; the chunk index is XOR-swizzled.  Both patterns are conflict
// free for R / 8 even.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lds_row_off(uint32_t row, uint32_t chunk) {
    return row * 128u + (((chunk ^ (row >> 1)) & 7u) << 4);
}
template <int R> __device__ __forceinline__ uint32_t lds_col_off(uint32_t row, uint32_t chunk) {
    const uint32_t pos = (row & 7u) * (R / 8) + (row >> 3);
    return pos * 128u + (((chunk ^ row ^ (row >> 4)) & 7u) << 4);
}

template <typename V> __device__ __forceinline__ V lds_read16(const char* smem, uint32_t off) {
    return __builtin_bit_cast(V, *reinterpret_cast<const u32x4*>(smem + off));
}
__device__ __forceinline__ void lds_write16(char* smem, uint32_t off, u32x4 v) {
    *reinterpret_cast<u32x4*>(smem + off) = v;
}

// ---------------------------------------------------------------------------------------
// Activations in fp32 (inputs are complete K-sums).  exp via v_exp_f32, 1/x via v_rcp_f32:
// relative error ~1e-6, far below the 16-bit rounding that follows.  They run in the tile
// epilogues with one wave per SIMD, where every instruction is exposed (a 256 x 256 tile's
// epilogue is 256 values per lane), so they are written for instruction count.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float sigmoid_fast(float z) {  // 1 / (1 + exp(-z))
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}
template <int ACT> __device__ __forceinline__ float activate(float x) {
    // median of (x, 0, +inf): one instruction (fmaxf is two: it quiets signalling NaNs first)
    if (ACT == ACT_RELU) return __builtin_amdgcn_fmed3f(x, 0.0f, __builtin_inff());
    if (ACT == ACT_SILU) return x * sigmoid_fast(x);
    if (ACT == ACT_GELU_TANH) {
        // 0.5 (1 + tanh z) = sigmoid(2 z),  z = sqrt(2/pi) (x + 0.044715 x^3); with the constants
        // folded: x / (1 + 2^(x (A + B x^2))),  A = -2 sqrt(2/pi) log2(e),  B = 0.044715 A
        const float t = x * x;
        const float u = __builtin_fmaf(t, -0.10294323958f, -2.3022081983f);
        return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * u));
    }
    return x;
}

// fp32 -> 16-bit operand type, round-to-nearest-even (hardware converts on gfx950)
template <typename T> __device__ __forceinline__ uint32_t pack2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) T t2;
    t2 v;
    v[0] = static_cast<T>(a);
    v[1] = static_cast<T>(b);
    return __builtin_bit_cast(uint32_t, v);
}

// the two 16-bit operands of a dword, widened exactly to fp32 (low half first)
template <typename T> __device__ __forceinline__ void unpack2(uint32_t w, float& a, float& b);
template <> __device__ __forceinline__ void unpack2<__bf16>(uint32_t w, float& a, float& b) {
    a = __builtin_bit_cast(float, w << 16);
    b = __builtin_bit_cast(float, w & 0xffff0000u);
}
template <> __device__ __forceinline__ void unpack2<_Float16>(uint32_t w, float& a, float& b) {
    a = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
    b = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
}

}  // namespace ffuse
