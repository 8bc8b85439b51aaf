// Shared device/host helpers of the gfx950 kernels (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qblora.h"

namespace qblora {

constexpr int kBlock = 64;   // quantization block: 64 contiguous k of one output row

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct Codebook {
    float c[16];
};

// Two fp32 -> one dword of two bf16 (round to nearest even); lo in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 p;
    p[0] = (__bf16)lo;
    p[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, p);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// OCP E4M3 bit pattern -> fp32 (NaN patterns are never produced by the encoder).
__device__ __forceinline__ float e4m3_to_float(uint32_t c) {
    uint32_t e = (c >> 3) & 0xf, m = c & 7;
    float v = e ? __uint_as_float(((e + 120u) << 23) | (m << 20)) : (float)m * 0x1p-9f;
    return (c & 0x80) ? -v : v;
}

// Byte `idx` (0 .. 3, a constant after unrolling) of v as a float: one v_cvt_f32_ubyteN, provided the compiler knows
// nothing about v's bits (see opaque_bits): from a shift and a mask of a value whose upper nibbles it knows to be zero
// it makes a bit-field extract and a conversion.
__device__ __forceinline__ float byte_to_float(uint32_t v, int idx) { return (float)((v >> (8 * idx)) & 0xffu); }

// The same value in a register the compiler cannot see through (no instruction).  Used instead of writing vector
// instructions as inline assembly: the compiler's hazard handling around MFMAs does not look inside assembly
// statements (an assembly instruction that reuses a register of an MFMA result still in flight is overwritten by it).
__device__ __forceinline__ uint32_t opaque_bits(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

// Reconstructed block scale under the grouped E4M3 second-level quantization.
__device__ __forceinline__ float grouped_scale(const uint8_t* __restrict__ scale_codes,
                                               const float* __restrict__ step,
                                               const float* __restrict__ mid, int64_t i, int group) {
    int64_t g = i / group;
    return __fmaf_rn(e4m3_to_float(scale_codes[i]), step[g], mid[g]);
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? QBLORA_OK : QBLORA_ERR_LAUNCH; }

// Records the caller's registered event pair of slot `which` (qblora_profile_events; none by default) on the
// stream around the launches made while the object lives.
struct ProfileScope {
    int which; hipStream_t st;
    ProfileScope(int which, hipStream_t st);
    ~ProfileScope();
    ProfileScope(const ProfileScope&) = delete;
    ProfileScope& operator=(const ProfileScope&) = delete;
};

// ---- kernels' host launchers (defined in the .hip files) -------------------------------------

// `tiled` (may be NULL) receives the second, tile-ordered copy of the codes described in qblora.h
int launch_quantize_codebook(const float* W, int d_out, int d_in, const Codebook& cb, uint8_t* codes,
                             uint8_t* tiled, float* absmax, hipStream_t st, int block_rows = 1, int block_cols = 8);
int launch_quantize_minmax(const float* W, int d_out, int d_in, uint8_t* codes, uint8_t* tiled, float* alpha,
                           float* beta, hipStream_t st, int block_rows = 1, int block_cols = 8);
int launch_prepack_codes(const uint8_t* codes, int d_out, int d_in, uint8_t* tiled, hipStream_t st, int regroup = 0);

// byte offset of the 32-byte run of (row n, 64-block b) in the tiled code copy
__host__ __device__ inline int64_t tiled_run_offset(int64_t n, int64_t b, int64_t blocks_per_row) {
    return (((n >> 8) * blocks_per_row + b) * 256 + (n & 255)) * 32;
}
int launch_scales_double_quantize(const float* scales, int64_t n, int group, uint8_t* scale_codes,
                                  float* step, float* mid, hipStream_t st);
int launch_scales_reconstruct(const uint8_t* scale_codes, const float* step, const float* mid, int64_t n,
                              int group, float* scales, hipStream_t st);
int launch_dequantize_bf16(const qblora_qweight& qw, const float* scales, qblora_bf16* Wt, hipStream_t st);
// The bf16 compute weight in the order the contraction kernel's waves load it (qmode 3): for the operand
// matrix Wop[N, K] -- the weight itself, N = d_out, K = d_in (transposed = 0), or its transpose, N = d_in,
// K = d_out -- the 16 bytes Wop[32i + (l & 31)][16j + 8(l >> 5) .. + 7] sit at ((i*(K/16) + j)*64 + l)*16.
// d_out*d_in*2 bytes, 16-byte aligned; d_in % 64 == 0, d_out % 64 == 0.
int launch_dequantize_operand(const qblora_qweight& qw, const float* scales, int transposed, qblora_bf16* Wop,
                              hipStream_t st);

// Builds K-contiguous bf16 copies of the adapter matrices for the GEMM kernels:
//   At_x [R, d_in]        At_x[j,k] = A[k/lam1, j]     (transpose, expand along k)
//   Bt   [d_out/lam2, R]  Bt[q,j]   = B[j, q]          (transpose)
//   Bx   [R, d_out]       Bx[j,n]   = B[j, n/lam2]     (expand along n)
// Any output pointer may be NULL to skip it.
// Optional extra job of the same launch: the block scales (fp32, or reconstructed from the grouped E4M3
// form when scale_codes is set) re-ordered to [row tile of 256][64-block][row in tile] for the forward kernel.
struct ScaleTiling {
    const float* scales; const uint8_t* scale_codes; const float* scale_step; const float* scale_mid;
    int scale_group, d_out, d_in;
    float* out;
};
int launch_adapter_prep(const qblora_bf16* A, const qblora_bf16* B, int d_in, int d_out, int R, int lam1,
                        int lam2, qblora_bf16* At_x, qblora_bf16* Bt, qblora_bf16* Bx, hipStream_t st,
                        const ScaleTiling* sc = nullptr);

// One GEMM launch description.  C[M,N] = out_scale1 * ( X1[M,K1] * Wq^T  +  X2[M,K2] * W2[N/div2, K2]^T )
// "token" operands X1/X2 are bf16 row-major; the quantized segment is optional (qmode 0).
struct GemmDesc {
    int qmode;                 // 0: no quantized segment; 1: forward (N = d_out, K1 = d_in);
                               // 2: transposed use (N = d_in, K1 = d_out);
                               // 3: first segment on a bf16 weight dequantized beforehand, in operand order
    const qblora_bf16* X1; int64_t ldx1;
    const qblora_bf16* W1; int K1;                     // qmode 3 only: see launch_dequantize_operand
    const uint8_t* codes; const float* scales; const float* beta; int d_out, d_in;
    const uint8_t* codes_tiled;            // optional tile-ordered copy (forward only)
    const float* scales_tiled;             // optional tile-ordered scales (forward only)
    Codebook cb;
    const qblora_bf16* X2; int64_t ldx2;
    const qblora_bf16* W2; int64_t ldw2; int K2; int div2;
    void* C; int64_t ldc; int out_f32;     // bf16 or fp32 output
    qblora_bf16* C2; float c2_scale;       // optional second bf16 output = bf16(c2_scale * value), same shape
    qblora_bf16* C_lo;                     // optional bf16 residual: bf16(value - bf16(value)), same shape
    float out_scale;
    int64_t M; int N;
    int block_rows;            // rows of a quantization block: 0/1 = 64 inputs of one row, 8 = 8 rows x 8 inputs
    int dup2;                  // qmode 0, narrow form only: 2 = W2 has K2/2 columns, column m serves k = 2m, 2m+1
};
int launch_gemm(const GemmDesc& d, hipStream_t st);
// the quantized segments (qmode 1, 2) with an 8-wave 256x256 tile; called by launch_gemm
int launch_qlinear(const GemmDesc& d, hipStream_t st);
// narrow-output plain bf16 GEMM (qmode 0, N = inner rank); called by launch_gemm when it applies
bool skinny_applies(const GemmDesc& d);
bool skinny_dup_applies(int64_t M, int N, int K, int64_t ldw);
int launch_skinny(const GemmDesc& d, hipStream_t st);

// Token-contraction GEMM with split-T partials:  part[z][i][j] = sum_{t in slice z} L[t,i] * S[t,j]
// followed by the reduction  out = sum_z part, pooled over `pool` adjacent i (scaled by out_scale),
// written row-major [I/pool, J] or, when transpose_out, [J, I/pool].
struct GradDesc {
    const qblora_bf16* L; int64_t ldl; int I;
    const qblora_bf16* S; int64_t lds; int J;
    const qblora_bf16* S_lo;               // optional low-order part of S (S = S + S_lo, both bf16), same layout
    int64_t T;
    float* part; int splits;
    float* out; int pool; float out_scale; int transpose_out;
};
int grad_splits(int64_t T, int I, int J = 1);    // slices of the token range for an [I, J] gradient
int launch_pool_rows(const qblora_bf16* in, int64_t T, int d, int lam, float scale, qblora_bf16* out,
                     qblora_bf16* out_lo, hipStream_t st);
int launch_grad(const GradDesc& d, hipStream_t st);
// two independent gradients whose partial buffers do not overlap: one launch for both where the shapes allow
int launch_grad_pair(const GradDesc& a, const GradDesc& b, hipStream_t st);
// out[t, c] = in[t, lam*c] for c < d/lam (every lam-th feature of each row), bf16
int launch_sample_rows(const qblora_bf16* in, int64_t T, int d, int lam, qblora_bf16* out, hipStream_t st);

// Index maps of the expanded adapter operands: output index -> source index, or "zero".
enum { MAP_ID = 0, MAP_DIV = 1, MAP_FRONT = 2, MAP_STRIDE = 3 };
// out[r][c] (bf16 [out_rows, out_cols]) = src(map_row(r), map_col(c)), 0 where a map says zero.  The source
// has src_rows x src_cols elements, stored row-major [src_rows, src_cols], or [src_cols, src_rows] when `transpose`.
int launch_expand_op(const qblora_bf16* in, int src_rows, int src_cols, int transpose, int out_rows, int out_cols,
                     int row_map, int row_lam, int col_map, int col_lam, qblora_bf16* out, hipStream_t st);

struct MergeDesc {
    const uint8_t* codes; const float* scales; const float* beta;
    const uint8_t* scale_codes; const float* scale_step; const float* scale_mid; int scale_group;
    Codebook cb; int d_out, d_in;
    const float* H; int lam1, lam2; float s;
    uint8_t* codes_out; float* alpha_out; float* beta_out;
    qblora_bf16* w16_out;                  // 16-bit merge only
    int block_rows;                        // 1 or 8
    int block_cols;                        // with block_rows 8: inputs per block, 8 or 4
    uint32_t kgroups_magic;                // set by the launcher: reciprocal for the tile index arithmetic
};
int launch_merge_requant(const MergeDesc& d, hipStream_t st);
// several weights in one launch; QBLORA_ERR_UNSUPPORTED (nothing launched) when they cannot share one
int launch_merge_requant_batch(const MergeDesc* ds, int count, hipStream_t st);
int launch_merge_bf16(const MergeDesc& d, hipStream_t st);
// H = A * B (fp32) for whole 64 x 128 tiles and R % 16 == 0; QBLORA_ERR_UNSUPPORTED otherwise (nothing launched)
int launch_tile_product(const qblora_bf16* A, const qblora_bf16* B, int rows, int cols, int R, float* H, hipStream_t st);
int launch_w4_decode(const uint8_t* codes, const float* scales, const float* beta, const Codebook& cb, int tiled,
                     int d_out, int d_in, const qblora_bf16* X, int T, qblora_bf16* Y, hipStream_t st, int block_rows = 1, int regrouped = 0);
// The same layer for 1 <= T <= 128 tokens on the bf16 compute weight (w4mid.hip); `part` holds
// w4_mid_part_bytes() bytes of split-K partial tiles (may be NULL when that is 0)
int w4_mid_splits(int d_out, int d_in, int T);
size_t w4_mid_part_bytes(int d_out, int d_in, int T);
int launch_w4_mid(const uint8_t* codes, const float* scales, const float* beta, const Codebook& cb, int tiled, int d_out,
                  int d_in, const qblora_bf16* X, int T, qblora_bf16* Y, float* part, hipStream_t st, int block_rows = 1,
                  int regrouped = 0, int block_cols = 8);
int launch_merge_beta_shift(const MergeDesc& d, hipStream_t st);

}  // namespace qblora
