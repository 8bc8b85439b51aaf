// Re-layout of the (small) adapter matrices into the K-contiguous bf16 operands the MFMA GEMM
// kernels read.  The non-parametric operators of Sec. 3.2 are folded into these copies:
// AvgPool(lambda1) on the input equals contracting X with A repeated lambda1 times along k and
// scaling by 1/lambda1; repeat_interleave(lambda2) on the output equals using row n/lambda2 of B^T
// for output column n (the tiling conditions stated after Eq. 2).
#include "common.h"

namespace qblora {

namespace {

// out[b][a*e + i] = in[a][b]  for i < e;  in is [na, nb] row-major, out is [nb, na*e] row-major.
__global__ __launch_bounds__(256) void k_transpose_expand(const uint16_t* __restrict__ in, int na, int nb, int e,
                                                          uint16_t* __restrict__ out) {
    __shared__ uint16_t tile[64][66];
    int a0 = blockIdx.x * 64, b0 = blockIdx.y * 64;
    int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;   // 64 x 4
    for (int r = ty; r < 64; r += 4) {
        int a = a0 + r, b = b0 + tx;
        tile[r][tx] = (a < na && b < nb) ? in[(int64_t)a * nb + b] : (uint16_t)0;
    }
    __syncthreads();
    int64_t ld = (int64_t)na * e;
    int width = 64 * e;                                  // output columns covered by this tile
    for (int r = ty; r < 64; r += 4) {
        int b = b0 + r;
        if (b >= nb) continue;
        for (int c = tx; c < width; c += 64) {
            int a = a0 + c / e;
            if (a < na) out[(int64_t)b * ld + (int64_t)a0 * e + c] = tile[c / e][r];
        }
    }
}

// out[j][n] = in[j][n / e];  in is [rows, cols], out is [rows, cols*e].
__global__ __launch_bounds__(256) void k_expand_cols(const uint16_t* __restrict__ in, int rows, int cols, int e,
                                                     uint16_t* __restrict__ out) {
    int64_t total = (int64_t)rows * cols * e;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int64_t ld = (int64_t)cols * e;
    int64_t j = i / ld, n = i - j * ld;
    out[i] = in[j * cols + n / e];
}

}  // namespace

int launch_adapter_prep(const qblora_bf16* A, const qblora_bf16* B, int d_in, int d_out, int R, int lam1,
                        int lam2, qblora_bf16* At_x, qblora_bf16* Bt, qblora_bf16* Bx, hipStream_t st) {
    if (At_x) {
        int na = d_in / lam1, nb = R;
        hipLaunchKernelGGL(k_transpose_expand, dim3((na + 63) / 64, (nb + 63) / 64), dim3(256), 0, st, A, na, nb,
                           lam1, At_x);
    }
    if (Bt) {
        int na = R, nb = d_out / lam2;
        hipLaunchKernelGGL(k_transpose_expand, dim3((na + 63) / 64, (nb + 63) / 64), dim3(256), 0, st, B, na, nb,
                           1, Bt);
    }
    if (Bx) {
        int64_t total = (int64_t)R * d_out;
        hipLaunchKernelGGL(k_expand_cols, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, B, R,
                           d_out / lam2, lam2, Bx);
    }
    return launch_status();
}

}  // namespace qblora
