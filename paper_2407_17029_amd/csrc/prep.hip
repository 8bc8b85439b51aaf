// Re-layout of the (small) adapter matrices into the K-contiguous bf16 operands the MFMA GEMM
// kernels read.  The non-parametric operators of Sec. 3.2 are folded into these copies:
// AvgPool(lambda1) on the input equals contracting X with A repeated lambda1 times along k and
// scaling by 1/lambda1; repeat_interleave(lambda2) on the output equals using row n/lambda2 of B^T
// for output column n (the tiling conditions stated after Eq. 2).
#include "common.h"

namespace qblora {

namespace {

// out[b][a*e + i] = in[a][b]  for i < e;  in is [na, nb] row-major, out is [nb, na*e] row-major.
// One call handles the 64 x 64 input tile (ta, tb).
__device__ __forceinline__ void transpose_expand_tile(const uint16_t* __restrict__ in, int na, int nb, int e,
                                                      uint16_t* __restrict__ out, int ta, int tb,
                                                      uint16_t (*tile)[66]) {
    const int a0 = ta * 64, b0 = tb * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;   // 64 x 4
    // all 16 loads of a thread are independent and issued together
    uint16_t v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int a = a0 + ty + 4 * i, b = b0 + tx;
        v[i] = (a < na && b < nb) ? in[(int64_t)a * nb + b] : (uint16_t)0;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[ty + 4 * i][tx] = v[i];
    __syncthreads();
    const int64_t ld = (int64_t)na * e;
    const int width = 64 * e;                                  // output columns covered by this tile
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int r = ty + 4 * i;
        const int b = b0 + r;
        if (b >= nb) continue;
        for (int c = tx; c < width; c += 64) {
            const int a = a0 + c / e;
            if (a < na) out[(int64_t)b * ld + (int64_t)a0 * e + c] = tile[c / e][r];
        }
    }
}

struct PrepDesc {
    const uint16_t* A; const uint16_t* B;
    int na_A, R, lam1;          // A is [na_A, R]
    int cols_B, lam2;           // B is [R, cols_B]
    uint16_t* At_x; uint16_t* Bt; uint16_t* Bx;
    int tilesA_a, tilesA_b, nA;     // tile grid of the A job and its block count (0 when skipped)
    int tilesB_a, tilesB_b, nB;     // tile grid of the B-transpose job
    int nX;                         // blocks of the column-expansion job (2048 outputs each)
    // block scales in the order the forward kernel streams them: [row tile of 256][64-block][row in tile]
    const float* scales; const uint8_t* scale_codes; const float* scale_step; const float* scale_mid;
    int scale_group, d_out, bpr;
    float* scales_tiled; int nS;    // blocks of this job (256 outputs each)
};

// All re-layouts of one call in a single launch: blocks [0,nA) transpose-expand A, the next nB
// transpose B, the last nX expand B along its columns.
__global__ __launch_bounds__(256) void k_adapter_prep(PrepDesc d) {
    __shared__ uint16_t tile[64][66];
    int b = blockIdx.x;
    if (b < d.nA) {
        transpose_expand_tile(d.A, d.na_A, d.R, d.lam1, d.At_x, b % d.tilesA_a, b / d.tilesA_a, tile);
        return;
    }
    b -= d.nA;
    if (b < d.nB) {
        transpose_expand_tile(d.B, d.R, d.cols_B, 1, d.Bt, b % d.tilesB_a, b / d.tilesB_a, tile);
        return;
    }
    b -= d.nB;
    if (b < d.nS) {
        const int64_t o = (int64_t)b * 256 + threadIdx.x;             // ((tile*bpr + blk)*256 + r)
        const int r = threadIdx.x;
        const int64_t tb = b;
        const int64_t tile = tb / d.bpr, blk = tb - tile * d.bpr;
        const int64_t n = tile * 256 + r;
        float v = 0.0f;
        if (n < d.d_out) {
            const int64_t i = n * d.bpr + blk;
            v = d.scale_codes ? grouped_scale(d.scale_codes, d.scale_step, d.scale_mid, i, d.scale_group) : d.scales[i];
        }
        d.scales_tiled[o] = v;
        return;
    }
    b -= d.nS;
    // Bx[j][n] = B[j][n / lam2]
    const int64_t ld = (int64_t)d.cols_B * d.lam2;
    const int64_t total = (int64_t)d.R * ld;
    const int64_t base = (int64_t)b * 2048;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int64_t i = base + u * 256 + threadIdx.x;
        if (i < total) {
            const int64_t j = i / ld, n = i - j * ld;
            d.Bx[i] = d.B[j * d.cols_B + n / d.lam2];
        }
    }
}

}  // namespace

int launch_adapter_prep(const qblora_bf16* A, const qblora_bf16* B, int d_in, int d_out, int R, int lam1,
                        int lam2, qblora_bf16* At_x, qblora_bf16* Bt, qblora_bf16* Bx, hipStream_t st,
                        const ScaleTiling* sc) {
    PrepDesc d{};
    if (sc && sc->out) {
        d.scales = sc->scales; d.scale_codes = sc->scale_codes; d.scale_step = sc->scale_step; d.scale_mid = sc->scale_mid;
        d.scale_group = sc->scale_group; d.d_out = sc->d_out; d.bpr = sc->d_in / kBlock; d.scales_tiled = sc->out;
        d.nS = ((sc->d_out + 255) / 256) * d.bpr;
    }
    if (!A || !B) At_x = Bt = Bx = nullptr;
    d.A = A; d.B = B; d.na_A = d_in / lam1; d.R = R; d.lam1 = lam1; d.cols_B = d_out / lam2; d.lam2 = lam2;
    d.At_x = At_x; d.Bt = Bt; d.Bx = Bx;
    if (At_x) { d.tilesA_a = (d.na_A + 63) / 64; d.tilesA_b = (R + 63) / 64; d.nA = d.tilesA_a * d.tilesA_b; }
    if (Bt) { d.tilesB_a = (R + 63) / 64; d.tilesB_b = (d.cols_B + 63) / 64; d.nB = d.tilesB_a * d.tilesB_b; }
    if (Bx) d.nX = (int)(((int64_t)R * d_out + 2047) / 2048);
    const int blocks = d.nA + d.nB + d.nS + d.nX;
    if (blocks == 0) return QBLORA_OK;
    hipLaunchKernelGGL(k_adapter_prep, dim3(blocks), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
