// Re-layout of the (small) adapter matrices into the K-contiguous bf16 operands the MFMA GEMM
// kernels read.  The non-parametric operators of Sec. 3.2 are folded into these copies:
// AvgPool(lambda1) on the input equals contracting X with A repeated lambda1 times along k and
// scaling by 1/lambda1; repeat_interleave(lambda2) on the output equals using row n/lambda2 of B^T
// for output column n (the tiling conditions stated after Eq. 2).
#include "common.h"

namespace qblora {

namespace {

// out[b][a*e + i] = in[a][b]  for i < e;  in is [na, nb] row-major, out is [nb, na*e] row-major.
// One call handles the 64 x 64 input tile (ta, tb).  When rows are whole 16-byte chunks on both sides
// (nb % 8 == 0 and 16-byte aligned bases) the tile is moved with 16-byte loads and stores.
__device__ __forceinline__ void transpose_expand_tile(const uint16_t* __restrict__ in, int na, int nb, int e,
                                                      uint16_t* __restrict__ out, int ta, int tb,
                                                      uint16_t (*tile)[66]) {
    const int a0 = ta * 64, b0 = tb * 64;
    const int64_t ld = (int64_t)na * e;
    const bool wide = (nb & 7) == 0 && (ld & 7) == 0 && ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    if (wide) {
        // 64 rows x 8 chunks of 8 elements: two chunks per thread
        uint4 v[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int a = a0 + (threadIdx.x >> 3) + 32 * i, bb = b0 + 8 * (threadIdx.x & 7);
            v[i] = (a < na && bb < nb) ? *reinterpret_cast<const uint4*>(in + (int64_t)a * nb + bb) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ar = (threadIdx.x >> 3) + 32 * i, bc = 8 * (threadIdx.x & 7);
            const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                tile[ar][bc + 2 * q] = (uint16_t)(w[q] & 0xffffu);
                tile[ar][bc + 2 * q + 1] = (uint16_t)(w[q] >> 16);
            }
        }
        __syncthreads();
        // output row b0 + r holds 64*e elements of this tile = 8*e chunks; only whole tiles take this
        // path, the ragged edge falls through to the loop below
        if (a0 + 64 <= na && b0 + 64 <= nb) {
            const int chunks = 8 * e;                              // per output row
            for (int idx = threadIdx.x; idx < 64 * chunks; idx += 256) {
                const int r = idx / chunks, c = (idx - r * chunks) * 8;
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t lo = tile[(c + 2 * q) / e][r], hi = tile[(c + 2 * q + 1) / e][r];
                    w[q] = lo | (hi << 16);
                }
                *reinterpret_cast<uint4*>(out + (int64_t)(b0 + r) * ld + (int64_t)a0 * e + c) = make_uint4(w[0], w[1], w[2], w[3]);
            }
            return;
        }
    } else {
        const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;   // 64 x 4
        uint16_t v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int a = a0 + ty + 4 * i, bb = b0 + tx;
            v[i] = (a < na && bb < nb) ? in[(int64_t)a * nb + bb] : (uint16_t)0;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) tile[ty + 4 * i][tx] = v[i];
        __syncthreads();
    }
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int width = 64 * e;                                  // output columns covered by this tile
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int r = ty + 4 * i;
        const int bb = b0 + r;
        if (bb >= nb) continue;
        for (int c = tx; c < width; c += 64) {
            const int a = a0 + c / e;
            if (a < na) out[(int64_t)bb * ld + (int64_t)a0 * e + c] = tile[c / e][r];
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
    float* scales_tiled; int nS;    // blocks of this job (256 rows x 16 blocks each)
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
        // 256 rows x 16 blocks per workgroup: rows are read along their (contiguous) blocks, written
        // per block along the 256 rows of the tile, through LDS
        __shared__ float st[16][257];
        const int groups = (d.bpr + 15) / 16;
        const int rt = b / groups, blk0 = (b - rt * groups) * 16;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int idx = i * 256 + threadIdx.x;
            const int r = idx >> 4, q = idx & 15;
            const int64_t n = (int64_t)rt * 256 + r;
            float v = 0.0f;
            if (n < d.d_out && blk0 + q < d.bpr) {
                const int64_t i0 = n * d.bpr + blk0 + q;
                v = d.scale_codes ? grouped_scale(d.scale_codes, d.scale_step, d.scale_mid, i0, d.scale_group) : d.scales[i0];
            }
            st[q][r] = v;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (blk0 + q < d.bpr)
                d.scales_tiled[((int64_t)rt * d.bpr + blk0 + q) * 256 + threadIdx.x] = st[q][threadIdx.x];
        return;
    }
    b -= d.nS;
    // Bx[j][n] = B[j][n / lam2]: 8 consecutive n (16 bytes) per store when rows are whole chunks
    const int64_t ld = (int64_t)d.cols_B * d.lam2;
    const int64_t total = (int64_t)d.R * ld;
    if ((ld & 7) == 0 && (reinterpret_cast<uintptr_t>(d.Bx) & 15) == 0) {
        const int64_t base = (int64_t)b * 2048;
        const int64_t i = base + 8 * (int64_t)threadIdx.x;
        if (i < total) {
            const int64_t j = i / ld;
            const int n = (int)(i - j * ld);
            const uint16_t* src = d.B + j * d.cols_B;
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t lo = src[(n + 2 * q) / d.lam2], hi = src[(n + 2 * q + 1) / d.lam2];
                w[q] = lo | (hi << 16);
            }
            *reinterpret_cast<uint4*>(d.Bx + i) = make_uint4(w[0], w[1], w[2], w[3]);
        }
        return;
    }
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

// Expanded adapter operand for the alternative scale operators (Sec. 4.3 "The scale operators"):
// every output element copies one source element or is zero.  Small (at most d x R elements), so one
// element per thread is enough.
struct ExpandDesc {
    const uint16_t* in; int src_rows, src_cols, transpose;
    int out_rows, out_cols, row_map, row_lam, col_map, col_lam;
    uint16_t* out;
};

__device__ __forceinline__ int map_index(int idx, int map, int lam, int n_src) {
    switch (map) {
        case MAP_DIV: return idx / lam;
        case MAP_FRONT: return idx < n_src ? idx : -1;
        case MAP_STRIDE: return idx % lam == 0 ? idx / lam : -1;
        default: return idx;
    }
}

__global__ __launch_bounds__(256) void k_expand_op(ExpandDesc d) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)d.out_rows * d.out_cols) return;
    const int r = (int)(i / d.out_cols), c = (int)(i - (int64_t)r * d.out_cols);
    const int sr = map_index(r, d.row_map, d.row_lam, d.src_rows);
    const int sc = map_index(c, d.col_map, d.col_lam, d.src_cols);
    uint16_t v = 0;
    if (sr >= 0 && sc >= 0 && sr < d.src_rows && sc < d.src_cols)
        v = d.transpose ? d.in[(int64_t)sc * d.src_rows + sr] : d.in[(int64_t)sr * d.src_cols + sc];
    d.out[i] = v;
}

}  // namespace

int launch_adapter_prep(const qblora_bf16* A, const qblora_bf16* B, int d_in, int d_out, int R, int lam1,
                        int lam2, qblora_bf16* At_x, qblora_bf16* Bt, qblora_bf16* Bx, hipStream_t st,
                        const ScaleTiling* sc) {
    PrepDesc d{};
    if (sc && sc->out) {
        d.scales = sc->scales; d.scale_codes = sc->scale_codes; d.scale_step = sc->scale_step; d.scale_mid = sc->scale_mid;
        d.scale_group = sc->scale_group; d.d_out = sc->d_out; d.bpr = sc->d_in / kBlock; d.scales_tiled = sc->out;
        d.nS = ((sc->d_out + 255) / 256) * ((d.bpr + 15) / 16);
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

int launch_expand_op(const qblora_bf16* in, int src_rows, int src_cols, int transpose, int out_rows, int out_cols,
                     int row_map, int row_lam, int col_map, int col_lam, qblora_bf16* out, hipStream_t st) {
    if (!in || !out || src_rows <= 0 || src_cols <= 0 || out_rows <= 0 || out_cols <= 0 || row_lam <= 0 || col_lam <= 0)
        return QBLORA_ERR_SHAPE;
    ExpandDesc d{reinterpret_cast<const uint16_t*>(in), src_rows, src_cols, transpose, out_rows, out_cols,
                 row_map, row_lam, col_map, col_lam, reinterpret_cast<uint16_t*>(out)};
    const int64_t total = (int64_t)out_rows * out_cols;
    hipLaunchKernelGGL(k_expand_op, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
