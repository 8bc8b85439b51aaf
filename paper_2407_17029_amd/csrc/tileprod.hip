// Tile product of the adapter, H = A * B (Alg. 1 get_delta_weight before the expansion; the matrix H of
// Sec. 3.3): A bf16 [rows, R], B bf16 [R, cols], H fp32 [rows, cols], fp32 accumulation.
//
// R is small (lambda * r), so the job is to write rows * cols * 4 bytes.  A workgroup owns 64 rows x 128
// columns and the whole contraction in chunks of 128: the A chunk goes into LDS as it is stored (k along the
// row); B is stored with k down the columns, so every thread fetches one 8 x 8 block of it (eight 16-byte
// loads), transposes it in registers with byte permutes and writes eight 16-byte rows -- the [column][k]
// tile the MFMA operand wants, without a transposed copy of B in HBM and without a second launch.  Rows of
// both tiles are 256 bytes with the 16-byte chunks XOR-swizzled by (row ^ row >> 3) & 15, which makes the fragment
// reads and the tile writes conflict-free.  The B tile is the MFMA A operand and the A tile the B operand,
// so a lane ends up with 4 consecutive columns of one row of H; the wave lays its 32 x 64 part out in LDS
// and stores whole 256-byte row segments.
#include "common.h"

namespace qblora {

namespace {

constexpr int kTpRows = 64, kTpCols = 128, kTpK = 128;
constexpr int kTpPitch = 64 * 4 + 16;                      // bytes per staged output row of a wave

// 16 consecutive rows (fragment reads) and 16 rows 8 apart (the transposed writes of one k block) both land
// on 16 different chunks
__device__ __forceinline__ int tp_swz(int row, int chunk) { return row * 256 + ((chunk ^ ((row ^ (row >> 3)) & 15)) << 4); }

__global__ __launch_bounds__(256) void k_tile_product(const qblora_bf16* __restrict__ A, const qblora_bf16* __restrict__ B,
                                                      int rows, int cols, int R, float* __restrict__ H) {
    __shared__ __align__(16) unsigned char smem[(kTpRows + kTpCols) * 256];
    unsigned char* sA = smem;                                   // [64 rows][128 k]
    unsigned char* sB = smem + kTpRows * 256;                   // [128 columns][128 k]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int tiles_c = cols / kTpCols;
    const int row0 = (blockIdx.x / tiles_c) * kTpRows, col0 = (blockIdx.x % tiles_c) * kTpCols;
    const int wr = wave & 1, wc = wave >> 1;                    // the wave's 32 rows x 64 columns
    const int r = lane & 31, hi = lane >> 5;

    f32x16 acc[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.0f;

    for (int kc = 0; kc < R; kc += kTpK) {
        const int kchunks = min(kTpK, R - kc) >> 3;             // 16-byte chunks of k in this pass
        if (kc) __syncthreads();                                // the previous pass is done with the tiles
        // A: 64 rows x kchunks chunks
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = t + 256 * i, row = c >> 4, ch = c & 15;
            if (ch < kchunks)
                *reinterpret_cast<uint4*>(sA + tp_swz(row, ch)) =
                    *reinterpret_cast<const uint4*>(A + (int64_t)(row0 + row) * R + kc + ch * 8);
        }
        // B: thread = (k block kb, column block nb) of 8 x 8 values
        {
            const int kb = t >> 4, nb = t & 15;
            if (kb < kchunks) {
                uint4 b[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    b[i] = *reinterpret_cast<const uint4*>(B + (int64_t)(kc + kb * 8 + i) * cols + col0 + nb * 8);
#pragma unroll
                for (int n = 0; n < 8; ++n) {
                    const uint32_t sel = (n & 1) ? 0x07060302u : 0x05040100u;   // halves n of two rows, side by side
                    uint32_t o[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 &x = b[2 * j], &y = b[2 * j + 1];
                        const uint32_t xs = n < 2 ? x.x : n < 4 ? x.y : n < 6 ? x.z : x.w;
                        const uint32_t ys = n < 2 ? y.x : n < 4 ? y.y : n < 6 ? y.z : y.w;
                        o[j] = __builtin_amdgcn_perm(ys, xs, sel);
                    }
                    *reinterpret_cast<uint4*>(sB + tp_swz(nb * 8 + n, kb)) = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        }
        __syncthreads();
        for (int ks = 0; ks < (kchunks >> 1); ++ks) {
            const bf16x8 fa = *reinterpret_cast<const bf16x8*>(sA + tp_swz(32 * wr + r, 2 * ks + hi));
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const bf16x8 fb = *reinterpret_cast<const bf16x8*>(sB + tp_swz(64 * wc + 32 * c + r, 2 * ks + hi));
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc[c], 0, 0, 0);
            }
        }
    }

    // acc[c][4q + j] is H[row r of the wave][column 32c + 8q + 4hi + j]
    __syncthreads();
    unsigned char* eb = smem + wave * (32 * kTpPitch);
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4*>(eb + r * kTpPitch + (32 * c + 8 * q + 4 * hi) * 4) =
                make_float4(acc[c][4 * q], acc[c][4 * q + 1], acc[c][4 * q + 2], acc[c][4 * q + 3]);
    // the wave reads back its own part only: no barrier, the writes above are complete when their data returns
    const int rr = lane >> 4, cc = lane & 15;
    float* out = H + (int64_t)(row0 + 32 * wr) * cols + col0 + 64 * wc + cc * 4;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = 4 * i + rr;
        // H is far larger than the caches and read by a later launch: a streaming store
        __builtin_nontemporal_store(*reinterpret_cast<const f32x4*>(eb + row * kTpPitch + cc * 16),
                                    reinterpret_cast<f32x4*>(out + (int64_t)row * cols));
    }
}

}  // namespace

// QBLORA_ERR_UNSUPPORTED when the shape is not made of whole tiles (the caller then takes the general path).
int launch_tile_product(const qblora_bf16* A, const qblora_bf16* B, int rows, int cols, int R, float* H, hipStream_t st) {
    auto aligned16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    if (rows <= 0 || cols <= 0 || R <= 0 || rows % kTpRows || cols % kTpCols || R % 16 || !aligned16(A) || !aligned16(B) ||
        !aligned16(H))
        return QBLORA_ERR_UNSUPPORTED;
    const int64_t tiles = (int64_t)(rows / kTpRows) * (cols / kTpCols);
    if (tiles > INT32_MAX) return QBLORA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_tile_product, dim3((unsigned)tiles), dim3(256), 0, st, A, B, rows, cols, R, H);
    return launch_status();
}

}  // namespace qblora
