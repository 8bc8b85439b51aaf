// Adapter-parameter gradients: reductions over all tokens (backward of Sec. 3.2's A and B).
//
//   dA = P^T dU = (1/lambda1) * pool_rows_lambda1( X^T dU )          [d_in/lambda1, R]
//   dB = U^T dV = transpose( pool_rows_lambda2( dY^T (s U) ) )        [R, d_out/lambda2]
//
// Both are "token-contraction" GEMMs  part[z][i][j] = sum_{t in slice z} L[t,i] * S[t,j]  with a
// wide L (X or dY) and a narrow S (dU or s*U, inner rank columns).  The token range is split over
// `splits` workgroup slices so the launch fills the chip; the partial sums are written to scratch
// and a second kernel adds them in a fixed order (deterministic), pools adjacent rows and applies
// the scale.  Operand tiles are transposed in registers on their way into LDS so that each MFMA
// lane reads 8 consecutive tokens of one feature as a single 16-byte word.  The narrow operand is
// produced by this library in fp32 and handed over as a bf16 pair (high part + residual); both parts
// are contracted, so the gradients carry fp32-accumulation error only.
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 512;
constexpr int BI = 128, BJ = 128, BT = 64;

__device__ __forceinline__ int swz(int row, int chunk) {
    return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

__global__ __launch_bounds__(kThreads) void k_grad_partial(GradDesc d, int64_t slice_len) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char (*sL)[BI * 128] = reinterpret_cast<unsigned char (*)[BI * 128]>(smem);
    unsigned char (*sS)[BJ * 128] = reinterpret_cast<unsigned char (*)[BJ * 128]>(smem + 2 * BI * 128);
    unsigned char (*sSlo)[BJ * 128] = reinterpret_cast<unsigned char (*)[BJ * 128]>(smem + 2 * BI * 128 + 2 * BJ * 128);
    const bool has_lo = d.S_lo != nullptr;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int i0 = blockIdx.x * BI, j0 = blockIdx.y * BJ, z = blockIdx.z;
    const int64_t t_begin = (int64_t)z * slice_len;
    int64_t t_end = t_begin + slice_len;
    if (t_end > d.T) t_end = d.T;
    const int nsteps = t_begin < t_end ? (int)((t_end - t_begin + BT - 1) / BT) : 0;

    // wave tile: 32 j (MFMA rows) x 64 i (MFMA columns, two blocks)
    const int wj0 = (wave & 3) * 32, wi0 = (wave >> 2) * 64;
    f32x16 acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

    // loader: threads 0..255 move the L tile, 256..511 the S tile; an item is 8 tokens x 4 columns
    const bool isL = t < 256;
    const int item = t & 255, cg = item & 31, tg = item >> 5;
    const qblora_bf16* src = isL ? d.L : d.S;
    const int64_t ld = isL ? d.ldl : d.lds;
    const int width = isL ? d.I : d.J;
    int col = (isL ? i0 : j0) + 4 * cg;
    if (col > width - 4) col = width - 4;          // clamped columns are never stored
    uint2 reg[8], reg_lo[8];

    auto load_global = [&](int step) {
        const int64_t tb = t_begin + (int64_t)step * BT + 8 * tg;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int64_t tt = tb + q;
            reg[q] = (tt < t_end) ? *reinterpret_cast<const uint2*>(src + tt * ld + col) : make_uint2(0, 0);
            if (!isL && has_lo)
                reg_lo[q] = (tt < t_end) ? *reinterpret_cast<const uint2*>(d.S_lo + tt * ld + col) : make_uint2(0, 0);
        }
    };
    auto transpose_store = [&](const uint2 (&rg)[8], unsigned char* base) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t h[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint32_t w = (c < 2) ? rg[q].x : rg[q].y;
                h[q] = (c & 1) ? (w >> 16) : (w & 0xffffu);
            }
            uint4 o;
            o.x = h[0] | (h[1] << 16); o.y = h[2] | (h[3] << 16);
            o.z = h[4] | (h[5] << 16); o.w = h[6] | (h[7] << 16);
            *reinterpret_cast<uint4*>(base + swz(4 * cg + c, tg)) = o;
        }
    };
    auto store_lds = [&](int buf) {
        transpose_store(reg, isL ? sL[buf] : sS[buf]);
        if (!isL && has_lo) transpose_store(reg_lo, sSlo[buf]);
    };
    auto compute = [&](int buf) {
        const int r = lane & 31, hi = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 sf = *reinterpret_cast<const bf16x8*>(sS[buf] + swz(wj0 + r, ks * 2 + hi));
            bf16x8 sf_lo = sf;
            if (has_lo) sf_lo = *reinterpret_cast<const bf16x8*>(sSlo[buf] + swz(wj0 + r, ks * 2 + hi));
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                bf16x8 lf = *reinterpret_cast<const bf16x8*>(sL[buf] + swz(wi0 + b * 32 + r, ks * 2 + hi));
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, lf, acc[b], 0, 0, 0);
                if (has_lo) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf_lo, lf, acc[b], 0, 0, 0);
            }
        }
    };

    if (nsteps > 0) {
        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int step = 0; step < nsteps; ++step) {
            const bool more = step + 1 < nsteps;
            if (more) load_global(step + 1);
            compute(step & 1);
            if (more) store_lds((step + 1) & 1);
            __syncthreads();
        }
    }

    // accumulator rows are j (4 consecutive per lane), columns are i
    float* part = d.part + (int64_t)z * d.I * d.J;
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int i = i0 + wi0 + b * 32 + r;
        if (i >= d.I) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int j = j0 + wj0 + q * 8 + hi * 4;
            if (j >= d.J) continue;
            *reinterpret_cast<float4*>(part + (int64_t)i * d.J + j) =
                make_float4(acc[b][q * 4 + 0], acc[b][q * 4 + 1], acc[b][q * 4 + 2], acc[b][q * 4 + 3]);
        }
    }
}

// out[i', j] (or out[j, i'] when transposed) = out_scale * sum_{p < pool} sum_z part[z][i'*pool+p][j],
// summed in ascending (p, z) order.
__global__ __launch_bounds__(256) void k_grad_reduce(GradDesc d) {
    const int Ip = d.I / d.pool;
    const int64_t total = (int64_t)Ip * d.J;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % d.J);
    const int ip = (int)(idx / d.J);
    const int64_t plane = (int64_t)d.I * d.J;
    float sum = 0.0f;
    for (int p = 0; p < d.pool; ++p) {
        const float* src = d.part + (int64_t)(ip * d.pool + p) * d.J + j;
        for (int z = 0; z < d.splits; ++z) sum += src[z * plane];
    }
    sum *= d.out_scale;
    if (d.transpose_out) d.out[(int64_t)j * Ip + ip] = sum;
    else d.out[(int64_t)ip * d.J + j] = sum;
}

}  // namespace

int grad_splits(int64_t T, int I) {
    int tiles_i = (I + BI - 1) / BI;
    int want = (256 + tiles_i - 1) / tiles_i;          // one workgroup per CU
    int64_t max_splits = (T + BT - 1) / BT;
    if (want > max_splits) want = (int)max_splits;
    if (want > 32) want = 32;
    if (want < 1) want = 1;
    return want;
}

int launch_grad(const GradDesc& d, hipStream_t st) {
    if (d.T <= 0) return QBLORA_ERR_SHAPE;      // the entry point handles the empty batch itself
    int64_t slice_len = (d.T + d.splits - 1) / d.splits;
    slice_len = (slice_len + BT - 1) / BT * BT;
    dim3 grid((d.I + BI - 1) / BI, (d.J + BJ - 1) / BJ, d.splits);
    constexpr size_t smem = 2 * BI * 128 + 4 * BJ * 128;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_grad_partial),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_grad_partial, grid, dim3(kThreads), smem, st, d, slice_len);
    int64_t total = (int64_t)(d.I / d.pool) * d.J;
    hipLaunchKernelGGL(k_grad_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
