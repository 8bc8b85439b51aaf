// QA-BLoRA merge (Sec. 3.3, Alg. 2 get_new_beta) for gfx950: fold the adapter's tile matrix H into
// block-wise INT4 parameters.  Streaming, HBM-bound kernels.
//
// The shift of stored element (n,k) is delta = (s * H[k/lambda1, n/lambda2]) / lambda1 (fp32).
//   beta-shift : blocks lie inside tiles, so delta is constant per block and only beta changes.
//   requantize : w' = w~ + delta per element, then the min-max quantizer of Eq. 1 per block.
//
// Requantize tiling: a workgroup owns 64 output rows x 256 input columns.  It first stages the
// deltas of that tile in LDS, transposed to [n/lambda2][k/lambda1] so that the per-element reads
// along k are contiguous (H itself is stored with k/lambda1 as the slow index, so the global reads
// run along n).  A thread then handles one dword of 8 codes; the 8 lanes that share a 64-block
// reduce min/max with shuffles.
#include "common.h"

namespace qblora {

namespace {

constexpr int NT = 64, KT = 256;

struct TileGeom {
    int hrow0, hrows, hcol0, hcols;
};

__device__ __forceinline__ TileGeom tile_geom(const MergeDesc& d, int n0, int k0) {
    TileGeom g;
    int k1 = min(k0 + KT, d.d_in) - 1, n1 = min(n0 + NT, d.d_out) - 1;
    g.hrow0 = k0 / d.lam1; g.hrows = k1 / d.lam1 - g.hrow0 + 1;
    g.hcol0 = n0 / d.lam2; g.hcols = n1 / d.lam2 - g.hcol0 + 1;
    return g;
}

template <bool GROUPED>
__global__ __launch_bounds__(256) void k_merge_requant(MergeDesc d) {
    extern __shared__ __align__(16) float smem_f[];
    float* lut = smem_f;                 // 16 code values
    float* dl = smem_f + 16;             // deltas, [hcols][hrows + 1]
    const int t = threadIdx.x;
    const int k0 = blockIdx.x * KT, n0 = blockIdx.y * NT;
    const TileGeom g = tile_geom(d, n0, k0);
    const int ldH = d.d_out / d.lam2, stride = g.hrows + 1;
    if (t < 16) lut[t] = d.cb.c[t];
    const float lam1f = (float)d.lam1;
    for (int idx = t; idx < g.hrows * g.hcols; idx += 256) {
        int r = idx / g.hcols, c = idx - r * g.hcols;
        float h = d.H[(int64_t)(g.hrow0 + r) * ldH + g.hcol0 + c];
        dl[c * stride + r] = __fdiv_rn(__fmul_rn(d.s, h), lam1f);
    }
    __syncthreads();

    const int bpr = d.d_in / kBlock;
    const int words_per_row = KT / 8;                        // 32
    for (int it = 0; it < NT * words_per_row / 256; ++it) {
        const int wi = it * 256 + t;
        const int n = n0 + wi / words_per_row;
        const int k = k0 + (wi % words_per_row) * 8;
        const bool live = n < d.d_out && k < d.d_in;         // whole 64-blocks are live or not
        float w[8];
        float lo = INFINITY, hi = -INFINITY;
        int64_t blk = 0;
        if (live) {
            blk = (int64_t)n * bpr + k / kBlock;
            const uint32_t cw = *reinterpret_cast<const uint32_t*>(d.codes + ((int64_t)n * d.d_in + k) / 2);
            float a;
            if constexpr (GROUPED) a = grouped_scale(d.scale_codes, d.scale_step, d.scale_mid, blk, d.scale_group);
            else a = d.scales[blk];
            const float* drow = dl + (n / d.lam2 - g.hcol0) * stride - g.hrow0;
            if (d.beta) {
                const float b = d.beta[blk];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    w[j] = __fadd_rn(__fmaf_rn(lut[(cw >> (4 * j)) & 15], a, b), drow[(k + j) / d.lam1]);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    w[j] = __fadd_rn(__fmul_rn(lut[(cw >> (4 * j)) & 15], a), drow[(k + j) / d.lam1]);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) { lo = fminf(lo, w[j]); hi = fmaxf(hi, w[j]); }
        }
        // the 8 lanes of a block reduce together (dead blocks carry +-inf and are not stored)
        lo = fminf(lo, __shfl_xor(lo, 4, 8)); hi = fmaxf(hi, __shfl_xor(hi, 4, 8));
        lo = fminf(lo, __shfl_xor(lo, 2, 8)); hi = fmaxf(hi, __shfl_xor(hi, 2, 8));
        lo = fminf(lo, __shfl_xor(lo, 1, 8)); hi = fmaxf(hi, __shfl_xor(hi, 1, 8));
        if (!live) continue;
        const float range = __fsub_rn(hi, lo);
        const float al = __fdiv_rn(range, 15.0f);
        uint32_t packed = 0;
        if (al != 0.0f) {
            const float inv = __fdiv_rn(15.0f, range);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float q = rintf(__fmul_rn(__fsub_rn(w[j], lo), inv));
                q = fminf(fmaxf(q, 0.0f), 15.0f);
                packed |= (uint32_t)q << (4 * j);
            }
        }
        *reinterpret_cast<uint32_t*>(d.codes_out + ((int64_t)n * d.d_in + k) / 2) = packed;
        if ((t & 7) == 0) {
            d.alpha_out[blk] = al;
            d.beta_out[blk] = lo;
        }
    }
}

// beta'[n,b] = beta[n,b] + delta(n, k = b*64); also emits fp32 alpha when the base scales are grouped.
template <bool GROUPED>
__global__ __launch_bounds__(256) void k_merge_beta_shift(MergeDesc d) {
    const int bpr = d.d_in / kBlock;
    const int64_t total = (int64_t)d.d_out * bpr;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int n = (int)(idx % d.d_out), b = (int)(idx / d.d_out);     // n fastest: H reads run along n
    const int64_t blk = (int64_t)n * bpr + b;
    const float h = d.H[(int64_t)((b * kBlock) / d.lam1) * (d.d_out / d.lam2) + n / d.lam2];
    const float delta = __fdiv_rn(__fmul_rn(d.s, h), (float)d.lam1);
    d.beta_out[blk] = d.beta ? __fadd_rn(d.beta[blk], delta) : delta;
    if constexpr (GROUPED)
        d.alpha_out[blk] = grouped_scale(d.scale_codes, d.scale_step, d.scale_mid, blk, d.scale_group);
}

}  // namespace

int launch_merge_requant(const MergeDesc& d, hipStream_t st) {
    // worst-case LDS: (KT/lam1 + 2) x (NT/lam2 + 1) deltas
    int hrows = KT / d.lam1 + 2, hcols = NT / d.lam2 + 2;
    size_t smem = sizeof(float) * (16 + (size_t)(hrows + 1) * hcols);
    dim3 grid((d.d_in + KT - 1) / KT, (d.d_out + NT - 1) / NT);
    auto launch = [&](auto kern) -> int {
        if (smem > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, d);
        return launch_status();
    };
    return d.scale_codes ? launch(k_merge_requant<true>) : launch(k_merge_requant<false>);
}

int launch_merge_beta_shift(const MergeDesc& d, hipStream_t st) {
    int64_t total = (int64_t)d.d_out * (d.d_in / kBlock);
    unsigned grid = (unsigned)((total + 255) / 256);
    if (d.scale_codes) hipLaunchKernelGGL(k_merge_beta_shift<true>, dim3(grid), dim3(256), 0, st, d);
    else hipLaunchKernelGGL(k_merge_beta_shift<false>, dim3(grid), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
