// QA-BLoRA merge (Sec. 3.3, Alg. 2 get_new_beta) for gfx950: fold the adapter's tile matrix H into
// block-wise INT4 parameters.  Streaming, HBM-bound kernels.
//
// The shift of stored element (n,k) is delta = (s * H[k/lambda1, n/lambda2]) / lambda1 (fp32).
//   beta-shift : blocks lie inside tiles, so delta is constant per block and only beta changes.
//   requantize : w' = w~ + delta per element, then the min-max quantizer of Eq. 1 per block.
//
// Requantize tiling: a workgroup of 256 threads owns 64 output rows x 256 input columns and every
// thread owns one whole 64-block of one row, so the block minimum and maximum are thread-local
// (no shuffles) and all of a thread's global loads (32 bytes of codes, scale, beta) are issued
// before anything else.  Meanwhile the workgroup stages the deltas of its tile in LDS, transposed
// to [n/lambda2][k/lambda1] so that a thread's deltas are contiguous (H itself is stored with
// k/lambda1 as the slow index, so the global reads run along n).  When lambda1 divides 64 the run
// of 64/lambda1 deltas of a block is read with 16-byte LDS loads; runs are padded by 4 floats so the
// four blocks of a row hit different banks.
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

// LDS position of delta (c, r) inside the staged tile.  L1 > 0: r = 4 runs of RUN = 64/L1 deltas, each
// padded by 4 floats.  L1 == 0 (lambda1 does not divide 64): plain rows.
template <int L1>
__device__ __forceinline__ int delta_pos(int c, int r, int stride) {
    if constexpr (L1 > 0) return c * stride + r + 4 * (r / (64 / L1));
    else return c * stride + r;
}

// Row stride (floats) of the staged tile; host and device use the same rule.
template <int L1>
__host__ __device__ inline int delta_stride(int lam1) {
    if constexpr (L1 > 0) return KT / L1 + 16 + 4;          // 4 padded runs, +4 skews consecutive columns
    else return KT / lam1 + 3;
}

template <bool GROUPED, bool BETA, int L1>
__global__ __launch_bounds__(256) void k_merge_requant(MergeDesc d) {
    __shared__ float lut[16];
    extern __shared__ __align__(16) float dl[];          // deltas, [hcols][stride]
    const int t = threadIdx.x;
    const int k0 = blockIdx.x * KT, n0 = blockIdx.y * NT;
    const int row = t >> 2, bk = t & 3;
    const int n = n0 + row, k = k0 + kBlock * bk;
    const bool live = n < d.d_out && k < d.d_in;
    const int bpr = d.d_in / kBlock;

    // this thread's block: all global loads first
    uint4 c0 = make_uint4(0, 0, 0, 0), c1 = c0;
    float a = 0.f, b = 0.f;
    int64_t blk = 0;
    if (live) {
        blk = (int64_t)n * bpr + k / kBlock;
        const uint4* cp = reinterpret_cast<const uint4*>(d.codes + ((int64_t)n * d.d_in + k) / 2);
        c0 = cp[0]; c1 = cp[1];
        if constexpr (GROUPED) a = grouped_scale(d.scale_codes, d.scale_step, d.scale_mid, blk, d.scale_group);
        else a = d.scales[blk];
        if constexpr (BETA) b = d.beta[blk];
    }

    // stage the deltas of the tile
    const TileGeom g = tile_geom(d, n0, k0);
    const int ldH = d.d_out / d.lam2, stride = delta_stride<L1>(d.lam1);
    if (t < 16) lut[t] = d.cb.c[t];
    const float lam1f = (float)d.lam1;
    for (int idx = t; idx < g.hrows * g.hcols; idx += 256) {
        const int r = idx / g.hcols, c = idx - r * g.hcols;
        const float h = d.H[(int64_t)(g.hrow0 + r) * ldH + g.hcol0 + c];
        dl[delta_pos<L1>(c, r, stride)] = __fdiv_rn(__fmul_rn(d.s, h), lam1f);
    }
    __syncthreads();
    if (!live) return;

    // w' = w~ + delta for the 64 elements of the block
    const uint32_t cw[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    float w[64];
    const int c = n / d.lam2 - g.hcol0;
    if constexpr (L1 > 0) {
        constexpr int RUN = 64 / L1;
        const float* drow = dl + c * stride + bk * (RUN + 4);
#pragma unroll
        for (int q = 0; q < RUN / 4; ++q) {
            const float4 dv = *reinterpret_cast<const float4*>(drow + 4 * q);
            const float de[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int u = 0; u < L1; ++u) {
                    const int j = (4 * q + e) * L1 + u;
                    const float cv = lut[(cw[j >> 3] >> (4 * (j & 7))) & 15];
                    const float wt = BETA ? __fmaf_rn(cv, a, b) : __fmul_rn(cv, a);
                    w[j] = __fadd_rn(wt, de[e]);
                }
        }
    } else {
        const float* drow = dl + c * stride - g.hrow0;
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            const float cv = lut[(cw[j >> 3] >> (4 * (j & 7))) & 15];
            const float wt = BETA ? __fmaf_rn(cv, a, b) : __fmul_rn(cv, a);
            w[j] = __fadd_rn(wt, drow[(k + j) / d.lam1]);
        }
    }
    float lo = w[0], hi = w[0];
#pragma unroll
    for (int j = 1; j < 64; ++j) { lo = fminf(lo, w[j]); hi = fmaxf(hi, w[j]); }

    // min-max INT4 of the block: one division for the scale, one for its reciprocal
    const float range = __fsub_rn(hi, lo);
    const float al = __fdiv_rn(range, 15.0f);
    uint32_t packed[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (al != 0.0f) {
        const float inv = __fdiv_rn(15.0f, range);
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            // (w-lo)*inv lies in [0, 15*(1+2^-23)], so rint() of it already lies in 0..15: adding
            // 1.5*2^23 rounds to the nearest integer (ties to even) and leaves it in the low mantissa bits
            const float q = __fadd_rn(__fmul_rn(__fsub_rn(w[j], lo), inv), 12582912.0f);
            packed[j >> 3] |= (__float_as_uint(q) - 0x4B400000u) << (4 * (j & 7));
        }
    }
    uint4* op = reinterpret_cast<uint4*>(d.codes_out + ((int64_t)n * d.d_in + k) / 2);
    op[0] = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    op[1] = make_uint4(packed[4], packed[5], packed[6], packed[7]);
    d.alpha_out[blk] = al;
    d.beta_out[blk] = lo;
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

template <int L1>
int launch_requant_l1(const MergeDesc& d, hipStream_t st) {
    const int hcols = NT / d.lam2 + 2;
    const size_t smem = sizeof(float) * (size_t)delta_stride<L1>(d.lam1) * hcols;
    dim3 grid((d.d_in + KT - 1) / KT, (d.d_out + NT - 1) / NT);
    auto launch = [&](auto kern) -> int {
        if (smem > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, d);
        return launch_status();
    };
    if (d.scale_codes) return d.beta ? launch(k_merge_requant<true, true, L1>) : launch(k_merge_requant<true, false, L1>);
    return d.beta ? launch(k_merge_requant<false, true, L1>) : launch(k_merge_requant<false, false, L1>);
}

int launch_merge_requant(const MergeDesc& d, hipStream_t st) {
    switch (d.lam1) {
        case 1: return launch_requant_l1<1>(d, st);
        case 2: return launch_requant_l1<2>(d, st);
        case 4: return launch_requant_l1<4>(d, st);
        case 8: return launch_requant_l1<8>(d, st);
        default: return launch_requant_l1<0>(d, st);
    }
}

int launch_merge_beta_shift(const MergeDesc& d, hipStream_t st) {
    int64_t total = (int64_t)d.d_out * (d.d_in / kBlock);
    unsigned grid = (unsigned)((total + 255) / 256);
    if (d.scale_codes) hipLaunchKernelGGL(k_merge_beta_shift<true>, dim3(grid), dim3(256), 0, st, d);
    else hipLaunchKernelGGL(k_merge_beta_shift<false>, dim3(grid), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
