// QA-BLoRA merge (Sec. 3.3, Alg. 2 get_new_beta) for gfx950: fold the adapter's tile matrix H into
// block-wise INT4 parameters.  Streaming, HBM-bound kernels.
//
// The shift of stored element (n,k) is delta = (s * H[k/lambda1, n/lambda2]) / lambda1 (fp32).
//   beta-shift : blocks lie inside tiles, so delta is constant per block and only beta changes.
//   requantize : w' = w~ + delta per element, then the min-max quantizer of Eq. 1 per block.
//
// Requantize tiling: a workgroup of 512 threads owns 64 output rows x 256 input columns and every
// thread owns half (32 elements) of one 64-block; the block minimum and maximum are combined over
// the two lanes with DPP.  Measured on a 22016 x 8192 weight, lambda 2 (95 us before the streaming stores, 82-85
// with them): the memory accesses alone, arithmetic removed, take as long as the whole kernel (a model of the
// kernel that keeps only its loads, the LDS staging and its stores: 95 us; its loads alone 57 us = 5.1 TB/s; the
// code stores add 24 us, the 16-byte pieces of block parameters 14 more on top of them and 2 on their own), and the
// vector ALU is busy 0.73 of the time underneath.  Tile shapes from 16 x 2048 to 128 x 256, one block per
// thread, linear / grouped / 8 x 8 super-tile orders and two or three resident workgroups per CU were all equal
// or slower in that model; a variant that walks eight tiles per workgroup with the next tile's loads in flight and
// stores whole lines of block parameters was slower too (fewer waves).  What helps is the streaming hint on the
// code stores.  For scale: a plain elementwise add of two arrays into a third runs at 0.72-0.75 of the HBM peak
// on this chip and a plain copy at 0.66; this kernel's 2 : 1 mix of reads and writes in 128-byte pieces (codes:
// 4 KB apart, H: 44 KB apart) reaches 0.52-0.60.  With lambda 8
// (H a sixteenth of the bytes) the vector ALU is the limit: one thread
// per block (64 elements) keeps the per-thread overhead (addresses, the two divisions of a block)
// lowest but gives only 4 waves per SIMD over a 4096 x 4096 weight, all resident at once and moving
// through load, compute and store phases in lockstep; a quarter block per thread overlaps those
// phases but doubles the overhead per element.  A thread's global loads (16 bytes of codes, scale, beta) are issued
// before anything else.  Meanwhile the workgroup stages the deltas of its tile in LDS, transposed
// to [n/lambda2][k/lambda1] so that a thread's deltas are contiguous (H itself is stored with
// k/lambda1 as the slow index, so the global reads run along n).  When lambda1 divides 64 the run
// of 32/lambda1 deltas of a half is read with 16-byte LDS loads; the runs of a block are
// padded by 4 floats so the four blocks of a row start in different banks.
#include "common.h"

namespace qblora {

namespace {

constexpr int NT = 64, KT = 256;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kMergeThreads = 512;            // 64 rows x 8 half blocks

struct TileGeom {
    int hrow0, hrows, hcol0, hcols;
};

// x / lam with the division spelled out only where it is one: lam a power of two (shift >= 0) shifts.  Integer
// division has no instruction on this chip; even for a workgroup-uniform value it expands to some fifteen
// vector instructions, and the tile arithmetic below had seven of them -- a fifth of the kernel's issue slots.
__device__ __forceinline__ int div_by(int x, int lam, int shift) { return shift >= 0 ? x >> shift : x / lam; }
__device__ __forceinline__ int shift_of(int lam) { return (lam & (lam - 1)) == 0 ? 31 - __builtin_clz(lam) : -1; }

template <int L1>
__device__ __forceinline__ TileGeom tile_geom(const MergeDesc& d, int n0, int k0, int sh2) {
    TileGeom g;
    int k1 = min(k0 + KT, d.d_in) - 1, n1 = min(n0 + NT, d.d_out) - 1;
    if constexpr (L1 > 0) { g.hrow0 = k0 / L1; g.hrows = k1 / L1 - g.hrow0 + 1; }
    else { g.hrow0 = k0 / d.lam1; g.hrows = k1 / d.lam1 - g.hrow0 + 1; }
    g.hcol0 = div_by(n0, d.lam2, sh2); g.hcols = div_by(n1, d.lam2, sh2) - g.hcol0 + 1;
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

// the two lanes of a block (lanes 2i, 2i+1) exchange values: minimum / maximum over the pair
__device__ __forceinline__ float pair_min(float v) {
    return fminf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, false)));
}
__device__ __forceinline__ float pair_max(float v) {
    return fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, false)));
}

// OUT16: write the shifted weights themselves as bf16 (the 16-bit merge) instead of requantizing them.
template <bool GROUPED, bool BETA, int L1, bool OUT16>
__device__ __forceinline__ void merge_requant_tile(const MergeDesc& d, const unsigned wg) {
    __shared__ float lut[16];
    extern __shared__ __align__(16) float dl[];          // deltas, [hcols][stride]
    const int t = threadIdx.x;
    // Workgroup -> tile.  Eight neighbouring k-tiles of a row tile touch the same 128-byte lines of the
    // scale arrays (4 blocks = 16 bytes per tile and row), in and out; workgroup id mod 8 is the XCD, so the
    // eight are given ids with equal id mod 8 (and consecutive id / 8): one L2 then sees whole lines instead
    // of eight L2s each fetching the line and writing back an eighth of it.  Ids past the ragged end of a
    // group of eight, or past the last group, have no tile.
    const int ktiles = (d.d_in + KT - 1) / KT, ntiles = (d.d_out + NT - 1) / NT;
    const int kgroups = (ktiles + 7) >> 3;
    const int xcd = wg & 7, seq = wg >> 3;
    const int group = (seq >> 3) * 8 + xcd;
    // group / kgroups by the host's reciprocal (exact for group < 2^24, kgroups < 2^8: the launcher checks)
    const int nt = kgroups == 1 ? group : (int)__umulhi((uint32_t)group, d.kgroups_magic);
    const int kt = (group - nt * kgroups) * 8 + (seq & 7);
    if (kt >= ktiles || nt >= ntiles) return;
    const int k0 = kt * KT, n0 = nt * NT;
    const int row = t >> 3, bk = (t >> 1) & 3, sub = t & 1;
    const int n = n0 + row, k = k0 + kBlock * bk + 32 * sub;
    const bool live = n < d.d_out && k < d.d_in;         // the same for the two lanes of a block
    const int bpr = d.d_in / kBlock;

    // this thread's half block: all global loads first
    uint4 cq = make_uint4(0, 0, 0, 0);
    float a = 0.f, b = 0.f;
    int64_t blk = 0;
    if (live) {
        blk = (int64_t)n * bpr + k / kBlock;
        cq = *reinterpret_cast<const uint4*>(d.codes + ((int64_t)n * d.d_in + k) / 2);
        if constexpr (GROUPED) {
            const int gs = shift_of(d.scale_group);
            const int64_t grp = gs >= 0 ? blk >> gs : blk / d.scale_group;
            a = __fmaf_rn(e4m3_to_float(d.scale_codes[blk]), d.scale_step[grp], d.scale_mid[grp]);   // = grouped_scale()
        } else {
            a = d.scales[blk];
        }
        if constexpr (BETA) b = d.beta[blk];
    }

    // stage the deltas of the tile: delta = (s*H)/lambda1, a division unless lambda1 is one of the
    // powers of two with a code path of their own, where multiplying by the (exact) reciprocal gives
    // the same bits
    const int sh2 = shift_of(d.lam2);
    const TileGeom g = tile_geom<L1>(d, n0, k0, sh2);
    const int ldH = div_by(d.d_out, d.lam2, sh2), stride = delta_stride<L1>(d.lam1);
    if (t < 16) lut[t] = d.cb.c[t];
    const float lam1f = (float)d.lam1;
    auto delta_of = [&](float h) __attribute__((always_inline)) {
        const float sh = __fmul_rn(d.s, h);
        if constexpr (L1 > 0) return __fmul_rn(sh, 1.0f / (float)L1);
        else return __fdiv_rn(sh, lam1f);
    };
    const int hc4 = g.hcols >> 2;
    if ((g.hcols & 3) == 0 && (hc4 & (hc4 - 1)) == 0 && (ldH & 3) == 0 && (g.hcol0 & 3) == 0 &&
        (reinterpret_cast<uintptr_t>(d.H) & 15) == 0) {
        // whole tiles of power-of-two lambdas: 16-byte loads along n, no division in the index
        const int sh = 31 - __builtin_clz(hc4);
        for (int idx = t; idx < g.hrows * hc4; idx += kMergeThreads) {
            const int r = idx >> sh, c = (idx & (hc4 - 1)) << 2;
            const float4 h = *reinterpret_cast<const float4*>(d.H + (int64_t)(g.hrow0 + r) * ldH + g.hcol0 + c);
            dl[delta_pos<L1>(c, r, stride)] = delta_of(h.x);
            dl[delta_pos<L1>(c + 1, r, stride)] = delta_of(h.y);
            dl[delta_pos<L1>(c + 2, r, stride)] = delta_of(h.z);
            dl[delta_pos<L1>(c + 3, r, stride)] = delta_of(h.w);
        }
    } else {
        for (int idx = t; idx < g.hrows * g.hcols; idx += kMergeThreads) {
            const int r = idx / g.hcols, c = idx - r * g.hcols;
            dl[delta_pos<L1>(c, r, stride)] = delta_of(d.H[(int64_t)(g.hrow0 + r) * ldH + g.hcol0 + c]);
        }
    }
    __syncthreads();
    if (!live) return;

    // w' = w~ + delta for the 32 elements of the half
    float w[32];
    const uint32_t cw[4] = {cq.x, cq.y, cq.z, cq.w};
    const int c = div_by(n, d.lam2, sh2) - g.hcol0;
    auto element = [&](int j, float de) __attribute__((always_inline)) {
        const float cv = lut[(cw[j >> 3] >> (4 * (j & 7))) & 15];
        const float wt = BETA ? __fmaf_rn(cv, a, b) : __fmul_rn(cv, a);
        w[j] = __fadd_rn(wt, de);
    };
    if constexpr (L1 > 0) {
        constexpr int RUN = 64 / L1, QR = 32 / L1;       // deltas per block / per half
        const float* dq = dl + c * stride + bk * (RUN + 4) + sub * QR;
        float de[QR];
#pragma unroll
        for (int v = 0; v < QR / 4; ++v) {
            const float4 x = *reinterpret_cast<const float4*>(dq + 4 * v);
            de[4 * v] = x.x; de[4 * v + 1] = x.y; de[4 * v + 2] = x.z; de[4 * v + 3] = x.w;
        }
#pragma unroll
        for (int j = 0; j < 32; ++j) element(j, de[j / L1]);
    } else {
        const float* drow = dl + c * stride - g.hrow0;
#pragma unroll
        for (int j = 0; j < 32; ++j) element(j, drow[(k + j) / d.lam1]);
    }
    if constexpr (OUT16) {
        uint4* wp = reinterpret_cast<uint4*>(d.w16_out + (int64_t)n * d.d_in + k);
#pragma unroll
        for (int v = 0; v < 4; ++v)
            wp[v] = make_uint4(pack_bf16(w[8 * v], w[8 * v + 1]), pack_bf16(w[8 * v + 2], w[8 * v + 3]),
                               pack_bf16(w[8 * v + 4], w[8 * v + 5]), pack_bf16(w[8 * v + 6], w[8 * v + 7]));
        return;
    }
    float lo = w[0], hi = w[0];
#pragma unroll
    for (int j = 1; j < 32; ++j) { lo = fminf(lo, w[j]); hi = fmaxf(hi, w[j]); }
    lo = pair_min(lo); hi = pair_max(hi);                // minimum and maximum are exact: any order

    // min-max INT4 of the block: one division for the scale, one for its reciprocal
    const float range = __fsub_rn(hi, lo);
    const float al = __fdiv_rn(range, 15.0f);
    const float inv = al != 0.0f ? __fdiv_rn(15.0f, range) : 0.0f;     // a flat block gets codes 0
    // (w-lo)*inv lies in [0, 15*(1+2^-23)], so rint() of it already lies in 0..15: adding 1.5*2^23
    // rounds to the nearest integer (ties to even) and leaves it in the low mantissa bits, above the
    // constant 0x4B400000.  Eight such words are summed with their nibble shifts (mod 2^32) and the
    // constants' sum, 0x4B400000 * 0x11111111 mod 2^32, is taken off once.
    constexpr uint32_t kMagicSum = (uint32_t)(0x4B400000ull * 0x11111111ull);
    uint32_t p[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const float q = __fadd_rn(__fmul_rn(__fsub_rn(w[j], lo), inv), 12582912.0f);
        p[j >> 3] += __float_as_uint(q) << (4 * (j & 7));
    }
    // written once and not read again here: a streaming store (measured 10 % off a 22016 x 8192 merge; on the
    // loads the same hint gains nothing or, where neighbouring tiles share lines of H, costs)
    const u32x4 pv = {p[0] - kMagicSum, p[1] - kMagicSum, p[2] - kMagicSum, p[3] - kMagicSum};
    __builtin_nontemporal_store(pv, reinterpret_cast<u32x4*>(d.codes_out + ((int64_t)n * d.d_in + k) / 2));
    if (sub == 0) {
        d.alpha_out[blk] = al;
        d.beta_out[blk] = lo;
    }
}

template <bool GROUPED, bool BETA, int L1, bool OUT16>
__global__ __launch_bounds__(kMergeThreads) void k_merge_requant(MergeDesc d) {
    merge_requant_tile<GROUPED, BETA, L1, OUT16>(d, blockIdx.x);
}

// Several weights in one launch (the projections of a layer): the workgroup ids of weight m start at first[m], a
// multiple of 64, so the id -> XCD pattern of the single launch is kept; between the weights there is no idle
// tail and no launch gap.
constexpr int kMergeBatchMax = 8;
struct MergeBatch {
    MergeDesc d[kMergeBatchMax];
    unsigned first[kMergeBatchMax + 1];
    int count;
};
template <bool GROUPED, bool BETA, int L1>
__global__ __launch_bounds__(kMergeThreads) void k_merge_requant_batch(MergeBatch b) {
    int m = 0;
#pragma unroll
    for (int i = 1; i < kMergeBatchMax; ++i)
        if (i < b.count && blockIdx.x >= b.first[i]) m = i;
    merge_requant_tile<GROUPED, BETA, L1, false>(b.d[m], blockIdx.x - b.first[m]);
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

// The same shift on 8 x 8 blocks (block (i, j): rows 8i.., inputs 8j.., index i*(d_in/8) + j); with 8 | lambda1
// and 8 | lambda2 the whole block sees one element of H, so the merged weight is exact (Alg. 2 get_new_beta).
__global__ __launch_bounds__(256) void k_merge_beta_shift_tile8(MergeDesc d) {
    const int bc = d.block_cols, nbc = d.d_in / bc;               // blocks of 8 rows x bc inputs
    const int64_t total = (int64_t)(d.d_out / 8) * nbc;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx / nbc), j = (int)(idx - (int64_t)i * nbc);
    const float h = d.H[(int64_t)((bc * j) / d.lam1) * (d.d_out / d.lam2) + (8 * i) / d.lam2];
    const float delta = __fdiv_rn(__fmul_rn(d.s, h), (float)d.lam1);
    d.beta_out[idx] = d.beta ? __fadd_rn(d.beta[idx], delta) : delta;
}

// Requantizing merge and 16-bit merge on 8 x 8 blocks (any lambdas; with 8 | lambda1 and 8 | lambda2 the offset
// shift above is the exact and cheaper way).  A thread owns one block: eight code dwords, one per row, the lanes
// of a wave along the block columns (256 contiguous bytes per row and load), its scale and offset; the shift of
// element (n, k) is read from H where it is (the 64 elements see at most (8/lambda1 + 1)(8/lambda2 + 1) entries,
// served by the cache).  Same arithmetic as on 64-blocks: fp32 w~ = fma(c, alpha, beta) or c * alpha, + delta,
// then the min-max quantizer of Eq. 1 over the block, or one rounding to bf16.
// BC = 4: blocks of 8 rows x 4 inputs (two code bytes per row).
template <bool BETA, bool OUT16, int BC>
__global__ __launch_bounds__(256) void k_merge_tile8(MergeDesc d) {
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = d.cb.c[threadIdx.x];
    __syncthreads();
    const int nbc = d.d_in / BC;
    const int64_t total = (int64_t)(d.d_out / 8) * nbc;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int bi = (int)(idx / nbc), bj = (int)(idx - (int64_t)bi * nbc);
    const int n0 = 8 * bi, k0 = BC * bj;
    const float a = d.scales[idx], b = BETA ? d.beta[idx] : 0.0f;
    const int ldH = d.d_out / d.lam2;
    const float lam1f = (float)d.lam1;
    float w[8][BC];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint8_t* cp = d.codes + ((int64_t)(n0 + i) * d.d_in + k0) / 2;
        const uint32_t cw = BC == 8 ? *reinterpret_cast<const uint32_t*>(cp) : (uint32_t)*reinterpret_cast<const uint16_t*>(cp);
        const float* hrow = d.H + (n0 + i) / d.lam2;
#pragma unroll
        for (int j = 0; j < BC; ++j) {
            const float cv = lut[(cw >> (4 * j)) & 15];
            const float wt = BETA ? __fmaf_rn(cv, a, b) : __fmul_rn(cv, a);
            const float delta = __fdiv_rn(__fmul_rn(d.s, hrow[(int64_t)((k0 + j) / d.lam1) * ldH]), lam1f);
            w[i][j] = __fadd_rn(wt, delta);
        }
    }
    if constexpr (OUT16) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            qblora_bf16* wp = d.w16_out + (int64_t)(n0 + i) * d.d_in + k0;
            if constexpr (BC == 8)
                *reinterpret_cast<uint4*>(wp) = make_uint4(pack_bf16(w[i][0], w[i][1]), pack_bf16(w[i][2], w[i][3]),
                                                           pack_bf16(w[i][4], w[i][5]), pack_bf16(w[i][6], w[i][7]));
            else
                *reinterpret_cast<uint2*>(wp) = make_uint2(pack_bf16(w[i][0], w[i][1]), pack_bf16(w[i][2], w[i][3]));
        }
        return;
    }
    float lo = w[0][0], hi = w[0][0];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < BC; ++j) { lo = fminf(lo, w[i][j]); hi = fmaxf(hi, w[i][j]); }
    const float range = __fsub_rn(hi, lo);
    const float al = __fdiv_rn(range, 15.0f);
    const float inv = al != 0.0f ? __fdiv_rn(15.0f, range) : 0.0f;     // a flat block gets codes 0
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t p = 0;
#pragma unroll
        for (int j = 0; j < BC; ++j) {
            // (w-lo)*inv lies in [0, 15*(1+2^-23)]: rint() of it is already a code
            const float q = rintf(__fmul_rn(__fsub_rn(w[i][j], lo), inv));
            p |= (uint32_t)q << (4 * j);
        }
        uint8_t* op = d.codes_out + ((int64_t)(n0 + i) * d.d_in + k0) / 2;
        if constexpr (BC == 8) *reinterpret_cast<uint32_t*>(op) = p;
        else *reinterpret_cast<uint16_t*>(op) = (uint16_t)p;
    }
    d.alpha_out[idx] = al;
    d.beta_out[idx] = lo;
}

}  // namespace

template <int L1, bool OUT16>
int launch_requant_l1(const MergeDesc& d, hipStream_t st) {
    const int hcols = NT / d.lam2 + 2;
    const size_t smem = sizeof(float) * (size_t)delta_stride<L1>(d.lam1) * hcols;
    // one id per (group of eight k-tiles, member), groups dealt round-robin to the eight XCDs
    const int64_t groups = (int64_t)(((d.d_in + KT - 1) / KT + 7) / 8) * ((d.d_out + NT - 1) / NT);
    const int64_t kgroups = ((d.d_in + KT - 1) / KT + 7) / 8;
    if (groups > (int64_t)1 << 24 || kgroups >= 256) return QBLORA_ERR_UNSUPPORTED;
    MergeDesc dd = d;
    dd.kgroups_magic = kgroups > 1 ? (uint32_t)((((uint64_t)1 << 32) / (uint64_t)kgroups) + 1) : 0u;
    dim3 grid((unsigned)(((groups + 7) / 8) * 64));
    auto launch = [&](auto kern) -> int {
        if (smem > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, grid, dim3(kMergeThreads), smem, st, dd);
        return launch_status();
    };
    if (d.scale_codes)
        return d.beta ? launch(k_merge_requant<true, true, L1, OUT16>) : launch(k_merge_requant<true, false, L1, OUT16>);
    return d.beta ? launch(k_merge_requant<false, true, L1, OUT16>) : launch(k_merge_requant<false, false, L1, OUT16>);
}

// workgroups of the requantizing launch for one weight (a multiple of 64) and its reciprocal; 0 when the shape
// is beyond the index arithmetic
unsigned requant_grid(const MergeDesc& d, uint32_t* magic) {
    const int64_t kgroups = ((d.d_in + KT - 1) / KT + 7) / 8;
    const int64_t groups = kgroups * ((d.d_out + NT - 1) / NT);
    if (groups > (int64_t)1 << 24 || kgroups >= 256) return 0;
    *magic = kgroups > 1 ? (uint32_t)((((uint64_t)1 << 32) / (uint64_t)kgroups) + 1) : 0u;
    return (unsigned)(((groups + 7) / 8) * 64);
}

template <int L1>
int launch_requant_batch_l1(const MergeDesc* ds, int count, hipStream_t st) {
    MergeBatch b{};
    b.count = count;
    unsigned total = 0;
    size_t smem = 0;
    for (int m = 0; m < count; ++m) {
        b.d[m] = ds[m];
        const unsigned g = requant_grid(ds[m], &b.d[m].kgroups_magic);
        if (g == 0) return QBLORA_ERR_UNSUPPORTED;
        b.first[m] = total;
        total += g;
        smem = sizeof(float) * (size_t)delta_stride<L1>(ds[m].lam1) * (NT / ds[m].lam2 + 2);
    }
    b.first[count] = total;
    auto launch = [&](auto kern) -> int {
        if (smem > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(total), dim3(kMergeThreads), smem, st, b);
        return launch_status();
    };
    if (ds[0].scale_codes)
        return ds[0].beta ? launch(k_merge_requant_batch<true, true, L1>) : launch(k_merge_requant_batch<true, false, L1>);
    return ds[0].beta ? launch(k_merge_requant_batch<false, true, L1>) : launch(k_merge_requant_batch<false, false, L1>);
}

// One launch for `count` (2 .. 8) row-segment weights that share lambdas, scale format and the presence of offsets;
// QBLORA_ERR_UNSUPPORTED (nothing launched) when they do not -- the caller then merges them one by one.
int launch_merge_requant_batch(const MergeDesc* ds, int count, hipStream_t st) {
    if (count < 2 || count > kMergeBatchMax) return QBLORA_ERR_UNSUPPORTED;
    for (int m = 0; m < count; ++m)
        if (ds[m].block_rows == 8 || ds[m].lam1 != ds[0].lam1 || ds[m].lam2 != ds[0].lam2 ||
            (ds[m].scale_codes == nullptr) != (ds[0].scale_codes == nullptr) || (ds[m].beta == nullptr) != (ds[0].beta == nullptr))
            return QBLORA_ERR_UNSUPPORTED;
    switch (ds[0].lam1) {
        case 1: return launch_requant_batch_l1<1>(ds, count, st);
        case 2: return launch_requant_batch_l1<2>(ds, count, st);
        case 4: return launch_requant_batch_l1<4>(ds, count, st);
        case 8: return launch_requant_batch_l1<8>(ds, count, st);
        default: return launch_requant_batch_l1<0>(ds, count, st);
    }
}

template <bool OUT16>
int launch_merge_elementwise(const MergeDesc& d, hipStream_t st) {
    if (d.block_rows == 8) {
        if (d.scale_codes || d.d_out % 8 != 0 || d.d_in % 8 != 0 || (d.block_cols != 8 && d.block_cols != 4))
            return QBLORA_ERR_UNSUPPORTED;
        const int64_t total = (int64_t)(d.d_out / 8) * (d.d_in / d.block_cols);
        const dim3 grid((unsigned)((total + 255) / 256));
        if (d.block_cols == 4) {
            if (d.beta) hipLaunchKernelGGL((k_merge_tile8<true, OUT16, 4>), grid, dim3(256), 0, st, d);
            else hipLaunchKernelGGL((k_merge_tile8<false, OUT16, 4>), grid, dim3(256), 0, st, d);
        } else {
            if (d.beta) hipLaunchKernelGGL((k_merge_tile8<true, OUT16, 8>), grid, dim3(256), 0, st, d);
            else hipLaunchKernelGGL((k_merge_tile8<false, OUT16, 8>), grid, dim3(256), 0, st, d);
        }
        return launch_status();
    }
    switch (d.lam1) {
        case 1: return launch_requant_l1<1, OUT16>(d, st);
        case 2: return launch_requant_l1<2, OUT16>(d, st);
        case 4: return launch_requant_l1<4, OUT16>(d, st);
        case 8: return launch_requant_l1<8, OUT16>(d, st);
        default: return launch_requant_l1<0, OUT16>(d, st);
    }
}

int launch_merge_requant(const MergeDesc& d, hipStream_t st) { return launch_merge_elementwise<false>(d, st); }
int launch_merge_bf16(const MergeDesc& d, hipStream_t st) { return launch_merge_elementwise<true>(d, st); }

int launch_merge_beta_shift(const MergeDesc& d, hipStream_t st) {
    int64_t total = d.block_rows == 8 ? (int64_t)(d.d_out / 8) * (d.d_in / d.block_cols) : (int64_t)d.d_out * (d.d_in / kBlock);
    unsigned grid = (unsigned)((total + 255) / 256);
    if (d.block_rows == 8) {
        hipLaunchKernelGGL(k_merge_beta_shift_tile8, dim3(grid), dim3(256), 0, st, d);
        return launch_status();
    }
    if (d.scale_codes) hipLaunchKernelGGL(k_merge_beta_shift<true>, dim3(grid), dim3(256), 0, st, d);
    else hipLaunchKernelGGL(k_merge_beta_shift<false>, dim3(grid), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
