// Block-wise quantizers and the standalone dequantizer (Eq. 1, Sec. 3.1) for gfx950.
//
// Both quantizers are HBM-streaming kernels: a thread owns 16 consecutive fp32 weights (four
// 16-byte loads), 4 lanes own one 64-wide block and reduce its absmax / min / max with
// cross-lane swaps; the codes of a workgroup are gathered in LDS and stored 16 bytes per
// thread.  All decision
// arithmetic is written with explicit single-rounding intrinsics so that no FMA contraction
// can change a code.
#include "common.h"

namespace qblora {

namespace {

struct Midpoints {
    float m[15];   // (c_j + c_{j+1}) * 0.5 in fp32, computed on the host
};

// All-reduce over the 4 lanes of a quad (one block held as 4 x 16 weights): two DPP quad permutations and
// combines leave the result in every lane; DPP keeps this in the vector ALU (the generic lane shuffle would go
// through the LDS crossbar).
template <int PERM>
__device__ __forceinline__ float quad_swap(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), PERM, 0xf, 0xf, false));
}
__device__ __forceinline__ float quad_max(float v) {
    v = fmaxf(v, quad_swap<0xB1>(v));
    return fmaxf(v, quad_swap<0x4E>(v));
}
__device__ __forceinline__ float quad_min(float v) {
    v = fminf(v, quad_swap<0xB1>(v));
    return fminf(v, quad_swap<0x4E>(v));
}

// Four codes of one float4 against the block's absmax a: code = #{ j : w > t_j } with t_j = m_j * a.
// Rounding is monotone, so the t_j ascend (weakly) and the count is found by bisection: four comparisons
// per weight against thresholds selected by the earlier outcomes, instead of fifteen.
__device__ __forceinline__ uint32_t codes4_codebook(const float4& w, float a, const Midpoints& mp) {
    const float t0 = __fmul_rn(mp.m[0], a), t1 = __fmul_rn(mp.m[1], a), t2 = __fmul_rn(mp.m[2], a),
                t3 = __fmul_rn(mp.m[3], a), t4 = __fmul_rn(mp.m[4], a), t5 = __fmul_rn(mp.m[5], a),
                t6 = __fmul_rn(mp.m[6], a), t7 = __fmul_rn(mp.m[7], a), t8 = __fmul_rn(mp.m[8], a),
                t9 = __fmul_rn(mp.m[9], a), t10 = __fmul_rn(mp.m[10], a), t11 = __fmul_rn(mp.m[11], a),
                t12 = __fmul_rn(mp.m[12], a), t13 = __fmul_rn(mp.m[13], a), t14 = __fmul_rn(mp.m[14], a);
    auto code_of = [&](float x) -> uint32_t {
        const bool b3 = x > t7;
        const float u2 = b3 ? t11 : t3;
        const bool b2 = x > u2;
        const float u1lo = b2 ? t5 : t1, u1hi = b2 ? t13 : t9;
        const bool b1 = x > (b3 ? u1hi : u1lo);
        const float q0 = b1 ? t2 : t0, q1 = b1 ? t6 : t4, q2 = b1 ? t10 : t8, q3 = b1 ? t14 : t12;
        const float u0lo = b2 ? q1 : q0, u0hi = b2 ? q3 : q2;
        const bool b0 = x > (b3 ? u0hi : u0lo);
        return (b3 ? 8u : 0u) + (b2 ? 4u : 0u) + (b1 ? 2u : 0u) + (b0 ? 1u : 0u);
    };
    const uint32_t c0 = code_of(w.x), c1 = code_of(w.y), c2 = code_of(w.z), c3 = code_of(w.w);
    return c0 | (c1 << 4) | (c2 << 8) | (c3 << 12);
}

// The same bisection with the thresholds of the lower three levels in LDS instead of registers: choosing a
// register by the earlier outcomes takes 1 + 3 + 7 select instructions per weight, and with the compares
// and the assembly of the code the register form spends 24 vector instructions per weight, which makes the
// kernel issue-bound, not HBM-bound.  Here a level is: one LDS read at (base + 4 * path), one compare, one
// add-with-carry that appends the outcome to the path (path = 2 * path + (x > t)); after four levels the path
// is the code.  Level l of a block's tree is an array of 2^(l-1) thresholds, [t3, t11], [t1, t5, t9, t13],
// [t0, t2, ..., t14]; the root t7 stays in a register.
// Level arrays of the 16 blocks of a wave side by side: [block][position], so that the 16 quads of a wave read
// different banks on levels 2 and 3 (32 and 64 words) and each half-wave does on level 4 (128 words).
struct WaveTrees {
    float2 l2[16]; float4 l3[16]; float4 l4[16][2];
};
__device__ __forceinline__ void append_gt(uint32_t& path, float x, float t) {
    asm("v_cmp_gt_f32_e32 vcc, %1, %2\n\tv_addc_co_u32_e32 %0, vcc, %0, %0, vcc" : "+v"(path) : "v"(x), "v"(t) : "vcc");
}
struct BlockTree {                       // the three level arrays of one block
    const float* l2; const float* l3; const float* l4;
};
__device__ __forceinline__ uint32_t code_by_tree(float x, float t7, const BlockTree& tree) {
    uint32_t path = x > t7 ? 1u : 0u;
    append_gt(path, x, tree.l2[path]);
    append_gt(path, x, tree.l3[path]);
    append_gt(path, x, tree.l4[path]);
    return path;
}
// thresholds t_j = m_j * a of block j into the wave's trees (every lane of the block writes the same values);
// returns t7
__device__ __forceinline__ float build_tree(WaveTrees& w, int j, float a, const Midpoints& mp, BlockTree& tree) {
    auto t = [&](int i) { return __fmul_rn(mp.m[i], a); };
    w.l2[j] = make_float2(t(3), t(11));
    w.l3[j] = make_float4(t(1), t(5), t(9), t(13));
    w.l4[j][0] = make_float4(t(0), t(2), t(4), t(6));
    w.l4[j][1] = make_float4(t(8), t(10), t(12), t(14));
    tree.l2 = reinterpret_cast<const float*>(&w.l2[j]);
    tree.l3 = reinterpret_cast<const float*>(&w.l3[j]);
    tree.l4 = reinterpret_cast<const float*>(&w.l4[j][0]);
    return t(7);
}
__device__ __forceinline__ uint32_t codes4_by_tree(const float4& w, float t7, const BlockTree& tree) {
    const uint32_t c0 = code_by_tree(w.x, t7, tree), c1 = code_by_tree(w.y, t7, tree), c2 = code_by_tree(w.z, t7, tree),
                   c3 = code_by_tree(w.w, t7, tree);
    return c0 | (c1 << 4) | (c2 << 8) | (c3 << 12);
}

// Four min-max codes of one float4 given the block's extremes; also returns alpha = (hi-lo)/15.
__device__ __forceinline__ uint32_t codes4_minmax(const float4& w, float lo, float hi, float& al) {
    const float range = __fsub_rn(hi, lo);
    al = __fdiv_rn(range, 15.0f);
    uint32_t packed = 0;
    if (al != 0.0f) {
        const float inv = __fdiv_rn(15.0f, range);
        float q0 = rintf(__fmul_rn(__fsub_rn(w.x, lo), inv));
        float q1 = rintf(__fmul_rn(__fsub_rn(w.y, lo), inv));
        float q2 = rintf(__fmul_rn(__fsub_rn(w.z, lo), inv));
        float q3 = rintf(__fmul_rn(__fsub_rn(w.w, lo), inv));
        q0 = fminf(fmaxf(q0, 0.0f), 15.0f);
        q1 = fminf(fmaxf(q1, 0.0f), 15.0f);
        q2 = fminf(fmaxf(q2, 0.0f), 15.0f);
        q3 = fminf(fmaxf(q3, 0.0f), 15.0f);
        packed = (uint32_t)q0 | ((uint32_t)q1 << 4) | ((uint32_t)q2 << 8) | ((uint32_t)q3 << 12);
    }
    return packed;
}

// Work split of both quantizers: a workgroup owns 4 consecutive weight rows x 16 consecutive 64-blocks
// (4 x 4 KB of contiguous fp32 input), wave u row u; a thread owns a quarter block (16 consecutive
// weights), so the four lanes of a quad hold one block.  Codes (8 bytes per thread) and block scales are
// collected in LDS and leave as 16-byte stores: 512 contiguous bytes per row in the canonical layout,
// and -- because the 4 rows are neighbours inside one 256-row tile -- 128 contiguous bytes per block
// column in the tile-ordered copy.
constexpr int kQRows = 4, kQBlocks = 16;

struct QuantTile {
    int row0, blk0, jt;
};

// grid: x = tile along the row (fastest, as consecutive workgroups should read consecutive memory), y and z = row
// tile (two dimensions only because one is limited to 65535) -- no division by a run-time count in the kernel
constexpr int kQGridY = 32768;
__device__ __forceinline__ QuantTile quant_tile() {
    QuantTile q;
    q.jt = blockIdx.x;
    q.row0 = ((int)blockIdx.z * kQGridY + (int)blockIdx.y) * kQRows;     // rows past the end are handled by the callers
    q.blk0 = q.jt * kQBlocks;
    return q;
}
inline dim3 quant_grid(int d_out, int bpr) {
    const int row_tiles = (d_out + kQRows - 1) / kQRows;
    return dim3((unsigned)((bpr + kQBlocks - 1) / kQBlocks), (unsigned)(row_tiles < kQGridY ? row_tiles : kQGridY),
                (unsigned)((row_tiles + kQGridY - 1) / kQGridY));
}

// 16 bytes of codes from LDS to global memory with the streaming hint: written once, read by a later launch (5 %
// off a 22016 x 8192 quantization; the same hint on the loads of W costs 30 %)
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__device__ __forceinline__ void stream16(uint8_t* dst, const void* lds_src) {
    __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(lds_src), reinterpret_cast<u32x4*>(dst));
}

// codes of the tile from LDS (cs[u][g] = 4 codes of float4 group g of row u) to both global layouts
__device__ __forceinline__ void store_tile_codes(const uint16_t (&cs)[kQRows][256], const QuantTile& q, int d_out, int bpr,
                                                 uint8_t* __restrict__ codes, uint8_t* __restrict__ tiled) {
    const int t = threadIdx.x;
    if (t < 128) {
        const int u = t >> 5, piece = t & 31;                 // 16-byte piece of the row's 512 bytes
        const int row = q.row0 + u, blk = q.blk0 + (piece >> 1);
        if (row < d_out && blk < bpr)
            stream16(codes + ((int64_t)row * bpr + blk) * 32 + (piece & 1) * 16, &cs[u][piece * 8]);
    } else if (tiled) {
        const int tt = t - 128, b = tt >> 3, u = (tt >> 1) & 3, half = tt & 1;
        const int row = q.row0 + u, blk = q.blk0 + b;
        if (row < d_out && blk < bpr)
            stream16(tiled + tiled_run_offset(row, blk, bpr) + half * 16, &cs[u][b * 16 + half * 8]);
    }
}

// Absmax / codebook quantizer.  Wave u of the workgroup takes row u of the tile; a thread owns 16
// consecutive weights (a quarter block, four 16-byte loads), so the 15 thresholds of its block are
// computed once per thread and the block reduction is two quad swaps.
__global__ __launch_bounds__(256) void k_quantize_codebook(const float4* __restrict__ W, int d_out, int bpr,
                                                           Midpoints mp, uint8_t* __restrict__ codes,
                                                           uint8_t* __restrict__ tiled, float* __restrict__ absmax) {
    __shared__ __align__(16) uint16_t cs[kQRows][256];
    __shared__ float as[kQRows][kQBlocks];
    __shared__ __align__(16) WaveTrees trees[kQRows];
    const QuantTile q = quant_tile();
    const int t = threadIdx.x, u = t >> 6, lane = t & 63, j = lane >> 2;
    const int row = q.row0 + u;
    // Lanes outside the matrix read the first block instead: their results are never stored, and the four
    // lanes of a block are inside or outside together.
    const bool ok = row < d_out && q.blk0 + j < bpr;
    const float4* src = W + (ok ? ((int64_t)row * bpr + q.blk0) * 16 + lane * 4 : (lane & 3) * 4);
    float4 wv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) wv[i] = src[i];
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        a = fmaxf(a, fmaxf(fmaxf(fabsf(wv[i].x), fabsf(wv[i].y)), fmaxf(fabsf(wv[i].z), fabsf(wv[i].w))));
    a = quad_max(a);
    // the block's tree is written and read by the lanes of its own quad only: DS operations of a wave execute in
    // order, so no barrier stands between the build and the look-ups
    BlockTree tree;
    const float t7 = build_tree(trees[u], j, a, mp, tree);
    uint32_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = codes4_by_tree(wv[i], t7, tree);
    *reinterpret_cast<uint2*>(&cs[u][lane * 4]) = make_uint2(c[0] | (c[1] << 16), c[2] | (c[3] << 16));
    if ((lane & 3) == 0) as[u][j] = a;
    __syncthreads();
    store_tile_codes(cs, q, d_out, bpr, codes, tiled);
    if (t < kQRows * kQBlocks) {
        const int r = q.row0 + (t >> 4), blk = q.blk0 + (t & 15);
        if (r < d_out && blk < bpr) absmax[(int64_t)r * bpr + blk] = as[t >> 4][t & 15];
    }
}

// Min-max INT4 quantizer: alpha = (hi-lo)/15, beta = lo, code = rint((w-lo) * (15/(hi-lo))).  Same work
// split as the codebook quantizer.
__global__ __launch_bounds__(256) void k_quantize_minmax(const float4* __restrict__ W, int d_out, int bpr,
                                                         uint8_t* __restrict__ codes, uint8_t* __restrict__ tiled,
                                                         float* __restrict__ alpha, float* __restrict__ beta) {
    __shared__ __align__(16) uint16_t cs[kQRows][256];
    __shared__ float as[kQRows][kQBlocks], bs[kQRows][kQBlocks];
    const QuantTile q = quant_tile();
    const int t = threadIdx.x, u = t >> 6, lane = t & 63, j = lane >> 2;
    const int row = q.row0 + u;
    const bool ok = row < d_out && q.blk0 + j < bpr;         // lanes outside the matrix read the first block
    const float4* src = W + (ok ? ((int64_t)row * bpr + q.blk0) * 16 + lane * 4 : (lane & 3) * 4);
    float4 wv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) wv[i] = src[i];
    float lo = wv[0].x, hi = wv[0].x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        lo = fminf(lo, fminf(fminf(wv[i].x, wv[i].y), fminf(wv[i].z, wv[i].w)));
        hi = fmaxf(hi, fmaxf(fmaxf(wv[i].x, wv[i].y), fmaxf(wv[i].z, wv[i].w)));
    }
    lo = quad_min(lo);
    hi = quad_max(hi);
    float al = 0.0f;
    uint32_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = codes4_minmax(wv[i], lo, hi, al);
    *reinterpret_cast<uint2*>(&cs[u][lane * 4]) = make_uint2(c[0] | (c[1] << 16), c[2] | (c[3] << 16));
    if ((lane & 3) == 0) { as[u][j] = al; bs[u][j] = lo; }
    __syncthreads();
    store_tile_codes(cs, q, d_out, bpr, codes, tiled);
    if (t < kQRows * kQBlocks) {
        const int r = q.row0 + (t >> 4), blk = q.blk0 + (t & 15);
        if (r < d_out && blk < bpr) {
            alpha[(int64_t)r * bpr + blk] = as[t >> 4][t & 15];
            beta[(int64_t)r * bpr + blk] = bs[t >> 4][t & 15];
        }
    }
}

// Both quantizers on 8 x 8 blocks (the two-dimensional block shapes of Sec. 3.3): a block is 8 output
// rows x 8 inputs, scale index (n/8)*(d_in/8) + k/8.  A workgroup owns 8 rows x 512 inputs = 64 blocks; the
// four lanes of a quad hold block t/4, lane q of the quad its rows 2q and 2q+1 (two 16-byte loads each), so
// a wave reads 512 contiguous bytes of each of the 8 rows and the block reduction is two quad swaps.
// Codes go through LDS as [row][256 bytes] and leave 16 bytes per thread in both layouts.
// BC: inputs per block, 8 (8 x 8) or 4 (blocks of 8 rows x 4 inputs, block size 32: the other shape Sec. 3.3
// names).  With BC = 4 a lane's eight inputs of a row are two blocks: wv[0], wv[2] (inputs 0..3 of its two rows) belong
// to the left one, wv[1], wv[3] to the right one, each reduced over the quad on its own.
template <bool MINMAX, int BC>
__global__ __launch_bounds__(256) void k_quantize_tile8(const float4* __restrict__ W, int d_out, int d_in, Midpoints mp,
                                                        uint8_t* __restrict__ codes, uint8_t* __restrict__ tiled,
                                                        float* __restrict__ alpha, float* __restrict__ beta) {
    constexpr int NB = 8 / BC;                                     // blocks per lane and row: 1 or 2
    __shared__ __align__(16) uint8_t cs[8][256];
    __shared__ float as[64 * NB], bs[64 * NB];
    const int ntj = (d_in + 511) / 512;
    const int jt = blockIdx.x % ntj, row0 = (blockIdx.x / ntj) * 8, col0 = jt * 512;
    const int t = threadIdx.x, j = t >> 2, q = t & 3;              // block of the workgroup, lane of its quad
    const int col = col0 + 8 * j;
    // d_out % 8 == 0: whole blocks are in or out; a block outside the matrix reads block (0, 0) instead and
    // its results are never stored
    const bool ok = col < d_in && row0 < d_out;
    const int rbase = ok ? row0 : 0, cbase = ok ? col : 0;
    float4 wv[4];                                                  // [2*rr + c]: row 2q+rr, inputs 4c .. 4c+3
#pragma unroll
    for (int i = 0; i < 4; ++i) wv[i] = W[((int64_t)(rbase + 2 * q + (i >> 1)) * d_in + cbase + 4 * (i & 1)) >> 2];
    uint32_t c[4];
#pragma unroll
    for (int h = 0; h < NB; ++h) {                                 // h: the lane's block (BC = 4: left, right)
        if constexpr (MINMAX) {
            float lo = wv[h].x, hi = wv[h].x;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (NB == 2 && (i & 1) != h) continue;
                lo = fminf(lo, fminf(fminf(wv[i].x, wv[i].y), fminf(wv[i].z, wv[i].w)));
                hi = fmaxf(hi, fmaxf(fmaxf(wv[i].x, wv[i].y), fmaxf(wv[i].z, wv[i].w)));
            }
            lo = quad_min(lo);
            hi = quad_max(hi);
            float al = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (NB == 1 || (i & 1) == h) c[i] = codes4_minmax(wv[i], lo, hi, al);
            if (q == 0) { as[NB * j + h] = al; bs[NB * j + h] = lo; }
        } else {
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (NB == 2 && (i & 1) != h) continue;
                a = fmaxf(a, fmaxf(fmaxf(fabsf(wv[i].x), fabsf(wv[i].y)), fmaxf(fabsf(wv[i].z), fabsf(wv[i].w))));
            }
            a = quad_max(a);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (NB == 1 || (i & 1) == h) c[i] = codes4_codebook(wv[i], a, mp);
            if (q == 0) as[NB * j + h] = a;
        }
    }
    *reinterpret_cast<uint32_t*>(&cs[2 * q][4 * j]) = c[0] | (c[1] << 16);
    *reinterpret_cast<uint32_t*>(&cs[2 * q + 1][4 * j]) = c[2] | (c[3] << 16);
    __syncthreads();
    const int bpr64 = d_in / kBlock;
    if (t < 128) {
        const int r = t >> 4, piece = t & 15;                // 16-byte piece of the row's 256 bytes (32 inputs)
        if (row0 + r < d_out && col0 + 32 * piece < d_in)
            stream16(codes + ((int64_t)(row0 + r) * d_in + col0) / 2 + 16 * piece, &cs[r][16 * piece]);
    } else if (tiled) {
        const int tt = t - 128, ks = tt >> 4, r = (tt >> 1) & 7, half = tt & 1;   // 64-wide input step of the tile copy
        if (row0 + r < d_out && col0 + 64 * ks < d_in)
            stream16(tiled + tiled_run_offset(row0 + r, col0 / 64 + ks, bpr64) + half * 16, &cs[r][32 * ks + 16 * half]);
    }
    if (t < 64 * NB && col0 + BC * t < d_in && row0 < d_out) {
        const int64_t blk = (int64_t)(row0 / 8) * (d_in / BC) + col0 / BC + t;
        alpha[blk] = as[t];
        if constexpr (MINMAX) beta[blk] = bs[t];
    }
}

// fp32 magnitude -> E4M3 magnitude bits (7 bits), round to nearest even, saturating at 448.
__device__ __forceinline__ uint32_t e4m3_encode_mag(float a) {
    if (a < 0x1p-6f) return (uint32_t)rintf(a * 512.0f);          // subnormal grid 2^-9 (8 -> smallest normal)
    uint32_t u = __float_as_uint(a);
    u += 0x7ffffu + ((u >> 20) & 1u);                              // RNE to 3 mantissa bits, carry into exponent
    uint32_t code = (u >> 20) - (120u << 3);
    return code > 0x7eu ? 0x7eu : code;
}

// One workgroup of 256 threads per group of up to 256 consecutive scales.
__global__ __launch_bounds__(256) void k_scales_double_quantize(const float* __restrict__ scales, int64_t n,
                                                                int group, uint8_t* __restrict__ scale_codes,
                                                                float* __restrict__ step,
                                                                float* __restrict__ mid) {
    __shared__ float s_lo[256], s_hi[256];
    int64_t base = (int64_t)blockIdx.x * group;
    int cnt = (int)((n - base) < group ? (n - base) : group);
    int t = threadIdx.x;
    float lo = INFINITY, hi = -INFINITY;
    for (int i = t; i < cnt; i += 256) {
        float v = scales[base + i];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    s_lo[t] = lo; s_hi[t] = hi;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (t < o) { s_lo[t] = fminf(s_lo[t], s_lo[t + o]); s_hi[t] = fmaxf(s_hi[t], s_hi[t + o]); }
        __syncthreads();
    }
    float m = __fmul_rn(__fadd_rn(s_lo[0], s_hi[0]), 0.5f);
    __syncthreads();
    float dmax = 0.0f;
    for (int i = t; i < cnt; i += 256) dmax = fmaxf(dmax, fabsf(__fsub_rn(scales[base + i], m)));
    s_hi[t] = dmax;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (t < o) s_hi[t] = fmaxf(s_hi[t], s_hi[t + o]);
        __syncthreads();
    }
    dmax = s_hi[0];
    float st = dmax == 0.0f ? 0.0f : __fdiv_rn(dmax, 448.0f);
    if (t == 0) { step[blockIdx.x] = st; mid[blockIdx.x] = m; }
    for (int i = t; i < cnt; i += 256) {
        uint32_t code = 0;
        if (dmax != 0.0f) {
            float q = __fdiv_rn(__fsub_rn(scales[base + i], m), st);
            code = e4m3_encode_mag(fabsf(q)) | (signbit(q) ? 0x80u : 0u);
        }
        scale_codes[base + i] = (uint8_t)code;
    }
}

__global__ __launch_bounds__(256) void k_scales_reconstruct(const uint8_t* __restrict__ scale_codes,
                                                            const float* __restrict__ step,
                                                            const float* __restrict__ mid, int64_t n, int group,
                                                            float* __restrict__ scales) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) scales[i] = grouped_scale(scale_codes, step, mid, i, group);
}

// Standalone dequantize: thread = 8 consecutive k (one dword of codes) -> 8 bf16 (16 bytes).
__global__ __launch_bounds__(256) void k_dequantize_bf16(const uint32_t* __restrict__ codes32,
                                                         const float* __restrict__ scales,
                                                         const float* __restrict__ beta, Codebook cb,
                                                         int64_t n_words, int words_per_row, int block_cols,
                                                         uint4* __restrict__ out) {
    __shared__ float lut[16];
    if (threadIdx.x < 16) lut[threadIdx.x] = cb.c[threadIdx.x];
    __syncthreads();
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_words) return;
    uint32_t w = codes32[i];
    int64_t blk = i >> 3, blk2 = blk;    // 8 words of 8 codes per 64-block
    if (words_per_row > 0) { // blocks of 8 rows: a word is one row of block (n/8, word in row), or of two blocks of 4 inputs
        const int64_t n = i / words_per_row, wd = i - n * words_per_row;
        blk = blk2 = (n >> 3) * words_per_row + wd;
        if (block_cols == 4) { blk = (n >> 3) * (2 * (int64_t)words_per_row) + 2 * wd; blk2 = blk + 1; }
    }
    const float a = scales[blk], a2 = scales[blk2];
    float v[8];
    if (beta) {
        const float b = beta[blk], b2 = beta[blk2];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __fmaf_rn(lut[(w >> (4 * j)) & 15], j < 4 ? a : a2, j < 4 ? b : b2);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __fmul_rn(lut[(w >> (4 * j)) & 15], j < 4 ? a : a2);
    }
    uint4 o;
    o.x = pack_bf16(v[0], v[1]); o.y = pack_bf16(v[2], v[3]);
    o.z = pack_bf16(v[4], v[5]); o.w = pack_bf16(v[6], v[7]);
    out[i] = o;
}

// The bf16 compute weight in MFMA operand order (see launch_dequantize_operand): the weight itself.
// A workgroup owns 64 stored rows x 128 inputs.  A thread dequantizes 32 inputs of one stored row (16 bytes of
// codes; four lanes read 64 contiguous bytes of a row) into four 16-byte chunks of an LDS tile [n][16 chunks], chunk
// c of row n at position c ^ (n & 15); operand order only regroups whole chunks -- lane l = r + 32*hi of the k slice
// j takes chunk 2j + hi of row r -- so each wave reads its pieces back with 16-byte LDS loads (16 consecutive rows of
// one chunk lie in 16 different positions) and stores 1 KB per instruction, 4 KB contiguous per wave.  (The first form
// let a lane load the 32 code bytes of its row's block, twice per row: both lanes of a row need every other dword;
// it streamed at 0.60 of the HBM peak.)
// BETA: offsets present; GEOM: 0 = 64-blocks, 1 = 8 x 8 blocks, 2 = blocks of 8 rows x 4 inputs -- compile-time, so that
// a launch carries neither the other geometries' loads nor both of multiply and multiply-add with a select per weight
// (380 -> 230 vector instructions per thread).
template <bool BETA, int GEOM>
__global__ __launch_bounds__(256) void k_dequantize_operand(const uint8_t* __restrict__ codes,
                                                            const float* __restrict__ scales,
                                                            const float* __restrict__ beta, Codebook cb,
                                                            int d_out, int d_in,
                                                            uint4* __restrict__ out) {
    constexpr int block_rows = GEOM == 0 ? 1 : 8, block_cols = GEOM == 2 ? 4 : 8;
    __shared__ float lut[16];
    __shared__ __align__(16) uint4 tile[64][16];                // [n][chunk of 8 k], positions swizzled
    const int t = threadIdx.x;
    if (t < 16) lut[t] = cb.c[t];
    __syncthreads();
    const int n_tiles = (d_out + 63) / 64;                      // d_out is a multiple of 32 here
    const int kt = blockIdx.x / n_tiles;                        // 128 inputs
    const int nt = blockIdx.x % n_tiles;                        // 64 stored rows
    {
        const int row = t >> 2, piece = t & 3;                  // stored row in tile, 32 inputs
        const int64_t n = min((int64_t)nt * 64 + row, (int64_t)d_out - 1);    // rows past the end: computed, never stored
        const int k0 = kt * 128 + piece * 32;
        uint4 cq = make_uint4(0, 0, 0, 0);
        float a1 = 0.0f, b1 = 0.0f;
        float4 a4 = make_float4(0.f, 0.f, 0.f, 0.f), b4 = make_float4(0.f, 0.f, 0.f, 0.f), a4b = a4, b4b = b4;
        if (k0 < d_in) {                                        // d_in % 64 == 0: the last tile may be half
            cq = *reinterpret_cast<const uint4*>(codes + n * (d_in / 2) + k0 / 2);
            if constexpr (block_rows == 8 && block_cols == 4) {  // eight block columns of 4 inputs
                const int64_t blk = (n >> 3) * (int64_t)(d_in / 4) + k0 / 4;
                a4 = *reinterpret_cast<const float4*>(scales + blk);
                a4b = *reinterpret_cast<const float4*>(scales + blk + 4);
                if constexpr (BETA) { b4 = *reinterpret_cast<const float4*>(beta + blk); b4b = *reinterpret_cast<const float4*>(beta + blk + 4); }
            } else if constexpr (block_rows == 8) {              // four block columns of 8 inputs
                const int64_t blk = (n >> 3) * (int64_t)(d_in / 8) + k0 / 8;
                a4 = *reinterpret_cast<const float4*>(scales + blk);
                if constexpr (BETA) b4 = *reinterpret_cast<const float4*>(beta + blk);
            } else {
                const int64_t blk = n * (int64_t)(d_in / kBlock) + k0 / kBlock;
                a1 = scales[blk];
                if constexpr (BETA) b1 = beta[blk];
            }
        }
        const uint32_t cw[4] = {cq.x, cq.y, cq.z, cq.w};
        const float as[8] = {a4.x, a4.y, a4.z, a4.w, a4b.x, a4b.y, a4b.z, a4b.w};
        const float bs[8] = {b4.x, b4.y, b4.z, b4.w, b4b.x, b4b.y, b4b.z, b4b.w};
        constexpr bool half = block_rows == 8 && block_cols == 4;   // two blocks per chunk of 8 inputs
#pragma unroll
        for (int c = 0; c < 4; ++c) {                           // chunk 4*piece + c: 8 inputs
            const float a = half ? as[2 * c] : block_rows == 8 ? as[c] : a1, be = half ? bs[2 * c] : block_rows == 8 ? bs[c] : b1;
            const float a_hi = half ? as[2 * c + 1] : a, be_hi = half ? bs[2 * c + 1] : be;    // inputs 4 .. 7 of the chunk
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float cv = lut[(cw[c] >> (4 * j)) & 15];
                v[j] = BETA ? __fmaf_rn(cv, j < 4 ? a : a_hi, j < 4 ? be : be_hi) : __fmul_rn(cv, j < 4 ? a : a_hi);
            }
            tile[row][(4 * piece + c) ^ (row & 15)] =
                make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
        }
    }
    __syncthreads();
    {
        const int w = t >> 6, lane = t & 63, r = lane & 31, hi = lane >> 5;
        const int rb = w >> 1;                                  // 32-row block of the tile
        const int64_t nb = (int64_t)nt * 2 + rb;                // 32-row block of the weight
        if (nb * 32 < d_out) {
            const int64_t kb_count = d_in / 16;                 // 16-wide k slices of a row block
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = (w & 1) * 4 + q;                  // slice inside the tile
                const int64_t js = (int64_t)kt * 8 + j;
                const int row = rb * 32 + r;
                const uint4 o = tile[row][(2 * j + hi) ^ (row & 15)];
                if (js < kb_count) out[(nb * kb_count + js) * 64 + lane] = o;
            }
        }
    }
}

// The same for the transposed weight (operand rows = inputs k, contraction = stored rows n), which the
// backward contraction reads.  A workgroup owns 64 stored rows x 128 inputs.  A thread dequantizes 32 inputs of
// one stored row (16 bytes of codes; four lanes read 64 contiguous bytes of a row) and writes them as four
// 16-byte chunks into an LDS tile in the stored orientation, [n][128 k] with 256-byte rows; the transposition is
// left to the transposing LDS read ds_read_b64_tr_b16 (a group of 16 lanes that points at 4 rows x 16 columns
// gets, lane i, column i of the four rows): two of them give a lane the 8 consecutive n of its k that the
// operand order wants.  Logical chunk c of row n sits at chunk position c ^ ((n & 3) << 2), so that the four
// rows of a transposing read lie in different banks.  Each wave then stores 1 KB pieces (lane l = r + 32*hi
// holds k = r, n = 16q + 8hi .. + 7).  (The first form read 4 bytes of codes per thread and wrote 2-byte elements
// into a [k][n] tile: 57 % of its LDS cycles were bank conflicts and it streamed at 0.49 of the HBM peak.)
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
template <bool BETA, int GEOM>
__global__ __launch_bounds__(256) void k_dequantize_operand_t(const uint8_t* __restrict__ codes,
                                                              const float* __restrict__ scales,
                                                              const float* __restrict__ beta, Codebook cb,
                                                              int d_out, int d_in,
                                                              uint4* __restrict__ out) {
    constexpr int block_rows = GEOM == 0 ? 1 : 8, block_cols = GEOM == 2 ? 4 : 8;
    __shared__ float lut[16];
    __shared__ __align__(16) unsigned char tile[64 * 256];      // [n][128 k] bf16, chunks swizzled
    const int t = threadIdx.x;
    if (t < 16) lut[t] = cb.c[t];
    __syncthreads();
    const int n_tiles = d_out / 64;                             // d_out is a multiple of 64 here
    const int kt = blockIdx.x / n_tiles;                        // 128 inputs
    const int nt = blockIdx.x % n_tiles;                        // 64 stored rows
    {
        const int row = t >> 2, piece = t & 3;                  // stored row in tile, 32 inputs
        const int64_t n = (int64_t)nt * 64 + row;
        const int k0 = kt * 128 + piece * 32;
        uint4 cq = make_uint4(0, 0, 0, 0);
        float a1 = 0.0f, b1 = 0.0f;
        float4 a4 = make_float4(0.f, 0.f, 0.f, 0.f), b4 = make_float4(0.f, 0.f, 0.f, 0.f), a4b = a4, b4b = b4;
        if (k0 < d_in) {                                        // d_in % 64 == 0: the last tile may be half
            cq = *reinterpret_cast<const uint4*>(codes + n * (d_in / 2) + k0 / 2);
            if constexpr (block_rows == 8 && block_cols == 4) {  // eight block columns of 4 inputs
                const int64_t blk = (n >> 3) * (int64_t)(d_in / 4) + k0 / 4;
                a4 = *reinterpret_cast<const float4*>(scales + blk);
                a4b = *reinterpret_cast<const float4*>(scales + blk + 4);
                if constexpr (BETA) { b4 = *reinterpret_cast<const float4*>(beta + blk); b4b = *reinterpret_cast<const float4*>(beta + blk + 4); }
            } else if constexpr (block_rows == 8) {              // four block columns of 8 inputs
                const int64_t blk = (n >> 3) * (int64_t)(d_in / 8) + k0 / 8;
                a4 = *reinterpret_cast<const float4*>(scales + blk);
                if constexpr (BETA) b4 = *reinterpret_cast<const float4*>(beta + blk);
            } else {
                const int64_t blk = n * (int64_t)(d_in / kBlock) + k0 / kBlock;
                a1 = scales[blk];
                if constexpr (BETA) b1 = beta[blk];
            }
        }
        const uint32_t cw[4] = {cq.x, cq.y, cq.z, cq.w};
        const float as[8] = {a4.x, a4.y, a4.z, a4.w, a4b.x, a4b.y, a4b.z, a4b.w};
        const float bs[8] = {b4.x, b4.y, b4.z, b4.w, b4b.x, b4b.y, b4b.z, b4b.w};
        constexpr bool half = block_rows == 8 && block_cols == 4;   // two blocks per chunk of 8 inputs
#pragma unroll
        for (int c = 0; c < 4; ++c) {                           // chunk 4*piece + c: 8 inputs
            const float a = half ? as[2 * c] : block_rows == 8 ? as[c] : a1, be = half ? bs[2 * c] : block_rows == 8 ? bs[c] : b1;
            const float a_hi = half ? as[2 * c + 1] : a, be_hi = half ? bs[2 * c + 1] : be;    // inputs 4 .. 7 of the chunk
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float cv = lut[(cw[c] >> (4 * j)) & 15];
                v[j] = BETA ? __fmaf_rn(cv, j < 4 ? a : a_hi, j < 4 ? be : be_hi) : __fmul_rn(cv, j < 4 ? a : a_hi);
            }
            const int pos = (4 * piece + c) ^ ((row & 3) << 2);
            *reinterpret_cast<uint4*>(tile + row * 256 + pos * 16) =
                make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
        }
    }
    __syncthreads();
    {
        const int q = t >> 6, lane = t & 63;                    // wave q: stored rows 16q .. 16q+15 of the tile
        const int g = lane >> 4, sl = lane & 15;
        const int frow = 8 * (g >> 1) + (sl >> 2);              // row inside the 16-row slice this lane points at
        const int64_t kb_count = d_out / 16;                    // slices of the contraction (stored rows)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {                        // 32 inputs each
            const int col = 32 * kb + 16 * (g & 1) + 4 * (sl & 3);
            const unsigned char* p = tile + (16 * q + frow) * 256 + ((((col >> 3) ^ ((frow & 3) << 2)) & 15) << 4) +
                                     ((col >> 2) & 1) * 8;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p + 4 * 256));
            const int64_t kb32 = (int64_t)kt * 4 + kb;
            if (kb32 * 32 < d_in) {
                uint4 o;
                o.x = __builtin_bit_cast(uint2, lo).x; o.y = __builtin_bit_cast(uint2, lo).y;
                o.z = __builtin_bit_cast(uint2, hi).x; o.w = __builtin_bit_cast(uint2, hi).y;
                out[(kb32 * kb_count + (int64_t)nt * 4 + q) * 64 + lane] = o;
            }
        }
    }
}

// Nibbles of a code dword regrouped for the table-free decode: position p of the result holds input k(p),
// k = 0, 2, 4, 6, 1, 3, 5, 7 -- the even inputs in the low half, the odd ones in the high half, so that
// (w >> 4i) & 0x000F000F is the pair (input 2i, input 2i+1) in the low bits of two 16-bit lanes.
__device__ __forceinline__ uint32_t regroup_nibbles(uint32_t w) {
    uint32_t e = w & 0x0F0F0F0Fu, o = (w >> 4) & 0x0F0F0F0Fu;
    e = (e | (e >> 4)) & 0x00FF00FFu; e = (e | (e >> 8)) & 0x0000FFFFu;
    o = (o | (o >> 4)) & 0x00FF00FFu; o = (o | (o >> 8)) & 0x0000FFFFu;
    return e | (o << 16);
}

// Tile-ordered copy of the codes: one thread moves one 16-byte half of a (row, 64-block) run; rows past
// d_out inside the last tile are written as zeros.  `regroup`: the decode pack of an INT4 model (above).
__global__ __launch_bounds__(256) void k_prepack_codes(const uint8_t* __restrict__ codes, int d_out, int bpr,
                                                       int64_t n_halves, uint8_t* __restrict__ tiled, int regroup) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;        // index of a 16-byte piece of the tiled copy
    if (i >= n_halves) return;
    const int half = (int)(i & 1);
    const int64_t run = i >> 1;                                       // (tile, block, row-in-tile)
    const int r = (int)(run & 255);
    const int64_t tb = run >> 8;
    const int64_t tile = tb / bpr, b = tb - tile * bpr;
    const int64_t n = tile * 256 + r;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < d_out) v = *reinterpret_cast<const uint4*>(codes + (n * bpr + b) * 32 + half * 16);
    if (regroup) v = make_uint4(regroup_nibbles(v.x), regroup_nibbles(v.y), regroup_nibbles(v.z), regroup_nibbles(v.w));
    *reinterpret_cast<uint4*>(tiled + i * 16) = v;
}

}  // namespace

int launch_prepack_codes(const uint8_t* codes, int d_out, int d_in, uint8_t* tiled, hipStream_t st, int regroup) {
    const int bpr = d_in / kBlock;
    const int64_t n_halves = (int64_t)((d_out + 255) / 256) * 256 * bpr * 2;
    hipLaunchKernelGGL(k_prepack_codes, dim3((unsigned)((n_halves + 255) / 256)), dim3(256), 0, st, codes, d_out, bpr,
                       n_halves, tiled, regroup);
    return launch_status();
}

int launch_quantize_codebook(const float* W, int d_out, int d_in, const Codebook& cb, uint8_t* codes,
                             uint8_t* tiled, float* absmax, hipStream_t st, int block_rows, int block_cols) {
    Midpoints mp;
    for (int j = 0; j < 15; ++j) {
        volatile float sum = cb.c[j] + cb.c[j + 1];   // two separate fp32 roundings
        volatile float m = sum * 0.5f;
        mp.m[j] = m;
    }
    if (block_rows == 8) {
        const unsigned grid8 = (unsigned)(((d_in + 511) / 512) * (d_out / 8));
        if (block_cols == 4)
            hipLaunchKernelGGL((k_quantize_tile8<false, 4>), dim3(grid8), dim3(256), 0, st, reinterpret_cast<const float4*>(W),
                               d_out, d_in, mp, codes, tiled, absmax, static_cast<float*>(nullptr));
        else
            hipLaunchKernelGGL((k_quantize_tile8<false, 8>), dim3(grid8), dim3(256), 0, st, reinterpret_cast<const float4*>(W),
                               d_out, d_in, mp, codes, tiled, absmax, static_cast<float*>(nullptr));
        return launch_status();
    }
    const int bpr = d_in / kBlock;
    hipLaunchKernelGGL(k_quantize_codebook, quant_grid(d_out, bpr), dim3(256), 0, st, reinterpret_cast<const float4*>(W),
                       d_out, bpr, mp, codes, tiled, absmax);
    return launch_status();
}

int launch_quantize_minmax(const float* W, int d_out, int d_in, uint8_t* codes, uint8_t* tiled, float* alpha,
                           float* beta, hipStream_t st, int block_rows, int block_cols) {
    if (block_rows == 8) {
        const unsigned grid8 = (unsigned)(((d_in + 511) / 512) * (d_out / 8));
        if (block_cols == 4)
            hipLaunchKernelGGL((k_quantize_tile8<true, 4>), dim3(grid8), dim3(256), 0, st, reinterpret_cast<const float4*>(W),
                               d_out, d_in, Midpoints{}, codes, tiled, alpha, beta);
        else
            hipLaunchKernelGGL((k_quantize_tile8<true, 8>), dim3(grid8), dim3(256), 0, st, reinterpret_cast<const float4*>(W),
                               d_out, d_in, Midpoints{}, codes, tiled, alpha, beta);
        return launch_status();
    }
    const int bpr = d_in / kBlock;
    hipLaunchKernelGGL(k_quantize_minmax, quant_grid(d_out, bpr), dim3(256), 0, st, reinterpret_cast<const float4*>(W),
                       d_out, bpr, codes, tiled, alpha, beta);
    return launch_status();
}

int launch_scales_double_quantize(const float* scales, int64_t n, int group, uint8_t* scale_codes,
                                  float* step, float* mid, hipStream_t st) {
    unsigned grid = (unsigned)((n + group - 1) / group);
    hipLaunchKernelGGL(k_scales_double_quantize, dim3(grid), dim3(256), 0, st, scales, n, group, scale_codes,
                       step, mid);
    return launch_status();
}

int launch_scales_reconstruct(const uint8_t* scale_codes, const float* step, const float* mid, int64_t n,
                              int group, float* scales, hipStream_t st) {
    unsigned grid = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(k_scales_reconstruct, dim3(grid), dim3(256), 0, st, scale_codes, step, mid, n, group,
                       scales);
    return launch_status();
}

int launch_dequantize_bf16(const qblora_qweight& qw, const float* scales, qblora_bf16* Wt, hipStream_t st) {
    Codebook cb;
    for (int j = 0; j < 16; ++j) cb.c[j] = qw.codebook[j];
    int64_t n_words = (int64_t)qw.d_out * qw.d_in / 8;
    unsigned grid = (unsigned)((n_words + 255) / 256);
    hipLaunchKernelGGL(k_dequantize_bf16, dim3(grid), dim3(256), 0, st,
                       reinterpret_cast<const uint32_t*>(qw.codes), scales, qw.beta, cb, n_words,
                       qw.block_rows == 8 ? qw.d_in / 8 : 0, qw.block_rows == 8 ? qw.block / 8 : 8,
                       reinterpret_cast<uint4*>(Wt));
    return launch_status();
}

int launch_dequantize_operand(const qblora_qweight& qw, const float* scales, int transposed, qblora_bf16* Wop,
                              hipStream_t st) {
    if (qw.d_in % 64 != 0 || qw.d_out % 64 != 0 || (reinterpret_cast<uintptr_t>(Wop) & 15) ||
        (reinterpret_cast<uintptr_t>(qw.codes) & 15))
        return QBLORA_ERR_UNSUPPORTED;
    if (qw.block_rows == 8 &&                             // four block parameters per 16-byte load
        ((reinterpret_cast<uintptr_t>(scales) & 15) || (reinterpret_cast<uintptr_t>(qw.beta) & 15)))
        return QBLORA_ERR_UNSUPPORTED;
    Codebook cb;
    for (int j = 0; j < 16; ++j) cb.c[j] = qw.codebook[j];
    const int br = qw.block_rows == 8 ? 8 : 1, bc = br == 8 ? qw.block / 8 : qw.block;
    const int64_t blocks = transposed ? (int64_t)((qw.d_in + 127) / 128) * (qw.d_out / 64)
                                      : (int64_t)((qw.d_out + 63) / 64) * ((qw.d_in + 127) / 128);
    if (blocks > 0x7fffffff) return QBLORA_ERR_UNSUPPORTED;
    auto go = [&](auto plain, auto trans) {
        if (transposed)
            hipLaunchKernelGGL(trans, dim3((unsigned)blocks), dim3(256), 0, st, qw.codes, scales, qw.beta, cb, qw.d_out, qw.d_in,
                               reinterpret_cast<uint4*>(Wop));
        else
            hipLaunchKernelGGL(plain, dim3((unsigned)blocks), dim3(256), 0, st, qw.codes, scales, qw.beta, cb, qw.d_out, qw.d_in,
                               reinterpret_cast<uint4*>(Wop));
    };
    const int geom = br == 1 ? 0 : bc == 8 ? 1 : 2;
    if (qw.beta) {
        if (geom == 0) go(k_dequantize_operand<true, 0>, k_dequantize_operand_t<true, 0>);
        else if (geom == 1) go(k_dequantize_operand<true, 1>, k_dequantize_operand_t<true, 1>);
        else go(k_dequantize_operand<true, 2>, k_dequantize_operand_t<true, 2>);
    } else {
        if (geom == 0) go(k_dequantize_operand<false, 0>, k_dequantize_operand_t<false, 0>);
        else if (geom == 1) go(k_dequantize_operand<false, 1>, k_dequantize_operand_t<false, 1>);
        else go(k_dequantize_operand<false, 2>, k_dequantize_operand_t<false, 2>);
    }
    return launch_status();
}

}  // namespace qblora
