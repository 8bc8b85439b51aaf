// Dequantize-and-contract GEMM for gfx950 (Alg. 1 qblora_forward: W_tilde = dequantize(...),
// x @ W_tilde, plus the adapter term; and its transpose for the backward pass).
//
//   C[M,N] = X1[M,K1] * Wq^T  +  X2[M,K2] * W2[N/div2, K2]^T
//
// Segment 1 reads the 4-bit codes and block scales of the frozen base weight from HBM,
// rebuilds bf16 weights (Eq. 1: c[code]*alpha (+beta), fp32 then round-to-nearest-even) straight
// into an LDS tile and feeds them to v_mfma_f32_32x32x16_bf16 with fp32 accumulation; the
// dequantized weight never exists in HBM.  qmode 1 contracts along d_in (forward), qmode 2
// uses the same stored tile transposed and contracts along d_out (backward w.r.t. activations);
// in qmode 2 the scale varies along the contraction index, which is why it is applied while
// building the tile and not to the accumulator.
// Segment 2 is a plain bf16 K-extension: the adapter's rank-R product rides in the same
// accumulators as R extra contraction steps (forward: X2 = s*U, W2 = B^T with output row n using
// row n/lambda2, i.e. repeat_interleave; backward: X2 = dU/lambda1, W2 = A with row k/lambda1).
//
// Tiling: one workgroup of 512 threads (8 wave64) owns a BM x BN output tile and walks K in steps
// of 64 (one quantization block).  Both operand tiles live in LDS as [row][64 k] bf16 with the
// 16-byte chunks of a row XOR-swizzled by (row ^ row>>3) & 7, double buffered, one barrier per
// step; global loads for step i+1 are issued before the MFMAs of step i.  The weight tile is the
// MFMA A operand and the token tile the B operand, so a lane ends up with 4 consecutive output
// features of one token and stores them as one 8-byte word.
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 512;
constexpr int kBK = 64;

__device__ __forceinline__ int swz(int row, int chunk) {
    return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

template <int BM, int BN, int WM, int WN, int QMODE>
__global__ __launch_bounds__(kThreads) void k_qgemm(GemmDesc d) {
    static_assert(WM * WN == 8, "8 waves");
    constexpr int TM = BM / WM, TN = BN / WN;       // wave tile: tokens x features
    constexpr int FM = TM / 32, FN = TN / 32;
    constexpr int XV = BM / 64;                      // 16-byte loads per thread for a token tile
    constexpr int WV = BN / 64;                      // ... for a plain bf16 weight tile
    constexpr int PER_ROW = kThreads / BN;           // qmode 1: threads sharing one weight row
    constexpr int CW = 8 / PER_ROW;                  // qmode 1: dwords of codes per thread
    constexpr int BWD_ITEMS = (BN / 4) * 8;          // qmode 2: (4 columns x 8 rows) work items

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* sX = smem;                                   // 2 * BM*128 bytes
    unsigned char* sW = smem + 2 * BM * 128;                    // 2 * BN*128 bytes
    float* lut = reinterpret_cast<float*>(smem + 2 * (BM + BN) * 128);

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm0 = (wave % WM) * TM, wn0 = (wave / WM) * TN;

    // ---- tile assignment: XCD-contiguous, grouped along tokens ---------------------------------
    const int tiles_m = (int)((d.M + BM - 1) / BM), tiles_n = (d.N + BN - 1) / BN;
    const int ntiles = tiles_m * tiles_n;
    int L = blockIdx.x;
    if ((ntiles & 7) == 0) L = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
    constexpr int GM = 4;
    const int in_group = GM * tiles_n;
    const int first_m = (L / in_group) * GM;
    const int gsize = min(tiles_m - first_m, GM);
    const int mt = first_m + (L % in_group) % gsize, nt = (L % in_group) / gsize;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * BN;

    if (t < 16) lut[t] = d.cb.c[t];

    const int K1 = QMODE == 0 ? 0 : (QMODE == 1 ? d.d_in : d.d_out);
    const int steps1 = K1 / kBK, steps2 = (d.K2 + kBK - 1) / kBK;
    const int nsteps = steps1 + steps2;
    const int bpr = d.d_in / kBlock;                // blocks per stored weight row

    f32x16 acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // ---- prefetch registers ----------------------------------------------------------------------
    uint4 xr[XV];
    uint4 wr[WV];                   // plain bf16 weight tile (segment 2)
    uint32_t cw[QMODE == 1 ? CW : 1];
    float sc1 = 0.f, be1 = 0.f;     // qmode 1 scale / beta of this thread's row and step
    uint16_t c16[8];
    float sc2[8], be2[8];           // qmode 2

    const int lrow = t >> 3, lchunk = t & 7;        // plain tile loader coordinates

    auto load_tokens = [&](const qblora_bf16* X, int64_t ld, int K, int k0) {
        int k = k0 + lchunk * 8;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            int64_t row = m0 + lrow + 64 * i;
            if (row > d.M - 1) row = d.M - 1;
            xr[i] = (k < K) ? *reinterpret_cast<const uint4*>(X + row * ld + k) : make_uint4(0, 0, 0, 0);
        }
    };

    auto load_global = [&](int step) {
        if (step < steps1) {
            const int k0 = step * kBK;
            load_tokens(d.X1, d.ldx1, K1, k0);
            if constexpr (QMODE == 1) {
                int row = n0 + t / PER_ROW;
                if (row > d.N - 1) row = d.N - 1;
                const int part = t % PER_ROW;
                const uint32_t* p = reinterpret_cast<const uint32_t*>(d.codes + (int64_t)row * (d.d_in / 2) +
                                                                      k0 / 2 + part * (CW * 4));
                if constexpr (CW == 4) {
                    uint4 v = *reinterpret_cast<const uint4*>(p);
                    cw[0] = v.x; cw[1] = v.y; cw[2] = v.z; cw[3] = v.w;
                } else if constexpr (CW == 2) {
                    uint2 v = *reinterpret_cast<const uint2*>(p);
                    cw[0] = v.x; cw[1] = v.y;
                } else {
                    cw[0] = *p;
                }
                int64_t blk = (int64_t)row * bpr + step;
                sc1 = d.scales[blk];
                if (d.beta) be1 = d.beta[blk];
            } else if constexpr (QMODE == 2) {
                if (t < BWD_ITEMS) {
                    int c = n0 + 4 * (t % (BN / 4));
                    if (c > d.N - 4) c = d.N - 4;
                    const int nb = k0 + 8 * (t / (BN / 4));
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        int64_t n = nb + i;
                        c16[i] = *reinterpret_cast<const uint16_t*>(d.codes + n * (d.d_in / 2) + c / 2);
                        int64_t blk = n * bpr + c / kBlock;
                        sc2[i] = d.scales[blk];
                        if (d.beta) be2[i] = d.beta[blk];
                    }
                }
            }
        } else {
            const int k0 = (step - steps1) * kBK;
            load_tokens(d.X2, d.ldx2, d.K2, k0);
            int k = k0 + lchunk * 8;
#pragma unroll
            for (int i = 0; i < WV; ++i) {
                int row = n0 + lrow + 64 * i;
                if (row > d.N - 1) row = d.N - 1;
                row /= d.div2;
                wr[i] = (k < d.K2) ? *reinterpret_cast<const uint4*>(d.W2 + (int64_t)row * d.ldw2 + k)
                                   : make_uint4(0, 0, 0, 0);
            }
        }
    };

    auto store_lds = [&](int step, int buf) {
        unsigned char* bx = sX + buf * BM * 128;
        unsigned char* bw = sW + buf * BN * 128;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            int row = lrow + 64 * i;
            *reinterpret_cast<uint4*>(bx + swz(row, lchunk)) = xr[i];
        }
        if (step < steps1) {
            if constexpr (QMODE == 1) {
                const int row = t / PER_ROW, part = t % PER_ROW;
                const bool hb = d.beta != nullptr;
#pragma unroll
                for (int w = 0; w < CW; ++w) {
                    float v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        float c = lut[(cw[w] >> (4 * j)) & 15];
                        v[j] = hb ? __fmaf_rn(c, sc1, be1) : __fmul_rn(c, sc1);
                    }
                    uint4 o;
                    o.x = pack_bf16(v[0], v[1]); o.y = pack_bf16(v[2], v[3]);
                    o.z = pack_bf16(v[4], v[5]); o.w = pack_bf16(v[6], v[7]);
                    *reinterpret_cast<uint4*>(bw + swz(row, part * CW + w)) = o;
                }
            } else if constexpr (QMODE == 2) {
                if (t < BWD_ITEMS) {
                    const int cg = t % (BN / 4), ng = t / (BN / 4);
                    const bool hb = d.beta != nullptr;
                    float v[8][4];
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            float c = lut[(c16[i] >> (4 * j)) & 15];
                            v[i][j] = hb ? __fmaf_rn(c, sc2[i], be2[i]) : __fmul_rn(c, sc2[i]);
                        }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        uint4 o;
                        o.x = pack_bf16(v[0][j], v[1][j]); o.y = pack_bf16(v[2][j], v[3][j]);
                        o.z = pack_bf16(v[4][j], v[5][j]); o.w = pack_bf16(v[6][j], v[7][j]);
                        *reinterpret_cast<uint4*>(bw + swz(4 * cg + j, ng)) = o;
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < WV; ++i) {
                int row = lrow + 64 * i;
                *reinterpret_cast<uint4*>(bw + swz(row, lchunk)) = wr[i];
            }
        }
    };

    auto compute = [&](int buf) {
        const unsigned char* bx = sX + buf * BM * 128;
        const unsigned char* bw = sW + buf * BN * 128;
        const int r = lane & 31, hi = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 wf[FN], xf[FM];
#pragma unroll
            for (int a = 0; a < FN; ++a)
                wf[a] = *reinterpret_cast<const bf16x8*>(bw + swz(wn0 + a * 32 + r, ks * 2 + hi));
#pragma unroll
            for (int b = 0; b < FM; ++b)
                xf[b] = *reinterpret_cast<const bf16x8*>(bx + swz(wm0 + b * 32 + r, ks * 2 + hi));
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
        }
    };

    // ---- main loop ---------------------------------------------------------------------------------
    if (nsteps > 0) {
        load_global(0);
        __syncthreads();            // lut visible
        store_lds(0, 0);
        __syncthreads();
        for (int step = 0; step < nsteps; ++step) {
            const int buf = step & 1;
            const bool more = step + 1 < nsteps;
            if (more) load_global(step + 1);
            compute(buf);
            if (more) store_lds(step + 1, buf ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: lane holds features n..n+3 of one token per accumulator quad -----------------------
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b) {
            const int64_t m = m0 + wm0 + b * 32 + r;
            if (m >= d.M) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn0 + a * 32 + q * 8 + hi * 4;
                if (n >= d.N) continue;
                float v0 = acc[a][b][q * 4 + 0] * d.out_scale, v1 = acc[a][b][q * 4 + 1] * d.out_scale;
                float v2 = acc[a][b][q * 4 + 2] * d.out_scale, v3 = acc[a][b][q * 4 + 3] * d.out_scale;
                if (d.out_f32) {
                    *reinterpret_cast<float4*>(reinterpret_cast<float*>(d.C) + m * d.ldc + n) =
                        make_float4(v0, v1, v2, v3);
                } else {
                    uint2 o;
                    o.x = pack_bf16(v0, v1); o.y = pack_bf16(v2, v3);
                    *reinterpret_cast<uint2*>(reinterpret_cast<qblora_bf16*>(d.C) + m * d.ldc + n) = o;
                }
                if (d.C_lo) {
                    uint2 h;
                    h.x = pack_bf16(v0, v1); h.y = pack_bf16(v2, v3);
                    uint2 o;
                    o.x = pack_bf16(v0 - bf16_bits_to_float(h.x & 0xffffu), v1 - bf16_bits_to_float(h.x >> 16));
                    o.y = pack_bf16(v2 - bf16_bits_to_float(h.y & 0xffffu), v3 - bf16_bits_to_float(h.y >> 16));
                    *reinterpret_cast<uint2*>(d.C_lo + m * d.ldc + n) = o;
                }
                if (d.C2) {
                    uint2 o;
                    o.x = pack_bf16(v0 * d.c2_scale, v1 * d.c2_scale);
                    o.y = pack_bf16(v2 * d.c2_scale, v3 * d.c2_scale);
                    *reinterpret_cast<uint2*>(d.C2 + m * d.ldc + n) = o;
                }
            }
        }
}

template <int BM, int BN, int WM, int WN, int QMODE>
int launch_cfg(const GemmDesc& d, hipStream_t st) {
    constexpr size_t smem = 2 * (BM + BN) * 128 + 64;
    auto kern = k_qgemm<BM, BN, WM, WN, QMODE>;
    // set once per instantiation; the initialisation of a function-local static is thread safe
    static const bool attr_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!attr_ok) return QBLORA_ERR_LAUNCH;
    int64_t tiles = ((d.M + BM - 1) / BM) * ((d.N + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kThreads), smem, st, d);
    return launch_status();
}

}  // namespace

int launch_gemm(const GemmDesc& d, hipStream_t st) {
    if (d.M <= 0 || d.N <= 0) return QBLORA_OK;
    if (d.qmode == 1 || d.qmode == 2 || d.qmode == 3) return launch_qlinear(d, st);
    if (skinny_applies(d)) return launch_skinny(d, st);
    // plain bf16 GEMMs of the adapter path that are not narrow (the tile product): 128 x 128 tiles unless
    // 256 x 256 tiles alone give every CU at least two workgroups
    const int64_t big_tiles = ((d.M + 255) / 256) * ((d.N + 255) / 256);
    if (d.N <= 128 || big_tiles < 512) return launch_cfg<128, 128, 2, 4, 0>(d, st);
    return launch_cfg<256, 256, 2, 4, 0>(d, st);
}

}  // namespace qblora
