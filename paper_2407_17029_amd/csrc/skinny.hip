// Narrow-output bf16 GEMM of the adapter path for gfx950:
//
//   C[M,N] = out_scale * X[M,K] * W[N,K]^T,   N = the adapter's inner rank R (tens to a few hundred)
//
// used for U = P A (Sec. 3.2; the average pool is folded into W = A^T repeated lambda1 times along
// k, so X is the raw activation) and for dU = dV B^T of the backward pass (the sum pool over lambda2
// folded the same way).  M is the token count and K the layer width, so the kernel reads X once
// from HBM and is bound by that stream, not by the MFMAs: the design goal is bytes in flight.
//
// One workgroup of 4 wave64 owns BM tokens x BN output columns and walks K through a ring of LDS
// stages (one or two 64-wide k-steps per stage and barrier).  Both operand tiles of a stage arrive by
// direct global -> LDS copies issued STAGES-1 stages ahead.  X comes from HBM once; W (1 MB for rank
// 128 at K = 4096) is re-read from L2 by every token tile, so the traffic through the CUs is a few
// times the X stream and that, not HBM latency, sets the pace: measured times do not change between
// 3 and 9 stages.  With a token count that gives only 128 tiles of 64 tokens, 64 x 64 tiles put a
// workgroup on every CU; the two workgroups that share a token tile sit on the same XCD and the second
// finds X in L2.  Tiles are [row][64 k] bf16 with the 16-byte chunks XOR-swizzled by
// (row ^ row>>3) & 7, applied by choosing which global chunk a lane fetches.
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 256;
constexpr int kBK = 64;

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding
constexpr int vmcnt_imm(int n) { return (n & 15) | 0x0F70 | ((n >> 4) << 14); }

__device__ __forceinline__ int swz(int row, int chunk) {
    return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

__device__ __forceinline__ void copy16_to_lds(const void* uniform_base, uint32_t lane_offset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(lane_offset), "s"(uniform_base) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// kDup = 2: W is stored with K/2 columns and column m serves k = 2m and 2m+1 (the adapter operand
// before its expansion along k: the pool over pairs of features is then folded into the fragment,
// which halves the W stream from L2 and its LDS tile).  Only in the k-split form with two k-steps per
// stage: the W columns of both k-steps are 128 contiguous bytes per row and form one tile per stage,
// behind the stage's two X sub-tiles.
template <int BM, int BN, int kStages, int kSub, bool kSplitK, int kDup = 1>
__global__ __launch_bounds__(kThreads) void k_skinny(GemmDesc d) {
    static_assert(!kSplitK || (BM == 64 && (BN == 64 || BN == 128)), "the k-split form is written for 64 x 64 and 64 x 128 tiles");
    static_assert(kDup == 1 || (kDup == 2 && kSplitK && kSub == 2), "column duplication: k-split form, two k-steps per stage");
    // a stage holds kSub consecutive k-steps (sub-tiles of 64 k each): one barrier per kSub * 64 k
    constexpr int kXBytes = BM * 128, kWBytes = BN * 128 / kDup, kSubBytes = kXBytes + kWBytes, kStageBytes = kSub * kSubBytes;
    constexpr int XC = BM / 32, WC = BN / 32;     // copies per wave and sub-tile (kDup = 2: W copies per stage)
    // byte offsets of the X sub-tile u and of its W tile inside a stage
    auto x_at = [](int u) { return kDup == 2 ? u * kXBytes : u * kSubBytes; };
    auto w_at = [](int u) { return kDup == 2 ? kSub * kXBytes : u * kSubBytes + kXBytes; };
    constexpr int WN = BN / 32, WM = 4 / WN;      // waves along the columns / along the tokens
    constexpr int MF = BM / (32 * WM);            // 32-token blocks per wave
    static_assert(MF >= 1 && WN * WM == 4, "tile shape");
    extern __shared__ __align__(16) unsigned char smem[];
    const int64_t M = d.M;
    const int N = d.N, K = d.K2;
    const qblora_bf16* const X = d.X2; const int64_t ldx = d.ldx2;
    const qblora_bf16* const W = d.W2; const int64_t ldw = d.ldw2;
    qblora_bf16* const C = reinterpret_cast<qblora_bf16*>(d.C);
    qblora_bf16* const C2 = d.C2;
    qblora_bf16* const C_lo = d.C_lo;
    const int64_t ldc = d.ldc;
    const float out_scale = d.out_scale, c2_scale = d.c2_scale;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    // blockIdx.x % 8 is the XCD: the column tiles of one token tile are 8 apart
    const int tiles_n = (N + BN - 1) / BN;
    const int grp = blockIdx.x / (8 * tiles_n), within = blockIdx.x % (8 * tiles_n);
    const int64_t m0 = ((int64_t)grp * 8 + (within & 7)) * BM;
    const int n0 = (within >> 3) * BN;
    if (m0 >= M) return;                          // the grid is rounded up to whole groups of 8 token tiles
    const int wave_n = wave % WN, wave_m = wave / WN;
    const int nsteps = K / (kBK * kSub);

    // per-lane byte offsets of the copies, relative to the first row of the tile
    const int crow = lane >> 3;
    uint32_t xoff[XC], woff[WC];
#pragma unroll
    for (int i = 0; i < XC; ++i) {
        int64_t lrow = wave * (8 * XC) + i * 8 + crow;
        if (m0 + lrow > M - 1) lrow = M - 1 - m0;
        xoff[i] = (uint32_t)(lrow * ldx * 2) + (((lane & 7) ^ crow ^ ((XC * wave + i) & 7)) << 4);
    }
#pragma unroll
    for (int i = 0; i < WC; ++i) {
        int lrow = wave * (8 * WC) + i * 8 + crow;
        if (n0 + lrow > N - 1) lrow = N - 1 - n0;
        woff[i] = (uint32_t)((int64_t)lrow * ldw * 2) + (((lane & 7) ^ crow ^ ((WC * wave + i) & 7)) << 4);
    }
    const qblora_bf16* const x_tile = X + m0 * ldx;
    const qblora_bf16* const w_tile = W + (int64_t)n0 * ldw;
    const uint32_t lds_x = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * (8 * XC) * 128);
    const uint32_t lds_w = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * (8 * WC) * 128);
    auto issue = [&](int step) __attribute__((always_inline)) {
        const uint32_t stage = (step % kStages) * kStageBytes;
#pragma unroll
        for (int u = 0; u < kSub; ++u) {
            const qblora_bf16* xb = x_tile + (step * kSub + u) * kBK;
            const qblora_bf16* wb = w_tile + (step * kSub + u) * (kBK / kDup);
#pragma unroll
            for (int i = 0; i < XC; ++i) copy16_to_lds(xb, xoff[i], lds_x + stage + x_at(u) + i * 8 * 128);
            if (kDup == 2 && u > 0) continue;     // one W tile per stage: 64 stored columns = both k-steps
#pragma unroll
            for (int i = 0; i < WC; ++i) copy16_to_lds(wb, woff[i], lds_w + stage + w_at(u) + i * 8 * 128);
        }
    };

    // Plain form: a wave owns 32 columns x MF token blocks and keeps one accumulator chain per
    // sub-tile (added at the end).  k-split form (64 tokens x 64 or 128 columns): a 32 x 32 wave tile would
    // read two fragments per MFMA, which is all the LDS can deliver; instead every wave computes the whole
    // tile (acc[column block][token block]) for one quarter of each sub-tile's k (slice ks == wave), one
    // fragment read per MFMA (three per four with 128 columns), and the four partial tiles are added through
    // LDS at the end, 64 columns at a time.
    constexpr int NA = kSplitK ? BN / 32 : kSub, NB = kSplitK ? 2 : MF;
    f32x16 acc[NA][NB];
#pragma unroll
    for (int u = 0; u < NA; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[u][b][i] = 0.0f;

    const int r = lane & 31, hi = lane >> 5;
    auto compute = [&](int step) __attribute__((always_inline)) {
        if constexpr (kSplitK) {
#pragma unroll
            for (int u = 0; u < kSub; ++u) {
                const unsigned char* bx = smem + (step % kStages) * kStageBytes + x_at(u);
                const unsigned char* bw = smem + (step % kStages) * kStageBytes + w_at(u);
                bf16x8 wf[NA], xf[2];
#pragma unroll
                for (int a = 0; a < 2; ++a) xf[a] = *reinterpret_cast<const bf16x8*>(bx + swz(a * 32 + r, wave * 2 + hi));
#pragma unroll
                for (int a = 0; a < NA; ++a) {
                    if constexpr (kDup == 2) {
                        // stored columns 32*u + 8*wave + 4*hi .. +3 of row a*32 + r, each used for two k
                        const uint2 v = *reinterpret_cast<const uint2*>(bw + swz(a * 32 + r, 4 * u + wave) + 8 * hi);
                        const uint4 e = make_uint4(__builtin_amdgcn_perm(v.x, v.x, 0x01000100u), __builtin_amdgcn_perm(v.x, v.x, 0x03020302u),
                                                   __builtin_amdgcn_perm(v.y, v.y, 0x01000100u), __builtin_amdgcn_perm(v.y, v.y, 0x03020302u));
                        wf[a] = __builtin_bit_cast(bf16x8, e);
                    } else {
                        wf[a] = *reinterpret_cast<const bf16x8*>(bw + swz(a * 32 + r, wave * 2 + hi));
                    }
                }
#pragma unroll
                for (int a = 0; a < NA; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int u = 0; u < kSub; ++u) {
                const unsigned char* bx = smem + (step % kStages) * kStageBytes + x_at(u);
                const unsigned char* bw = smem + (step % kStages) * kStageBytes + w_at(u);
                const bf16x8 wf = *reinterpret_cast<const bf16x8*>(bw + swz(wave_n * 32 + r, ks * 2 + hi));
#pragma unroll
                for (int b = 0; b < MF; ++b) {
                    const bf16x8 xf = *reinterpret_cast<const bf16x8*>(bx + swz((wave_m * MF + b) * 32 + r, ks * 2 + hi));
                    acc[u][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[u][b], 0, 0, 0);
                }
            }
    };

    constexpr int kAhead = kStages - 1;           // stages in flight
#pragma unroll
    for (int i = 0; i < kAhead; ++i)
        if (i < nsteps) issue(i);
    int s = 0;
    for (; s + kAhead < nsteps; ++s) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((kAhead - 1) * (XC * kSub + WC * (kDup == 2 ? 1 : kSub))));   // the younger stages may be in flight
        __syncthreads();                          // stage s landed for all; everyone is done with step s-1
        issue(s + kAhead);                        // into the buffer step s-1 used
        compute(s);
    }
    for (; s < nsteps; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
        __syncthreads();
        compute(s);
    }

    // lane holds columns n..n+3 of one token per accumulator quad of a 32 x 32 block
    auto emit = [&](const f32x16& v, const int out_n, const int out_m) __attribute__((always_inline)) {
        const int64_t m = m0 + out_m + r;
        if (m >= M) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n0 + out_n + q * 8 + hi * 4;
            if (n >= N) continue;
            const float v0 = v[q * 4 + 0] * out_scale, v1 = v[q * 4 + 1] * out_scale;
            const float v2 = v[q * 4 + 2] * out_scale, v3 = v[q * 4 + 3] * out_scale;
            uint2 h;
            h.x = pack_bf16(v0, v1); h.y = pack_bf16(v2, v3);
            *reinterpret_cast<uint2*>(C + m * ldc + n) = h;
            if (C_lo) {
                uint2 o;
                o.x = pack_bf16(v0 - bf16_bits_to_float(h.x & 0xffffu), v1 - bf16_bits_to_float(h.x >> 16));
                o.y = pack_bf16(v2 - bf16_bits_to_float(h.y & 0xffffu), v3 - bf16_bits_to_float(h.y >> 16));
                *reinterpret_cast<uint2*>(C_lo + m * ldc + n) = o;
            }
            if (C2) {
                uint2 o;
                o.x = pack_bf16(v0 * c2_scale, v1 * c2_scale);
                o.y = pack_bf16(v2 * c2_scale, v3 * c2_scale);
                *reinterpret_cast<uint2*>(C2 + m * ldc + n) = o;
            }
        }
    };
    if constexpr (kSplitK) {
        // partial tiles -> LDS, 64 columns (two column blocks) per pass: register i of block (a, b) of wave w at
        // float [((w*4 + a*2+b)*16 + i)*64 + lane]; wave w then adds the four partials of block (a, b) =
        // (w >> 1, w & 1) in wave order.  The first barrier also ends the last step's reads of the ring.
        float* red = reinterpret_cast<float*>(smem);
#pragma unroll
        for (int p = 0; p < NA / 2; ++p) {
            __syncthreads();
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) red[((wave * 4 + a * 2 + b) * 16 + i) * 64 + lane] = acc[2 * p + a][b][i];
            __syncthreads();
            f32x16 sum;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = red[((0 * 4 + wave) * 16 + i) * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) v += red[((w * 4 + wave) * 16 + i) * 64 + lane];
                sum[i] = v;
            }
            emit(sum, p * 64 + (wave >> 1) * 32, (wave & 1) * 32);
        }
    } else {
#pragma unroll
        for (int u = 1; u < kSub; ++u)
#pragma unroll
            for (int b = 0; b < MF; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[0][b][i] += acc[u][b][i];
#pragma unroll
        for (int b = 0; b < MF; ++b) emit(acc[0][b], wave_n * 32, (wave_m * MF + b) * 32);
    }
}

}  // namespace

// Whether the narrow GEMM can take W with K/2 columns, each serving two adjacent k (GemmDesc::dup2 = 2): the
// problem must be one the k-split form with two k-steps per stage handles (at every token count: with 512 or more
// tiles of 64 x 128 the plain form on the expanded operand measured slower, 13B layer at rank 128 21.0 -> 20.8 ms).
bool skinny_dup_applies(int64_t /*M*/, int N, int K, int64_t ldw) {
    return N > 64 && N % 4 == 0 && N <= 512 && K % (2 * kBK) == 0 && ldw % 8 == 0;
}

// Whether launch_skinny can take this problem (otherwise the general tile kernel does).
bool skinny_applies(const GemmDesc& d) {
    return d.qmode == 0 && !d.out_f32 && d.div2 == 1 && d.N % 4 == 0 && d.N <= 512 && d.K2 > 0 &&
           d.K2 % kBK == 0 && d.M >= 1 && (int64_t)128 * d.ldw2 * 2 < (int64_t)1 << 31 &&
           (int64_t)64 * d.ldx2 * 2 < (int64_t)1 << 31;
}

template <int BM, int BN, int kStages, int kSub, bool kSplitK, int kDup = 1>
int launch_skinny_cfg(const GemmDesc& d, hipStream_t st) {
    constexpr size_t smem = kStages * kSub * (BM * 128 + BN * 128 / kDup);
    auto kern = k_skinny<BM, BN, kStages, kSub, kSplitK, kDup>;
    // set once per instantiation; the initialisation of a function-local static is thread safe
    static const bool attr_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!attr_ok) return QBLORA_ERR_LAUNCH;
    const int64_t tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
    dim3 grid((unsigned)((tiles_m + 7) / 8 * 8 * tiles_n));
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, st, d);
    return launch_status();
}

int launch_skinny(const GemmDesc& d, hipStream_t st) {
    // 64 x 128 tiles once they alone fill the chip twice over; below that 64 x 64 tiles with a deep
    // ring (a narrower output has nothing to split: 32-token tiles, 128 columns)
    const int64_t wgs = ((d.M + 63) / 64) * ((d.N + 127) / 128);
    if (d.dup2 == 2) {                                                             // see skinny_dup_applies
        // 128 columns per workgroup once that still puts a workgroup on every CU: the token tile is then fetched by
        // two workgroups instead of four (65B gate projection, inner rank 256: 2.16 -> 1.44 GB through the CUs,
        // backward 200 -> 157 us, forward 77 -> 62 us; three or four stages measure the same, two are slower)
        if (d.N > 64 && wgs >= 256) return launch_skinny_cfg<64, 128, 3, 2, true, 2>(d, st);
        return launch_skinny_cfg<64, 64, 5, 2, true, 2>(d, st);
    }
    if (wgs >= 512) return launch_skinny_cfg<64, 128, 4, 1, false>(d, st);
    if (d.N > 64) {
        if (d.K2 % (2 * kBK) == 0) return launch_skinny_cfg<64, 64, 5, 2, true>(d, st);
        return launch_skinny_cfg<64, 64, 9, 1, true>(d, st);
    }
    return launch_skinny_cfg<32, 128, 6, 1, false>(d, st);
}

}  // namespace qblora
