// Narrow-output bf16 GEMM of the adapter path for gfx950:
//
//   C[M,N] = out_scale * X[M,K] * W[N,K]^T,   N = the adapter's inner rank R (tens to a few hundred)
//
// used for U = P A (Sec. 3.2; the average pool is folded into W = A^T repeated lambda1 times along
// k, so X is the raw activation) and for dU = dV B^T of the backward pass (the sum pool over lambda2
// folded the same way).  M is the token count and K the layer width, so the kernel reads X once
// from HBM and is bound by that stream, not by the MFMAs: the design goal is bytes in flight.
//
// One workgroup of 4 wave64 owns BM (32 or 64) tokens x 128 output columns and walks K in steps of 64
// through a ring of LDS stages (6 for BM = 32, 4 for BM = 64).  Both operand tiles of a stage arrive
// by direct global -> LDS copies issued STAGES-1 steps ahead, so 70 to 100 KB per workgroup are in
// flight; one barrier per step.  BM = 32 doubles the number of workgroups (the token count of the
// workloads gives only 128 workgroups of 64 tokens, half the CUs) at the price of re-reading W from L2
// twice as often.  Tiles are [row][64 k] bf16 with the 16-byte chunks XOR-swizzled by
// (row ^ row>>3) & 7, applied by choosing which global chunk a lane fetches.  Wave w owns output
// columns 32w..32w+31 (MFMA A operand) for both 32-token halves (B operand).
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 256;
constexpr int BN = 128, kBK = 64;
constexpr int kWBytes = BN * 128;

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

template <int BM, int kStages>
__global__ __launch_bounds__(kThreads) void k_skinny(GemmDesc d) {
    constexpr int kXBytes = BM * 128, kStageBytes = kXBytes + kWBytes;
    constexpr int XC = BM / 32;                   // activation copies per wave and stage
    constexpr int MF = BM / 32;                   // 32-token blocks per wave
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
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int nsteps = K / kBK;

    // per-lane byte offsets of the copies, relative to the first row of the tile
    const int crow = lane >> 3;
    uint32_t xoff[XC], woff[4];
#pragma unroll
    for (int i = 0; i < XC; ++i) {
        int64_t lrow = wave * (8 * XC) + i * 8 + crow;
        if (m0 + lrow > M - 1) lrow = M - 1 - m0;
        xoff[i] = (uint32_t)(lrow * ldx * 2) + (((lane & 7) ^ crow ^ ((XC * wave + i) & 7)) << 4);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int lrow = wave * 32 + i * 8 + crow;
        if (n0 + lrow > N - 1) lrow = N - 1 - n0;
        woff[i] = (uint32_t)((int64_t)lrow * ldw * 2) + (((lane & 7) ^ crow ^ ((4 * wave + i) & 7)) << 4);
    }
    const qblora_bf16* const x_tile = X + m0 * ldx;
    const qblora_bf16* const w_tile = W + (int64_t)n0 * ldw;
    const uint32_t lds_x = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * (8 * XC) * 128);
    const uint32_t lds_w = __builtin_amdgcn_readfirstlane(lds_address(smem) + kXBytes + wave * 32 * 128);
    auto issue = [&](int step) __attribute__((always_inline)) {
        const uint32_t stage = (step % kStages) * kStageBytes;
        const qblora_bf16* xb = x_tile + step * kBK;
        const qblora_bf16* wb = w_tile + step * kBK;
#pragma unroll
        for (int i = 0; i < XC; ++i) copy16_to_lds(xb, xoff[i], lds_x + stage + i * 8 * 128);
#pragma unroll
        for (int i = 0; i < 4; ++i) copy16_to_lds(wb, woff[i], lds_w + stage + i * 8 * 128);
    };

    f32x16 acc[MF];
#pragma unroll
    for (int b = 0; b < MF; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

    const int r = lane & 31, hi = lane >> 5;
    auto compute = [&](int step) __attribute__((always_inline)) {
        const unsigned char* bx = smem + (step % kStages) * kStageBytes;
        const unsigned char* bw = bx + kXBytes;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 wf = *reinterpret_cast<const bf16x8*>(bw + swz(wave * 32 + r, ks * 2 + hi));
#pragma unroll
            for (int b = 0; b < MF; ++b) {
                const bf16x8 xf = *reinterpret_cast<const bf16x8*>(bx + swz(b * 32 + r, ks * 2 + hi));
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[b], 0, 0, 0);
            }
        }
    };

    constexpr int kAhead = kStages - 1;           // stages in flight
#pragma unroll
    for (int i = 0; i < kAhead; ++i)
        if (i < nsteps) issue(i);
    int s = 0;
    for (; s + kAhead < nsteps; ++s) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((kAhead - 1) * (XC + 4)));   // the younger stages may be in flight
        __syncthreads();                          // stage s landed for all; everyone is done with step s-1
        issue(s + kAhead);                        // into the buffer step s-1 used
        compute(s);
    }
    for (; s < nsteps; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
        __syncthreads();
        compute(s);
    }

    // lane holds columns n..n+3 of one token per accumulator quad
#pragma unroll
    for (int b = 0; b < MF; ++b) {
        const int64_t m = m0 + b * 32 + r;
        if (m >= M) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n0 + wave * 32 + q * 8 + hi * 4;
            if (n >= N) continue;
            const float v0 = acc[b][q * 4 + 0] * out_scale, v1 = acc[b][q * 4 + 1] * out_scale;
            const float v2 = acc[b][q * 4 + 2] * out_scale, v3 = acc[b][q * 4 + 3] * out_scale;
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
    }
}

}  // namespace

// Whether launch_skinny can take this problem (otherwise the general tile kernel does).
bool skinny_applies(const GemmDesc& d) {
    return d.qmode == 0 && !d.out_f32 && d.div2 == 1 && d.N % 4 == 0 && d.N <= 512 && d.K2 > 0 &&
           d.K2 % kBK == 0 && d.M >= 1 && (int64_t)BN * d.ldw2 * 2 < (int64_t)1 << 31 &&
           (int64_t)64 * d.ldx2 * 2 < (int64_t)1 << 31;
}

template <int BM, int kStages>
int launch_skinny_cfg(const GemmDesc& d, hipStream_t st) {
    constexpr size_t smem = kStages * (BM * 128 + kWBytes);
    auto kern = k_skinny<BM, kStages>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        attr_set = true;
    }
    dim3 grid((unsigned)((d.M + BM - 1) / BM), (unsigned)((d.N + BN - 1) / BN));
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, st, d);
    return launch_status();
}

int launch_skinny(const GemmDesc& d, hipStream_t st) {
    // 64-token tiles once they alone fill the chip twice over, 32-token tiles below that
    const int64_t wgs64 = ((d.M + 63) / 64) * ((d.N + BN - 1) / BN);
    if (wgs64 >= 512) return launch_skinny_cfg<64, 4>(d, st);
    return launch_skinny_cfg<32, 6>(d, st);
}

}  // namespace qblora
