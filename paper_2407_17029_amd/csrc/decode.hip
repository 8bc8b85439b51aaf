// Small-batch forward of a 4-bit block-quantized layer (merged-model inference: the INT4 weights
// (codes, alpha, beta) that the QA-BLoRA merge of Sec. 3.3 produces, or any other quantized base):
//
//   Y[t, n] = sum_k X[t, k] * w~[n, k],   w~ = bf16(c[code] * alpha) or bf16(fma(c[code], alpha, beta)),
//
// for T <= 16 tokens.  Every weight is used once per token, so the kernel is bound by streaming the
// codes and block parameters from HBM (0.5 + 4/64 (+ 4/64) bytes per weight); the dequantize-and-
// contract kernel for training batches would spend its time filling 256-token tiles with padding.
//
// A workgroup of 4 waves owns 16 output rows; the waves split the input dimension (wave w takes the
// groups of 4 blocks j = w, w+4, ...) and add their partial tiles through LDS at the end.  Inside a
// wave, lane l works on row (l & 15) and on block 4j + (l >> 4) of the group: it loads that block's 32
// code bytes and parameters, dequantizes 8 weights at a time into the A operand of
// v_mfma_f32_16x16x32_bf16 and contracts them with the 8 matching activations of token (l & 15) (B
// operand, zero for tokens >= T), so one MFMA retires 16 rows x 16 tokens x 32 inputs and the vector
// ALU only dequantizes.  The contraction order inside a group is this lane assignment (any order is
// valid as long as both operands agree); accumulation is fp32.
#include "common.h"

namespace qblora {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;

struct DecodeDesc {
    const uint8_t* codes; const float* scales; const float* beta; Codebook cb;
    int d_out, d_in;
    const qblora_bf16* X; int T;
    qblora_bf16* Y;
};

struct DecodeRegs {
    uint4 c0, c1;          // the lane's block: 64 codes
    float a, b;            // its scale and offset
    uint4 x[8];            // activations of the lane's token for the block, 8 per MFMA
};

template <bool BETA>
__global__ __launch_bounds__(256) void k_w4_decode(DecodeDesc d) {
    __shared__ float lut[16];
    __shared__ float red[4][4][64];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int nl = lane & 15, kg = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int n = min(n0 + nl, d.d_out - 1);                  // rows past the end are computed, not stored
    const int bpr = d.d_in / kBlock;
    const int groups = (bpr + 3) / 4;
    if (t < 16) lut[t] = d.cb.c[t];
    __syncthreads();

    const uint8_t* crow = d.codes + (int64_t)n * (d.d_in / 2);
    const float* srow = d.scales + (int64_t)n * bpr;
    const float* brow = BETA ? d.beta + (int64_t)n * bpr : nullptr;
    const qblora_bf16* xrow = d.X + (int64_t)min(nl, d.T - 1) * d.d_in;
    const bool token = nl < d.T;

    auto load = [&](DecodeRegs& r, int j) __attribute__((always_inline)) {
        const int b = 4 * j + kg;
        if (b < bpr) {
            const uint4* cp = reinterpret_cast<const uint4*>(crow + b * 32);
            r.c0 = cp[0]; r.c1 = cp[1];
            r.a = srow[b];
            r.b = BETA ? brow[b] : 0.0f;
        } else {
            r.c0 = r.c1 = make_uint4(0, 0, 0, 0); r.a = 0.0f; r.b = 0.0f;
        }
#pragma unroll
        for (int m = 0; m < 8; ++m)
            r.x[m] = (token && b < bpr) ? *reinterpret_cast<const uint4*>(xrow + b * kBlock + 8 * m) : make_uint4(0, 0, 0, 0);
    };

    f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    auto compute = [&](const DecodeRegs& r) __attribute__((always_inline)) {
        const uint32_t cw[8] = {r.c0.x, r.c0.y, r.c0.z, r.c0.w, r.c1.x, r.c1.y, r.c1.z, r.c1.w};
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            uint32_t p[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float c_lo = lut[(cw[m] >> (8 * q)) & 15], c_hi = lut[(cw[m] >> (8 * q + 4)) & 15];
                const float w_lo = BETA ? __fmaf_rn(c_lo, r.a, r.b) : __fmul_rn(c_lo, r.a);
                const float w_hi = BETA ? __fmaf_rn(c_hi, r.a, r.b) : __fmul_rn(c_hi, r.a);
                p[q] = pack_bf16(w_lo, w_hi);
            }
            const uint4 wv = make_uint4(p[0], p[1], p[2], p[3]);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv), __builtin_bit_cast(bf16x8, r.x[m]),
                                                          acc, 0, 0, 0);
        }
    };

    // two register sets: the loads of the wave's next group are in flight while this one is contracted
    DecodeRegs r0, r1;
    int j = wave;
    if (j < groups) load(r0, j);
    for (; j < groups; j += 8) {
        if (j + 4 < groups) load(r1, j + 4);
        compute(r0);
        if (j + 4 < groups) {
            if (j + 8 < groups) load(r0, j + 8);
            compute(r1);
        }
    }

    // partial tiles of the four waves -> LDS, added in wave order by wave 0
#pragma unroll
    for (int e = 0; e < 4; ++e) red[wave][e][lane] = acc[e];
    __syncthreads();
    if (wave == 0 && token) {
        // the lane holds token nl, rows 4*kg .. 4*kg+3
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = ((red[0][e][lane] + red[1][e][lane]) + red[2][e][lane]) + red[3][e][lane];
        const int nb = n0 + 4 * kg;
        qblora_bf16* yp = d.Y + (int64_t)nl * d.d_out + nb;
        if (nb + 3 < d.d_out && (d.d_out & 3) == 0) {
            *reinterpret_cast<uint2*>(yp) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (nb + e < d.d_out) reinterpret_cast<uint16_t*>(yp)[e] = (uint16_t)(pack_bf16(v[e], 0.0f) & 0xffffu);
        }
    }
}

}  // namespace

int launch_w4_decode(const uint8_t* codes, const float* scales, const float* beta, const Codebook& cb, int d_out,
                     int d_in, const qblora_bf16* X, int T, qblora_bf16* Y, hipStream_t st) {
    DecodeDesc d{codes, scales, beta, cb, d_out, d_in, X, T, Y};
    const dim3 grid((unsigned)((d_out + 15) / 16));
    if (beta) hipLaunchKernelGGL(k_w4_decode<true>, grid, dim3(256), 0, st, d);
    else hipLaunchKernelGGL(k_w4_decode<false>, grid, dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace qblora
