// Row pooling for the single-matrix adapter (QA-BLoRA, Sec. 3.3, Alg. 2): the compressed input
// AvgPool_lambda1(X) and the compressed output gradient sum_lambda2(dY) are materialised once per call
// as bf16 operands of the K-extension of the dequantize-and-contract kernel and of the dH contraction,
//
//   out[t, m] = bf16( scale * sum_{i < lam} in[t, lam*m + i] )      (sum and product in fp32)
//
// and optionally the bf16 residual out_lo = bf16(value - out), which the dH contraction adds as a
// second operand part so that only one of its two operands carries a bf16 rounding.
//
// Streaming, HBM-bound: a thread produces 8 consecutive outputs (one 16-byte store) from 8*lam
// consecutive inputs (lam 16-byte loads) when rows are whole chunks, one output otherwise.
#include "common.h"

namespace qblora {

namespace {

template <int LAM>
__global__ __launch_bounds__(256) void k_pool_rows8(const uint4* __restrict__ in, int64_t n_chunks, float scale,
                                                    uint4* __restrict__ out, uint4* __restrict__ out_lo) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;         // output chunk (8 values)
    if (c >= n_chunks) return;
    uint4 v[LAM];
#pragma unroll
    for (int i = 0; i < LAM; ++i) v[i] = in[c * LAM + i];
    float x[8 * LAM];
#pragma unroll
    for (int i = 0; i < LAM; ++i) {
        const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            x[8 * i + 2 * q] = bf16_bits_to_float(w[q] & 0xffffu);
            x[8 * i + 2 * q + 1] = bf16_bits_to_float(w[q] >> 16);
        }
    }
    float o[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        float acc = x[LAM * m];
#pragma unroll
        for (int i = 1; i < LAM; ++i) acc += x[LAM * m + i];
        o[m] = acc * scale;
    }
    const uint4 h = make_uint4(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]), pack_bf16(o[4], o[5]), pack_bf16(o[6], o[7]));
    out[c] = h;
    if (out_lo) {
        const uint32_t hw[4] = {h.x, h.y, h.z, h.w};
        uint32_t lw[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            lw[q] = pack_bf16(o[2 * q] - bf16_bits_to_float(hw[q] & 0xffffu), o[2 * q + 1] - bf16_bits_to_float(hw[q] >> 16));
        out_lo[c] = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    }
}

__global__ __launch_bounds__(256) void k_pool_rows1(const uint16_t* __restrict__ in, int64_t n_out, int lam,
                                                    float scale, uint16_t* __restrict__ out,
                                                    uint16_t* __restrict__ out_lo) {
    const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= n_out) return;
    float acc = 0.0f;
    for (int i = 0; i < lam; ++i) acc += bf16_bits_to_float(in[o * lam + i]);
    const float v = acc * scale;
    const uint32_t h = pack_bf16(v, 0.0f) & 0xffffu;
    out[o] = (uint16_t)h;
    if (out_lo) out_lo[o] = (uint16_t)(pack_bf16(v - bf16_bits_to_float(h), 0.0f) & 0xffffu);
}

// Interval sampling (the "interval_sampling" compress operator of the ablation, Sec. 4.3):
// out[t, c] = in[t, lam*c]; 8 outputs (one 16-byte store) per thread when rows are whole chunks.
__global__ __launch_bounds__(256) void k_sample_rows(const uint16_t* __restrict__ in, int64_t T, int d, int lam,
                                                     uint16_t* __restrict__ out) {
    const int dq = d / lam;
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;   // first of 8 consecutive outputs
    const int64_t total = T * dq;
    if (i >= total) return;
    if ((dq & 7) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        const int64_t t = i / dq;
        const int c = (int)(i - t * dq);
        const uint16_t* src = in + t * d + (int64_t)c * lam;
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = (uint32_t)src[(2 * q) * lam] | ((uint32_t)src[(2 * q + 1) * lam] << 16);
        *reinterpret_cast<uint4*>(out + i) = make_uint4(w[0], w[1], w[2], w[3]);
        return;
    }
    for (int64_t j = i; j < i + 8 && j < total; ++j) {
        const int64_t t = j / dq;
        out[j] = in[t * d + (j - t * dq) * lam];
    }
}

}  // namespace

// in: bf16 [T, d] with d % lam == 0 (rows are contiguous, so the whole matrix is one run of groups of
// lam values); out (and out_lo, or NULL): bf16 [T, d/lam].
int launch_pool_rows(const qblora_bf16* in, int64_t T, int d, int lam, float scale, qblora_bf16* out,
                     qblora_bf16* out_lo, hipStream_t st) {
    const int64_t n_out = T * (int64_t)(d / lam);
    if (n_out <= 0) return QBLORA_OK;
    const bool aligned = ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out) |
                           reinterpret_cast<uintptr_t>(out_lo)) & 15) == 0;
    if (aligned && n_out % 8 == 0 && (lam == 1 || lam == 2 || lam == 4 || lam == 8)) {
        const int64_t n_chunks = n_out / 8;
        const dim3 grid((unsigned)((n_chunks + 255) / 256));
        const uint4* src = reinterpret_cast<const uint4*>(in);
        uint4* dst = reinterpret_cast<uint4*>(out);
        uint4* dlo = reinterpret_cast<uint4*>(out_lo);
        switch (lam) {
            case 1: hipLaunchKernelGGL(k_pool_rows8<1>, grid, dim3(256), 0, st, src, n_chunks, scale, dst, dlo); break;
            case 2: hipLaunchKernelGGL(k_pool_rows8<2>, grid, dim3(256), 0, st, src, n_chunks, scale, dst, dlo); break;
            case 4: hipLaunchKernelGGL(k_pool_rows8<4>, grid, dim3(256), 0, st, src, n_chunks, scale, dst, dlo); break;
            default: hipLaunchKernelGGL(k_pool_rows8<8>, grid, dim3(256), 0, st, src, n_chunks, scale, dst, dlo); break;
        }
    } else {
        hipLaunchKernelGGL(k_pool_rows1, dim3((unsigned)((n_out + 255) / 256)), dim3(256), 0, st,
                           reinterpret_cast<const uint16_t*>(in), n_out, lam, scale, reinterpret_cast<uint16_t*>(out),
                           reinterpret_cast<uint16_t*>(out_lo));
    }
    return launch_status();
}

int launch_sample_rows(const qblora_bf16* in, int64_t T, int d, int lam, qblora_bf16* out, hipStream_t st) {
    if (T <= 0 || d <= 0 || lam <= 0 || d % lam != 0) return QBLORA_ERR_SHAPE;
    const int64_t total = T * (d / lam);
    hipLaunchKernelGGL(k_sample_rows, dim3((unsigned)((total + 2047) / 2048)), dim3(256), 0, st,
                       reinterpret_cast<const uint16_t*>(in), T, d, lam, reinterpret_cast<uint16_t*>(out));
    return launch_status();
}

}  // namespace qblora
