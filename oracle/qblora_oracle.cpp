// CPU oracle for the adapted quantized linear layer (Q-BLoRA / QA-BLoRA).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
// library is checked against.  It is used by the tests, by the smoke check and
// by the benchmark's CPU-baseline leg, never by the product path, and it shares
// no code, table or helper with the GPU kernels.
//
// Conventions
//   * Storage layout of the base weight is [d_out, d_in] row-major (the
//     nn.Linear layout); the paper writes W as D_in x D_out and y = W^T x
//     (Sec. 3.1), so Y = X * Wt^T here.
//   * A quantization block is `block` contiguous input indices k inside one
//     output row n; block b of row n covers k in [b*block, (b+1)*block).
//   * 4-bit codes are packed two per byte: element (n,k) lives in byte
//     (n*d_in+k)/2, even k in the low nibble.
//   * bf16 tensors are passed as uint16 bit patterns and widened exactly.
//   * Forward / backward are evaluated in fp64 from the exact input values with
//     no intermediate rounding.  The integer-producing paths (quantize, merge)
//     follow a fixed sequence of single IEEE fp32 operations (each realised as
//     the fp64 operation followed by one rounding to fp32, which is exact for
//     + - * / because 53 >= 2*24+2), so their outputs are reproducible to the
//     bit.
//   * Parallelism: independent output rows are split over std::thread workers;
//     every output element is produced by exactly one thread with a fixed
//     summation order, so results do not depend on the thread count.
//
// Pins (tests/test_oracle_*.py): brute-force nearest-codebook search, closed
// forms and error bounds of Eq. 1, dense-matmul equivalence with the full-size
// delta weight (Sec. 3.2 "Merging Q-BLoRA", Eq. 2), B = 0 and lambda = 1
// special cases, central finite differences, adjoint identity, merge
// invariants, E4M3 round trips; the single-matrix (QA-BLoRA) layer against the
// dense delta weight, against the two-matrix layer with A = identity and by
// finite differences; the alternative scale operators against dense operator
// matrices, against the default layer (op 0, lambda = 1) and by finite
// differences; the two-dimensional block variants against the row-segment
// functions (br = 1), brute force, and the exactness of the offset-shift merge.
// No function here is unpinned.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>

namespace {

int g_threads = 0;

int n_threads() {
    if (g_threads > 0) return g_threads;
    unsigned hc = std::thread::hardware_concurrency();
    return hc ? (int)hc : 1;
}

// Run fn(begin, end) over [0, n) split into contiguous chunks, one per worker.
void parallel_rows(int64_t n, const std::function<void(int64_t, int64_t)>& fn) {
    int nt = (int)std::min<int64_t>(n_threads(), std::max<int64_t>(n, 1));
    if (nt <= 1) { fn(0, n); return; }
    std::vector<std::thread> pool;
    int64_t chunk = (n + nt - 1) / nt;
    for (int i = 0; i < nt; ++i) {
        int64_t b = i * chunk, e = std::min<int64_t>(n, b + chunk);
        if (b >= e) break;
        pool.emplace_back(fn, b, e);
    }
    for (auto& t : pool) t.join();
}

inline double bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

// one IEEE fp32 operation = fp64 operation + one rounding
inline float f32_add(float a, float b) { return (float)((double)a + (double)b); }
inline float f32_sub(float a, float b) { return (float)((double)a - (double)b); }
inline float f32_mul(float a, float b) { return (float)((double)a * (double)b); }
inline float f32_div(float a, float b) { return (float)((double)a / (double)b); }

// fp32 -> nearest bf16 value (ties to even), returned as fp32
inline float round_to_bf16(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x;  // NaN stays NaN
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    float r;
    std::memcpy(&r, &u, 4);
    return r;
}

inline int get_code(const uint8_t* codes, int64_t idx) {
    uint8_t byte = codes[idx >> 1];
    return (idx & 1) ? (byte >> 4) : (byte & 0xf);
}

inline void put_code(uint8_t* codes, int64_t idx, int code) {
    uint8_t& byte = codes[idx >> 1];
    if (idx & 1) byte = (uint8_t)((byte & 0x0f) | (code << 4));
    else byte = (uint8_t)((byte & 0xf0) | code);
}

// Min-max quantizer of Eq. 1 with alpha = (max-min)/(2^4-1), beta = min
// (Sec. 3.1), applied to one block held in fp32.
void minmax_encode_block(const float* w, int n, int* code, float* alpha, float* beta) {
    float lo = w[0], hi = w[0];
    for (int i = 1; i < n; ++i) { lo = std::min(lo, w[i]); hi = std::max(hi, w[i]); }
    float range = f32_sub(hi, lo);
    *alpha = f32_div(range, 15.0f);
    *beta = lo;
    if (*alpha == 0.0f) {
        for (int i = 0; i < n; ++i) code[i] = 0;
        return;
    }
    float inv = f32_div(15.0f, range);          // one division per block
    for (int i = 0; i < n; ++i) {
        float q = f32_mul(f32_sub(w[i], lo), inv);
        double r = std::nearbyint((double)q);    // ties to even (default rounding mode)
        int c = (int)r;
        code[i] = std::min(15, std::max(0, c));
    }
}

// The OCP 8-bit E4M3 value set: sign, 4 exponent bits (bias 7), 3 mantissa
// bits, no infinities, exponent 15 / mantissa 7 is NaN, largest finite 448.
double e4m3_value(int code7) {   // magnitude of the 7 low bits
    int e = (code7 >> 3) & 0xf, m = code7 & 7;
    if (e == 0) return std::ldexp((double)m / 8.0, -6);
    return std::ldexp(1.0 + (double)m / 8.0, e - 7);
}

}  // namespace

extern "C" {

void oracle_set_threads(int n) { g_threads = n; }
int oracle_get_threads() { return n_threads(); }

// ---------------------------------------------------------------------------
// Block-wise quantizers (Eq. 1, Sec. 3.1)
// ---------------------------------------------------------------------------

// Codebook quantizer with an absmax scale (the NF4-style base of Sec. 3.2):
// alpha = max|w| of the block, code = index of the codebook entry nearest to
// w/alpha.  Nearest is decided by thresholds: m_j = (c_j + c_{j+1}) * 0.5,
// t_j = m_j * alpha, code = #{ j : w > t_j }, so a value exactly on a
// threshold takes the lower index.
void oracle_quantize_codebook(const float* W, int64_t d_out, int64_t d_in, int block,
                              const float* codebook, uint8_t* codes, float* absmax) {
    int64_t bpr = d_in / block;
    std::memset(codes, 0, (size_t)(d_out * d_in / 2));
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t b = 0; b < bpr; ++b) {
                const float* w = W + n * d_in + b * block;
                float a = 0.0f;
                for (int i = 0; i < block; ++i) a = std::max(a, std::fabs(w[i]));
                absmax[n * bpr + b] = a;
                float t[15];
                for (int j = 0; j < 15; ++j) {
                    float m = f32_mul(f32_add(codebook[j], codebook[j + 1]), 0.5f);
                    t[j] = f32_mul(m, a);
                }
                for (int i = 0; i < block; ++i) {
                    int c = 0;
                    for (int j = 0; j < 15; ++j) c += (w[i] > t[j]) ? 1 : 0;
                    put_code(codes, n * d_in + b * block + i, c);
                }
            }
    });
}

// Min-max INT4 quantizer: codes 0..15, alpha = (max-min)/15, beta = min.
void oracle_quantize_minmax(const float* W, int64_t d_out, int64_t d_in, int block,
                            uint8_t* codes, float* alpha, float* beta) {
    int64_t bpr = d_in / block;
    std::memset(codes, 0, (size_t)(d_out * d_in / 2));
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        std::vector<int> c(block);
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t b = 0; b < bpr; ++b) {
                minmax_encode_block(W + n * d_in + b * block, block, c.data(),
                                    &alpha[n * bpr + b], &beta[n * bpr + b]);
                for (int i = 0; i < block; ++i) put_code(codes, n * d_in + b * block + i, c[i]);
            }
    });
}

// ---------------------------------------------------------------------------
// Second-level quantization of the block scales (8-bit E4M3 codes, groups of
// `group` consecutive scales).  Not in the paper; the reading is: per group,
// mid = (min+max)*0.5, d_i = s_i - mid, step = max|d_i| / 448,
// code_i = nearest E4M3 value to d_i/step (ties to the even code, saturating
// at 448), reconstructed scale = fma(value(code_i), step, mid).
// ---------------------------------------------------------------------------
float oracle_e4m3_decode(uint8_t code) {
    double v = e4m3_value(code & 0x7f);
    if ((code & 0x7f) == 0x7f) return std::nanf("");
    return (float)((code & 0x80) ? -v : v);
}

uint8_t oracle_e4m3_encode(float x) {
    double a = std::fabs((double)x);
    int best = 0;
    double best_err = a;   // distance to code 0 (value 0)
    for (int c = 1; c < 0x7f; ++c) {          // 0x7f is NaN, never chosen
        double err = std::fabs(a - e4m3_value(c));
        if (err < best_err || (err == best_err && (c & 1) == 0)) { best = c; best_err = err; }
    }
    return (uint8_t)(best | (std::signbit(x) ? 0x80 : 0));
}

void oracle_scales_double_quantize(const float* scales, int64_t n, int group,
                                   uint8_t* scale_codes, float* step, float* mid) {
    int64_t ng = (n + group - 1) / group;
    for (int64_t g = 0; g < ng; ++g) {
        int64_t b = g * group, e = std::min<int64_t>(n, b + group);
        float lo = scales[b], hi = scales[b];
        for (int64_t i = b + 1; i < e; ++i) { lo = std::min(lo, scales[i]); hi = std::max(hi, scales[i]); }
        float m = f32_mul(f32_add(lo, hi), 0.5f);
        float dmax = 0.0f;
        for (int64_t i = b; i < e; ++i) dmax = std::max(dmax, std::fabs(f32_sub(scales[i], m)));
        mid[g] = m;
        if (dmax == 0.0f) {
            step[g] = 0.0f;
            for (int64_t i = b; i < e; ++i) scale_codes[i] = 0;
            continue;
        }
        float st = f32_div(dmax, 448.0f);
        step[g] = st;
        for (int64_t i = b; i < e; ++i)
            scale_codes[i] = oracle_e4m3_encode(f32_div(f32_sub(scales[i], m), st));
    }
}

void oracle_scales_double_dequantize(const uint8_t* scale_codes, int64_t n, int group,
                                     const float* step, const float* mid, float* scales) {
    for (int64_t i = 0; i < n; ++i)
        scales[i] = std::fmaf(oracle_e4m3_decode(scale_codes[i]), step[i / group], mid[i / group]);
}

// ---------------------------------------------------------------------------
// Dequantize (Eq. 1): w~ = alpha * c[code] + beta, beta = 0 when absent.
//   mode 0: the real-number formula evaluated in fp64
//   mode 1: fp32 arithmetic, c*alpha (one multiply) or fma(c, alpha, beta)
//   mode 3: the small-batch inference weight: the code value is rounded to bf16 (exact for the integer
//           codebook 0..15 of merged INT4 models), scale and offset are applied unrounded -- evaluated in fp64
//   mode 2: mode 1 followed by rounding to bf16 -- the 16-bit compute weight
//           the paper contracts activations with (Sec. 3.1: the dequantized
//           base is held in BF16/FP16)
// ---------------------------------------------------------------------------
void oracle_dequantize(const uint8_t* codes, const float* alpha, const float* beta,
                       const float* codebook, int64_t d_out, int64_t d_in, int block,
                       int mode, double* Wt) {
    int64_t bpr = d_in / block;
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t k = 0; k < d_in; ++k) {
                int64_t blk = n * bpr + k / block;
                float c = codebook[get_code(codes, n * d_in + k)];
                double v;
                if (mode == 0) {
                    v = (double)alpha[blk] * (double)c + (beta ? (double)beta[blk] : 0.0);
                } else if (mode == 3) {
                    v = (double)alpha[blk] * (double)round_to_bf16(c) + (beta ? (double)beta[blk] : 0.0);
                } else {
                    float f = beta ? std::fmaf(c, alpha[blk], beta[blk]) : f32_mul(c, alpha[blk]);
                    v = (double)(mode == 2 ? round_to_bf16(f) : f);
                }
                Wt[n * d_in + k] = v;
            }
    });
}

// ---------------------------------------------------------------------------
// Adapted forward (Sec. 3.2, Alg. 1 qblora_forward with the scaling applied to
// the adapter term only):
//   P[t,m] = (1/lam1) sum_{i<lam1} X[t, lam1*m+i]          AvgPool(lam1)
//   U = P A,  V = U B                                      higher-rank product
//   Y[t,n] = sum_k X[t,k] Wt[n,k] + s * V[t, n / lam2]     repeat_interleave(lam2)
// A is [d_in/lam1, R], B is [R, d_out/lam2], row-major.  A == NULL or R == 0
// gives the base layer.  P_out/U_out/V_out may be NULL.
// ---------------------------------------------------------------------------
void oracle_forward(const double* Wt, int64_t d_out, int64_t d_in, const uint16_t* X, int64_t T,
                    const uint16_t* A, const uint16_t* B, int64_t R, int lam1, int lam2, double s,
                    double* Y, double* P_out, double* U_out, double* V_out) {
    bool adapted = A && B && R > 0;
    int64_t dp = adapted ? d_in / lam1 : 0, dq = adapted ? d_out / lam2 : 0;
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> x(d_in), P(dp), U(R > 0 ? R : 1), V(dq);
        for (int64_t t = t0; t < t1; ++t) {
            for (int64_t k = 0; k < d_in; ++k) x[k] = bf16_to_f64(X[t * d_in + k]);
            if (adapted) {
                for (int64_t m = 0; m < dp; ++m) {
                    double acc = 0.0;
                    for (int i = 0; i < lam1; ++i) acc += x[lam1 * m + i];
                    P[m] = acc / (double)lam1;
                }
                for (int64_t r = 0; r < R; ++r) {
                    double acc = 0.0;
                    for (int64_t m = 0; m < dp; ++m) acc += P[m] * bf16_to_f64(A[m * R + r]);
                    U[r] = acc;
                }
                for (int64_t j = 0; j < dq; ++j) {
                    double acc = 0.0;
                    for (int64_t r = 0; r < R; ++r) acc += U[r] * bf16_to_f64(B[r * dq + j]);
                    V[j] = acc;
                }
                if (P_out) std::copy(P.begin(), P.end(), P_out + t * dp);
                if (U_out) std::copy(U.begin(), U.begin() + R, U_out + t * R);
                if (V_out) std::copy(V.begin(), V.end(), V_out + t * dq);
            }
            for (int64_t n = 0; n < d_out; ++n) {
                const double* w = Wt + n * d_in;
                double acc = 0.0;
                for (int64_t k = 0; k < d_in; ++k) acc += x[k] * w[k];
                if (adapted) acc += s * V[n / lam2];
                Y[t * d_out + n] = acc;
            }
        }
    });
}

// ---------------------------------------------------------------------------
// Backward of the forward above with respect to X, A and B (the base weight is
// frozen, Sec. 3.1).  With G = dY:
//   dV[t,j] = s * sum_{i<lam2} G[t, lam2*j+i]
//   dB = U^T dV,  dU = dV B^T,  dA = P^T dU,  dP = dU A^T
//   dX[t,k] = sum_n G[t,n] Wt[n,k] + (1/lam1) dP[t, k / lam1]
// dX is skipped when compute_dx == 0 (dX may then be NULL); dA/dB are skipped
// when dA == NULL.
// ---------------------------------------------------------------------------
void oracle_backward(const double* Wt, int64_t d_out, int64_t d_in, const uint16_t* X,
                     const uint16_t* dY, int64_t T, const uint16_t* A, const uint16_t* B, int64_t R,
                     int lam1, int lam2, double s, int compute_dx, double* dX, double* dA, double* dB) {
    bool adapted = A && B && R > 0;
    int64_t dp = adapted ? d_in / lam1 : 0, dq = adapted ? d_out / lam2 : 0;
    std::vector<double> P, U, dV, dU;
    if (adapted) {
        P.resize(T * dp); U.resize(T * R); dV.resize(T * dq); dU.resize(T * R);
        parallel_rows(T, [&](int64_t t0, int64_t t1) {
            for (int64_t t = t0; t < t1; ++t) {
                for (int64_t m = 0; m < dp; ++m) {
                    double acc = 0.0;
                    for (int i = 0; i < lam1; ++i) acc += bf16_to_f64(X[t * d_in + lam1 * m + i]);
                    P[t * dp + m] = acc / (double)lam1;
                }
                for (int64_t r = 0; r < R; ++r) {
                    double acc = 0.0;
                    for (int64_t m = 0; m < dp; ++m) acc += P[t * dp + m] * bf16_to_f64(A[m * R + r]);
                    U[t * R + r] = acc;
                }
                for (int64_t j = 0; j < dq; ++j) {
                    double acc = 0.0;
                    for (int i = 0; i < lam2; ++i) acc += bf16_to_f64(dY[t * d_out + lam2 * j + i]);
                    dV[t * dq + j] = s * acc;
                }
                for (int64_t r = 0; r < R; ++r) {
                    double acc = 0.0;
                    for (int64_t j = 0; j < dq; ++j) acc += dV[t * dq + j] * bf16_to_f64(B[r * dq + j]);
                    dU[t * R + r] = acc;
                }
            }
        });
        if (dA) {
            parallel_rows(dp, [&](int64_t m0, int64_t m1) {
                for (int64_t m = m0; m < m1; ++m)
                    for (int64_t r = 0; r < R; ++r) {
                        double acc = 0.0;
                        for (int64_t t = 0; t < T; ++t) acc += P[t * dp + m] * dU[t * R + r];
                        dA[m * R + r] = acc;
                    }
            });
        }
        if (dB) {
            parallel_rows(R, [&](int64_t r0, int64_t r1) {
                for (int64_t r = r0; r < r1; ++r)
                    for (int64_t j = 0; j < dq; ++j) {
                        double acc = 0.0;
                        for (int64_t t = 0; t < T; ++t) acc += U[t * R + r] * dV[t * dq + j];
                        dB[r * dq + j] = acc;
                    }
            });
        }
    }
    if (!compute_dx) return;
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> dP(dp);
        for (int64_t t = t0; t < t1; ++t) {
            double* dx = dX + t * d_in;
            for (int64_t k = 0; k < d_in; ++k) dx[k] = 0.0;
            for (int64_t n = 0; n < d_out; ++n) {
                double g = bf16_to_f64(dY[t * d_out + n]);
                const double* w = Wt + n * d_in;
                for (int64_t k = 0; k < d_in; ++k) dx[k] += g * w[k];
            }
            if (adapted) {
                for (int64_t m = 0; m < dp; ++m) {
                    double acc = 0.0;
                    for (int64_t r = 0; r < R; ++r) acc += dU[t * R + r] * bf16_to_f64(A[m * R + r]);
                    dP[m] = acc;
                }
                for (int64_t k = 0; k < d_in; ++k) dx[k] += dP[k / lam1] / (double)lam1;
            }
        }
    });
}

// ---------------------------------------------------------------------------
// The adapted layer with the alternative non-parametric scale operators of the
// ablation (Sec. 4.3 "The scale operators", Table 6).  The compress operator C
// maps the d_in input features to d_in/lam1, the expand operator E maps the
// d_out/lam2 adapter outputs to d_out features:
//   op 0  AvgPool & repeat_interleave (Sec. 3.2):  P[m] = mean_i x[lam1*m+i];
//         the expanded output at n is V[n / lam2]
//   op 1  truncation & supplement_0:  P[m] = x[m] (the front part is kept);
//         the expanded output at n is V[n] for n < d_out/lam2 and 0 behind it
//   op 2  interval_sampling & interpolation with zeros:  P[m] = x[lam1*m];
//         the expanded output at n is V[n / lam2] where lam2 divides n, else 0
//   Y[t,n] = sum_k X[t,k] Wt[n,k] + s * E(C(x) A B)[n]
// The backward applies the transposed operators: dV = s * E^T(G),
// dB = U^T dV, dU = dV B^T, dA = P^T dU, dX = G Wt + C^T(dU A^T).
// ---------------------------------------------------------------------------
static void compress_row(const double* x, int64_t dp, int lam1, int op, double* P) {
    for (int64_t m = 0; m < dp; ++m) {
        if (op == 0) {
            double acc = 0.0;
            for (int i = 0; i < lam1; ++i) acc += x[lam1 * m + i];
            P[m] = acc / (double)lam1;
        } else if (op == 1) {
            P[m] = x[m];
        } else {
            P[m] = x[(int64_t)lam1 * m];
        }
    }
}

// y[n] += scale * E(V)[n]
static void expand_add_row(const double* V, int64_t dq, int64_t d_out, int lam2, int op, double scale, double* y) {
    for (int64_t n = 0; n < d_out; ++n) {
        if (op == 0) y[n] += scale * V[n / lam2];
        else if (op == 1) { if (n < dq) y[n] += scale * V[n]; }
        else { if (n % lam2 == 0) y[n] += scale * V[n / lam2]; }
    }
}

// dV[j] = scale * E^T(g)[j]
static void expand_transposed_row(const double* g, int64_t dq, int lam2, int op, double scale, double* dV) {
    for (int64_t j = 0; j < dq; ++j) {
        if (op == 0) {
            double acc = 0.0;
            for (int i = 0; i < lam2; ++i) acc += g[lam2 * j + i];
            dV[j] = scale * acc;
        } else if (op == 1) {
            dV[j] = scale * g[j];
        } else {
            dV[j] = scale * g[(int64_t)lam2 * j];
        }
    }
}

// dx[k] += C^T(dP)[k]
static void compress_transposed_add_row(const double* dP, int64_t dp, int64_t d_in, int lam1, int op, double* dx) {
    for (int64_t k = 0; k < d_in; ++k) {
        if (op == 0) dx[k] += dP[k / lam1] / (double)lam1;
        else if (op == 1) { if (k < dp) dx[k] += dP[k]; }
        else { if (k % lam1 == 0) dx[k] += dP[k / lam1]; }
    }
}

void oracle_forward_op(const double* Wt, int64_t d_out, int64_t d_in, const uint16_t* X, int64_t T,
                       const uint16_t* A, const uint16_t* B, int64_t R, int lam1, int lam2, int op, double s,
                       double* Y) {
    const int64_t dp = d_in / lam1, dq = d_out / lam2;
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> x(d_in), P(dp), U(R), V(dq);
        for (int64_t t = t0; t < t1; ++t) {
            for (int64_t k = 0; k < d_in; ++k) x[k] = bf16_to_f64(X[t * d_in + k]);
            compress_row(x.data(), dp, lam1, op, P.data());
            for (int64_t r = 0; r < R; ++r) {
                double acc = 0.0;
                for (int64_t m = 0; m < dp; ++m) acc += P[m] * bf16_to_f64(A[m * R + r]);
                U[r] = acc;
            }
            for (int64_t j = 0; j < dq; ++j) {
                double acc = 0.0;
                for (int64_t r = 0; r < R; ++r) acc += U[r] * bf16_to_f64(B[r * dq + j]);
                V[j] = acc;
            }
            double* y = Y + t * d_out;
            for (int64_t n = 0; n < d_out; ++n) {
                const double* w = Wt + n * d_in;
                double acc = 0.0;
                for (int64_t k = 0; k < d_in; ++k) acc += x[k] * w[k];
                y[n] = acc;
            }
            expand_add_row(V.data(), dq, d_out, lam2, op, s, y);
        }
    });
}

// Wt may be NULL when compute_dx == 0; dA/dB are skipped when dA == NULL.
void oracle_backward_op(const double* Wt, int64_t d_out, int64_t d_in, const uint16_t* X, const uint16_t* dY,
                        int64_t T, const uint16_t* A, const uint16_t* B, int64_t R, int lam1, int lam2, int op,
                        double s, int compute_dx, double* dX, double* dA, double* dB) {
    const int64_t dp = d_in / lam1, dq = d_out / lam2;
    std::vector<double> P(T * dp), U(T * R), dV(T * dq), dU(T * R);
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> x(d_in), g(d_out);
        for (int64_t t = t0; t < t1; ++t) {
            for (int64_t k = 0; k < d_in; ++k) x[k] = bf16_to_f64(X[t * d_in + k]);
            for (int64_t n = 0; n < d_out; ++n) g[n] = bf16_to_f64(dY[t * d_out + n]);
            compress_row(x.data(), dp, lam1, op, &P[t * dp]);
            for (int64_t r = 0; r < R; ++r) {
                double acc = 0.0;
                for (int64_t m = 0; m < dp; ++m) acc += P[t * dp + m] * bf16_to_f64(A[m * R + r]);
                U[t * R + r] = acc;
            }
            expand_transposed_row(g.data(), dq, lam2, op, s, &dV[t * dq]);
            for (int64_t r = 0; r < R; ++r) {
                double acc = 0.0;
                for (int64_t j = 0; j < dq; ++j) acc += dV[t * dq + j] * bf16_to_f64(B[r * dq + j]);
                dU[t * R + r] = acc;
            }
        }
    });
    if (dA) {
        parallel_rows(dp, [&](int64_t m0, int64_t m1) {
            for (int64_t m = m0; m < m1; ++m)
                for (int64_t r = 0; r < R; ++r) {
                    double acc = 0.0;
                    for (int64_t t = 0; t < T; ++t) acc += P[t * dp + m] * dU[t * R + r];
                    dA[m * R + r] = acc;
                }
        });
        parallel_rows(R, [&](int64_t r0, int64_t r1) {
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t j = 0; j < dq; ++j) {
                    double acc = 0.0;
                    for (int64_t t = 0; t < T; ++t) acc += U[t * R + r] * dV[t * dq + j];
                    dB[r * dq + j] = acc;
                }
        });
    }
    if (!compute_dx) return;
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> dP(dp);
        for (int64_t t = t0; t < t1; ++t) {
            double* dx = dX + t * d_in;
            for (int64_t k = 0; k < d_in; ++k) dx[k] = 0.0;
            for (int64_t n = 0; n < d_out; ++n) {
                const double gn = bf16_to_f64(dY[t * d_out + n]);
                const double* w = Wt + n * d_in;
                for (int64_t k = 0; k < d_in; ++k) dx[k] += gn * w[k];
            }
            for (int64_t m = 0; m < dp; ++m) {
                double acc = 0.0;
                for (int64_t r = 0; r < R; ++r) acc += dU[t * R + r] * bf16_to_f64(A[m * R + r]);
                dP[m] = acc;
            }
            compress_transposed_add_row(dP.data(), dp, d_in, lam1, op, dx);
        }
    });
}

// ---------------------------------------------------------------------------
// QA-BLoRA single-matrix adapter (Sec. 3.3, Alg. 2 qablora_forward, scaling on
// the adapter term only): the adapter is one matrix H [d_in/lam1, d_out/lam2],
//   P[t,m] = (1/lam1) sum_{i<lam1} X[t, lam1*m+i]
//   V = P H
//   Y[t,n] = sum_k X[t,k] Wt[n,k] + s * V[t, n / lam2]
// and its backward with respect to X and H (the base weight is frozen):
//   dV[t,j] = s * sum_{i<lam2} G[t, lam2*j+i],  dH = P^T dV,  dP = dV H^T,
//   dX[t,k] = sum_n G[t,n] Wt[n,k] + (1/lam1) dP[t, k / lam1].
// H is bf16 (bit patterns), like the other trainable operands.
// ---------------------------------------------------------------------------
void oracle_qa_forward(const double* Wt, int64_t d_out, int64_t d_in, const uint16_t* X, int64_t T,
                       const uint16_t* H, int lam1, int lam2, double s, double* Y) {
    int64_t dp = d_in / lam1, dq = d_out / lam2;
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> x(d_in), P(dp), V(dq);
        for (int64_t t = t0; t < t1; ++t) {
            for (int64_t k = 0; k < d_in; ++k) x[k] = bf16_to_f64(X[t * d_in + k]);
            for (int64_t m = 0; m < dp; ++m) {
                double acc = 0.0;
                for (int i = 0; i < lam1; ++i) acc += x[lam1 * m + i];
                P[m] = acc / (double)lam1;
            }
            for (int64_t j = 0; j < dq; ++j) V[j] = 0.0;
            for (int64_t m = 0; m < dp; ++m)
                for (int64_t j = 0; j < dq; ++j) V[j] += P[m] * bf16_to_f64(H[m * dq + j]);
            for (int64_t n = 0; n < d_out; ++n) {
                const double* w = Wt + n * d_in;
                double acc = 0.0;
                for (int64_t k = 0; k < d_in; ++k) acc += x[k] * w[k];
                Y[t * d_out + n] = acc + s * V[n / lam2];
            }
        }
    });
}

void oracle_qa_backward(const double* Wt, int64_t d_out, int64_t d_in, const uint16_t* X,
                        const uint16_t* dY, int64_t T, const uint16_t* H, int lam1, int lam2, double s,
                        int compute_dx, double* dX, double* dH) {
    int64_t dp = d_in / lam1, dq = d_out / lam2;
    std::vector<double> P(T * dp), dV(T * dq);
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        for (int64_t t = t0; t < t1; ++t) {
            for (int64_t m = 0; m < dp; ++m) {
                double acc = 0.0;
                for (int i = 0; i < lam1; ++i) acc += bf16_to_f64(X[t * d_in + lam1 * m + i]);
                P[t * dp + m] = acc / (double)lam1;
            }
            for (int64_t j = 0; j < dq; ++j) {
                double acc = 0.0;
                for (int i = 0; i < lam2; ++i) acc += bf16_to_f64(dY[t * d_out + lam2 * j + i]);
                dV[t * dq + j] = s * acc;
            }
        }
    });
    if (dH) {
        parallel_rows(dp, [&](int64_t m0, int64_t m1) {
            for (int64_t m = m0; m < m1; ++m)
                for (int64_t j = 0; j < dq; ++j) {
                    double acc = 0.0;
                    for (int64_t t = 0; t < T; ++t) acc += P[t * dp + m] * dV[t * dq + j];
                    dH[m * dq + j] = acc;
                }
        });
    }
    if (!compute_dx) return;
    parallel_rows(T, [&](int64_t t0, int64_t t1) {
        std::vector<double> dP(dp);
        for (int64_t t = t0; t < t1; ++t) {
            double* dx = dX + t * d_in;
            for (int64_t k = 0; k < d_in; ++k) dx[k] = 0.0;
            for (int64_t n = 0; n < d_out; ++n) {
                double g = bf16_to_f64(dY[t * d_out + n]);
                const double* w = Wt + n * d_in;
                for (int64_t k = 0; k < d_in; ++k) dx[k] += g * w[k];
            }
            for (int64_t m = 0; m < dp; ++m) {
                double acc = 0.0;
                for (int64_t j = 0; j < dq; ++j) acc += dV[t * dq + j] * bf16_to_f64(H[m * dq + j]);
                dP[m] = acc;
            }
            for (int64_t k = 0; k < d_in; ++k) dx[k] += dP[k / lam1] / (double)lam1;
        }
    });
}

// ---------------------------------------------------------------------------
// Tile matrix H = A B ([d_in/lam1, d_out/lam2]) and the equivalent full-size
// delta weight in the paper's D_in x D_out layout (Sec. 3.2 "Merging Q-BLoRA";
// Alg. 1 get_delta_weight): dW[k,n] = H[k/lam1, n/lam2] / lam1 -- each
// (lam1 x lam2) tile holds one value; the 1/lam1 comes from the average pool,
// the output side is a plain copy.
// ---------------------------------------------------------------------------
void oracle_tile_product(const uint16_t* A, const uint16_t* B, int64_t rows, int64_t R, int64_t cols,
                         double* H) {
    parallel_rows(rows, [&](int64_t m0, int64_t m1) {
        for (int64_t m = m0; m < m1; ++m)
            for (int64_t j = 0; j < cols; ++j) {
                double acc = 0.0;
                for (int64_t r = 0; r < R; ++r) acc += bf16_to_f64(A[m * R + r]) * bf16_to_f64(B[r * cols + j]);
                H[m * cols + j] = acc;
            }
    });
}

void oracle_delta_weight(const double* H, int64_t d_in, int64_t d_out, int lam1, int lam2, double* dW) {
    int64_t cols = d_out / lam2;
    for (int64_t k = 0; k < d_in; ++k)
        for (int64_t n = 0; n < d_out; ++n)
            dW[k * d_out + n] = H[(k / lam1) * cols + n / lam2] / (double)lam1;
}

// ---------------------------------------------------------------------------
// QA-BLoRA merge (Sec. 3.3, Alg. 2 get_new_beta).  H is fp32 [d_in/lam1,
// d_out/lam2]; the shift of element (n,k) is delta = (s*H[k/lam1, n/lam2]) / lam1
// in fp32 (one multiply, one division).
//
// beta-shift: allowed when every quantization block lies inside one
// (lam1 x lam2) tile, i.e. lam1 % block == 0 for blocks running along k.
// beta'_b = beta_b + delta (beta absent => delta); codes and alpha untouched.
// Returns 0, or -1 when the alignment condition does not hold.
// ---------------------------------------------------------------------------
int oracle_merge_beta_shift(const float* beta, const float* H, int64_t d_out, int64_t d_in, int block,
                            int lam1, int lam2, float s, float* beta_out) {
    if (lam1 % block != 0) return -1;
    int64_t bpr = d_in / block, cols = d_out / lam2;
    for (int64_t n = 0; n < d_out; ++n)
        for (int64_t b = 0; b < bpr; ++b) {
            int64_t k = b * block;
            float delta = f32_div(f32_mul(s, H[(k / lam1) * cols + n / lam2]), (float)lam1);
            beta_out[n * bpr + b] = beta ? f32_add(beta[n * bpr + b], delta) : delta;
        }
    return 0;
}

// ---------------------------------------------------------------------------
// Two-dimensional quantization blocks (the 4 x 8 and 8 x 8 shapes named in
// Sec. 3.3): a block is br consecutive output rows x bc
// consecutive inputs; its scale / offset live at [(n/br) * (d_in/bc) + k/bc].
// With lam1 % bc == 0 and lam2 % br == 0 every block lies inside one
// (lam1 x lam2) tile of the adapter, so get_new_beta (Alg. 2) is exact: the
// merge is the offset shift alone.  Codes keep the [d_out, d_in/2] packing.
// Elements of a block are visited row by row; br = 1 gives the row-segment
// blocks of the functions above.
// ---------------------------------------------------------------------------
void oracle_quantize_codebook_tile(const float* W, int64_t d_out, int64_t d_in, int br, int bc,
                                   const float* codebook, uint8_t* codes, float* absmax) {
    const int64_t nbr = d_out / br, nbc = d_in / bc;
    std::memset(codes, 0, (size_t)(d_out * d_in / 2));
    parallel_rows(nbr, [&](int64_t r0, int64_t r1) {
        for (int64_t rb = r0; rb < r1; ++rb)
            for (int64_t cbk = 0; cbk < nbc; ++cbk) {
                float a = 0.0f;
                for (int i = 0; i < br; ++i)
                    for (int j = 0; j < bc; ++j) a = std::max(a, std::fabs(W[(rb * br + i) * d_in + cbk * bc + j]));
                absmax[rb * nbc + cbk] = a;
                float t[15];
                for (int j = 0; j < 15; ++j) t[j] = f32_mul(f32_mul(f32_add(codebook[j], codebook[j + 1]), 0.5f), a);
                for (int i = 0; i < br; ++i)
                    for (int j = 0; j < bc; ++j) {
                        const int64_t idx = (rb * br + i) * d_in + cbk * bc + j;
                        int c = 0;
                        for (int q = 0; q < 15; ++q) c += (W[idx] > t[q]) ? 1 : 0;
                        put_code(codes, idx, c);
                    }
            }
    });
}

void oracle_quantize_minmax_tile(const float* W, int64_t d_out, int64_t d_in, int br, int bc,
                                 uint8_t* codes, float* alpha, float* beta) {
    const int64_t nbr = d_out / br, nbc = d_in / bc;
    std::memset(codes, 0, (size_t)(d_out * d_in / 2));
    parallel_rows(nbr, [&](int64_t r0, int64_t r1) {
        std::vector<float> w(br * bc);
        std::vector<int> c(br * bc);
        for (int64_t rb = r0; rb < r1; ++rb)
            for (int64_t cbk = 0; cbk < nbc; ++cbk) {
                for (int i = 0; i < br; ++i)
                    for (int j = 0; j < bc; ++j) w[i * bc + j] = W[(rb * br + i) * d_in + cbk * bc + j];
                minmax_encode_block(w.data(), br * bc, c.data(), &alpha[rb * nbc + cbk], &beta[rb * nbc + cbk]);
                for (int i = 0; i < br; ++i)
                    for (int j = 0; j < bc; ++j) put_code(codes, (rb * br + i) * d_in + cbk * bc + j, c[i * bc + j]);
            }
    });
}

// modes as in oracle_dequantize
void oracle_dequantize_tile(const uint8_t* codes, const float* alpha, const float* beta, const float* codebook,
                            int64_t d_out, int64_t d_in, int br, int bc, int mode, double* Wt) {
    const int64_t nbc = d_in / bc;
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t k = 0; k < d_in; ++k) {
                const int64_t blk = (n / br) * nbc + k / bc;
                const float c = codebook[get_code(codes, n * d_in + k)];
                double v;
                if (mode == 0) {
                    v = (double)alpha[blk] * (double)c + (beta ? (double)beta[blk] : 0.0);
                } else if (mode == 3) {
                    v = (double)alpha[blk] * (double)round_to_bf16(c) + (beta ? (double)beta[blk] : 0.0);
                } else {
                    float f = beta ? std::fmaf(c, alpha[blk], beta[blk]) : f32_mul(c, alpha[blk]);
                    v = (double)(mode == 2 ? round_to_bf16(f) : f);
                }
                Wt[n * d_in + k] = v;
            }
    });
}

// Alg. 2 get_new_beta on two-dimensional blocks: beta' = beta + (s * H[k/lam1, n/lam2]) / lam1 for the
// block at rows n.., inputs k..; -1 when a block would straddle two tiles.
int oracle_merge_beta_shift_tile(const float* beta, const float* H, int64_t d_out, int64_t d_in, int br, int bc,
                                 int lam1, int lam2, float s, float* beta_out) {
    if (lam1 % bc != 0 || lam2 % br != 0) return -1;
    const int64_t nbr = d_out / br, nbc = d_in / bc, cols = d_out / lam2;
    for (int64_t rb = 0; rb < nbr; ++rb)
        for (int64_t cbk = 0; cbk < nbc; ++cbk) {
            const int64_t n = rb * br, k = cbk * bc;
            const float delta = f32_div(f32_mul(s, H[(k / lam1) * cols + n / lam2]), (float)lam1);
            beta_out[rb * nbc + cbk] = beta ? f32_add(beta[rb * nbc + cbk], delta) : delta;
        }
    return 0;
}

// Requantizing merge for tiles that do not cover whole blocks: per block,
// w' = w~ + delta with w~ dequantized in fp32 (mode 1 above), then the min-max
// quantizer of Eq. 1 gives (codes', alpha', beta').
void oracle_merge_requant(const uint8_t* codes, const float* alpha, const float* beta,
                          const float* codebook, const float* H, int64_t d_out, int64_t d_in,
                          int block, int lam1, int lam2, float s,
                          uint8_t* codes_out, float* alpha_out, float* beta_out) {
    int64_t bpr = d_in / block, cols = d_out / lam2;
    std::memset(codes_out, 0, (size_t)(d_out * d_in / 2));
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        std::vector<float> w(block);
        std::vector<int> c(block);
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t b = 0; b < bpr; ++b) {
                int64_t blk = n * bpr + b;
                for (int i = 0; i < block; ++i) {
                    int64_t k = b * block + i;
                    float cv = codebook[get_code(codes, n * d_in + k)];
                    float wt = beta ? std::fmaf(cv, alpha[blk], beta[blk]) : f32_mul(cv, alpha[blk]);
                    float delta = f32_div(f32_mul(s, H[(k / lam1) * cols + n / lam2]), (float)lam1);
                    w[i] = f32_add(wt, delta);
                }
                minmax_encode_block(w.data(), block, c.data(), &alpha_out[blk], &beta_out[blk]);
                for (int i = 0; i < block; ++i) put_code(codes_out, n * d_in + b * block + i, c[i]);
            }
    });
}

// The same requantizing merge on two-dimensional blocks of br output rows x bc inputs (Sec. 3.3 names 4 x 8
// and 8 x 8; block (i, j) has index i*(d_in/bc) + j): per block, w' = w~ + delta element by element in fp32,
// then the min-max quantizer of Eq. 1 over the block's br*bc values.
void oracle_merge_requant_tile(const uint8_t* codes, const float* alpha, const float* beta,
                               const float* codebook, const float* H, int64_t d_out, int64_t d_in,
                               int br, int bc, int lam1, int lam2, float s,
                               uint8_t* codes_out, float* alpha_out, float* beta_out) {
    const int64_t nbr = d_out / br, nbc = d_in / bc, cols = d_out / lam2;
    std::memset(codes_out, 0, (size_t)(d_out * d_in / 2));
    parallel_rows(nbr, [&](int64_t r0, int64_t r1) {
        std::vector<float> w(br * bc);
        std::vector<int> c(br * bc);
        for (int64_t rb = r0; rb < r1; ++rb)
            for (int64_t cbk = 0; cbk < nbc; ++cbk) {
                const int64_t blk = rb * nbc + cbk;
                for (int i = 0; i < br; ++i)
                    for (int j = 0; j < bc; ++j) {
                        const int64_t n = rb * br + i, k = cbk * bc + j;
                        float cv = codebook[get_code(codes, n * d_in + k)];
                        float wt = beta ? std::fmaf(cv, alpha[blk], beta[blk]) : f32_mul(cv, alpha[blk]);
                        float delta = f32_div(f32_mul(s, H[(k / lam1) * cols + n / lam2]), (float)lam1);
                        w[i * bc + j] = f32_add(wt, delta);
                    }
                minmax_encode_block(w.data(), br * bc, c.data(), &alpha_out[blk], &beta_out[blk]);
                for (int i = 0; i < br; ++i)
                    for (int j = 0; j < bc; ++j)
                        put_code(codes_out, (rb * br + i) * d_in + cbk * bc + j, c[i * bc + j]);
            }
    });
}

// ---------------------------------------------------------------------------
// Merge into a 16-bit weight (Sec. 3.2 "Merging Q-BLoRA", Alg. 1 get_delta_weight): W'[n,k] = w~[n,k] +
// delta(n,k), delta = (s*H[k/lam1, n/lam2]) / lam1, with w~ and the sum in fp32 exactly as in the
// requantizing merge above, then one rounding to bf16 (ties to even).  Returns bf16 bit patterns
// [d_out, d_in].
// ---------------------------------------------------------------------------
void oracle_merge_bf16(const uint8_t* codes, const float* alpha, const float* beta, const float* codebook,
                       const float* H, int64_t d_out, int64_t d_in, int block, int lam1, int lam2, float s,
                       uint16_t* W16) {
    int64_t bpr = d_in / block, cols = d_out / lam2;
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t k = 0; k < d_in; ++k) {
                int64_t blk = n * bpr + k / block;
                float cv = codebook[get_code(codes, n * d_in + k)];
                float wt = beta ? std::fmaf(cv, alpha[blk], beta[blk]) : f32_mul(cv, alpha[blk]);
                float delta = f32_div(f32_mul(s, H[(k / lam1) * cols + n / lam2]), (float)lam1);
                float w = f32_add(wt, delta);
                uint32_t bits;
                float r = round_to_bf16(w);
                std::memcpy(&bits, &r, 4);
                W16[n * d_in + k] = (uint16_t)(bits >> 16);
            }
    });
}

// ... and on br x bc blocks (scale and offset of block (n/br, k/bc)).
void oracle_merge_bf16_tile(const uint8_t* codes, const float* alpha, const float* beta, const float* codebook,
                            const float* H, int64_t d_out, int64_t d_in, int br, int bc, int lam1, int lam2, float s,
                            uint16_t* W16) {
    const int64_t nbc = d_in / bc, cols = d_out / lam2;
    parallel_rows(d_out, [&](int64_t n0, int64_t n1) {
        for (int64_t n = n0; n < n1; ++n)
            for (int64_t k = 0; k < d_in; ++k) {
                const int64_t blk = (n / br) * nbc + k / bc;
                float cv = codebook[get_code(codes, n * d_in + k)];
                float wt = beta ? std::fmaf(cv, alpha[blk], beta[blk]) : f32_mul(cv, alpha[blk]);
                float delta = f32_div(f32_mul(s, H[(k / lam1) * cols + n / lam2]), (float)lam1);
                float r = round_to_bf16(f32_add(wt, delta));
                uint32_t bits;
                std::memcpy(&bits, &r, 4);
                W16[n * d_in + k] = (uint16_t)(bits >> 16);
            }
    });
}

}  // extern "C"
