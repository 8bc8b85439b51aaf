// C-ABI entry points (include/qblora.h): host-side validation, workspace layout and kernel
// sequencing.  Every step of the method runs in the kernels; nothing here touches tensor data.
#include <algorithm>
#include <cstring>
#include <mutex>

#include "common.h"

using namespace qblora;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += align_up(count * sizeof(T));
        return r;
    }
};

bool has_adapter(const qblora_adapter* ad) { return ad && ad->A && ad->B && ad->R > 0; }
// Whether the narrow GEMM over `width` features takes the unexpanded adapter operand (pool / repeat factor 2)
bool pooled_pair_operand(int64_t T, int R, int width, int lam) {
    return lam == 2 && skinny_dup_applies(T, R, width, width / 2);
}
int scale_op_of(const qblora_adapter* ad) { return has_adapter(ad) ? ad->scale_op : QBLORA_OP_AVGPOOL_REPEAT; }
// index map of an expanded operand for the compress / expand operator `op`
int op_map(int op) { return op == QBLORA_OP_TRUNCATE_PAD0 ? MAP_FRONT : op == QBLORA_OP_SAMPLE_ZEROFILL ? MAP_STRIDE : MAP_DIV; }

// rows of a quantization block: 1 (row segments of 64 inputs) or 8 (8 x 8 blocks)
int block_rows_of(const qblora_qweight* qw) { return qw->block_rows == 8 ? 8 : 1; }
// inputs per block: 64 (row segments), or with 8-row blocks 8 (block size 64) or 4 (block size 32)
int block_cols_of(const qblora_qweight* qw) { return qw->block_rows == 8 ? qw->block / 8 : qw->block; }
// Blocks of 8 rows x 4 inputs: the kernels that rebuild weights inside a contraction (training calls on few tokens,
// the inference kernels) do not know this shape; every training call takes the dequantize-once form instead.
bool half_blocks(const qblora_qweight* qw) { return qw->block_rows == 8 && qw->block == 32; }

int check_qweight(const qblora_qweight* qw, bool need_codes, bool allow_tile8 = false) {
    if (!qw) return QBLORA_ERR_NULL;
    if (qw->d_out <= 0 || qw->d_in <= 0) return QBLORA_ERR_SHAPE;
    if (qw->block != kBlock && !(qw->block == 32 && qw->block_rows == 8 && allow_tile8))
        return qw->block > 0 ? QBLORA_ERR_UNSUPPORTED : QBLORA_ERR_SHAPE;
    if (qw->d_in % kBlock != 0) return QBLORA_ERR_SHAPE;
    if (qw->block_rows != 0 && qw->block_rows != 1 && qw->block_rows != 8) return QBLORA_ERR_UNSUPPORTED;
    if (qw->block_rows == 8) {
        if (!allow_tile8 || qw->scale_mode != QBLORA_SCALES_FP32) return QBLORA_ERR_UNSUPPORTED;
        if (qw->d_out % 8 != 0) return QBLORA_ERR_SHAPE;
    }
    if (need_codes) {
        if (!qw->codes) return QBLORA_ERR_NULL;
        if (qw->scale_mode == QBLORA_SCALES_FP32) {
            if (!qw->scales) return QBLORA_ERR_NULL;
        } else if (qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED) {
            if (!qw->scale_codes || !qw->scale_step || !qw->scale_mid) return QBLORA_ERR_NULL;
            if (qw->scale_group <= 0) return QBLORA_ERR_SHAPE;
        } else {
            return QBLORA_ERR_UNSUPPORTED;
        }
    }
    return QBLORA_OK;
}

int check_layer(const qblora_qweight* qw, const qblora_adapter* ad) {
    int rc = check_qweight(qw, true, true);
    if (rc) return rc;
    if (qw->d_out % 64 != 0) return QBLORA_ERR_SHAPE;      // contraction step of the transposed use
    if (ad && (ad->A || ad->B || ad->R)) {
        if (ad->R < 0 || ad->lambda1 <= 0 || ad->lambda2 <= 0) return QBLORA_ERR_SHAPE;
        if (has_adapter(ad)) {
            if (qw->d_in % ad->lambda1 != 0 || qw->d_out % ad->lambda2 != 0) return QBLORA_ERR_SHAPE;
            if (ad->R % 8 != 0) return QBLORA_ERR_SHAPE;
            if (ad->scale_op < QBLORA_OP_AVGPOOL_REPEAT || ad->scale_op > QBLORA_OP_SAMPLE_ZEROFILL)
                return QBLORA_ERR_UNSUPPORTED;
            if (ad->scale_op != QBLORA_OP_AVGPOOL_REPEAT &&
                ((qw->d_in / ad->lambda1) % 8 != 0 || (qw->d_out / ad->lambda2) % 8 != 0))
                return QBLORA_ERR_SHAPE;
        } else if (ad->R > 0) {
            return QBLORA_ERR_NULL;                         // a rank was given but a matrix is missing
        }
    }
    return QBLORA_OK;
}

Codebook codebook_of(const qblora_qweight* qw) {
    Codebook cb;
    for (int j = 0; j < 16; ++j) cb.c[j] = qw->codebook[j];
    return cb;
}

int64_t n_blocks(const qblora_qweight* qw) { return (int64_t)qw->d_out * (qw->d_in / qw->block); }

// From this many tokens on, a call dequantizes the weight ONCE into a bf16 buffer in its workspace and contracts
// that (direct copies of both operand tiles); below it, every 256-token tile rebuilds its weight tiles in LDS.
// Rebuilding costs about a quarter of the contraction kernel's time for every token tile; the one-off pass
// costs one sweep over the weight (0.56 B read + 2 B written per element), which 2048 tokens amortize.
constexpr int64_t kDenseMinTokens = 2048;
// (the contraction kernel addresses the dequantized weight with 32-bit byte offsets)
bool use_dense(const qblora_qweight* qw, int64_t T) {
    return (T >= kDenseMinTokens || half_blocks(qw)) && (int64_t)qw->d_out * qw->d_in * 2 < ((int64_t)1 << 32);
}

struct FwdSpace {
    float* scales; qblora_bf16 *At_x, *Bt, *U, *W16;
    size_t bytes;
};
FwdSpace carve_fwd(const qblora_qweight* qw, const qblora_adapter* ad, int64_t T, void* ws, bool dense) {
    Carver c(ws);
    FwdSpace s{};
    if (dense) {
        s.W16 = c.take<qblora_bf16>((size_t)qw->d_out * qw->d_in);
        if (qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED) s.scales = c.take<float>(n_blocks(qw));   // reconstructed
    } else {
        s.scales = c.take<float>((size_t)((qw->d_out + 255) / 256) * 256 * (qw->d_in / qw->block));   // tile-ordered
    }
    if (has_adapter(ad)) {
        s.At_x = c.take<qblora_bf16>((size_t)ad->R * qw->d_in);
        // the alternative scale operators use a full [d_out, R] expansion (zero rows included)
        const size_t bt_rows = scale_op_of(ad) ? (size_t)qw->d_out : (size_t)(qw->d_out / ad->lambda2);
        s.Bt = c.take<qblora_bf16>(bt_rows * ad->R);
        s.U = c.take<qblora_bf16>((size_t)T * ad->R);
    }
    s.bytes = c.off;
    return s;
}

struct BwdSpace {
    float* scales; qblora_bf16 *At_x, *Bx, *U, *U_lo, *dU, *dU_lo, *dUs, *A_op, *Xs, *dYs, *W16t; float *part, *part_b;
    int splits_a, splits_b;
    size_t bytes;
};
BwdSpace carve_bwd(const qblora_qweight* qw, const qblora_adapter* ad, int64_t T, void* ws, bool dense) {
    Carver c(ws);
    BwdSpace s{};
    if (qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED) s.scales = c.take<float>(n_blocks(qw));
    if (dense) s.W16t = c.take<qblora_bf16>((size_t)qw->d_out * qw->d_in);
    if (has_adapter(ad)) {
        s.At_x = c.take<qblora_bf16>((size_t)ad->R * qw->d_in);
        s.Bx = c.take<qblora_bf16>((size_t)ad->R * qw->d_out);
        s.U = c.take<qblora_bf16>((size_t)T * ad->R);
        s.U_lo = c.take<qblora_bf16>((size_t)T * ad->R);
        s.dU = c.take<qblora_bf16>((size_t)T * ad->R);
        s.dU_lo = c.take<qblora_bf16>((size_t)T * ad->R);
        s.dUs = c.take<qblora_bf16>((size_t)T * ad->R);
        s.splits_a = grad_splits(T, qw->d_in);
        s.splits_b = grad_splits(T, qw->d_out);
        size_t pa = (size_t)s.splits_a * qw->d_in * ad->R, pb = (size_t)s.splits_b * qw->d_out * ad->R;
        s.part = c.take<float>(pa);             // dA and dB are computed in one launch: a buffer each
        s.part_b = c.take<float>(pb);
        if (scale_op_of(ad)) s.A_op = c.take<qblora_bf16>((size_t)qw->d_in * ad->R);
        if (scale_op_of(ad) == QBLORA_OP_SAMPLE_ZEROFILL) {
            s.Xs = c.take<qblora_bf16>((size_t)T * (qw->d_in / ad->lambda1));
            s.dYs = c.take<qblora_bf16>((size_t)T * (qw->d_out / ad->lambda2));
        }
    }
    s.bytes = c.off;
    return s;
}

}  // namespace

// measurement hook (qblora_profile_events): the registration belongs to the calling host thread
namespace qblora {
namespace {
thread_local hipEvent_t g_events[QBLORA_PROFILE_SLOTS][2] = {};
}
ProfileScope::ProfileScope(int w, hipStream_t s) : which(w), st(s) {
    if (g_events[which][0]) (void)hipEventRecord(g_events[which][0], st);
}
ProfileScope::~ProfileScope() {
    if (g_events[which][1]) (void)hipEventRecord(g_events[which][1], st);
}
}  // namespace qblora

namespace {

using ScopedEvents = qblora::ProfileScope;

__global__ void k_fill_zero(float* p, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// fp32 block scales the GEMM kernels read: the stored ones, or reconstructed into scratch.
int resolve_scales(const qblora_qweight* qw, float* scratch, hipStream_t st, const float** out) {
    if (qw->scale_mode == QBLORA_SCALES_FP32) { *out = qw->scales; return QBLORA_OK; }
    *out = scratch;
    return launch_scales_reconstruct(qw->scale_codes, qw->scale_step, qw->scale_mid, n_blocks(qw),
                                     qw->scale_group, scratch, st);
}

// ---- QA-BLoRA merge: validation (touches nothing), description + output header, offset-shift launch ------------

int merge_check(const qblora_qweight* base, const float* H, int32_t lambda1, int32_t lambda2, int32_t mode,
                const qblora_qweight* out) {
    int rc = check_qweight(base, true, true);
    if (rc) return rc;
    if (!H || !out) return QBLORA_ERR_NULL;
    if (lambda1 <= 0 || lambda2 <= 0) return QBLORA_ERR_SHAPE;
    if (base->d_in % lambda1 || base->d_out % lambda2) return QBLORA_ERR_SHAPE;
    if (mode != QBLORA_MERGE_BETA_SHIFT && mode != QBLORA_MERGE_REQUANT_MINMAX) return QBLORA_ERR_UNSUPPORTED;
    if (!out->codes || !out->scales || !out->beta) return QBLORA_ERR_NULL;
    if (mode == QBLORA_MERGE_BETA_SHIFT &&
        (block_rows_of(base) == 8 ? (lambda1 % block_cols_of(base) != 0 || lambda2 % 8 != 0) : (lambda1 % base->block != 0)))
        return QBLORA_ERR_ALIGNMENT;
    return QBLORA_OK;
}

// after merge_check: the kernels' description, and the header of `out` (which may alias `base`)
MergeDesc merge_fill(const qblora_qweight* base, const float* H, int32_t lambda1, int32_t lambda2, float s, int32_t mode,
                     qblora_qweight* out) {
    const bool grouped = base->scale_mode == QBLORA_SCALES_E4M3_GROUPED;
    MergeDesc d{};
    d.codes = base->codes; d.scales = base->scales; d.beta = base->beta;
    if (grouped) {
        d.scale_codes = base->scale_codes; d.scale_step = base->scale_step; d.scale_mid = base->scale_mid;
        d.scale_group = base->scale_group;
    }
    d.cb = codebook_of(base); d.d_out = base->d_out; d.d_in = base->d_in;
    d.H = H; d.lam1 = lambda1; d.lam2 = lambda2; d.s = s;
    d.codes_out = out->codes; d.alpha_out = out->scales; d.beta_out = out->beta;
    d.block_rows = block_rows_of(base); d.block_cols = block_cols_of(base);
    float cbk[16];
    std::memcpy(cbk, base->codebook, sizeof(cbk));
    out->d_out = base->d_out; out->d_in = base->d_in; out->block = base->block; out->block_rows = base->block_rows;
    out->scale_mode = QBLORA_SCALES_FP32; out->scale_group = 0;
    out->scale_codes = nullptr; out->scale_step = nullptr; out->scale_mid = nullptr; out->codes_tiled = nullptr;
    if (mode == QBLORA_MERGE_BETA_SHIFT) std::memcpy(out->codebook, cbk, sizeof(cbk));
    else for (int j = 0; j < 16; ++j) out->codebook[j] = (float)j;
    return d;
}

// offset-shift merge: codes and alpha are copied when the output is a separate weight, beta is shifted
int merge_shift(const qblora_qweight* base, const MergeDesc& d, const qblora_qweight* out, hipStream_t st) {
    const bool grouped = d.scale_codes != nullptr;
    if (d.codes_out != d.codes &&
        hipMemcpyAsync(d.codes_out, d.codes, (size_t)d.d_out * d.d_in / 2, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return QBLORA_ERR_LAUNCH;
    if (!grouped && d.alpha_out != d.scales &&
        hipMemcpyAsync(d.alpha_out, d.scales, sizeof(float) * (size_t)n_blocks(base), hipMemcpyDeviceToDevice, st) !=
            hipSuccess)
        return QBLORA_ERR_LAUNCH;
    (void)out;
    ScopedEvents ev(QBLORA_PROFILE_MERGE, st);
    return launch_merge_beta_shift(d, st);
}

}  // namespace

extern "C" {

const char* qblora_strerror(int code) {
    switch (code) {
        case QBLORA_OK: return "ok";
        case QBLORA_ERR_NULL: return "a required pointer is NULL";
        case QBLORA_ERR_SHAPE: return "a size is non-positive or not divisible as the method requires";
        case QBLORA_ERR_UNSUPPORTED: return "configuration not implemented by these kernels";
        case QBLORA_ERR_WORKSPACE: return "workspace missing or too small";
        case QBLORA_ERR_ALIGNMENT: return "beta-shift merge needs every quantization block inside one adapter tile";
        case QBLORA_ERR_LAUNCH: return "the HIP runtime refused a launch";
        default: return "unknown error code";
    }
}

int qblora_profile_events(int32_t which, void* start_event, void* stop_event) {
    if (which < 0 || which >= QBLORA_PROFILE_SLOTS) return QBLORA_ERR_SHAPE;
    if ((start_event == nullptr) != (stop_event == nullptr)) return QBLORA_ERR_NULL;
    qblora::g_events[which][0] = static_cast<hipEvent_t>(start_event);
    qblora::g_events[which][1] = static_cast<hipEvent_t>(stop_event);
    return QBLORA_OK;
}

int qblora_quantize_blockwise(const float* W, int32_t d_out, int32_t d_in, int32_t block, int32_t quantizer,
                              const float* codebook, int32_t scale_mode, qblora_qweight* out, void* stream) {
    if (!W || !out) return QBLORA_ERR_NULL;
    if (d_out <= 0 || d_in <= 0 || block <= 0) return QBLORA_ERR_SHAPE;
    if (block != kBlock && !(block == 32 && out->block_rows == 8)) return QBLORA_ERR_UNSUPPORTED;
    if (d_in % kBlock != 0) return QBLORA_ERR_SHAPE;
    if (quantizer != QBLORA_QUANT_ABSMAX_CODEBOOK && quantizer != QBLORA_QUANT_MINMAX_INT4)
        return QBLORA_ERR_UNSUPPORTED;
    if (scale_mode != QBLORA_SCALES_FP32 && scale_mode != QBLORA_SCALES_E4M3_GROUPED) return QBLORA_ERR_UNSUPPORTED;
    if (!out->codes || !out->scales) return QBLORA_ERR_NULL;
    if (out->block_rows != 0 && out->block_rows != 1 && out->block_rows != 8) return QBLORA_ERR_UNSUPPORTED;
    const int block_rows = out->block_rows == 8 ? 8 : 1;
    if (block_rows == 8 && scale_mode != QBLORA_SCALES_FP32) return QBLORA_ERR_UNSUPPORTED;
    if (block_rows == 8 && d_out % 8 != 0) return QBLORA_ERR_SHAPE;
    hipStream_t st = as_stream(stream);
    if (quantizer == QBLORA_QUANT_MINMAX_INT4) {
        if (scale_mode != QBLORA_SCALES_FP32) return QBLORA_ERR_UNSUPPORTED;
        if (!out->beta) return QBLORA_ERR_NULL;
    } else {
        if (!codebook) return QBLORA_ERR_NULL;
        for (int j = 0; j < 15; ++j)
            if (!(codebook[j] < codebook[j + 1])) return QBLORA_ERR_SHAPE;
        if (scale_mode == QBLORA_SCALES_E4M3_GROUPED &&
            (!out->scale_codes || !out->scale_step || !out->scale_mid))
            return QBLORA_ERR_NULL;
    }
    out->d_out = d_out; out->d_in = d_in; out->block = block; out->scale_mode = scale_mode;
    out->scale_group = 256;
    if (quantizer == QBLORA_QUANT_MINMAX_INT4) {
        for (int j = 0; j < 16; ++j) out->codebook[j] = (float)j;
        ScopedEvents ev(QBLORA_PROFILE_QUANTIZE, st);
        return launch_quantize_minmax(W, d_out, d_in, out->codes, out->codes_tiled, out->scales, out->beta, st, block_rows,
                                      block_rows == 8 ? block / 8 : 8);
    }
    Codebook cb;
    for (int j = 0; j < 16; ++j) { cb.c[j] = codebook[j]; out->codebook[j] = codebook[j]; }
    out->beta = nullptr;
    int rc;
    {
        ScopedEvents ev(QBLORA_PROFILE_QUANTIZE, st);
        rc = launch_quantize_codebook(W, d_out, d_in, cb, out->codes, out->codes_tiled, out->scales, st, block_rows,
                                      block_rows == 8 ? block / 8 : 8);
    }
    if (rc) return rc;
    if (scale_mode == QBLORA_SCALES_E4M3_GROUPED)
        rc = launch_scales_double_quantize(out->scales, n_blocks(out), out->scale_group, out->scale_codes,
                                           out->scale_step, out->scale_mid, st);
    return rc;
}

size_t qblora_codes_tiled_bytes(int32_t d_out, int32_t d_in) {
    if (d_out <= 0 || d_in <= 0 || d_in % kBlock != 0) return 0;
    return (size_t)((d_out + 255) / 256) * 256 * (size_t)(d_in / 2);
}

int qblora_prepack_codes(const qblora_qweight* qw, void* stream) {
    int rc = check_qweight(qw, false, true);                 // the code packing does not depend on the block shape
    if (rc) return rc;
    if (!qw->codes || !qw->codes_tiled) return QBLORA_ERR_NULL;
    return launch_prepack_codes(qw->codes, qw->d_out, qw->d_in, qw->codes_tiled, as_stream(stream));
}

int qblora_dequantize_bf16(const qblora_qweight* qw, qblora_bf16* Wt, void* stream) {
    int rc = check_qweight(qw, true, true);
    if (rc) return rc;
    if (!Wt) return QBLORA_ERR_NULL;
    if (qw->scale_mode != QBLORA_SCALES_FP32) return QBLORA_ERR_UNSUPPORTED;   // reconstruct needs scratch
    return launch_dequantize_bf16(*qw, qw->scales, Wt, as_stream(stream));
}

size_t qblora_linear_fwd_workspace_bytes(const qblora_qweight* qw, const qblora_adapter* ad, int64_t T) {
    if (check_layer(qw, ad) || T < 0) return 0;
    return carve_fwd(qw, ad, T, nullptr, use_dense(qw, T)).bytes;
}

size_t qblora_linear_bwd_workspace_bytes(const qblora_qweight* qw, const qblora_adapter* ad, int64_t T) {
    if (check_layer(qw, ad) || T < 0) return 0;
    return carve_bwd(qw, ad, T, nullptr, use_dense(qw, T)).bytes;
}

int64_t qblora_dense_min_tokens(void) { return kDenseMinTokens; }

size_t qblora_saved_bytes(const qblora_adapter* ad, int64_t T) {
    if (!has_adapter(ad) || T <= 0) return 0;
    return (size_t)2 * (size_t)T * (size_t)ad->R * sizeof(qblora_bf16);
}

namespace {

int linear_fwd_impl(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                    qblora_bf16* Y, qblora_bf16* saved, void* workspace, size_t workspace_bytes, void* stream,
                    bool allow_dense = true) {
    int rc = check_layer(qw, ad);
    if (rc) return rc;
    if (T < 0) return QBLORA_ERR_SHAPE;
    if (T == 0) return QBLORA_OK;
    if (!X || !Y) return QBLORA_ERR_NULL;
    const bool dense = allow_dense && use_dense(qw, T);
    if (half_blocks(qw) && !dense) return QBLORA_ERR_UNSUPPORTED;
    FwdSpace ws = carve_fwd(qw, ad, T, workspace, dense);
    if (ws.bytes > 0 && (!workspace || workspace_bytes < ws.bytes)) return QBLORA_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    const bool adapted = has_adapter(ad);

    GemmDesc g{};
    g.qmode = dense ? 3 : 1;
    // one launch re-orders the block scales for the forward kernel (reconstructing grouped ones) and,
    // with an adapter, builds its K-contiguous operands
    ScaleTiling sct{};
    const bool grouped = qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED;
    sct.scales = grouped ? nullptr : qw->scales;
    if (grouped) { sct.scale_codes = qw->scale_codes; sct.scale_step = qw->scale_step; sct.scale_mid = qw->scale_mid; }
    sct.scale_group = qw->scale_group; sct.d_out = qw->d_out; sct.d_in = qw->d_in; sct.out = ws.scales;
    g.scales = nullptr; g.scales_tiled = ws.scales;
    g.block_rows = block_rows_of(qw);
    if (g.block_rows == 8) { sct.out = nullptr; g.scales = qw->scales; g.scales_tiled = nullptr; }   // read in place
    if (dense) {
        // the weight once, as the bf16 compute weight of Eq. 1, for all token tiles of this call
        sct.out = nullptr;
        const float* plain = nullptr;
        if ((rc = resolve_scales(qw, ws.scales, st, &plain))) return rc;
        {
            ScopedEvents ev(QBLORA_PROFILE_DEQUANT, st);
            rc = launch_dequantize_operand(*qw, plain, 0, ws.W16, st);
        }
        if (rc) return rc;
        g.W1 = ws.W16; g.K1 = qw->d_in;
    }
    const int op = scale_op_of(ad);
    const bool prep_adapter = adapted && op == QBLORA_OP_AVGPOOL_REPEAT;
    // lambda1 = 2: A^T stays unexpanded and the narrow GEMM uses each of its columns for two adjacent k
    const bool dup_a = prep_adapter && pooled_pair_operand(T, ad->R, qw->d_in, ad->lambda1);
    {
        ScopedEvents ev(QBLORA_PROFILE_PREP, st);
        rc = launch_adapter_prep(prep_adapter ? ad->A : nullptr, prep_adapter ? ad->B : nullptr,
                                 dup_a ? qw->d_in / 2 : qw->d_in, qw->d_out,
                                 adapted ? ad->R : 0, adapted ? (dup_a ? 1 : ad->lambda1) : 1, adapted ? ad->lambda2 : 1,
                                 ws.At_x, ws.Bt, nullptr, st, sct.out ? &sct : nullptr);
    }
    if (rc) return rc;
    if (adapted && op != QBLORA_OP_AVGPOOL_REPEAT) {
        // At_x[j][k] = A[C-map(k)][j] and Bt[n][j] = B[j][E-map(n)], zero where the operator drops the index
        const int na = qw->d_in / ad->lambda1, nb = qw->d_out / ad->lambda2;
        if ((rc = launch_expand_op(ad->A, ad->R, na, 1, ad->R, qw->d_in, MAP_ID, 1, op_map(op), ad->lambda1, ws.At_x, st)))
            return rc;
        if ((rc = launch_expand_op(ad->B, nb, ad->R, 1, qw->d_out, ad->R, op_map(op), ad->lambda2, MAP_ID, 1, ws.Bt, st)))
            return rc;
    }
    if (adapted) {
        // s*U = (s/lambda1) * X * expand(A): average pool folded into the contraction
        GemmDesc u{};
        u.qmode = 0;
        u.X2 = X; u.ldx2 = qw->d_in; u.W2 = ws.At_x; u.ldw2 = qw->d_in; u.K2 = qw->d_in; u.div2 = 1;
        if (dup_a) { u.ldw2 = qw->d_in / 2; u.dup2 = 2; }
        qblora_bf16* su = saved ? saved : ws.U;               // kept for the backward: high part, then residual
        u.C = su; u.C_lo = saved ? saved + T * ad->R : nullptr;
        u.ldc = ad->R; u.out_scale = op ? ad->s : ad->s / (float)ad->lambda1; u.M = T; u.N = ad->R;
        {
            ScopedEvents ev(QBLORA_PROFILE_ADAPTER_FWD, st);
            rc = launch_gemm(u, st);
        }
        if (rc) return rc;
        g.X2 = su; g.ldx2 = ad->R; g.W2 = ws.Bt; g.ldw2 = ad->R; g.K2 = ad->R; g.div2 = op ? 1 : ad->lambda2;
    } else {
        g.K2 = 0; g.div2 = 1;
    }
    g.X1 = X; g.ldx1 = qw->d_in;
    g.codes = qw->codes; g.beta = qw->beta; g.d_out = qw->d_out; g.d_in = qw->d_in; g.cb = codebook_of(qw);
    g.codes_tiled = qw->codes_tiled;
    g.C = Y; g.ldc = qw->d_out; g.out_scale = 1.0f; g.M = T; g.N = qw->d_out;
    ScopedEvents ev(QBLORA_PROFILE_FWD_GEMM, st);
    return launch_gemm(g, st);
}

int linear_bwd_impl(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X,
                    const qblora_bf16* dY, int64_t T, const qblora_bf16* saved, qblora_bf16* dX, float* dA,
                    float* dB, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_layer(qw, ad);
    if (rc) return rc;
    if (T < 0) return QBLORA_ERR_SHAPE;
    const bool adapted = has_adapter(ad);
    const bool want_grads = dA || dB;
    if (want_grads && !(dA && dB)) return QBLORA_ERR_NULL;
    if (want_grads && !adapted) return QBLORA_ERR_NULL;
    if (!dX && !want_grads) return QBLORA_ERR_NULL;
    hipStream_t st = as_stream(stream);
    if (T == 0) {
        if (want_grads) {
            int64_t na = (int64_t)(qw->d_in / ad->lambda1) * ad->R, nb = (int64_t)ad->R * (qw->d_out / ad->lambda2);
            hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, st, dA, na);
            hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, st, dB, nb);
            return launch_status();
        }
        return QBLORA_OK;
    }
    if (!dY || (adapted && !X)) return QBLORA_ERR_NULL;
    const bool dense = use_dense(qw, T) && dX;
    if (half_blocks(qw) && dX && !dense) return QBLORA_ERR_UNSUPPORTED;
    BwdSpace ws = carve_bwd(qw, ad, T, workspace, use_dense(qw, T));
    if (ws.bytes > 0 && (!workspace || workspace_bytes < ws.bytes)) return QBLORA_ERR_WORKSPACE;

    GemmDesc g{};
    g.qmode = dense ? 3 : 2;
    g.block_rows = block_rows_of(qw);
    if (dX && (rc = resolve_scales(qw, ws.scales, st, &g.scales))) return rc;
    if (dense) {
        // the transposed bf16 compute weight once, for all token tiles of this call
        {
            ScopedEvents ev(QBLORA_PROFILE_DEQUANT, st);
            rc = launch_dequantize_operand(*qw, g.scales, 1, ws.W16t, st);
        }
        if (rc) return rc;
        g.W1 = ws.W16t; g.K1 = qw->d_out;
    }
    if (adapted) {
        const int R = ad->R;
        const int op = scale_op_of(ad);
        const int na = qw->d_in / ad->lambda1, nb = qw->d_out / ad->lambda2;
        // lambda = 2: the narrow GEMMs read B (and A^T) unexpanded, each column serving two adjacent features
        const bool dup_b = op == QBLORA_OP_AVGPOOL_REPEAT && pooled_pair_operand(T, R, qw->d_out, ad->lambda2) &&
                           (reinterpret_cast<uintptr_t>(ad->B) & 15) == 0;      // B is copied in 16-byte chunks
        const bool dup_a = op == QBLORA_OP_AVGPOOL_REPEAT && pooled_pair_operand(T, R, qw->d_in, ad->lambda1);
        if (op == QBLORA_OP_AVGPOOL_REPEAT) {
            if ((rc = launch_adapter_prep(ad->A, ad->B, dup_a ? qw->d_in / 2 : qw->d_in, qw->d_out, R,
                                          dup_a ? 1 : ad->lambda1, ad->lambda2,
                                          (want_grads && !saved) ? ws.At_x : nullptr, nullptr, dup_b ? nullptr : ws.Bx, st)))
                return rc;
        } else {
            // Bx[j][n] = B[j][E-map(n)], A_op[k][j] = A[C-map(k)][j] (and At_x as in the forward), zeros elsewhere
            if ((rc = launch_expand_op(ad->B, R, nb, 0, R, qw->d_out, MAP_ID, 1, op_map(op), ad->lambda2, ws.Bx, st)))
                return rc;
            if (dX && (rc = launch_expand_op(ad->A, na, R, 0, qw->d_in, R, op_map(op), ad->lambda1, MAP_ID, 1, ws.A_op, st)))
                return rc;
            if (want_grads && !saved &&
                (rc = launch_expand_op(ad->A, R, na, 1, R, qw->d_in, MAP_ID, 1, op_map(op), ad->lambda1, ws.At_x, st)))
                return rc;
        }
        // dU = s * dY * expand(B)^T (sum pool over lambda2 folded into the contraction); dUs = dU/lambda1
        GemmDesc du{};
        du.qmode = 0;
        du.X2 = dY; du.ldx2 = qw->d_out; du.W2 = ws.Bx; du.ldw2 = qw->d_out; du.K2 = qw->d_out; du.div2 = 1;
        if (dup_b) { du.W2 = ad->B; du.ldw2 = nb; du.dup2 = 2; }
        du.C = ws.dU; du.ldc = R; du.out_scale = ad->s; du.C2 = ws.dUs; du.c2_scale = op ? 1.0f : 1.0f / (float)ad->lambda1;
        du.C_lo = want_grads ? ws.dU_lo : nullptr;
        du.M = T; du.N = R;
        {
            ScopedEvents ev(QBLORA_PROFILE_ADAPTER_BWD, st);
            rc = launch_gemm(du, st);
        }
        if (rc) return rc;
        if (want_grads) {
            const qblora_bf16* su = saved; const qblora_bf16* su_lo = saved ? saved + T * R : nullptr;
            if (!saved) {                                     // s*U again from X, as the forward computed it
                GemmDesc u{};
                u.qmode = 0;
                u.X2 = X; u.ldx2 = qw->d_in; u.W2 = ws.At_x; u.ldw2 = qw->d_in; u.K2 = qw->d_in; u.div2 = 1;
                if (dup_a) { u.ldw2 = qw->d_in / 2; u.dup2 = 2; }
                u.C = ws.U; u.ldc = R; u.out_scale = op ? ad->s : ad->s / (float)ad->lambda1; u.M = T; u.N = R; u.C_lo = ws.U_lo;
                if ((rc = launch_gemm(u, st))) return rc;
                su = ws.U; su_lo = ws.U_lo;
            }
            GradDesc ga{};
            ga.L = X; ga.ldl = qw->d_in; ga.I = qw->d_in; ga.S = ws.dU; ga.S_lo = ws.dU_lo; ga.lds = R; ga.J = R; ga.T = T;
            ga.part = ws.part; ga.splits = ws.splits_a; ga.out = dA; ga.pool = ad->lambda1;
            ga.out_scale = 1.0f / (float)ad->lambda1; ga.transpose_out = 0;
            GradDesc gb{};
            gb.L = dY; gb.ldl = qw->d_out; gb.I = qw->d_out; gb.S = su; gb.S_lo = su_lo; gb.lds = R; gb.J = R; gb.T = T;
            gb.part = ws.part_b; gb.splits = ws.splits_b; gb.out = dB; gb.pool = ad->lambda2;
            gb.out_scale = 1.0f; gb.transpose_out = 1;
            if (op != QBLORA_OP_AVGPOOL_REPEAT) {
                // dA = C(X)^T dU and dB = (sU)^T E^T(dY): the kept features are the first ones of each
                // row (truncation) or are gathered into a dense copy first (interval sampling)
                ga.I = na; ga.pool = 1; ga.out_scale = 1.0f;
                gb.I = nb; gb.pool = 1;
                if (op == QBLORA_OP_SAMPLE_ZEROFILL) {
                    if ((rc = launch_sample_rows(X, T, qw->d_in, ad->lambda1, ws.Xs, st))) return rc;
                    if ((rc = launch_sample_rows(dY, T, qw->d_out, ad->lambda2, ws.dYs, st))) return rc;
                    ga.L = ws.Xs; ga.ldl = na; gb.L = ws.dYs; gb.ldl = nb;
                }
            }
            if ((rc = launch_grad_pair(ga, gb, st))) return rc;
        }
        g.X2 = ws.dUs; g.ldx2 = R; g.K2 = R;
        if (op == QBLORA_OP_AVGPOOL_REPEAT) { g.W2 = ad->A; g.ldw2 = R; g.div2 = ad->lambda1; }
        else { g.W2 = ws.A_op; g.ldw2 = R; g.div2 = 1; }
    } else {
        g.K2 = 0; g.div2 = 1;
    }
    if (!dX) return QBLORA_OK;
    g.X1 = dY; g.ldx1 = qw->d_out;
    g.codes = qw->codes; g.beta = qw->beta; g.d_out = qw->d_out; g.d_in = qw->d_in; g.cb = codebook_of(qw);
    g.C = dX; g.ldc = qw->d_in; g.out_scale = 1.0f; g.M = T; g.N = qw->d_in;
    ScopedEvents ev(QBLORA_PROFILE_BWD_GEMM, st);
    return launch_gemm(g, st);
}

}  // namespace

int qblora_linear_fwd(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                      qblora_bf16* Y, void* workspace, size_t workspace_bytes, void* stream) {
    return linear_fwd_impl(qw, ad, X, T, Y, nullptr, workspace, workspace_bytes, stream);
}

int qblora_linear_fwd_save(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                           qblora_bf16* Y, qblora_bf16* saved, void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (has_adapter(ad) && T > 0 && !saved) return QBLORA_ERR_NULL;
    return linear_fwd_impl(qw, ad, X, T, Y, has_adapter(ad) ? saved : nullptr, workspace, workspace_bytes, stream);
}

int qblora_linear_bwd(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X,
                      const qblora_bf16* dY, int64_t T, qblora_bf16* dX, float* dA, float* dB,
                      void* workspace, size_t workspace_bytes, void* stream) {
    return linear_bwd_impl(qw, ad, X, dY, T, nullptr, dX, dA, dB, workspace, workspace_bytes, stream);
}

int qblora_linear_bwd_saved(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X,
                            const qblora_bf16* dY, int64_t T, const qblora_bf16* saved, qblora_bf16* dX,
                            float* dA, float* dB, void* workspace, size_t workspace_bytes, void* stream) {
    if (has_adapter(ad) && T > 0 && (dA || dB) && !saved) return QBLORA_ERR_NULL;
    return linear_bwd_impl(qw, ad, X, dY, T, has_adapter(ad) ? saved : nullptr, dX, dA, dB, workspace,
                           workspace_bytes, stream);
}

// ---- forward on a scratch array of the library's own -----------------------------------------------

namespace {

constexpr size_t kStaticScratchBytes = QBLORA_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// Scratch of qblora_linear_fwd_noalloc.  Every GPU the library runs on holds its own copy of the array at
// its own address; in host code the name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QBLORA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QBLORA_ERR_LAUNCH;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return QBLORA_OK;
}

}  // namespace

size_t qblora_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

int qblora_linear_fwd_noalloc(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                              qblora_bf16* Y, void* stream) {
    int rc = check_layer(qw, ad);
    if (rc) return rc;
    if (T < 0) return QBLORA_ERR_SHAPE;
    if (T == 0) return QBLORA_OK;
    if (!X || !Y) return QBLORA_ERR_NULL;
    // always the form that rebuilds weight tiles in LDS: its scratch does not grow with the weight
    if (carve_fwd(qw, ad, T, nullptr, false).bytes > kStaticScratchBytes) return QBLORA_ERR_WORKSPACE;
    void* ptr = nullptr;
    if ((rc = static_scratch(&ptr))) return rc;
    // every part of the forward's scratch is written by this call's own kernels before it is read, so
    // nothing has to be cleared between calls
    return linear_fwd_impl(qw, ad, X, T, Y, nullptr, ptr, kStaticScratchBytes, stream, false);
}

// ---- single-matrix adapter (QA-BLoRA) ------------------------------------------------------------

namespace {

int check_qa(const qblora_qweight* qw, const qblora_bf16* H, int32_t lam1, int32_t lam2) {
    int rc = check_qweight(qw, true, true);
    if (rc) return rc;
    if (qw->d_out % 64 != 0) return QBLORA_ERR_SHAPE;
    if (!H) return QBLORA_ERR_NULL;
    if (lam1 <= 0 || lam2 <= 0 || qw->d_in % lam1 != 0 || qw->d_out % lam2 != 0) return QBLORA_ERR_SHAPE;
    // the pooled widths are contraction lengths of 16-byte chunk copies
    if ((qw->d_in / lam1) % 8 != 0 || (qw->d_out / lam2) % 8 != 0) return QBLORA_ERR_SHAPE;
    return QBLORA_OK;
}

struct QaFwdSpace { float* scales; qblora_bf16 *Ht, *P, *W16; size_t bytes; };
QaFwdSpace carve_qa_fwd(const qblora_qweight* qw, int lam1, int lam2, int64_t T, void* ws) {
    Carver c(ws);
    QaFwdSpace s{};
    if (use_dense(qw, T)) {
        s.W16 = c.take<qblora_bf16>((size_t)qw->d_out * qw->d_in);
        if (qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED) s.scales = c.take<float>(n_blocks(qw));
    } else {
        s.scales = c.take<float>((size_t)((qw->d_out + 255) / 256) * 256 * (qw->d_in / qw->block));
    }
    s.Ht = c.take<qblora_bf16>((size_t)(qw->d_out / lam2) * (qw->d_in / lam1));
    s.P = c.take<qblora_bf16>((size_t)T * (qw->d_in / lam1));
    s.bytes = c.off;
    return s;
}

struct QaBwdSpace { float* scales; qblora_bf16 *P, *dVs, *dVs_lo, *W16t; float* part; int splits; size_t bytes; };
QaBwdSpace carve_qa_bwd(const qblora_qweight* qw, int lam1, int lam2, int64_t T, void* ws) {
    Carver c(ws);
    QaBwdSpace s{};
    const int I = qw->d_in / lam1, J = qw->d_out / lam2;
    if (qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED) s.scales = c.take<float>(n_blocks(qw));
    if (use_dense(qw, T)) s.W16t = c.take<qblora_bf16>((size_t)qw->d_out * qw->d_in);
    s.P = c.take<qblora_bf16>((size_t)T * I);
    s.dVs = c.take<qblora_bf16>((size_t)T * J);
    s.dVs_lo = c.take<qblora_bf16>((size_t)T * J);
    s.splits = grad_splits(T, I, J);
    s.part = c.take<float>((size_t)s.splits * I * J);
    s.bytes = c.off;
    return s;
}

}  // namespace

size_t qablora_linear_fwd_workspace_bytes(const qblora_qweight* qw, int32_t lambda1, int32_t lambda2, int64_t T) {
    if (check_qweight(qw, false, true) || lambda1 <= 0 || lambda2 <= 0 || T < 0) return 0;
    return carve_qa_fwd(qw, lambda1, lambda2, T, nullptr).bytes;
}

size_t qablora_linear_bwd_workspace_bytes(const qblora_qweight* qw, int32_t lambda1, int32_t lambda2, int64_t T) {
    if (check_qweight(qw, false, true) || lambda1 <= 0 || lambda2 <= 0 || T < 0) return 0;
    return carve_qa_bwd(qw, lambda1, lambda2, T, nullptr).bytes;
}

int qablora_linear_fwd(const qblora_qweight* qw, const qblora_bf16* H, int32_t lambda1, int32_t lambda2, float s,
                       const qblora_bf16* X, int64_t T, qblora_bf16* Y, void* workspace, size_t workspace_bytes,
                       void* stream) {
    int rc = check_qa(qw, H, lambda1, lambda2);
    if (rc) return rc;
    if (T < 0) return QBLORA_ERR_SHAPE;
    if (T == 0) return QBLORA_OK;
    if (!X || !Y) return QBLORA_ERR_NULL;
    QaFwdSpace ws = carve_qa_fwd(qw, lambda1, lambda2, T, workspace);
    if (!workspace || workspace_bytes < ws.bytes) return QBLORA_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    const int I = qw->d_in / lambda1, J = qw->d_out / lambda2;

    // block scales in tile order and H^T (the K-contiguous weight operand of the K-extension), one launch
    ScaleTiling sct{};
    const bool grouped = qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED;
    sct.scales = grouped ? nullptr : qw->scales;
    if (grouped) { sct.scale_codes = qw->scale_codes; sct.scale_step = qw->scale_step; sct.scale_mid = qw->scale_mid; }
    sct.scale_group = qw->scale_group; sct.d_out = qw->d_out; sct.d_in = qw->d_in; sct.out = ws.scales;
    const bool tile8 = block_rows_of(qw) == 8;               // 8 x 8 blocks: scales are read in place
    const bool dense = use_dense(qw, T);                     // many tokens: the weight is dequantized once
    if (half_blocks(qw) && !dense) return QBLORA_ERR_UNSUPPORTED;
    if (tile8 || dense) sct.out = nullptr;
    if ((rc = launch_adapter_prep(H, H, I, J, J, 1, 1, ws.Ht, nullptr, nullptr, st, sct.out ? &sct : nullptr))) return rc;
    if (dense) {
        const float* plain = nullptr;
        if ((rc = resolve_scales(qw, ws.scales, st, &plain))) return rc;
        if ((rc = launch_dequantize_operand(*qw, plain, 0, ws.W16, st))) return rc;
    }
    // s * AvgPool_lambda1(X)
    if ((rc = launch_pool_rows(X, T, qw->d_in, lambda1, s / (float)lambda1, ws.P, nullptr, st))) return rc;

    GemmDesc g{};
    g.qmode = 1;
    g.scales = nullptr; g.scales_tiled = ws.scales;
    if (tile8) { g.scales = qw->scales; g.scales_tiled = nullptr; g.block_rows = 8; }
    if (dense) { g.qmode = 3; g.W1 = ws.W16; g.K1 = qw->d_in; }
    g.X2 = ws.P; g.ldx2 = I; g.W2 = ws.Ht; g.ldw2 = I; g.K2 = I; g.div2 = lambda2;
    g.X1 = X; g.ldx1 = qw->d_in;
    g.codes = qw->codes; g.beta = qw->beta; g.d_out = qw->d_out; g.d_in = qw->d_in; g.cb = codebook_of(qw);
    g.codes_tiled = qw->codes_tiled;
    g.C = Y; g.ldc = qw->d_out; g.out_scale = 1.0f; g.M = T; g.N = qw->d_out;
    return launch_gemm(g, st);
}

int qablora_linear_bwd(const qblora_qweight* qw, const qblora_bf16* H, int32_t lambda1, int32_t lambda2, float s,
                       const qblora_bf16* X, const qblora_bf16* dY, int64_t T, qblora_bf16* dX, float* dH,
                       void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_qa(qw, H, lambda1, lambda2);
    if (rc) return rc;
    if (T < 0) return QBLORA_ERR_SHAPE;
    if (!dX && !dH) return QBLORA_ERR_NULL;
    hipStream_t st = as_stream(stream);
    const int I = qw->d_in / lambda1, J = qw->d_out / lambda2;
    if (T == 0) {
        if (dH) {
            const int64_t nh = (int64_t)I * J;
            hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((nh + 255) / 256)), dim3(256), 0, st, dH, nh);
            return launch_status();
        }
        return QBLORA_OK;
    }
    if (!dY || (dH && !X)) return QBLORA_ERR_NULL;
    QaBwdSpace ws = carve_qa_bwd(qw, lambda1, lambda2, T, workspace);
    if (!workspace || workspace_bytes < ws.bytes) return QBLORA_ERR_WORKSPACE;

    // (s/lambda1) * sum_lambda2(dY): operand of the dX K-extension and, rescaled by lambda1 at the end, of dH
    // (there with its bf16 residual, so that only the pooled input carries a bf16 rounding)
    if ((rc = launch_pool_rows(dY, T, qw->d_out, lambda2, s / (float)lambda1, ws.dVs, dH ? ws.dVs_lo : nullptr, st)))
        return rc;
    if (dH) {
        if ((rc = launch_pool_rows(X, T, qw->d_in, lambda1, 1.0f / (float)lambda1, ws.P, nullptr, st))) return rc;
        GradDesc gh{};
        gh.L = ws.P; gh.ldl = I; gh.I = I; gh.S = ws.dVs; gh.S_lo = ws.dVs_lo; gh.lds = J; gh.J = J; gh.T = T;
        gh.part = ws.part; gh.splits = ws.splits; gh.out = dH; gh.pool = 1;
        gh.out_scale = (float)lambda1; gh.transpose_out = 0;
        if ((rc = launch_grad(gh, st))) return rc;
    }
    if (!dX) return QBLORA_OK;
    GemmDesc g{};
    g.qmode = 2;
    g.block_rows = block_rows_of(qw);
    if ((rc = resolve_scales(qw, ws.scales, st, &g.scales))) return rc;
    if (use_dense(qw, T)) {
        if ((rc = launch_dequantize_operand(*qw, g.scales, 1, ws.W16t, st))) return rc;
        g.qmode = 3; g.W1 = ws.W16t; g.K1 = qw->d_out;
    } else if (half_blocks(qw)) {
        return QBLORA_ERR_UNSUPPORTED;
    }
    g.X2 = ws.dVs; g.ldx2 = J; g.W2 = H; g.ldw2 = J; g.K2 = J; g.div2 = lambda1;
    g.X1 = dY; g.ldx1 = qw->d_out;
    g.codes = qw->codes; g.beta = qw->beta; g.d_out = qw->d_out; g.d_in = qw->d_in; g.cb = codebook_of(qw);
    g.C = dX; g.ldc = qw->d_in; g.out_scale = 1.0f; g.M = T; g.N = qw->d_in;
    return launch_gemm(g, st);
}

size_t qblora_tile_product_workspace_bytes(const qblora_adapter* ad, int32_t d_in, int32_t d_out) {
    if (!has_adapter(ad) || d_out <= 0 || ad->lambda2 <= 0 || d_out % ad->lambda2) return 0;
    (void)d_in;
    return align_up((size_t)(d_out / ad->lambda2) * ad->R * sizeof(qblora_bf16));
}

int qblora_tile_product(const qblora_adapter* ad, int32_t d_in, int32_t d_out, float* H, void* workspace,
                        size_t workspace_bytes, void* stream) {
    if (!ad || !ad->A || !ad->B || !H) return QBLORA_ERR_NULL;
    if (d_in <= 0 || d_out <= 0 || ad->R <= 0 || ad->lambda1 <= 0 || ad->lambda2 <= 0) return QBLORA_ERR_SHAPE;
    if (d_in % ad->lambda1 || d_out % ad->lambda2 || ad->R % 8) return QBLORA_ERR_SHAPE;
    if (ad->scale_op != QBLORA_OP_AVGPOOL_REPEAT) return QBLORA_ERR_UNSUPPORTED;   // no tile-constant delta weight
    const int rows = d_in / ad->lambda1, cols = d_out / ad->lambda2;
    if (cols % 4) return QBLORA_ERR_UNSUPPORTED;
    size_t need = qblora_tile_product_workspace_bytes(ad, d_in, d_out);
    if (!workspace || workspace_bytes < need) return QBLORA_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    // whole tiles: one kernel that transposes B on the fly; otherwise a transposed copy and the general GEMM
    ScopedEvents ev(QBLORA_PROFILE_TILE_PRODUCT, st);
    int rc = launch_tile_product(ad->A, ad->B, rows, cols, ad->R, H, st);
    if (rc != QBLORA_ERR_UNSUPPORTED) return rc;
    qblora_bf16* Bt = static_cast<qblora_bf16*>(workspace);
    rc = launch_adapter_prep(ad->A, ad->B, d_in, d_out, ad->R, ad->lambda1, ad->lambda2, nullptr, Bt, nullptr, st);
    if (rc) return rc;
    GemmDesc g{};
    g.qmode = 0;
    g.X2 = ad->A; g.ldx2 = ad->R; g.W2 = Bt; g.ldw2 = ad->R; g.K2 = ad->R; g.div2 = 1;
    g.C = H; g.ldc = cols; g.out_f32 = 1; g.out_scale = 1.0f; g.M = rows; g.N = cols;
    return launch_gemm(g, st);
}

int qablora_merge_quantize(const qblora_qweight* base, const float* H, int32_t lambda1, int32_t lambda2, float s,
                           int32_t mode, qblora_qweight* out, void* stream) {
    int rc = merge_check(base, H, lambda1, lambda2, mode, out);
    if (rc) return rc;
    hipStream_t st = as_stream(stream);
    const MergeDesc d = merge_fill(base, H, lambda1, lambda2, s, mode, out);
    if (mode == QBLORA_MERGE_BETA_SHIFT) return merge_shift(base, d, out, st);
    ScopedEvents ev(QBLORA_PROFILE_MERGE, st);
    return launch_merge_requant(d, st);
}

int qablora_merge_quantize_batch(int32_t count, const qblora_qweight* const* bases, const float* const* H,
                                 int32_t lambda1, int32_t lambda2, float s, int32_t mode, qblora_qweight* const* outs,
                                 void* stream) {
    if (count < 0) return QBLORA_ERR_SHAPE;
    if (count == 0) return QBLORA_OK;
    if (!bases || !H || !outs) return QBLORA_ERR_NULL;
    for (int32_t m = 0; m < count; ++m) {                   // every check of every weight before any `out` is touched
        if (!bases[m] || !outs[m]) return QBLORA_ERR_NULL;
        const int rc = merge_check(bases[m], H[m], lambda1, lambda2, mode, outs[m]);
        if (rc) return rc;
    }
    hipStream_t st = as_stream(stream);
    constexpr int32_t kChunk = 8;                           // weights per launch
    for (int32_t m0 = 0; m0 < count; m0 += kChunk) {
        const int32_t n = std::min(kChunk, count - m0);
        MergeDesc ds[kChunk];
        for (int32_t m = 0; m < n; ++m) ds[m] = merge_fill(bases[m0 + m], H[m0 + m], lambda1, lambda2, s, mode, outs[m0 + m]);
        int rc = QBLORA_ERR_UNSUPPORTED;
        if (mode == QBLORA_MERGE_REQUANT_MINMAX) {
            ScopedEvents ev(QBLORA_PROFILE_MERGE, st);
            rc = launch_merge_requant_batch(ds, n, st);
        }
        if (rc == QBLORA_ERR_UNSUPPORTED) {                 // one by one (nothing was launched)
            for (int32_t m = 0; m < n; ++m) {
                if (mode == QBLORA_MERGE_BETA_SHIFT) rc = merge_shift(bases[m0 + m], ds[m], outs[m0 + m], st);
                else rc = launch_merge_requant(ds[m], st);
                if (rc) return rc;
            }
        } else if (rc) {
            return rc;
        }
    }
    return QBLORA_OK;
}

int qblora_merge_bf16(const qblora_qweight* base, const float* H, int32_t lambda1, int32_t lambda2, float s,
                      qblora_bf16* W16, void* stream) {
    int rc = check_qweight(base, true, true);
    if (rc) return rc;
    if (!H || !W16) return QBLORA_ERR_NULL;
    if (lambda1 <= 0 || lambda2 <= 0) return QBLORA_ERR_SHAPE;
    if (base->d_in % lambda1 || base->d_out % lambda2) return QBLORA_ERR_SHAPE;
    const bool grouped = base->scale_mode == QBLORA_SCALES_E4M3_GROUPED;
    MergeDesc d{};
    d.codes = base->codes; d.scales = base->scales; d.beta = base->beta;
    if (grouped) {
        d.scale_codes = base->scale_codes; d.scale_step = base->scale_step; d.scale_mid = base->scale_mid;
        d.scale_group = base->scale_group;
    }
    d.cb = codebook_of(base); d.d_out = base->d_out; d.d_in = base->d_in;
    d.H = H; d.lam1 = lambda1; d.lam2 = lambda2; d.s = s;
    d.w16_out = W16;
    d.block_rows = block_rows_of(base); d.block_cols = block_cols_of(base);
    return launch_merge_bf16(d, as_stream(stream));
}

namespace {

struct DecodePack { uint8_t* codes; float* scales; float* beta; size_t bytes; };
constexpr int32_t kDecodeMaxTokens = 16;     // up to here: the streaming kernel that scales block sums
constexpr int32_t kMidChunk = 128;           // above: the bf16 compute weight, at most this many tokens per launch
constexpr int32_t kMidMaxTokens = 256;

// An INT4 model in 64-blocks (codebook exactly 0, 1, ..., 15 and offsets present): its pack holds the codes
// with the nibbles of every dword regrouped for the table-free decode kernel.  Pack and decode both decide
// from the weight's description, which a pack belongs to.
bool decode_regrouped(const qblora_qweight* qw) {
    if (!qw->beta || block_rows_of(qw) != 1) return false;
    for (int j = 0; j < 16; ++j)
        if (qw->codebook[j] != (float)j) return false;
    return true;
}
DecodePack carve_pack(const qblora_qweight* qw, void* base) {
    Carver c(base);
    DecodePack p{};
    const size_t rows = (size_t)((qw->d_out + 255) / 256) * 256, bpr = (size_t)(qw->d_in / kBlock);   // 64-input runs of codes
    p.codes = c.take<uint8_t>(rows * bpr * 32);
    if (block_rows_of(qw) == 8) {            // scales and offsets of 8 x 8 blocks are read where they are
        p.scales = qw->scales; p.beta = qw->beta;
    } else {
        p.scales = c.take<float>(rows * bpr);
        if (qw->beta) p.beta = c.take<float>(rows * bpr);
    }
    p.bytes = c.off;
    return p;
}

}  // namespace

size_t qblora_decode_pack_bytes(const qblora_qweight* qw) {
    if (check_qweight(qw, false, true)) return 0;
    return carve_pack(qw, nullptr).bytes;
}

int qblora_decode_pack(const qblora_qweight* qw, void* pack, void* stream) {
    int rc = check_qweight(qw, true, true);
    if (rc) return rc;
    if (!pack) return QBLORA_ERR_NULL;
    hipStream_t st = as_stream(stream);
    DecodePack p = carve_pack(qw, pack);
    if ((rc = launch_prepack_codes(qw->codes, qw->d_out, qw->d_in, p.codes, st, decode_regrouped(qw)))) return rc;
    if (block_rows_of(qw) == 8) return QBLORA_OK;
    ScaleTiling sct{};
    const bool grouped = qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED;
    sct.scales = grouped ? nullptr : qw->scales;
    if (grouped) { sct.scale_codes = qw->scale_codes; sct.scale_step = qw->scale_step; sct.scale_mid = qw->scale_mid; }
    sct.scale_group = qw->scale_group; sct.d_out = qw->d_out; sct.d_in = qw->d_in; sct.out = p.scales;
    if ((rc = launch_adapter_prep(nullptr, nullptr, qw->d_in, qw->d_out, 0, 1, 1, nullptr, nullptr, nullptr, st, &sct)))
        return rc;
    if (qw->beta) {
        ScaleTiling bt{};
        bt.scales = qw->beta; bt.d_out = qw->d_out; bt.d_in = qw->d_in; bt.out = p.beta;
        if ((rc = launch_adapter_prep(nullptr, nullptr, qw->d_in, qw->d_out, 0, 1, 1, nullptr, nullptr, nullptr, st, &bt)))
            return rc;
    }
    return QBLORA_OK;
}

size_t qblora_linear_decode_workspace_bytes(const qblora_qweight* qw) {
    if (check_qweight(qw, false, true)) return 0;
    return qw->scale_mode == QBLORA_SCALES_E4M3_GROUPED ? align_up(sizeof(float) * (size_t)n_blocks(qw)) : 0;
}
size_t qblora_linear_decode_tokens_workspace_bytes(const qblora_qweight* qw, int32_t T) {
    if (check_qweight(qw, false, true)) return 0;
    size_t part = 0;
    for (int32_t t0 = (kDecodeMaxTokens < T || half_blocks(qw)) ? 0 : T; t0 < T; t0 += kMidChunk)   // chunks of the mid-batch form
        part = std::max(part, w4_mid_part_bytes(qw->d_out, qw->d_in, std::min(kMidChunk, T - t0)));
    return qblora_linear_decode_workspace_bytes(qw) + align_up(part);
}
int qblora_linear_decode(const qblora_qweight* qw, const void* pack, const qblora_bf16* X, int32_t T, qblora_bf16* Y,
                         void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_qweight(qw, true, true);
    if (rc) return rc;
    if (T < 0 || T > kMidMaxTokens) return QBLORA_ERR_SHAPE;
    if (T == 0) return QBLORA_OK;
    if (!X || !Y) return QBLORA_ERR_NULL;
    if (qw->d_in % 8 != 0 || (reinterpret_cast<uintptr_t>(X) & 15) || (reinterpret_cast<uintptr_t>(qw->codes) & 15) ||
        (reinterpret_cast<uintptr_t>(pack) & 255))
        return QBLORA_ERR_SHAPE;
    hipStream_t st = as_stream(stream);
    const bool mid = T > kDecodeMaxTokens || half_blocks(qw);   // 8 x 4 blocks: the mid-batch kernel at every token count
    const size_t scale_bytes = qblora_linear_decode_workspace_bytes(qw);
    const size_t need = mid ? qblora_linear_decode_tokens_workspace_bytes(qw, T) : (pack ? 0 : scale_bytes);
    if (need > 0 && (!workspace || workspace_bytes < need)) return QBLORA_ERR_WORKSPACE;
    if (mid && need > scale_bytes && (reinterpret_cast<uintptr_t>(workspace) & 15)) return QBLORA_ERR_WORKSPACE;
    // the mid-batch kernel stores 8-byte words and, with 8 x 8 blocks, loads four block parameters at a time
    if (mid && ((reinterpret_cast<uintptr_t>(Y) & 7) || qw->d_in % kBlock != 0 ||
                (block_rows_of(qw) == 8 && ((reinterpret_cast<uintptr_t>(qw->scales) & 15) ||
                                            (reinterpret_cast<uintptr_t>(qw->beta) & 15)))))
        return QBLORA_ERR_SHAPE;
    const uint8_t* codes = qw->codes;
    const float* scales = nullptr;
    const float* beta = qw->beta;
    const int regrouped = pack ? decode_regrouped(qw) : 0;
    if (pack) {
        DecodePack p = carve_pack(qw, const_cast<void*>(pack));
        codes = p.codes; scales = p.scales; beta = p.beta;
    } else if ((rc = resolve_scales(qw, static_cast<float*>(workspace), st, &scales))) {
        return rc;
    }
    if (!mid)
        return launch_w4_decode(codes, scales, beta, codebook_of(qw), pack ? 1 : 0, qw->d_out, qw->d_in, X, T, Y, st,
                                block_rows_of(qw), regrouped);
    float* part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + scale_bytes);
    for (int32_t t0 = 0; t0 < T; t0 += kMidChunk) {
        const int32_t tc = std::min(kMidChunk, T - t0);
        if ((rc = launch_w4_mid(codes, scales, beta, codebook_of(qw), pack ? 1 : 0, qw->d_out, qw->d_in,
                                X + (int64_t)t0 * qw->d_in, tc, Y + (int64_t)t0 * qw->d_out,
                                w4_mid_part_bytes(qw->d_out, qw->d_in, tc) ? part : nullptr, st, block_rows_of(qw), regrouped,
                                block_rows_of(qw) == 8 ? block_cols_of(qw) : 8)))
            return rc;
    }
    return QBLORA_OK;
}

}  // extern "C"
