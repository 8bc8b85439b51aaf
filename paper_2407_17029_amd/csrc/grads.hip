// Adapter-parameter gradients: reductions over all tokens (backward of Sec. 3.2's A and B).
//
//   dA = P^T dU = (1/lambda1) * pool_rows_lambda1( X^T dU )          [d_in/lambda1, R]
//   dB = U^T dV = transpose( pool_rows_lambda2( dY^T (s U) ) )        [R, d_out/lambda2]
//
// Both are "token-contraction" GEMMs  part[z][i][j] = sum_{t in slice z} L[t,i] * S[t,j]  with a
// wide L (X or dY) and a narrow S (dU or s*U, inner rank columns).  The token range is split over
// `splits` workgroup slices so the launch fills the chip; the partial sums are written to scratch
// and a second kernel adds them in a fixed order (deterministic), pools adjacent rows and applies
// the scale.  The narrow operand is produced by this library in fp32 and handed over as a bf16 pair
// (high part + residual); both parts are contracted, so the gradients carry fp32-accumulation error
// only.
//
// Both operands are token-major in memory while an MFMA lane needs consecutive tokens of one
// feature.  k_grad_tr (the fast path) copies token-major tiles straight into an LDS ring and lets
// the transposing LDS read (ds_read_b64_tr_b16) deliver the operand layout; k_grad_partial (any
// shape and alignment) transposes in registers on the way into LDS.
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 512;
constexpr int BI = 128, BJ = 128, BT = 64;

__device__ __forceinline__ int swz(int row, int chunk) {
    return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

__global__ __launch_bounds__(kThreads) void k_grad_partial(GradDesc d, int64_t slice_len) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char (*sL)[BI * 128] = reinterpret_cast<unsigned char (*)[BI * 128]>(smem);
    unsigned char (*sS)[BJ * 128] = reinterpret_cast<unsigned char (*)[BJ * 128]>(smem + 2 * BI * 128);
    unsigned char (*sSlo)[BJ * 128] = reinterpret_cast<unsigned char (*)[BJ * 128]>(smem + 2 * BI * 128 + 2 * BJ * 128);
    const bool has_lo = d.S_lo != nullptr;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int i0 = blockIdx.x * BI, j0 = blockIdx.y * BJ, z = blockIdx.z;
    const int64_t t_begin = (int64_t)z * slice_len;
    int64_t t_end = t_begin + slice_len;
    if (t_end > d.T) t_end = d.T;
    const int nsteps = t_begin < t_end ? (int)((t_end - t_begin + BT - 1) / BT) : 0;

    // wave tile: 32 j (MFMA rows) x 64 i (MFMA columns, two blocks)
    const int wj0 = (wave & 3) * 32, wi0 = (wave >> 2) * 64;
    f32x16 acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

    // loader: threads 0..255 move the L tile, 256..511 the S tile; an item is 8 tokens x 4 columns
    const bool isL = t < 256;
    const int item = t & 255, cg = item & 31, tg = item >> 5;
    const qblora_bf16* src = isL ? d.L : d.S;
    const int64_t ld = isL ? d.ldl : d.lds;
    const int width = isL ? d.I : d.J;
    int col = (isL ? i0 : j0) + 4 * cg;
    if (col > width - 4) col = width - 4;          // clamped columns are never stored
    uint2 reg[8], reg_lo[8];

    auto load_global = [&](int step) {
        const int64_t tb = t_begin + (int64_t)step * BT + 8 * tg;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int64_t tt = tb + q;
            reg[q] = (tt < t_end) ? *reinterpret_cast<const uint2*>(src + tt * ld + col) : make_uint2(0, 0);
            if (!isL && has_lo)
                reg_lo[q] = (tt < t_end) ? *reinterpret_cast<const uint2*>(d.S_lo + tt * ld + col) : make_uint2(0, 0);
        }
    };
    auto transpose_store = [&](const uint2 (&rg)[8], unsigned char* base) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t h[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint32_t w = (c < 2) ? rg[q].x : rg[q].y;
                h[q] = (c & 1) ? (w >> 16) : (w & 0xffffu);
            }
            uint4 o;
            o.x = h[0] | (h[1] << 16); o.y = h[2] | (h[3] << 16);
            o.z = h[4] | (h[5] << 16); o.w = h[6] | (h[7] << 16);
            *reinterpret_cast<uint4*>(base + swz(4 * cg + c, tg)) = o;
        }
    };
    auto store_lds = [&](int buf) {
        transpose_store(reg, isL ? sL[buf] : sS[buf]);
        if (!isL && has_lo) transpose_store(reg_lo, sSlo[buf]);
    };
    auto compute = [&](int buf) {
        const int r = lane & 31, hi = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 sf = *reinterpret_cast<const bf16x8*>(sS[buf] + swz(wj0 + r, ks * 2 + hi));
            bf16x8 sf_lo = sf;
            if (has_lo) sf_lo = *reinterpret_cast<const bf16x8*>(sSlo[buf] + swz(wj0 + r, ks * 2 + hi));
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                bf16x8 lf = *reinterpret_cast<const bf16x8*>(sL[buf] + swz(wi0 + b * 32 + r, ks * 2 + hi));
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, lf, acc[b], 0, 0, 0);
                if (has_lo) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf_lo, lf, acc[b], 0, 0, 0);
            }
        }
    };

    if (nsteps > 0) {
        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int step = 0; step < nsteps; ++step) {
            const bool more = step + 1 < nsteps;
            if (more) load_global(step + 1);
            compute(step & 1);
            if (more) store_lds((step + 1) & 1);
            __syncthreads();
        }
    }

    // accumulator rows are j (4 consecutive per lane), columns are i
    float* part = d.part + (int64_t)z * d.I * d.J;
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int i = i0 + wi0 + b * 32 + r;
        if (i >= d.I) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int j = j0 + wj0 + q * 8 + hi * 4;
            if (j >= d.J) continue;
            *reinterpret_cast<float4*>(part + (int64_t)i * d.J + j) =
                make_float4(acc[b][q * 4 + 0], acc[b][q * 4 + 1], acc[b][q * 4 + 2], acc[b][q * 4 + 3]);
        }
    }
}

// ---- fast path: direct copies + transposing LDS reads -------------------------------------------
//
// A stage holds 32 tokens of three token-major tiles (L, S, S_lo), each 32 rows x 128 features of
// bf16 = 256-byte rows of sixteen 16-byte chunks.  Logical chunk c of row t sits at chunk position
// c ^ ((t & 3) << 2): a direct copy instruction fills four whole rows (lane l: row l>>4, position
// l&15, so it fetches chunk (l&15) ^ ((l>>4)<<2)), and the transposing read below touches every
// bank exactly once.
//
// ds_read_b64_tr_b16 works on groups of 16 lanes: if lane s of a group points at four consecutive
// features of token row s>>2, starting at feature 4*(s&3) of a 16-feature block, lane i of the
// group receives feature i of the block for the group's four token rows, in row order.  Two such
// reads (rows +0..3 and +4..7) give a lane the 8 consecutive tokens of one feature that
// v_mfma_f32_32x32x16_bf16 wants: lane groups 0/1 serve features 0-15 / 16-31 of a 32-feature block
// for tokens 0-7 of a 16-token slice, groups 2/3 the same features for tokens 8-15.
constexpr int kTrBT = 32, kTrStages = 3;         // 72 KB: two workgroups fit a CU (6 stages measured the same)
constexpr int kTrTile = kTrBT * 256, kTrStage = 3 * kTrTile;
constexpr int kTrThreads = 512;

__device__ __align__(16) const uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};

constexpr int vmcnt_imm(int n) { return (n & 15) | 0x0F70 | ((n >> 4) << 14); }

__device__ __forceinline__ void copy16_to_lds(const void* p, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(lds_base), "v"(p) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// 8 consecutive tokens of this lane's feature: rows +0..3 and +4..7 of the 16-token slice half
__device__ __forceinline__ bf16x8 tr_fragment(const unsigned char* p) {
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * 256));
    const s16x8 v = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// Two gradients in one launch (dA and dB of a layer are independent): the first n_a workgroups work on `a`,
// the others on `b`.  With one workgroup per CU each, the dispatcher puts one of either on every CU, and one's
// MFMAs run under the other's waits for its copies.
struct GradPair {
    GradDesc a, b;
    int n_a;
    int64_t slice_a, slice_b;
};

template <bool HAS_LO>
__global__ __launch_bounds__(kTrThreads) void k_grad_tr(GradPair p) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kPer = HAS_LO ? 3 : 2;             // copy instructions per wave and stage
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const bool second = (int)blockIdx.x >= p.n_a;
    const GradDesc& d = second ? p.b : p.a;
    const int64_t slice_len = second ? p.slice_b : p.slice_a;
    const int bid = (int)blockIdx.x - (second ? p.n_a : 0);
    // Consecutive workgroup ids go to different XCDs (id % 8).  The column tiles of one (row tile, token
    // slice) read the same stream of L, the wide operand: they get ids 8 apart inside a run of 8 * tiles_j
    // ids, so they start together on one XCD and its L2 fetches L once for all of them.  The grid is
    // rounded up to whole runs; ids past the last (row tile, slice) leave.
    const int tiles_i = (d.I + BI - 1) / BI, tiles_j = (d.J + BJ - 1) / BJ;
    const int run = bid / (8 * tiles_j), within = bid % (8 * tiles_j);
    const int unit = run * 8 + (within & 7);
    if (unit >= tiles_i * d.splits) return;
    const int z = unit % d.splits;
    const int i0 = (unit / d.splits) * BI, j0 = (within >> 3) * BJ;
    const int64_t t_begin = (int64_t)z * slice_len;
    int64_t t_end = t_begin + slice_len;
    if (t_end > d.T) t_end = d.T;
    const int nsteps = t_begin < t_end ? (int)((t_end - t_begin + kTrBT - 1) / kTrBT) : 0;

    const qblora_bf16* const Lp = d.L; const int64_t ldl = d.ldl;
    const qblora_bf16* const Sp = d.S; const qblora_bf16* const Slo = d.S_lo; const int64_t lds = d.lds;

    // copies: wave w fills rows 4w .. 4w+3 of each tile with one instruction
    const int drow = lane >> 4;
    const int dchunk = (lane & 15) ^ (drow << 2);
    const int lcol = i0 + 8 * dchunk, scol = j0 + 8 * dchunk;
    const bool lcol_ok = lcol < d.I, scol_ok = scol < d.J;      // widths are multiples of 8: a chunk is in or out
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * 4 * 256);
    const void* const zero = g_zero16;
    // Whole steps (every token row inside the slice) walk per-lane pointers: a lane whose chunk lies
    // beyond the operand's width keeps fetching the zero chunk (increment 0).  Steps are issued in
    // ascending order, so the pointers simply advance by 32 rows per call.
    const unsigned char* pl[1]; const unsigned char* ps[1]; const unsigned char* pslo[1];
#pragma unroll
    for (int i = 0; i < 1; ++i) {
        const int64_t tt = t_begin + wave * 4 + drow;
        pl[i] = lcol_ok ? reinterpret_cast<const unsigned char*>(Lp + tt * ldl + lcol) : static_cast<const unsigned char*>(zero);
        ps[i] = scol_ok ? reinterpret_cast<const unsigned char*>(Sp + tt * lds + scol) : static_cast<const unsigned char*>(zero);
        pslo[i] = (HAS_LO && scol_ok) ? reinterpret_cast<const unsigned char*>(Slo + tt * lds + scol)
                                      : static_cast<const unsigned char*>(zero);
    }
    const int64_t inc_l = lcol_ok ? kTrBT * ldl * 2 : 0, inc_s = scol_ok ? kTrBT * lds * 2 : 0;
    auto issue = [&](int step) __attribute__((always_inline)) {
        const uint32_t stage = lds0 + (uint32_t)(step % kTrStages) * kTrStage;
        if (t_begin + (int64_t)(step + 1) * kTrBT <= t_end) {
#pragma unroll
            for (int i = 0; i < 1; ++i) {
                copy16_to_lds(pl[i], stage + i * 1024);
                copy16_to_lds(ps[i], stage + kTrTile + i * 1024);
                if constexpr (HAS_LO) copy16_to_lds(pslo[i], stage + 2 * kTrTile + i * 1024);
                pl[i] += inc_l; ps[i] += inc_s;
                if constexpr (HAS_LO) pslo[i] += inc_s;
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < 1; ++i) {                           // the ragged last step of the last slice
            const int64_t tt = t_begin + (int64_t)step * kTrBT + wave * 4 + drow;
            const bool ok = tt < t_end;                         // rows past the slice contribute zeros
            copy16_to_lds((ok && lcol_ok) ? (const void*)(Lp + tt * ldl + lcol) : zero, stage + i * 1024);
            copy16_to_lds((ok && scol_ok) ? (const void*)(Sp + tt * lds + scol) : zero, stage + kTrTile + i * 1024);
            if constexpr (HAS_LO)
                copy16_to_lds((ok && scol_ok) ? (const void*)(Slo + tt * lds + scol) : zero,
                              stage + 2 * kTrTile + i * 1024);
        }
    };

    // wave tile: 64 j (MFMA rows, two blocks) x 32 i (MFMA columns); two waves share a SIMD
    const int wj0 = (wave & 1) * 64, wi0 = (wave >> 1) * 32;
    const int g = lane >> 4, sl = lane & 15;
    const int frow = 8 * (g >> 1) + (sl >> 2);                  // token row inside a 16-token slice
    uint32_t soff[2], loff[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int cs = wj0 + b * 32 + 16 * (g & 1) + 4 * (sl & 3);
        const int cl = wi0 + 16 * (g & 1) + 4 * (sl & 3);
        soff[b] = frow * 256 + ((((cs >> 3) ^ ((frow & 3) << 2)) & 15) << 4) + ((cs >> 2) & 1) * 8;
        loff[b] = frow * 256 + ((((cl >> 3) ^ ((frow & 3) << 2)) & 15) << 4) + ((cl >> 2) & 1) * 8;
    }
    f32x16 acc[2][1];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][0][i] = 0.0f;

    // A wave is alone on its SIMD, so LDS latency is hidden by hand: the fragments of the next
    // 16-token slice are read while the MFMAs of the current one issue (two fragment sets with fixed
    // names), and the barrier that publishes the next stage sits between the two slices of a step.
    struct Frags { bf16x8 sf[2], sflo[2], lf[1]; };
    auto read_frags = [&](Frags& f, int buf, int kk) __attribute__((always_inline)) {
        const unsigned char* base = smem + buf * kTrStage + kk * 16 * 256;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            f.sf[b] = tr_fragment(base + kTrTile + soff[b]);
            if constexpr (HAS_LO) f.sflo[b] = tr_fragment(base + 2 * kTrTile + soff[b]);
            if (b == 0) f.lf[0] = tr_fragment(base + loff[0]);
        }
    };
    auto mfmas = [&](const Frags& f) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 1; ++b) {
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.sf[a], f.lf[b], acc[a][b], 0, 0, 0);
                if constexpr (HAS_LO)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.sflo[a], f.lf[b], acc[a][b], 0, 0, 0);
            }
    };
    auto interleave = [&]() __attribute__((always_inline)) {        // one MFMA, then two of the pending LDS reads
#pragma unroll
        for (int m = 0; m < (HAS_LO ? 4 : 2); ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // Ring: every buffer is filled up front; step s hands its buffer to step s + kTrStages as soon as
    // all waves have read it (the barrier in the middle of the step).
    static_assert(kTrBT == 32, "a step is two 16-token slices");
    if (nsteps > 0) {
        for (int q = 0; q < kTrStages && q < nsteps; ++q) issue(q);
        if (nsteps >= kTrStages) __builtin_amdgcn_s_waitcnt(vmcnt_imm((kTrStages - 1) * kPer));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        Frags f0, f1;
        read_frags(f0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        int s = 0, buf = 0;
        for (; s + kTrStages < nsteps; ++s) {
            const int nxt = buf + 1 == kTrStages ? 0 : buf + 1;
            read_frags(f1, buf, 1);
            mfmas(f0);
            interleave();
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((kTrStages - 2) * kPer));   // stage s+1 is in; younger ones may fly
            __syncthreads();                         // ... for every wave, and all reads of this buffer are done
            issue(s + kTrStages);                    // refill this buffer
            read_frags(f0, nxt, 0);
            mfmas(f1);
            interleave();
            buf = nxt;
        }
        for (; s < nsteps; ++s) {
            const int nxt = buf + 1 == kTrStages ? 0 : buf + 1;
            const bool more = s + 1 < nsteps;
            read_frags(f1, buf, 1);
            mfmas(f0);
            interleave();
            if (more) {
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
                __syncthreads();
                read_frags(f0, nxt, 0);
            }
            mfmas(f1);
            interleave();
            buf = nxt;
        }
    }

    // accumulator rows are j (4 consecutive per lane), columns are i
    float* part = d.part + (int64_t)z * d.I * d.J;
    const int r = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int b = 0; b < 1; ++b) {
        const int i = i0 + wi0 + b * 32 + r;
        if (i >= d.I) continue;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + wj0 + a * 32 + q * 8 + hi * 4;
                if (j >= d.J) continue;
                *reinterpret_cast<float4*>(part + (int64_t)i * d.J + j) =
                    make_float4(acc[a][b][q * 4 + 0], acc[a][b][q * 4 + 1], acc[a][b][q * 4 + 2], acc[a][b][q * 4 + 3]);
            }
    }
}

// out[i', j] (or out[j, i'] when transposed) = out_scale * sum_{p < pool} sum_z part[z][i'*pool+p][j],
// summed in ascending (p, z) order.
__device__ __forceinline__ void grad_reduce_plain(const GradDesc& d, const unsigned bid) {
    const int Ip = d.I / d.pool;
    const int64_t total = (int64_t)Ip * d.J;
    const int64_t idx = (int64_t)bid * 256 + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % d.J);
    const int ip = (int)(idx / d.J);
    const int64_t plane = (int64_t)d.I * d.J;
    float sum = 0.0f;
    for (int p = 0; p < d.pool; ++p) {
        const float* src = d.part + (int64_t)(ip * d.pool + p) * d.J + j;
        // eight slices at a time: the loads are independent and issued together, the additions keep
        // their order
        for (int z0 = 0; z0 < d.splits; z0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)min(z0 + u, d.splits - 1) * plane];   // unconditional, in bounds
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (z0 + u < d.splits) sum += v[u];
        }
    }
    sum *= d.out_scale;
    if (d.transpose_out) d.out[(int64_t)j * Ip + ip] = sum;
    else d.out[(int64_t)ip * d.J + j] = sum;
}

// The same sums (same order, same bits) for J % 4 == 0, Ip % 4 == 0 and 16-byte aligned buffers; used for
// the transposed output.  A workgroup owns 32 pooled rows x 32 columns, a thread one pooled row and 4
// consecutive columns, so every load instruction of a wave reads eight whole 128-byte lines and all
// pool * splits loads of a thread are issued together; the transposed output goes through LDS so that its
// stores are whole lines too (one thread per output element wrote 4 bytes into each of 64 lines).
__device__ __forceinline__ void grad_reduce_tile(const GradDesc& d, const unsigned bid, float (&tr)[32][33]) {
    const int Ip = d.I / d.pool;
    const int tiles_j = (d.J + 31) / 32;
    const int j0 = (bid % tiles_j) * 32, ip0 = (bid / tiles_j) * 32;
    const int t = threadIdx.x, r = t >> 3, c4 = (t & 7) * 4;
    const int ip = min(ip0 + r, Ip - 1), j = min(j0 + c4, d.J - 4);      // clamped lanes compute, never store
    const int64_t plane = (int64_t)d.I * d.J;
    const float* src = d.part + (int64_t)ip * d.pool * d.J + j;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    const int n = d.pool * d.splits;
    for (int q0 = 0; q0 < n; q0 += 16) {                                 // q = p * splits + z: ascending (p, z)
        float4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int q = min(q0 + u, n - 1), pp = q / d.splits, z = q - pp * d.splits;
            v[u] = *reinterpret_cast<const float4*>(src + (int64_t)pp * d.J + (int64_t)z * plane);
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (q0 + u < n) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
    }
    sum.x *= d.out_scale; sum.y *= d.out_scale; sum.z *= d.out_scale; sum.w *= d.out_scale;
    const bool live = ip0 + r < Ip && j0 + c4 < d.J;
    if (!d.transpose_out) {
        if (live) *reinterpret_cast<float4*>(d.out + (int64_t)ip * d.J + j) = sum;
        return;
    }
    tr[c4][r] = sum.x; tr[c4 + 1][r] = sum.y; tr[c4 + 2][r] = sum.z; tr[c4 + 3][r] = sum.w;
    __syncthreads();
    const int jj = t >> 3, iq = (t & 7) * 4;                             // output row j0 + jj, pooled rows ip0 + iq .. +3
    if (j0 + jj < d.J && ip0 + iq < Ip)
        *reinterpret_cast<float4*>(d.out + (int64_t)(j0 + jj) * Ip + ip0 + iq) =
            make_float4(tr[jj][iq], tr[jj][iq + 1], tr[jj][iq + 2], tr[jj][iq + 3]);
}

__global__ __launch_bounds__(256) void k_grad_reduce(GradDesc d) { grad_reduce_plain(d, blockIdx.x); }

__global__ __launch_bounds__(256) void k_grad_reduce_tile(GradDesc d) {
    __shared__ float tr[32][33];
    grad_reduce_tile(d, blockIdx.x, tr);
}

// Both second stages of a layer's gradients in one launch: blocks below n_a reduce `a` element-wise, the
// others reduce `b` by tiles (transposed output).
__global__ __launch_bounds__(256) void k_grad_reduce_pair(GradPair p) {
    __shared__ float tr[32][33];
    if ((int)blockIdx.x < p.n_a) grad_reduce_plain(p.a, blockIdx.x);
    else grad_reduce_tile(p.b, blockIdx.x - p.n_a, tr);
}

}  // namespace

int grad_splits(int64_t T, int I, int J) {
    int tiles = ((I + BI - 1) / BI) * ((J + BJ - 1) / BJ);
    int want = (256 + tiles - 1) / tiles;              // one workgroup per CU
    int64_t max_splits = (T + BT - 1) / BT;
    if (want > max_splits) want = (int)max_splits;
    if (want > 32) want = 32;
    if (want < 1) want = 1;
    return want;
}

namespace {

// The fast path fetches 16-byte chunks: rows and widths must keep every chunk whole and aligned.
bool tr_applies(const GradDesc& d) {
    auto aligned16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    return d.I % 8 == 0 && d.J % 8 == 0 && d.ldl % 8 == 0 && d.lds % 8 == 0 && aligned16(d.L) && aligned16(d.S) &&
           (d.S_lo == nullptr || aligned16(d.S_lo));
}

// raises a kernel's dynamic LDS limit; callers keep the result in a function-local static (set once, thread safe)
template <typename K>
bool set_lds(K kernel, size_t smem) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)smem) == hipSuccess;
}

}  // namespace

namespace {

int64_t slice_of(const GradDesc& d) {
    int64_t slice_len = (d.T + d.splits - 1) / d.splits;
    return (slice_len + BT - 1) / BT * BT;
}

unsigned tr_blocks(const GradDesc& d) {              // whole runs of 8 (row tile, slice) units x column tiles
    const unsigned units = (unsigned)(((d.I + BI - 1) / BI) * d.splits);
    return (units + 7) / 8 * 8 * (unsigned)((d.J + BJ - 1) / BJ);
}

// partial sums of one or two gradients on the copy path (both with or both without a low-order part)
int launch_tr(const GradDesc& a, const GradDesc* b, hipStream_t st) {
    constexpr size_t smem = (size_t)kTrStages * kTrStage;
    GradPair p{};
    p.a = a; p.slice_a = slice_of(a); p.n_a = (int)tr_blocks(a);
    unsigned blocks = tr_blocks(a);
    if (b) { p.b = *b; p.slice_b = slice_of(*b); blocks += tr_blocks(*b); }
    if (a.S_lo) {
        static const bool ok = set_lds(k_grad_tr<true>, smem);
        if (!ok) return QBLORA_ERR_LAUNCH;
        hipLaunchKernelGGL(k_grad_tr<true>, dim3(blocks), dim3(kTrThreads), smem, st, p);
    } else {
        static const bool ok = set_lds(k_grad_tr<false>, smem);
        if (!ok) return QBLORA_ERR_LAUNCH;
        hipLaunchKernelGGL(k_grad_tr<false>, dim3(blocks), dim3(kTrThreads), smem, st, p);
    }
    return launch_status();
}

int launch_partial(const GradDesc& d, hipStream_t st) {
    constexpr size_t smem = 2 * BI * 128 + 4 * BJ * 128;
    static const bool ok = set_lds(k_grad_partial, smem);
    if (!ok) return QBLORA_ERR_LAUNCH;
    dim3 grid((d.I + BI - 1) / BI, (d.J + BJ - 1) / BJ, d.splits);
    hipLaunchKernelGGL(k_grad_partial, grid, dim3(kThreads), smem, st, d, slice_of(d));
    return launch_status();
}

// measured: the plain kernel is the faster one when the output is not transposed (5.1 vs 5.5 us), the tiled
// one when it is (5.8 vs 7.5 us)
bool reduce_by_tiles(const GradDesc& d) {
    const int Ip = d.I / d.pool;
    auto aligned16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    return d.transpose_out && d.J % 4 == 0 && Ip % 4 == 0 && aligned16(d.part) && aligned16(d.out);
}
unsigned reduce_blocks(const GradDesc& d) {
    const int Ip = d.I / d.pool;
    if (reduce_by_tiles(d)) return (unsigned)(((d.J + 31) / 32) * ((Ip + 31) / 32));
    return (unsigned)(((int64_t)Ip * d.J + 255) / 256);
}

int launch_reduce(const GradDesc& d, hipStream_t st) {
    if (reduce_by_tiles(d)) hipLaunchKernelGGL(k_grad_reduce_tile, dim3(reduce_blocks(d)), dim3(256), 0, st, d);
    else hipLaunchKernelGGL(k_grad_reduce, dim3(reduce_blocks(d)), dim3(256), 0, st, d);
    return launch_status();
}

}  // namespace

int launch_grad(const GradDesc& d, hipStream_t st) {
    if (d.T <= 0) return QBLORA_ERR_SHAPE;      // the entry point handles the empty batch itself
    int rc = tr_applies(d) ? launch_tr(d, nullptr, st) : launch_partial(d, st);
    if (rc) return rc;
    return launch_reduce(d, st);
}

// Two independent gradients with partial buffers of their own: one launch of the copy path for both when
// both qualify, else one after the other.
int launch_grad_pair(const GradDesc& a, const GradDesc& b, hipStream_t st) {
    if (a.T <= 0 || b.T <= 0) return QBLORA_ERR_SHAPE;
    if (a.part == b.part || !tr_applies(a) || !tr_applies(b) || (a.S_lo == nullptr) != (b.S_lo == nullptr)) {
        int rc = launch_grad(a, st);
        return rc ? rc : launch_grad(b, st);
    }
    int rc;
    {
        ProfileScope ev(QBLORA_PROFILE_ADAPTER_GRADS, st);
        rc = launch_tr(a, &b, st);
    }
    if (rc) return rc;
    ProfileScope ev(QBLORA_PROFILE_GRAD_REDUCE, st);
    if (!reduce_by_tiles(a) && reduce_by_tiles(b)) {         // the usual case (dA plain, dB transposed): one launch
        GradPair p{};
        p.a = a; p.b = b; p.n_a = (int)reduce_blocks(a);
        hipLaunchKernelGGL(k_grad_reduce_pair, dim3(reduce_blocks(a) + reduce_blocks(b)), dim3(256), 0, st, p);
        return launch_status();
    }
    if ((rc = launch_reduce(a, st))) return rc;
    return launch_reduce(b, st);
}

}  // namespace qblora
