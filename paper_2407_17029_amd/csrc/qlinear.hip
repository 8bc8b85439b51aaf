// Dequantize-and-contract kernel of the adapted layer for gfx950 (Alg. 1 qblora_forward:
// W_tilde = dequantize(...), x @ W_tilde, plus the adapter term; and its transpose for the
// backward pass with respect to the activations).
//
//   C[M,N] = X1[M,K1] * Wq^T  +  X2[M,K2] * W2[N/div2, K2]^T
//
// Segment 1 reads the 4-bit codes and block scales of the frozen base weight from HBM, rebuilds
// bf16 weights (Eq. 1: c[code]*alpha (+beta), fp32 then round-to-nearest-even) straight into an
// LDS tile and feeds them to v_mfma_f32_32x32x16_bf16 with fp32 accumulation; the dequantized
// weight never exists in HBM.  QMODE 1 contracts along d_in (forward); QMODE 2 uses the same
// stored tile transposed and contracts along d_out (backward w.r.t. activations) -- there the
// scale varies along the contraction index, which is why it is applied while building the tile
// and not to the accumulator.  Segment 2 is a plain bf16 K-extension: the adapter's rank-R product
// rides in the same accumulators as R extra contraction steps (forward: X2 = s*U, W2 = B^T with
// output row n using row n/lambda2, i.e. repeat_interleave; backward: X2 = dU/lambda1, W2 = A with
// row k/lambda1).
//
// Shape of the computation on a CU: one workgroup of 256 threads (4 wave64, one per SIMD) owns a
// 256 x 256 output tile; every wave owns a 128 x 128 quadrant, i.e. 16 MFMA accumulators of
// 32 x 32 (256 registers), so one k-step of 64 issues 64 MFMAs against 32 16-byte LDS fragment
// reads per wave.  Both operand tiles live in LDS as [row][64 k] bf16 (128 bytes per row) with the
// 16-byte chunks of a row XOR-swizzled by (row ^ row>>3) & 7, double buffered, one barrier per
// k-step.  Activation tiles (and the bf16 tiles of segment 2) go from global memory directly into
// LDS (global_load_lds, 16 bytes per lane; the swizzle is applied by choosing which global chunk a
// lane fetches).  Codes and scales are fetched two k-steps ahead into registers and dequantized
// between the MFMAs of the step before they are needed.
// The weight tile is the MFMA A operand and the token tile the B operand, so a lane ends up with 4
// consecutive output features of one token and stores them as one 8-byte word.
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 256;
constexpr int BM = 256, BN = 256, kBK = 64;
constexpr int kTileBytes = 256 * 128;                       // one operand tile: 256 rows x 128 bytes
constexpr int kTableBytes = 256 * 128;                      // byte-indexed pair table, 16 replicas

__device__ __align__(16) const uint32_t g_zero_chunk[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ int swz(int row, int chunk) {
    return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

// One wave-wide global -> LDS copy: lane i fetches the 16 bytes at base + offset_i and they land at
// lds_base + 16*i (M0 carries the wave-uniform LDS byte address).  Written as assembly so that the
// compiler's wait-count bookkeeping does not tie later LDS accesses to these copies; every copy is
// completed by the explicit vmcnt(0) in front of the barrier that publishes the tile.
__device__ __forceinline__ void copy16_to_lds(const void* src, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_base), "v"(src) : "memory");
}
__device__ __forceinline__ void copy16_to_lds(const void* uniform_base, uint32_t lane_offset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(lane_offset), "s"(uniform_base) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// codes / scales of one k-step held in registers
template <int QMODE>
struct Staged {
    uint32_t cw[8];          // QMODE 1: the 64 codes of this thread's row; QMODE 2: 8 codes of each of 8 rows
    float sc[QMODE == 2 ? 8 : 1];
    float be[QMODE == 2 ? 8 : 1];
};

template <int QMODE, bool BETA>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_qlinear(GemmDesc d) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* sX = smem;                                   // 2 tiles
    unsigned char* sW = sX + 2 * kTileBytes;                    // 2 tiles
    unsigned char* sT = smem + 4 * kTileBytes;                  // pair table, see below

    // Every field of the descriptor the loop touches is copied into a local first: the copies in
    // the loop are assembly statements that clobber memory, and values must not be re-read around them.
    const int64_t M = d.M;
    const int N = d.N, d_in = d.d_in, d_out = d.d_out, K2 = d.K2, div2 = d.div2;
    const qblora_bf16* const X1 = d.X1; const int64_t ldx1 = d.ldx1;
    const qblora_bf16* const X2 = d.X2; const int64_t ldx2 = d.ldx2;
    const qblora_bf16* const W2 = d.W2; const int64_t ldw2 = d.ldw2;
    const uint8_t* const codes = d.codes;
    const float* const scales = d.scales;
    const float* const beta = d.beta;
    qblora_bf16* const C = reinterpret_cast<qblora_bf16*>(d.C);
    const int64_t ldc = d.ldc;
    const float out_scale = d.out_scale;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm0 = (wave & 1) * 128, wn0 = (wave >> 1) * 128;

    // ---- tile assignment: XCD-contiguous, grouped along tokens ---------------------------------
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
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

    // Pair table: a byte of codes (two adjacent k, low nibble first) selects the 8-byte entry
    // (c[lo], c[hi]) -- one LDS read dequantizes two weights.  The 256 entries are replicated 16 times,
    // entry b of replica q at b*128 + q*8, and lane l reads replica l & 15: whatever the bytes are, the
    // 16 lanes the LDS serves together touch 16 different bank pairs.
    if (t < 16) reinterpret_cast<float*>(sT)[t] = d.cb.c[t];
    __syncthreads();
    {
        const float c_lo = reinterpret_cast<const float*>(sT)[t & 15], c_hi = reinterpret_cast<const float*>(sT)[t >> 4];
        __syncthreads();
        const float4 e = make_float4(c_lo, c_hi, c_lo, c_hi);
#pragma unroll
        for (int q = 0; q < 8; ++q) *reinterpret_cast<float4*>(sT + t * 128 + q * 16) = e;
    }

    const int K1 = QMODE == 1 ? d_in : d_out;
    const int steps1 = K1 / kBK, steps2 = (K2 + kBK - 1) / kBK;
    const int nsteps = steps1 + steps2;
    const int bpr = d_in / kBlock;                // blocks per stored weight row

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // ---- direct global -> LDS copies -------------------------------------------------------------
    // Wave w fills rows 64w .. 64w+63 of a tile with 8 copies of 8 rows each.  In copy i, lane l
    // lands on row 64w + 8i + (l>>3), physical chunk l&7, which must hold logical chunk
    // (l&7) ^ swizzle(row); with row&7 = l>>3 and (row>>3)&7 = i that is (l&7) ^ (l>>3) ^ i.
    const int crow = lane >> 3;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * 64 * 128);
    // CHECK_K: chunks at or beyond K are fetched from a zero constant instead (K-extension only)
    auto copy_tile = [&](const bool check_k, const qblora_bf16* src, int64_t ld, int64_t row_base, int64_t row_max,
                         int div, int K, int k0, uint32_t tile_off) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int64_t row = row_base + wave * 64 + i * 8 + crow;
            row = row > row_max ? row_max : row;
            if (div != 1) row = (int64_t)((uint32_t)row / (uint32_t)div);      // only weight rows (< 2^31) are divided
            const int k = k0 + (((lane & 7) ^ crow ^ i) << 3);
            const qblora_bf16* p = src + row * ld + k;
            if (check_k)
                p = (k < K) ? p : reinterpret_cast<const qblora_bf16*>(g_zero_chunk);
            copy16_to_lds(p, lds0 + tile_off + i * 8 * 128);
        }
    };

    // ---- codes / scales -> registers -------------------------------------------------------------
    int qrow = 0, qcol = 0;
    const uint8_t* fwd_codes = nullptr;              // QMODE 1: this thread's 32 bytes of step 0 ...
    int fwd_stride = 32;                             // ... and the distance to the next step's
    const float* fwd_scales = nullptr;               // likewise for its block scale
    int fwd_scale_stride = 1;
    if constexpr (QMODE == 1) {
        qrow = n0 + t;                               // this thread's stored weight row
        if (qrow > N - 1) qrow = N - 1;
        if (d.codes_tiled) {                         // tile-ordered copy: the workgroup's step is one 8 KiB block
            fwd_codes = d.codes_tiled + tiled_run_offset(n0 + t, 0, bpr);
            fwd_stride = 256 * 32;
        } else {
            fwd_codes = codes + (int64_t)qrow * (d_in / 2);
        }
        if (d.scales_tiled) {
            fwd_scales = d.scales_tiled + tiled_run_offset(n0 + t, 0, bpr) / 32;
            fwd_scale_stride = 256;
        } else {
            fwd_scales = scales + (int64_t)qrow * bpr;
        }
    } else {
        qcol = n0 + 8 * (t & 31);                    // this thread's 8 stored columns (k of the layer)
        if (qcol > N - 8) qcol = N - 8;
    }
    auto load_staged = [&](Staged<QMODE>& s, int step) __attribute__((always_inline)) {
        const int k0 = step * kBK;
        if constexpr (QMODE == 1) {
            const uint4* p = reinterpret_cast<const uint4*>(fwd_codes + (int64_t)step * fwd_stride);
            uint4 v0 = p[0], v1 = p[1];
            s.cw[0] = v0.x; s.cw[1] = v0.y; s.cw[2] = v0.z; s.cw[3] = v0.w;
            s.cw[4] = v1.x; s.cw[5] = v1.y; s.cw[6] = v1.z; s.cw[7] = v1.w;
            s.sc[0] = fwd_scales[(int64_t)step * fwd_scale_stride];
            if constexpr (BETA) s.be[0] = beta[(int64_t)qrow * bpr + step];
        } else {
            const int nb = k0 + 8 * (t >> 5);        // 8 stored rows (contraction index)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t n = nb + i;
                s.cw[i] = *reinterpret_cast<const uint32_t*>(codes + n * (d_in / 2) + qcol / 2);
                const int64_t blk = n * bpr + qcol / kBlock;
                s.sc[i] = scales[blk];
                if constexpr (BETA) s.be[i] = beta[blk];
            }
        }
    };

    // Segment-1 activation tiles: per-lane byte offsets relative to the tile's first row are fixed for
    // the whole kernel, the uniform base walks along k.
    uint32_t xoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int64_t lrow = wave * 64 + i * 8 + crow;
        if (m0 + lrow > M - 1) lrow = M - 1 - m0;
        xoff[i] = (uint32_t)(lrow * ldx1 * 2) + ((((lane & 7) ^ crow ^ i)) << 4);
    }
    const qblora_bf16* const x1_tile = X1 + m0 * ldx1;
    // Copies of a quantized step's token tile in two halves of 4, and all copies of any step.
    auto issue_x1_half = [&](int step, int buf, int half) __attribute__((always_inline)) {
        const qblora_bf16* base = x1_tile + step * kBK;
#pragma unroll
        for (int i = 4 * half; i < 4 * half + 4; ++i)
            copy16_to_lds(base, xoff[i], lds0 + buf * kTileBytes + i * 8 * 128);
    };
    auto issue_copies = [&](int step, int buf) __attribute__((always_inline)) {
        if (step < steps1) {
            issue_x1_half(step, buf, 0);
            issue_x1_half(step, buf, 1);
        } else {
            const int k0 = (step - steps1) * kBK;
            copy_tile(true, X2, ldx2, m0, M - 1, 1, K2, k0, buf * kTileBytes);
            copy_tile(true, W2, ldw2, n0, N - 1, div2, K2, k0, (2 + buf) * kTileBytes);
        }
    };

    // ---- one k-step ----------------------------------------------------------------------------------
    // A wave runs alone on its SIMD, so nothing hides an LDS round trip or a barrier but its own
    // MFMAs.  The 64 MFMAs of a step are cut into 8 slices of 8 (about 256 cycles each) and all other
    // work is pinned to slices (plan at run_step): fragments and table values are read two slices
    // before their use; the barrier that publishes the next tiles sits in front of slice 6, so the
    // last 16 MFMAs of a step cover it and the first fragment reads of the next step.
    // Scheduling barriers keep work inside its slice; group barriers spread it between the MFMAs.
    const int r = lane & 31, hi = lane >> 5;
    bf16x8 wf[2][4], xf[2][4];      // two fragment sets; set 0 holds quarter 0 when a step starts
    auto read_wf = [&](const unsigned char* bw, int ks, bf16x8 (&f)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 4; ++a) f[a] = *reinterpret_cast<const bf16x8*>(bw + swz(wn0 + a * 32 + r, ks * 2 + hi));
    };
    auto read_xf = [&](const unsigned char* bx, int ks, bf16x8 (&f)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < 4; ++b) f[b] = *reinterpret_cast<const bf16x8*>(bx + swz(wm0 + b * 32 + r, ks * 2 + hi));
    };
    // Dequantization of a staged k-step in 4 pieces of 16 elements (two 16-byte LDS stores each):
    //   QMODE 1: piece q = dwords 2q, 2q+1 of this thread's row (8 bytes of codes) -> chunks 2q, 2q+1 of LDS row t;
    //   QMODE 2: piece q = byte q (columns 2q, 2q+1) of each of the 8 stored rows of this thread's 8x8
    //            patch -> LDS rows 8*kg+2q and 8*kg+2q+1, chunk ng (packing down the columns transposes).
    const uint32_t table_lane = lds_address(sT) - lds_address(smem) + ((lane & 15) << 3);
    auto table_offsets = [&](const Staged<QMODE>& s, int q, uint32_t (&li)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t w = QMODE == 1 ? s.cw[2 * q + (i >> 2)] : s.cw[i];
            const int byte = QMODE == 1 ? (i & 3) : q;
            const uint32_t sh = byte == 0 ? (w << 7) : (w >> (8 * byte - 7));
            li[i] = (sh & 0x7f80u) | table_lane;
        }
    };
    auto table_reads = [&](const uint32_t (&li)[8], float2 (&lv)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) lv[i] = *reinterpret_cast<const float2*>(smem + li[i]);
    };
    auto finish_piece = [&](const Staged<QMODE>& s, int q, const float2 (&lv)[8], unsigned char* tile)
        __attribute__((always_inline)) {
        float lo[8], hi[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int si = QMODE == 1 ? 0 : i;
            lo[i] = BETA ? __fmaf_rn(lv[i].x, s.sc[si], s.be[si]) : __fmul_rn(lv[i].x, s.sc[si]);
            hi[i] = BETA ? __fmaf_rn(lv[i].y, s.sc[si], s.be[si]) : __fmul_rn(lv[i].y, s.sc[si]);
        }
        if constexpr (QMODE == 1) {
            // byte i holds elements 2i, 2i+1 of the 16: adjacent k, packed as they come
            uint4 o0, o1;
            o0.x = pack_bf16(lo[0], hi[0]); o0.y = pack_bf16(lo[1], hi[1]);
            o0.z = pack_bf16(lo[2], hi[2]); o0.w = pack_bf16(lo[3], hi[3]);
            o1.x = pack_bf16(lo[4], hi[4]); o1.y = pack_bf16(lo[5], hi[5]);
            o1.z = pack_bf16(lo[6], hi[6]); o1.w = pack_bf16(lo[7], hi[7]);
            *reinterpret_cast<uint4*>(tile + swz(t, 2 * q)) = o0;
            *reinterpret_cast<uint4*>(tile + swz(t, 2 * q + 1)) = o1;
        } else {
            // lo[i] / hi[i] are columns 2q / 2q+1 of stored row i: pack down each column
            uint4 o0, o1;
            o0.x = pack_bf16(lo[0], lo[1]); o0.y = pack_bf16(lo[2], lo[3]);
            o0.z = pack_bf16(lo[4], lo[5]); o0.w = pack_bf16(lo[6], lo[7]);
            o1.x = pack_bf16(hi[0], hi[1]); o1.y = pack_bf16(hi[2], hi[3]);
            o1.z = pack_bf16(hi[4], hi[5]); o1.w = pack_bf16(hi[6], hi[7]);
            *reinterpret_cast<uint4*>(tile + swz(8 * (t & 31) + 2 * q, t >> 5)) = o0;
            *reinterpret_cast<uint4*>(tile + swz(8 * (t & 31) + 2 * q + 1, t >> 5)) = o1;
        }
    };
    auto dequant_store = [&](const Staged<QMODE>& s, unsigned char* tile) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t li[8];
            float2 lv[8];
            table_offsets(s, q, li);
            table_reads(li, lv);
            finish_piece(s, q, lv, tile);
        }
    };
    auto mfma_row = [&](int a, const bf16x8 (&fw)[4], const bf16x8 (&fx)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < 4; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[a], fx[b], acc[a][b], 0, 0, 0);
    };
    // dq: dequantize `sdq` into bw_next during this step; has_next: a step follows (its tiles are in
    // bx_next / bw_next once the barrier is passed).  Both are literal `true` in the steady state.
    //
    // Slice plan (8 MFMAs per slice; fragment set = quarter & 1; every LDS read two slices before use):
    //   0: table reads of piece 0, fragments of quarter 1, offsets of piece 1
    //   1: table reads of piece 1, offsets of piece 2
    //   2: table reads of piece 2, fragments of quarter 2, finish piece 0, offsets of piece 3
    //   3: table reads of piece 3, finish piece 1
    //   4: fragments of quarter 3, finish piece 2
    //   5: finish piece 3
    //   6: wait for the copies, barrier, fragments of quarter 0 of the next step; with `refill`, first
    //      half of the token-tile copies of quantized step `step2` (the step after next) into the
    //      buffer this step has just finished reading
    //   7: second half of those copies
    auto run_step = [&](const unsigned char* bx, const unsigned char* bw, const unsigned char* bx_next,
                        unsigned char* bw_next, const bool dq, const Staged<QMODE>& sdq, const bool has_next,
                        const bool refill, const int step2, const int buf2) __attribute__((always_inline)) {
        float2 lv[3][8];
        uint32_t li[3][8];
        if (dq) table_offsets(sdq, 0, li[0]);
#pragma unroll
        for (int h = 0; h < 8; ++h) {
            const int ks = h >> 1, half = h & 1, cur = ks & 1, nxt = cur ^ 1;
            if (h == 6 && has_next) {
                __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): direct copies and staged codes
                __syncthreads();                           // next tiles published; this step's tiles free
                read_wf(bw_next, 0, wf[0]);
                read_xf(bx_next, 0, xf[0]);
                if (refill) issue_x1_half(step2, buf2, 0);  // this step's token buffer is free: refill it
                __builtin_amdgcn_sched_barrier(0);
            }
            if (h == 7 && has_next && refill) issue_x1_half(step2, buf2, 1);
            if (dq) {
                if (h >= 2 && h <= 5) finish_piece(sdq, h - 2, lv[(h - 2) % 3], bw_next);
                if (h <= 3) table_reads(li[h % 3], lv[h % 3]);
                if (h == 0) table_offsets(sdq, 1, li[1]);
                if (h == 1) { table_offsets(sdq, 2, li[2]); table_offsets(sdq, 3, li[0]); }
            }
            if (half == 0 && ks < 3) {
                read_wf(bw, ks + 1, wf[nxt]);
                read_xf(bx, ks + 1, xf[nxt]);
            }
            mfma_row(2 * half, wf[cur], xf[cur]);
            mfma_row(2 * half + 1, wf[cur], xf[cur]);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                   // vector ALU
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                   // LDS reads
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);                   // vector ALU
                if (i == 3 || i == 7) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // a piece's LDS stores
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ---------------------------------------------------------------------------------
    // Invariant at the top of step s: tile buffers s&1 hold step s and fragment set 0 holds its first
    // quarter; st[(s+1)&1] holds the codes of step s+1 (if that is a quantized step).
    Staged<QMODE> st[2];
    if (nsteps > 0) {
        issue_copies(0, 0);
        int issued = 0;                                    // copies are in flight or done for steps <= issued
        if (steps1 > 1) { issue_copies(1, 1); issued = 1; }
        if (steps1 > 0) load_staged(st[0], 0);
        if (steps1 > 1) load_staged(st[1], 1);
        __syncthreads();                                   // pair table visible
        if (steps1 > 0) dequant_store(st[0], sW);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        read_wf(sW, 0, wf[0]);
        read_xf(sX, 0, xf[0]);
        int s = 0;
        // Quantized steps whose successor is quantized too (the successor's tile is dequantized during
        // the step), unrolled by two so that the staging registers and the tile buffers have fixed
        // names.  Codes are fetched two steps ahead; past the end the last quantized step is fetched
        // again (in bounds, unused) so that the body has no conditions.  A step refills its own token
        // buffer with the copies of the step after next (when that is a quantized step) behind its
        // barrier, under its last 16 MFMAs.
        const int last_q = steps1 - 1;
        for (; s + 2 < steps1; s += 2) {
            load_staged(st[0], min(s + 2, last_q));
            run_step(sX, sW, sX + kTileBytes, sW + kTileBytes, true, st[1], true, true, s + 2, 0);
            load_staged(st[1], min(s + 3, last_q));
            const bool more = s + 3 < steps1;
            run_step(sX + kTileBytes, sW + kTileBytes, sX, sW, true, st[0], true, more, s + 3, 1);
            issued = more ? s + 3 : s + 2;
        }
        if (s + 1 < steps1) {
            run_step(sX, sW, sX + kTileBytes, sW + kTileBytes, true, st[1], true, false, 0, 0);
            ++s;
        }
        // the last quantized step and the K-extension steps: nothing to dequantize; copies of the next
        // step are issued at the top of a step when no earlier step has done it
        for (; s < nsteps; ++s) {
            const int buf = s & 1;
            const bool has_next = s + 1 < nsteps;
            if (has_next && issued < s + 1) { issue_copies(s + 1, buf ^ 1); issued = s + 1; }
            run_step(sX + buf * kTileBytes, sW + buf * kTileBytes, sX + (buf ^ 1) * kTileBytes,
                     sW + (buf ^ 1) * kTileBytes, false, st[0], has_next, false, 0, 0);
        }
    }

    __builtin_amdgcn_s_waitcnt(0x0F70);                    // nothing may still be writing this workgroup's LDS

    // ---- epilogue ---------------------------------------------------------------------------------------
    // A lane holds features n..n+3 of one token per accumulator quad, i.e. 8 bytes of an output row.
    // The wave first lays its 128 x 128 quadrant out in LDS (the tiles are dead by now) as bf16 rows of
    // 256 bytes (pitch 272), then reads it back 16 bytes per lane so that every global store
    // instruction writes four complete 256-byte row segments.
    __syncthreads();                                       // every wave is done reading the tiles
    {
        constexpr int kPitch = 272;
        unsigned char* eb = smem + wave * (128 * kPitch);
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 o;
                    o.x = pack_bf16(acc[a][b][q * 4 + 0] * out_scale, acc[a][b][q * 4 + 1] * out_scale);
                    o.y = pack_bf16(acc[a][b][q * 4 + 2] * out_scale, acc[a][b][q * 4 + 3] * out_scale);
                    *reinterpret_cast<uint2*>(eb + (b * 32 + r) * kPitch + (a * 32 + q * 8 + hi * 4) * 2) = o;
                }
        const int erow = lane >> 4, echunk = lane & 15;
        const int n = n0 + wn0 + echunk * 8;
#pragma unroll 8
        for (int i = 0; i < 32; ++i) {
            const int row = i * 4 + erow;
            const uint4 v = *reinterpret_cast<const uint4*>(eb + row * kPitch + echunk * 16);
            const int64_t m = m0 + wm0 + row;
            if (m < M && n < N) *reinterpret_cast<uint4*>(C + m * ldc + n) = v;
        }
    }
}

template <int QMODE, bool BETA>
int launch_cfg(const GemmDesc& d, hipStream_t st) {
    constexpr size_t smem = 4 * kTileBytes + kTableBytes;
    auto kern = k_qlinear<QMODE, BETA>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return QBLORA_ERR_LAUNCH;
        attr_set = true;
    }
    int64_t tiles = ((d.M + BM - 1) / BM) * ((d.N + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kThreads), smem, st, d);
    return launch_status();
}

}  // namespace

// The quantized GEMMs of the layer (qmode 1 or 2, bf16 output, no auxiliary outputs).
int launch_qlinear(const GemmDesc& d, hipStream_t st) {
    if (d.M <= 0 || d.N <= 0) return QBLORA_OK;
    if (d.out_f32 || d.C2 || d.C_lo) return QBLORA_ERR_UNSUPPORTED;
    if (d.qmode == 1) return d.beta ? launch_cfg<1, true>(d, st) : launch_cfg<1, false>(d, st);
    if (d.qmode == 2) return d.beta ? launch_cfg<2, true>(d, st) : launch_cfg<2, false>(d, st);
    return QBLORA_ERR_UNSUPPORTED;
}

}  // namespace qblora
