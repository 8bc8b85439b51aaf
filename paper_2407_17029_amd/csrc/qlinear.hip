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
// row k/lambda1).  QMODE 0 is the same contraction on a weight that has already been dequantized once (the
// layer does that when the batch is large, so that a weight is not rebuilt by every token tile) into a bf16
// buffer in MFMA operand order: the 16 bytes lane l needs for rows 32i..32i+31 and the 16-wide k slice j sit at
// ((i*(K1/16) + j)*64 + l)*16.  A wave then loads its weight fragments straight from global memory into
// registers, one step ahead, 1 KB contiguous per instruction, and only the token tile goes through LDS: filling
// LDS is the slow side of this CU (direct copies 64 B/clk, ds_write_b128 85 B/clk against 200 B/clk reads).
//
// Shape of the computation on a CU: one workgroup of 512 threads (8 wave64, two per SIMD) owns a
// 256 x 256 output tile; a wave owns 128 tokens x 64 features = 8 MFMA accumulators of 32 x 32
// (128 registers).  Two waves per SIMD matter: a single wave cannot issue MFMAs back to back at the
// full rate of the matrix pipe, and the dequantization arithmetic of one wave issues in the shadow
// of the other wave's MFMAs.  Both operand tiles live in LDS as [row][64 k] bf16 (128 bytes per
// row) with the 16-byte chunks of a row XOR-swizzled by (row ^ row>>3) & 7, double buffered, one
// barrier per k-step.  Activation tiles (and both bf16 tiles of segment 2) go from global memory
// directly into LDS (global_load_lds, 16 bytes per lane; the swizzle is applied by choosing which
// global chunk a lane fetches).  Codes and scales are fetched two k-steps ahead into registers and
// dequantized between the MFMAs of the step before they are needed, through a byte-indexed table
// in LDS that turns one byte of codes into two fp32 code values.
// The weight tile is the MFMA A operand and the token tile the B operand, so a lane ends up with 4
// consecutive output features of one token and stores them as one 8-byte word.
#include "common.h"

namespace qblora {

namespace {

constexpr int kThreads = 512;
constexpr int BM = 256, BN = 256, kBK = 64;
constexpr int kTileBytes = 256 * 128;                       // one operand tile: 256 rows x 128 bytes
constexpr int kTableBytes = 256 * 128;                      // byte-indexed pair table, 16 replicas

__device__ __align__(16) const uint32_t g_zero_chunk[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ int swz(int row, int chunk) {
    return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

// One wave-wide global -> LDS copy: lane i fetches 16 bytes and they land at lds_base + 16*i (M0
// carries the wave-uniform LDS byte address).  Written as assembly so that the compiler's wait-count
// bookkeeping does not tie later LDS accesses to these copies; every copy is completed by the
// explicit vmcnt(0) in front of the barrier that publishes the tile.
__device__ __forceinline__ void copy16_to_lds(const void* src, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_base), "v"(src) : "memory");
}
__device__ __forceinline__ void copy16_to_lds(const void* uniform_base, uint32_t lane_offset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(lane_offset), "s"(uniform_base) : "memory");
}

// 16 bytes per lane from uniform_base + lane_offset + IMM into registers.  The data arrive asynchronously: the
// value may only be used behind a wait_vm that names it (vmcnt counts every copy and load of this kernel's
// loop, which are all issued by statements like these, in program order).
template <int IMM>
__device__ __forceinline__ void load_operand16(bf16x8& v, uint32_t lane_offset, const void* uniform_base) {
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3"
                 : "=&v"(v) : "v"(lane_offset), "s"(uniform_base), "n"(IMM) : "memory");
}
// waits until at most N of this wave's copies / loads are outstanding; a and b are usable afterwards
template <int N>
__device__ __forceinline__ void wait_vm(bf16x8& a, bf16x8& b) {
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}

// value of lane `src` (0..3, a constant after unrolling) of the caller's quad
__device__ __forceinline__ float quad_broadcast(float v, int src) {
    const int x = __float_as_int(v);
    switch (src) {
        case 0: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x00, 0xf, 0xf, false));
        case 1: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x55, 0xf, 0xf, false));
        case 2: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xAA, 0xf, 0xf, false));
        default: return __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xFF, 0xf, 0xf, false));
    }
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// codes / scales of one k-step held in registers: 32 weights per thread
//   QMODE 1: half a stored row (16 bytes of codes), one scale -- or, with 8 x 8 quantization blocks
//            (BR = 8), one scale per code dword (8 inputs = one block column)
//   QMODE 2: a patch of 4 stored rows x 8 columns (one dword per row); one scale per thread: the
//            patch's own with BR = 8, else that of row (lane & 3) of the patch, shared inside the quad
template <int QMODE, int BR>
struct Staged {
    uint32_t cw[4];
    float sc[(QMODE == 1 && BR == 8) ? 4 : 1];
    float be[(QMODE == 1 && BR == 8) ? 4 : 1];
};

template <int QMODE, bool BETA, int BR>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_qlinear(GemmDesc d) {
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
    const int wm0 = (wave & 1) * 128, wn0 = (wave >> 1) * 64;

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
    // entry b of replica q at b*128 + q*8, and lane l reads replica l & 15, so that lanes of one
    // 16-lane group never collide whatever their bytes are.
    if constexpr (QMODE != 0) {
        if (t < 16) reinterpret_cast<float*>(sT)[t] = d.cb.c[t];
        __syncthreads();
        const int b = t & 255;
        const float c_lo = reinterpret_cast<const float*>(sT)[b & 15], c_hi = reinterpret_cast<const float*>(sT)[b >> 4];
        __syncthreads();
        const float4 e = make_float4(c_lo, c_hi, c_lo, c_hi);
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<float4*>(sT + b * 128 + (t >> 8) * 64 + q * 16) = e;
    }

    const int K1 = QMODE == 0 ? d.K1 : QMODE == 1 ? d_in : d_out;
    const int steps1 = K1 / kBK, steps2 = (K2 + kBK - 1) / kBK;
    const int nsteps = steps1 + steps2;
    const int bpr = d_in / kBlock;                // blocks per stored weight row

    f32x16 acc[2][4];                             // [feature block][token block]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // ---- direct global -> LDS copies -------------------------------------------------------------
    // Wave w fills rows 32w .. 32w+31 of a tile with 4 copies of 8 rows each.  In copy i, lane l
    // lands on row 32w + 8i + (l>>3), physical chunk l&7, which must hold logical chunk
    // (l&7) ^ swizzle(row); with row&7 = l>>3 and (row>>3)&7 = (4w+i)&7 that is (l&7) ^ (l>>3) ^ (4w+i).
    const int crow = lane >> 3;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + wave * 32 * 128);
    // check_k: chunks at or beyond K are fetched from a zero constant instead (K-extension only)
    auto copy_tile = [&](const bool check_k, const qblora_bf16* src, int64_t ld, int64_t row_base, int64_t row_max,
                         int div, int K, int k0, uint32_t tile_off) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int64_t row = row_base + wave * 32 + i * 8 + crow;
            row = row > row_max ? row_max : row;
            if (div != 1) row = (int64_t)((uint32_t)row / (uint32_t)div);      // only weight rows (< 2^31) are divided
            const int k = k0 + (((lane & 7) ^ crow ^ ((4 * wave + i) & 7)) << 3);
            const qblora_bf16* p = src + row * ld + k;
            if (check_k)
                p = (k < K) ? p : reinterpret_cast<const qblora_bf16*>(g_zero_chunk);
            copy16_to_lds(p, lds0 + tile_off + i * 8 * 128);
        }
    };
    // Segment-1 activation tiles: per-lane byte offsets relative to the tile's first row are fixed for
    // the whole kernel, the uniform base walks along k.
    uint32_t xoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t lrow = wave * 32 + i * 8 + crow;
        if (m0 + lrow > M - 1) lrow = M - 1 - m0;
        xoff[i] = (uint32_t)(lrow * ldx1 * 2) + (((lane & 7) ^ crow ^ ((4 * wave + i) & 7)) << 4);
    }
    const qblora_bf16* const x1_tile = X1 + m0 * ldx1;
    auto issue_x1 = [&](int step, int buf) __attribute__((always_inline)) {
        const qblora_bf16* base = x1_tile + step * kBK;
#pragma unroll
        for (int i = 0; i < 4; ++i) copy16_to_lds(base, xoff[i], lds0 + buf * kTileBytes + i * 8 * 128);
    };
    // QMODE 0: per-lane byte offsets of this wave's two 32-row blocks in the operand-ordered weight
    uint32_t wvoff[2] = {0u, 0u};
    const unsigned char* const wop = reinterpret_cast<const unsigned char*>(d.W1);
    if constexpr (QMODE == 0) {
        const int blocks32 = (N + 31) / 32;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            int nb = (n0 + wn0) / 32 + a;
            nb = nb > blocks32 - 1 ? blocks32 - 1 : nb;      // rows past N: any valid block, results never stored
            wvoff[a] = (uint32_t)nb * (uint32_t)(d.K1 / 16) * 1024u + (uint32_t)lane * 16u;
        }
    }
    auto issue_copies = [&](int step, int buf) __attribute__((always_inline)) {
        if (step < steps1) {
            issue_x1(step, buf);
        } else {
            const int k0 = (step - steps1) * kBK;
            copy_tile(true, X2, ldx2, m0, M - 1, 1, K2, k0, buf * kTileBytes);
            copy_tile(true, W2, ldw2, n0, N - 1, div2, K2, k0, (2 + buf) * kTileBytes);
        }
    };

    // ---- codes / scales -> registers -------------------------------------------------------------
    int qrow = 0, qcol = 0;
    const uint8_t* fwd_codes = nullptr; int fwd_stride = 32;
    const float* fwd_scales = nullptr; int fwd_scale_stride = 1;
    if constexpr (QMODE == 1) {
        qrow = n0 + (t >> 1);                        // this thread's stored weight row (it owns half of it)
        if (qrow > N - 1) qrow = N - 1;
        if (d.codes_tiled) { fwd_codes = d.codes_tiled + tiled_run_offset(n0 + (t >> 1), 0, bpr) + (t & 1) * 16; fwd_stride = 256 * 32; }
        else fwd_codes = codes + (int64_t)qrow * (d_in / 2) + (t & 1) * 16;
        if (d.scales_tiled) { fwd_scales = d.scales_tiled + tiled_run_offset(n0 + (t >> 1), 0, bpr) / 32; fwd_scale_stride = 256; }
        else fwd_scales = scales + (int64_t)qrow * bpr;
    } else if constexpr (QMODE == 2) {
        qcol = n0 + 8 * (t & 31);                    // this thread's 8 stored columns (k of the layer)
        if (qcol > N - 8) qcol = N - 8;
    }
    auto load_staged = [&](Staged<QMODE, BR>& s, int step) __attribute__((always_inline)) {
        const int k0 = step * kBK;
        if constexpr (QMODE == 1) {
            const uint4 v = *reinterpret_cast<const uint4*>(fwd_codes + (int64_t)step * fwd_stride);
            s.cw[0] = v.x; s.cw[1] = v.y; s.cw[2] = v.z; s.cw[3] = v.w;
            if constexpr (BR == 8) {
                // block columns 8*step + 4*half .. +3 of block row qrow/8: one scale per code dword
                const int64_t b0 = (int64_t)(qrow >> 3) * (d_in >> 3) + 8 * step + 4 * (t & 1);
                const float4 a4 = *reinterpret_cast<const float4*>(scales + b0);
                s.sc[0] = a4.x; s.sc[1] = a4.y; s.sc[2] = a4.z; s.sc[3] = a4.w;
                if constexpr (BETA) {
                    const float4 b4 = *reinterpret_cast<const float4*>(beta + b0);
                    s.be[0] = b4.x; s.be[1] = b4.y; s.be[2] = b4.z; s.be[3] = b4.w;
                }
            } else {
                s.sc[0] = fwd_scales[(int64_t)step * fwd_scale_stride];
                if constexpr (BETA) s.be[0] = beta[(int64_t)qrow * bpr + step];
            }
        } else {
            const int nb = k0 + 4 * (t >> 5);        // 4 stored rows (contraction index)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t n = nb + i;
                s.cw[i] = *reinterpret_cast<const uint32_t*>(codes + n * (d_in / 2) + qcol / 2);
            }
            // One scale load per thread: with 8 x 8 blocks the patch lies in one block; with row-segment
            // blocks the four lanes of a quad (32 consecutive columns, inside one 64-block) each fetch
            // the scale of one of the four rows and the multiply reads it through a quad broadcast.
            const int64_t blk = BR == 8 ? (int64_t)(nb >> 3) * (d_in >> 3) + (qcol >> 3)
                                        : (int64_t)(nb + (t & 3)) * bpr + qcol / kBlock;
            s.sc[0] = scales[blk];
            if constexpr (BETA) s.be[0] = beta[blk];
        }
    };

    // ---- dequantization of a staged k-step: 4 pieces of 8 weights (4 table reads each) per thread ----------
    //   QMODE 1: piece p = code dword p of this thread's half row -> chunk 4*half+p of LDS row t>>1;
    //   QMODE 2: piece p = byte p (columns 2p, 2p+1) of each of the 4 stored rows of the patch -> 8-byte halves
    //            of LDS rows 8*kg+2p and 8*kg+2p+1 (packing down the columns transposes).
    constexpr int kPieces = 4, kReads = 4;
    const uint32_t table_lane = lds_address(sT) - lds_address(smem) + ((lane & 15) << 3);
    auto table_offsets = [&](const Staged<QMODE, BR>& s, int p, uint32_t (&li)[kReads]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kReads; ++i) {
            // QMODE 1: i = byte of dword p;  QMODE 2: i = stored row, byte p of its dword
            const uint32_t w = QMODE == 1 ? s.cw[p] : s.cw[i];
            const int byte = QMODE == 1 ? i : p;
            const uint32_t sh = byte == 0 ? (w << 7) : (w >> (8 * byte - 7));
            li[i] = (sh & 0x7f80u) | table_lane;
        }
    };
    auto table_reads = [&](const uint32_t (&li)[kReads], float2 (&lv)[kReads]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kReads; ++i) lv[i] = *reinterpret_cast<const float2*>(smem + li[i]);
    };
    auto finish_piece = [&](const Staged<QMODE, BR>& s, int p, const float2 (&lv)[kReads], unsigned char* tile)
        __attribute__((always_inline)) {
        float lo[kReads], hi[kReads];
#pragma unroll
        for (int i = 0; i < kReads; ++i) {
            float sc, be = 0.0f;
            if constexpr (QMODE == 2 && BR == 1) {           // row i of the patch: lane i of the quad holds its scale
                sc = quad_broadcast(s.sc[0], i);
                if constexpr (BETA) be = quad_broadcast(s.be[0], i);
            } else {
                const int si = QMODE == 2 ? 0 : (BR == 8 ? p : 0);
                sc = s.sc[si];
                if constexpr (BETA) be = s.be[si];
            }
            lo[i] = BETA ? __fmaf_rn(lv[i].x, sc, be) : __fmul_rn(lv[i].x, sc);
            hi[i] = BETA ? __fmaf_rn(lv[i].y, sc, be) : __fmul_rn(lv[i].y, sc);
        }
        if constexpr (QMODE == 1) {
            // byte i holds elements 2i, 2i+1 of the 8: adjacent k, packed as they come
            uint4 o0;
            o0.x = pack_bf16(lo[0], hi[0]); o0.y = pack_bf16(lo[1], hi[1]);
            o0.z = pack_bf16(lo[2], hi[2]); o0.w = pack_bf16(lo[3], hi[3]);
            *reinterpret_cast<uint4*>(tile + swz(t >> 1, 4 * (t & 1) + p)) = o0;
        } else {
            // lv[i] is (column 2p, column 2p+1) of stored row i: pack down each column
            const int kg = t & 31, ng = t >> 5;
            uint2 c0, c1;
            c0.x = pack_bf16(lo[0], lo[1]); c0.y = pack_bf16(lo[2], lo[3]);
            c1.x = pack_bf16(hi[0], hi[1]); c1.y = pack_bf16(hi[2], hi[3]);
            const int row = 8 * kg + 2 * p;
            *reinterpret_cast<uint2*>(tile + swz(row, ng >> 1) + 8 * (ng & 1)) = c0;
            *reinterpret_cast<uint2*>(tile + swz(row + 1, ng >> 1) + 8 * (ng & 1)) = c1;
        }
    };
    auto dequant_store = [&](const Staged<QMODE, BR>& s, unsigned char* tile) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < kPieces; ++p) {
            uint32_t li[kReads];
            float2 lv[kReads];
            table_offsets(s, p, li);
            table_reads(li, lv);
            finish_piece(s, p, lv, tile);
        }
    };

    // ---- one k-step ----------------------------------------------------------------------------------
    // Four quarters of 8 MFMAs (one 16-wide slice of k each).  Fragments of quarter q+1 are read during
    // quarter q (two fragment sets); the dequantization of the next weight tile is spread over the
    // first three quarters (table reads one quarter before the values are scaled and stored); the
    // barrier that publishes the next tiles sits in front of the last quarter, whose MFMAs cover it and
    // the first fragment reads of the next step.
    const int r = lane & 31, hi = lane >> 5;
    bf16x8 wf[2][2], xf[2][4];      // two fragment sets; set 0 holds quarter 0 when a step starts
    // Fragment addresses: row base + 32a + r, chunk 2ks + hi sits at (base + r)*128 + 4096a +
    // 16*[(hi ^ r ^ r>>3) & 7 ^ (2ks ^ 4(a&1))] -- one per-lane value XOR a constant plus an immediate;
    // the empty asm in run_step keeps the variants from being hoisted and held in registers.
    uint32_t frag_w = (uint32_t)(sW - smem) + (uint32_t)((wn0 + r) * 128 + (((hi ^ r ^ (r >> 3)) & 7) << 4));
    uint32_t frag_x = (uint32_t)(sX - smem) + (uint32_t)((wm0 + r) * 128 + (((hi ^ r ^ (r >> 3)) & 7) << 4));
    auto read_frags = [&](const unsigned char* bx, const unsigned char* bw, int ks, bf16x8 (&fw)[2], bf16x8 (&fx)[4])
        __attribute__((always_inline)) {
        const uint32_t wo = (uint32_t)(bw - sW), xo = (uint32_t)(bx - sX);
#pragma unroll
        for (int a = 0; a < 2; ++a)
            fw[a] = *reinterpret_cast<const bf16x8*>(smem + ((frag_w ^ (uint32_t)(((2 * ks) ^ (4 * (a & 1))) << 4)) + (wo + a * 4096)));
#pragma unroll
        for (int b = 0; b < 4; ++b)
            fx[b] = *reinterpret_cast<const bf16x8*>(smem + ((frag_x ^ (uint32_t)(((2 * ks) ^ (4 * (b & 1))) << 4)) + (xo + b * 4096)));
    };
    // dq: dequantize `sdq` into bw_next during this step; has_next: a step follows (its tiles are in
    // bx_next / bw_next once the barrier is passed); dq_next: the following step dequantizes `sdq_next`, whose
    // first piece is looked up behind this step's barrier (lv0 carries the values across the step boundary).
    // All flags are literal `true` in the steady state.
    float2 lv0[kReads];
    auto run_step = [&](const unsigned char* bx, const unsigned char* bw, const unsigned char* bx_next,
                        unsigned char* bw_next, const bool dq, const Staged<QMODE, BR>& sdq, const bool has_next,
                        const bool refill, const int step2, const int buf2, const bool dq_next,
                        const Staged<QMODE, BR>& sdq_next) __attribute__((always_inline)) {
        float2 lv[2][kReads];
        uint32_t li[kReads];
        asm volatile("" : "+v"(frag_w), "+v"(frag_x));
        if (dq) {
#pragma unroll
            for (int i = 0; i < kReads; ++i) lv[0][i] = lv0[i];
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            // the last piece is stored in front of the barrier that publishes the tile
            if (ks == 3 && dq) finish_piece(sdq, 3, lv[1], bw_next);
            if (ks == 3 && has_next) {
                __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): direct copies and staged codes
                __syncthreads();                           // next tiles published; this step's tiles free
                read_frags(bx_next, bw_next, 0, wf[0], xf[0]);
                if (refill) issue_x1(step2, buf2);         // this step's token buffer is free: refill it
            }
            if (ks < 3) read_frags(bx, bw, ks + 1, wf[nxt], xf[nxt]);
            if (dq && ks < 3) {
                // piece ks+1 is looked up while piece ks is scaled and stored
                table_offsets(sdq, ks + 1, li);
                table_reads(li, lv[nxt]);
            }
            if (ks == 3 && dq_next) {                      // the staged codes of the next step's tile have arrived
                // (the empty statement pins the address arithmetic behind the barrier: hoisted to the top of
                // the step it would wait for the code loads issued there)
                Staged<QMODE, BR> nx = sdq_next;
#pragma unroll
                for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(nx.cw[i]));
                table_offsets(nx, 0, li);
                table_reads(li, lv0);
            }
            __builtin_amdgcn_sched_barrier(0);             // LDS reads of the next quarter go out before this quarter's MFMAs
            if (dq && ks < 3) finish_piece(sdq, ks, lv[cur], bw_next);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][a], xf[cur][b], acc[a][b], 0, 0, 0);
            // the scaling arithmetic of the piece goes into the shadow of the MFMAs, two vector instructions each
#pragma unroll
            for (int i = 0; i < 7; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- QMODE 0: steps on the operand-ordered weight ---------------------------------------------------
    // wreg[ks][a] holds the weight fragment of quarter ks, feature block a.  In the steady state a step loads
    // the next step's fragment of a quarter right behind that quarter's MFMAs (into the registers they have
    // just read), so a load has a whole step to arrive.  Every copy and load of the loop is issued by an asm
    // statement in program order, per step: W(s+1,0) x2, W(s+1,1) x2, W(s+1,2) x2, X copies of step s+2 x4,
    // W(s+1,3) x2.  The fragment of quarter q < 3 was issued one step earlier and 10 operations have been
    // issued since, hence vmcnt(10); in front of the barrier of the last quarter the token copies of step s+1
    // and W(s,3) have the 6 loads of this step behind them, hence vmcnt(6).
    bf16x8 wreg[4][2];
    auto read_x = [&](const unsigned char* bx, int ks, bf16x8 (&fx)[4]) __attribute__((always_inline)) {
        const uint32_t xo = (uint32_t)(bx - sX);
#pragma unroll
        for (int b = 0; b < 4; ++b)
            fx[b] = *reinterpret_cast<const bf16x8*>(smem + ((frag_x ^ (uint32_t)(((2 * ks) ^ (4 * (b & 1))) << 4)) + (xo + b * 4096)));
    };
    auto mfma_quarter = [&](const int ks, const int cur) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks][a], xf[cur][b], acc[a][b], 0, 0, 0);
    };
    auto load_w_quarter = [&](const int ks, const void* base) __attribute__((always_inline)) {
        if (ks == 0) { load_operand16<0>(wreg[0][0], wvoff[0], base); load_operand16<0>(wreg[0][1], wvoff[1], base); }
        if (ks == 1) { load_operand16<1024>(wreg[1][0], wvoff[0], base); load_operand16<1024>(wreg[1][1], wvoff[1], base); }
        if (ks == 2) { load_operand16<2048>(wreg[2][0], wvoff[0], base); load_operand16<2048>(wreg[2][1], wvoff[1], base); }
        if (ks == 3) { load_operand16<3072>(wreg[3][0], wvoff[0], base); load_operand16<3072>(wreg[3][1], wvoff[1], base); }
    };
    // a step that is followed by another step on the operand-ordered weight (step + 1 < steps1)
    auto dense_step = [&](const unsigned char* bx, const unsigned char* bx_next, const bool refill, const int step,
                          const int buf2) __attribute__((always_inline)) {
        const void* const next_w = wop + (int64_t)(step + 1) * 4096;          // 4 slices of 1 KB per step
        asm volatile("" : "+v"(frag_x));
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks < 3) {
                read_x(bx, ks + 1, xf[nxt]);
                wait_vm<10>(wreg[ks][0], wreg[ks][1]);
            } else {
                wait_vm<6>(wreg[3][0], wreg[3][1]);        // also: this wave's token copies of the next step
                __syncthreads();                           // next token tile published; this step's tile free
                read_x(bx_next, 0, xf[0]);
                if (refill) issue_x1(step + 2, buf2);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_quarter(ks, cur);
            __builtin_amdgcn_sched_barrier(0);
            load_w_quarter(ks, next_w);
        }
    };
    // the last step on the operand-ordered weight: nothing more is loaded; if a K-extension step follows, its
    // tiles (8 copies, issued just before) are the youngest operations
    auto dense_last = [&](const unsigned char* bx, const unsigned char* bx_next, const unsigned char* bw_next,
                          const bool has_next) __attribute__((always_inline)) {
        asm volatile("" : "+v"(frag_w), "+v"(frag_x));
        if (has_next) wait_vm<8>(wreg[0][0], wreg[0][1]); else wait_vm<0>(wreg[0][0], wreg[0][1]);
#pragma unroll
        for (int ks = 1; ks < 4; ++ks) asm volatile("" : "+v"(wreg[ks][0]), "+v"(wreg[ks][1]));
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks < 3) read_x(bx, ks + 1, xf[nxt]);
            if (ks == 3 && has_next) {
                __builtin_amdgcn_s_waitcnt(0x0F70);
                __syncthreads();
                read_frags(bx_next, bw_next, 0, wf[0], xf[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_quarter(ks, cur);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto dense_loop = [&]() __attribute__((always_inline)) {
        if (nsteps <= 0) return;
        Staged<QMODE, BR> none{};
        int s = 0, issued = 0;
        if (steps1 > 0) {
            issue_x1(0, 0);
            if (steps1 > 1) { issue_x1(1, 1); issued = 1; }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) load_w_quarter(ks, wop);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            read_x(sX, 0, xf[0]);
            for (; s + 2 < steps1; s += 2) {
                dense_step(sX, sX + kTileBytes, true, s, 0);
                const bool more = s + 3 < steps1;
                dense_step(sX + kTileBytes, sX, more, s + 1, 1);
                issued = more ? s + 3 : s + 2;
            }
            if (s + 1 < steps1) {
                dense_step(sX, sX + kTileBytes, false, s, 0);
                ++s;
            }
            const int buf = s & 1;
            const bool has_next = s + 1 < nsteps;
            if (has_next) { issue_copies(s + 1, buf ^ 1); issued = s + 1; }
            dense_last(sX + buf * kTileBytes, sX + (buf ^ 1) * kTileBytes, sW + (buf ^ 1) * kTileBytes, has_next);
            ++s;
        } else {
            issue_copies(0, 0);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            read_frags(sX, sW, 0, wf[0], xf[0]);
        }
        // K-extension steps: both tiles through LDS
        for (; s < nsteps; ++s) {
            const int buf = s & 1;
            const bool has_next = s + 1 < nsteps;
            if (has_next && issued < s + 1) { issue_copies(s + 1, buf ^ 1); issued = s + 1; }
            run_step(sX + buf * kTileBytes, sW + buf * kTileBytes, sX + (buf ^ 1) * kTileBytes,
                     sW + (buf ^ 1) * kTileBytes, false, none, has_next, false, 0, 0, false, none);
        }
    };

    // ---- main loop ---------------------------------------------------------------------------------
    // Invariant at the top of step s: tile buffers s&1 hold step s and fragment set 0 holds its first
    // quarter; st[(s+1)&1] holds the codes of step s+1 (if that is a quantized step).
    Staged<QMODE, BR> st[2];
    if constexpr (QMODE == 0) {
        dense_loop();
    } else if (nsteps > 0) {
        issue_copies(0, 0);
        int issued = 0;                                    // copies are in flight or done for steps <= issued
        if (steps1 > 1) { issue_copies(1, 1); issued = 1; }
        constexpr bool kDq = QMODE != 0;                   // segment 1 is dequantized in the kernel
        if constexpr (kDq) {
            if (steps1 > 0) load_staged(st[0], 0);
            if (steps1 > 1) load_staged(st[1], 1);
            __syncthreads();                               // pair table visible
            if (steps1 > 0) dequant_store(st[0], sW);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        read_frags(sX, sW, 0, wf[0], xf[0]);
        if (kDq && steps1 > 1) {                           // first piece of the tile the first step dequantizes
            uint32_t li[kReads];
            table_offsets(st[1], 0, li);
            table_reads(li, lv0);
        }
        int s = 0;
        // Quantized steps whose successor is quantized too (the successor's tile is dequantized during
        // the step), unrolled by two so that the staging registers and the tile buffers have fixed
        // names.  Codes are fetched two steps ahead; past the end the last quantized step is fetched
        // again (in bounds, unused) so that the body has no conditions.  A step refills its own token
        // buffer with the copies of the step after next (when that is a quantized step) behind its
        // barrier, under its last 8 MFMAs.
        const int last_q = steps1 - 1;
        for (; s + 2 < steps1; s += 2) {
            if constexpr (kDq) load_staged(st[0], min(s + 2, last_q));
            run_step(sX, sW, sX + kTileBytes, sW + kTileBytes, kDq, st[1], true, true, s + 2, 0, kDq, st[0]);
            if constexpr (kDq) load_staged(st[1], min(s + 3, last_q));
            const bool more = s + 3 < steps1;
            // (past the last dequantizing step the looked-up piece is simply not used)
            run_step(sX + kTileBytes, sW + kTileBytes, sX, sW, kDq, st[0], true, more, s + 3, 1, kDq, st[1]);
            issued = more ? s + 3 : s + 2;
        }
        if (s + 1 < steps1) {
            run_step(sX, sW, sX + kTileBytes, sW + kTileBytes, kDq, st[1], true, false, 0, 0, false, st[0]);
            ++s;
        }
        // the last quantized step and the K-extension steps: nothing to dequantize; copies of the next
        // step are issued at the top of a step when no earlier step has done it
        for (; s < nsteps; ++s) {
            const int buf = s & 1;
            const bool has_next = s + 1 < nsteps;
            if (has_next && issued < s + 1) { issue_copies(s + 1, buf ^ 1); issued = s + 1; }
            run_step(sX + buf * kTileBytes, sW + buf * kTileBytes, sX + (buf ^ 1) * kTileBytes,
                     sW + (buf ^ 1) * kTileBytes, false, st[0], has_next, false, 0, 0, false, st[0]);
        }
    }

    __builtin_amdgcn_s_waitcnt(0x0F70);                    // nothing may still be writing this workgroup's LDS

    // ---- epilogue ---------------------------------------------------------------------------------------
    // A lane holds features n..n+3 of one token per accumulator quad, i.e. 8 bytes of an output row.
    // The wave first lays its 128 x 64 quadrant out in LDS (the tiles are dead by now) as bf16 rows of
    // 128 bytes (pitch 144), then reads it back 16 bytes per lane so that every global store
    // instruction writes eight complete 128-byte row segments.
    __syncthreads();                                       // every wave is done reading the tiles
    {
        constexpr int kPitch = 144;
        unsigned char* eb = smem + wave * (128 * kPitch);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 o;
                    o.x = pack_bf16(acc[a][b][q * 4 + 0] * out_scale, acc[a][b][q * 4 + 1] * out_scale);
                    o.y = pack_bf16(acc[a][b][q * 4 + 2] * out_scale, acc[a][b][q * 4 + 3] * out_scale);
                    *reinterpret_cast<uint2*>(eb + (b * 32 + r) * kPitch + (a * 32 + q * 8 + hi * 4) * 2) = o;
                }
        const int erow = lane >> 3, echunk = lane & 7;
        const int n = n0 + wn0 + echunk * 8;
#pragma unroll 8
        for (int i = 0; i < 16; ++i) {
            const int row = i * 8 + erow;
            const uint4 v = *reinterpret_cast<const uint4*>(eb + row * kPitch + echunk * 16);
            const int64_t m = m0 + wm0 + row;
            if (m < M && n < N) {
                typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
                const u32x4 vv = {v.x, v.y, v.z, v.w};
                __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(C + m * ldc + n));
            }
        }
    }
}

template <int QMODE, bool BETA, int BR>
int launch_cfg(const GemmDesc& d, hipStream_t st) {
    constexpr size_t smem = 4 * kTileBytes + kTableBytes;
    auto kern = k_qlinear<QMODE, BETA, BR>;
    // set once per instantiation; the initialisation of a function-local static is thread safe
    static const bool attr_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!attr_ok) return QBLORA_ERR_LAUNCH;
    int64_t tiles = ((d.M + BM - 1) / BM) * ((d.N + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kThreads), smem, st, d);
    return launch_status();
}

}  // namespace

// The quantized GEMMs of the layer (qmode 1 or 2, bf16 output, no auxiliary outputs).
int launch_qlinear(const GemmDesc& d, hipStream_t st) {
    if (d.M <= 0 || d.N <= 0) return QBLORA_OK;
    if (d.out_f32 || d.C2 || d.C_lo) return QBLORA_ERR_UNSUPPORTED;
    if (d.block_rows == 8 && d.qmode != 3) {
        // scales / offsets are read as 16-byte groups of 4 block columns; tile-ordered scales do not exist
        if (d.scales_tiled || !d.scales || d.d_out % 8 != 0 || (reinterpret_cast<uintptr_t>(d.scales) & 15) ||
            (reinterpret_cast<uintptr_t>(d.beta) & 15))
            return QBLORA_ERR_UNSUPPORTED;
        if (d.qmode == 1) return d.beta ? launch_cfg<1, true, 8>(d, st) : launch_cfg<1, false, 8>(d, st);
        if (d.qmode == 2) return d.beta ? launch_cfg<2, true, 8>(d, st) : launch_cfg<2, false, 8>(d, st);
        return QBLORA_ERR_UNSUPPORTED;
    }
    if (d.qmode == 3) {
        // dense first segment: whole 64-wide steps of 16-byte chunks
        // whole 64-wide steps, whole 32-row blocks, 32-bit byte offsets into the operand-ordered weight
        if (!d.W1 || d.K1 <= 0 || d.K1 % kBK != 0 || d.N % 32 != 0 || (reinterpret_cast<uintptr_t>(d.W1) & 15) ||
            (int64_t)d.N * d.K1 * 2 >= ((int64_t)1 << 32))
            return QBLORA_ERR_UNSUPPORTED;
        return launch_cfg<0, false, 1>(d, st);
    }
    if (d.qmode == 1) return d.beta ? launch_cfg<1, true, 1>(d, st) : launch_cfg<1, false, 1>(d, st);
    if (d.qmode == 2) return d.beta ? launch_cfg<2, true, 1>(d, st) : launch_cfg<2, false, 1>(d, st);
    return QBLORA_ERR_UNSUPPORTED;
}

}  // namespace qblora
