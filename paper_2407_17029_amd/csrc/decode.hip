// Small-batch forward of a 4-bit block-quantized layer (merged-model inference: the INT4 weights
// (codes, alpha, beta) that the QA-BLoRA merge of Sec. 3.3 produces, or any other quantized base):
//
//   Y[t, n] = sum_b ( alpha[n,b] * sum_{k in b} X[t,k] * c^[n,k]  +  beta[n,b] * sum_{k in b} X[t,k] ),
//
// c^ = bf16(c[code]) (exact for the codebook 0..15 of INT4 models), for T <= 16 tokens.  Every weight is
// used once per token, so the job is to stream the codes and block parameters from HBM (0.5 + 4/64
// (+ 4/64) bytes per weight) with as little vector arithmetic per weight as possible: scale and offset
// are constant inside a 64-block, so they are applied to the block's partial sums, not to the weights,
// and a code byte becomes two bf16 operand values with one LDS read.
//
// A workgroup of 4 waves (8 on layers with few rows) owns 16 output rows (32 on tall layers); the waves split
// the input dimension (wave w takes the groups of 4 or 2 consecutive blocks j = w, w+4, ...) and add their partial
// tiles through LDS at the end.
// Inside a wave, lane l works on row (l & 15): for block b it loads 8 of the block's 32 code bytes
// (quarter l >> 4), turns them into the B operand of two v_mfma_f32_16x16x32_bf16 whose A operand is the
// matching 8 activations of token (l & 15) (zero for tokens >= T): the two MFMAs give the lane the
// block's sums for its row and tokens 4*(l>>4) .. +3.  A third and fourth MFMA against a B operand of
// ones give sum_k X[t,k] of the block when there are offsets.  Then one FMA per token applies alpha
// (and one beta).  Any assignment of k to lanes is valid as long as both operands agree.
//
// With 8 x 8 quantization blocks (BR = 8) the scale changes every 8 inputs, inside the contraction of one
// MFMA, so it cannot act on partial sums: there the lane builds the bf16 compute weight
// bf16(fma(c, alpha, beta)) of its 16 inputs (two block columns; the byte table then holds fp32 pairs) and
// the MFMAs accumulate directly -- the arithmetic of the training forward.  The table entries of an operand are read
// one operand ahead of their use; for an INT4 model (codebook exactly 0..15) a code is its own value, so there is no
// table at all: two masks per code dword and one byte-to-float conversion per code.  That form is bound by its vector
// arithmetic (some 4 instructions per weight: conversion, scale-and-shift, half a packing, loop overhead), not by HBM.
//
// INT4 models (codebook exactly 0..15, offsets present, packed arrays: DIRECT) need no table: the bf16 with
// bits 0x4300 | c is 128 + c, so two shift/and-or instructions turn a code dword into an operand dword
// (the pack regroups the nibbles of every dword for that), and the 128 comes off through the block's
// sum of activations, which the offset term computes anyway:
// alpha * sum x (128 + c) + (beta - 128 alpha) * sum x.
#include "common.h"
#include <type_traits>

namespace qblora {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;

struct DecodeDesc {
    const uint8_t* codes; const float* scales; const float* beta; Codebook cb;
    int tiled;                 // the three arrays are in tile order (256-row tiles, rows of a block adjacent);
                               // with 8 x 8 blocks only the codes are, scales and offsets stay [d_out/8, d_in/8]
    int block_rows;            // 1 or 8
    int d_out, d_in;
    const qblora_bf16* X; int T;
    qblora_bf16* Y;
};

constexpr int kReplicas = 16;               // copies of the byte -> (bf16 c[lo], bf16 c[hi]) table

template <int G, int R>
struct DecodeRegs {                         // one group = G consecutive blocks of the lane's R rows (16 rows apart)
    uint2 c[G][R];                          // the lane's quarter of each block's codes: 16 codes
    float a[G][R], b[G][R];                 // scale and offset of each block
    float2 a2[G][R], b2[G][R];              // BR = 8: scales and offsets of the lane's two block columns
    int xb[G];                              // XALL: the (redirected) block whose activations go with c[q]
    uint4 x[G][2];                          // activations of the lane's token, 8 per MFMA (fetched in operand order)
};

// XLDS: the activations of a group as fetched.  (A native vector type: with HIP's uint4, a struct that is copied as
// memory, the compiler kept these registers in scratch memory -- a store, a wait for it and a load per group.)
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
template <int N>
struct StagedRegs { u32x4_t v[N]; };

// XLDS: the activations go through LDS.  In operand order a load instruction touches 16 token rows, 64 bytes of
// each; with more than a few tokens these loads, not the codes, fill the address path (T = 16: 55 us against 29 at
// T = 1).  Fetched as whole row segments (512 bytes with four-block sets, 256 with two-block sets) and re-read from
// the wave's own LDS region in operand order they cost half the cache-line accesses.  With two-block sets the region
// holds two buffers and the staging runs one group ahead of the MFMAs (see the loop); as first written -- the group's
// activations held in scratch memory by the compiler and written to LDS right before they were read -- this form
// only paid above 8 tokens (T = 16: 44 us); now it is the form of the table-free kernels from two tokens on.
// XMODE 2 (few tokens, rows short enough: at most kXAllBytes of activations): the workgroup copies all of X into
// LDS once, and the loop has no activation loads at all.  With one token the operand-order loads above move 16 x
// the bytes of the codes through the vector memory path (every lane fetches its own copy of the 16 activations
// it shares with 15 others), and that path, not HBM, set the time.
constexpr int kXAllBytes = 40 * 1024;
constexpr int kXAllBytesFew = 59 * 1024;     // with the 4 KB of static LDS inside the 64 KB a launch may ask for without more ado
constexpr int kBufferWord3 = 0x00020000;    // buffer descriptor, last word: untyped 32-bit data, no swizzle, no stride
template <bool BETA, int BR, bool DIRECT, int XMODE, int G = 4, int R = 1, int NE = 4, int NW = 4>
__device__ __forceinline__ void w4_decode(const DecodeDesc& d);

template <bool BETA, int BR, bool DIRECT = false, int XMODE = 0, int G = 4, int R = 1, int NE = 4>
__global__ __launch_bounds__(256) void k_w4_decode(DecodeDesc d) { w4_decode<BETA, BR, DIRECT, XMODE, G, R, NE>(d); }

// G: blocks per register set.  Four keep the most bytes in flight per wave and use 108 registers (four waves per
// SIMD, 1024 workgroups resident); two use 76, six waves per SIMD, so that the 1376 workgroups of a 22016-row layer
// are resident at once (25.2 against 26.0 us; limiting the four-block form to 84 registers instead spills 24 of
// them and nearly doubles the time).  Layers that fit the 1024 slots are faster with four (4096 rows: 5.4 against 6.0).
// NE: tokens per lane that are kept (a lane holds tokens 4 * (lane / 16) .. + 3 of its row): with one or two tokens
// the scale-and-offset FMAs of the others are left out (8 -> 2 or 4 per block and row group).
// NW: waves per workgroup.  Layers with at most two workgroups of four waves per CU (8192 rows and fewer) have too few
// waves to keep enough loads in flight; eight waves split the input dimension finer instead.
template <bool BETA, bool DIRECT, int G, int BR = 1, int R = 1, int NE = 4, int NW = 4>
__global__ __launch_bounds__(NW * 64) void k_w4_decode_xall(DecodeDesc d) {
    w4_decode<BETA, BR, DIRECT, 2, G, R, NE, NW>(d);
}

// R: row groups of 16 per workgroup.  With two, the activation operands (which every workgroup fetches for its own
// rows: at 16 tokens four times the bytes of the codes) serve 32 rows, and so do the block sums of the activations.
template <bool BETA, int BR, bool DIRECT, int XMODE, int G, int R, int NE, int NW>
__device__ __forceinline__ void w4_decode(const DecodeDesc& d) {
    static_assert(NW == 4 || DIRECT, "the table is filled by 256 threads");
    constexpr bool XLDS = XMODE == 1, XALL = XMODE == 2;
    static_assert(!DIRECT || BR == 8 || BETA, "the table-free form of 64-blocks needs offsets");
    extern __shared__ __align__(16) unsigned char x_all[];       // XALL: [T][d_in * 2 + 16] bytes
    // entry e of replica q at e*kReplicas + q: bf16 pairs (4 bytes), or fp32 pairs (8 bytes) for BR = 8
    __shared__ __align__(8) uint32_t pair[DIRECT ? 2 : 256 * kReplicas * (BR == 8 ? 2 : 1)];
    __shared__ float red[NW][4][64];
    // Activations of one group of G blocks (16 tokens x 128 G bytes), one region per wave: fetched as whole
    // row segments (two or four token rows per load instruction) and read back in operand order.  A row is
    // 128 G + 16 bytes so that the 16 tokens of an operand read start 16 bytes apart modulo 256.
    constexpr int kXPitch = G * 128 + 16;
    constexpr int kLPR = 8 * G, kTPL = 64 / kLPR, kNX = 16 / kTPL;    // lanes per staged token row, token rows per load, loads
    constexpr int kXBufs = G <= 2 ? 2 : 1;                     // LDS buffers per wave (two: 35 KB per workgroup at G = 2)
    __shared__ __align__(16) unsigned char xs_all[XLDS ? NW : 1][XLDS ? kXBufs * 16 * kXPitch : 16];
    const int t = threadIdx.x, lane = t & 63;
    // the wave id as a scalar: block indices, the redirects of blocks past the end and the block part of every address
    // are then scalar arithmetic, and the loads take a scalar base with a 32-bit lane offset
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int nl = lane & 15, kg = lane >> 4;
    // Row groups 2i and 2i+1 share the 128-byte lines of the tile-ordered scales and offsets (16 rows = 64
    // bytes per block): they are given workgroup ids x and x + 8 of a run of 16 ids, which are dispatched to
    // the same XCD, so that one L2 fetches each line.  The grid is a multiple of 16; ids past the end leave.
    // (With two row groups per workgroup the pair is in one workgroup anyway.)
    const int rg = R == 1 ? (int)((blockIdx.x & ~15) | ((blockIdx.x & 7) << 1) | ((blockIdx.x >> 3) & 1)) : (int)blockIdx.x;
    if (rg * 16 * R >= d.d_out) return;
    const int n0 = rg * 16 * R;
    int n[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) n[rr] = min(n0 + 16 * rr + nl, d.d_out - 1);    // rows past the end are computed, not stored
    const int bpr = d.d_in / kBlock;
    const int groups = (bpr + G - 1) / G;
    if constexpr (DIRECT) {
        // no table
    } else if constexpr (BR == 8) {
        const float2 e = make_float2(d.cb.c[t & 15], d.cb.c[t >> 4]);
#pragma unroll
        for (int q = 0; q < kReplicas; ++q) reinterpret_cast<float2*>(pair)[t * kReplicas + q] = e;
    } else {
        const uint32_t e = pack_bf16(d.cb.c[t & 15], d.cb.c[t >> 4]);
#pragma unroll
        for (int q = 0; q < kReplicas; ++q) pair[t * kReplicas + q] = e;
    }
    __syncthreads();
    const uint32_t* my_pair = pair + (lane & (kReplicas - 1));
    const float2* my_pairf = reinterpret_cast<const float2*>(pair) + (lane & (kReplicas - 1));

    // Row-major arrays: a wave's load of one block touches 16 rows, i.e. 16 cache lines.  In tile order
    // (the layout of the forward kernel's code copy) the 16 rows of a block are adjacent: 4 lines of codes
    // and one of scales per load, which is what keeps the address path from being the bottleneck.
    const int bstep = d.tiled ? 256 : 1;                                                            // next block
    // the lane's part of every address, in bytes (the launcher has checked that the arrays are below 4 GB)
    uint32_t coff[R], soff[R];
    uint32_t off8[R];                       // BR = 8: block row n/8, block columns 8*b + 2*kg, +1 of 64-input step b
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const uint32_t run = d.tiled ? ((uint32_t)(n[rr] >> 8) * bpr * 256 + (n[rr] & 255)) : (uint32_t)n[rr] * bpr;   // block 0 of the row
        coff[rr] = run * 32 + 8 * kg;
        soff[rr] = run * 4;
        off8[rr] = ((uint32_t)(n[rr] >> 3) * (d.d_in >> 3) + 2 * kg) * 4;
    }
    const int cstep = bstep * 32;
    // Codes, scales and offsets come through buffer loads: scalar base (the descriptor), scalar block offset and the
    // lane's constant 32-bit offset, so that no load needs vector address arithmetic (as global loads every one cost
    // a 64-bit vector add, a quarter of the loop's vector instructions).  num_records = the array's size: an offset
    // past it would read zero instead of faulting.
    const uint32_t rows_held = d.tiled ? (uint32_t)((d.d_out + 255) & ~255) : (uint32_t)d.d_out;
    const uint32_t param_bytes = BR == 8 ? (uint32_t)((d.d_out + 7) >> 3) * (d.d_in >> 3) * 4 : rows_held * bpr * 4;
    const auto rsrc_c = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(d.codes), 0, rows_held * bpr * 32, kBufferWord3);
    const auto rsrc_s = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(d.scales), 0, param_bytes, kBufferWord3);
    const auto rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(BETA ? d.beta : d.scales), 0, param_bytes, kBufferWord3);
    unsigned char* xs = xs_all[XLDS ? wave : 0];
    const int xtok = lane / kLPR, xchunk = lane % kLPR;
    const qblora_bf16* xrow = d.X + (int64_t)min(nl, d.T - 1) * d.d_in + 16 * kg;
    const int x_pitch = d.d_in * 2 + 16;                      // token rows start 16 bytes apart modulo the banks
    const unsigned char* x_mine = x_all + min(nl, d.T - 1) * x_pitch + 32 * kg;      // XALL: inputs 16 kg .. of block 0

    // Every load is unconditional: a block past the end of the row is redirected to the last block and
    // given scale = offset = 0; lanes whose token does not exist read the last token's row and produce
    // output rows that are never stored.
    // (a group that lies wholly inside the row -- every group of a layer whose input size is a multiple of 64 G --
    // takes a copy of the code without the redirects and selects: FULL)
    auto load_as = [&](DecodeRegs<G, R>& r, int j, auto full) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full)::value;
#pragma unroll
        for (int q = 0; q < G; ++q) {
            const int b = G * j + q;
            const bool in = FULL || b < bpr;
            const int bc = in ? b : bpr - 1;
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                r.c[q][rr] = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rsrc_c, coff[rr], bc * cstep, 0));
                if constexpr (BR == 8) {
                    const float2 a = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(rsrc_s, off8[rr], 32 * bc, 0));
                    r.a2[q][rr] = in ? a : make_float2(0.0f, 0.0f);
                    r.b2[q][rr] = make_float2(0.0f, 0.0f);
                    if constexpr (BETA) {
                        const float2 bt = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(rsrc_b, off8[rr], 32 * bc, 0));
                        if (in) r.b2[q][rr] = bt;
                    }
                } else {
                    const float a = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_s, soff[rr], bc * bstep * 4, 0));
                    r.a[q][rr] = in ? a : 0.0f;
                    if constexpr (BETA) {
                        const float bt = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_b, soff[rr], bc * bstep * 4, 0));
                        r.b[q][rr] = in ? bt : 0.0f;
                        if constexpr (DIRECT) r.b[q][rr] = __builtin_fmaf(-128.0f, r.a[q][rr], r.b[q][rr]);
                    } else {
                        r.b[q][rr] = 0.0f;
                    }
                }
            }
            if constexpr (XALL) {
                r.xb[q] = bc;
            } else if constexpr (!XLDS) {
#pragma unroll
                for (int m = 0; m < 2; ++m) r.x[q][m] = *reinterpret_cast<const uint4*>(xrow + bc * kBlock + 8 * m);
            }
        }
    };
    using XRegs = StagedRegs<kNX>;
    // XLDS: the activations of group j as fetched, 64 / (8 G) token rows per load, 16-byte chunk lane % (8 G) of the
    // group.  Token rows that do not exist are not fetched (their LDS rows keep old contents and feed output rows
    // that are never stored); chunks of blocks past the end of the row are redirected to the last block, whose
    // scale and offset are zero there.
    auto load_x = [&](XRegs& x, int j) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < kNX; ++p) {
            if (kTPL * p < d.T) {
                const int tk = min(kTPL * p + xtok, d.T - 1);
                const int bc = min(G * j + (xchunk >> 3), bpr - 1);
                x.v[p] = *reinterpret_cast<const u32x4_t*>(d.X + (int64_t)tk * d.d_in + bc * kBlock + 8 * (xchunk & 7));
            }
        }
    };
    // ... and into the wave's LDS buffer `buf`
    auto stage = [&](const XRegs& x, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < kNX; ++p)
            if (kTPL * p < d.T) *reinterpret_cast<u32x4_t*>(xs + buf * (16 * kXPitch) + (kTPL * p + xtok) * kXPitch + xchunk * 16) = x.v[p];
    };
    auto load = [&](DecodeRegs<G, R>& r, int j) __attribute__((always_inline)) {
        if constexpr (XLDS) {              // (two copies cost the staged form ten registers and with them a wave per SIMD)
            load_as(r, j, std::false_type{});
        } else {
            if (G * j + G <= bpr) load_as(r, j, std::true_type{});
            else load_as(r, j, std::false_type{});
        }
    };

    const f32x4_t zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4_t acc[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) acc[rr] = zero;
    const uint4 ones4 = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones4);
    // The two constants of the table-free operand sit in registers the compiler cannot see through: with literals it
    // emits an AND and an OR per operand dword (the three-operand AND-OR cannot encode two literals), with registers
    // the one instruction.  (The instruction is left to the compiler rather than written as inline assembly, so that
    // its hazard handling next to the MFMAs sees it.)
    const uint32_t nib_mask = opaque_bits(0x000F000Fu), bf16_128 = opaque_bits(0x43004300u);
    auto operand = [&](uint32_t w) __attribute__((always_inline)) {
        if constexpr (DIRECT) {
            const uint4 v = make_uint4((w & nib_mask) | bf16_128, ((w >> 4) & nib_mask) | bf16_128,
                                       ((w >> 8) & nib_mask) | bf16_128, ((w >> 12) & nib_mask) | bf16_128);
            return __builtin_bit_cast(bf16x8, v);
        }
        const uint4 v = make_uint4(my_pair[(w & 0xffu) * kReplicas], my_pair[((w >> 8) & 0xffu) * kReplicas],
                                   my_pair[((w >> 16) & 0xffu) * kReplicas], my_pair[(w >> 24) * kReplicas]);
        return __builtin_bit_cast(bf16x8, v);
    };
    // BR = 8: the four table entries of an operand (one code dword) are read one operand ahead of their use, so that
    // a wave has LDS reads in flight under the scaling arithmetic of the previous operand instead of waiting for
    // each operand's reads in turn (the compiler's order: eight exposed LDS round trips per group of blocks)
    // (DIRECT with BR = 8: the codebook is exactly 0 .. 15, so a code is its own value and the byte-to-float
    // conversions replace the table; its reads, two-way bank conflicts included, otherwise cost as much LDS time as the
    // codes cost HBM time)
    auto fetch8 = [&](uint32_t w, float2 (&cv)[4]) __attribute__((always_inline)) {
        if constexpr (DIRECT) {
            // one byte-to-float conversion per code on the two masked dwords (whose known zero nibbles are hidden from
            // the compiler: otherwise it makes a bit-field extract and a conversion per code)
            const uint32_t lo = opaque_bits(w & 0x0F0F0F0Fu), hi = opaque_bits((w >> 4) & 0x0F0F0F0Fu);
            cv[0] = make_float2(byte_to_float(lo, 0), byte_to_float(hi, 0));
            cv[1] = make_float2(byte_to_float(lo, 1), byte_to_float(hi, 1));
            cv[2] = make_float2(byte_to_float(lo, 2), byte_to_float(hi, 2));
            cv[3] = make_float2(byte_to_float(lo, 3), byte_to_float(hi, 3));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) cv[i] = my_pairf[((w >> (8 * i)) & 0xffu) * kReplicas];
        }
    };
    auto build8 = [&](const float2 (&cv)[4], float a, float b) __attribute__((always_inline)) {
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            o[i] = BETA ? pack_bf16(__fmaf_rn(cv[i].x, a, b), __fmaf_rn(cv[i].y, a, b)) : pack_bf16(__fmul_rn(cv[i].x, a), __fmul_rn(cv[i].y, a));
        return __builtin_bit_cast(bf16x8, make_uint4(o[0], o[1], o[2], o[3]));
    };
    auto compute8 = [&](const DecodeRegs<G, R>& r, const unsigned char* xsb) __attribute__((always_inline)) {
        float2 cv[2][4];
        auto dword = [&](int v) __attribute__((always_inline)) {      // operand v = (block, code dword, row group)
            const int u = v / R, rr = v % R;
            return (u & 1) ? r.c[u >> 1][rr].y : r.c[u >> 1][rr].x;
        };
        fetch8(dword(0), cv[0]);
        bf16x8 x;
#pragma unroll
        for (int v = 0; v < 2 * G * R; ++v) {
            const int u = v / R, rr = v % R, q = u >> 1;
            if (v + 1 < 2 * G * R) fetch8(dword(v + 1 < 2 * G * R ? v + 1 : v), cv[(v + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            if (rr == 0) {
                if constexpr (XLDS) x = *reinterpret_cast<const bf16x8*>(xsb + nl * kXPitch + 128 * q + 32 * kg + 16 * (u & 1));
                else if constexpr (XALL) x = *reinterpret_cast<const bf16x8*>(x_mine + r.xb[q] * (kBlock * 2) + 16 * (u & 1));
                else x = __builtin_bit_cast(bf16x8, r.x[q][u & 1]);
            }
            const bf16x8 wv = build8(cv[v & 1], (u & 1) ? r.a2[q][rr].y : r.a2[q][rr].x, (u & 1) ? r.b2[q][rr].y : r.b2[q][rr].x);
            acc[rr] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wv, acc[rr], 0, 0, 0);
        }
    };
    // (buf: the wave's LDS buffer that holds the group's activations, XLDS only)
    auto compute = [&](const DecodeRegs<G, R>& r, int buf = 0) __attribute__((always_inline)) {
        const unsigned char* xsb = xs + buf * (16 * kXPitch);
        if constexpr (BR == 8) { compute8(r, xsb); return; }
#pragma unroll
        for (int q = 0; q < G; ++q) {
            bf16x8 x0, x1;
            if constexpr (XLDS) {
                const unsigned char* xq = xsb + nl * kXPitch + 128 * q + 32 * kg;    // k = 64q + 16kg .. +15 of token nl
                x0 = *reinterpret_cast<const bf16x8*>(xq); x1 = *reinterpret_cast<const bf16x8*>(xq + 16);
            } else if constexpr (XALL) {
                const unsigned char* xq = x_mine + r.xb[q] * (kBlock * 2);
                x0 = *reinterpret_cast<const bf16x8*>(xq); x1 = *reinterpret_cast<const bf16x8*>(xq + 16);
            } else {
                x0 = __builtin_bit_cast(bf16x8, r.x[q][0]); x1 = __builtin_bit_cast(bf16x8, r.x[q][1]);
            }
            f32x4_t sx = zero;
            if constexpr (BETA) {
                sx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x0, ones, zero, 0, 0, 0);
                sx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x1, ones, sx, 0, 0, 0);
            }
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                f32x4_t blk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x0, operand(r.c[q][rr].x), zero, 0, 0, 0);
                blk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x1, operand(r.c[q][rr].y), blk, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < NE; ++e) acc[rr][e] = __builtin_fmaf(r.a[q][rr], blk[e], acc[rr][e]);
                if constexpr (BETA) {
#pragma unroll
                    for (int e = 0; e < NE; ++e) acc[rr][e] = __builtin_fmaf(r.b[q][rr], sx[e], acc[rr][e]);
                }
            }
        }
    };

    // two register sets: the loads of the wave's next group are in flight while this one is contracted
    DecodeRegs<G, R> r0, r1;
    int j = wave;
    if (j < groups) load(r0, j);
    if constexpr (XALL) {                                     // behind the first loads of codes: both are in flight together
        const int chunks = d.d_in / 8;                        // 16-byte pieces per token row
        for (int i0 = t; i0 < d.T * chunks; i0 += 4 * NW * 64) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = min(i0 + u * NW * 64, d.T * chunks - 1);
                const int tk = i / chunks, c = i - tk * chunks;
                v[u] = *reinterpret_cast<const uint4*>(d.X + (int64_t)tk * d.d_in + c * 8);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * NW * 64;
                if (i >= d.T * chunks) break;
                const int tk = i / chunks, c = i - tk * chunks;
                *reinterpret_cast<uint4*>(x_all + tk * x_pitch + c * 16) = v[u];
            }
        }
        __syncthreads();
    }
    if constexpr (XLDS && kXBufs == 2) {
        // Two LDS buffers per wave: while group g is contracted out of one, the activations of group g + 1 (fetched
        // during the contraction of group g - 1) are written into the other and those of group g + 2 set out -- the
        // write -> read -> MFMA round trip of a group is then not waited for in front of its MFMAs.
        XRegs xq;
        if (j < groups) { load_x(xq, j); stage(xq, 0); }       // (the codes of group j are already on their way)
        if (j + NW < groups) load_x(xq, j + NW);
        for (; j < groups; j += 2 * NW) {
            if (j + NW < groups) {
                load(r1, j + NW);
                stage(xq, 1);
                if (j + 2 * NW < groups) load_x(xq, j + 2 * NW);
            }
            compute(r0, 0);
            if (j + NW < groups) {
                if (j + 2 * NW < groups) {
                    load(r0, j + 2 * NW);
                    stage(xq, 0);
                    if (j + 3 * NW < groups) load_x(xq, j + 3 * NW);
                }
                compute(r1, 1);
            }
        }
    } else if constexpr (XLDS) {                               // one buffer: written just before it is read
        XRegs xq;
        if (j < groups) load_x(xq, j);
        for (; j < groups; j += 2 * NW) {
            if (j + NW < groups) load(r1, j + NW);
            stage(xq, 0);
            if (j + NW < groups) load_x(xq, j + NW);
            compute(r0, 0);
            if (j + NW < groups) {
                if (j + 2 * NW < groups) load(r0, j + 2 * NW);
                stage(xq, 0);
                if (j + 2 * NW < groups) load_x(xq, j + 2 * NW);
                compute(r1, 0);
            }
        }
    } else {
        for (; j < groups; j += 2 * NW) {
            if (j + NW < groups) load(r1, j + NW);
            compute(r0);
            if (j + NW < groups) {
                if (j + 2 * NW < groups) load(r0, j + 2 * NW);
                compute(r1);
            }
        }
    }

    // The lane holds row nl, tokens 4*kg .. 4*kg+3.  Partial tiles of the waves -> LDS; wave 0 adds
    // them in wave order, lane l taking token l >> 2 and rows 4*(l & 3) .. +3 so that stores run along n.
    const int tok = lane >> 2, nq = 4 * (lane & 3);
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        if (rr) __syncthreads();                               // wave 0 has read the previous row group's partial tiles
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][e][lane] = acc[rr][e];
        __syncthreads();
        if (wave == 0 && tok < d.T) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int src = (nq + i) + 16 * (tok >> 2), e = tok & 3;
                float sum = red[0][e][src];
#pragma unroll
                for (int w = 1; w < NW; ++w) sum += red[w][e][src];
                v[i] = sum;
            }
            const int nb = n0 + 16 * rr + nq;
            qblora_bf16* yp = d.Y + (int64_t)tok * d.d_out + nb;
            if (nb + 3 < d.d_out && (d.d_out & 3) == 0) {
                *reinterpret_cast<uint2*>(yp) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (nb + i < d.d_out) reinterpret_cast<uint16_t*>(yp)[i] = (uint16_t)(pack_bf16(v[i], 0.0f) & 0xffffu);
            }
        }
    }
}

// the form with all of X in LDS (at most kXAllBytes of it: inside the default limit of dynamic LDS; a limit of 66 KB
// measured slower wherever it applied -- 22016 x 8192 at four tokens 48 against 33 us, two workgroups per CU)
template <bool BETA, bool DIRECT, int G, int BR = 1, int R = 1, int NE = 4, int NW = 4>
int launch_xall(const DecodeDesc& d, dim3 grid, size_t x_all_bytes, hipStream_t st) {
    hipLaunchKernelGGL((k_w4_decode_xall<BETA, DIRECT, G, BR, R, NE, NW>), grid, dim3(NW * 64), x_all_bytes, st, d);
    return launch_status();
}

}  // namespace

int launch_w4_decode(const uint8_t* codes, const float* scales, const float* beta, const Codebook& cb, int tiled,
                     int d_out, int d_in, const qblora_bf16* X, int T, qblora_bf16* Y, hipStream_t st, int block_rows,
                     int regrouped) {
    DecodeDesc d{codes, scales, beta, cb, tiled, block_rows, d_out, d_in, X, T, Y};
    // the kernels address codes, scales and offsets with 32-bit byte offsets
    if (((int64_t)d_out + 255) / 256 * 256 * (int64_t)d_in / 2 >= (int64_t)1 << 31) return QBLORA_ERR_UNSUPPORTED;
    if (regrouped && (!beta || !tiled || block_rows == 8)) return QBLORA_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(((d_out + 15) / 16 + 15) / 16 * 16));       // 16 rows per workgroup
    const dim3 grid2((unsigned)(((d_out + 31) / 32 + 15) / 16 * 16));      // 32 rows (two row groups)
    const size_t per_cu = (grid.x + 255) / 256, per_cu2 = (grid2.x + 255) / 256;
    const bool tall = grid2.x > 512;            // more than 16384 rows: the forms with two row groups pay
    auto launch = [&](auto kernel, dim3 g) -> int {
        hipLaunchKernelGGL(kernel, g, dim3(256), 0, st, d);
        return launch_status();
    };
    // All of X in LDS: when it is small enough, and when the workgroups of the launch still fit the CUs together with
    // their copies (160 KB of LDS per CU; 22016 x 8192 at two tokens: 31.3 us with six 36 KB workgroups wanted per CU,
    // 29.9 without the copy).  With at most two workgroups per CU a larger copy costs no residency (8192 x 22016 at
    // one token, 44 KB).
    const size_t x_all_bytes = (size_t)T * ((size_t)d_in * 2 + 16);
    auto x_all_fits = [&](size_t workgroups_per_cu, size_t limit) {
        return d_in % 8 == 0 && x_all_bytes <= limit && workgroups_per_cu * (x_all_bytes + 5 * 1024) <= 150 * 1024;
    };
    bool int4 = true;                           // codes are their own values: no table
    for (int j = 0; j < 16; ++j) int4 = int4 && cb.c[j] == (float)j;

    // ---- packed INT4 model in 64-blocks (table-free, codes regrouped by the pack) --------------------------------------
    // Measured on 22016 x 8192 / 8192 x 22016 / 8192 x 8192 / 11008 x 4096, warm us (cold in brackets where it decides):
    //   one token: the LDS-copy forms win (20.5 / 20.7 / 9.9 / 7.0 against 21.1 / 24.4 / 11.4 / 7.6 staged);
    //   two and more: the staged forms (two tokens 20.9 / 24.2 / 11.2 / 7.6 against 22.0 / 25.4 / 10.9 / 7.5 -- level
    //   warm, 1 us ahead cold; four tokens 20.8 / 25.8 / 11.8 / 7.8 against 25.3 / 28.5 / 12.9 / 8.7), except where the
    //   eight-wave copy form applies (at most two workgroups per CU: 8192 x 8192 at two / three tokens 10.9 (12.9) /
    //   11.9 (13.8) against 11.2 (13.9) / 11.8 (14.7)) and on layers with one workgroup per CU (4096 x 4096: 4.4 to
    //   5.5 us against 5.3 to 5.8).
    if (regrouped) {
        if (per_cu <= 2 && x_all_fits(per_cu, kXAllBytesFew)) {
            // eight waves per workgroup (8192 x 8192 at one token 11.1 -> 10.0 us, from HBM 13.7 -> 11.9; 8192 x 22016:
            // 24.2 -> 20.8 and 30.2 -> 24.7 us; with two-block sets 10.4 / 12.7 and 21.7 / 27.1)
            if (T == 1) return launch_xall<true, true, 4, 1, 1, 1, 8>(d, grid, x_all_bytes, st);
            if (T == 2) return launch_xall<true, true, 4, 1, 1, 2, 8>(d, grid, x_all_bytes, st);
            return launch_xall<true, true, 4, 1, 1, 4, 8>(d, grid, x_all_bytes, st);
        }
        if (T == 1) {
            // tall layers: two row groups per workgroup, half as many copies of X (22016 x 8192: 25.8 -> 23.6 us before
            // the changes to the loads, 20.5 now); otherwise two-block sets when there are more workgroups than the
            // four-block form's 1024 slots
            if (tall && x_all_fits(per_cu2, kXAllBytes)) return launch_xall<true, true, 2, 1, 2, 1>(d, grid2, x_all_bytes, st);
            if (x_all_fits(per_cu, kXAllBytes))
                return grid.x > 1024 ? launch_xall<true, true, 2, 1, 1, 1>(d, grid, x_all_bytes, st)
                                     : launch_xall<true, true, 4, 1, 1, 1>(d, grid, x_all_bytes, st);
            return grid.x > 768 ? launch(k_w4_decode<true, 1, true, 0, 2, 1, 1>, grid) : launch(k_w4_decode<true, 1, true, 0, 4, 1, 1>, grid);
        }
        if (per_cu <= 1 && T <= 8) return launch(k_w4_decode<true, 1, true, 0>, grid);
        // staged: two row groups and two-block sets on tall layers (22016 x 8192 at 8 / 16 tokens 22.8 / 24.7 us; with
        // one row group and four-block sets 52 / 54 us before the staging was pipelined), else one and four
        if (tall) return launch(k_w4_decode<true, 1, true, 1, 2, 2>, grid2);
        return launch(k_w4_decode<true, 1, true, 1>, grid);
    }

    // ---- 8 x 8 blocks ----------------------------------------------------------------------------------------------
    if (block_rows == 8) {
        if (!int4) {                            // table of fp32 pairs: with the activation rows too it leaves two workgroups
                                                // per CU, measured slower (68 vs 64 us at T = 16): the plain form only
            return beta ? launch(k_w4_decode<true, 8, false, 0>, grid) : launch(k_w4_decode<false, 8, false, 0>, grid);
        }
        // INT4 model, one token: no table, all of X in LDS (22016 x 8192: 35.8 -> 28.2 us, with two row groups level;
        // with at most two workgroups per CU the copy costs more than it saves: 4096 rows 6.3 against 5.9 us)
        if (T == 1 && tall && x_all_fits(per_cu2, kXAllBytes))
            return beta ? launch_xall<true, true, 2, 8, 2>(d, grid2, x_all_bytes, st) : launch_xall<false, true, 2, 8, 2>(d, grid2, x_all_bytes, st);
        if (T == 1 && grid.x > 512 && x_all_fits(per_cu, kXAllBytes)) {
            if (grid.x > 1024) return beta ? launch_xall<true, true, 2, 8>(d, grid, x_all_bytes, st) : launch_xall<false, true, 2, 8>(d, grid, x_all_bytes, st);
            return beta ? launch_xall<true, true, 4, 8>(d, grid, x_all_bytes, st) : launch_xall<false, true, 4, 8>(d, grid, x_all_bytes, st);
        }
        // otherwise staged (22016 x 8192 at 2 / 4 / 8 / 16 tokens 26.4 / 26.5 / 27.9 / 30.8 us; 8192 x 8192 at one token
        // 13.8 against 14.7 us plain), unless the layer has at most one workgroup per CU (4096 rows)
        if (tall) return beta ? launch(k_w4_decode<true, 8, true, 1, 2, 2>, grid2) : launch(k_w4_decode<false, 8, true, 1, 2, 2>, grid2);
        if (grid.x > 256) return beta ? launch(k_w4_decode<true, 8, true, 1>, grid) : launch(k_w4_decode<false, 8, true, 1>, grid);
        return beta ? launch(k_w4_decode<true, 8, true, 0>, grid) : launch(k_w4_decode<false, 8, true, 0>, grid);
    }

    // ---- 64-blocks with a code table (any codebook; row-major or tile-ordered arrays) ------------------------------------
    if (x_all_fits(per_cu, kXAllBytes)) {
        const bool small_sets = grid.x > 1024;  // more workgroups than fit at four waves per SIMD
        if (beta) return small_sets ? launch_xall<true, false, 2>(d, grid, x_all_bytes, st) : launch_xall<true, false, 4>(d, grid, x_all_bytes, st);
        return small_sets ? launch_xall<false, false, 2>(d, grid, x_all_bytes, st) : launch_xall<false, false, 4>(d, grid, x_all_bytes, st);
    }
    // above 8 tokens the activations go through LDS (with the table in LDS as well, two workgroups per CU: the staged
    // form starts to pay later than in the table-free kernels -- 22016 x 8192 at 6 tokens 32.2 plain, 35.8 staged)
    if (T > 8) return beta ? launch(k_w4_decode<true, 1, false, 1>, grid) : launch(k_w4_decode<false, 1, false, 1>, grid);
    return beta ? launch(k_w4_decode<true, 1, false, 0>, grid) : launch(k_w4_decode<false, 1, false, 0>, grid);
}

}  // namespace qblora
