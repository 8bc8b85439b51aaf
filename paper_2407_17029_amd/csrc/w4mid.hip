// Mid-batch forward of a 4-bit block-quantized layer without adapter (merged-model inference, Sec. 3.3, with
// a few dozen to 128 tokens in flight; larger batches are cut into chunks of 128 by the caller):
//
//   Y[t, n] = sum_k X[t, k] * w~[n, k],   w~ = bf16( c[code] * alpha (+ beta) )   (Eq. 1, the bf16 compute
//                                                                                  weight of the training forward)
//
// The regime: every weight is used T times, so up to a few dozen tokens the weight stream from HBM (0.5 byte
// of codes + the block parameters per weight) sets the time and at 128 tokens the MFMAs do.  A token tile of
// 256 (the training kernel) would waste most of its MFMAs here and, with one workgroup per 256 output rows,
// leave most of the chip idle.  Here a workgroup of 4 waves owns 128 output rows (32 per wave), ALL tokens
// (32 * TB of them, TB = 1, 2, 4) and one slice of the input dimension; the slices of a row tile (split-K, as
// many as it takes to put two workgroups on every CU) write fp32 partial tiles that a second kernel adds in
// slice order (deterministic).
//
// A wave dequantizes its own MFMA operand in registers: lane l owns row (l & 31) and the 32 inputs
// 32*(l >> 5) .. +31 of each 64-input step, i.e. 16 bytes of codes, fetched with one load instruction (in the
// tile-ordered code copy the 32 rows of a step are adjacent: 1 KB contiguous per wave); dword j of them is the
// A operand (32 rows x 16 inputs, 8 per lane) of the j-th v_mfma_f32_32x32x16_bf16 of the step.  The weight
// tile never crosses LDS.  The token tile does ([token][64 inputs] bf16, 16-byte chunks XOR-swizzled by
// (row ^ row>>3) & 7): it is shared by the four waves, arrives by direct global -> LDS copies into a ring of
// four stages, and is read as the B operand (lane l: token l & 31, the same 8 inputs).  All vector-memory
// operations of the loop are issued from assembly statements three steps ahead (codes: four) and counted by
// hand (the compiler would tie every LDS access to them): a step waits until only the two youngest batches are
// outstanding.  The operands of step s+1 are built between the MFMAs of step s.
//
// A lane ends up with 4 consecutive output rows of one token per accumulator quad and stores them as one
// 8-byte word (bf16) or one 16-byte word (fp32 partials).
#include "common.h"

namespace qblora {

namespace {

constexpr int kMidThreads = 256;
constexpr int kMidRows = 128;                   // output rows per workgroup
constexpr int kStages = 4;                      // ring of token tiles; operations are issued kStages - 1 steps ahead
constexpr int kTableReplicas = 8;

struct MidDesc {
    const uint8_t* codes; const float* scales; const float* beta; Codebook cb;
    int tiled;                 // codes (and, with 64-blocks, scales and offsets) in tile order
    int d_out, d_in;
    const qblora_bf16* X; int T;
    qblora_bf16* Y;            // splits == 1
    float* part;               // splits > 1: [splits][T][d_out] fp32
    int splits, steps_per_split;
};

__device__ __forceinline__ void copy16_to_lds(const void* uniform_base, uint32_t lane_offset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(lane_offset), "s"(uniform_base) : "memory");
}
// The data of these loads arrive asynchronously: a destination may only be used behind a wait_slot that names it.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__device__ __forceinline__ void load16(u32x4& v, uint32_t lane_offset, const void* uniform_base) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(v) : "v"(lane_offset), "s"(uniform_base) : "memory");
}
__device__ __forceinline__ void load4(float& v, uint32_t lane_offset, const void* uniform_base) {
    asm volatile("global_load_dword %0, %1, %2" : "=&v"(v) : "v"(lane_offset), "s"(uniform_base) : "memory");
}
__device__ __forceinline__ void load16f(f32x4& v, uint32_t lane_offset, const void* uniform_base) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(v) : "v"(lane_offset), "s"(uniform_base) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// codes and block parameters of one step, as fetched
template <int BR>
struct Slot {
    u32x4 cw;
    float sc, be;              // 64-blocks: the row's scale and offset of this step
    f32x4 sc4, be4;            // 8 x 8 blocks: those of the lane's four block columns
    f32x4 sc4b, be4b;          // blocks of 8 rows x 4 inputs (BR = 84): the lane has eight block columns, these are 4 .. 7
};

template <int N, int BR, bool BETA>
__device__ __forceinline__ void wait_slot(Slot<BR>& s) {
    if constexpr (BR == 84) {
        if constexpr (BETA)
            asm volatile("s_waitcnt vmcnt(%5)" : "+v"(s.cw), "+v"(s.sc4), "+v"(s.sc4b), "+v"(s.be4), "+v"(s.be4b) : "n"(N) : "memory");
        else asm volatile("s_waitcnt vmcnt(%3)" : "+v"(s.cw), "+v"(s.sc4), "+v"(s.sc4b) : "n"(N) : "memory");
    } else if constexpr (BR == 8) {
        if constexpr (BETA) asm volatile("s_waitcnt vmcnt(%3)" : "+v"(s.cw), "+v"(s.sc4), "+v"(s.be4) : "n"(N) : "memory");
        else asm volatile("s_waitcnt vmcnt(%2)" : "+v"(s.cw), "+v"(s.sc4) : "n"(N) : "memory");
    } else {
        if constexpr (BETA) asm volatile("s_waitcnt vmcnt(%3)" : "+v"(s.cw), "+v"(s.sc), "+v"(s.be) : "n"(N) : "memory");
        else asm volatile("s_waitcnt vmcnt(%2)" : "+v"(s.cw), "+v"(s.sc) : "n"(N) : "memory");
    }
}

// TB: 32-token blocks; BETA: offsets present; BR: 1 (64 inputs of one row), 8 (8 rows x 8 inputs) or 84 (8 rows x 4 inputs);
// REGROUPED: INT4 model whose code dwords were regrouped by the decode pack (codebook 0..15, offsets present)
template <int TB, bool BETA, int BR, bool REGROUPED>
__global__ __launch_bounds__(kMidThreads) void k_w4_mid(MidDesc d) {
    static_assert(!REGROUPED || (BETA && BR == 1), "regrouped codes belong to INT4 models in 64-blocks");
    constexpr int kStageBytes = TB * 32 * 128;
    static_assert(BR == 1 || BR == 8 || BR == 84, "block shape");
    constexpr int kParamLoads = BR == 84 ? 2 : 1;              // 16-byte (or 4-byte) loads of scales per step; as many of offsets
    constexpr int kOps = TB + 1 + kParamLoads * (BETA ? 2 : 1);   // vector-memory operations per wave and step
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* const sX = smem;                                              // kStages token tiles
    float2* const sT = reinterpret_cast<float2*>(smem + kStages * kStageBytes);  // byte -> (c[lo], c[hi]), replicated

    const int d_out = d.d_out, d_in = d.d_in, T = d.T;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int tiles_n = (d_out + kMidRows - 1) / kMidRows;
    const int nt = blockIdx.x % tiles_n, z = blockIdx.x / tiles_n;
    const int n0 = nt * kMidRows + wave * 32;
    const int n = min(n0 + r, d_out - 1);                       // rows past the end are computed, never stored
    const int steps_total = d_in / kBlock;
    const int s_begin = z * d.steps_per_split;
    const int s_end = min(steps_total, s_begin + d.steps_per_split);

    if constexpr (!REGROUPED) {
        const float2 e = make_float2(d.cb.c[t & 15], d.cb.c[t >> 4]);
#pragma unroll
        for (int q = 0; q < kTableReplicas; ++q) sT[t * kTableReplicas + q] = e;
    }
    const float2* const my_table = sT + (lane & (kTableReplicas - 1));

    // ---- addresses: per-lane byte offsets are fixed, the wave-uniform bases walk along the steps --------------
    const int64_t bpr = steps_total;
    const int64_t run = d.tiled ? (((int64_t)(n >> 8) * bpr) * 256 + (n & 255)) : (int64_t)n * bpr;   // block 0 of row n
    const int64_t bstep = d.tiled ? 256 : 1;                                                          // next block
    const uint32_t c_off = (uint32_t)(run * 32 + 16 * h);
    uint32_t s_off;
    int64_t s_step;                                            // bytes per step in the scale / offset arrays
    if constexpr (BR == 84) {                                  // 16 block columns per step, the lane's half: 8
        s_off = (uint32_t)((((int64_t)(n >> 3) * (d_in >> 2)) + 8 * h) * 4);
        s_step = 64;
    } else if constexpr (BR == 8) {
        s_off = (uint32_t)((((int64_t)(n >> 3) * (d_in >> 3)) + 4 * h) * 4);
        s_step = 32;
    } else {
        s_off = (uint32_t)(run * 4);
        s_step = bstep * 4;
    }
    const int64_t c_step = bstep * 32;
    // copies of the token tile: wave w fills rows 8*TB*w .. +8*TB-1, copy i rows 8*(TB*w + i) + (lane >> 3)
    uint32_t x_off[TB];
#pragma unroll
    for (int i = 0; i < TB; ++i) {
        const int row = 8 * (TB * wave + i) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row ^ (row >> 3)) & 7);
        x_off[i] = (uint32_t)((int64_t)min(row, T - 1) * d_in * 2 + chunk * 16);
    }
    const uint32_t lds_x = __builtin_amdgcn_readfirstlane(lds_address(sX) + wave * TB * 1024);
    const unsigned char* const cbase = d.codes;
    const unsigned char* const sbase = reinterpret_cast<const unsigned char*>(d.scales);
    const unsigned char* const bbase = reinterpret_cast<const unsigned char*>(d.beta);
    const unsigned char* const xbase = reinterpret_cast<const unsigned char*>(d.X);

    // One batch of operations per step, the same count (kOps) whatever the step: the codes and block parameters of
    // step `sc` into register slot `sl`, and the token tile of step `sx` into ring stage `stage`.  Steps past the
    // slice are redirected to its last step (fetched, never used).
    auto issue_codes = [&](Slot<BR>& sl, int step) __attribute__((always_inline)) {
        const int64_t sc = min(step, s_end - 1);
        load16(sl.cw, c_off, cbase + sc * c_step);
        if constexpr (BR == 84) {
            load16f(sl.sc4, s_off, sbase + sc * s_step);
            load16f(sl.sc4b, s_off + 16, sbase + sc * s_step);
            if constexpr (BETA) { load16f(sl.be4, s_off, bbase + sc * s_step); load16f(sl.be4b, s_off + 16, bbase + sc * s_step); }
        } else if constexpr (BR == 8) {
            load16f(sl.sc4, s_off, sbase + sc * s_step);
            if constexpr (BETA) load16f(sl.be4, s_off, bbase + sc * s_step);
        } else {
            load4(sl.sc, s_off, sbase + sc * s_step);
            if constexpr (BETA) load4(sl.be, s_off, bbase + sc * s_step);
        }
    };
    auto issue_x = [&](int step, int stage) __attribute__((always_inline)) {
        const int64_t sx = min(step, s_end - 1);
#pragma unroll
        for (int i = 0; i < TB; ++i) copy16_to_lds(xbase + sx * 128, x_off[i], lds_x + stage * kStageBytes + i * 1024);
    };

    // fragment addresses of the token tile: token 32*tb + r, logical chunk 4h + j
    uint32_t f_off[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int row = 32 * tb + r;
        f_off[tb] = row * 128 + (((4 * h) ^ ((row ^ (row >> 3)) & 7)) << 4);
    }

    f32x16 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[tb][i] = 0.0f;

    auto weight = [&](float c, float a, float b) __attribute__((always_inline)) {
        return BETA ? __fmaf_rn(c, a, b) : __fmul_rn(c, a);
    };
    // Dequantization in 16 units per step: unit k = 4j + i makes dword i (two weights, inputs 2i and 2i+1 of the
    // 8) of the j-th A operand (code dword j).  Table form: unit_a fetches the byte's (c[lo], c[hi]) pair from LDS,
    // unit_b scales, offsets and rounds; an INT4 model's regrouped dword holds input 0, 2, 4, 6, 1, 3, 5, 7 in its
    // nibbles, so the bytes of (w & 0x0F0F0F0F) are inputs 0, 4, 1, 5 and those of ((w >> 4) & 0x0F0F0F0F) 2, 6, 3, 7.
    struct Params { uint32_t cw[4]; float a[8], b[8]; };       // scale / offset of inputs 0..3 and 4..7 of each code dword
    auto params = [&](const Slot<BR>& sl) __attribute__((always_inline)) {
        Params p;
        p.cw[0] = sl.cw.x; p.cw[1] = sl.cw.y; p.cw[2] = sl.cw.z; p.cw[3] = sl.cw.w;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int j = e >> 1;
            if constexpr (BR == 84) {
                p.a[e] = e < 4 ? sl.sc4[e] : sl.sc4b[e - 4];
                p.b[e] = !BETA ? 0.0f : e < 4 ? sl.be4[e] : sl.be4b[e - 4];
            } else {
                p.a[e] = BR == 8 ? sl.sc4[j] : sl.sc;
                p.b[e] = !BETA ? 0.0f : BR == 8 ? sl.be4[j] : sl.be;
            }
        }
        return p;
    };
    auto unit_a = [&](const Params& p, int k, float2& tv) __attribute__((always_inline)) {
        if constexpr (!REGROUPED) tv = my_table[((p.cw[k >> 2] >> (8 * (k & 3))) & 0xffu) * kTableReplicas];
    };
    auto unit_b = [&](const Params& p, int k, const float2& tv) __attribute__((always_inline)) {
        const int j = k >> 2, i = k & 3;
        float lo, hi;
        if constexpr (REGROUPED) {
            const uint32_t t = (p.cw[j] >> (4 * (i & 1))) & 0x0F0F0F0Fu;       // i odd: inputs 2, 6, 3, 7
            lo = (float)((t >> (8 * (i >> 1))) & 0xffu);                          // i < 2: bytes 0 and 2, else 1 and 3
            hi = (float)((t >> (16 + 8 * (i >> 1))) & 0xffu);
        } else {
            lo = tv.x; hi = tv.y;
        }
        const int e = 2 * j + (i >> 1);                        // byte i of the dword: inputs 2i, 2i+1
        return pack_bf16(weight(lo, p.a[e], p.b[e]), weight(hi, p.a[e], p.b[e]));
    };
    // all four operands at once (before the loop)
    auto dequantize = [&](const Slot<BR>& sl, bf16x8 (&wf)[4]) __attribute__((always_inline)) {
        const Params p = params(sl);
        uint32_t o[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) { float2 tv = make_float2(0.f, 0.f); unit_a(p, k, tv); o[k] = unit_b(p, k, tv); }
#pragma unroll
        for (int j = 0; j < 4; ++j) wf[j] = __builtin_bit_cast(bf16x8, make_uint4(o[4 * j], o[4 * j + 1], o[4 * j + 2], o[4 * j + 3]));
    };
    // One step: the 4 * TB MFMAs on this step's operands `wf`, and between them the units that build the next
    // step's operands `wn` from slot `sl` -- written in issue order and fenced after every MFMA: a wave issues in
    // order, so vector work has to sit between the MFMAs to run in their shadow.  LDS reads are issued one MFMA
    // (token fragment) or one unit (table pair) ahead of their use.
    auto step = [&](const bf16x8 (&wf)[4], int stage, const Slot<BR>& sl, bf16x8 (&wn)[4]) __attribute__((always_inline)) {
        constexpr int M = 4 * TB, U = 16 / M;
        const unsigned char* xs = sX + stage * kStageBytes;
        const Params p = params(sl);
        uint32_t o[16];
        float2 tv[2] = {make_float2(0.f, 0.f), make_float2(0.f, 0.f)};
        bf16x8 xf[2];
        auto read_x = [&](int m) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8*>(xs + (f_off[m % TB] ^ ((m / TB) << 4)));
        };
        unit_a(p, 0, tv[0]);
        xf[0] = read_x(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < M; ++m) {
            if (m + 1 < M) xf[(m + 1) & 1] = read_x(m + 1);
            acc[m % TB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[m / TB], xf[m & 1], acc[m % TB], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int k = m * U + q;
                if (k + 1 < 16) unit_a(p, k + 1, tv[(k + 1) & 1]);
                o[k] = unit_b(p, k, tv[k & 1]);
                asm volatile("" : "+v"(o[k]));                  // computed here
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            wn[j] = __builtin_bit_cast(bf16x8, make_uint4(o[4 * j], o[4 * j + 1], o[4 * j + 2], o[4 * j + 3]));
    };

    Slot<BR> slot[kStages];
#pragma unroll
    for (int u = 0; u < kStages; ++u) {                         // defined values for the fields a variant never loads
        slot[u].sc = 0.0f; slot[u].be = 0.0f;
        slot[u].sc4 = f32x4{0.f, 0.f, 0.f, 0.f}; slot[u].be4 = f32x4{0.f, 0.f, 0.f, 0.f};
        slot[u].sc4b = f32x4{0.f, 0.f, 0.f, 0.f}; slot[u].be4b = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    bf16x8 wf[2][4];                                            // operands of this step and of the next
    __syncthreads();                                            // the table is complete
    // The weights of step s+1 are dequantized while the MFMAs of step s issue, so the codes run one step ahead of
    // the token tiles: batch b carries the codes of step b+4 and the tile of step b+3.
    issue_codes(slot[0], s_begin);
#pragma unroll
    for (int u = 0; u < kStages - 1; ++u) { issue_codes(slot[u + 1], s_begin + u + 1); issue_x(s_begin + u, u); }
    wait_slot<(kStages - 1) * kOps, BR, BETA>(slot[0]);
    dequantize(slot[0], wf[0]);
    for (int s = s_begin; s < s_end; s += kStages) {
#pragma unroll
        for (int u = 0; u < kStages; ++u) {
            // the batch issued three steps ago is in when at most the two after it are outstanding
            wait_slot<(kStages - 2) * kOps, BR, BETA>(slot[(u + 1) % kStages]);
            __syncthreads();                                    // every wave's part of the tile is in; all waves are past
                                                                // the step before, whose stage is refilled now
            issue_codes(slot[u], s + u + kStages);              // slot u was turned into operands a step ago
            issue_x(s + u + kStages - 1, (u + kStages - 1) % kStages);
            if (s + u < s_end) step(wf[u & 1], u, slot[(u + 1) % kStages], wf[(u + 1) & 1]);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");            // the redirected look-ahead operations

    // ---- store: lane = token 32*tb + r; registers 4q .. 4q+3 = rows 8q + 4h .. +3 of the wave's 32 ----------
    const bool whole = (d_out & 3) == 0;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int tok = 32 * tb + r;
        if (tok >= T) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int nb = n0 + 8 * q + 4 * h;
            if (nb >= d_out) continue;
            const float v0 = acc[tb][4 * q], v1 = acc[tb][4 * q + 1], v2 = acc[tb][4 * q + 2], v3 = acc[tb][4 * q + 3];
            if (d.splits > 1) {
                float* p = d.part + ((int64_t)z * T + tok) * d_out + nb;
                if (whole) { *reinterpret_cast<float4*>(p) = make_float4(v0, v1, v2, v3); continue; }
                p[0] = v0;
                if (nb + 1 < d_out) p[1] = v1;
                if (nb + 2 < d_out) p[2] = v2;
                if (nb + 3 < d_out) p[3] = v3;
            } else {
                uint16_t* p = reinterpret_cast<uint16_t*>(d.Y) + (int64_t)tok * d_out + nb;
                const uint32_t lo = pack_bf16(v0, v1), hi = pack_bf16(v2, v3);
                if (whole) { *reinterpret_cast<uint2*>(p) = make_uint2(lo, hi); continue; }
                p[0] = (uint16_t)(lo & 0xffffu);
                if (nb + 1 < d_out) p[1] = (uint16_t)(lo >> 16);
                if (nb + 2 < d_out) p[2] = (uint16_t)(hi & 0xffffu);
                if (nb + 3 < d_out) p[3] = (uint16_t)(hi >> 16);
            }
        }
    }
}

// Y = bf16( sum_z part[z] ), slices added in ascending order
__global__ __launch_bounds__(256) void k_w4_mid_reduce(const float* __restrict__ part, int splits, int64_t count,
                                                       qblora_bf16* __restrict__ Y) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 2;
    if (i >= count) return;
    float a = 0.0f, b = 0.0f;
    const bool two = i + 1 < count;
    for (int zz = 0; zz < splits; ++zz) {
        a += part[zz * count + i];
        if (two) b += part[zz * count + i + 1];
    }
    const uint32_t p = pack_bf16(a, b);
    uint16_t* y = reinterpret_cast<uint16_t*>(Y) + i;
    if (two) *reinterpret_cast<uint32_t*>(y) = p;               // i is even: 4-byte aligned
    else y[0] = (uint16_t)(p & 0xffffu);
}

template <int TB>
constexpr size_t mid_lds(bool regrouped) {
    return (size_t)kStages * TB * 32 * 128 + (regrouped ? 0 : 256 * kTableReplicas * sizeof(float2));
}

template <typename K>
bool set_lds(K kernel, size_t smem) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)smem) == hipSuccess;
}

template <int TB, bool BETA, int BR, bool REGROUPED>
int launch_one(const MidDesc& d, unsigned blocks, hipStream_t st) {
    constexpr size_t smem = mid_lds<TB>(REGROUPED);
    static const bool ok = set_lds(k_w4_mid<TB, BETA, BR, REGROUPED>, smem);
    if (!ok) return QBLORA_ERR_LAUNCH;
    hipLaunchKernelGGL((k_w4_mid<TB, BETA, BR, REGROUPED>), dim3(blocks), dim3(kMidThreads), smem, st, d);
    return launch_status();
}

template <int TB>
int launch_tb(const MidDesc& d, unsigned blocks, hipStream_t st, int block_rows, int regrouped, int block_cols) {
    if (block_rows == 8 && block_cols == 4)
        return d.beta ? launch_one<TB, true, 84, false>(d, blocks, st) : launch_one<TB, false, 84, false>(d, blocks, st);
    if (block_rows == 8)
        return d.beta ? launch_one<TB, true, 8, false>(d, blocks, st) : launch_one<TB, false, 8, false>(d, blocks, st);
    if (regrouped) return d.beta ? launch_one<TB, true, 1, true>(d, blocks, st) : QBLORA_ERR_UNSUPPORTED;
    return d.beta ? launch_one<TB, true, 1, false>(d, blocks, st) : launch_one<TB, false, 1, false>(d, blocks, st);
}

}  // namespace

int w4_mid_token_blocks(int T) { return T <= 32 ? 1 : T <= 64 ? 2 : 4; }

// Slices of the input dimension for T <= 128 tokens.  Measured over 2 / 3 / 4 waves per workgroup and 1 .. 8 slices on
// 4096 x 4096, 11008 x 4096 and 22016 x 8192: what counts is the number of workgroups -- about 700 up to 64 tokens
// (the weight stream wants loads in flight), about 400 at 128 (two resident per CU; more slices only add partial
// tiles) -- while 64- or 96-row workgroups differ from 128-row ones by a few percent at most; one slice per row tile,
// which the balance of matrix work alone would choose at 128 tokens, is 20 % slower than two.  At least 4 steps per
// slice, at most 8 slices, no empty slice.
int w4_mid_splits(int d_out, int d_in, int T) {
    const int tiles_n = (d_out + kMidRows - 1) / kMidRows, steps = d_in / kBlock;
    const int target = w4_mid_token_blocks(T) == 4 ? 400 : 700;
    int want = (target + tiles_n / 2) / tiles_n;
    if (want > steps / 4) want = steps / 4;
    if (want > 8) want = 8;
    if (want < 1) want = 1;
    const int per = (steps + want - 1) / want;
    return (steps + per - 1) / per;
}

size_t w4_mid_part_bytes(int d_out, int d_in, int T) {
    const int splits = w4_mid_splits(d_out, d_in, T);
    return splits > 1 ? sizeof(float) * (size_t)splits * (size_t)T * (size_t)d_out : 0;
}

int launch_w4_mid(const uint8_t* codes, const float* scales, const float* beta, const Codebook& cb, int tiled, int d_out,
                  int d_in, const qblora_bf16* X, int T, qblora_bf16* Y, float* part, hipStream_t st, int block_rows,
                  int regrouped, int block_cols) {
    if (T < 1 || T > 128 || d_in % kBlock != 0 || d_out < 1) return QBLORA_ERR_SHAPE;
    // 32-bit lane offsets: the arrays of one weight and the token rows must stay below 4 GiB
    if ((int64_t)((d_out + 255) / 256) * 256 * (d_in / 2) >= ((int64_t)1 << 32) || (int64_t)T * d_in * 2 >= ((int64_t)1 << 32))
        return QBLORA_ERR_SHAPE;
    if (block_rows == 8 && (d_out % 8 != 0)) return QBLORA_ERR_SHAPE;
    const int splits = w4_mid_splits(d_out, d_in, T), steps = d_in / kBlock;
    if (splits > 1 && !part) return QBLORA_ERR_WORKSPACE;
    MidDesc d{codes, scales, beta, cb, tiled, d_out, d_in, X, T, Y, part, splits, (steps + splits - 1) / splits};
    const unsigned blocks = (unsigned)(((d_out + kMidRows - 1) / kMidRows) * splits);
    int rc;
    switch (w4_mid_token_blocks(T)) {
        case 1: rc = launch_tb<1>(d, blocks, st, block_rows, regrouped, block_cols); break;
        case 2: rc = launch_tb<2>(d, blocks, st, block_rows, regrouped, block_cols); break;
        default: rc = launch_tb<4>(d, blocks, st, block_rows, regrouped, block_cols); break;
    }
    if (rc || splits == 1) return rc;
    const int64_t count = (int64_t)T * d_out;
    hipLaunchKernelGGL(k_w4_mid_reduce, dim3((unsigned)((count / 2 + 256) / 256)), dim3(256), 0, st, part, splits, count, Y);
    return launch_status();
}

}  // namespace qblora
