// Prefill product for int4 weights on the fp16 matrix cores:
//   y[m,n] = sum_k x[m,k] * (s * Wq[n,k]),  fp32 accumulation,
// with s = s[n, k/32] (group scales) or s[n] (per-channel scales).
// FP16 activations with quantized weights (section 4.2 of the paper), computed
// on matrix units as the compute-bound prefill stage wants (section 3.7).
//
// Two kernels.  The main one (K a multiple of 128; described in front of it)
// never writes dequantized weights anywhere: packed tiles are copied verbatim
// into LDS, a lane reads the dword that is its MFMA operand, converts it in
// registers and feeds the matrix core.  Int4 weights are a quarter of the
// activation bytes, so LDS carries far fewer bytes per MFMA than with a
// dequantized weight tile.  The second kernel is the general fallback (any K
// that is a multiple of 32):
//
// Per K stage of 128 (one packed weight tile per 16 rows): every thread loads
// 16-byte vectors of packed codes (four octets, one per quantization group of
// the tile) plus the four group scales of its row, dequantizes in registers
// (exact int -> binary16, then one binary16 multiply by the scale) and writes
// 16-byte binary16 vectors to LDS.  Activations are copied to LDS as they are.
// LDS holds both tiles octet-major ([k/8][row], 16 B each), so an MFMA fragment
// (32 rows x 16 k, lane = row + 32 * (k/8)) is two runs of 512 contiguous
// bytes; the activation tile has a one-vector pad per octet so that its
// transposing writes are conflict free as well.
#include <type_traits>

#include "qfc_internal.h"

namespace qfc {
namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BN = 128, BM = 128, BK = 128;
constexpr int OCT = BK / 8;      // 16-byte octets (8 binary16) per row per stage
constexpr int LDW = BN;          // vectors per octet, weights
constexpr int LDX = BM + 1;      // vectors per octet, activations (padded)
constexpr size_t kLdsBytes = (size_t)OCT * (LDW + LDX) * 16;

struct GemmF16Args {
    const uint4 *w;   // packed int4 row tiles (W4G32 or W4C)
    const uint4 *x;   // binary16 [M, K] viewed as 16-byte vectors
    _Float16 *y;
    const _Float16 *res;  // [M, N] residual added before the rounding, or null
    const float *sw;  // W4C: fp32 scale per output channel [Np]
    int M, N, K, KT, rt_stride, n_tiles, m_tiles;
    int gated_act = -1;  // QFC_ACT_*: the layer is packed in pairs and y [M, N/2] = fp16(act(gate) * other)
};

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// eight biased codes -> eight scaled binary16 values, k ascending
__device__ __forceinline__ uint4 dequant8_scaled(uint32_t w, uint32_t scale_bits) {
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const _Float16 sh = __builtin_bit_cast(_Float16, (uint16_t)scale_bits);
    const h2 s = {sh, sh};
    const uint32_t lo = w & 0x0F0F0F0Fu, hi = w & 0xF0F0F0F0u;
    const h2 p0 = (as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u)) - c1032) * s;
    const h2 p1 = (as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u)) - c1032) * s;
    const h2 p2 = (as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u)) * c16th - c72) * s;
    const h2 p3 = (as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u)) * c16th - c72) * s;
    return make_uint4(as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3));
}

// eight int8 codes (two dwords) -> eight binary16 values, exactly (sign bit flipped: b + 128 under the
// exponent byte 0x64 is 1024 + b + 128)
__device__ __forceinline__ uint4 dequant_i8x8(uint32_t lo, uint32_t hi) {
    const h2 c1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
    const uint32_t a = lo ^ 0x80808080u, b = hi ^ 0x80808080u;
    const h2 p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, a, 0x04010400u)) - c1152;
    const h2 p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, a, 0x04030402u)) - c1152;
    const h2 p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, b, 0x04010400u)) - c1152;
    const h2 p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, b, 0x04030402u)) - c1152;
    return make_uint4(as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3));
}

// PC = per-channel scales (W4C): unscaled integer weights in the MFMA, fp32 scale in the epilogue.
// W8 (with PC) = int8 per-channel weights with binary16 activations (the "q8" scheme of section 4.2
// with FP16 activations at M > 8): two packed KiB tiles of 64 k per row tile and stage, converted
// exactly to binary16 on their way into LDS, fp32 scale in the epilogue.
template <bool PC, bool W8 = false>
__global__ __launch_bounds__(256) void gemm_f16_w4_kernel(GemmF16Args a) {
    static_assert(!W8 || PC, "int8 weights carry per-channel scales");
    extern __shared__ uint4 lds[];
    uint4 *lds_w = lds;
    uint4 *lds_x = lds + OCT * LDW;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;

    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles;
    const int mt = logical % a.m_tiles;

    // weights: thread -> two packed vectors per stage: row tile (tid / 64) and (tid / 64 + 4)
    const int c = lane & 15, q = lane >> 4;
    const uint4 *w_rt[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        w_rt[i] = a.w + (size_t)(nt * (BN / 16) + wave + 4 * i) * a.rt_stride * 64;
    const int K8 = a.K / 8;

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4 wreg[2], wreg2[W8 ? 2 : 1], xreg[8];
    uint2 sreg[2];
    auto load_stage = [&](int kt) {
        const int u = kt >> 3;
        const int wpos = W8 ? 2 * kt : PC ? kt : kt + u;       // weight tile kt of the row tile (int8: tiles 2 kt, 2 kt + 1)
        const int spos = min(8 * u + 8, a.KT) + u;             // scale tile of its unit
        const int soff = (((kt & 7) >> 1) * 16 + c) * 2 + (kt & 1);  // 8-byte index inside it
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            wreg[i] = w_rt[i][(size_t)wpos * 64 + lane];
            if (W8) wreg2[i] = w_rt[i][(size_t)(wpos + 1) * 64 + lane];
            sreg[i] = PC ? make_uint2(0x3C003C00u, 0x3C003C00u)  // 1.0: the multiply is exact
                         : reinterpret_cast<const uint2 *>(w_rt[i] + (size_t)spos * 64)[soff];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int v = tid + 256 * i;
            const int row = mt * BM + (v >> 4);
            const int o = kt * OCT + (v & 15);
            xreg[i] = (row < a.M && o < K8) ? a.x[(size_t)row * K8 + o] : make_uint4(0, 0, 0, 0);
        }
    };

    const int stages = W8 ? a.KT / 2 : a.KT;  // (int8 rows are padded to a multiple of 256 k: an even number of tiles)
    load_stage(0);
    for (int kt = 0; kt < stages; ++kt) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = (wave + 4 * i) * 16 + c;
            if (W8) {
                // lane (c, q) of tile h holds the codes k = 64 h + 16 q .. + 15: octets 8 h + 2 q and + 1 of the stage
                lds_w[(2 * q) * LDW + row] = dequant_i8x8(wreg[i].x, wreg[i].y);
                lds_w[(2 * q + 1) * LDW + row] = dequant_i8x8(wreg[i].z, wreg[i].w);
                lds_w[(8 + 2 * q) * LDW + row] = dequant_i8x8(wreg2[i].x, wreg2[i].y);
                lds_w[(8 + 2 * q + 1) * LDW + row] = dequant_i8x8(wreg2[i].z, wreg2[i].w);
                continue;
            }
            const uint32_t wd[4] = {wreg[i].x, wreg[i].y, wreg[i].z, wreg[i].w};
            const uint32_t sc[4] = {sreg[i].x & 0xFFFFu, sreg[i].x >> 16, sreg[i].y & 0xFFFFu, sreg[i].y >> 16};
#pragma unroll
            for (int j = 0; j < 4; ++j) lds_w[(j * 4 + q) * LDW + row] = dequant8_scaled(wd[j], sc[j]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int v = tid + 256 * i;
            lds_x[(v & 15) * LDX + (v >> 4)] = xreg[i];
        }
        __syncthreads();
        if (kt + 1 < stages) load_stage(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int o = 2 * ks + (lane >> 5);
            v8h fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fa[i] = __builtin_bit_cast(v8h, lds_w[o * LDW + wn * 64 + i * 32 + (lane & 31)]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fb[j] = __builtin_bit_cast(v8h, lds_x[o * LDX + wm * 64 + j * 32 + (lane & 31)]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // Epilogue.  A lane holds one token row (lane % 32) and groups of four
    // consecutive n; stored directly, every store instruction would touch 32 rows
    // of y with 8 bytes each.  The binary16 values go through LDS (32 token rows x
    // 64 channels per wavefront at a time) and leave as 16-byte stores along n.
    __syncthreads();  // all wavefronts are done with the tiles in LDS
    if ((a.N % 8) == 0) {
        constexpr int PITCH = (64 + 8) * 2;  // bytes per staged row
        char *region = reinterpret_cast<char *>(lds) + wave * (32 * PITCH);
        const int n0 = nt * BN + wn * 64;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int mrow0 = mt * BM + wm * 64 + j * 32;
            const bool has_res = a.res != nullptr;
            if (has_res) stage_residual_block<8, PITCH>(region, a.res, mrow0, n0, a.M, a.N, lane);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int nl = i * 32 + 8 * qq + 4 * (lane >> 5);
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    float4 sc = make_float4(1.0f, 1.0f, 1.0f, 1.0f);
                    if (PC) sc = *reinterpret_cast<const float4 *>(a.sw + n0 + nl);
                    float v[4] = {acc[i][j][4 * qq + 0] * sc.x, acc[i][j][4 * qq + 1] * sc.y,
                                  acc[i][j][4 * qq + 2] * sc.z, acc[i][j][4 * qq + 3] * sc.w};
                    if (has_res) {
                        float rv[4];
                        staged_residual4(region, (lane & 31) * PITCH + nl * 2, rv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += rv[e];
                    }
                    const h4 hv = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
                    *reinterpret_cast<h4 *>(region + (lane & 31) * PITCH + nl * 2) = hv;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int it = 0; it < 4; ++it) {  // 32 rows x 8 chunks of 16 bytes
                const int idx = it * 64 + lane;
                const int row = idx >> 3, ch = idx & 7;
                const uint4 v = *reinterpret_cast<const uint4 *>(region + row * PITCH + ch * 16);
                const int mm = mrow0 + row, nn = n0 + ch * 8;
                if (mm < a.M && nn < a.N) *reinterpret_cast<uint4 *>(a.y + (size_t)mm * a.N + nn) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        return;
    }
    const bool vec_ok = (a.N % 4) == 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int m = mt * BM + wm * 64 + j * 32 + (lane & 31);
        if (m >= a.M) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const int n = nt * BN + wn * 64 + i * 32 + 8 * qq + 4 * (lane >> 5);
                if (n >= a.N) continue;
                _Float16 *y = a.y + (size_t)m * a.N + n;
                _Float16 h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = PC ? acc[i][j][4 * qq + e] * a.sw[n + e] : acc[i][j][4 * qq + e];
                    if (a.res && n + e < a.N) v += (float)a.res[(size_t)m * a.N + n + e];
                    h[e] = (_Float16)v;
                }
                if (vec_ok) {
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    *reinterpret_cast<h4 *>(y) = h4{h[0], h[1], h[2], h[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < a.N) y[e] = h[e];
                }
            }
        }
    }
}


// ---------------------------------------------------------------------------
// Main kernel: weights never dequantized into LDS, activations through an LDS ring.
//
// Workgroup = 8 wavefronts over 256 output channels x 128 token rows: four
// groups of 64 channels (four packed row tiles each), times two halves of K.
// Both wavefronts of a channel group own the same 64 x 128 outputs as 2 x 4
// tiles of v_mfma_f32_32x32x16_f16; in every 128-k tile one takes quantization
// groups 0, 1 and the other groups 2, 3; at the end they swap halves of their
// accumulators through LDS and each stores half of the outputs.  The two share a SIMD, so that the integer -> binary16
// conversion of one (about 60 vector instructions per group, each done by exactly
// one wavefront of the chip) runs while the matrix core works for the other:
// from a single wavefront the conversion and the MFMAs mostly add up instead of
// overlapping.  (Measured on MI355X: this MFMA shape runs at the full matrix rate
// from one wavefront per SIMD; the 16x16x32 shape reaches less than half of it.)
// Weights are the row operand, so a lane ends up with groups of four consecutive
// n of one token row.
//
// Everything arrives by direct global -> LDS copies (16 bytes per lane, one KiB
// per wavefront instruction).  Per 128-k tile every wavefront issues one batch of
// 7 copies: 2 of the 16 packed KiB tiles of codes (tile j + 3), the scales of its
// channel group for tile j + 3 (lane = one of the 64 rows, 16 bytes = 8 groups;
// both wavefronts of the group write the same bytes), and 4 KiB of the 32 KiB
// activation stage j + 2 (128 rows x 128 k, stored as two halves of 64 k).
// Three-slot rings; nothing else touches vector memory inside the loop, so the
// copies complete in issue order and "the batch issued two tiles ago has landed"
// is "at most one batch is outstanding".  One workgroup barrier per tile.
//
// Inside a wavefront the loop is software pipelined by one quantization group:
// while the 16 MFMAs of a group run, the activations of the next group are read
// from LDS and its codes are converted (exact int -> binary16, one binary16
// multiply by the group scale); the codes and scales of a tile are read into
// registers at the end of the tile before.
//
// An MFMA operand is 32 rows x 16 k, lane = (row r, k octet kh).  For the
// weights, lane (r, kh) of row pair ip, k step s owns the 16-byte vector of row
// tile 2 ip + r / 16, lane (2 s + kh) * 16 + r % 16 of a packed tile: dword g of
// it is the lane's operand for group g.
// A half of an activation stage is 128 rows x 64 k, row-major with 128-byte
// rows; the 16-byte octet o of row r sits at octet position o ^ ((r >> 1) & 7),
// which makes the operand reads conflict free while a wavefront copy instruction
// still reads whole 128-byte rows from memory.
typedef __attribute__((address_space(3))) void *lptr_t;

constexpr int DBN = 256, DBM = 128;
constexpr int DRING = 3;
constexpr int DX_BYTES = DBM * 128 * 2;           // activation stage: 128 rows x 128 k
constexpr int DW_BYTES = 16 * 1024;               // codes of one tile: 16 row tiles
constexpr int DS_BYTES = 4 * 1024;                // scales for one tile: 4 channel groups x 64 rows x 16 B
constexpr int DW_OFF = DRING * DX_BYTES;
constexpr int DS_OFF = DW_OFF + DRING * DW_BYTES;
constexpr int kDirectRingBytes = DS_OFF + DRING * DS_BYTES;
constexpr int DSPARE_OFF = kDirectRingBytes;          // one spare KiB: destination of the copies past the end of K
constexpr int kDirectLdsBytes = kDirectRingBytes + 1024;
static_assert(kDirectLdsBytes <= 160 * 1024, "LDS of a compute unit");
constexpr int DBATCH = 2 + 1 + 4;                 // copies per wavefront per tile (one fewer without group scales)
constexpr int DEX_BYTES = 64 * 64 * 4;            // half of a wavefront's accumulators (exchange buffer)
constexpr int DEPI_PITCH = (64 + 8) * 2;
static_assert(8 * DEX_BYTES <= kDirectRingBytes && 32 * DEPI_PITCH <= DEX_BYTES, "exchange and store staging fit in the rings, below the spare KiB");
static_assert(3 * DBATCH <= 63, "outstanding copies of a wavefront (three batches at most) must fit the 6-bit counter");

// eight biased codes -> eight scaled binary16 values (k ascending) as an MFMA operand
__device__ __forceinline__ v8h dequant_frag(uint32_t w, h2 s) {
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t lo = w & 0x0F0F0F0Fu, hi = w & 0xF0F0F0F0u;
    const h2 p0 = (as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u)) - c1032) * s;
    const h2 p1 = (as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u)) - c1032) * s;
    const h2 p2 = (as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u)) * c16th - c72) * s;
    const h2 p3 = (as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u)) * c16th - c72) * s;
    return v8h{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// the same without a scale: the integer values themselves (W4C; the scale is applied to the output)
__device__ __forceinline__ v8h dequant_frag_unscaled(uint32_t w) {
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t lo = w & 0x0F0F0F0Fu, hi = w & 0xF0F0F0F0u;
    const h2 p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u)) - c1032;
    const h2 p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u)) - c1032;
    const h2 p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u)) * c16th - c72;
    const h2 p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u)) * c16th - c72;
    return v8h{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// One MFMA followed by a few vector instructions, four times: the order the
// instructions of a quarter of a "multiply one group, convert the next" block
// (4 MFMAs, the conversion of one operand) are issued in.
__device__ __forceinline__ void interleave_mfma_valu() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
    }
}

template <bool PC>
__global__ __launch_bounds__(512) void gemm_f16_w4_direct_kernel(GemmF16Args a) {
    constexpr int BATCH = PC ? DBATCH - 1 : DBATCH;
    extern __shared__ uint4 lds[];
    char *lds_b = reinterpret_cast<char *>(lds);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ng = wave & 3;   // channel group: output channels 64 ng .. 64 ng + 63 of the tile
    const int ks = wave >> 2;  // K half: quantization groups 2 ks, 2 ks + 1 of every 128-k tile
    const int c = lane & 15, q = lane >> 4;
    const int r = lane & 31, kh = lane >> 5;

    // Workgroups are dealt to the 8 XCDs round robin; each XCD has its own L2.  Where
    // the tile grid allows, an XCD gets a rectangle of (n_tiles / 2) x (m_tiles / 4)
    // tiles and walks it channel tile by channel tile, so that the workgroups in
    // flight on it (about 32) share 4 activation tiles and 8 weight tiles.
    const int total = a.n_tiles * a.m_tiles;
    int nt, mt;
    if (a.m_tiles % 4 == 0 && a.n_tiles % 2 == 0) {
        const int xcd = blockIdx.x % 8, j = blockIdx.x / 8;
        const int cm = a.m_tiles / 4, cn = a.n_tiles / 2;
        nt = (xcd & 1) * cn + j / cm;
        mt = (xcd >> 1) * cm + j % cm;
    } else {
        int logical = blockIdx.x;
        if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
        nt = logical / a.m_tiles;
        mt = logical % a.m_tiles;
    }

    const int KT = a.KT;  // packed weight tiles (128 k) per row tile; K is a multiple of 128 here

    // Sources of the copies: a wavefront-uniform base that advances along K, plus
    // a per-lane byte offset that never changes.
    // activations: block b = wave + 8 i (i < 4) = rows 8 (b % 16) .. + 7 of half b / 16 = i / 2
    const char *xbase = reinterpret_cast<const char *>(a.x) + (size_t)mt * DBM * a.K * 2;
    uint32_t xlane[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int rl = 8 * (wave + 8 * i) + (lane >> 3);
        const int oct = (lane & 7) ^ ((rl >> 1) & 7);
        const int row = min(mt * DBM + rl, a.M - 1) - mt * DBM;  // rows past M: any finite data, never stored
        xlane[i] = (uint32_t)row * (uint32_t)a.K * 2u + oct * 16;
    }
    // codes: row tiles 2 ks, 2 ks + 1 of the channel group; lane l takes vector l of a packed tile
    const char *wbase = reinterpret_cast<const char *>(a.w) + (size_t)(nt * (DBN / 16) + ng * 4 + ks * 2) * a.rt_stride * 1024;
    const uint32_t wlane = lane * 16;
    // scales: lane l = (row tile l / 16, row l % 16) takes the 16-byte vector of its row
    const char *sbase = reinterpret_cast<const char *>(a.w) + (size_t)(nt * (DBN / 16) + ng * 4) * a.rt_stride * 1024;
    const uint32_t slane = (uint32_t)q * a.rt_stride * 1024u + c * 16;
    const size_t rt_bytes = (size_t)a.rt_stride * 1024;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)lds;  // LDS byte address of the rings
    // The 7 copies of a batch, one at a time (they are spread over the MFMA blocks of
    // a tile: issued together by all eight wavefronts right after the barrier they
    // would queue up behind each other in the memory pipeline while the matrix
    // cores idle).  Past the end of K the copies start over at tile 0, so that the
    // count of outstanding copies is the same on every iteration, and all land in
    // one spare KiB behind the rings that nothing reads and the exchange and store
    // phases never use (distinct sources, not the last tile again and again: many
    // copies of the same lines in flight from one wavefront had been seen in ring
    // slots after the counter said they were done; the cause is not known, so no
    // late copy may have a destination that anything reads or reuses).
    // (bulk: the caller knows that tile t lies inside K; the tiles of the main loop's bulk part then
    // carry no end-of-K tests)
    constexpr bool kBulk = true, kEdge = false;  // (constants at every call site: the tests fold away)
    auto issue_w = [&](int t, int i, const bool bulk) __attribute__((always_inline)) {  // codes of tile t, row tile 2 ks + i of the channel group
        const bool real = bulk || t < KT;
        const int tc = real ? t : min(t - KT, KT - 1);
        const size_t wpos = (size_t)(PC ? tc : tc + (tc >> 3)) * 1024;
        copy16_to_lds(wbase + i * rt_bytes + wpos, wlane,
                      lds0 + (real ? DW_OFF + (t % DRING) * DW_BYTES + (ng * 4 + ks * 2 + i) * 1024 : DSPARE_OFF));
    };
    auto issue_s = [&](int t, const bool bulk) __attribute__((always_inline)) {  // scales of tile t: vector (t % 8) / 2 * 16 + row of the unit's scale tile (8 groups = 2 tiles)
        const bool real = bulk || t < KT;
        const int tc = real ? t : min(t - KT, KT - 1), u = tc >> 3;
        const size_t spos = (size_t)(min(8 * u + 8, KT) + u) * 1024 + (size_t)((tc & 7) >> 1) * 256;
        copy16_to_lds(sbase + spos, slane, lds0 + (real ? DS_OFF + (t % DRING) * DS_BYTES + ng * 1024 : DSPARE_OFF));
    };
    auto issue_x = [&](int t, int i, const bool bulk) __attribute__((always_inline)) {  // activation stage t, block wave + 8 (i % 2) of half i / 2
        const bool real = bulk || t < KT;
        const int tc = real ? t : min(t - KT, KT - 1);
        copy16_to_lds(xbase + (size_t)tc * 256 + (i >> 1) * 128, xlane[i & 1],
                      lds0 + (real ? (t % DRING) * DX_BYTES + wave * 1024 + (i >> 1) * (DX_BYTES / 2) + (i & 1) * 8192 : DSPARE_OFF));
    };
    auto issue_batch = [&](int tw, int tx) {
        issue_w(tw, 0, kEdge); issue_w(tw, 1, kEdge);
        if (!PC) issue_s(tw, kEdge);
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_x(tx, i, kEdge);
    };

    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // operand read addresses of this lane
    int xoff[2][2];  // [group of the half][k step s]: row r, octet (4 g + 2 s + kh) ^ ((r >> 1) & 7)
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int s = 0; s < 2; ++s) xoff[g][s] = ks * (DX_BYTES / 2) + r * 128 + (((4 * g + 2 * s + kh) ^ ((r >> 1) & 7)) << 4);
    const char *wring = lds_b + DW_OFF + ng * 4096 + ((r >> 4) * 64 + kh * 16 + (r & 15)) * 16 + ks * 8;
    const char *sring = lds_b + DS_OFF + ng * 1024 + r * 16 + ks * 4;

    uint4 x0[4][2], x1[4][2];  // activations of a group: [token row block jp][k step s]
    uint2 wv[2][2];            // codes of the current tile: [row pair ip][k step s], .x / .y = this wavefront's two groups
    uint32_t sv[2];            // their scales: [row pair ip], two binary16
    v8h fa0[2][2], fa1[2][2];  // converted weights of a group

    auto read_x = [&](uint4 (&x)[4][2], int g, int t) {
        const char *lx = lds_b + (t % DRING) * DX_BYTES;
#pragma unroll
        for (int jp = 0; jp < 4; ++jp)
#pragma unroll
            for (int s = 0; s < 2; ++s) x[jp][s] = *reinterpret_cast<const uint4 *>(lx + xoff[g][s] + jp * 4096);
    };
    auto read_ws = [&](int t) {
#pragma unroll
        for (int ip = 0; ip < 2; ++ip) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
                wv[ip][s] = *reinterpret_cast<const uint2 *>(wring + (t % DRING) * DW_BYTES + ip * 2048 + s * 512);
            if (!PC) sv[ip] = *reinterpret_cast<const uint32_t *>(sring + (t % DRING) * DS_BYTES + ip * 512 + (t & 1) * 8);
        }
    };
    // quarter qb of the conversion of a group: operand (ip, s) = (qb / 2, qb % 2)
    auto convert = [&](v8h (&fa)[2][2], int g, int qb) {  // g = 0, 1: group of this wavefront's half of the tile
        const int ip = qb >> 1, sx = qb & 1;
        if (PC) {
            fa[ip][sx] = dequant_frag_unscaled(g ? wv[ip][sx].y : wv[ip][sx].x);
        } else {
            const h2 s2 = as_h2(__builtin_amdgcn_perm(0u, sv[ip], g ? 0x03020302u : 0x01000100u));
            fa[ip][sx] = dequant_frag(g ? wv[ip][sx].y : wv[ip][sx].x, s2);
        }
    };
    // quarter qb of the product of a group: k step qb / 2, token row blocks 2 (qb % 2), + 1
    auto multiply = [&](const v8h (&fa)[2][2], const uint4 (&x)[4][2], int qb) {
        const int sx = qb >> 1;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int jp = 2 * (qb & 1) + jj;
#pragma unroll
            for (int ip = 0; ip < 2; ++ip)
                acc[ip][jp] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ip][sx], __builtin_bit_cast(v8h, x[jp][sx]),
                                                                     acc[ip][jp], 0, 0, 0);
        }
    };

    // Copies in issue order: codes/scales 0, codes/scales 1, stage 0 | codes/scales 2,
    // stage 1 | then during tile t: codes/scales t + 3, stage t + 2.
    issue_w(0, 0, kEdge); issue_w(0, 1, kEdge);
    if (!PC) issue_s(0, kEdge);
    issue_w(1, 0, kEdge); issue_w(1, 1, kEdge);
    if (!PC) issue_s(1, kEdge);
#pragma unroll
    for (int i = 0; i < 4; ++i) issue_x(0, i, kEdge);
    issue_batch(2, 1);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) fa1[i][j] = v8h{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) x1[i][j] = make_uint4(0, 0, 0, 0);
    wait_vmcnt<BATCH>();
    asm volatile("s_barrier" ::: "memory");
    read_ws(0);
    auto tile = [&](int t, const bool bulk) __attribute__((always_inline)) {
        // What was issued two tiles ago has landed once only the newest batch is
        // outstanding: stage t, codes and scales of tile t + 1.  The barrier makes
        // the other wavefronts' copies visible and says that every wavefront is done
        // with stage t - 1 and has the codes of tile t in registers: their slots are
        // overwritten by the copies issued during this tile.
        wait_vmcnt<BATCH>();
        asm volatile("s_barrier" ::: "memory");
        read_x(x0, 0, t);
        __builtin_amdgcn_sched_barrier(0);  // the reads are in flight before the MFMAs start
#pragma unroll
        for (int qb = 0; qb < 4; ++qb) {  // group before x converted group 0; activation copies in between
            multiply(fa1, x1, qb);
            convert(fa0, 0, qb);
            interleave_mfma_valu();
            __builtin_amdgcn_sched_barrier(0);
            issue_x(t + 2, qb, bulk);
        }
        read_x(x1, 1, t);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int qb = 0; qb < 4; ++qb) {
            multiply(fa0, x0, qb);
            convert(fa1, 1, qb);
            interleave_mfma_valu();
            __builtin_amdgcn_sched_barrier(0);
            if (qb == 0) issue_w(t + 3, 0, bulk);
            if (qb == 1) issue_w(t + 3, 1, bulk);
            if (qb == 2 && !PC) issue_s(t + 3, bulk);
        }
        read_ws(t + 1);
    };
    {
        int t = 0;
        for (; t + 3 < KT; ++t) tile(t, kBulk);  // every copy issued during these tiles lies inside K
        for (; t < KT; ++t) tile(t, kEdge);
    }
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) multiply(fa1, x1, qb);
    wait_vmcnt<0>();

    // The two wavefronts of a channel group hold partial sums of the same outputs.
    // Each keeps two of the four 32-row blocks and hands the other two to its
    // partner through LDS ([wavefront][16-byte vector][lane], 16 KiB per wavefront
    // over the dead rings), adds what it receives, and stores its half.
    asm volatile("s_barrier" ::: "memory");  // every wavefront is done with the rings
    const int keep = 2 * ks;                  // token row blocks keep, keep + 1 stay here
    {
        float4 *mine = reinterpret_cast<float4 *>(lds_b + wave * DEX_BYTES) + lane;
#pragma unroll
        for (int ip = 0; ip < 2; ++ip)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const v16f &v = ks ? acc[ip][jj] : acc[ip][2 + jj];
                    mine[((ip * 2 + jj) * 4 + qq) * 64] = make_float4(v[4 * qq], v[4 * qq + 1], v[4 * qq + 2], v[4 * qq + 3]);
                }
    }
    __syncthreads();
    v16f out[2][2];  // [ip][jj]: block keep + jj
    {
        const float4 *theirs = reinterpret_cast<const float4 *>(lds_b + (wave ^ 4) * DEX_BYTES) + lane;
#pragma unroll
        for (int ip = 0; ip < 2; ++ip)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const float4 p = theirs[((ip * 2 + jj) * 4 + qq) * 64];
                    const v16f &v = ks ? acc[ip][2 + jj] : acc[ip][jj];
                    out[ip][jj][4 * qq + 0] = v[4 * qq + 0] + p.x;
                    out[ip][jj][4 * qq + 1] = v[4 * qq + 1] + p.y;
                    out[ip][jj][4 * qq + 2] = v[4 * qq + 2] + p.z;
                    out[ip][jj][4 * qq + 3] = v[4 * qq + 3] + p.w;
                }
    }
    __syncthreads();  // the exchange buffers are free: each wavefront stages its stores in its own
    if (PC) {  // per-channel scale of the lane's output channels
#pragma unroll
        for (int ip = 0; ip < 2; ++ip)
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const float4 sc = *reinterpret_cast<const float4 *>(a.sw + nt * DBN + ng * 64 + ip * 32 + 8 * qq + 4 * kh);
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    out[ip][jj][4 * qq + 0] *= sc.x;
                    out[ip][jj][4 * qq + 1] *= sc.y;
                    out[ip][jj][4 * qq + 2] *= sc.z;
                    out[ip][jj][4 * qq + 3] *= sc.w;
                }
            }
    }

    // Epilogue: a lane holds one token row (lane % 32) and groups of four
    // consecutive n.  The binary16 values go through a per-wavefront LDS block
    // (32 token rows x 64 channels) and leave as 16-byte stores along n.
    const int n0 = nt * DBN + ng * 64;
    if (a.gated_act >= 0) {
        // Layer packed in pairs (operator fusion, section 3.6 of the paper): physical rows 32 t .. + 15
        // are gate rows and 32 t + 16 .. + 31 the other branch's rows of the same 16 channels, so the
        // registers 4 qq + e (qq = 0, 1) and 4 (qq + 2) + e of a 32 x 32 tile are the two branches of one
        // channel.  32 output channels per wavefront, rows of N / 2 values.
        const GateCoeffs gc = gate_coeffs(a.gated_act);
        const int half = a.N / 2, o0 = n0 / 2;
        char *region = lds_b + wave * DEX_BYTES;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int mrow0 = mt * DBM + (keep + jj) * 32;
#pragma unroll
            for (int ip = 0; ip < 2; ++ip)
#pragma unroll
                for (int qq = 0; qq < 2; ++qq) {
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    h4 hv;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        hv[e] = (_Float16)(gate_activation(out[ip][jj][4 * qq + e], gc) * out[ip][jj][4 * (qq + 2) + e]);
                    *reinterpret_cast<h4 *>(region + r * DEPI_PITCH + (ip * 16 + 8 * qq + 4 * kh) * 2) = hv;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int it = 0; it < 2; ++it) {  // 32 rows x 4 chunks of 16 bytes
                const int idx = it * 64 + lane;
                const int row = idx >> 2, ch = idx & 3;
                const uint4 v = *reinterpret_cast<const uint4 *>(region + row * DEPI_PITCH + ch * 16);
                const int mm = mrow0 + row, nn = o0 + ch * 8;
                if (mm < a.M && nn < half) *reinterpret_cast<uint4 *>(a.y + (size_t)mm * half + nn) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        return;
    }
    if ((a.N % 8) == 0) {
        char *region = lds_b + wave * DEX_BYTES;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int mrow0 = mt * DBM + (keep + jj) * 32;
            const bool has_res = a.res != nullptr;
            if (has_res) stage_residual_block<8, DEPI_PITCH>(region, a.res, mrow0, n0, a.M, a.N, lane);
#pragma unroll
            for (int ip = 0; ip < 2; ++ip) {
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int nl = ip * 32 + 8 * qq + 4 * kh;
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    float v[4] = {out[ip][jj][4 * qq + 0], out[ip][jj][4 * qq + 1], out[ip][jj][4 * qq + 2],
                                  out[ip][jj][4 * qq + 3]};
                    if (has_res) {
                        float rv[4];
                        staged_residual4(region, r * DEPI_PITCH + nl * 2, rv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += rv[e];
                    }
                    const h4 hv = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
                    *reinterpret_cast<h4 *>(region + r * DEPI_PITCH + nl * 2) = hv;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int it = 0; it < 4; ++it) {  // 32 rows x 8 chunks of 16 bytes
                const int idx = it * 64 + lane;
                const int row = idx >> 3, ch = idx & 7;
                const uint4 v = *reinterpret_cast<const uint4 *>(region + row * DEPI_PITCH + ch * 16);
                const int mm = mrow0 + row, nn = n0 + ch * 8;
                if (mm < a.M && nn < a.N) *reinterpret_cast<uint4 *>(a.y + (size_t)mm * a.N + nn) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        return;
    }
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
        const int m = mt * DBM + (keep + jj) * 32 + r;
        if (m >= a.M) continue;
#pragma unroll
        for (int ip = 0; ip < 2; ++ip)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int n = n0 + ip * 32 + 8 * (e >> 2) + 4 * kh + (e & 3);
                if (n < a.N) {
                    float v = out[ip][jj][e];
                    if (a.res) v += (float)a.res[(size_t)m * a.N + n];
                    a.y[(size_t)m * a.N + n] = (_Float16)v;
                }
            }
    }
}

template <bool PC>
hipError_t launch_direct(GemmF16Args a, int M, hipStream_t st) {
    if (const hipError_t e = allow_dynamic_lds<gemm_f16_w4_direct_kernel<PC>>(kDirectLdsBytes); e != hipSuccess) return e;
    a.n_tiles = (a.N + DBN - 1) / DBN;
    a.m_tiles = (M + DBM - 1) / DBM;
    gemm_f16_w4_direct_kernel<PC><<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 512, kDirectLdsBytes, st>>>(a);
    return hipGetLastError();
}

template <bool PC, bool W8 = false>
hipError_t launch_fallback(GemmF16Args a, int M, hipStream_t st) {
    if (const hipError_t e = allow_dynamic_lds<gemm_f16_w4_kernel<PC, W8>>(kLdsBytes); e != hipSuccess) return e;
    a.n_tiles = (a.N + BN - 1) / BN;
    a.m_tiles = (M + BM - 1) / BM;
    gemm_f16_w4_kernel<PC, W8><<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, kLdsBytes, st>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f16(const Geometry &g, const void *packed, const void *x, int M, void *y,
                           const void *residual, int gated_act, int num_cus, hipStream_t st) {
    // only the kernel that converts in registers has the merged gating (int4 formats, K a multiple of 128)
    if (gated_act >= 0 && (!g.pair_half || (g.K % 128) != 0 || g.fmt == kW8C)) return hipErrorNotSupported;
    (void)num_cus;
    GemmF16Args a;
    a.w = static_cast<const uint4 *>(packed);
    a.x = static_cast<const uint4 *>(x);
    a.y = static_cast<_Float16 *>(y);
    a.res = static_cast<const _Float16 *>(residual);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.M = M;
    a.N = g.N;
    a.K = g.K;
    a.KT = g.KT;
    a.rt_stride = g.rt_stride;
    a.n_tiles = a.m_tiles = 0;
    a.gated_act = gated_act;
    if (g.fmt == kW8C) return launch_fallback<true, true>(a, M, st);
    const bool pc = g.fmt == kW4C;
    if ((g.K % 128) == 0 && (tuning().gemm_variant != 9 || gated_act >= 0)) return pc ? launch_direct<true>(a, M, st) : launch_direct<false>(a, M, st);
    return pc ? launch_fallback<true>(a, M, st) : launch_fallback<false>(a, M, st);
}

}  // namespace qfc
