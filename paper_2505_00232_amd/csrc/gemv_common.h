// Device-side pieces shared by the decode kernels (one launch per layer, and the persistent
// kernel that runs a chain of layers): code conversion, the staging of the token rows in LDS and
// the argument block of one layer.
#pragma once

#include "qfc_internal.h"

namespace qfc {
namespace gemv_detail {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// Eight biased int4 codes of one dword -> eight binary16 values, k ascending,
// exactly.  A byte permute puts a code byte under the high byte 0x64:
// 0x6400 | u is 1024 + u and 0x6400 | (u << 4) is 1024 + 16 u, both exact in
// binary16, as are the subtraction of 1032 and the fused (x / 16 - 72).
// (Plain C only: hand-placed VALU instructions next to MFMAs would escape the
// compiler's hazard tracking.)
__device__ __forceinline__ v8h dequant8(uint32_t w) {
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t lo = w & 0x0F0F0F0Fu, hi = w & 0xF0F0F0F0u;
    const h2 p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u)) - c1032;
    const h2 p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u)) - c1032;
    const h2 p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u)) * c16th - c72;
    const h2 p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u)) * c16th - c72;
    const u32x4 r = {as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3)};
    return __builtin_bit_cast(v8h, r);
}

// Eight int8 codes (two dwords) -> eight binary16 values, exactly: flipping the
// sign bit gives b + 128 in [0, 255]; 0x64 in the high byte makes 1024 + that.
__device__ __forceinline__ v8h dequant_i8x8(uint32_t lo, uint32_t hi) {
    const h2 c1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
    const uint32_t a = lo ^ 0x80808080u, b = hi ^ 0x80808080u;
    const h2 p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, a, 0x04010400u)) - c1152;
    const h2 p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, a, 0x04030402u)) - c1152;
    const h2 p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, b, 0x04010400u)) - c1152;
    const h2 p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, b, 0x04030402u)) - c1152;
    const u32x4 r = {as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3)};
    return __builtin_bit_cast(v8h, r);
}

__device__ __forceinline__ u32x4 gated_input8(const u32x4 &gate, const u32x4 &x, int act) {
    return __builtin_bit_cast(u32x4, gated_input8_u4(__builtin_bit_cast(uint4, gate), __builtin_bit_cast(uint4, x), act));
}

// eight binary16 pairs (weight, x) -> eight binary16 values fp16(x * (offset + weight))
__device__ __forceinline__ u32x4 weighted_input8(const u32x4 &w, const u32x4 &x, float offset) {
    const v8h wv = __builtin_bit_cast(v8h, w), xv = __builtin_bit_cast(v8h, x);
    v8h r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (_Float16)((float)xv[e] * (offset + (float)wv[e]));
    return __builtin_bit_cast(u32x4, r);
}

struct GemvArgs {
    const u32x4 *packed;
    const u32x4 *x;     // binary16 [M, K] as 16-byte vectors (8 values)
    const u32x4 *gate;  // prologue 1: binary16 [M, K], the layer's input is fp16(act(gate) * x);
                        // prologue 2: binary16 [K], the weight of the merged RMS normalization
    float norm_eps, norm_offset;  // prologue 2
    const _Float16 *res;  // binary16 [M, N] added before the final rounding, or null
    int act;            // QFC_ACT_* of the gate
    _Float16 *y;        // [M, N]
    const float *sw;    // per-channel scales [Np] (W8C, W4C)
    int N, K, RT, KT, KU, rt_stride;
    int row_tiles;           // R: row tiles per workgroup
    int rt_step;             // distance between a workgroup's row tiles (1; RT / 2 for a gated output)
    int gated_out;           // 1: rows [0, N/2) are the gate, rows [N/2, N) the other branch; y is [M, N/2]
    int units_q, units_rem;  // KU = units_q * waves + units_rem
};

// LDS view of one wavefront's staged activations: vector (slot * M + m).
// int4 unit: 1024 k = 128 octets, slot = octet index (4 * group + q).
// W8C unit:   512 k =  64 octets, slot = tile * 8 + j * 4 + q for octet 2q + j of the tile.
// Prologues.  PRO = 1: the gate branch travels with x and the two are merged on the way into LDS (operator
// fusion, section 3.6 of the paper: element-wise operators of two branches merged into the
// fully connected operator).  PRO = 2: RMS normalization merged into the layer: normalizing scales
// a row by one number rs, which commutes with the product, so the row goes into LDS multiplied by
// the normalization weight only and the output is multiplied by rs at the end; every workgroup
// computes the rows' sums of squares for itself (one pass over x).
template <int M, int FMT, int PRO>
struct XStage {
    static constexpr int OCT = FMT == kW8C ? 64 : 128;  // octets per unit
    static constexpr int XV = M * OCT / 64;               // 16-byte vectors per lane per unit
    u32x4 v[XV];
    u32x4 g[PRO ? XV : 1];

    // global -> registers (zeros beyond K)
    __device__ __forceinline__ void load(const GemvArgs &a, int unit, int lane) {
        const int K8 = a.K / 8;
        const int o_base = unit * OCT;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = i * 64 + lane;
            const int m = p / OCT, o = p % OCT;
            const u32x4 zero = {0, 0, 0, 0};
            v[i] = o_base + o < K8 ? a.x[(size_t)m * K8 + o_base + o] : zero;
            if (PRO == 1) g[i] = o_base + o < K8 ? a.gate[(size_t)m * K8 + o_base + o] : zero;
            if (PRO == 2) g[i] = o_base + o < K8 ? a.gate[o_base + o] : zero;
        }
    }
    // registers -> this wavefront's LDS region, A-operand order
    __device__ __forceinline__ void store(u32x4 *lds, int lane, int act, float offset) const {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = i * 64 + lane;
            const int m = p / OCT, o = p % OCT;
            int slot = o;
            if (FMT == kW8C) slot = (o & ~7) | ((o & 1) << 2) | ((o >> 1) & 3);
            lds[slot * M + m] = PRO == 1 ? gated_input8(g[i], v[i], act) : PRO == 2 ? weighted_input8(g[i], v[i], offset) : v[i];
        }
    }
};

// The argument block of one layer for plan p (prologue pointer: the gate; the caller replaces it
// by the normalization weight for a merged RMS normalization).
inline GemvArgs make_gemv_args(const Geometry &g, const void *packed, const void *x, void *y, const Fusion &f,
                               const GemvPlan &p) {
    GemvArgs a;
    a.packed = static_cast<const u32x4 *>(packed);
    a.x = static_cast<const u32x4 *>(x);
    a.gate = static_cast<const u32x4 *>(f.gate);
    a.res = static_cast<const _Float16 *>(f.residual);
    a.act = f.activation;
    a.y = static_cast<_Float16 *>(y);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.N = g.N;
    a.K = g.K;
    a.RT = g.RT;
    a.KT = g.KT;
    a.KU = g.KU;
    a.rt_stride = g.rt_stride;
    a.row_tiles = p.row_tiles;
    a.rt_step = f.gated_output ? g.RT / 2 : 1;
    a.gated_out = f.gated_output ? 1 : 0;
    a.units_q = g.KU / p.waves;
    a.units_rem = g.KU % p.waves;
    a.norm_eps = f.norm_eps;
    a.norm_offset = f.norm_offset;
    return a;
}

}  // namespace gemv_detail
}  // namespace qfc
