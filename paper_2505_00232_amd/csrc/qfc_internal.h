// Internal declarations shared by the translation units of libqfc.so.
//
// Physical weight layouts (the "weights conversion" of section 3.4 of the
// paper; the layouts themselves are this library's own, chosen for 64-lane
// wavefronts, 16-byte lane loads and the CDNA4 matrix-core operand shapes).
// A wavefront load of 16 B per lane always covers one contiguous KiB "tile" of
// 16 output rows; lane l = (c, q) with c = l % 16 the row inside the tile and
// q = l / 16 a quarter of the tile's k range.  This is exactly the B-operand
// shape of the 16x16 MFMA instructions, so a tile goes from HBM to a matrix
// core without any cross-lane shuffle.
//
// W8C (int8 codes, one fp32 scale per output channel)
//   tile = 16 rows x 64 k; lane (c, q) holds the 16 codes (row c, k = 16q .. 16q+15).
//   Tiles are stored [row tile][k tile].  N is padded to a multiple of 256 and
//   K to a multiple of 256 with zero codes.  The fp32 scales [Np] follow.
//   The 16 bytes of a lane are an int8 MFMA fragment as they are
//   (v_mfma_i32_16x16x64_i8 / 32x32x32), and two fp16 MFMA fragments after
//   conversion (k = 16q + 8j + e for j = 0, 1).
//
// W4G32 (int4 codes, one binary16 scale per 32 consecutive k)
//   weight tile = 16 rows x 128 k (four quantization groups); lane (c, q) holds
//   four dwords, dword j = the eight codes (row c, k = 32 (4t + j) + 8q .. + 7)
//   of tile t: octet q of group j, i.e. one fp16 MFMA B fragment whose whole k
//   range lies inside one quantization group, so the group scale can be applied
//   to the MFMA result.  Codes are stored biased (q + 8); byte i of a dword holds
//   code i in its low nibble and code 4 + i in its high nibble, so that one mask
//   per nibble plane and one byte permute per pair yield k-adjacent binary16
//   pairs.
//   Up to eight weight tiles (1024 k) are followed by one scale tile holding the
//   32 group scales of each of the 16 rows: 16-byte vector p * 16 + c = scales
//   of row c for groups 8p .. 8p+7 of the unit.  A row tile is the sequence
//   [8 tiles][scales][8 tiles][scales]...[last <= 8 tiles][scales].
//   K is padded to a multiple of 128 (codes 8 = zero, scales 0), N to 256.
//
// W4C (int4 codes, one fp32 scale per output channel: the per-channel 4-bit
//   scheme of section 4.2 of the paper)
//   the same 16 rows x 128 k weight tiles as W4G32, stored [row tile][k tile]
//   with no scale tiles in between; the fp32 scales [Np] follow, as for W8C.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/qfc.h"

namespace qfc {

constexpr int kTileRows = 16;
constexpr int kPadN = 256;
constexpr int kMaxDecodeM = 8;

enum Format { kW8C = 0, kW4G32 = 1, kW4C = 2 };

struct Geometry {
    int N, K;    // logical
    int Np, Kp;  // padded
    int RT;      // row tiles holding real rows: ceil(N / 16)
    int RTp;     // Np / 16
    int KT;      // k tiles per row tile (64 k for W8C, 128 k for the int4 formats)
    int KU;      // units of 8 tiles per row tile: ceil(KT / 8)
    int rt_stride;       // KiB tiles per row tile (W4G32: KT + KU, else KT)
    int fmt;
    int pair_half;       // N / 2 for a layer packed with its two branches' row tiles interleaved, else 0
    size_t code_bytes;   // bytes of the code (+ group scale) region
    size_t scale_off;    // W8C, W4C: byte offset of the fp32 scales
    size_t total_bytes;
};

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

inline Geometry make_geometry(int N, int K, int fmt, bool paired = false) {
    Geometry g;
    g.N = N; g.K = K; g.fmt = fmt;
    g.pair_half = paired ? N / 2 : 0;
    g.Np = round_up(N, kPadN);
    g.RT = (N + kTileRows - 1) / kTileRows;
    g.RTp = g.Np / kTileRows;
    if (fmt == kW8C) {
        g.Kp = round_up(K, 256);
        g.KT = g.Kp / 64;
        g.KU = (g.KT + 7) / 8;
        g.rt_stride = g.KT;
        g.code_bytes = (size_t)g.Np * g.Kp;
        g.scale_off = g.code_bytes;
        g.total_bytes = g.code_bytes + (size_t)g.Np * 4;
    } else if (fmt == kW4G32) {
        g.Kp = round_up(K, 128);
        g.KT = g.Kp / 128;
        g.KU = (g.KT + 7) / 8;
        g.rt_stride = g.KT + g.KU;
        g.code_bytes = (size_t)g.RTp * g.rt_stride * 1024;
        g.scale_off = 0;
        g.total_bytes = g.code_bytes;
    } else {
        g.Kp = round_up(K, 128);
        g.KT = g.Kp / 128;
        g.KU = (g.KT + 7) / 8;
        g.rt_stride = g.KT;
        g.code_bytes = (size_t)g.RTp * g.KT * 1024;
        g.scale_off = g.code_bytes;
        g.total_bytes = g.code_bytes + (size_t)g.Np * 4;
    }
    return g;
}

struct GemvPlan {
    int waves;       // wavefronts per workgroup, each owning a range of units
    int row_tiles;   // row tiles a workgroup walks through (shares staged x)
    bool half = false;  // items are half units (four weight tiles)
    bool copy = false;  // token rows staged by direct global -> LDS copies
    int units = 0;      // items per row tile along K
};

// Tunables (set through qfc_tune of qfc_experimental.h by tests and sweeps, read by the planners).
// Each is one relaxed atomic: a launch being planned on another thread reads whole values.
struct Tunable {
    std::atomic<int> v;
    Tunable(int init) : v(init) {}
    operator int() const { return v.load(std::memory_order_relaxed); }
    Tunable &operator=(int x) {
        v.store(x, std::memory_order_relaxed);
        return *this;
    }
};
struct Tuning {
    Tunable gemv_target_waves{0};   // 0: automatic (8192 up to two token rows, 2048 above)
    Tunable gemv_max_row_tiles{0};  // 0: automatic (2 up to two token rows, 4 above)
    Tunable gemm_variant{0};
    Tunable act_quant_rows{0};  // 0: automatic
    Tunable attn_chunks{-1};    // prefill attention, walks cut into chunks: -1 automatic, 0 never, 1 always
    Tunable attn_pair{-1};      // prefill attention, two blocks per workgroup: -1 automatic, 0 never, 1 always
    Tunable gemv_half{-1};      // half-unit items of the decode kernel: -1 automatic, 0 never, 1 where possible
};
Tuning &tuning();

// pro: the prologue fused into the launch (0 none, 1 gated input, 2 merged normalization); -1 for
// the kernels that only take the basic plan
GemvPlan plan_gemv(const Geometry &g, int M, int num_cus, int pro = -1);

// Launchers.  Every one validates nothing (the C ABI layer did) and returns
// the hipError_t of the launch.
hipError_t launch_pack(const Geometry &g, const int8_t *wq, const void *scales, void *packed,
                       hipStream_t st);
hipError_t launch_unpack(const Geometry &g, const void *packed, int8_t *wq, void *scales,
                         hipStream_t st);
// rows ids[0 .. M) of the table as binary16 [M, K]
hipError_t launch_embedding(const Geometry &g, const void *packed, const int32_t *ids, int M, void *y,
                            hipStream_t st);
// Allow kernel Kernel `bytes` of dynamic LDS (above the default limit of 64 KiB): set once per
// kernel and device, from whichever thread gets there first (setting it twice is harmless).
template <auto Kernel>
hipError_t allow_dynamic_lds(size_t bytes) {
    static std::atomic<uint64_t> done{0};  // one bit per device (devices beyond 63 set it every time)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t(1) << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// ---- helpers of the kernels that copy tiles from memory straight into LDS
// Wait until at most N vector-memory operations are outstanding and all LDS operations are done
// (gfx9 s_waitcnt encoding: vmcnt in bits 3:0 and 15:14, lgkmcnt in bits 11:8, expcnt left at its
// maximum).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

// Direct global -> LDS copy of one wavefront: lane l moves 16 bytes from base + lane_offset(l) to
// LDS byte address lds_base + 16 l.  Written as assembly because the compiler, when it knows
// about such a copy, makes every later LDS read wait for ALL outstanding copies (it cannot tell
// ring slots apart), which would serialize a prefetch ring; the kernels place their waits
// themselves.  M0 carries the LDS base (declared as clobbered; nothing else in those kernels uses M0).
__device__ __forceinline__ void copy16_to_lds(const void *base, uint32_t lane_offset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_offset), "s"(base), "s"(lds_base)
                 : "memory", "m0");
}

// ---- per-token int8 quantization steps shared by the kernels that produce quantized activations
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

// Four binary16 values -> four int8 codes in one dword.  The product is rounded to fp32 first and
// then to the nearest integer (ties to even) by adding 1.5 * 2^23, which leaves the two's complement
// code in the low mantissa byte: the same two roundings as rintf(x * inv).  |x * inv| cannot exceed
// 127 by more than two units in the last place, so the clamp to +-127 of the definition never acts.
__device__ __forceinline__ uint32_t quant4(const _Float16 *h, float inv) {
    uint32_t b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma clang fp contract(off)  // a fused multiply-add would round once, not twice
        const float v = (float)h[i] * inv;
        b[i] = __float_as_uint(v + 12582912.0f);
    }
    const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
    return lo | (hi << 16);
}

// Running maximum of |x| over pairs of binary16 values, on the bit patterns with the sign cleared:
// for finite values the order of the magnitudes is the order of these 15-bit integers.
__device__ __forceinline__ us2 fold_abs(us2 acc, uint32_t d) {
    return __builtin_elementwise_max(acc, __builtin_bit_cast(us2, d & 0x7FFF7FFFu));
}

// Gate activations of the fused input act(gate) * x.  Both are g * sigmoid(t): t = g for SiLU,
// t = 2 sqrt(2/pi) (g + 0.044715 g^3) for the tanh form of GELU (0.5 (1 + tanh z) = sigmoid(2 z)).
// Written as t = g (c1 + c3 g^2) with the pair (c1, c3) chosen once per kernel.  EXACT = false
// (decode kernels, where every workgroup repeats the evaluation): fast exponential and the hardware
// reciprocal (1 ulp) in place of an IEEE division; the result is rounded to binary16 anyway.
// EXACT = true (the quantizer of the int8 prefill path, where the rounded value goes on to decide
// an 8-bit code): library exponential and an IEEE division, so that the fp32 value is within a
// few units in the last place of the real one and a code differs from the definition's only when
// the real value lies that close to a rounding boundary.
struct GateCoeffs {
    float c1, c3;
};
__device__ __forceinline__ GateCoeffs gate_coeffs(int act) {
    GateCoeffs c;
    c.c1 = act == QFC_ACT_GELU_TANH ? 1.5957691216f : 1.0f;
    c.c3 = act == QFC_ACT_GELU_TANH ? 1.5957691216f * 0.044715f : 0.0f;
    return c;
}
template <bool EXACT = false>
__device__ __forceinline__ float gate_activation(float g, const GateCoeffs &c) {
    const float t = g * fmaf(c.c3, g * g, c.c1);
    if constexpr (EXACT) return g / (1.0f + expf(-t));
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-t));
}

// Eight binary16 pairs (gate, x) -> eight binary16 values fp16(act(gate) * x): fp32 arithmetic,
// one rounding to binary16.
template <bool EXACT = false>
__device__ __forceinline__ uint4 gated_input8_u4(const uint4 &gate, const uint4 &x, int act) {
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    const half8 g = __builtin_bit_cast(half8, gate), u = __builtin_bit_cast(half8, x);
    const GateCoeffs c = gate_coeffs(act);
    half8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (_Float16)(gate_activation<EXACT>((float)g[e], c) * (float)u[e]);
    return __builtin_bit_cast(uint4, r);
}

// Residual connection merged into the store phase of the prefill kernels (operator fusion,
// section 3.6 of the paper).  Those kernels stage a block of 32 token rows x 8 CH channels of
// binary16 outputs per wavefront in LDS and store it with 16 bytes per lane along n.  The
// residual's block is copied into the same LDS positions with the same access pattern first;
// each lane then adds the four values under its own outputs in fp32, before the one rounding.
template <int CH, int PITCH>
__device__ __forceinline__ void stage_residual_block(char *region, const _Float16 *res, int mrow0, int n0, int M,
                                                     int N, int lane) {
#pragma unroll
    for (int it = 0; it < 32 * CH / 64; ++it) {
        const int idx = it * 64 + lane;
        const int row = idx / CH, ch = idx % CH;
        const int mm = mrow0 + row, nn = n0 + ch * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (mm < M && nn < N) v = *reinterpret_cast<const uint4 *>(res + (size_t)mm * N + nn);
        *reinterpret_cast<uint4 *>(region + row * PITCH + ch * 16) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// the four residual values staged at byte offset `off` of the region, as fp32
__device__ __forceinline__ void staged_residual4(const char *region, int off, float (&r)[4]) {
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    const half4 v = *reinterpret_cast<const half4 *>(region + off);
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = (float)v[e];
}

// Element-wise parts fused with the layer (null pointer = absent), see qfc_fusion_t.
// Rotary embedding, QKV layout transformation and KV-cache append merged into the decode kernel of
// the QKV layer (the M token rows are M sequences at the same position `pos`).
struct RopeOut {
    int d = 0, h_q = 0, h_kv = 0, C = 0, pos = 0;
    const float *table = nullptr;  // [positions][d / 2][2]: cos, sin of pos * base^(-2 i / d)
    void *q = nullptr, *kc = nullptr, *vc = nullptr;  // binary16, layouts of the attention operators
};

struct Fusion {
    const RopeOut *rope = nullptr;   // decode only; y is not written
    const void *gate = nullptr;      // binary16 [M, K]
    int activation = 0;              // QFC_ACT_*
    const void *residual = nullptr;  // binary16 [M, N]
    bool gated_output = false;       // y [M, N/2] = fp16(act(rows [0, N/2)) * rows [N/2, N))
    const void *norm_gamma = nullptr;  // binary16 [K]: the layer's input is rmsnorm(x) * (norm_offset + gamma)
    float norm_eps = 0.0f, norm_offset = 0.0f;
};

hipError_t launch_gemv(const Geometry &g, const void *packed, const void *x, int M, void *y,
                       const Fusion &f, int num_cus, hipStream_t st);
// Decode with 8-bit activations (per-channel weight formats).  src 0: x is binary16 and is
// quantized in the kernel; 1: x is int8 with scales sx.  out_mode 0: binary16 y; 1: int32 sums.
hipError_t launch_gemv_q8(const Geometry &g, const void *packed, const void *x, const float *sx, int src,
                          int M, void *out, int out_mode, int num_cus, hipStream_t st);
// `gate` (binary16 [M, K] or null): the rows quantized are fp16(act(gate) * x).
hipError_t launch_act_quant(const void *x, const void *gate, int act, int M, int K, int8_t *xq, float *sx,
                            int tiled, int Mp, int Kp, int num_cus, hipStream_t st);
// RMS normalization with the residual connection merged in; see qfc_rmsnorm_t.
struct RmsNormArgs {
    const void *x, *residual, *gamma;
    void *h_out, *y;
    int8_t *xq;
    float *sx;
    float eps, gamma_offset;
    int tiled = 0, Mp = 0, Kp = 0;  // tiled output for an int8 prefill layer (see the kernel)
};
hipError_t launch_rmsnorm(const RmsNormArgs &a, int M, int K, int num_cus, hipStream_t st);
// Attention-side operators (see qfc_rope_qkv / qfc_attention).  G = batch * h_kv groups.
constexpr int kAttnMaxSplits = 64;
constexpr int kPrefillMaxChunks = 8;  // chunks a block's walk is cut into at most (prefill, few blocks)
// Bytes of workspace the many-query-rows path needs for G groups of M query rows of d values.
size_t attn_prefill_workspace(int G, int M, int d, int num_cus);
int attn_splits(int G, int n_ctx, int num_cus);
// cos and sin of pos * base^(-2 i / d) for pos < positions, i < d / 2, evaluated in fp64: [positions][d / 2][2] floats
hipError_t launch_rope_table(int d, float base, int positions, float *table, hipStream_t st);
hipError_t launch_rope_qkv(const void *qkv, int B, int S, int h_q, int h_kv, int d, int C, int pos0, float base,
                           void *q_out, void *kc, void *vc, hipStream_t st);
hipError_t launch_attention(const void *q, const void *kc, const void *vc, int G, int S, int g, int d, int C,
                            int n_ctx, void *workspace, void *out, int num_cus, hipStream_t st);
hipError_t launch_retile_xq(const int8_t *xq, int M, int K, int8_t *tiled, int Mp, int Kp, bool int4_order,
                            hipStream_t st);
// out_mode 0: binary16 y with scales; 1: raw int32 accumulators.
// `residual` (binary16 [M, N] or null) is added before the final rounding (out_mode 0 only).
// gated_act (QFC_ACT_* or -1): the layer is packed in pairs (g.pair_half) and y [M, N/2] is
// fp16(act(gate) * other) of the fp32 outputs of the two branches (out_mode 0, no residual).
hipError_t launch_gemm_i8(const Geometry &g, const void *packed, const int8_t *xq_tiled,
                          const float *sx, int M, int Mp, void *out, int out_mode, const void *residual,
                          int gated_act, int num_cus, hipStream_t st);
// Returns hipErrorNotSupported for a gated output when K is not a multiple of 128.
hipError_t launch_gemm_f16(const Geometry &g, const void *packed, const void *x, int M, void *y,
                           const void *residual, int gated_act, int num_cus, hipStream_t st);

}  // namespace qfc
