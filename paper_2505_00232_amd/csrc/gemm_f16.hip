// Prefill product for group-quantized int4 weights on the fp16 matrix cores:
//   y[m,n] = sum_k x[m,k] * (s[n, k/32] * Wq[n,k]),  fp32 accumulation.
// FP16 activations with quantized weights (section 4.2 of the paper), computed
// on matrix units as the compute-bound prefill stage wants (section 3.7).
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
    const uint4 *w;   // packed W4G32 row tiles
    const uint4 *x;   // binary16 [M, K] viewed as 16-byte vectors
    _Float16 *y;
    int M, N, K, KT, rt_stride, n_tiles, m_tiles;
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

__global__ __launch_bounds__(256) void gemm_f16_w4_kernel(GemmF16Args a) {
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

    uint4 wreg[2], xreg[8];
    uint2 sreg[2];
    auto load_stage = [&](int kt) {
        const int u = kt >> 3;
        const int wpos = kt + u;                               // weight tile kt of the row tile
        const int spos = min(8 * u + 8, a.KT) + u;             // scale tile of its unit
        const int soff = (((kt & 7) >> 1) * 16 + c) * 2 + (kt & 1);  // 8-byte index inside it
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            wreg[i] = w_rt[i][(size_t)wpos * 64 + lane];
            sreg[i] = reinterpret_cast<const uint2 *>(w_rt[i] + (size_t)spos * 64)[soff];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int v = tid + 256 * i;
            const int row = mt * BM + (v >> 4);
            const int o = kt * OCT + (v & 15);
            xreg[i] = (row < a.M && o < K8) ? a.x[(size_t)row * K8 + o] : make_uint4(0, 0, 0, 0);
        }
    };

    const int stages = a.KT;
    load_stage(0);
    for (int kt = 0; kt < stages; ++kt) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = (wave + 4 * i) * 16 + c;
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
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int nl = i * 32 + 8 * qq + 4 * (lane >> 5);
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    const h4 hv = {(_Float16)acc[i][j][4 * qq + 0], (_Float16)acc[i][j][4 * qq + 1],
                                   (_Float16)acc[i][j][4 * qq + 2], (_Float16)acc[i][j][4 * qq + 3]};
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
                for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[i][j][4 * qq + e];
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

}  // namespace

hipError_t launch_gemm_f16(const Geometry &g, const void *packed, const void *x, int M, void *y,
                           hipStream_t st) {
    if (g.fmt != kW4G32) return hipErrorNotSupported;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_f16_w4_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    GemmF16Args a;
    a.w = static_cast<const uint4 *>(packed);
    a.x = static_cast<const uint4 *>(x);
    a.y = static_cast<_Float16 *>(y);
    a.M = M;
    a.N = g.N;
    a.K = g.K;
    a.KT = g.KT;
    a.rt_stride = g.rt_stride;
    a.n_tiles = (g.N + BN - 1) / BN;
    a.m_tiles = (M + BM - 1) / BM;
    gemm_f16_w4_kernel<<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, kLdsBytes, st>>>(a);
    return hipGetLastError();
}

}  // namespace qfc
