// Prefill product for group-quantized int4 weights on the fp16 matrix cores:
//   y[m,n] = sum_k x[m,k] * (s[n, k/32] * Wq[n,k]),  fp32 accumulation.
// FP16 activations with quantized weights (section 4.2 of the paper), computed
// on matrix units as the compute-bound prefill stage wants (section 3.7).
//
// Per K stage of 64: every thread loads one 16-byte vector of packed codes
// (32 codes of one row and group) plus that group's scale, dequantizes in
// registers (exact int -> binary16, then one binary16 multiply by the scale)
// and writes four 16-byte binary16 vectors to LDS.  Activations are copied
// to LDS as they are.  LDS holds both tiles chunk-major ([k/8][row], 16 B
// each), so an MFMA fragment (32 rows x 16 k, lane = row + 32 * (k/8)) is two
// runs of 512 contiguous bytes; the activation tile has a one-vector pad per
// chunk so that its transposing writes are conflict free as well.
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BN = 128, BM = 128, BK = 64;
constexpr int CH = BK / 8;       // 16-byte chunks (8 binary16) per row per stage
constexpr int LDW = BN;          // vectors per chunk, weights
constexpr int LDX = BM + 1;      // vectors per chunk, activations (padded)

struct GemmF16Args {
    const uint4 *w;   // packed W4G32 units
    const uint4 *x;   // binary16 [M, K] viewed as 16-byte vectors
    _Float16 *y;
    int M, N, K, G8, n_tiles, m_tiles;
};

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// eight biased codes -> eight scaled binary16 values, k ascending
__device__ __forceinline__ uint4 dequant8_scaled(uint32_t w, h2 s) {
    const uint32_t magic = 0x64006400u;
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t ws = w >> 8;
    const h2 p0 = (as_h2((w & 0x000F000Fu) | magic) - c1032) * s;
    const h2 p1 = (as_h2((w & 0x00F000F0u) | magic) * c16th - c72) * s;
    const h2 p2 = (as_h2((ws & 0x000F000Fu) | magic) - c1032) * s;
    const h2 p3 = (as_h2((ws & 0x00F000F0u) | magic) * c16th - c72) * s;
    return make_uint4(as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3));
}

__global__ __launch_bounds__(256) void gemm_f16_w4_kernel(GemmF16Args a) {
    __shared__ uint4 lds_w[CH * LDW];
    __shared__ uint4 lds_x[CH * LDX];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;

    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles;
    const int mt = logical % a.m_tiles;

    // weights: thread -> (row block of the tile, group of the stage, row)
    const int w_rbl = tid >> 7, w_jj = (tid >> 6) & 1, w_r = tid & 63;
    const uint4 *w_rb = a.w + (size_t)(nt * (BN / 64) + w_rbl) * a.G8 * kW4UnitVecs;
    // activations: thread -> 4 vectors (row = v / 8, chunk = v % 8)
    const int K8 = a.K / 8;

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4 wreg, xreg[4];
    uint32_t sreg;
    auto load_stage = [&](int kt) {
        const int g = 2 * kt + w_jj;  // group index along K
        const uint4 *unit = w_rb + (size_t)(g >> 3) * kW4UnitVecs;
        wreg = unit[(g & 7) * 64 + w_r];
        sreg = reinterpret_cast<const uint16_t *>(unit + 8 * 64 + w_r)[g & 7];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + 256 * i;
            const int row = mt * BM + (v >> 3);
            const int c = kt * CH + (v & 7);
            xreg[i] = (row < a.M && c < K8) ? a.x[(size_t)row * K8 + c] : make_uint4(0, 0, 0, 0);
        }
    };

    const int stages = (a.K + BK - 1) / BK;
    load_stage(0);
    for (int kt = 0; kt < stages; ++kt) {
        __syncthreads();
        {
            const _Float16 sh = __builtin_bit_cast(_Float16, (uint16_t)sreg);
            const h2 s = {sh, sh};
            const int row = w_rbl * 64 + w_r;
            lds_w[(4 * w_jj + 0) * LDW + row] = dequant8_scaled(wreg.x, s);
            lds_w[(4 * w_jj + 1) * LDW + row] = dequant8_scaled(wreg.y, s);
            lds_w[(4 * w_jj + 2) * LDW + row] = dequant8_scaled(wreg.z, s);
            lds_w[(4 * w_jj + 3) * LDW + row] = dequant8_scaled(wreg.w, s);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int v = tid + 256 * i;
                lds_x[(v & 7) * LDX + (v >> 3)] = xreg[i];
            }
        }
        __syncthreads();
        if (kt + 1 < stages) load_stage(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            v8h fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fa[i] = __builtin_bit_cast(v8h, lds_w[c * LDW + wn * 64 + i * 32 + (lane & 31)]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fb[j] = __builtin_bit_cast(v8h, lds_x[c * LDX + wm * 64 + j * 32 + (lane & 31)]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    const bool vec_ok = (a.N % 4) == 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int m = mt * BM + wm * 64 + j * 32 + (lane & 31);
        if (m >= a.M) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = nt * BN + wn * 64 + i * 32 + 8 * q + 4 * (lane >> 5);
                if (n >= a.N) continue;
                _Float16 *y = a.y + (size_t)m * a.N + n;
                _Float16 h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = (_Float16)acc[i][j][4 * q + e];
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
    GemmF16Args a;
    a.w = static_cast<const uint4 *>(packed);
    a.x = static_cast<const uint4 *>(x);
    a.y = static_cast<_Float16 *>(y);
    a.M = M;
    a.N = g.N;
    a.K = g.K;
    a.G8 = g.Kp / 256;
    a.n_tiles = (g.N + BN - 1) / BN;
    a.m_tiles = (M + BM - 1) / BM;
    gemm_f16_w4_kernel<<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace qfc
