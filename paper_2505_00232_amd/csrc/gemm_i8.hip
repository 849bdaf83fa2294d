// Prefill int8 product and its dequantizing epilogue (section 3.7 of the paper:
// int8 activations x pre-quantized int8 weights with integer instructions, then
// dequantization of the output):
//   acc[m,n] = sum_k xq[m,k] * Wq[n,k]        (int32, exact)
//   y[m,n]   = fp16(float(acc) * sx[m] * sw[n])
//
// Both operands arrive tiled the same way (KiB tiles of 16 rows x 64 k, lane
// (c, q) = 16 codes of row c at k = 16q), so a stage of the K loop is a
// verbatim, fully coalesced copy of KiB tiles into LDS, and an MFMA operand
// fragment (32 rows x 32 k, lane = row + 32 * (k / 16)) is made of runs of 256
// contiguous LDS bytes: bank-conflict free without padding or swizzling.
//
// Workgroup: 256 threads = 4 wavefronts in a 2 x 2 grid over a BN x BM tile
// (weights rows x token rows); each wavefront owns (BN/2) x (BM/2) outputs as
// 32x32 MFMA tiles (v_mfma_i32_32x32x32_i8).  The weights are the row operand
// of the MFMA so that a lane ends up with 4 consecutive n of one token row:
// 8-byte binary16 stores along the contiguous axis of y.
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK = 128;            // k per stage
constexpr int KCH = BK / 16;       // 16-byte chunks per row per stage

struct GemmI8Args {
    const uint4 *w;      // packed weights, tiles [row tile][Kp/64][64]
    const uint4 *x;      // tiled activations, tiles [row tile][Kp/64][64]
    const float *sw;     // [Np]
    const float *sx;     // [Mp] (null for raw accumulators)
    void *out;
    int M, N, Kp, n_tiles, m_tiles;
};

template <int BN, int BM, int OUT_MODE>
__global__ __launch_bounds__(256) void gemm_i8_kernel(GemmI8Args a) {
    constexpr int WN = BN / 2, WM = BM / 2;      // per-wavefront tile
    constexpr int TN = WN / 32, TM = WM / 32;    // 32x32 MFMA tiles per wavefront
    constexpr int W_VECS = BN * KCH, X_VECS = BM * KCH;  // 16-byte vectors per stage
    constexpr int W_LD = W_VECS / 256, X_LD = X_VECS / 256;
    __shared__ uint4 lds_w[W_VECS];
    __shared__ uint4 lds_x[X_VECS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;

    // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs, so
    // give each XCD a contiguous range of logical tiles; the token tiles that
    // share one weight tile are neighbours and hit the same L2.
    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles;
    const int mt = logical % a.m_tiles;
    const int KT = a.Kp / 64;  // k tiles per row tile
    constexpr int KTS = BK / 64;  // k tiles per stage

    // global source of this thread's vectors for stage 0 (LDS vector v = tile * 64 + lane,
    // tile = row tile of the block * KTS + k tile of the stage)
    const uint4 *wsrc[W_LD];
    const uint4 *xsrc[X_LD];
#pragma unroll
    for (int i = 0; i < W_LD; ++i) {
        const int v = tid + 256 * i;
        const int rtl = v / (KTS * 64), ktl = (v / 64) % KTS, ln = v % 64;
        wsrc[i] = a.w + ((size_t)(nt * (BN / 16) + rtl) * KT + ktl) * 64 + ln;
    }
#pragma unroll
    for (int i = 0; i < X_LD; ++i) {
        const int v = tid + 256 * i;
        const int rtl = v / (KTS * 64), ktl = (v / 64) % KTS, ln = v % 64;
        xsrc[i] = a.x + ((size_t)(mt * (BM / 16) + rtl) * KT + ktl) * 64 + ln;
    }

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    uint4 wreg[W_LD], xreg[X_LD];
#pragma unroll
    for (int i = 0; i < W_LD; ++i) wreg[i] = wsrc[i][0];
#pragma unroll
    for (int i = 0; i < X_LD; ++i) xreg[i] = xsrc[i][0];

    const int stages = a.Kp / BK;
    for (int kt = 0; kt < stages; ++kt) {
        __syncthreads();  // previous stage fully consumed
#pragma unroll
        for (int i = 0; i < W_LD; ++i) lds_w[tid + 256 * i] = wreg[i];
#pragma unroll
        for (int i = 0; i < X_LD; ++i) lds_x[tid + 256 * i] = xreg[i];
        __syncthreads();
        if (kt + 1 < stages) {
            const size_t adv = (size_t)(kt + 1) * KTS * 64;
#pragma unroll
            for (int i = 0; i < W_LD; ++i) wreg[i] = wsrc[i][adv];
#pragma unroll
            for (int i = 0; i < X_LD; ++i) xreg[i] = xsrc[i][adv];
        }
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            const int kc = 2 * ks + (lane >> 5);           // 16-code chunk inside the stage
            const int koff = (kc >> 2) * 64 + (kc & 3) * 16;  // k tile and quarter
            v4i fa[TN], fb[TM];
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                const int row = wn * WN + i * 32 + (lane & 31);
                fa[i] = __builtin_bit_cast(v4i, lds_w[(row >> 4) * (KTS * 64) + koff + (row & 15)]);
            }
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int row = wm * WM + j * 32 + (lane & 31);
                fb[j] = __builtin_bit_cast(v4i, lds_x[(row >> 4) * (KTS * 64) + koff + (row & 15)]);
            }
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // epilogue: lane holds token m = .. + lane % 32 and, per group of four
    // accumulator registers, four consecutive n.
    const bool vec_ok = (a.N % 4) == 0;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = mt * BM + wm * WM + j * 32 + (lane & 31);
        if (m >= a.M) continue;
        float sxm = 1.0f;
        if (OUT_MODE == 0) sxm = a.sx[m];
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = nt * BN + wn * WN + i * 32 + 8 * q + 4 * (lane >> 5);
                if (n >= a.N) continue;
                if (OUT_MODE == 0) {
                    _Float16 *y = static_cast<_Float16 *>(a.out) + (size_t)m * a.N + n;
                    const float4 s = *reinterpret_cast<const float4 *>(a.sw + n);
                    const float sv[4] = {s.x, s.y, s.z, s.w};
                    _Float16 h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = (_Float16)((float)acc[i][j][4 * q + e] * sxm * sv[e]);
                    if (vec_ok) {
                        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                        *reinterpret_cast<h4 *>(y) = h4{h[0], h[1], h[2], h[3]};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < a.N) y[e] = h[e];
                    }
                } else {
                    int32_t *o = static_cast<int32_t *>(a.out) + (size_t)m * a.N + n;
                    if (vec_ok) {
                        *reinterpret_cast<int4 *>(o) = make_int4(acc[i][j][4 * q], acc[i][j][4 * q + 1],
                                                                 acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < a.N) o[e] = acc[i][j][4 * q + e];
                    }
                }
            }
        }
    }
}

template <int BN, int BM>
hipError_t launch_tile(const GemmI8Args &args, int out_mode, hipStream_t st) {
    GemmI8Args a = args;
    a.n_tiles = (a.N + BN - 1) / BN;
    a.m_tiles = (a.M + BM - 1) / BM;
    const dim3 grid((unsigned)(a.n_tiles * a.m_tiles));
    if (out_mode == 0)
        gemm_i8_kernel<BN, BM, 0><<<grid, 256, 0, st>>>(a);
    else
        gemm_i8_kernel<BN, BM, 1><<<grid, 256, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_i8(const Geometry &g, const void *packed, const int8_t *xq_tiled,
                          const float *sx, int M, int Mp, void *out, int out_mode, hipStream_t st) {
    (void)Mp;
    GemmI8Args a;
    a.w = static_cast<const uint4 *>(packed);
    a.x = reinterpret_cast<const uint4 *>(xq_tiled);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.sx = sx;
    a.out = out;
    a.M = M;
    a.N = g.N;
    a.Kp = g.Kp;
    a.n_tiles = a.m_tiles = 0;
    return launch_tile<128, 128>(a, out_mode, st);
}

}  // namespace qfc
