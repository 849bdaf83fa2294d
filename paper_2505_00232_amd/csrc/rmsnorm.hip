// RMS normalization with the residual connection and the following quantization
// merged into one kernel (operator fusion, section 3.6 of the paper and the
// right half of its figure: residual connection and element-wise operators
// merged with a hand-written RMS normalization operator).  Per token row:
//   h = fp16(x + residual)                      (the residual stream as it is stored; h = x without one)
//   y[k] = fp16(h[k] * rs * (gamma_offset + gamma[k])),  rs = 1 / sqrt(mean_k h^2 + eps)   in fp32
//   optionally (xq, sx) = the per-token int8 quantization of y, the input of the next layer.
// Any of h, y, (xq, sx) is written if its pointer is given.
//
// Mapping as in the activation quantization kernel: a workgroup of 2 ROWS wavefronts takes ROWS
// token rows; a lane holds 16 consecutive k of one row per step and keeps the row in registers
// between the reductions (K <= 14336), so x and the residual are read once.
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

struct RmsDev {
    const uint4 *x, *res, *gamma;
    uint4 *h_out, *y, *xq;
    float *sx;
    float eps, goff;
    int M, K;
    // tiled != 0: xq / sx are the tiled activations and scales of an int8 prefill layer (see the
    // activation quantization kernel: 1 = order of 8-bit weights, 2 = order of 4-bit weights), padded
    // with zeros to [Mp, Kp]; the grid then covers Mp rows
    int tiled, Mp, Kp;
};

template <int ROWS>
__global__ __launch_bounds__(128 * ROWS) void rmsnorm_kernel(RmsDev a) {
    constexpr int T = 16 / ROWS;  // tiles of 64 k per wavefront instruction
    constexpr int NW = 2 * ROWS;  // wavefronts; NW * T = 32 tiles per step
    constexpr int KEEP = 7;       // steps kept in registers: 7 * 2048 = 14336 k
    __shared__ float part[2][NW][ROWS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane % ROWS, q = (lane / ROWS) & 3, t = lane / (4 * ROWS);
    const int m = blockIdx.x * ROWS + c;
    const bool real = m < a.M;
    const int K = a.K;
    const int steps = ((K + 63) / 64 + 31) / 32;

    uint4 keep[KEEP][2];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        if (i < steps) {
            const int k0 = (T * (NW * i + wave) + t) * 64 + q * 16;
            const bool in = real && k0 < K;
            const size_t off = in ? (size_t)m * (K / 8) + k0 / 8 : 0;
            uint4 v0 = a.x[off], v1 = a.x[off + 1];
            if (a.res) {
                const uint4 r0 = a.res[off], r1 = a.res[off + 1];
                v0 = __builtin_bit_cast(uint4, __builtin_bit_cast(h8, v0) + __builtin_bit_cast(h8, r0));
                v1 = __builtin_bit_cast(uint4, __builtin_bit_cast(h8, v1) + __builtin_bit_cast(h8, r1));
            }
            if (!in) v0 = v1 = make_uint4(0, 0, 0, 0);
            if (a.h_out && in) {
                a.h_out[off] = v0;
                a.h_out[off + 1] = v1;
            }
            keep[i][0] = v0;
            keep[i][1] = v1;
            const h8 h0 = __builtin_bit_cast(h8, v0), h1 = __builtin_bit_cast(h8, v1);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ss = fmaf((float)h0[e], (float)h0[e], ss);
                ss = fmaf((float)h1[e], (float)h1[e], ss);
            }
        }
    }
#pragma unroll
    for (int off = ROWS; off < 64; off <<= 1) ss += __shfl_xor(ss, off, 64);
    if (lane < ROWS) part[0][wave][lane] = ss;
    __syncthreads();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) tot += part[0][w][c];
    const float rs = 1.0f / sqrtf(tot / (float)K + a.eps);

    // y replaces h in the registers
    us2 amax = {0, 0};
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        if (i < steps) {
            const int k0 = (T * (NW * i + wave) + t) * 64 + q * 16;
            const bool in = real && k0 < K;
            const size_t goff = k0 < K ? k0 / 8 : 0;
            const uint4 gv[2] = {a.gamma[goff], a.gamma[goff + 1]};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const h8 h = __builtin_bit_cast(h8, keep[i][j]), g = __builtin_bit_cast(h8, gv[j]);
                h8 y;
#pragma unroll
                for (int e = 0; e < 8; ++e) y[e] = (_Float16)(((float)h[e] * rs) * (a.goff + (float)g[e]));
                keep[i][j] = in ? __builtin_bit_cast(uint4, y) : make_uint4(0, 0, 0, 0);
            }
            if (a.y && in) {
                const size_t off = (size_t)m * (K / 8) + k0 / 8;
                a.y[off] = keep[i][0];
                a.y[off + 1] = keep[i][1];
            }
            amax = fold_abs(fold_abs(fold_abs(fold_abs(amax, keep[i][0].x), keep[i][0].y), keep[i][0].z), keep[i][0].w);
            amax = fold_abs(fold_abs(fold_abs(fold_abs(amax, keep[i][1].x), keep[i][1].y), keep[i][1].z), keep[i][1].w);
        }
    }
    if (!a.xq) return;

    // per-token int8 quantization of y (the steps of the activation quantization kernel)
    const unsigned short top = amax.x > amax.y ? amax.x : amax.y;
    float am = (float)__builtin_bit_cast(_Float16, top);
#pragma unroll
    for (int off = ROWS; off < 64; off <<= 1) am = fmaxf(am, __shfl_xor(am, off, 64));
    if (lane < ROWS) part[1][wave][lane] = am;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) am = fmaxf(am, part[1][w][c]);
    float scale = 0.0f, inv = 0.0f;
    if (am != 0.0f) {
        scale = am / 127.0f;
        inv = 127.0f / am;
    }
    if (wave == 0 && lane < ROWS && (real || a.tiled)) a.sx[m] = scale;
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        if (i < steps) {
            const int kt = T * (NW * i + wave) + t;
            const int k0 = kt * 64 + q * 16;
            const bool in = real && k0 < K;
            if (!in && !(a.tiled && kt * 64 < a.Kp)) continue;
            const h8 h0 = __builtin_bit_cast(h8, keep[i][0]), h1 = __builtin_bit_cast(h8, keep[i][1]);  // (zeros outside the row)
            _Float16 v[16];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[e] = h0[e];
                v[8 + e] = h1[e];
            }
            const uint4 out = make_uint4(quant4(v, inv), quant4(v + 4, inv), quant4(v + 8, inv), quant4(v + 12, inv));
            if (a.tiled == 2) {
                uint2 *dst = reinterpret_cast<uint2 *>(a.xq + ((size_t)(m >> 4) * (a.Kp / 64) + kt) * 64 + (m & 15)) + (q >> 1);
                dst[(2 * (q & 1)) * 16 * 2] = make_uint2(out.x, out.y);
                dst[(2 * (q & 1) + 1) * 16 * 2] = make_uint2(out.z, out.w);
            } else if (a.tiled) {
                a.xq[((size_t)(m >> 4) * (a.Kp / 64) + kt) * 64 + q * 16 + (m & 15)] = out;
            } else {
                a.xq[(size_t)m * (K / 16) + kt * 4 + q] = out;
            }
        }
    }
}

}  // namespace

// K a multiple of 32, at most 14336 (checked by the caller).
hipError_t launch_rmsnorm(const RmsNormArgs &h, int M, int K, int num_cus, hipStream_t st) {
    RmsDev a;
    a.x = static_cast<const uint4 *>(h.x);
    a.res = static_cast<const uint4 *>(h.residual);
    a.gamma = static_cast<const uint4 *>(h.gamma);
    a.h_out = static_cast<uint4 *>(h.h_out);
    a.y = static_cast<uint4 *>(h.y);
    a.xq = reinterpret_cast<uint4 *>(h.xq);
    a.sx = h.sx;
    a.eps = h.eps;
    a.goff = h.gamma_offset;
    a.M = M;
    a.K = K;
    a.tiled = h.tiled;
    a.Mp = h.Mp;
    a.Kp = h.Kp;
    const int rows_total = h.tiled ? h.Mp : M;  // (Mp is a multiple of 16)
    const int rows = rows_total >= 16 * num_cus ? 8 : rows_total >= 8 * num_cus ? 4 : 2;
    const unsigned grid = (unsigned)((rows_total + rows - 1) / rows);
    if (rows == 8)
        rmsnorm_kernel<8><<<grid, 1024, 0, st>>>(a);
    else if (rows == 4)
        rmsnorm_kernel<4><<<grid, 512, 0, st>>>(a);
    else
        rmsnorm_kernel<2><<<grid, 256, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace qfc
