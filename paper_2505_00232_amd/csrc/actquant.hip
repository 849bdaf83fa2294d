// Activation quantization kernel of the prefill stage (section 3.7 of the
// paper: float activations -> 8-bit integers plus their quantization
// parameter).  One scale per token row, symmetric, in fp32 exactly as follows:
//   a = max_k |x|;  sx = a / 127;  inv = 127 / a;  xq = clamp(rne(x * inv), +-127)
// with IEEE division, one rounding for the product and round-half-to-even.
// An all-zero row gives sx = 0 and xq = 0.
//
// Output either row-major [M, K] (the public entry point) or tiled for the
// int8 product exactly like the int8 weights: KiB tiles of 16 token rows x 64 k,
// lane (c, q) of a tile = the 16 codes (row c, k = 16q .. 16q+15), tiles stored
// [row tile][k tile], padded with zeros to [Mp, Kp].
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ uint32_t quant4(const float *v, float inv) {
    uint32_t d = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float r = rintf(v[i] * inv);
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        d |= ((uint32_t)(int)r & 0xFFu) << (8 * i);
    }
    return d;
}

template <bool kTiled>
__global__ __launch_bounds__(256) void act_quant_kernel(const uint4 *__restrict__ x, int M, int K,
                                                        uint4 *__restrict__ xq, float *__restrict__ sx,
                                                        int Kp) {
    __shared__ float wmax[4];
    const int m = blockIdx.x;
    const int tid = threadIdx.x;
    const bool real = m < M;
    float a = 0.0f;
    if (real) {
        const uint4 *row = x + (size_t)m * (K / 8);
        for (int v = tid; v < K / 8; v += 256) {
            const h8 h = __builtin_bit_cast(h8, row[v]);
#pragma unroll
            for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf((float)h[i]));
        }
    }
    a = wave_max(a);
    if ((tid & 63) == 0) wmax[tid >> 6] = a;
    __syncthreads();
    a = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    float scale = 0.0f, inv = 0.0f;
    if (a != 0.0f) {
        scale = a / 127.0f;
        inv = 127.0f / a;
    }
    if (tid == 0) sx[m] = scale;

    const int chunks = (kTiled ? Kp : K) / 16;
    for (int c = tid; c < chunks; c += 256) {
        uint4 out = make_uint4(0, 0, 0, 0);
        if (real && c * 16 < K) {
            const uint4 *src = x + (size_t)m * (K / 8) + c * 2;
            const h8 h0 = __builtin_bit_cast(h8, src[0]);
            const h8 h1 = __builtin_bit_cast(h8, src[1]);
            float v[16];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[i] = (float)h0[i];
                v[8 + i] = (float)h1[i];
            }
            out = make_uint4(quant4(v, inv), quant4(v + 4, inv), quant4(v + 8, inv), quant4(v + 12, inv));
        }
        if (kTiled)
            xq[((size_t)(m >> 4) * (Kp / 64) + (c >> 2)) * 64 + (c & 3) * 16 + (m & 15)] = out;
        else
            xq[(size_t)m * (K / 16) + c] = out;
    }
}

__global__ __launch_bounds__(256) void retile_xq_kernel(const uint4 *__restrict__ xq, int M, int K,
                                                        uint4 *__restrict__ tiled, int Mp, int Kp) {
    const size_t total = (size_t)Mp * (Kp / 16);
    const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int kt = (int)(tile % (Kp / 64));
    const int m = (int)(tile / (Kp / 64)) * 16 + (lane & 15);
    const int c = kt * 4 + (lane >> 4);
    uint4 out = make_uint4(0, 0, 0, 0);
    if (m < M && c * 16 < K) out = xq[(size_t)m * (K / 16) + c];
    tiled[v] = out;
}

}  // namespace

hipError_t launch_act_quant(const void *x, int M, int K, int8_t *xq, float *sx, int tiled, int Mp,
                            int Kp, hipStream_t st) {
    if (tiled)
        act_quant_kernel<true><<<Mp, 256, 0, st>>>(static_cast<const uint4 *>(x), M, K,
                                                   reinterpret_cast<uint4 *>(xq), sx, Kp);
    else
        act_quant_kernel<false><<<M, 256, 0, st>>>(static_cast<const uint4 *>(x), M, K,
                                                   reinterpret_cast<uint4 *>(xq), sx, K);
    return hipGetLastError();
}

hipError_t launch_retile_xq(const int8_t *xq, int M, int K, int8_t *tiled, int Mp, int Kp,
                            hipStream_t st) {
    const size_t total = (size_t)Mp * (Kp / 16);
    retile_xq_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(
        reinterpret_cast<const uint4 *>(xq), M, K, reinterpret_cast<uint4 *>(tiled), Mp, Kp);
    return hipGetLastError();
}

}  // namespace qfc
