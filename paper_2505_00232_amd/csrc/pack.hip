// Weights conversion (section 3.4 of the paper): logical [N, K] quantized codes
// and scales -> the physical layouts described in qfc_internal.h, and back.
// Pure byte shuffling, bit exact.  One thread produces (or consumes) one
// 16-byte vector of the packed form.
#include "qfc_internal.h"

namespace qfc {
namespace {

// ---------------------------------------------------------------- W8C
__global__ __launch_bounds__(256) void pack_w8c_kernel(const int8_t *__restrict__ wq,
                                                       const float *__restrict__ scales,
                                                       uint4 *__restrict__ packed, float *__restrict__ ps,
                                                       int N, int K, int Np, int Kp) {
    const int KC = Kp / 16;
    const size_t total = (size_t)(Np / 64) * KC * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < (size_t)Np) ps[v] = v < (size_t)N ? scales[v] : 0.0f;
    if (v >= total) return;
    const int r = (int)(v % 64);
    const size_t tile = v / 64;
    const int kc = (int)(tile % KC);
    const int rb = (int)(tile / KC);
    const int n = rb * 64 + r;
    const int k = kc * 16;
    uint4 out = make_uint4(0, 0, 0, 0);
    if (n < N && k < K) out = *reinterpret_cast<const uint4 *>(wq + (size_t)n * K + k);
    packed[v] = out;
}

__global__ __launch_bounds__(256) void unpack_w8c_kernel(const uint4 *__restrict__ packed,
                                                         const float *__restrict__ ps,
                                                         int8_t *__restrict__ wq, float *__restrict__ scales,
                                                         int N, int K, int Np, int Kp) {
    const int KC = Kp / 16;
    const size_t total = (size_t)(Np / 64) * KC * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < (size_t)N) scales[v] = ps[v];
    if (v >= total) return;
    const int r = (int)(v % 64);
    const size_t tile = v / 64;
    const int kc = (int)(tile % KC);
    const int rb = (int)(tile / KC);
    const int n = rb * 64 + r;
    const int k = kc * 16;
    if (n < N && k < K) *reinterpret_cast<uint4 *>(wq + (size_t)n * K + k) = packed[v];
}

// ---------------------------------------------------------------- W4G32
// Eight consecutive codes -> one dword, biased by 8, code e in nibble (e>>1)+4*(e&1).
__device__ inline uint32_t pack8(const int8_t *c) {
    uint32_t d = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t u = ((uint32_t)(c[e] + 8)) & 0xFu;
        d |= u << (4 * ((e >> 1) + 4 * (e & 1)));
    }
    return d;
}

__device__ inline void unpack8(uint32_t d, int8_t *c) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t u = (d >> (4 * ((e >> 1) + 4 * (e & 1)))) & 0xFu;
        c[e] = (int8_t)((int)u - 8);
    }
}

__global__ __launch_bounds__(256) void pack_w4g32_kernel(const int8_t *__restrict__ wq,
                                                         const uint16_t *__restrict__ scales,
                                                         uint4 *__restrict__ packed, int N, int K,
                                                         int Np, int Kp) {
    const int G8 = Kp / 256;
    const int Kg = K / 32;
    const size_t total = (size_t)(Np / 64) * G8 * kW4UnitVecs;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= total) return;
    const int r = (int)(v % 64);
    const int j = (int)((v / 64) % 9);
    const size_t unit = v / kW4UnitVecs;
    const int b = (int)(unit % G8);
    const int rb = (int)(unit / G8);
    const int n = rb * 64 + r;
    uint4 out;
    if (j < 8) {
        const int g = b * 8 + j;
        if (n < N && g < Kg) {
            alignas(16) int8_t c[32];
            const uint4 *src = reinterpret_cast<const uint4 *>(wq + (size_t)n * K + (size_t)g * 32);
            *reinterpret_cast<uint4 *>(c) = src[0];
            *reinterpret_cast<uint4 *>(c + 16) = src[1];
            out = make_uint4(pack8(c), pack8(c + 8), pack8(c + 16), pack8(c + 24));
        } else {
            out = make_uint4(0x88888888u, 0x88888888u, 0x88888888u, 0x88888888u);
        }
    } else {
        uint32_t s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = b * 8 + i;
            s[i] = (n < N && g < Kg) ? scales[(size_t)n * Kg + g] : 0u;
        }
        out = make_uint4(s[0] | (s[1] << 16), s[2] | (s[3] << 16), s[4] | (s[5] << 16), s[6] | (s[7] << 16));
    }
    packed[v] = out;
}

__global__ __launch_bounds__(256) void unpack_w4g32_kernel(const uint4 *__restrict__ packed,
                                                           int8_t *__restrict__ wq,
                                                           uint16_t *__restrict__ scales, int N, int K,
                                                           int Np, int Kp) {
    const int G8 = Kp / 256;
    const int Kg = K / 32;
    const size_t total = (size_t)(Np / 64) * G8 * kW4UnitVecs;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= total) return;
    const int r = (int)(v % 64);
    const int j = (int)((v / 64) % 9);
    const size_t unit = v / kW4UnitVecs;
    const int b = (int)(unit % G8);
    const int rb = (int)(unit / G8);
    const int n = rb * 64 + r;
    if (n >= N) return;
    const uint4 in = packed[v];
    if (j < 8) {
        const int g = b * 8 + j;
        if (g >= Kg) return;
        alignas(16) int8_t c[32];
        unpack8(in.x, c);
        unpack8(in.y, c + 8);
        unpack8(in.z, c + 16);
        unpack8(in.w, c + 24);
        uint4 *dst = reinterpret_cast<uint4 *>(wq + (size_t)n * K + (size_t)g * 32);
        dst[0] = *reinterpret_cast<uint4 *>(c);
        dst[1] = *reinterpret_cast<uint4 *>(c + 16);
    } else {
        const uint32_t w[4] = {in.x, in.y, in.z, in.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = b * 8 + i;
            if (g < Kg) scales[(size_t)n * Kg + g] = (uint16_t)((w[i / 2] >> (16 * (i & 1))) & 0xFFFFu);
        }
    }
}

inline unsigned blocks_for(size_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

hipError_t launch_pack(const Geometry &g, const int8_t *wq, const void *scales, void *packed,
                       hipStream_t st) {
    if (g.fmt == kW8C) {
        const size_t total = (size_t)g.RBp * (g.Kp / 16) * 64;
        pack_w8c_kernel<<<blocks_for(total), 256, 0, st>>>(
            wq, static_cast<const float *>(scales), static_cast<uint4 *>(packed),
            reinterpret_cast<float *>(static_cast<char *>(packed) + g.scale_off), g.N, g.K, g.Np, g.Kp);
    } else {
        const size_t total = (size_t)g.RBp * (g.Kp / 256) * kW4UnitVecs;
        pack_w4g32_kernel<<<blocks_for(total), 256, 0, st>>>(
            wq, static_cast<const uint16_t *>(scales), static_cast<uint4 *>(packed), g.N, g.K, g.Np, g.Kp);
    }
    return hipGetLastError();
}

hipError_t launch_unpack(const Geometry &g, const void *packed, int8_t *wq, void *scales,
                         hipStream_t st) {
    if (g.fmt == kW8C) {
        const size_t total = (size_t)g.RBp * (g.Kp / 16) * 64;
        unpack_w8c_kernel<<<blocks_for(total), 256, 0, st>>>(
            static_cast<const uint4 *>(packed),
            reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off), wq,
            static_cast<float *>(scales), g.N, g.K, g.Np, g.Kp);
    } else {
        const size_t total = (size_t)g.RBp * (g.Kp / 256) * kW4UnitVecs;
        unpack_w4g32_kernel<<<blocks_for(total), 256, 0, st>>>(
            static_cast<const uint4 *>(packed), wq, static_cast<uint16_t *>(scales), g.N, g.K, g.Np, g.Kp);
    }
    return hipGetLastError();
}

}  // namespace qfc
