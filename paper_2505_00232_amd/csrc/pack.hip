// Weights conversion (section 3.4 of the paper): logical [N, K] quantized codes
// and scales -> the physical layouts described in qfc_internal.h, and back.
// Pure byte shuffling, bit exact.  One thread produces (or consumes) one
// 16-byte vector of the packed form.
#include "qfc_internal.h"

namespace qfc {
namespace {

// Paired packing of a layer that produces the two branches of a gated feed-forward block (rows
// [0, N/2) = gate, rows [N/2, N) = the other branch; operator fusion, section 3.6 of the paper):
// physical row tile 2 t holds gate rows 16 t .. 16 t + 15 and tile 2 t + 1 the other branch's rows
// of the same 16 channels, so that every 32-row MFMA tile of a product holds both branches of its
// channels in the same lanes.  `half` = N / 2 for such a layer (N a multiple of 32), 0 otherwise.
__device__ inline int logical_row(int p, int N, int half) {
    if (!half || p >= N) return p;
    const int tp = p >> 4;
    return (tp & 1) * half + (tp >> 1) * 16 + (p & 15);
}

// ---------------------------------------------------------------- W8C
__global__ __launch_bounds__(256) void pack_w8c_kernel(const int8_t *__restrict__ wq,
                                                       const float *__restrict__ scales,
                                                       uint4 *__restrict__ packed, float *__restrict__ ps,
                                                       int N, int K, int Np, int KT, int half) {
    const size_t total = (size_t)(Np / 16) * KT * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < (size_t)Np) ps[v] = v < (size_t)N ? scales[logical_row((int)v, N, half)] : 0.0f;
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int kt = (int)(tile % KT);
    const int rt = (int)(tile / KT);
    const int n = logical_row(rt * 16 + (lane & 15), N, half);
    const int k = kt * 64 + (lane >> 4) * 16;
    uint4 out = make_uint4(0, 0, 0, 0);
    if (n < N && k < K) out = *reinterpret_cast<const uint4 *>(wq + (size_t)n * K + k);
    packed[v] = out;
}

__global__ __launch_bounds__(256) void unpack_w8c_kernel(const uint4 *__restrict__ packed,
                                                         const float *__restrict__ ps,
                                                         int8_t *__restrict__ wq, float *__restrict__ scales,
                                                         int N, int K, int Np, int KT, int half) {
    const size_t total = (size_t)(Np / 16) * KT * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < (size_t)N) scales[logical_row((int)v, N, half)] = ps[v];
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int kt = (int)(tile % KT);
    const int rt = (int)(tile / KT);
    const int n = logical_row(rt * 16 + (lane & 15), N, half);
    const int k = kt * 64 + (lane >> 4) * 16;
    if (n < N && k < K) *reinterpret_cast<uint4 *>(wq + (size_t)n * K + k) = packed[v];
}

// ---------------------------------------------------------------- W4G32
// Eight consecutive codes -> one dword, biased by 8: byte i holds code i in its
// low nibble and code 4 + i in its high nibble.
__device__ inline uint32_t pack8(const int8_t *c) {
    uint32_t d = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t u = ((uint32_t)(c[e] + 8)) & 0xFu;
        d |= u << (8 * (e & 3) + 4 * (e >> 2));
    }
    return d;
}

__device__ inline void unpack8(uint32_t d, int8_t *c) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t u = (d >> (8 * (e & 3) + 4 * (e >> 2))) & 0xFu;
        c[e] = (int8_t)((int)u - 8);
    }
}

// Position `pos` inside a row tile's sequence -> weight tile index (>= 0) or
// scale tile of unit u (returned as -1 - u).
__device__ inline int classify(int pos, int KT) {
    const int u = pos / 9;
    const int s = pos % 9;
    const int nt = min(8, KT - 8 * u);
    return s < nt ? 8 * u + s : -1 - u;
}

__global__ __launch_bounds__(256) void pack_w4g32_kernel(const int8_t *__restrict__ wq,
                                                         const uint16_t *__restrict__ scales,
                                                         uint4 *__restrict__ packed, int N, int K,
                                                         int RTp, int KT, int stride, int half) {
    const int Kg = K / 32;
    const size_t total = (size_t)RTp * stride * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int pos = (int)(tile % stride);
    const int rt = (int)(tile / stride);
    const int what = classify(pos, KT);
    uint4 out;
    if (what >= 0) {
        const int n = logical_row(rt * 16 + (lane & 15), N, half);
        const int q = lane >> 4;
        uint32_t d[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int g = 4 * what + j;
            if (n < N && g < Kg) {
                alignas(8) int8_t c[8];
                *reinterpret_cast<uint2 *>(c) =
                    *reinterpret_cast<const uint2 *>(wq + (size_t)n * K + (size_t)g * 32 + 8 * q);
                d[j] = pack8(c);
            } else {
                d[j] = 0x88888888u;
            }
        }
        out = make_uint4(d[0], d[1], d[2], d[3]);
    } else {
        const int u = -1 - what;
        const int n = logical_row(rt * 16 + (lane & 15), N, half);
        const int p = lane >> 4;
        uint32_t s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = 32 * u + 8 * p + i;
            s[i] = (n < N && g < Kg) ? scales[(size_t)n * Kg + g] : 0u;
        }
        out = make_uint4(s[0] | (s[1] << 16), s[2] | (s[3] << 16), s[4] | (s[5] << 16), s[6] | (s[7] << 16));
    }
    packed[v] = out;
}

__global__ __launch_bounds__(256) void unpack_w4g32_kernel(const uint4 *__restrict__ packed,
                                                           int8_t *__restrict__ wq,
                                                           uint16_t *__restrict__ scales, int N, int K,
                                                           int RTp, int KT, int stride, int half) {
    const int Kg = K / 32;
    const size_t total = (size_t)RTp * stride * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int pos = (int)(tile % stride);
    const int rt = (int)(tile / stride);
    const int what = classify(pos, KT);
    const int n = logical_row(rt * 16 + (lane & 15), N, half);
    if (n >= N) return;
    const uint4 in = packed[v];
    const uint32_t w[4] = {in.x, in.y, in.z, in.w};
    if (what >= 0) {
        const int q = lane >> 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int g = 4 * what + j;
            if (g < Kg) {
                alignas(8) int8_t c[8];
                unpack8(w[j], c);
                *reinterpret_cast<uint2 *>(wq + (size_t)n * K + (size_t)g * 32 + 8 * q) =
                    *reinterpret_cast<uint2 *>(c);
            }
        }
    } else {
        const int u = -1 - what;
        const int p = lane >> 4;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int g = 32 * u + 8 * p + i;
            if (g < Kg) scales[(size_t)n * Kg + g] = (uint16_t)((w[i / 2] >> (16 * (i & 1))) & 0xFFFFu);
        }
    }
}

// ---------------------------------------------------------------- W4C
// The weight tiles of W4G32 without scale tiles; fp32 scales per row like W8C.
__global__ __launch_bounds__(256) void pack_w4c_kernel(const int8_t *__restrict__ wq,
                                                       const float *__restrict__ scales,
                                                       uint4 *__restrict__ packed, float *__restrict__ ps,
                                                       int N, int K, int Np, int KT, int half) {
    const int Kg = K / 32;
    const size_t total = (size_t)(Np / 16) * KT * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < (size_t)Np) ps[v] = v < (size_t)N ? scales[logical_row((int)v, N, half)] : 0.0f;
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int kt = (int)(tile % KT);
    const int rt = (int)(tile / KT);
    const int n = logical_row(rt * 16 + (lane & 15), N, half);
    const int q = lane >> 4;
    uint32_t d[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int g = 4 * kt + j;
        if (n < N && g < Kg) {
            alignas(8) int8_t c[8];
            *reinterpret_cast<uint2 *>(c) = *reinterpret_cast<const uint2 *>(wq + (size_t)n * K + (size_t)g * 32 + 8 * q);
            d[j] = pack8(c);
        } else {
            d[j] = 0x88888888u;
        }
    }
    packed[v] = make_uint4(d[0], d[1], d[2], d[3]);
}

__global__ __launch_bounds__(256) void unpack_w4c_kernel(const uint4 *__restrict__ packed,
                                                         const float *__restrict__ ps,
                                                         int8_t *__restrict__ wq, float *__restrict__ scales,
                                                         int N, int K, int Np, int KT, int half) {
    const int Kg = K / 32;
    const size_t total = (size_t)(Np / 16) * KT * 64;
    const size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < (size_t)N) scales[logical_row((int)v, N, half)] = ps[v];
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int kt = (int)(tile % KT);
    const int rt = (int)(tile / KT);
    const int n = logical_row(rt * 16 + (lane & 15), N, half);
    if (n >= N) return;
    const int q = lane >> 4;
    const uint4 in = packed[v];
    const uint32_t w[4] = {in.x, in.y, in.z, in.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int g = 4 * kt + j;
        if (g < Kg) {
            alignas(8) int8_t c[8];
            unpack8(w[j], c);
            *reinterpret_cast<uint2 *>(wq + (size_t)n * K + (size_t)g * 32 + 8 * q) = *reinterpret_cast<uint2 *>(c);
        }
    }
}

// ---------------------------------------------------------------- embedding lookup
// Rows ids[m] of the quantized table as binary16: y[m, k] = fp16(s * q), the product taken in fp32
// (exact for binary16 group scales; rounded to fp32 first for fp32 channel scales).  The table is
// the packed layer itself (the tied embedding / LM-head matrix of the int4 and int8 schemes of
// section 4.2 of the paper): one thread per 16-byte vector of the row's tiles.  Ids outside
// [0, N) give a row of zeros.
template <int FMT>
__global__ __launch_bounds__(256) void embedding_kernel(const uint4 *__restrict__ packed, const float *__restrict__ ps,
                                                        const int32_t *__restrict__ ids, _Float16 *__restrict__ y,
                                                        int N, int K, int KT, int rt_stride) {
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    const int m = blockIdx.y;
    const int v = blockIdx.x * 256 + threadIdx.x;  // vector of the row: tile v / 4, quarter v % 4
    if (v >= KT * 4) return;
    const int kt = v >> 2, q = v & 3;
    const int n = ids[m];
    const bool valid = n >= 0 && n < N;
    const int rt = valid ? n >> 4 : 0, c = n & 15;
    _Float16 *row = y + (size_t)m * K;
    if (FMT == kW8C) {
        const int k0 = kt * 64 + q * 16;
        if (k0 >= K) return;
        const uint4 in = packed[((size_t)rt * rt_stride + kt) * 64 + q * 16 + c];
        const float sc = valid ? ps[n] : 0.0f;
        const uint32_t w[4] = {in.x, in.y, in.z, in.w};
        half8 o[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int code = (int)(int8_t)((w[e >> 2] >> (8 * (e & 3))) & 0xFFu);
            o[e >> 3][e & 7] = (_Float16)(valid ? sc * (float)code : 0.0f);
        }
        *reinterpret_cast<half8 *>(row + k0) = o[0];
        *reinterpret_cast<half8 *>(row + k0 + 8) = o[1];
        return;
    }
    // int4 formats: dword j of the lane's vector = codes k = 128 kt + 32 j + 8 q .. + 7
    const int pos = FMT == kW4G32 ? kt + (kt >> 3) : kt;  // a scale tile follows every 8 weight tiles
    const uint4 in = packed[((size_t)rt * rt_stride + pos) * 64 + q * 16 + c];
    const uint32_t w[4] = {in.x, in.y, in.z, in.w};
    uint4 sv = make_uint4(0, 0, 0, 0);
    float sc = 0.0f;
    if (FMT == kW4G32) {
        const int u = kt >> 3, ntu = min(8, KT - 8 * u);  // the unit's scale tile: after its ntu weight tiles
        const int gl0 = 4 * (kt & 7);                      // first group of this tile inside the unit
        sv = packed[((size_t)rt * rt_stride + 9 * u + ntu) * 64 + (gl0 >> 3) * 16 + c];
    } else if (valid) {
        sc = ps[n];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k0 = kt * 128 + 32 * j + 8 * q;
        if (k0 >= K) continue;
        if (FMT == kW4G32) {
            const int gi = (4 * (kt & 7) + j) & 7;  // group inside the scale vector
            const uint32_t sd = gi < 2 ? sv.x : gi < 4 ? sv.y : gi < 6 ? sv.z : sv.w;
            sc = (float)__builtin_bit_cast(_Float16, (uint16_t)(sd >> (16 * (gi & 1))));
        }
        alignas(8) int8_t code[8];
        unpack8(w[j], code);
        half8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (_Float16)(valid ? sc * (float)code[e] : 0.0f);
        *reinterpret_cast<half8 *>(row + k0) = o;
    }
}

inline unsigned blocks_for(size_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

hipError_t launch_pack(const Geometry &g, const int8_t *wq, const void *scales, void *packed,
                       hipStream_t st) {
    if (g.fmt == kW8C) {
        const size_t total = (size_t)g.RTp * g.KT * 64;
        pack_w8c_kernel<<<blocks_for(total), 256, 0, st>>>(
            wq, static_cast<const float *>(scales), static_cast<uint4 *>(packed),
            reinterpret_cast<float *>(static_cast<char *>(packed) + g.scale_off), g.N, g.K, g.Np, g.KT, g.pair_half);
    } else if (g.fmt == kW4C) {
        const size_t total = (size_t)g.RTp * g.KT * 64;
        pack_w4c_kernel<<<blocks_for(total > (size_t)g.Np ? total : (size_t)g.Np), 256, 0, st>>>(
            wq, static_cast<const float *>(scales), static_cast<uint4 *>(packed),
            reinterpret_cast<float *>(static_cast<char *>(packed) + g.scale_off), g.N, g.K, g.Np, g.KT, g.pair_half);
    } else {
        const size_t total = (size_t)g.RTp * g.rt_stride * 64;
        pack_w4g32_kernel<<<blocks_for(total), 256, 0, st>>>(
            wq, static_cast<const uint16_t *>(scales), static_cast<uint4 *>(packed), g.N, g.K, g.RTp, g.KT,
            g.rt_stride, g.pair_half);
    }
    return hipGetLastError();
}

hipError_t launch_embedding(const Geometry &g, const void *packed, const int32_t *ids, int M, void *y,
                            hipStream_t st) {
    const uint4 *pv = static_cast<const uint4 *>(packed);
    const float *ps = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    _Float16 *yo = static_cast<_Float16 *>(y);
    const dim3 grid(blocks_for((size_t)g.KT * 4), (unsigned)M);
    if (g.fmt == kW8C)
        embedding_kernel<kW8C><<<grid, 256, 0, st>>>(pv, ps, ids, yo, g.N, g.K, g.KT, g.rt_stride);
    else if (g.fmt == kW4C)
        embedding_kernel<kW4C><<<grid, 256, 0, st>>>(pv, ps, ids, yo, g.N, g.K, g.KT, g.rt_stride);
    else
        embedding_kernel<kW4G32><<<grid, 256, 0, st>>>(pv, ps, ids, yo, g.N, g.K, g.KT, g.rt_stride);
    return hipGetLastError();
}

hipError_t launch_unpack(const Geometry &g, const void *packed, int8_t *wq, void *scales,
                         hipStream_t st) {
    if (g.fmt == kW8C) {
        const size_t total = (size_t)g.RTp * g.KT * 64;
        unpack_w8c_kernel<<<blocks_for(total), 256, 0, st>>>(
            static_cast<const uint4 *>(packed),
            reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off), wq,
            static_cast<float *>(scales), g.N, g.K, g.Np, g.KT, g.pair_half);
    } else if (g.fmt == kW4C) {
        const size_t total = (size_t)g.RTp * g.KT * 64;
        unpack_w4c_kernel<<<blocks_for(total > (size_t)g.Np ? total : (size_t)g.Np), 256, 0, st>>>(
            static_cast<const uint4 *>(packed),
            reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off), wq,
            static_cast<float *>(scales), g.N, g.K, g.Np, g.KT, g.pair_half);
    } else {
        const size_t total = (size_t)g.RTp * g.rt_stride * 64;
        unpack_w4g32_kernel<<<blocks_for(total), 256, 0, st>>>(
            static_cast<const uint4 *>(packed), wq, static_cast<uint16_t *>(scales), g.N, g.K, g.RTp, g.KT,
            g.rt_stride, g.pair_half);
    }
    return hipGetLastError();
}

}  // namespace qfc
