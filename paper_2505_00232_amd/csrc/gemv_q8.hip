// Decode kernel with 8-bit activations (M <= 8 token rows), the decode design of
// section 3.7 of the paper: the fully connected kernel quantizes its input
// activations itself and works on integers; the output is dequantized at the
// end:
//   a_m = max_k |x[m,k]|,  sx[m] = a_m / 127,  xq[m,k] = clamp(rne(x[m,k] * (127 / a_m)), +-127)
//   acc[m,n] = sum_k xq[m,k] * Wq[n,k]                      (int32, exact)
//   y[m,n]   = fp16(float(acc[m,n]) * sx[m] * sw[n])
// for weights with one scale per output channel (int8, or the per-channel
// 4-bit scheme of section 4.2).  The quantization steps are those of the
// prefill quantization kernel, in the same fp32 arithmetic, so both produce
// the same codes.
//
// Same mapping as the binary16 decode kernel: a wavefront streams KiB tiles of
// 16 output rows; here a tile goes to the matrix core with no conversion at all
// (int8: the 16 bytes of a lane are its v_mfma_i32_16x16x64_i8 operand) or with
// three instructions per eight codes (int4: the two nibble planes of two dwords
// are the 16 operand bytes; codes stay biased by 8, and 8 * sum_k xq[m,k] is
// subtracted from the integer accumulators at the end, exactly).  The quantized
// activations of the k range a wavefront works on sit in a private LDS region
// in operand order.  Wavefronts of a workgroup split K; their integer partial
// sums meet in LDS.
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GemvQ8Args {
    const u32x4 *packed;
    const u32x4 *x;      // SRC 0: binary16 [M, K] as 16-byte vectors
    const int8_t *xq;    // SRC 1: int8 [M, K]
    const float *sx_in;  // SRC 1: scales of the rows (null with raw output)
    _Float16 *y;         // [M, N] (OUT 0)
    int32_t *acc_out;    // [M, N] (OUT 1)
    const float *sw;     // per-channel weight scales [Np]
    int N, K, RT, KT, KU, rt_stride;
    int row_tiles;
    int units_q, units_rem;
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// sum of the four signed bytes of a dword, added to acc
__device__ __forceinline__ int bytes_sum(uint32_t d, int acc) {
    return __builtin_amdgcn_sdot4((int)d, 0x01010101, acc, false);
}

// FMT: kW8C or kW4C.  SRC 0: binary16 activations, quantized here; 1: int8 activations given.
// OUT 0: binary16 y; 1: raw int32 accumulators.
template <int M, int FMT, int SRC, int OUT>
__global__ __launch_bounds__(512) void gemv_q8_kernel(GemvQ8Args a) {
    constexpr int TILES = 8;
    constexpr int UK = FMT == kW8C ? 512 : 1024;  // k per unit
    constexpr int SLOTS = UK / 16;                // 16-byte operand slots per token row per unit
    constexpr int NCH = (M * SLOTS + 63) / 64;    // slots a lane stages per unit
    constexpr int MI = M < 4 ? M : 4;
    extern __shared__ u32x4 lds_all[];
    __shared__ float s_amax[8][M];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int rt0 = blockIdx.x * a.row_tiles;
    const int R = min(a.row_tiles, a.RT - rt0);
    const int u0 = wave * a.units_q + min(wave, a.units_rem);
    const int u1 = u0 + a.units_q + (wave < a.units_rem ? 1 : 0);
    u32x4 *lds_x = lds_all + wave * (SLOTS * M);

    // The weights of the first item are requested before anything else: they do not depend on
    // the activations, and their latency then covers the quantization parameters' pass over x.
    const int items = (u1 - u0) * R;
    auto load_w = [&](u32x4 (&w)[TILES], int u, int r) {
        const int nt = min(TILES, a.KT - TILES * u);
        const u32x4 *base = a.packed + ((size_t)(rt0 + r) * a.rt_stride + TILES * u) * 64 + lane;
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const u32x4 zero = {0, 0, 0, 0};
            w[t] = t < nt ? __builtin_nontemporal_load(base + t * 64) : zero;
        }
    };
    u32x4 w[TILES];
    if (items > 0) load_w(w, u0, 0);

    // ---- quantization parameters of the token rows (every workgroup computes them for itself)
    float inv[M], sxr[M];
    if (SRC == 0) {
        float am[M];
#pragma unroll
        for (int m = 0; m < M; ++m) am[m] = 0.0f;
        const int K8 = a.K / 8;
        for (int v = threadIdx.x; v < M * K8; v += blockDim.x) {
            const int m = v / K8;
            const h8 h = __builtin_bit_cast(h8, a.x[v]);
            float t = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) t = fmaxf(t, fabsf((float)h[i]));
#pragma unroll
            for (int mm = 0; mm < M; ++mm)
                if (mm == m) am[mm] = fmaxf(am[mm], t);
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            am[m] = wave_max(am[m]);
            if (lane == 0) s_amax[wave][m] = am[m];
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float t = 0.0f;
            for (int w = 0; w < nwaves; ++w) t = fmaxf(t, s_amax[w][m]);
            sxr[m] = t != 0.0f ? t / 127.0f : 0.0f;
            inv[m] = t != 0.0f ? 127.0f / t : 0.0f;
        }
    } else {
#pragma unroll
        for (int m = 0; m < M; ++m) {
            sxr[m] = (OUT == 0) ? a.sx_in[m] : 1.0f;
            inv[m] = 0.0f;
        }
    }

    int acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[r][i] = 0;
    int xsum[M];  // sum of the quantized activations this wavefront has staged, per token row (int4: bias removal)
#pragma unroll
    for (int m = 0; m < M; ++m) xsum[m] = 0;

    // Operand slot s of a unit (16 bytes of one token row):
    //   int8: tile s / 4, quarter s % 4: k = 64 (s / 4) + 16 (s % 4) .. + 15
    //   int4: group pair s / 4, octet s % 4: k = 64 (s / 4) + 8 (s % 4) .. + 7 and the same + 32
    auto stage = [&](int u) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int p = i * 64 + lane;
            if (p >= M * SLOTS) continue;
            const int m = p / SLOTS, s = p % SLOTS;
            const int ka = u * UK + (s >> 2) * 64 + (FMT == kW8C ? 16 : 8) * (s & 3);
            const int kb = FMT == kW8C ? ka + 8 : ka + 32;
            // addresses past K are clamped to the row's start and the loaded values replaced by zero
            const bool ina = ka < a.K, inb = kb < a.K;
            const size_t ea = (size_t)m * a.K + (ina ? ka : 0), eb = (size_t)m * a.K + (inb ? kb : 0);
            u32x4 out;
            if (SRC == 0) {
                const u32x4 zero = {0, 0, 0, 0};
                u32x4 va = a.x[ea / 8], vb = a.x[eb / 8];
                va = ina ? va : zero;
                vb = inb ? vb : zero;
                const h8 ha = __builtin_bit_cast(h8, va), hb = __builtin_bit_cast(h8, vb);
                _Float16 t[16];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    t[e] = ha[e];
                    t[8 + e] = hb[e];
                }
                float invm = 0.0f;
#pragma unroll
                for (int mm = 0; mm < M; ++mm)
                    if (mm == m) invm = inv[mm];
                out.x = quant4(t, invm);
                out.y = quant4(t + 4, invm);
                out.z = quant4(t + 8, invm);
                out.w = quant4(t + 12, invm);
            } else {
                const uint2 *pa = reinterpret_cast<const uint2 *>(a.xq + ea);
                const uint2 *pb = reinterpret_cast<const uint2 *>(a.xq + eb);
                const uint2 va = *pa, vb = *pb;
                out.x = ina ? va.x : 0u;
                out.y = ina ? va.y : 0u;
                out.z = inb ? vb.x : 0u;
                out.w = inb ? vb.y : 0u;
            }
            const int sum = bytes_sum(out.x, bytes_sum(out.y, bytes_sum(out.z, bytes_sum(out.w, 0))));
            if (FMT == kW4C) {
#pragma unroll
                for (int mm = 0; mm < M; ++mm)
                    if (mm == m) xsum[mm] += sum;
            }
            lds_x[s * M + m] = out;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    int u = u0, r = 0;
    for (int it = 0; it < items; ++it) {
        const int nt = min(TILES, a.KT - TILES * u);
        if (it > 0) load_w(w, u, r);
        if (r == 0) stage(u);
        // lanes whose row index is >= M read row c % M: that row of the result is never used
        const u32x4 *xrow = lds_x + q * M + (c % M);
        v4i d0 = {0, 0, 0, 0}, d1 = {0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            if (t < nt) {
                if (FMT == kW8C) {
                    const v4i xa = __builtin_bit_cast(v4i, xrow[(t * 4) * M]);
                    const v4i wb = __builtin_bit_cast(v4i, w[t]);
                    if (t & 1) d1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, wb, d1, 0, 0, 0);
                    else d0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, wb, d0, 0, 0, 0);
                } else {
                    // dwords 0, 1 = groups 4 t, 4 t + 1 (pair 2 t); dwords 2, 3 = pair 2 t + 1
                    const v4i xa0 = __builtin_bit_cast(v4i, xrow[((2 * t) * 4) * M]);
                    const v4i xa1 = __builtin_bit_cast(v4i, xrow[((2 * t + 1) * 4) * M]);
                    const u32x4 b0 = {w[t].x & 0x0F0F0F0Fu, (w[t].x >> 4) & 0x0F0F0F0Fu, w[t].y & 0x0F0F0F0Fu, (w[t].y >> 4) & 0x0F0F0F0Fu};
                    const u32x4 b1 = {w[t].z & 0x0F0F0F0Fu, (w[t].z >> 4) & 0x0F0F0F0Fu, w[t].w & 0x0F0F0F0Fu, (w[t].w >> 4) & 0x0F0F0F0Fu};
                    d0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa0, __builtin_bit_cast(v4i, b0), d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa1, __builtin_bit_cast(v4i, b1), d1, 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            if (rr == r) {
#pragma unroll
                for (int i = 0; i < MI; ++i) acc[rr][i] += d0[i] + d1[i];
            }
        if (++r == R) {
            r = 0;
            ++u;
        }
    }

    if (FMT == kW4C) {
        // stored codes are Wq + 8: remove 8 * (sum of this wavefront's quantized activations) per token row
        int tot[M];
#pragma unroll
        for (int m = 0; m < M; ++m) tot[m] = wave_sum(xsum[m]);
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            int t = 0;
#pragma unroll
            for (int m = 0; m < M; ++m)
                if (m == 4 * q + i) t = tot[m];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[rr][i] -= 8 * t;
        }
    }

    // meet in LDS: red[wave][r][m][16 rows]; lane (c, q) holds token rows 4q .. 4q+3 of row c
    __syncthreads();
    int *red = reinterpret_cast<int *>(lds_all);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int m = 4 * q + i;
            if (rr < R && m < M) red[((wave * 4 + rr) * M + m) * 16 + c] = acc[rr][i];
        }
    __syncthreads();
    for (int e = threadIdx.x; e < R * M * 16; e += blockDim.x) {
        const int cc = e & 15, m = (e >> 4) % M, rr = (e >> 4) / M;
        int s = 0;
        for (int w = 0; w < nwaves; ++w) s += red[((w * 4 + rr) * M + m) * 16 + cc];
        const int n = (rt0 + rr) * 16 + cc;
        if (n < a.N) {
            if (OUT == 0) {
                float sm = 0.0f;
#pragma unroll
                for (int mm = 0; mm < M; ++mm)
                    if (mm == m) sm = sxr[mm];
                a.y[(size_t)m * a.N + n] = (_Float16)((float)s * sm * a.sw[n]);
            } else {
                a.acc_out[(size_t)m * a.N + n] = s;
            }
        }
    }
}

template <int M, int SRC, int OUT>
hipError_t launch_m(const Geometry &g, const GemvQ8Args &a, int waves, hipStream_t st) {
    const dim3 grid((unsigned)((g.RT + a.row_tiles - 1) / a.row_tiles));
    const dim3 block((unsigned)(waves * 64));
    const int slots = g.fmt == kW8C ? 32 : 64;
    size_t lds = (size_t)waves * slots * M * 16;
    const size_t red = (size_t)waves * 4 * M * 16 * sizeof(int);
    if (red > lds) lds = red;
    if (g.fmt == kW8C)
        gemv_q8_kernel<M, kW8C, SRC, OUT><<<grid, block, lds, st>>>(a);
    else
        gemv_q8_kernel<M, kW4C, SRC, OUT><<<grid, block, lds, st>>>(a);
    return hipGetLastError();
}

template <int SRC, int OUT>
hipError_t launch_any_m(const Geometry &g, const GemvQ8Args &a, int M, int waves, hipStream_t st) {
    switch (M) {
        case 1: return launch_m<1, SRC, OUT>(g, a, waves, st);
        case 2: return launch_m<2, SRC, OUT>(g, a, waves, st);
        case 3: return launch_m<3, SRC, OUT>(g, a, waves, st);
        case 4: return launch_m<4, SRC, OUT>(g, a, waves, st);
        case 5: return launch_m<5, SRC, OUT>(g, a, waves, st);
        case 6: return launch_m<6, SRC, OUT>(g, a, waves, st);
        case 7: return launch_m<7, SRC, OUT>(g, a, waves, st);
        case 8: return launch_m<8, SRC, OUT>(g, a, waves, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// src 0: x is binary16 [M, K] and is quantized in the kernel; src 1: x is int8 [M, K] with
// scales sx (ignored when out_mode is 1).  out_mode 0: binary16 y; 1: raw int32 accumulators.
hipError_t launch_gemv_q8(const Geometry &g, const void *packed, const void *x, const float *sx, int src,
                          int M, void *out, int out_mode, int num_cus, hipStream_t st) {
    if (g.fmt != kW8C && g.fmt != kW4C) return hipErrorNotSupported;
    const GemvPlan p = plan_gemv(g, M, num_cus);
    GemvQ8Args a;
    a.packed = static_cast<const u32x4 *>(packed);
    a.x = static_cast<const u32x4 *>(x);
    a.xq = static_cast<const int8_t *>(x);
    a.sx_in = sx;
    a.y = static_cast<_Float16 *>(out);
    a.acc_out = static_cast<int32_t *>(out);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.N = g.N;
    a.K = g.K;
    a.RT = g.RT;
    a.KT = g.KT;
    a.KU = g.KU;
    a.rt_stride = g.rt_stride;
    a.row_tiles = p.row_tiles;
    a.units_q = g.KU / p.waves;
    a.units_rem = g.KU % p.waves;
    if (src == 0) return launch_any_m<0, 0>(g, a, M, p.waves, st);
    return out_mode == 0 ? launch_any_m<1, 0>(g, a, M, p.waves, st) : launch_any_m<1, 1>(g, a, M, p.waves, st);
}

}  // namespace qfc
