// Decode kernels (M <= 8 token rows): y[m,n] = sum_k x[m,k] * s * Wq[n,k].
// The memory-bound fully connected kernel of the decode stage (section 3.7 of
// the paper), here with binary16 activations and the weights dequantized in
// registers.
//
// Mapping.  A wavefront owns 64 output rows (lane = row) and a contiguous range
// of K.  Every 16-byte lane load is one contiguous KiB for the wavefront; the
// activations of the current k range are the same for all 64 lanes, so they are
// read through the scalar unit and used as scalar operands of v_dot2_f32_f16.
// No lane ever needs another lane's data: there is no cross-lane reduction in
// the streaming loop.  K is split over the wavefronts of a workgroup (summed in
// LDS, fixed order) and, when there are too few row blocks to fill 256 CUs,
// over several workgroups (fp32 partials in the workspace, summed in fixed
// order by the workgroup that arrives last; no floating-point atomics, so the
// result is deterministic).
#include "qfc_internal.h"

namespace qfc {

Tuning &tuning() {
    static Tuning t;
    return t;
}

GemvPlan plan_gemv(const Geometry &g, int M, int num_cus) {
    (void)M;
    (void)num_cus;
    GemvPlan p;
    p.units = g.fmt == kW8C ? (g.K + 127) / 128 : (g.K + 255) / 256;
    const Tuning &t = tuning();
    int per_rb = (t.gemv_target_waves + g.RB - 1) / g.RB;
    if (per_rb < 1) per_rb = 1;
    if (per_rb > p.units) per_rb = p.units;
    int maxw = t.gemv_max_waves_per_wg;
    if (maxw > 8) maxw = 8;  // LDS reduction buffer holds 8 wavefronts
    if (maxw < 1) maxw = 1;
    p.splits = (per_rb + maxw - 1) / maxw;
    p.waves = (per_rb + p.splits - 1) / p.splits;
    return p;
}

static size_t ticket_bytes(const Geometry &g) { return (size_t)round_up(g.RB * 4, 256); }

size_t gemv_workspace_bytes(const Geometry &g, int M, int num_cus) {
    const GemvPlan p = plan_gemv(g, M, num_cus);
    size_t b = ticket_bytes(g);
    if (p.splits > 1) b += (size_t)p.splits * M * g.RB * 64 * sizeof(float);
    return b;
}

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }

__device__ __forceinline__ float dot2(h2 a, h2 b, float c) {
    return __builtin_amdgcn_fdot2(a, b, c, false);
}

__device__ __forceinline__ float f16_bits_to_f32(uint32_t bits) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}

struct GemvArgs {
    const u32x4 *packed;
    const uint32_t *x;  // binary16 pairs, [M, K/2]
    _Float16 *y;        // [M, N]
    const float *sw;    // W8C scales [Np]
    float *partial;     // [splits][M][RB*64]
    unsigned *tickets;  // [RB]
    int N, K, units_q, units_rem, waves, splits, units_stride, ld;
};

// Sum the per-wavefront partials in LDS, then either store y or hand the
// workgroup's partial to the cross-workgroup reduction.
template <int M, bool kPerChannelScale>
__device__ __forceinline__ void finish(const GemvArgs &a, float (&acc)[M], int rb, int split, int wave,
                                       int lane) {
    __shared__ float red[kMaxDecodeM * 8 * 64];
    if (a.waves > 1) {
#pragma unroll
        for (int m = 0; m < M; ++m) red[(wave * M + m) * 64 + lane] = acc[m];
        __syncthreads();
    }
    if (wave != 0) return;
    if (a.waves > 1) {
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float s = red[m * 64 + lane];
            for (int w = 1; w < a.waves; ++w) s += red[(w * M + m) * 64 + lane];
            acc[m] = s;
        }
    }
    const int n = rb * 64 + lane;
    const int ld = a.ld;  // RB * 64
    if (a.splits > 1) {
        // Publish this workgroup's partial, then take a ticket; the workgroup that
        // draws the last ticket of the row block sums all partials in split order.
#pragma unroll
        for (int m = 0; m < M; ++m) a.partial[(size_t)(split * M + m) * ld + n] = acc[m];
        __threadfence();
        unsigned last = 0;
        if (lane == 0) last = atomicAdd(&a.tickets[rb], 1u) == (unsigned)(a.splits - 1) ? 1u : 0u;
        last = __builtin_amdgcn_readfirstlane(last);
        if (!last) return;
        __threadfence();
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float s = 0.0f;
            for (int sp = 0; sp < a.splits; ++sp) s += a.partial[(size_t)(sp * M + m) * ld + n];
            acc[m] = s;
        }
        if (lane == 0) a.tickets[rb] = 0u;  // ready for the next call on this workspace
    }
    if (n < a.N) {
        float sc = 1.0f;
        if (kPerChannelScale) sc = a.sw[n];
#pragma unroll
        for (int m = 0; m < M; ++m) a.y[(size_t)m * a.N + n] = (_Float16)(acc[m] * sc);
    }
}

// ---------------------------------------------------------------- W4G32
// Eight biased int4 codes of one dword -> four binary16 pairs (k-adjacent),
// exactly: 0x6400 | u is 1024 + u, 0x6400 | (u << 4) is 1024 + 16 u.
// (w & mask) | magic in one VALU instruction; the compiler emits two otherwise.
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t magic) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(magic));
    return r;
}

__device__ __forceinline__ void dequant8(uint32_t w, h2 (&p)[4]) {
    const uint32_t magic = 0x64006400u;
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t ws = w >> 8;
    p[0] = as_h2(and_or(w, 0x000F000Fu, magic)) - c1032;
    p[1] = as_h2(and_or(w, 0x00F000F0u, magic)) * c16th - c72;
    p[2] = as_h2(and_or(ws, 0x000F000Fu, magic)) - c1032;
    p[3] = as_h2(and_or(ws, 0x00F000F0u, magic)) * c16th - c72;
}

template <int M>
__device__ __forceinline__ void w4_group(const u32x4 &wv, uint32_t scale_bits, const uint32_t *xg, int K2,
                                         float (&acc)[M]) {
    float part[M];
#pragma unroll
    for (int m = 0; m < M; ++m) part[m] = 0.0f;
    const uint32_t wd[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        h2 p[4];
        dequant8(wd[d], p);
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const uint32_t *xm = xg + (size_t)m * K2 + d * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) part[m] = dot2(p[i], as_h2(xm[i]), part[m]);
        }
    }
    const float s = f16_bits_to_f32(scale_bits);
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] = fmaf(s, part[m], acc[m]);
}

template <int M>
__global__ __launch_bounds__(512) void gemv_w4g32_kernel(GemvArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rb = blockIdx.y;
    const int split = blockIdx.x;
    const int t = split * a.waves + wave;
    // units = q * slots + rem: the first rem slots take q + 1 units
    const int u0 = t * a.units_q + (t < a.units_rem ? t : a.units_rem);
    const int u1 = u0 + a.units_q + (t < a.units_rem ? 1 : 0);
    const int Kg = a.K / 32;
    const int K2 = a.K / 2;

    float acc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] = 0.0f;

    const u32x4 *p = a.packed + ((size_t)rb * a.units_stride + u0) * kW4UnitVecs + lane;
    u32x4 cur[9];
    if (u0 < u1) {
#pragma unroll
        for (int j = 0; j < 9; ++j) cur[j] = __builtin_nontemporal_load(p + j * 64);
    }
    for (int u = u0; u < u1; ++u) {
        u32x4 nxt[9];
        p += kW4UnitVecs;
        if (u + 1 < u1) {
#pragma unroll
            for (int j = 0; j < 9; ++j) nxt[j] = __builtin_nontemporal_load(p + j * 64);
        }
        const uint32_t sc[4] = {cur[8].x, cur[8].y, cur[8].z, cur[8].w};
        const uint32_t *xu = a.x + (size_t)u * 128;  // 256 k = 128 pairs
        if (u * 8 + 8 <= Kg) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                w4_group<M>(cur[j], (sc[j >> 1] >> (16 * (j & 1))) & 0xFFFFu, xu + j * 16, K2, acc);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (u * 8 + j < Kg)
                    w4_group<M>(cur[j], (sc[j >> 1] >> (16 * (j & 1))) & 0xFFFFu, xu + j * 16, K2, acc);
        }
        if (u + 1 < u1) {
#pragma unroll
            for (int j = 0; j < 9; ++j) cur[j] = nxt[j];
        }
    }
    finish<M, false>(a, acc, rb, split, wave, lane);
}

// ---------------------------------------------------------------- W8C
// Four int8 codes of one dword -> two binary16 pairs, exactly: flipping the
// sign bit gives b + 128 in [0, 255]; 0x64 in the high byte makes 1024 + that.
__device__ __forceinline__ void dequant4(uint32_t w, h2 (&p)[2]) {
    const h2 c1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
    const uint32_t wx = w ^ 0x80808080u;
    p[0] = as_h2(__builtin_amdgcn_perm(0x64646464u, wx, 0x04010400u)) - c1152;
    p[1] = as_h2(__builtin_amdgcn_perm(0x64646464u, wx, 0x04030402u)) - c1152;
}

template <int M>
__device__ __forceinline__ void w8_chunk(const u32x4 &wv, const uint32_t *xc, int K2, float (&acc)[M]) {
    const uint32_t wd[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        h2 p[2];
        dequant4(wd[d], p);
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const uint32_t *xm = xc + (size_t)m * K2 + d * 2;
            acc[m] = dot2(p[0], as_h2(xm[0]), acc[m]);
            acc[m] = dot2(p[1], as_h2(xm[1]), acc[m]);
        }
    }
}

template <int M>
__global__ __launch_bounds__(512) void gemv_w8c_kernel(GemvArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rb = blockIdx.y;
    const int split = blockIdx.x;
    const int t = split * a.waves + wave;
    // units = q * slots + rem: the first rem slots take q + 1 units
    const int u0 = t * a.units_q + (t < a.units_rem ? t : a.units_rem);
    const int u1 = u0 + a.units_q + (t < a.units_rem ? 1 : 0);
    const int Kc = a.K / 16;
    const int K2 = a.K / 2;

    float acc[M];
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] = 0.0f;

    // a unit is 8 chunks of 16 k; chunk tiles of one row block are contiguous
    const u32x4 *p = a.packed + ((size_t)rb * a.units_stride + u0) * 8 * 64 + lane;
    u32x4 cur[8];
    if (u0 < u1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) cur[j] = __builtin_nontemporal_load(p + j * 64);
    }
    for (int u = u0; u < u1; ++u) {
        u32x4 nxt[8];
        p += 8 * 64;
        if (u + 1 < u1) {
#pragma unroll
            for (int j = 0; j < 8; ++j) nxt[j] = __builtin_nontemporal_load(p + j * 64);
        }
        const uint32_t *xu = a.x + (size_t)u * 64;  // 128 k = 64 pairs
        if (u * 8 + 8 <= Kc) {
#pragma unroll
            for (int j = 0; j < 8; ++j) w8_chunk<M>(cur[j], xu + j * 8, K2, acc);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (u * 8 + j < Kc) w8_chunk<M>(cur[j], xu + j * 8, K2, acc);
        }
        if (u + 1 < u1) {
#pragma unroll
            for (int j = 0; j < 8; ++j) cur[j] = nxt[j];
        }
    }
    finish<M, true>(a, acc, rb, split, wave, lane);
}

template <int M>
hipError_t launch_m(const Geometry &g, const GemvArgs &a, dim3 grid, dim3 block, hipStream_t st) {
    if (g.fmt == kW8C)
        gemv_w8c_kernel<M><<<grid, block, 0, st>>>(a);
    else
        gemv_w4g32_kernel<M><<<grid, block, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemv(const Geometry &g, const void *packed, const void *x, int M, void *y,
                       void *workspace, int num_cus, hipStream_t st) {
    const GemvPlan p = plan_gemv(g, M, num_cus);
    GemvArgs a;
    a.packed = static_cast<const u32x4 *>(packed);
    a.x = static_cast<const uint32_t *>(x);
    a.y = static_cast<_Float16 *>(y);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.tickets = static_cast<unsigned *>(workspace);
    a.partial = reinterpret_cast<float *>(static_cast<char *>(workspace) + ticket_bytes(g));
    a.N = g.N;
    a.K = g.K;
    a.units_q = p.units / (p.splits * p.waves);
    a.units_rem = p.units % (p.splits * p.waves);
    a.ld = g.RB * 64;
    a.waves = p.waves;
    a.splits = p.splits;
    a.units_stride = g.fmt == kW8C ? g.Kp / 128 : g.Kp / 256;
    const dim3 grid((unsigned)p.splits, (unsigned)g.RB);
    const dim3 block((unsigned)(p.waves * 64));
    switch (M) {
        case 1: return launch_m<1>(g, a, grid, block, st);
        case 2: return launch_m<2>(g, a, grid, block, st);
        case 3: return launch_m<3>(g, a, grid, block, st);
        case 4: return launch_m<4>(g, a, grid, block, st);
        case 5: return launch_m<5>(g, a, grid, block, st);
        case 6: return launch_m<6>(g, a, grid, block, st);
        case 7: return launch_m<7>(g, a, grid, block, st);
        case 8: return launch_m<8>(g, a, grid, block, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace qfc
