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
//
// Tiled for the int8 product with 4-bit weights (TILED = 2): the packed 4-bit tiles keep the eight
// codes of octet q of quantization-group-sized run g of a 128-k block in one dword, so the
// product takes k in that order, and the activations are laid out to match: the 16 codes of
// lane (c, q) of tile 2 t + op are k = 128 t + 32 (2 op) + 8 q .. + 7 followed by
// k = 128 t + 32 (2 op + 1) + 8 q .. + 7 (a permutation of the 8-byte pieces inside each 128-k
// block; the contraction does not care about the order of k as long as both operands agree).
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

// A workgroup of NW = 2 ROWS wavefronts takes ROWS token rows (8, 4 or 2).  With T = 16 / ROWS, lane
// (c, q, t) of wavefront w handles, in step i, the 16 values k = 64 kt + 16 q .. + 15 of row c,
// kt = T (NW i + w) + t: a wavefront instruction reads 256 T contiguous bytes of each of its rows
// and, in the tiled layout, writes 16 ROWS contiguous bytes per tile quarter.  The values of the
// first KEEP steps stay in registers between the maximum pass and the quantization pass (rows up
// to K = 14336 are read once); longer rows are read a second time.  Few rows per workgroup spread
// a small M over the whole chip (a compute unit streams only about 30 GB/s on its own); many rows
// per workgroup write whole 128-byte lines.
// `gate` (or null): the row that is quantized is fp16(act(gate) * x), the input of a layer whose
// two input branches are merged into it (operator fusion, section 3.6 of the paper).
template <int TILED, int ROWS, bool GLU>
__global__ __launch_bounds__(128 * ROWS) void act_quant_kernel(const uint4 *__restrict__ x,
                                                               const uint4 *__restrict__ gate, int act, int M,
                                                               int K, uint4 *__restrict__ xq,
                                                               float *__restrict__ sx, int Kp) {
    constexpr bool kTiled = TILED != 0;
    constexpr int T = 16 / ROWS;           // tiles per wavefront instruction
    constexpr int NW = 2 * ROWS;           // wavefronts; NW * T = 32 tiles per step
    constexpr int KEEP = 7;
    __shared__ float wmax[NW][ROWS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane % ROWS, q = (lane / ROWS) & 3, t = lane / (4 * ROWS);
    // Tiled output: the workgroups that share the lines of a tile run on one XCD (workgroup b runs
    // on XCD b % 8), so the pieces of a line meet in that XCD's L2.  The grid is a multiple of 8 then.
    const int wg = kTiled ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
    const int m = wg * ROWS + c;
    const bool real = m < M;
    const int tiles = (kTiled ? Kp : K + 63) / 64;
    const int steps = (tiles + 31) / 32;
    const uint4 *row = x + (size_t)(real ? m : 0) * (K / 8);

    uint4 keep[KEEP][2];
    us2 amax = {0, 0};
    auto load = [&](int i, uint4 &v0, uint4 &v1) {
        const int k0 = (T * (NW * i + wave) + t) * 64 + q * 16;
        const bool in = real && k0 < K;
        const size_t off = in ? k0 / 8 : 0;
        v0 = row[off];
        v1 = row[off + 1];
        if (GLU) {
            const uint4 *grow = gate + (size_t)(real ? m : 0) * (K / 8);
            v0 = gated_input8_u4<true>(grow[off], v0, act);
            v1 = gated_input8_u4<true>(grow[off + 1], v1, act);
        }
        if (!in) v0 = v1 = make_uint4(0, 0, 0, 0);
    };
    auto fold = [&](const uint4 &v0, const uint4 &v1) {
        amax = fold_abs(fold_abs(fold_abs(fold_abs(amax, v0.x), v0.y), v0.z), v0.w);
        amax = fold_abs(fold_abs(fold_abs(fold_abs(amax, v1.x), v1.y), v1.z), v1.w);
    };
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        if (i < steps) {
            load(i, keep[i][0], keep[i][1]);
            fold(keep[i][0], keep[i][1]);
        }
    }
    for (int i = KEEP; i < steps; ++i) {
        uint4 v0, v1;
        load(i, v0, v1);
        fold(v0, v1);
    }
    const unsigned short top = amax.x > amax.y ? amax.x : amax.y;
    float a = (float)__builtin_bit_cast(_Float16, top);
#pragma unroll
    for (int off = ROWS; off < 64; off <<= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
    if (lane < ROWS) wmax[wave][lane] = a;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) a = fmaxf(a, wmax[w][c]);
    float scale = 0.0f, inv = 0.0f;
    if (a != 0.0f) {
        scale = a / 127.0f;
        inv = 127.0f / a;
    }
    if (wave == 0 && lane < ROWS && (kTiled || real)) sx[m] = scale;

    auto emit = [&](int i, const uint4 &v0, const uint4 &v1) {
        const int kt = T * (NW * i + wave) + t;
        if (kt >= tiles) return;
        const h8 h0 = __builtin_bit_cast(h8, v0), h1 = __builtin_bit_cast(h8, v1);
        _Float16 v[16];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[e] = h0[e];
            v[8 + e] = h1[e];
        }
        const uint4 out = make_uint4(quant4(v, inv), quant4(v + 4, inv), quant4(v + 8, inv), quant4(v + 12, inv));
        if (TILED == 2) {
            // source octets 2 q and 2 q + 1 of tile kt = octets (q & 1) * 2 and (q & 1) * 2 + 1 of run
            // g = 2 (kt & 1) + (q >> 1): 8-byte half q >> 1 of vectors 2 (q & 1) and 2 (q & 1) + 1
            uint2 *dst = reinterpret_cast<uint2 *>(xq + ((size_t)(m >> 4) * (Kp / 64) + kt) * 64 + (m & 15)) + (q >> 1);
            dst[(2 * (q & 1)) * 16 * 2] = make_uint2(out.x, out.y);
            dst[(2 * (q & 1) + 1) * 16 * 2] = make_uint2(out.z, out.w);
        } else if (kTiled)
            xq[((size_t)(m >> 4) * (Kp / 64) + kt) * 64 + q * 16 + (m & 15)] = out;
        else if (real && kt * 64 + q * 16 < K)
            xq[(size_t)m * (K / 16) + kt * 4 + q] = out;
    };
#pragma unroll
    for (int i = 0; i < KEEP; ++i)
        if (i < steps) emit(i, keep[i][0], keep[i][1]);
    for (int i = KEEP; i < steps; ++i) {
        uint4 v0, v1;
        load(i, v0, v1);
        emit(i, v0, v1);
    }
}

// PERM: the k order of the product with 4-bit weights (see the head of this file).
template <bool PERM>
__global__ __launch_bounds__(256) void retile_xq_kernel(const uint4 *__restrict__ xq, int M, int K,
                                                        uint4 *__restrict__ tiled, int Mp, int Kp) {
    const size_t total = (size_t)Mp * (Kp / 16);
    const size_t v = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= total) return;
    const int lane = (int)(v % 64);
    const size_t tile = v / 64;
    const int kt = (int)(tile % (Kp / 64));
    const int m = (int)(tile / (Kp / 64)) * 16 + (lane & 15);
    uint4 out = make_uint4(0, 0, 0, 0);
    if (PERM) {
        const int q = lane >> 4;
        const uint2 *src = reinterpret_cast<const uint2 *>(xq);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int k = (kt >> 1) * 128 + 32 * (2 * (kt & 1) + j) + 8 * q;
            uint2 p = make_uint2(0, 0);
            if (m < M && k < K) p = src[((size_t)m * K + k) / 8];
            if (j == 0) { out.x = p.x; out.y = p.y; } else { out.z = p.x; out.w = p.y; }
        }
    } else {
        const int c = kt * 4 + (lane >> 4);
        if (m < M && c * 16 < K) out = xq[(size_t)m * (K / 16) + c];
    }
    tiled[v] = out;
}


template <int ROWS>
void launch_rows(const void *x, const void *gate, int act, int M, int K, int8_t *xq, float *sx, int tiled, int Mp,
                 int Kp, hipStream_t st) {
    const uint4 *xv = static_cast<const uint4 *>(x);
    const uint4 *gv = static_cast<const uint4 *>(gate);
    uint4 *qv = reinterpret_cast<uint4 *>(xq);
    const dim3 grid((unsigned)(tiled ? Mp / ROWS : (M + ROWS - 1) / ROWS)), block(128 * ROWS);
    if (tiled == 2) {
        if (gate)
            act_quant_kernel<2, ROWS, true><<<grid, block, 0, st>>>(xv, gv, act, M, K, qv, sx, Kp);
        else
            act_quant_kernel<2, ROWS, false><<<grid, block, 0, st>>>(xv, gv, act, M, K, qv, sx, Kp);
    } else if (tiled) {
        if (gate)
            act_quant_kernel<1, ROWS, true><<<grid, block, 0, st>>>(xv, gv, act, M, K, qv, sx, Kp);
        else
            act_quant_kernel<1, ROWS, false><<<grid, block, 0, st>>>(xv, gv, act, M, K, qv, sx, Kp);
    } else {
        if (gate)
            act_quant_kernel<0, ROWS, true><<<grid, block, 0, st>>>(xv, gv, act, M, K, qv, sx, K);
        else
            act_quant_kernel<0, ROWS, false><<<grid, block, 0, st>>>(xv, gv, act, M, K, qv, sx, K);
    }
}

}  // namespace

// tiled: 0 row-major, 1 tiled, 2 tiled in the k order of the product with 4-bit weights (Kp a multiple of 128).
// Mp (tiled output) must be a multiple of 16.  The most rows per workgroup that still give two
// workgroups per compute unit, else two.
hipError_t launch_act_quant(const void *x, const void *gate, int act, int M, int K, int8_t *xq, float *sx,
                            int tiled, int Mp, int Kp, int num_cus, hipStream_t st) {
    const int rows_total = tiled ? Mp : M;
    int rows = rows_total >= 16 * num_cus ? 8 : rows_total >= 8 * num_cus ? 4 : 2;
    const int forced = tuning().act_quant_rows;
    if (forced == 2 || forced == 4 || forced == 8) rows = forced;
    if (rows == 8)
        launch_rows<8>(x, gate, act, M, K, xq, sx, tiled, Mp, Kp, st);
    else if (rows == 4)
        launch_rows<4>(x, gate, act, M, K, xq, sx, tiled, Mp, Kp, st);
    else
        launch_rows<2>(x, gate, act, M, K, xq, sx, tiled, Mp, Kp, st);
    return hipGetLastError();
}

hipError_t launch_retile_xq(const int8_t *xq, int M, int K, int8_t *tiled, int Mp, int Kp, bool int4_order,
                            hipStream_t st) {
    const size_t total = (size_t)Mp * (Kp / 16);
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (int4_order)
        retile_xq_kernel<true><<<grid, 256, 0, st>>>(reinterpret_cast<const uint4 *>(xq), M, K, reinterpret_cast<uint4 *>(tiled), Mp, Kp);
    else
        retile_xq_kernel<false><<<grid, 256, 0, st>>>(reinterpret_cast<const uint4 *>(xq), M, K, reinterpret_cast<uint4 *>(tiled), Mp, Kp);
    return hipGetLastError();
}

}  // namespace qfc
