// Attention-side operators of the decode stage.
//
// 1. Rotary embedding fused with the layout transformation of the query, key and value
//    projections (section 3.6 of the paper): the QKV layer's output [B, S, (h_q + 2 h_kv) d] goes
//    to queries [B h_kv, S g, d] (g = h_q / h_kv query heads per KV head, row s g + j), the rotated
//    keys are appended to the K cache [B h_kv, C, d] as rows pos0 + s and the values to the V cache
//    (d, cache position) as columns pos0 + s.
// 2. The two matrix products of attention with the KV cache in the role of weights (section 3.8):
//    the K cache is stored (cache position, d), i.e. K^T of Q K^T, the V cache (d, cache position);
//    both are [N, K] operands exactly like a layer's logical weight matrix, and 16 bytes of a row
//    are one lane's MFMA operand.  Physically the V cache is cut into blocks of 64 positions,
//    [B h_kv, C / 64, d, 64]: a step of the kernel then reads 128 d contiguous bytes of V as it does
//    of K, instead of d pieces of 128 bytes that lie a whole cache row apart.  Here the two products and the softmax between them run
//    in one pass over the cache (the scores never leave registers): per step of 64 positions a
//    wavefront computes S^T = K Q^T with v_mfma_f32_16x16x32_f16 (keys as rows), updates the running
//    maximum and sum of every query row, and accumulates O^T += V P^T, where the positions are
//    taken in the order in which the score tiles leave them in the lanes (no cross-lane traffic:
//    the rows of the score tiles are assigned to positions so that lane (m, r) ends up with 2 x 8
//    contiguous positions for query row m, and reads the same positions of its V rows, 16 bytes each).  The context is split over workgroups and
//    wavefronts; partial (maximum, sum, O) triples meet in LDS and then in a second small kernel.
#include <type_traits>

#include "qfc_internal.h"

namespace qfc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;
static_assert(kAttnMaxSplits <= 64, "the combine kernel takes one split per lane");

// ---------------------------------------------------------------- rotary embedding + layouts
// One thread per (b, s, head, i), i < d / 2: the pair (i, i + d / 2) of one head of one token.
__global__ __launch_bounds__(256) void rope_qkv_kernel(const _Float16 *__restrict__ qkv, int B, int S, int h_q,
                                                       int h_kv, int d, int C, int pos0, double log_base,
                                                       _Float16 *__restrict__ q_out, _Float16 *__restrict__ kc,
                                                       _Float16 *__restrict__ vc) {
    const int half = d / 2;
    const int heads = h_q + 2 * h_kv;
    const long total = (long)B * S * heads * half;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half);
    const int head = (int)((idx / half) % heads);
    const int s = (int)((idx / ((long)half * heads)) % S);
    const int b = (int)(idx / ((long)half * heads * S));
    const _Float16 *src = qkv + ((size_t)(b * S + s) * heads + head) * d;
    const double x0 = (double)(float)src[i], x1 = (double)(float)src[i + half];
    const int g = h_q / h_kv;
    if (head >= h_q + h_kv) {  // value head: no rotation, transposed into the cache
        const int kv = head - h_q - h_kv;
        const int p = pos0 + s;
        _Float16 *dst = vc + (((size_t)(b * h_kv + kv) * (C / 64) + p / 64) * d) * 64 + p % 64;
        dst[(size_t)i * 64] = src[i];
        dst[(size_t)(i + half) * 64] = src[i + half];
        return;
    }
    // angle = pos * base^(-2 i / d), in double so that long contexts keep the low bits of the angle
    const double ang = (double)(pos0 + s) * exp(-2.0 * (double)i / (double)d * log_base);
    double sn, cs;
    sincos(ang, &sn, &cs);
    const _Float16 y0 = (_Float16)(float)(x0 * cs - x1 * sn);
    const _Float16 y1 = (_Float16)(float)(x1 * cs + x0 * sn);
    _Float16 *dst;
    if (head < h_q) {
        const int kv = head / g, j = head % g;
        dst = q_out + ((size_t)(b * h_kv + kv) * (S * g) + (s * g + j)) * d;
    } else {
        const int kv = head - h_q;
        dst = kc + ((size_t)(b * h_kv + kv) * C + (pos0 + s)) * d;
    }
    dst[i] = y0;
    dst[i + half] = y1;
}

// cos and sin of the rotary angles of `positions` positions: table[(pos * d / 2 + i) * 2] = cos, + 1 = sin
// of pos * base^(-2 i / d), the angle in fp64 as in the kernel above (long contexts keep its low bits).
__global__ __launch_bounds__(256) void rope_table_kernel(int d, int positions, double log_base, float *__restrict__ table) {
    const int half = d / 2;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)positions * half) return;
    const int i = (int)(idx % half);
    const int pos = (int)(idx / half);
    const double ang = (double)pos * exp(-2.0 * (double)i / (double)d * log_base);
    double sn, cs;
    sincos(ang, &sn, &cs);
    table[2 * idx] = (float)cs;
    table[2 * idx + 1] = (float)sn;
}

// ---------------------------------------------------------------- attention over the cache
struct AttnArgs {
    const _Float16 *q;   // [G, M, D]
    const _Float16 *kc;  // [G, C, D]
    const _Float16 *vc;  // [G, C / 64, D, 64]
    float *ws_o;         // [G, splits, M, D] partial outputs (unnormalized)
    float *ws_ml;        // [G, splits, M, 2] partial (maximum, sum)
    _Float16 *out;       // [G, M, D]
    int M, g, S, C, n_ctx, splits;
    int num_cus;
    int pair;  // prefill: a workgroup takes blocks (last - i, i) in turn
    int chunk_steps;  // prefill: > 0 = walks are cut into chunks of this many steps (one workgroup each)
    int max_chunks;   // prefill: chunk slots per query row in the workspace
    float scale;
};

// Workgroup = 4 wavefronts.  grid = (splits, G).  A step covers TP pairs of score tiles = 32 TP positions:
// 64 for head sizes up to 128, 32 for 256 (whose operands of 64 positions would leave one wavefront per SIMD).
// Two workgroups per compute unit (up to head size 128) are said in the launch bounds so that the accumulators stay in
// ordinary registers (with the whole register file at its disposal the compiler parks them in
// accumulation registers and copies them back and forth for the rescaling).
template <int D>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void attn_partial_kernel(AttnArgs a) {
    constexpr int TP = D <= 128 ? 2 : 1;
    constexpr int SP = 32 * TP;  // positions per step
    constexpr int DJ = D / 32;  // MFMA steps along d of the score product
    constexpr int DT = D / 16;  // row tiles of O^T
    constexpr int PITCH = D + 4;  // floats per staged query row: O^T column, maximum, sum (16-byte aligned rows)
    extern __shared__ float lds[];  // [4][16][PITCH]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, r = lane >> 4;
    const int G = blockIdx.y;
    const int part = blockIdx.x, parts = a.splits;
    const int nb = (a.n_ctx + SP - 1) / SP;  // steps
    // the workgroup takes a contiguous range of steps; its wavefronts take every fourth step of it
    const int b0 = (int)((long)part * nb / parts) + wave, b1 = (int)((long)(part + 1) * nb / parts);

    // Q^T operand: lane (m, r) holds Q[m][32 j + 8 r .. + 7]; rows >= M are zero
    u32x4 qf[DJ];
#pragma unroll
    for (int j = 0; j < DJ; ++j) {
        const u32x4 zero = {0, 0, 0, 0};
        qf[j] = m < a.M ? *reinterpret_cast<const u32x4 *>(a.q + ((size_t)G * a.M + m) * D + 32 * j + 8 * r) : zero;
    }
    // positions a query row may see: those before the end of its own token
    // (rows >= M are all-zero queries whose results are never stored: they see everything)
    const int lim = m < a.M ? a.n_ctx - a.S + m / a.g + 1 : a.n_ctx;

    v4f acc[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t) acc[t] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    float run_max = kNegBig, run_sum = 0.0f;  // run_sum: this lane's share (its 8 positions per block)

    const _Float16 *kbase = a.kc + (size_t)G * a.C * D;
    const _Float16 *vbase = a.vc + (size_t)G * D * a.C;
    // One step = 64 positions: four score tiles of 16 positions, two MFMA steps of 32 positions for
    // O^T.  All operands of a step are requested at once, so that each 128-byte line of a V row (64
    // positions) is fetched by one burst of one wavefront.  The loop is software pipelined without a
    // second set of registers: the next step's K operands are requested as soon as the score MFMAs
    // have consumed the current ones (they fly during the softmax and the O^T MFMAs), the next step's
    // V operands at the end of the step (they fly during the next score MFMAs and softmax).
    // Which position a row of a score tile stands for is free; row w of tile t is position
    //   k0 + 32 (t / 2) + 8 (w / 4) + 4 (t % 2) + w % 4,
    // so that the eight values lane (m, r) holds of tiles (2 u, 2 u + 1) are the contiguous positions
    // k0 + 32 u + 8 r .. + 7: its V operand of MFMA step u is one 16-byte load, and the four lanes r
    // of a V row read 64 contiguous bytes.  K: lane (w = lane & 15, r) reads d = 32 j + 8 r .. + 7 of
    // its position's row (a K row is contiguous whatever the order of the rows).
    u32x4 kf[2 * TP][DJ];
    u32x4 vf[DT][TP];
    auto load_k = [&](int blk) {
#pragma unroll
        for (int t = 0; t < 2 * TP; ++t) {
            const int pos = blk * SP + 32 * (t >> 1) + 8 * (m >> 2) + 4 * (t & 1) + (m & 3);
            const _Float16 *krow = kbase + (size_t)pos * D + 8 * r;
#pragma unroll
            for (int j = 0; j < DJ; ++j) kf[t][j] = *reinterpret_cast<const u32x4 *>(krow + 32 * j);
        }
    };
    auto load_v = [&](int blk) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int p0 = blk * SP;  // first position of the step: block p0 / 64 of the cache, column p0 % 64
            const _Float16 *vrow = vbase + ((size_t)(p0 / 64) * D + 16 * dt + m) * 64 + p0 % 64 + 8 * r;
#pragma unroll
            for (int u = 0; u < TP; ++u)
                vf[dt][u] = *reinterpret_cast<const u32x4 *>(vrow + 32 * u);
        }
    };
    if (b0 < b1) {
        load_k(b0);
        load_v(b0);
    }
    for (int blk = b0; blk < b1; blk += 4) {
        const int k0 = blk * SP;
        // ---- S^T = K Q^T; lane (m, r) holds positions k0 + 32 (t / 2) + 8 r + 4 (t % 2) + i
        v4f st[2 * TP];
#pragma unroll
        for (int t = 0; t < 2 * TP; ++t) {
            v4f acc_s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int j = 0; j < DJ; ++j)
                acc_s = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, kf[t][j]), __builtin_bit_cast(h8, qf[j]), acc_s, 0, 0, 0);
            st[t] = acc_s;
        }
        if (blk + 4 < b1) load_k(blk + 4);
        // ---- scaled (in units of log 2, so that exponentials are bare v_exp_f32) and, in the steps that
        // reach past the first query token's horizon, masked
        float sc[8 * TP];
        float bmax = kNegBig;
        const bool edge = k0 + SP > a.n_ctx - a.S + 1;  // same for the whole wavefront
        if (!edge) {
#pragma unroll
            for (int e = 0; e < 8 * TP; ++e) {
                sc[e] = st[e >> 2][e & 3] * a.scale;
                bmax = fmaxf(bmax, sc[e]);
            }
        } else {
#pragma unroll
            for (int t = 0; t < 2 * TP; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int pos = k0 + 32 * (t >> 1) + 8 * r + 4 * (t & 1) + i;
                    sc[4 * t + i] = pos < lim ? st[t][i] * a.scale : kNegBig;
                    bmax = fmaxf(bmax, sc[4 * t + i]);
                }
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float new_max = fmaxf(run_max, bmax);
        const float corr = __builtin_amdgcn_exp2f(run_max - new_max);
        run_max = new_max;
        float psum = 0.0f;
        h8 pv[TP];  // P^T operands of the MFMA steps: positions of tiles (0, 1), (2, 3)
#pragma unroll
        for (int e = 0; e < 8 * TP; ++e) {
            // a masked score is kNegBig: 2^(kNegBig - maximum) is 0 unless the row has seen no valid
            // position yet (maximum = kNegBig), which the test on the score itself excludes
            float p = __builtin_amdgcn_exp2f(sc[e] - new_max);
            if (edge) p = sc[e] > 0.5f * kNegBig ? p : 0.0f;
            psum += p;
            pv[e >> 3][e & 7] = (_Float16)p;
        }
        run_sum = run_sum * corr + psum;
        // positions at or past the end of the context may hold anything (0 * NaN would poison the sum)
        if (k0 + SP > a.n_ctx) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int u = 0; u < TP; ++u) {
                    const int p0 = k0 + 32 * u + 8 * r;
                    uint32_t w[4] = {vf[dt][u].x, vf[dt][u].y, vf[dt][u].z, vf[dt][u].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (p0 + 2 * e >= a.n_ctx) w[e] &= 0xFFFF0000u;
                        if (p0 + 2 * e + 1 >= a.n_ctx) w[e] &= 0x0000FFFFu;
                    }
                    vf[dt][u] = u32x4{w[0], w[1], w[2], w[3]};
                }
        }
        // ---- O^T = O^T corr + V P^T (the running maxima settle early: most steps have corr = 1 in every lane)
        const bool rescale = __any(corr != 1.0f);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            v4f o = acc[dt];
            if (rescale) {
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] *= corr;
            }
#pragma unroll
            for (int u = 0; u < TP; ++u) {
                o = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, vf[dt][u]), pv[u], o, 0, 0, 0);
            }
            acc[dt] = o;
        }
        if (blk + 4 < b1) load_v(blk + 4);
    }
    run_sum += __shfl_xor(run_sum, 16, 64);
    run_sum += __shfl_xor(run_sum, 32, 64);

    // ---- the four wavefronts meet in LDS: [wave][m][PITCH] = O^T column m, then (maximum, sum)
    float *mine = lds + (size_t)wave * 16 * PITCH + (size_t)m * PITCH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<v4f *>(mine + 16 * dt + 4 * r) = acc[dt];  // rows d = 16 dt + 4 r + i
    if (r == 0) {
        mine[D] = run_max;
        mine[D + 1] = run_sum;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < a.M * D; e += 256) {
        const int mm = e / D, dd = e % D;
        float mx = kNegBig;
#pragma unroll
        for (int w = 0; w < 4; ++w) mx = fmaxf(mx, lds[(size_t)w * 16 * PITCH + (size_t)mm * PITCH + D]);
        float o = 0.0f, l = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float *src = lds + (size_t)w * 16 * PITCH + (size_t)mm * PITCH;
            const float f = __builtin_amdgcn_exp2f(src[D] - mx);
            o += f * src[dd];
            l += f * src[D + 1];
        }
        if (a.splits == 1) {
            a.out[((size_t)G * a.M + mm) * D + dd] = (_Float16)(o / l);
        } else {
            const size_t p = ((size_t)G * a.splits + blockIdx.x) * a.M + mm;
            a.ws_o[p * D + dd] = o;
            if (dd == 0) {
                a.ws_ml[p * 2] = mx;
                a.ws_ml[p * 2 + 1] = l;
            }
        }
    }
}

// grid = (M, G, D / 64), one wavefront per query row and 64 columns: lane s first takes the (maximum,
// sum) pair of split s (splits <= 64) and the factors 2^(maximum_s - maximum) are shared by lane
// broadcast; then lane l sums column 64 z + l of the partial outputs in split order.
template <int D>
__global__ __launch_bounds__(64) void attn_combine_kernel(AttnArgs a) {
    const int G = blockIdx.y, mm = blockIdx.x, lane = threadIdx.x;
    const int col = 64 * blockIdx.z + lane;
    const size_t row0 = ((size_t)G * a.splits) * a.M + mm;  // partial row of split s: row0 + s * M
    float mx = kNegBig, l = 0.0f;
    if (lane < a.splits) {
        mx = a.ws_ml[(row0 + (size_t)lane * a.M) * 2];
        l = a.ws_ml[(row0 + (size_t)lane * a.M) * 2 + 1];
    }
    float top = mx;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) top = fmaxf(top, __shfl_xor(top, off, 64));
    const float f = lane < a.splits ? __builtin_amdgcn_exp2f(mx - top) : 0.0f;
    float lsum = f * l;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lsum += __shfl_xor(lsum, off, 64);
    float o = 0.0f;
    const float *src = a.ws_o + row0 * D + col;
    const size_t step = (size_t)a.M * D;
    int s = 0;
    for (; s + 8 <= a.splits; s += 8) {  // eight loads in flight
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(s + u) * step];
#pragma unroll
        for (int u = 0; u < 8; ++u) o = fmaf(__shfl(f, s + u, 64), v[u], o);
    }
    for (; s < a.splits; ++s) o = fmaf(__shfl(f, s, 64), src[(size_t)s * step], o);
    a.out[((size_t)G * a.M + mm) * D + col] = (_Float16)(o / lsum);
}

// ---------------------------------------------------------------- attention, many query rows (prefill)
// More than 16 query rows per KV head.  A workgroup of 4 wavefronts owns 128 query rows, a
// wavefront 32 of them (the columns of v_mfma_f32_32x32x16_f16), and they walk the positions the
// block may see together, in steps of 32: the step's K rows and V block are copied once into LDS
// (direct-to-LDS copies, ring of NS stages, one bare s_barrier per step) and every wavefront reads
// its MFMA operands from there: S^T = K Q^T (32 positions x 32 queries), running maximum / sum per
// query (a query's 16 scores of a step sit in two lanes), O^T += V P^T.  As in the decode kernel
// the rows of the score tile are assigned to positions so that a lane's eight probabilities of an
// MFMA step are eight contiguous positions (row i = 16 c + 8 b + 4 h + r is position
// k0 + 16 c + 8 h + 4 b + r): P goes from the first product's result registers into the second
// product's operand registers as it is, and a lane's V operand is one 16-byte read.
// LDS layouts (16-byte chunks, XOR-swizzled so that the operand reads are conflict free; the copy
// writes LDS linearly, so the swizzle is applied to the address it reads from memory):
//   K stage: row = position of the step (32), D / 8 chunks per row; chunk o of row p sits at o ^ swz(p)
//   V stage: row = d (D), 4 chunks per row (32 positions); chunk c of row d sits at c ^ ((d >> 2) & 3)
// Causal: rows of token s see positions 0 .. n_ctx - S + s; the block stops at the last position
// its last row sees, rows that see less mask the rest.  grid = (blocks of 128 query rows, or pairs
// of a long and a short block in large launches, G); which block a workgroup takes is decided at
// the start of the kernel.
template <int D>
struct PrefillCfg {
    static constexpr int CPR = D / 8;                   // 16-byte chunks per K row
    static constexpr int KBYTES = 32 * D * 2;           // K rows of a step
    static constexpr int STAGE = 2 * KBYTES;            // + the V block of the step
    static constexpr int NS = 4;                        // LDS stages
    static constexpr int HALVES = D > 128 ? 2 : 1;      // wavefronts that share 32 query rows (each a part of d)
    static constexpr int NW = 4 * HALVES;               // wavefronts per workgroup
    static constexpr int COPIES = STAGE / 1024 / NW;    // copies per wavefront and stage
    __device__ static int swz(int p) { return D >= 128 ? (p & 15) : ((p >> 1) & 7); }
};

// (Two workgroups per compute unit up to head size 128: said in the launch bounds, so that the
// accumulators stay in ordinary registers, where the softmax rescales them in place.)
template <int D>
__global__ __launch_bounds__(64 * PrefillCfg<D>::NW, 2) void attn_prefill_kernel(AttnArgs a) {
    typedef float v16f __attribute__((ext_vector_type(16)));
    typedef PrefillCfg<D> Cfg;
    constexpr int DJ = D / 16;  // MFMA steps along d of the score product
    // Head size 256: eight wavefronts; wavefronts w and w + 4 own the same 32 query rows and both
    // compute their scores and probabilities, but each accumulates one half of the d range of O^T
    // (with all of it a wavefront would need more than half the register file, i.e. one wavefront
    // per SIMD with nothing to overlap with).
    constexpr int HALVES = Cfg::HALVES, NW = Cfg::NW;
    constexpr int DT = D / 32 / HALVES;  // row tiles of O^T of this wavefront
    constexpr int NS = Cfg::NS, CP = Cfg::COPIES;
    extern __shared__ uint4 lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane & 31, h = lane >> 5;
    const int G = blockIdx.y;
    // Causal walks grow with the block index.  The first workgroups (one per compute unit) take the
    // blocks longest walk first; the next batch, which joins them on the same compute units, takes
    // them shortest first, and so on in turns: two workgroups that share a compute unit have
    // about the same work together everywhere.
    const int linear = (int)(blockIdx.y * gridDim.x + blockIdx.x);
    const bool ascending = ((linear / a.num_cus) & 1) != 0;
    // a.pair (launches of more than two workgroups per compute unit): a workgroup takes a long and a
    // short block, one after the other, so that all workgroups have the same work and there are
    // half as many (measured: S = 4096 231 -> 180 us, S = 8192 740 -> 645 us; slower for launches
    // that are a single batch anyway).
    const int nblocks = (a.M + 127) / 128;
    const int reps = a.pair && 2 * (int)blockIdx.x + 1 < nblocks ? 2 : 1;
    // a.chunk_steps > 0 (launches with fewer blocks than compute units): the walk of a block is cut
    // into chunks of that many steps, one workgroup each, longest blocks first; a block with more
    // than one chunk leaves unnormalized partial results that a second kernel combines.
    int chunk_block = 0, chunk = 0, chunks = 1;
    if (a.chunk_steps > 0) {
        int w = blockIdx.x;
        for (int j = nblocks - 1;; --j) {
            const int last = min(j * 128 + 127, a.M - 1);
            const int cj = ((a.n_ctx - a.S + last / a.g + 1 + 31) / 32 + a.chunk_steps - 1) / a.chunk_steps;
            if (w < cj || j == 0) {
                chunk_block = j;
                chunk = w;
                chunks = cj;
                break;
            }
            w -= cj;
        }
        if (chunk >= chunks) return;  // (a grid larger than the chunk count: nothing to do)
    }
  for (int rep = 0; rep < reps; ++rep) {
    if (rep > 0) asm volatile("s_barrier" ::: "memory");  // every wavefront is done with the ring
    const int block = a.chunk_steps > 0 ? chunk_block
                      : a.pair ? (rep == 0 ? nblocks - 1 - (int)blockIdx.x : (int)blockIdx.x)
                      : ascending ? (int)blockIdx.x : (int)gridDim.x - 1 - (int)blockIdx.x;
    const int r0 = (block * 4 + (wave & 3)) * 32;             // first query row of the wavefront
    const int m = r0 + q;
    const bool real = m < a.M;
    const int lim = real ? a.n_ctx - a.S + m / a.g + 1 : a.n_ctx;
    // (the same in every lane: said explicitly, the divisions would otherwise be carried out per lane
    // and drag the loop control and the copy addresses into vector registers)
    const int lo_full = __builtin_amdgcn_readfirstlane(a.n_ctx - a.S + min(r0, a.M - 1) / a.g + 1);  // positions every row of the wavefront sees
    const int block_last = min(block * 128 + 127, a.M - 1);
    const int nb_all = __builtin_amdgcn_readfirstlane((a.n_ctx - a.S + block_last / a.g + 1 + 31) / 32);  // steps of the block's walk
    // the steps this workgroup takes: [sb, nb)
    const int sb = a.chunk_steps > 0 ? chunk * a.chunk_steps : 0;
    const int nb = a.chunk_steps > 0 ? min(nb_all, sb + a.chunk_steps) : nb_all;

    // Q^T operand: lane (q, h) holds Q[m][16 j + 8 h .. + 7]
    u32x4 qf[DJ];
#pragma unroll
    for (int j = 0; j < DJ; ++j) {
        const u32x4 zero = {0, 0, 0, 0};
        qf[j] = real ? *reinterpret_cast<const u32x4 *>(a.q + ((size_t)G * a.M + m) * D + 16 * j + 8 * h) : zero;
    }
    v16f acc[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
    float run_max = kNegBig, run_sum = 0.0f;
    float run_max_final = kNegBig;  // the maximum over the steps actually taken (run_max runs a step ahead)

    // ---- copies: the stage's bytes are CP * 4 KiB pieces; wavefront w issues pieces w, w + 4, ..
    const char *kbase = reinterpret_cast<const char *>(a.kc + (size_t)G * a.C * D);
    const char *vbase = reinterpret_cast<const char *>(a.vc + (size_t)G * D * a.C);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds_raw;
    uint32_t src_off[CP];  // byte offset of this lane's 16 bytes inside the step's K rows / V block (step-invariant part)
#pragma unroll
    for (int i = 0; i < CP; ++i) {
        const int piece = wave + NW * i;     // KiB piece of the stage
        const int L = piece * 64 + lane;     // linear 16-byte chunk of the stage
        if (piece < Cfg::KBYTES / 1024) {
            const int p = L / Cfg::CPR, o = (L % Cfg::CPR) ^ Cfg::swz(p);
            src_off[i] = (uint32_t)(p * (2 * D) + o * 16);
        } else {
            const int Lv = L - Cfg::KBYTES / 16;
            const int d = Lv >> 2, c = (Lv & 3) ^ ((d >> 2) & 3);
            src_off[i] = (uint32_t)(d * 128 + c * 16);
        }
    }
    auto issue = [&](int blk) {
        // past the end the walk's first steps are copied again (constant operation counts), into one
        // spare KiB behind the ring that nothing reads (and from distinct sources: many copies of the
        // same lines in flight had been seen in ring slots after the counter said they were done;
        // the cause is not known, so a late copy gets no destination that anything reads)
        const int bc = blk < nb ? blk : min(sb + (blk - nb), nb - 1);
        const int p0 = bc * 32;
        const char *ksrc = kbase + (size_t)p0 * (2 * D);
        const char *vsrc = vbase + (size_t)(p0 / 64) * D * 128 + (p0 % 64) * 2;
#pragma unroll
        for (int i = 0; i < CP; ++i) {
            const int piece = wave + NW * i;
            const bool is_k = piece < Cfg::KBYTES / 1024;
            // (the address is the same in every lane; saying so keeps it in scalar registers for the copy)
            const uint64_t addr = reinterpret_cast<uint64_t>(is_k ? ksrc : vsrc);
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)addr);
            const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(addr >> 32));
            copy16_to_lds(reinterpret_cast<const void *>(((uint64_t)hi << 32) | lo), src_off[i],
                          __builtin_amdgcn_readfirstlane(lds0 + (blk < nb ? (blk % NS) * Cfg::STAGE + piece * 1024 : NS * Cfg::STAGE)));
        }
    };

    // operand read offsets of this lane inside a stage
    const int pp = 16 * (q >> 4) + 8 * ((q >> 2) & 1) + 4 * ((q >> 3) & 1) + (q & 3);  // position of score-tile row q
    int koff[DJ];
#pragma unroll
    for (int j = 0; j < DJ; ++j) koff[j] = pp * (2 * D) + (((2 * j + h) ^ Cfg::swz(pp)) * 16);
    int voff[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int d = 32 * (dt + (wave >> 2) * DT) + q;
            voff[dt][c] = Cfg::KBYTES + d * 64 + (((2 * c + h) ^ ((d >> 2) & 3)) * 16);
        }

#pragma unroll
    for (int p = 0; p < NS - 1; ++p) issue(sb + p);
    // The scores of step blk + 1 are computed while the softmax of step blk runs: their MFMAs do
    // not depend on it, so the matrix core works through them while the vector unit does the
    // exponentials (from one wavefront the two would otherwise take turns).
    auto scores = [&](int blk_) {
        const char *stage_ = reinterpret_cast<const char *>(lds_raw) + (blk_ % NS) * Cfg::STAGE;
        u32x4 kf[DJ];
#pragma unroll
        for (int j = 0; j < DJ; ++j) kf[j] = *reinterpret_cast<const u32x4 *>(stage_ + koff[j]);
        v16f r;
#pragma unroll
        for (int e = 0; e < 16; ++e) r[e] = 0.0f;
#pragma unroll
        for (int j = 0; j < DJ; ++j)
            r = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, kf[j]), __builtin_bit_cast(h8, qf[j]), r, 0, 0, 0);
        return r;
    };
    wait_vmcnt<(NS - 2) * CP>();
    asm volatile("s_barrier" ::: "memory");
    v16f st = scores(sb);
    // The softmax of a step is cut in two.  Its first part (running maximum and the correction of
    // the sums so far) only needs the step's scores, so it runs a step ahead, between the MFMAs of
    // the previous step's second product; its second part (exponentials, sums, conversion) runs
    // between the MFMAs of the next step's scores.  From one wavefront the matrix core and the
    // vector unit would otherwise take turns.
    // EDGE = some row of the wavefront does not see all 32 positions of the step (causal horizon or
    // end of the context); the steps before a wavefront's first such step run branch-free bodies in
    // which the compiler is told to issue the MFMAs one at a time between the vector instructions.
    auto max_part = [&](const v16f &sv, int k0, auto edge_c) {
        constexpr bool EDGE = decltype(edge_c)::value;
        // register e = 8 c + 4 b + r of lane (q, h): position k0 + 8 h + (16 c + 4 b + r)
        const int room = lim - k0 - 8 * h;
        float bmax = kNegBig;
#pragma unroll
        for (int e = 0; e < 16; ++e) bmax = fmaxf(bmax, !EDGE || 16 * (e >> 3) + (e & 7) < room ? sv[e] : kNegBig);
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float new_max = fmaxf(run_max, bmax * a.scale);  // kNegBig * scale stays hugely negative
        const float c = __builtin_amdgcn_exp2f(run_max - new_max);
        run_max = new_max;
        return c;
    };
    float corr = max_part(st, sb * 32, std::true_type{});
    auto step = [&](int blk, auto edge_c, auto edge_next_c) {
        constexpr bool EDGE = decltype(edge_c)::value;
        const int k0 = blk * 32;
        // stage blk + 1 has landed (past the end: a copy of the last stage), and every wavefront is
        // done with stage blk - 1, whose slot the next copies overwrite
        wait_vmcnt<(NS - 3) * CP>();
        asm volatile("s_barrier" ::: "memory");
        issue(blk + NS - 1);
        // (the one branch of a step comes first, so that the rest is one block for the scheduler)
        if (__any(corr != 1.0f)) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[dt][e] *= corr;
        }
        const char *stage = reinterpret_cast<const char *>(lds_raw) + (blk % NS) * Cfg::STAGE;
        u32x4 vf[DT][2];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int c = 0; c < 2; ++c) vf[dt][c] = *reinterpret_cast<const u32x4 *>(stage + voff[dt][c]);
        const v16f st_next = scores(blk + 1);
        // raw scores; the scale (in units of log 2) is applied inside the exponent: 2^(s scale - maximum)
        const int room = lim - k0 - 8 * h;
        const float cur_max = run_max;
        run_max_final = cur_max;
        float psum = 0.0f;
        h8 pv[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float p = __builtin_amdgcn_exp2f(fmaf(st[e], a.scale, -cur_max));
            if (EDGE) p = 16 * (e >> 3) + (e & 7) < room ? p : 0.0f;
            psum += p;
            pv[e >> 3][e & 7] = (_Float16)p;
        }
        run_sum = run_sum * corr + psum;
        if (EDGE && k0 + 32 > a.n_ctx) {  // positions past the context may hold anything
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int p0 = k0 + 16 * c + 8 * h;
                    uint32_t w[4] = {vf[dt][c].x, vf[dt][c].y, vf[dt][c].z, vf[dt][c].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (p0 + 2 * e >= a.n_ctx) w[e] &= 0xFFFF0000u;
                        if (p0 + 2 * e + 1 >= a.n_ctx) w[e] &= 0x0000FFFFu;
                    }
                    vf[dt][c] = u32x4{w[0], w[1], w[2], w[3]};
                }
        }
        __builtin_amdgcn_s_setprio(1);
        // (positions 0..15 of the step first: their probabilities are ready first)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, vf[dt][c]), pv[c], acc[dt], 0, 0, 0);
        // first part of the next step's softmax (past the last step: of scores nobody uses)
        corr = max_part(st_next, k0 + 32, edge_next_c);
        __builtin_amdgcn_s_setprio(0);
        if (!EDGE && !decltype(edge_next_c)::value) {
            // order asked of the scheduler: the operand reads, then every score MFMA followed by a
            // share of the exponential part, then every MFMA of the second product followed by a
            // share of the maximum part
            if (HALVES == 1) __builtin_amdgcn_sched_group_barrier(0x100, DJ + 2 * DT, 0);
#pragma unroll
            for (int j = 0; j < DJ; ++j) {  // score MFMAs, the exponentials of the step's first 16 positions
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 32 / DJ, 0);
            }
#pragma unroll
            for (int j = 0; j < DT; ++j) {  // second product over those positions, the other exponentials
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 32 / DT, 0);
            }
#pragma unroll
            for (int j = 0; j < DT; ++j) {  // second product over the rest, the next step's maximum part
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 16 / DT, 0);
            }
        }
        st = st_next;
    };
    const int nfull = min(nb, lo_full / 32);  // steps in which every row of the wavefront sees all positions
    int blk = sb;
    for (; blk < nfull - 1; ++blk) step(blk, std::false_type{}, std::false_type{});
    for (; blk < nfull; ++blk) step(blk, std::false_type{}, std::true_type{});
    for (; blk < nb; ++blk) step(blk, std::true_type{}, std::true_type{});
    wait_vmcnt<0>();  // the redundant copies past the end have landed before the workgroup leaves
    run_sum += __shfl_xor(run_sum, 32, 64);
    if (real && chunks > 1) {
        // partial result of this chunk: unnormalized O^T column, maximum (in units of log 2) and sum
        const size_t slot = ((size_t)G * a.M + m) * a.max_chunks + chunk;
        float *dst = a.ws_o + slot * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                *reinterpret_cast<v4f *>(dst + 32 * (dt + (wave >> 2) * DT) + 8 * b + 4 * h) =
                    v4f{acc[dt][4 * b + 0], acc[dt][4 * b + 1], acc[dt][4 * b + 2], acc[dt][4 * b + 3]};
        if (h == 0 && wave < 4) {
            a.ws_ml[slot * 2] = run_max_final;
            a.ws_ml[slot * 2 + 1] = run_sum;
        }
    } else if (real) {
        const float inv = 1.0f / run_sum;
        // lane (q, h) holds O^T rows d = 32 dt + 8 b + 4 h + r of column q: four consecutive d per b
        _Float16 *dst = a.out + ((size_t)G * a.M + m) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const h4 v = {(_Float16)(acc[dt][4 * b + 0] * inv), (_Float16)(acc[dt][4 * b + 1] * inv),
                              (_Float16)(acc[dt][4 * b + 2] * inv), (_Float16)(acc[dt][4 * b + 3] * inv)};
                *reinterpret_cast<h4 *>(dst + 32 * (dt + (wave >> 2) * DT) + 8 * b + 4 * h) = v;
            }
    }
  }
}

// steps of the walk of block j, and the chunks it is cut into (host side of what the kernels compute)
inline int prefill_steps(const AttnArgs &a, int j) {
    const int last = (j * 128 + 127 < a.M - 1) ? j * 128 + 127 : a.M - 1;
    return (a.n_ctx - a.S + last / a.g + 1 + 31) / 32;
}
inline int prefill_chunks(const AttnArgs &a, int j) {
    return (prefill_steps(a, j) + a.chunk_steps - 1) / a.chunk_steps;
}

// Chunked walks: the rows of blocks with more than one chunk.  One wavefront per query row; lane l
// takes the D / 64 consecutive values from d = l D / 64.
template <int D>
__global__ __launch_bounds__(256) void attn_prefill_combine_kernel(AttnArgs a) {
    constexpr int PER = D / 64;
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int G = blockIdx.y;
    if (m >= a.M) return;
    const int last = min((m / 128) * 128 + 127, a.M - 1);
    const int chunks = ((a.n_ctx - a.S + last / a.g + 1 + 31) / 32 + a.chunk_steps - 1) / a.chunk_steps;
    if (chunks <= 1) return;  // written by the first kernel
    const size_t slot0 = ((size_t)G * a.M + m) * a.max_chunks;
    // lane c < chunks holds chunk c's (maximum, sum); all loads of the row are requested at once
    static_assert(kPrefillMaxChunks == 8, "the reductions below cover eight lanes");
    float mx = kNegBig, l = 0.0f;
    if (lane < chunks) {
        mx = a.ws_ml[(slot0 + lane) * 2];
        l = a.ws_ml[(slot0 + lane) * 2 + 1];
    }
    float part[kPrefillMaxChunks][PER];
#pragma unroll
    for (int c = 0; c < kPrefillMaxChunks; ++c) {
        const float *src = a.ws_o + (slot0 + min(c, chunks - 1)) * D + lane * PER;
#pragma unroll
        for (int e = 0; e < PER; ++e) part[c][e] = src[e];
    }
    float top = mx;
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) top = fmaxf(top, __shfl_xor(top, off, 64));
    top = __shfl(top, 0, 64);
    const float f = lane < chunks ? __builtin_amdgcn_exp2f(mx - top) : 0.0f;
    float den = f * l;
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) den += __shfl_xor(den, off, 64);
    den = __shfl(den, 0, 64);
    float o[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) o[e] = 0.0f;
#pragma unroll
    for (int c = 0; c < kPrefillMaxChunks; ++c) {
        const float fc = __shfl(f, c, 64);  // 0 for c >= chunks (whose loads repeated the last chunk)
#pragma unroll
        for (int e = 0; e < PER; ++e) o[e] = fmaf(fc, part[c][e], o[e]);
    }
    const float inv = 1.0f / den;
    _Float16 *dst = a.out + ((size_t)G * a.M + m) * D + lane * PER;
#pragma unroll
    for (int e = 0; e < PER; ++e) dst[e] = (_Float16)(o[e] * inv);
}

template <int D>
hipError_t launch_attn_prefill(const AttnArgs &a, int G, hipStream_t st) {
    constexpr size_t lds = (size_t)PrefillCfg<D>::NS * PrefillCfg<D>::STAGE + 1024;  // the ring and the spare KiB
    static_assert(lds <= 160 * 1024, "LDS budget");
    static_assert((PrefillCfg<D>::NS - 1) * PrefillCfg<D>::COPIES <= 63, "outstanding copies must fit the 6-bit counter");
    if (const hipError_t e = allow_dynamic_lds<attn_prefill_kernel<D>>(lds); e != hipSuccess) return e;
    const int nblocks = (a.M + 127) / 128;
    if (a.chunk_steps > 0) {
        int total = 0;
        for (int j = 0; j < nblocks; ++j) total += prefill_chunks(a, j);
        attn_prefill_kernel<D><<<dim3((unsigned)total, (unsigned)G), 64 * PrefillCfg<D>::NW, lds, st>>>(a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        attn_prefill_combine_kernel<D><<<dim3((unsigned)((a.M + 3) / 4), (unsigned)G), 256, 0, st>>>(a);
        return hipGetLastError();
    }
    attn_prefill_kernel<D><<<dim3((unsigned)(a.pair ? (nblocks + 1) / 2 : nblocks), (unsigned)G), 64 * PrefillCfg<D>::NW, lds, st>>>(a);
    return hipGetLastError();
}

template <int D>
hipError_t launch_attn(const AttnArgs &a, int G, hipStream_t st) {
    const size_t lds = (size_t)4 * 16 * (D + 4) * sizeof(float);
    if (const hipError_t e = allow_dynamic_lds<attn_partial_kernel<D>>(lds); e != hipSuccess) return e;
    attn_partial_kernel<D><<<dim3((unsigned)a.splits, (unsigned)G), 256, lds, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1) return e;
    attn_combine_kernel<D><<<dim3((unsigned)a.M, (unsigned)G, D / 64), 64, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace

// Workgroups per (batch, KV head) group: enough wavefronts to fill the chip, at least one block
// of 32 positions per wavefront, at most kAttnMaxSplits.
int attn_splits(int G, int n_ctx, int num_cus) {
    const int nb = (n_ctx + 63) / 64;
    int s = (8 * num_cus + 4 * G - 1) / (4 * G);
    if (s > (nb + 3) / 4) s = (nb + 3) / 4;  // at least one step of 64 positions per wavefront
    if (s > kAttnMaxSplits) s = kAttnMaxSplits;
    if (s < 1) s = 1;
    return s;
}

// The many-query-rows path needs partial results only where it may cut walks into chunks: launches
// with no more blocks of 128 query rows than compute units.
static bool prefill_may_chunk(int G, int M, int num_cus) {
    const long wgs = (long)((M + 127) / 128) * G;
    const int forced = tuning().attn_chunks;
    return forced >= 0 ? forced != 0 : wgs <= num_cus;
}

size_t attn_prefill_workspace(int G, int M, int d, int num_cus) {
    if (!prefill_may_chunk(G, M, num_cus)) return 256;
    return (size_t)G * M * kPrefillMaxChunks * (d + 2) * sizeof(float);
}

hipError_t launch_rope_qkv(const void *qkv, int B, int S, int h_q, int h_kv, int d, int C, int pos0, float base,
                           void *q_out, void *kc, void *vc, hipStream_t st) {
    const long total = (long)B * S * (h_q + 2 * h_kv) * (d / 2);
    rope_qkv_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(
        static_cast<const _Float16 *>(qkv), B, S, h_q, h_kv, d, C, pos0, log((double)base),
        static_cast<_Float16 *>(q_out), static_cast<_Float16 *>(kc), static_cast<_Float16 *>(vc));
    return hipGetLastError();
}

hipError_t launch_rope_table(int d, float base, int positions, float *table, hipStream_t st) {
    const long total = (long)positions * (d / 2);
    rope_table_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(d, positions, log((double)base), table);
    return hipGetLastError();
}

hipError_t launch_attention(const void *q, const void *kc, const void *vc, int G, int S, int g, int d, int C,
                            int n_ctx, void *workspace, void *out, int num_cus, hipStream_t st) {
    AttnArgs a;
    a.q = static_cast<const _Float16 *>(q);
    a.kc = static_cast<const _Float16 *>(kc);
    a.vc = static_cast<const _Float16 *>(vc);
    a.M = S * g;
    a.g = g;
    a.S = S;
    a.C = C;
    a.n_ctx = n_ctx;
    a.splits = attn_splits(G, n_ctx, num_cus);
    a.num_cus = num_cus > 0 ? num_cus : 1;
    {
        const long wgs = (long)((a.M + 127) / 128) * G;
        const int forced = tuning().attn_pair;
        a.pair = forced >= 0 ? forced : (wgs > 2L * a.num_cus ? 1 : 0);
        // fewer blocks than compute units: cut the walks into chunks (at most kPrefillMaxChunks per
        // block, at least 4 steps each) that fill the chip in one batch
        a.chunk_steps = 0;
        a.max_chunks = kPrefillMaxChunks;
        if (a.M > 16 && prefill_may_chunk(G, a.M, a.num_cus)) {
            const int nblocks = (a.M + 127) / 128;
            long steps_total = 0;
            int longest = 0;
            for (int j = 0; j < nblocks; ++j) {
                const int last = (j * 128 + 127 < a.M - 1) ? j * 128 + 127 : a.M - 1;
                const int nbj = (n_ctx - S + last / g + 1 + 31) / 32;
                steps_total += nbj;
                if (nbj > longest) longest = nbj;
            }
            // the shortest chunk length whose chunks are all resident at once (two workgroups per
            // compute unit up to head size 128, one above)
            const long slots = (long)a.num_cus * (d <= 128 ? 2 : 1);
            long len = (steps_total * G + slots - 1) / slots;
            const int floor_len = (longest + kPrefillMaxChunks - 1) / kPrefillMaxChunks;
            if (len < floor_len) len = floor_len;
            if (len < 4) len = 4;
            for (; len < longest; ++len) {
                long total = 0;
                for (int j = 0; j < nblocks; ++j) {
                    const int last = (j * 128 + 127 < a.M - 1) ? j * 128 + 127 : a.M - 1;
                    const int nbj = (n_ctx - S + last / g + 1 + 31) / 32;
                    total += (nbj + len - 1) / len;
                }
                if (total * G <= slots) break;
            }
            if (len < longest) {  // else every block is one chunk anyway
                // Worth it?  The launch ends with its longest walk: chunks save (longest - len) steps
                // of a workgroup (measured: about 0.6 / 0.9 / 1.4 us per step at head size 64 / 128 /
                // 256) and cost a second launch plus the partial results written and read again
                // (taken at 4 TB/s).  Many query heads per KV head with short heads lose, few heads
                // with long ones (one step is twice the work) win by up to 2x.
                double partial_bytes = 0.0;
                for (int j = 0; j < nblocks; ++j) {
                    const int last = (j * 128 + 127 < a.M - 1) ? j * 128 + 127 : a.M - 1;
                    const int nbj = (n_ctx - S + last / g + 1 + 31) / 32;
                    const long cj = (nbj + len - 1) / len;
                    if (cj > 1) partial_bytes += (double)(last - j * 128 + 1) * cj * (d + 2) * 8.0;
                }
                partial_bytes *= G;
                const double step_us = d <= 64 ? 0.6 : d <= 128 ? 0.9 : 1.4;
                const double gain_us = (double)(longest - len) * step_us;
                const double cost_us = 3.0 + partial_bytes / 4.0e6;
                if (tuning().attn_chunks > 0 || gain_us > 1.2 * cost_us) {
                    a.chunk_steps = (int)len;
                    a.pair = 0;
                }
            }
        }
    }
    a.scale = 1.4426950408889634f / sqrtf((float)d);  // scores in units of log 2
    a.ws_o = static_cast<float *>(workspace);
    a.ws_ml = a.ws_o + (size_t)G * (a.M > 16 ? kPrefillMaxChunks : kAttnMaxSplits) * a.M * d;
    a.out = static_cast<_Float16 *>(out);
    if (a.M > 16) {
        switch (d) {
            case 64: return launch_attn_prefill<64>(a, G, st);
            case 128: return launch_attn_prefill<128>(a, G, st);
            case 256: return launch_attn_prefill<256>(a, G, st);
            default: return hipErrorInvalidValue;
        }
    }
    switch (d) {
        case 64: return launch_attn<64>(a, G, st);
        case 128: return launch_attn<128>(a, G, st);
        case 256: return launch_attn<256>(a, G, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace qfc
