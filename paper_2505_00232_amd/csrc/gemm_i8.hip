// Prefill int8 product and its dequantizing epilogue (section 3.7 of the paper:
// int8 activations x pre-quantized int8 weights with integer instructions, then
// dequantization of the output):
//   acc[m,n] = sum_k xq[m,k] * Wq[n,k]        (int32, exact)
//   y[m,n]   = fp16(float(acc) * sx[m] * sw[n])
//
// Both operands arrive tiled the same way (KiB tiles of 16 rows x 64 k, lane
// (c, q) = 16 codes of row c at k = 16q).  A stage of the K loop (128 k) is a
// verbatim copy of KiB tiles into LDS, done by global_load_lds_dwordx4 (one
// wavefront instruction moves one tile from memory straight into LDS, no
// staging registers), in a ring of LDS stages that keeps several stages in
// flight, with one workgroup barrier per stage.
// An MFMA operand fragment (32 rows x 32 k, lane = row + 32 * (k / 16)) is made
// of runs of 256 contiguous LDS bytes: conflict free without padding.
//
// Workgroup: 4 wavefronts in a 2 x 2 grid over a BN x BM tile (weight rows x
// token rows); each wavefront owns (BN/2) x (BM/2) outputs as 32x32 tiles of
// v_mfma_i32_32x32x32_i8.  The weights are the row operand of the MFMA so that
// a lane ends up with 4 consecutive n of one token row (8-byte fp16 stores
// along the contiguous axis of y).  Tile ids are dealt so that every XCD works
// on a contiguous range of (weight tile, token tile) pairs and the token tiles
// that share a weight tile hit the same L2.
#include "qfc_internal.h"

namespace qfc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

__host__ __device__ inline int stages_total(int Kp, int bk) { return Kp / bk; }

struct GemmI8Args {
    const uint4 *w;   // packed weights, tiles [row tile][Kp/64][64]
    const uint4 *x;   // tiled activations, tiles [row tile][Kp/64][64]
    const float *sw;  // [Np]
    const float *sx;  // [Mp] (null for raw accumulators)
    const _Float16 *res;  // [M, N] residual added before the rounding, or null
    void *out;
    int M, N, Kp, n_tiles, m_tiles;
    // 4-bit weights enter the MFMA as 16 q (the code's nibble in the top half of a byte): the sums are
    // 16 times the definition's, exactly; channel scales are multiplied by 1/16, raw sums shifted by 4
    float sw_mul = 1.0f;
    int acc_shift = 0;
    int gated_act = -1;  // QFC_ACT_*: the layer is packed in pairs and y [M, N/2] = fp16(act(gate) * other)
};

// Store phase of a layer packed in pairs (operator fusion, section 3.6 of the paper: the element-wise
// operators of the two branches merged into the fully connected operator that produces them).
// Physical rows 32 t .. 32 t + 15 are gate rows and 32 t + 16 .. 32 t + 31 the other branch's rows of
// the same 16 channels, so a lane's accumulator registers 4 q + e (q = 0, 1) and 4 (q + 2) + e of a
// 32 x 32 tile are the two branches of one channel: scale both, multiply act(gate) with the other
// in fp32, round once.  16 TN output channels per wavefront, staged through LDS like the plain
// store phase and written as 16-byte pieces of rows of N / 2 values.
template <int TN, int TM>
__device__ __forceinline__ void epilogue_gated(const GemmI8Args &a, v16i (&acc)[TN][TM], uint4 *lds, int n_base,
                                               int m_base, int wave, int lane) {
    constexpr int WO = TN * 16;
    constexpr int PITCH = (WO + 8) * 2;  // bytes per staged row
    char *region = reinterpret_cast<char *>(lds) + wave * (32 * PITCH);
    const int half = a.N / 2;
    const int o0 = n_base / 2;  // first output channel of the wavefront
    const GateCoeffs gc = gate_coeffs(a.gated_act);
    float4 scg[TN][2], scu[TN][2];
    float sxr[TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            float4 g = *reinterpret_cast<const float4 *>(a.sw + n_base + i * 32 + 8 * q + 4 * (lane >> 5));
            float4 u = *reinterpret_cast<const float4 *>(a.sw + n_base + i * 32 + 16 + 8 * q + 4 * (lane >> 5));
            g.x *= a.sw_mul, g.y *= a.sw_mul, g.z *= a.sw_mul, g.w *= a.sw_mul;
            u.x *= a.sw_mul, u.y *= a.sw_mul, u.z *= a.sw_mul, u.w *= a.sw_mul;
            scg[i][q] = g;
            scu[i][q] = u;
        }
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m_base + j * 32 + (lane & 31);
        sxr[j] = m < a.M ? a.sx[m] : 0.0f;
    }
    asm volatile("s_barrier" ::: "memory");  // all wavefronts are done with the stage buffers
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int mrow0 = m_base + j * 32;
        const float sxm = sxr[j];
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                const float gs[4] = {scg[i][q].x, scg[i][q].y, scg[i][q].z, scg[i][q].w};
                const float us[4] = {scu[i][q].x, scu[i][q].y, scu[i][q].z, scu[i][q].w};
                h4 hv;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float g = (float)acc[i][j][4 * q + e] * sxm * gs[e];
                    const float u = (float)acc[i][j][4 * (q + 2) + e] * sxm * us[e];
                    hv[e] = (_Float16)(gate_activation(g, gc) * u);
                }
                *reinterpret_cast<h4 *>(region + (lane & 31) * PITCH + (i * 16 + 8 * q + 4 * (lane >> 5)) * 2) = hv;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int CH = WO / 8;  // 16-byte chunks per staged row
#pragma unroll
        for (int it = 0; it < 32 * CH / 64; ++it) {
            const int idx = it * 64 + lane;
            const int row = idx / CH, ch = idx % CH;
            const uint4 v = *reinterpret_cast<const uint4 *>(region + row * PITCH + ch * 16);
            const int mm = mrow0 + row, nn = o0 + ch * 8;
            if (mm < a.M && nn < half)
                *reinterpret_cast<uint4 *>(static_cast<_Float16 *>(a.out) + (size_t)mm * half + nn) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// Epilogue shared by the product kernels.
// A wavefront holds TN x TM tiles of 32 x 32 outputs whose first weight row is n_base and first
// token row is m_base.
template <int OUT_MODE, int TN, int TM>
__device__ __forceinline__ void epilogue(const GemmI8Args &a, v16i (&acc)[TN][TM], uint4 *lds, int n_base, int m_base,
                                         int wave, int lane) {
    constexpr int WN = TN * 32;
    if (OUT_MODE == 0 && a.gated_act >= 0) {
        epilogue_gated<TN, TM>(a, acc, lds, n_base, m_base, wave, lane);
        return;
    }
    // Epilogue.  After the MFMAs a lane holds one token row m (lane % 32) and, per
    // group of four accumulator registers, four consecutive n: stored as they are,
    // every store instruction would touch 32 different rows of y with 8 bytes
    // each.  The scaled binary16 values therefore take a detour through LDS (one
    // block of 32 token rows x WN channels per wavefront at a time) and leave as
    // 16-byte stores that cover whole rows segments of 2 * WN contiguous bytes.
    if (OUT_MODE == 0 && (a.N % 8) == 0) {
        constexpr int PITCH = (WN + 8) * 2;  // bytes per staged row
        char *region = reinterpret_cast<char *>(lds) + wave * (32 * PITCH);
        const int n0 = n_base;
        // the scales of the lane's channels and token rows, requested once and before the barrier
        // (inside the loop over the row blocks they would be fetched again after every fence)
        float4 scw[TN][4];
        float sxr[TM];
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
            {
                float4 v = *reinterpret_cast<const float4 *>(a.sw + n0 + i * 32 + 8 * q + 4 * (lane >> 5));
                v.x *= a.sw_mul, v.y *= a.sw_mul, v.z *= a.sw_mul, v.w *= a.sw_mul;  // (1 or 1/16: exact)
                scw[i][q] = v;
            }
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m_base + j * 32 + (lane & 31);
            sxr[j] = m < a.M ? a.sx[m] : 0.0f;
        }
        asm volatile("s_barrier" ::: "memory");  // all wavefronts are done with the stage buffers
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int mrow0 = m_base + j * 32;
            const float sxm = sxr[j];
            const bool has_res = a.res != nullptr;
            if (has_res) stage_residual_block<WN / 8, PITCH>(region, a.res, mrow0, n0, a.M, a.N, lane);
#pragma unroll
            for (int i = 0; i < TN; ++i) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = i * 32 + 8 * q + 4 * (lane >> 5);
                    const float4 sc = scw[i][q];
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    float v[4] = {(float)acc[i][j][4 * q + 0] * sxm * sc.x, (float)acc[i][j][4 * q + 1] * sxm * sc.y,
                                  (float)acc[i][j][4 * q + 2] * sxm * sc.z, (float)acc[i][j][4 * q + 3] * sxm * sc.w};
                    if (has_res) {
                        float rv[4];
                        staged_residual4(region, (lane & 31) * PITCH + nl * 2, rv);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += rv[e];
                    }
                    const h4 hv = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
                    *reinterpret_cast<h4 *>(region + (lane & 31) * PITCH + nl * 2) = hv;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            constexpr int CH = WN / 8;  // 16-byte chunks per staged row
#pragma unroll
            for (int it = 0; it < 32 * CH / 64; ++it) {
                const int idx = it * 64 + lane;
                const int row = idx / CH, ch = idx % CH;
                const uint4 v = *reinterpret_cast<const uint4 *>(region + row * PITCH + ch * 16);
                const int mm = mrow0 + row, nn = n0 + ch * 8;
                if (mm < a.M && nn < a.N)
                    *reinterpret_cast<uint4 *>(static_cast<_Float16 *>(a.out) + (size_t)mm * a.N + nn) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        return;
    }
    asm volatile("s_barrier" ::: "memory");  // all wavefronts are done with the stage buffers
    // generic path (raw accumulators, or N not a multiple of 8): direct stores
    const bool vec_ok = (a.N % 4) == 0;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m_base + j * 32 + (lane & 31);
        if (m >= a.M) continue;
        float sxm = 1.0f;
        if (OUT_MODE == 0) sxm = a.sx[m];
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n_base + i * 32 + 8 * q + 4 * (lane >> 5);
                if (n >= a.N) continue;
                if (OUT_MODE == 0) {
                    _Float16 *y = static_cast<_Float16 *>(a.out) + (size_t)m * a.N + n;
                    const float4 s = *reinterpret_cast<const float4 *>(a.sw + n);
                    const float sv[4] = {s.x * a.sw_mul, s.y * a.sw_mul, s.z * a.sw_mul, s.w * a.sw_mul};
                    _Float16 h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float v = (float)acc[i][j][4 * q + e] * sxm * sv[e];
                        if (a.res && n + e < a.N) v += (float)a.res[(size_t)m * a.N + n + e];
                        h[e] = (_Float16)v;
                    }
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
                    const int sh = a.acc_shift;  // (arithmetic shift of an exact multiple: exact)
                    if (vec_ok) {
                        *reinterpret_cast<int4 *>(o) = make_int4(acc[i][j][4 * q] >> sh, acc[i][j][4 * q + 1] >> sh,
                                                                 acc[i][j][4 * q + 2] >> sh, acc[i][j][4 * q + 3] >> sh);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < a.N) o[e] = acc[i][j][4 * q + e] >> sh;
                    }
                }
            }
        }
    }
}

// KTS = KiB k tiles (64 k each) per stage, NS = LDS stages (prefetch distance NS - 1)
template <int BN, int BM, int KTS, int NS, int OUT_MODE>
__global__ __launch_bounds__(256, (BN * BM > 128 * 256) ? 1 : 2) void gemm_i8_kernel(GemmI8Args a) {
    constexpr int BK = KTS * 64;
    constexpr int WN = BN / 2, WM = BM / 2;    // per-wavefront tile
    constexpr int TN = WN / 32, TM = WM / 32;  // 32x32 MFMA tiles per wavefront
    constexpr int W_TILES = BN / 16 * KTS, X_TILES = BM / 16 * KTS;  // KiB tiles per stage
    constexpr int STAGE_VECS = (W_TILES + X_TILES) * 64;
    extern __shared__ uint4 lds[];  // NS stages: [stage][W tiles | X tiles][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1, wm = wave >> 1;

    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles;
    const int mt = logical % a.m_tiles;
    const int KT = a.Kp / 64;

    // One wavefront instruction copies one KiB tile: tile t of the stage, t = wave,
    // wave + 4, ...  The tiles of one row tile are contiguous along K, so the source
    // of a tile advances by a constant per stage; the stage-0 pointers are
    // computed once.
    constexpr int NLOAD = (W_TILES + X_TILES) / 4;
    const uint4 *src0[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int t = wave + 4 * i;
        if (t < W_TILES)
            src0[i] = a.w + ((size_t)(nt * (BN / 16) + t / KTS) * KT + t % KTS) * 64 + lane;
        else
            src0[i] = a.x + ((size_t)(mt * (BM / 16) + (t - W_TILES) / KTS) * KT + (t - W_TILES) % KTS) * 64 + lane;
    }
    auto issue_stage = [&](int kt, int buf) {
        uint4 *dst = lds + buf * STAGE_VECS + wave * 64;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(src0[i] + (size_t)kt * (KTS * 64)), (lptr_t)(dst + i * 256), 16, 0, 0);
    };

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    // Software pipeline over k steps of 32.  While the MFMAs of step s run, the
    // fragments of step s + 1 are already being read from LDS (double-buffered in
    // registers; scheduling barriers keep the reads ahead of the MFMA block), and
    // NS - 1 stages of global -> LDS copies are in flight.  When step s + 1 is the
    // first of the next stage, the wait for that stage and the workgroup barrier
    // come before its reads, i.e. before the MFMAs of the last step of the current
    // stage.  The barrier is a bare s_barrier: __syncthreads() would drain every
    // outstanding copy and cancel the prefetch distance.  The copy issued after the
    // barrier overwrites the buffer of the stage that is ending: every wavefront
    // waited for its own last LDS reads of that stage before the barrier.
    constexpr int KS = BK / 32;
    auto load_frags = [&](v4i(&fa)[TN], v4i(&fb)[TM], int buf, int ks) {
        const uint4 *lw = lds + buf * STAGE_VECS;
        const uint4 *lx = lw + W_TILES * 64;
        const int kc = 2 * ks + (lane >> 5);              // 16-code chunk inside the stage
        const int koff = (kc >> 2) * 64 + (kc & 3) * 16;  // k tile and quarter
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int row = wn * WN + i * 32 + (lane & 31);
            fa[i] = __builtin_bit_cast(v4i, lw[(row >> 4) * (KTS * 64) + koff + (row & 15)]);
        }
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int row = wm * WM + j * 32 + (lane & 31);
            fb[j] = __builtin_bit_cast(v4i, lx[(row >> 4) * (KTS * 64) + koff + (row & 15)]);
        }
    };
    auto stage_ready = [&](int kt) {  // stage kt has landed for the whole workgroup
        if (kt + NS - 2 < stages_total(a.Kp, BK))
            wait_vmcnt<(NS - 2) * NLOAD>();
        else
            wait_vmcnt<0>();
        asm volatile("s_barrier" ::: "memory");
    };
    const int stages = stages_total(a.Kp, BK);
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < stages) issue_stage(p, p);
    v4i fa[2][TN], fb[2][TM];
    stage_ready(0);
    if (NS - 1 < stages) issue_stage(NS - 1, NS - 1);
    load_frags(fa[0], fb[0], 0, 0);
    for (int kt = 0; kt < stages; ++kt) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            constexpr int kKsLast = KS - 1;
            if (ks < kKsLast) {
                load_frags(fa[(ks + 1) & 1], fb[(ks + 1) & 1], kt % NS, ks + 1);
            } else if (kt + 1 < stages) {
                stage_ready(kt + 1);
                if (kt + NS < stages) issue_stage(kt + NS, (kt + NS) % NS);
                load_frags(fa[(ks + 1) & 1], fb[(ks + 1) & 1], (kt + 1) % NS, 0);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of this step's MFMAs
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    epilogue<OUT_MODE, TN, TM>(a, acc, lds, nt * BN + wn * WN, mt * BM + wm * WM, wave, lane);
}

// int8 activations x 4-bit per-channel weights (the "8/4/4" scheme of section 4.2 in the prefill
// stage of section 3.7): the same pipeline as gemm_i8_kernel with stages of 128 k.  A stage holds
// one packed KiB tile per 16 weight rows (16 rows x 128 k of 4-bit codes, copied verbatim) and
// two activation tiles per 16 token rows, the latter written by the quantizer in the k order of
// the packed codes.  A lane reads the two dwords of its packed vector that belong to a k step and
// expands them in registers: code u = q + 8 in a nibble becomes the byte (u ^ 8) << 4, which the
// MFMA reads as the signed value 16 q (5 vector instructions per 8 codes), so the int32 sums are
// exactly 16 times the definition's and the epilogue divides them out (scale * 1/16, or a shift).
template <int BN, int BM, int NS, int OUT_MODE>
__global__ __launch_bounds__(256, 2) void gemm_i8_w4_kernel(GemmI8Args a) {
    constexpr int WN = BN / 2, WM = BM / 2;
    constexpr int TN = WN / 32, TM = WM / 32;
    constexpr int W_TILES = BN / 16, X_TILES = BM / 16 * 2;  // KiB tiles per stage
    constexpr int STAGE_VECS = (W_TILES + X_TILES) * 64;
    static_assert((W_TILES + X_TILES) % 4 == 0, "tiles of a stage are dealt to four wavefronts");
    extern __shared__ uint4 lds[];  // NS stages: [stage][W tiles | X tiles][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1, wm = wave >> 1;
    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles;
    const int mt = logical % a.m_tiles;
    const int stages = a.Kp / 128;

    constexpr int NLOAD = (W_TILES + X_TILES) / 4;
    const uint4 *src0[NLOAD];
    int adv[NLOAD];  // vectors a tile's source advances per stage
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int t = wave + 4 * i;
        if (t < W_TILES) {
            src0[i] = a.w + ((size_t)(nt * (BN / 16) + t) * stages) * 64 + lane;
            adv[i] = 64;
        } else {
            const int tx = t - W_TILES;
            src0[i] = a.x + ((size_t)(mt * (BM / 16) + tx / 2) * (2 * stages) + tx % 2) * 64 + lane;
            adv[i] = 128;
        }
    }
    auto issue_stage = [&](int kt, int buf) {
        uint4 *dst = lds + buf * STAGE_VECS + wave * 64;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(src0[i] + (size_t)kt * adv[i]), (lptr_t)(dst + i * 256), 16, 0, 0);
    };

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    constexpr int KS = 4;  // k steps of 32 per stage: step ks = (op, half step) = (ks >> 1, ks & 1)
    auto load_frags = [&](v4i(&fa)[TN], v4i(&fb)[TM], int buf, int ks) {
        const char *lw = reinterpret_cast<const char *>(lds + buf * STAGE_VECS);
        const uint4 *lx = lds + buf * STAGE_VECS + W_TILES * 64;
        const int q = 2 * (ks & 1) + (lane >> 5);  // octet of the runs 2 op, 2 op + 1 this lane takes
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int row = wn * WN + i * 32 + (lane & 31);
            const uint2 p = *reinterpret_cast<const uint2 *>(lw + ((row >> 4) * 64 + q * 16 + (row & 15)) * 16 + (ks >> 1) * 8);
            fa[i][0] = (int)(((p.x << 4) & 0xF0F0F0F0u) ^ 0x80808080u);  // codes 0..3 of the first run's octet
            fa[i][1] = (int)((p.x & 0xF0F0F0F0u) ^ 0x80808080u);         // codes 4..7
            fa[i][2] = (int)(((p.y << 4) & 0xF0F0F0F0u) ^ 0x80808080u);  // the second run's octet
            fa[i][3] = (int)((p.y & 0xF0F0F0F0u) ^ 0x80808080u);
        }
        const int kc = 2 * ks + (lane >> 5);  // 16-code chunk inside the stage: tile kc >> 2, quarter kc & 3
        const int koff = (kc >> 2) * 64 + (kc & 3) * 16;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int row = wm * WM + j * 32 + (lane & 31);
            fb[j] = __builtin_bit_cast(v4i, lx[(row >> 4) * 128 + koff + (row & 15)]);
        }
    };
    auto stage_ready = [&](int kt) {  // stage kt has landed for the whole workgroup
        if (kt + NS - 2 < stages)
            wait_vmcnt<(NS - 2) * NLOAD>();
        else
            wait_vmcnt<0>();
        asm volatile("s_barrier" ::: "memory");
    };
    static_assert((NS - 1) * NLOAD <= 63, "outstanding copies must fit the 6-bit counter");
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < stages) issue_stage(p, p);
    v4i fa[2][TN], fb[2][TM];
    stage_ready(0);
    if (NS - 1 < stages) issue_stage(NS - 1, NS - 1);
    load_frags(fa[0], fb[0], 0, 0);
    for (int kt = 0; kt < stages; ++kt) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks < KS - 1) {
                load_frags(fa[(ks + 1) & 1], fb[(ks + 1) & 1], kt % NS, ks + 1);
            } else if (kt + 1 < stages) {
                stage_ready(kt + 1);
                if (kt + NS < stages) issue_stage(kt + NS, (kt + NS) % NS);
                load_frags(fa[(ks + 1) & 1], fb[(ks + 1) & 1], (kt + 1) % NS, 0);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of this step's MFMAs
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    epilogue<OUT_MODE, TN, TM>(a, acc, lds, nt * BN + wn * WN, mt * BM + wm * WM, wave, lane);
}

// Variant with the weights going from memory straight into the MFMA operand registers.  The packed
// layout already is operand order (a lane's 16 bytes of a KiB tile are 16 consecutive k of one row),
// so only the activations, which all four wavefronts share, pass through LDS: 64 instead of 96-128
// LDS bytes per clock at full MFMA rate.  Tile 256 (n) x 128 (m); wavefront w owns weight rows
// 64 w .. 64 w + 63 and all 128 token rows (2 x 4 tiles of 32 x 32, 128 accumulator registers) and
// loads only its own weights, PW stages of 64 k ahead, into a ring of registers (slot = stage % PW,
// refilled right after the MFMAs that consumed it).  Activation stages: ring of NS LDS stages of
// 8 KiB (4 KiB for the 64-row tile), CP tile copies per wavefront and stage; the ring is deep (8-14
// stages) because the wait count that is safe for both kinds of operation grows with it (see below).  Copies and loads past the end of K start
// over at stage 0, so that every iteration issues the same number of operations and the waits are
// constants.  Such copies go to a spare KiB behind the ring that is never read (and their sources
// are distinct stages, not one stage over and over: with about ten copies of the same lines in
// flight from one wavefront, data had been seen in ring slots after the counter had dropped to zero;
// the cause is not known, so no late copy may have a destination that anything reads or reuses).
// The number of stages must be a multiple of PW.
// TM = 4: 256 x 128 tile; TM = 2: 256 x 64 tile (twice the tiles for small outputs, twice the weight
// loads per MFMA).
//
// PIPE: the operand reads of stage kt + 1 are issued in the middle of the MFMAs of stage kt (second set
// of fragment registers; the ring is one stage deeper because a stage must have landed one step
// earlier).  A wavefront that is alone on its SIMD (launches of at most one workgroup per compute unit)
// otherwise spends 180 of its ~640 clocks per stage between the barrier and the first MFMA waiting
// for LDS (cycle counters inside the kernel); measured 4-6 % on such launches in the steady state,
// level elsewhere.
//
// The weight loads carry no streaming hint: the workgroups of the same weight tile (one per token tile)
// run side by side on one XCD, and with the lines marked evict-first the later ones miss in L2
// (measured: 4-19 % slower on every shape).
//
// The weight loads are assembly too: the compiler counts only the loads it knows when it places its
// waits, and with the copies in between those waits would drain most of the prefetch.  A load's
// destination registers are handed back to the compiler (an empty asm that "redefines" them) right
// after the explicit wait that covers the load, so that no MFMA can be scheduled ahead of that wait.
template <int NS, int PW, int TM, int OUT_MODE, bool PIPE = false>
__global__ __launch_bounds__(256, 2) void gemm_i8_dw_kernel(GemmI8Args a) {
    constexpr int BN = 256, BM = 32 * TM, TN = 2;
    constexpr int XT = BM / 16;  // activation tiles (KiB) per stage
    constexpr int CP = XT / 4;   // copies per wavefront and stage
    static_assert(NS >= 3 && (TM == 2 || TM == 4), "tile shapes");
    extern __shared__ uint4 lds[];  // NS stages of XT tiles x 64 vectors
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles, mt = logical % a.m_tiles;
    const int KT = a.Kp / 64;  // stages

    // weights: operand (i, ks) of a stage = rows 32 i + (lane & 31) of the wavefront's 64, k = 32 ks + 16 (lane >> 5) ..
    const uint4 *wsrc[TN];
#pragma unroll
    for (int i = 0; i < TN; ++i) {
        const int row = 32 * i + (lane & 31);
        wsrc[i] = a.w + ((size_t)(nt * (BN / 16) + 4 * wave + (row >> 4)) * KT) * 64 + (lane >> 5) * 16 + (row & 15);
    }
    v4i wreg[PW][TN][2];
    auto load_w = [&](int slot, int kt, const bool bulk) __attribute__((always_inline)) {  // bulk: kt < KT is known
        const int kc = bulk || kt < KT ? kt : min(kt - KT, KT - 1);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                asm volatile("global_load_dwordx4 %0, %1, off"
                             : "=&v"(wreg[slot][i][ks])
                             : "v"(wsrc[i] + (size_t)kc * 64 + ks * 32)
                             : "memory");
    };
    // activations: tiles wave (and wave + 4) of the XT token-row tiles of a stage
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)lds;
    const uint4 *xsrc = a.x + ((size_t)(mt * (BM / 16)) * KT) * 64;
    // Copies past the end of K (issued so that every iteration has the same operation count and the
    // waits stay constants) read the first stages again and all land in one spare KiB behind the
    // ring that nothing ever reads and the store phase never uses: whatever their timing, they
    // cannot touch a stage or the staging area of the store phase.
    constexpr uint32_t kSpare = NS * XT * 1024;
    auto issue_x = [&](int kt, const bool bulk) __attribute__((always_inline)) {  // bulk: kt < KT is known
        const bool real = bulk || kt < KT;
        const int kc = real ? kt : min(kt - KT, KT - 1);
#pragma unroll
        for (int h = 0; h < CP; ++h) {
            const int t = wave + 4 * h;
            copy16_to_lds(xsrc + ((size_t)t * KT + kc) * 64, lane * 16, lds0 + (real ? ((kt % NS) * XT + t) * 1024 : kSpare));
        }
    };

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    // prologue: PW weight stages, then NS - 1 activation stages
    constexpr bool kBulk = true, kEdge = false;  // (constants at every call site: the tests fold away)
#pragma unroll
    for (int p = 0; p < PW; ++p) load_w(p, p, kEdge);
#pragma unroll
    for (int p = 0; p < NS - 1; ++p) issue_x(p, kEdge);

    // Waiting.  Copies into LDS and loads into registers share one counter (vmcnt) but do NOT complete
    // in order relative to each other - only within their own kind (measured: with waits that assumed
    // one common order, stages were read before their copies had landed).  At the top of iteration kt
    // a wavefront has issued, after the copies of stage kt, the copies of NS - 2 later stages (CP each),
    // and after the loads of stage kt the loads of PW - 1 later stages (4 each) - from iteration 0 on,
    // thanks to the prologue.  If at most kAllowed = min(CP (NS - 2), 4 (PW - 1)) operations are
    // outstanding, neither stage kt's copies nor its loads can be among them: an unfinished copy would
    // have all CP (NS - 2) later copies behind it, an unfinished load all 4 (PW - 1) later loads.
    // With PIPE it is stage kt + 1 whose copies must have landed (its operands are read during stage
    // kt), which has one stage fewer behind it.
    constexpr int kAfterCopies = CP * (NS - (PIPE ? 3 : 2)), kAfterLoads = 4 * (PW - 1);
    constexpr int kAllowed = kAfterCopies < kAfterLoads ? kAfterCopies : kAfterLoads;
    // The most vector-memory operations a wavefront ever has outstanding: the copies of NS - 1 stages
    // and the loads of PW stages (right after the refills of an iteration).  The counter has 6 bits.
    static_assert(kAllowed >= 0 && CP * (NS - 1) + 4 * PW <= 63, "wait counts must fit the 6-bit counter");
    v4i xf[PIPE ? 2 : 1][2][TM];
    auto read_x = [&](int b, int kt) {
        const uint4 *lx = lds + (kt % NS) * (XT * 64);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int row = 32 * j + (lane & 31);
                xf[b][ks][j] = __builtin_bit_cast(v4i, lx[(row >> 4) * 64 + (2 * ks + (lane >> 5)) * 16 + (row & 15)]);
            }
    };
    if (PIPE) {
        wait_vmcnt<kAfterCopies + CP < 4 * PW ? kAfterCopies + CP : 4 * PW>();  // stage 0's copies have landed
        asm volatile("s_barrier" ::: "memory");
        read_x(0, 0);
    }
    // PW stages per pass.  The passes whose copies and loads all lie inside K come first and carry no
    // end-of-K tests; the last ones redirect what lies past the end.
    auto stages_pw = [&](int kt0, const bool bulk) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < PW; ++u) {
            const int kt = kt0 + u;
            if (PIPE)
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kAllowed) : "memory");  // (not the LDS counter: the next stage's operand reads stay in flight)
            else
                wait_vmcnt<kAllowed>();
            asm volatile("s_barrier" ::: "memory");
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) asm volatile("" : "+v"(wreg[u][i][ks]));
            issue_x(kt + NS - 1, bulk);
            const int cur = PIPE ? (u & 1) : 0;
            if (!PIPE) read_x(0, kt);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int j = 0; j < TM; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[u][i][ks], xf[cur][ks][j], acc[i][j], 0, 0, 0);
                if (PIPE && ks == 0) read_x(cur ^ 1, kt + 1);
            }
            load_w(u, kt + PW, bulk);
        }
    };
    static_assert(NS - 1 >= PW, "a pass whose copies lie inside K has its loads inside K too");
    int kt0 = 0;
    for (; kt0 + PW - 1 + NS - 1 < KT; kt0 += PW) stages_pw(kt0, kBulk);
    for (; kt0 < KT; kt0 += PW) stages_pw(kt0, kEdge);
    wait_vmcnt<0>();
    // The loads issued past the end of K are still writing their destination registers until this
    // wait returns, and the compiler does not know (it sees registers that nobody reads any more).
    // Naming them as inputs here keeps them allocated until after the wait, and the memory clobber
    // keeps the store phase's own loads from being moved above it.
#pragma unroll
    for (int p = 0; p < PW; ++p)
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) asm volatile("" ::"v"(wreg[p][i][ks]) : "memory");
    epilogue<OUT_MODE, TN, TM>(a, acc, lds, nt * BN + wave * 64, mt * BM, wave, lane);
}

template <int NS, int PW, int TM, int OUT_MODE, bool PIPE = false>
hipError_t launch_dw(GemmI8Args a, hipStream_t st) {
    constexpr size_t ring_bytes = (size_t)NS * (2 * TM) * 1024;  // + one spare KiB for the copies past the end of K
    constexpr size_t lds_bytes = ring_bytes + 1024;
    static_assert(ring_bytes >= 4 * 32 * (64 + 8) * 2, "the store phase stages its blocks inside the ring, below the spare KiB");
    if ((a.Kp / 64) % PW != 0) return hipErrorInvalidValue;
    static_assert(lds_bytes <= 80 * 1024, "two workgroups per compute unit");
    if (const hipError_t e = allow_dynamic_lds<gemm_i8_dw_kernel<NS, PW, TM, OUT_MODE, PIPE>>(lds_bytes); e != hipSuccess) return e;
    a.n_tiles = (a.N + 255) / 256;
    a.m_tiles = (a.M + 32 * TM - 1) / (32 * TM);
    gemm_i8_dw_kernel<NS, PW, TM, OUT_MODE, PIPE><<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, lds_bytes, st>>>(a);
    return hipGetLastError();
}

// The same direct-weights form for 4-bit per-channel weights.  A stage is 128 k: a lane's two packed
// vectors of a row (octets h and 2 + h of the 128 codes, h = lane / 32) feed all four k steps of the
// stage, so a stage costs 4 loads per wavefront where the 8-bit kernel needs 8 for the same k, and
// the activations (two KiB tiles per 16 token rows and stage, in the k order of the packed dwords)
// are the only operand in LDS.  The codes are expanded as in the kernel above.  Waiting, the spare
// KiB for copies past the end of K and the hand-back of the load destinations are those of the
// 8-bit kernel; the operand reads of a k step are left to the compiler (they wait on the LDS
// counter, which no asm here touches).
template <int NS, int PW, int TM, int OUT_MODE>
__global__ __launch_bounds__(256, 2) void gemm_i8_dw4_kernel(GemmI8Args a) {
    constexpr int BN = 256, BM = 32 * TM, TN = 2;
    constexpr int XT = BM / 16 * 2;  // activation tiles (KiB) per stage
    constexpr int CP = XT / 4;       // copies per wavefront and stage
    static_assert(NS >= 3 && (TM == 2 || TM == 4), "tile shapes");
    extern __shared__ uint4 lds[];  // NS stages of XT tiles x 64 vectors
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int total = a.n_tiles * a.m_tiles;
    int logical = blockIdx.x;
    if (total % 8 == 0) logical = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const int nt = logical / a.m_tiles, mt = logical % a.m_tiles;
    const int KT = a.Kp / 128;  // stages

    // weights: vector v of operand row tile i = rows 32 i + (lane & 31) of the wavefront's 64, octet 2 v + lane / 32
    const uint4 *wsrc[TN];
#pragma unroll
    for (int i = 0; i < TN; ++i) {
        const int row = 32 * i + (lane & 31);
        wsrc[i] = a.w + ((size_t)(nt * (BN / 16) + 4 * wave + (row >> 4)) * KT) * 64 + (lane >> 5) * 16 + (row & 15);
    }
    v4i wreg[PW][TN][2];
    auto load_w = [&](int slot, int kt, const bool bulk) __attribute__((always_inline)) {  // bulk: kt < KT is known
        const int kc = bulk || kt < KT ? kt : min(kt - KT, KT - 1);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v = 0; v < 2; ++v)
                asm volatile("global_load_dwordx4 %0, %1, off"
                             : "=&v"(wreg[slot][i][v])
                             : "v"(wsrc[i] + (size_t)kc * 64 + v * 32)
                             : "memory");
    };
    // activations: tile t = 2 g + e of a stage is half e of the stage's 128 k for token rows 16 g ..
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)lds;
    const uint4 *xsrc = a.x + ((size_t)(mt * (BM / 16)) * 2 * KT) * 64;
    constexpr uint32_t kSpare = NS * XT * 1024;  // copies past the end of K land here; nothing reads it
    auto issue_x = [&](int kt, const bool bulk) __attribute__((always_inline)) {
        const bool real = bulk || kt < KT;
        const int kc = real ? kt : min(kt - KT, KT - 1);
#pragma unroll
        for (int h = 0; h < CP; ++h) {
            const int t = wave + 4 * h;
            copy16_to_lds(xsrc + ((size_t)(t >> 1) * 2 * KT + 2 * kc + (t & 1)) * 64, lane * 16,
                          lds0 + (real ? ((kt % NS) * XT + t) * 1024 : kSpare));
        }
    };

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    constexpr bool kBulk = true, kEdge = false;
#pragma unroll
    for (int p = 0; p < PW; ++p) load_w(p, p, kEdge);
#pragma unroll
    for (int p = 0; p < NS - 1; ++p) issue_x(p, kEdge);

    // (see the 8-bit kernel: at most kAllowed operations outstanding means stage kt's copies and loads are done)
    constexpr int kAfterCopies = CP * (NS - 2), kAfterLoads = 4 * (PW - 1);
    constexpr int kAllowed = kAfterCopies < kAfterLoads ? kAfterCopies : kAfterLoads;
    static_assert(CP * (NS - 1) + 4 * PW <= 63, "wait counts must fit the 6-bit counter");

    auto stages_pw = [&](int kt0, const bool bulk) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < PW; ++u) {
            const int kt = kt0 + u;
            wait_vmcnt<kAllowed>();
            asm volatile("s_barrier" ::: "memory");
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v = 0; v < 2; ++v) asm volatile("" : "+v"(wreg[u][i][v]));
            issue_x(kt + NS - 1, bulk);
            const uint4 *lx = lds + (kt % NS) * (XT * 64);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {  // k step = (dword pair, vector) = (ks >> 1, ks & 1)
                v4i fa[TN], fb[TM];
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    const uint32_t px = (uint32_t)wreg[u][i][ks & 1][2 * (ks >> 1)];
                    const uint32_t py = (uint32_t)wreg[u][i][ks & 1][2 * (ks >> 1) + 1];
                    fa[i][0] = (int)(((px << 4) & 0xF0F0F0F0u) ^ 0x80808080u);
                    fa[i][1] = (int)((px & 0xF0F0F0F0u) ^ 0x80808080u);
                    fa[i][2] = (int)(((py << 4) & 0xF0F0F0F0u) ^ 0x80808080u);
                    fa[i][3] = (int)((py & 0xF0F0F0F0u) ^ 0x80808080u);
                }
                const int kc = 2 * ks + (lane >> 5);  // 16-code chunk inside the stage: tile kc >> 2, quarter kc & 3
                const int koff = (kc >> 2) * 64 + (kc & 3) * 16;
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    const int row = 32 * j + (lane & 31);
                    fb[j] = __builtin_bit_cast(v4i, lx[(row >> 4) * 128 + koff + (row & 15)]);
                }
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int j = 0; j < TM; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
            load_w(u, kt + PW, bulk);
        }
    };
    constexpr int kAhead = NS - 1 > PW ? NS - 1 : PW;  // how far past kt a pass issues
    int kt0 = 0;
    for (; kt0 + PW - 1 + kAhead < KT; kt0 += PW) stages_pw(kt0, kBulk);
    for (; kt0 < KT; kt0 += PW) stages_pw(kt0, kEdge);
    wait_vmcnt<0>();
#pragma unroll
    for (int p = 0; p < PW; ++p)
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v = 0; v < 2; ++v) asm volatile("" ::"v"(wreg[p][i][v]) : "memory");
    epilogue<OUT_MODE, TN, TM>(a, acc, lds, nt * BN + wave * 64, mt * BM, wave, lane);
}

template <int NS, int PW, int TM, int OUT_MODE>
hipError_t launch_dw4(GemmI8Args a, hipStream_t st) {
    constexpr size_t ring_bytes = (size_t)NS * (4 * TM) * 1024;  // + one spare KiB for the copies past the end of K
    constexpr size_t lds_bytes = ring_bytes + 1024;
    static_assert(ring_bytes >= 4 * 32 * (64 + 8) * 2, "the store phase stages its blocks inside the ring, below the spare KiB");
    static_assert(lds_bytes <= 80 * 1024, "two workgroups per compute unit");
    if ((a.Kp / 128) % PW != 0) return hipErrorInvalidValue;
    if (const hipError_t e = allow_dynamic_lds<gemm_i8_dw4_kernel<NS, PW, TM, OUT_MODE>>(lds_bytes); e != hipSuccess) return e;
    a.n_tiles = (a.N + 255) / 256;
    a.m_tiles = (a.M + 32 * TM - 1) / (32 * TM);
    gemm_i8_dw4_kernel<NS, PW, TM, OUT_MODE><<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, lds_bytes, st>>>(a);
    return hipGetLastError();
}

template <int BN, int BM, int KTS, int NS, int OUT_MODE>
hipError_t launch_variant(GemmI8Args a, hipStream_t st) {
    constexpr size_t lds_bytes = (size_t)NS * ((BN + BM) / 16 * KTS) * 1024;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    if (const hipError_t e = allow_dynamic_lds<gemm_i8_kernel<BN, BM, KTS, NS, OUT_MODE>>(lds_bytes); e != hipSuccess) return e;
    a.n_tiles = (a.N + BN - 1) / BN;
    a.m_tiles = (a.M + BM - 1) / BM;
    gemm_i8_kernel<BN, BM, KTS, NS, OUT_MODE><<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, lds_bytes, st>>>(a);
    return hipGetLastError();
}

template <int BN, int BM, int NS, int OUT_MODE>
hipError_t launch_w4(GemmI8Args a, hipStream_t st) {
    constexpr size_t lds_bytes = (size_t)NS * (BN / 16 + BM / 8) * 1024;
    static_assert(lds_bytes <= 80 * 1024, "two workgroups per compute unit");
    static_assert(lds_bytes >= 4 * 32 * (BN / 2 + 8) * 2, "the store phase stages its blocks in the same LDS");
    if (const hipError_t e = allow_dynamic_lds<gemm_i8_w4_kernel<BN, BM, NS, OUT_MODE>>(lds_bytes); e != hipSuccess) return e;
    a.n_tiles = (a.N + BN - 1) / BN;
    a.m_tiles = (a.M + BM - 1) / BM;
    gemm_i8_w4_kernel<BN, BM, NS, OUT_MODE><<<dim3((unsigned)(a.n_tiles * a.m_tiles)), 256, lds_bytes, st>>>(a);
    return hipGetLastError();
}

template <int OUT_MODE>
hipError_t launch_mode(const GemmI8Args &a, int num_cus, hipStream_t st) {
    // Tile shapes measured on MI355X.  The direct-weights kernel with the 256 x 128 tile is used
    // wherever its tiles cover at least three quarters of the compute units: on the Llama shapes it
    // is level with the 128 x 128 kernel (both operands through LDS) at M = 1024 and 10-17 % faster at
    // M = 2048 and 4096 (1.9-1.95 POP/s).  Below that (N = 4096 at M = 1024 gives 128 such tiles) its
    // 256 x 64 form doubles the number of tiles and is 3-7 % faster than the 128 x 128 kernel; with
    // many tiles it is the slowest (two weight loads per MFMA pair).  The kernels that stage both
    // operands stay selectable for experiments.
    int variant = tuning().gemm_variant;
    if (variant == 0) {
        const long big_tiles = (long)((a.N + 255) / 256) * ((a.M + 127) / 128);
        variant = 4 * big_tiles >= 3L * num_cus ? 10 : 12;
    }
    switch (variant) {
        case 1: return launch_variant<256, 256, 1, 4, OUT_MODE>(a, st);
        case 2: return launch_variant<256, 128, 1, 4, OUT_MODE>(a, st);
        case 4: return launch_variant<128, 128, 2, 3, OUT_MODE>(a, st);
        case 5: return launch_variant<128, 256, 1, 3, OUT_MODE>(a, st);
        case 6: return launch_variant<256, 128, 1, 3, OUT_MODE>(a, st);
        case 10: return launch_dw<9, 4, 4, OUT_MODE, true>(a, st);
        case 11: return launch_dw<6, 4, 4, OUT_MODE>(a, st);
        case 12: return launch_dw<15, 4, 2, OUT_MODE, true>(a, st);
        case 13: return launch_dw<8, 4, 2, OUT_MODE>(a, st);
        case 14: return launch_dw<8, 4, 4, OUT_MODE>(a, st);
        case 15: return launch_dw<14, 4, 2, OUT_MODE>(a, st);
        default: return launch_variant<128, 128, 1, 4, OUT_MODE>(a, st);
    }
}

template <int OUT_MODE>
hipError_t launch_mode_w4(const GemmI8Args &a, int num_cus, hipStream_t st) {
    int variant = tuning().gemm_variant;
    const int stages = a.Kp / 128;
    if (variant == 0) {
        const long big_tiles = (long)((a.N + 255) / 256) * ((a.M + 127) / 128);
        variant = stages % 2 != 0 ? 20 : 4 * big_tiles >= 3L * num_cus ? 21 : 23;
    }
    switch (variant) {
        case 21: return launch_dw4<4, 2, 4, OUT_MODE>(a, st);
        case 22: return launch_dw4<4, 4, 4, OUT_MODE>(a, st);
        case 23: return launch_dw4<8, 2, 2, OUT_MODE>(a, st);
        case 24: return launch_dw4<8, 4, 2, OUT_MODE>(a, st);
        default: return launch_w4<128, 128, 3, OUT_MODE>(a, st);
    }
}

}  // namespace

hipError_t launch_gemm_i8(const Geometry &g, const void *packed, const int8_t *xq_tiled,
                          const float *sx, int M, int Mp, void *out, int out_mode, const void *residual,
                          int gated_act, int num_cus, hipStream_t st) {
    (void)Mp;
    GemmI8Args a;
    a.w = static_cast<const uint4 *>(packed);
    a.x = reinterpret_cast<const uint4 *>(xq_tiled);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.sx = sx;
    a.res = out_mode == 0 ? static_cast<const _Float16 *>(residual) : nullptr;
    a.out = out;
    a.M = M;
    a.N = g.N;
    a.Kp = g.Kp;
    a.n_tiles = a.m_tiles = 0;
    a.gated_act = out_mode == 0 && g.pair_half ? gated_act : -1;
    if (g.fmt == kW4C) {
        a.sw_mul = 0.0625f;
        a.acc_shift = 4;
        return out_mode == 0 ? launch_mode_w4<0>(a, num_cus, st) : launch_mode_w4<1>(a, num_cus, st);
    }
    return out_mode == 0 ? launch_mode<0>(a, num_cus, st) : launch_mode<1>(a, num_cus, st);
}

}  // namespace qfc
