// Decode kernels (M <= 8 token rows): y[m,n] = sum_k x[m,k] * s * Wq[n,k].
// The memory-bound fully connected kernel of the decode stage (section 3.7 of
// the paper), here with binary16 activations and the weights dequantized in
// registers.
//
// Mapping.  A wavefront streams KiB tiles of 16 output rows (one 16-byte load
// per lane, one contiguous KiB per wavefront load, several loads in flight),
// converts the codes to binary16 in registers (exactly) and feeds them to
// v_mfma_f32_16x16x32_f16 as the B operand; the A operand holds the token rows
// (rows >= M are zero).  The MFMA does the reduction across the lanes of the
// wavefront that a dot-product formulation would need DPP shuffles for, its
// cost does not depend on M, and the matrix pipe is idle in a bandwidth-bound
// kernel anyway.  For int4 group-quantized weights every MFMA covers exactly
// one quantization group, and its fp32 result is scaled and accumulated with
// one FMA per token row; per-channel weights (int8 or int4) accumulate inside
// the MFMA and are scaled once at the end.
//
// Activations of the k range a wavefront is working on are staged in a private
// LDS region in A-operand order (no workgroup barrier in the streaming loop).
// A workgroup owns 1..4 consecutive row tiles (which share the staged
// activations) and splits K over its wavefronts; their partial sums meet in
// LDS in fixed order, so results are deterministic.  There is no reduction
// across workgroups and no atomics.
#include <type_traits>

#include "qfc_internal.h"

namespace qfc {

Tuning &tuning() {
    static Tuning t;
    return t;
}

// Wavefronts per workgroup at most.  Up to two token rows (and no prologue) the kernel needs few
// enough registers for 16 wavefronts of a workgroup to be resident: a K of 9 to 16 units
// (K = 14336: 14 units) then has one unit per wavefront and all its weight vectors in flight at
// once, instead of two units per wavefront in turn.
static int wave_cap(int M, bool plain, int KU) {
    return M > 4 ? 4 : (M <= 2 && plain && KU > 8 && KU <= 16) ? 16 : 8;
}

GemvPlan plan_gemv(const Geometry &g, int M, int num_cus, int pro) {
    (void)num_cus;
    const bool plain = pro == 0;
    const Tuning &t = tuning();
    GemvPlan p;
    // Half-unit items (int4 formats, no prologue), where measured faster: launches of few
    // wavefronts with a short K (O and QKV projections: twice the wavefronts, each with half the
    // serial work), and for M > 4 a long K, where a wavefront's staged token rows (16 KB of LDS per
    // unit at M = 8) limit the wavefronts a compute unit holds.
    const long full_waves = (long)g.RT * g.KU;
    const bool gain = M > 4 ? (g.KU > 4 || full_waves <= 1024) : (g.KU <= 4 && full_waves <= 2048);
    const bool can = g.fmt != kW8C && (plain || (pro > 0 && M <= 4));  // kernels built with half-unit items
    p.half = can && (t.gemv_half >= 0 ? t.gemv_half != 0 : gain);
    p.copy = p.half && plain && M > 4 && g.KU > 4;  // long K at M > 4: token rows staged by direct copies
    p.units = p.half ? (g.KT + 3) / 4 : g.KU;
    const int cap = p.half ? 8 : wave_cap(M, plain, p.units);
    const int per_wave = (p.units + cap - 1) / cap;  // items per wavefront and row tile
    p.waves = (p.units + per_wave - 1) / per_wave;
    const long waves_total = (long)g.RT * p.waves;
    // Row tiles per workgroup (they share the staged token rows).  One or two token rows: launches of
    // up to 8192 wavefronts, at most two row tiles (more measured slower: gate+up projection of
    // Llama-3.1-8B at M = 1 13.5 -> 14.3-17.3 us).  From three token rows on, staging the rows costs as
    // much traffic between L2 and the compute units as the weights themselves, and sharing it among up
    // to four row tiles wins wherever there are enough row tiles (the same layer at M = 4: 16.6 -> 15.5 us,
    // at M = 8: 23.3 -> 17.4 us; the narrow projections are level).
    const int target = t.gemv_target_waves > 0 ? (int)t.gemv_target_waves : (M > 2 ? 2048 : 8192);
    const int most = t.gemv_max_row_tiles > 0 ? (int)t.gemv_max_row_tiles : (M > 2 ? 4 : 2);
    int r = (int)((waves_total + target - 1) / target);
    if (r > most) r = most;
    if (r > 4) r = 4;
    if (r < 1) r = 1;
    p.row_tiles = r;
    return p;
}

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// Eight biased int4 codes of one dword -> eight binary16 values, k ascending,
// exactly.  A byte permute puts a code byte under the high byte 0x64:
// 0x6400 | u is 1024 + u and 0x6400 | (u << 4) is 1024 + 16 u, both exact in
// binary16, as are the subtraction of 1032 and the fused (x / 16 - 72).
// (Plain C only: hand-placed VALU instructions next to MFMAs would escape the
// compiler's hazard tracking.)
__device__ __forceinline__ v8h dequant8(uint32_t w) {
    const h2 c1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const h2 c72 = {(_Float16)72.0f, (_Float16)72.0f};
    const h2 c16th = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t lo = w & 0x0F0F0F0Fu, hi = w & 0xF0F0F0F0u;
    const h2 p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u)) - c1032;
    const h2 p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u)) - c1032;
    const h2 p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u)) * c16th - c72;
    const h2 p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u)) * c16th - c72;
    const u32x4 r = {as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3)};
    return __builtin_bit_cast(v8h, r);
}

// Eight int8 codes (two dwords) -> eight binary16 values, exactly: flipping the
// sign bit gives b + 128 in [0, 255]; 0x64 in the high byte makes 1024 + that.
__device__ __forceinline__ v8h dequant_i8x8(uint32_t lo, uint32_t hi) {
    const h2 c1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
    const uint32_t a = lo ^ 0x80808080u, b = hi ^ 0x80808080u;
    const h2 p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, a, 0x04010400u)) - c1152;
    const h2 p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, a, 0x04030402u)) - c1152;
    const h2 p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, b, 0x04010400u)) - c1152;
    const h2 p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, b, 0x04030402u)) - c1152;
    const u32x4 r = {as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3)};
    return __builtin_bit_cast(v8h, r);
}

__device__ __forceinline__ u32x4 gated_input8(const u32x4 &gate, const u32x4 &x, int act) {
    return __builtin_bit_cast(u32x4, gated_input8_u4(__builtin_bit_cast(uint4, gate), __builtin_bit_cast(uint4, x), act));
}

// eight binary16 pairs (weight, x) -> eight binary16 values fp16(x * (offset + weight))
__device__ __forceinline__ u32x4 weighted_input8(const u32x4 &w, const u32x4 &x, float offset) {
    const v8h wv = __builtin_bit_cast(v8h, w), xv = __builtin_bit_cast(v8h, x);
    v8h r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (_Float16)((float)xv[e] * (offset + (float)wv[e]));
    return __builtin_bit_cast(u32x4, r);
}

struct GemvArgs {
    const u32x4 *packed;
    const u32x4 *x;     // binary16 [M, K] as 16-byte vectors (8 values)
    const u32x4 *gate;  // prologue 1: binary16 [M, K], the layer's input is fp16(act(gate) * x);
                        // prologue 2: binary16 [K], the weight of the merged RMS normalization
    float norm_eps, norm_offset;  // prologue 2
    const _Float16 *res;  // binary16 [M, N] added before the final rounding, or null
    int act;            // QFC_ACT_* of the gate
    _Float16 *y;        // [M, N]
    const float *sw;    // per-channel scales [Np] (W8C, W4C)
    int N, K, RT, KT, KU, rt_stride;
    int row_tiles;           // R: row tiles per workgroup
    int rt_step;             // distance between a workgroup's row tiles (1; RT / 2 for a gated output)
    int gated_out;           // 1: rows [0, N/2) are the gate, rows [N/2, N) the other branch; y is [M, N/2]
    int paired;              // 1: the layer is packed in pairs (physical row tiles 2 t, 2 t + 1 = the two branches)
    int units_q, units_rem;  // KU = units_q * waves + units_rem
    // Rotary embedding + layout transformation + cache append in the final reduction (QKV layer):
    // rope_per = d / 32 (0: off) is the distance, in row tiles, between the two rows of a rotary pair.
    int rope_per, rope_d, rope_hq, rope_hkv, rope_C, rope_pos;
    const float *rope_table;
    _Float16 *rope_q, *rope_kc, *rope_vc;
};

// LDS view of one wavefront's staged activations: vector (slot * M + m).
// int4 unit: 1024 k = 128 octets, slot = octet index (4 * group + q).
// W8C unit:   512 k =  64 octets, slot = tile * 8 + j * 4 + q for octet 2q + j of the tile.
// Prologues.  PRO = 1: the gate branch travels with x and the two are merged on the way into LDS (operator
// fusion, section 3.6 of the paper: element-wise operators of two branches merged into the
// fully connected operator).  PRO = 2: RMS normalization merged into the layer: normalizing scales
// a row by one number rs, which commutes with the product, so the row goes into LDS multiplied by
// the normalization weight only and the output is multiplied by rs at the end; every workgroup
// computes the rows' sums of squares for itself (one pass over x).
template <int M, int FMT, int PRO, int OCT>  // OCT: octets (8 k) per item
struct XStage {
    static constexpr int XV = M * OCT / 64;               // 16-byte vectors per lane per unit
    u32x4 v[XV];
    u32x4 g[PRO ? XV : 1];

    // global -> registers (zeros beyond K)
    __device__ __forceinline__ void load(const GemvArgs &a, int unit, int lane) {
        const int K8 = a.K / 8;
        const int o_base = unit * OCT;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = i * 64 + lane;
            const int m = p / OCT, o = p % OCT;
            const u32x4 zero = {0, 0, 0, 0};
            v[i] = o_base + o < K8 ? a.x[(size_t)m * K8 + o_base + o] : zero;
            if (PRO == 1) g[i] = o_base + o < K8 ? a.gate[(size_t)m * K8 + o_base + o] : zero;
            if (PRO == 2) g[i] = o_base + o < K8 ? a.gate[o_base + o] : zero;
        }
    }
    // global -> this wavefront's LDS region without passing registers (no prologue): vector p of
    // the region (p = 64 i + lane = slot * M + m) is copied from wherever its token row keeps that
    // octet.  Octets beyond K are read from the start of the row instead, each from its own place
    // (finite values that only meet zero weights of the padding; not all from one place: many copies
    // of the same line in flight have been seen to reach LDS after the counter said they were done).
    __device__ __forceinline__ void copy(const GemvArgs &a, int unit, int lane, u32x4 *lds) const {
        const int K8 = a.K / 8;
        const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = i * 64 + lane;
            const int slot = p / M, m = p % M;
            int o = slot;
            if (FMT == kW8C) o = (slot & ~7) | ((slot >> 2) & 1) | ((slot & 3) << 1);
            const int oo = unit * OCT + o;
            const uint32_t off = (uint32_t)(((size_t)m * K8 + (oo < K8 ? oo : oo - K8)) * 16);
            copy16_to_lds(a.x, off, __builtin_amdgcn_readfirstlane(lds_base + i * 1024));
        }
    }
    // registers -> this wavefront's LDS region, A-operand order
    __device__ __forceinline__ void store(u32x4 *lds, int lane, int act, float offset) const {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int p = i * 64 + lane;
            const int m = p / OCT, o = p % OCT;
            int slot = o;
            if (FMT == kW8C) slot = (o & ~7) | ((o & 1) << 2) | ((o >> 1) & 3);
            lds[slot * M + m] = PRO == 1 ? gated_input8(g[i], v[i], act) : PRO == 2 ? weighted_input8(g[i], v[i], offset) : v[i];
        }
    }
};

// HALF (int4 formats): an item is half a unit, four weight tiles and the two scale vectors of their
// 16 groups, and a wavefront stages 512 k of the token rows at a time: twice the wavefronts for
// short K, and half the LDS and registers per wavefront for M > 4, where the staged rows limit
// how many wavefronts a compute unit holds.  a.KU, a.units_q and a.units_rem then count half units.
// COPY (with HALF, M > 4, long K): the token rows go from memory into LDS by direct copies instead of
// through registers (a third of the registers of M = 8 otherwise hold them).  Such copies and the
// weight loads complete in order only among their own kind, so the wavefront waits for an empty
// counter before its first tile: slower for short K, faster for the down projections (M = 8: -17 %).
template <int M, int FMT, bool DB, int PRO, bool BIG = false, bool HALF = false, bool COPY = false>
__global__ __launch_bounds__(BIG ? 1024 : PRO && M > 4 ? 256 : 512) void gemv_kernel(GemvArgs a) {
    static_assert(!HALF || (FMT != kW8C && !DB), "half units: int4 formats, single buffer");
    static_assert(!COPY || (HALF && PRO == 0), "direct copies: half units without a prologue");
    constexpr int TILES = HALF ? 4 : 8;         // weight tiles per item
    constexpr int NV = FMT == kW4G32 ? TILES + TILES / 2 : TILES;  // 16-byte vectors per lane per (item, row tile)
    constexpr int OCT = FMT == kW8C ? 64 : HALF ? 64 : 128;
    constexpr int MI = M < 4 ? M : 4;           // accumulator rows that matter on a lane
    extern __shared__ u32x4 lds_all[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int c = lane & 15, q = lane >> 4;
    // Gated output: a workgroup owns the two row tiles (t, t + RT / 2) that hold the gate and the
    // other branch of the same 16 output channels.
    // (first row tile in the packed buffer: with the branches' tiles interleaved, the pair (2 b, 2 b + 1))
    // Rotary pairs: a workgroup owns the row tiles (t, t + d / 32) of one head, i.e. rows i and i + d / 2.
    const int rt0 = a.rope_per    ? (int)(blockIdx.x / a.rope_per) * (2 * a.rope_per) + (int)(blockIdx.x % a.rope_per)
                    : a.gated_out ? (a.paired ? 2 * blockIdx.x : blockIdx.x)
                                  : blockIdx.x * a.row_tiles;
    const int R = a.gated_out || a.rope_per ? 2 : min(a.row_tiles, a.RT - rt0);
    const int u0 = wave * a.units_q + min(wave, a.units_rem);
    const int u1 = u0 + a.units_q + (wave < a.units_rem ? 1 : 0);
    u32x4 *lds_x = lds_all + wave * (OCT * M);

    float acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[r][i] = 0.0f;

    // Merged RMS normalization: the rows' sums of squares, by the whole workgroup (fp32; partial
    // sums of the wavefronts are added in fixed order where they are used, at the end).
    __shared__ float s_ss[PRO == 2 ? 8 : 1][M];
    static_assert(!(BIG && PRO), "up to 16 wavefronts only without a prologue");
    if constexpr (PRO == 2) {
        float ss[M];
#pragma unroll
        for (int m = 0; m < M; ++m) ss[m] = 0.0f;
        const int K8 = a.K / 8;
        for (int v = threadIdx.x; v < M * K8; v += blockDim.x) {
            const int m = v / K8;
            const v8h hx = __builtin_bit_cast(v8h, a.x[v]);
            float t = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) t = fmaf((float)hx[i], (float)hx[i], t);
#pragma unroll
            for (int mm = 0; mm < M; ++mm)
                if (mm == m) ss[mm] += t;
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float t = ss[m];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, 64);
            if (lane == 0) s_ss[wave][m] = t;
        }
        // (made visible to the other wavefronts by the barriers before the final reduction)
    }

    // item = (unit, row tile); its vectors: (W4G32) 4 scale vectors, then weight tiles 0..nt-1.
    // `full` = all 8 tiles present: unconditional loads, so that the compiler can
    // count them and wait tile by tile instead of for everything.
    auto load_item = [&](u32x4(&buf)[NV], int u, int r, auto full) {
        const int nt = full ? TILES : min(TILES, a.KT - TILES * u);
        const int U = HALF ? u >> 1 : u, h = HALF ? u & 1 : 0;  // unit, half of it
        const int ntU = HALF ? min(8, a.KT - 8 * U) : nt;       // weight tiles before the unit's scale tile
        const int pos = FMT == kW4G32 ? 9 * U : 8 * U;
        const u32x4 *base = a.packed + ((size_t)(rt0 + r * a.rt_step) * a.rt_stride + pos) * 64;
        // scales first: loads return in order, and the first tile's results need them
        if (FMT == kW4G32) {
#pragma unroll
            for (int p = 0; p < TILES / 2; ++p)
                buf[TILES + p] = __builtin_nontemporal_load(base + ntU * 64 + (h * 2 + p) * 16 + c);
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            if (full || t < nt) buf[t] = __builtin_nontemporal_load(base + (h * 4 + t) * 64 + lane);
    };
    constexpr std::false_type kMaybePartial{};
    constexpr std::true_type kFull{};

    // Two variants.  DB = false: latency is hidden by occupancy, a wavefront
    // requests the activations and all weight vectors of an item at once, waits,
    // computes and moves on; the low register count (no second weight buffer)
    // buys extra resident wavefronts.  This suits launches whose wavefronts have
    // one or two items.  DB = true: the next item's vectors are requested before
    // the current item is computed, for long-lived wavefronts.  Vector loads
    // return in order, so the (small) activation loads are issued first.
    XStage<M, FMT, PRO, OCT> xs;
    u32x4 cur[NV];
    u32x4 nxt[DB ? NV : 1];
    const int items = (u1 - u0) * R;
    int u = u0, r = 0;
    if constexpr (DB) {
        if (items > 0) {
            xs.load(a, u0, lane);
            load_item(cur, u0, 0, kMaybePartial);
            if (items > 1) load_item(nxt, R > 1 ? u0 : u0 + 1, R > 1 ? 1 : 0, kMaybePartial);
        }
    }
    auto stage = [&]() {
        // the wavefront's earlier LDS reads are done (same wavefront, in order)
        xs.store(lds_x, lane, a.act, a.norm_offset);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    for (int it = 0; it < items; ++it) {
        const int nt = min(TILES, a.KT - TILES * u);
        float accr[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        v4f accw = {0.0f, 0.0f, 0.0f, 0.0f};
        v4f accw2 = {0.0f, 0.0f, 0.0f, 0.0f};  // second chain (W4C), so that MFMAs do not wait on each other
        // A operands (token rows) of one tile; lanes whose row index is >= M read
        // row c % M instead: an A row only feeds the D row of the same index, and
        // D rows >= M are never used, so no masking or zeroing is needed.
        constexpr int XA = FMT == kW8C ? 2 : 4;
        const u32x4 *xrow = lds_x + q * M + (c % M);
        auto load_xa = [&](v8h(&xa)[XA], int t) {
#pragma unroll
            for (int j = 0; j < XA; ++j)
                xa[j] = __builtin_bit_cast(v8h, xrow[(FMT == kW8C ? t * 8 + j * 4 : (4 * t + j) * 4) * M]);
        };
        // The scaled accumulation of an MFMA result is issued one step late, after the
        // next MFMA has been started, so that its latency is covered by the next
        // step's dequantization instead of a stall.
        v4f d_prev = {0.0f, 0.0f, 0.0f, 0.0f};
        _Float16 s_prev = (_Float16)0.0f;
        auto tile_math = [&](const v8h(&xa)[XA], int t) {
            if (FMT == kW4G32) {
                const uint32_t wd[4] = {cur[t].x, cur[t].y, cur[t].z, cur[t].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int gl = 4 * t + j;  // group inside the unit
                    const v8h wb = dequant8(wd[j]);
                    const v4f zero = {0.0f, 0.0f, 0.0f, 0.0f};
                    const v4f d = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[j], wb, zero, 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < MI; ++i) accr[i] = fmaf((float)s_prev, d_prev[i], accr[i]);
                    const u32x4 sv = cur[TILES + gl / 8];
                    const uint32_t sd = sv[(gl % 8) / 2];
                    s_prev = __builtin_bit_cast(_Float16, (uint16_t)(sd >> (16 * (gl & 1))));
                    d_prev = d;
                }
            } else if (FMT == kW4C) {
                accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[0], dequant8(cur[t].x), accw, 0, 0, 0);
                accw2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[1], dequant8(cur[t].y), accw2, 0, 0, 0);
                accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[2], dequant8(cur[t].z), accw, 0, 0, 0);
                accw2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[3], dequant8(cur[t].w), accw2, 0, 0, 0);
            } else {
                accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[0], dequant_i8x8(cur[t].x, cur[t].y), accw, 0, 0, 0);
                accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[1], dequant_i8x8(cur[t].z, cur[t].w), accw, 0, 0, 0);
            }
        };
        auto compute_full = [&]() {
            // full unit: straight-line code, A operands fetched one tile ahead
            v8h xa[XA], xn[XA];
            load_xa(xa, 0);
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                if (t + 1 < TILES) load_xa(xn, t + 1);
                tile_math(xa, t);
#pragma unroll
                for (int j = 0; j < XA; ++j) xa[j] = xn[j];
            }
        };
        auto compute_tail = [&]() {
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                if (t < nt) {
                    v8h xa[XA];
                    load_xa(xa, t);
                    tile_math(xa, t);
                }
            }
        };
        if constexpr (DB) {
            if (r == 0) stage();
            if (nt == TILES)
                compute_full();
            else
                compute_tail();
        } else {
            // single buffer: request, stage and compute inside one branch
            if (r == 0) {
                if constexpr (COPY)
                    xs.copy(a, u, lane, lds_x);
                else
                    xs.load(a, u, lane);
            }
            auto staged = [&]() {
                if constexpr (COPY) {
                    wait_vmcnt<0>();  // only an empty counter says that the copies have landed
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                } else {
                    stage();
                }
            };
            if (nt == TILES) {
                load_item(cur, u, r, kFull);
                if (r == 0) staged();
                compute_full();
            } else {
                load_item(cur, u, r, kMaybePartial);
                if (r == 0) staged();
                compute_tail();
            }
        }
        if (FMT == kW4G32) {
#pragma unroll
            for (int i = 0; i < MI; ++i) accr[i] = fmaf((float)s_prev, d_prev[i], accr[i]);
        }
        // add this item's contribution to the accumulators of its row tile
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            if (rr == r) {
#pragma unroll
                for (int i = 0; i < MI; ++i) acc[rr][i] += FMT == kW4G32 ? accr[i] : FMT == kW4C ? accw[i] + accw2[i] : accw[i];
            }
        if (++r == R) {
            r = 0;
            ++u;
        }
        if constexpr (DB) {
            if (it + 1 < items) {
                if (r == 0) xs.load(a, u, lane);
#pragma unroll
                for (int v = 0; v < NV; ++v) cur[v] = nxt[v];
                if (it + 2 < items) load_item(nxt, r + 1 == R ? u + 1 : u, r + 1 == R ? 0 : r + 1, kMaybePartial);
            }
        }
    }

    // meet in LDS: red[wave][r][m][16 rows]; lane (c, q) holds token rows 4q .. 4q+3 of row c
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds_all);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int m = 4 * q + i;
            if (rr < R && m < M) red[((wave * 4 + rr) * M + m) * 16 + c] = acc[rr][i];
        }
    __syncthreads();
    if (a.rope_per) {
        // Rotary embedding fused with the layout transformation of the query, key and value
        // projections (section 3.6 of the paper), here in the final reduction of the layer that
        // produces them: the workgroup holds the fp32 sums of rows i and i + d / 2 of one head for
        // every token row (= sequence b at position pos); queries and keys are rotated in fp32 and
        // rounded once, the results go to the query buffer and into the two caches.
        const int d = a.rope_d, halfd = d / 2, g = a.rope_hq / a.rope_hkv;
        const int head = (int)(blockIdx.x / a.rope_per);
        for (int e = threadIdx.x; e < M * 16; e += blockDim.x) {
            const int cc = e & 15, m = e >> 4;
            float s0 = 0.0f, s1 = 0.0f;
            for (int w = 0; w < nwaves; ++w) {
                s0 += red[((w * 4 + 0) * M + m) * 16 + cc];
                s1 += red[((w * 4 + 1) * M + m) * 16 + cc];
            }
            const int i = (int)(blockIdx.x % a.rope_per) * 16 + cc;  // index inside the first half of the head
            const int n0 = head * d + i;                             // output channel of s0; s1 is n0 + d / 2
            if (FMT != kW4G32) {
                s0 *= a.sw[n0];
                s1 *= a.sw[n0 + halfd];
            }
            if constexpr (PRO == 2) {
                float tot = 0.0f;
                for (int w = 0; w < nwaves; ++w) tot += s_ss[w][m];
                const float rs = 1.0f / sqrtf(tot / (float)a.K + a.norm_eps);
                s0 *= rs;
                s1 *= rs;
            }
            if (head >= a.rope_hq + a.rope_hkv) {  // value head: column pos of the transposed cache
                const int kv = head - a.rope_hq - a.rope_hkv;
                _Float16 *dst = a.rope_vc + (((size_t)(m * a.rope_hkv + kv) * (a.rope_C / 64) + a.rope_pos / 64) * d) * 64 + a.rope_pos % 64;
                dst[(size_t)i * 64] = (_Float16)s0;
                dst[(size_t)(i + halfd) * 64] = (_Float16)s1;
                continue;
            }
            const float cs = a.rope_table[((size_t)a.rope_pos * halfd + i) * 2];
            const float sn = a.rope_table[((size_t)a.rope_pos * halfd + i) * 2 + 1];
            _Float16 *dst;
            if (head < a.rope_hq)
                dst = a.rope_q + ((size_t)(m * a.rope_hkv + head / g) * g + head % g) * d;
            else
                dst = a.rope_kc + ((size_t)(m * a.rope_hkv + head - a.rope_hq) * a.rope_C + a.rope_pos) * d;
            dst[i] = (_Float16)(s0 * cs - s1 * sn);
            dst[i + halfd] = (_Float16)(s1 * cs + s0 * sn);
        }
        return;
    }
    if (a.gated_out) {
        // y[m, n] = fp16(act(gate) * other), both fp32 sums of this workgroup (operator fusion,
        // section 3.6 of the paper: the element-wise operators of the two branches are merged
        // into the fully connected operator that produces them)
        const GateCoeffs gc = gate_coeffs(a.act);
        const int half = a.N / 2;
        for (int e = threadIdx.x; e < M * 16; e += blockDim.x) {
            const int cc = e & 15, m = e >> 4;
            float sg = 0.0f, su = 0.0f;
            for (int w = 0; w < nwaves; ++w) {
                sg += red[((w * 4 + 0) * M + m) * 16 + cc];
                su += red[((w * 4 + 1) * M + m) * 16 + cc];
            }
            const int n = (int)blockIdx.x * 16 + cc;  // channel of the gated output
            if (n < half) {
                if (FMT != kW4G32) {  // (the scales follow the packed row order)
                    sg *= a.sw[a.paired ? rt0 * 16 + cc : n];
                    su *= a.sw[a.paired ? rt0 * 16 + 16 + cc : n + half];
                }
                if constexpr (PRO == 2) {
                    float tot = 0.0f;
                    for (int w = 0; w < nwaves; ++w) tot += s_ss[w][m];
                    const float rs = 1.0f / sqrtf(tot / (float)a.K + a.norm_eps);
                    sg *= rs;
                    su *= rs;
                }
                a.y[(size_t)m * half + n] = (_Float16)(gate_activation(sg, gc) * su);
            }
        }
        return;
    }
    for (int e = threadIdx.x; e < R * M * 16; e += blockDim.x) {
        const int cc = e & 15, m = (e >> 4) % M, rr = (e >> 4) / M;
        float s = 0.0f;
        for (int w = 0; w < nwaves; ++w) s += red[((w * 4 + rr) * M + m) * 16 + cc];
        const int n = (rt0 + rr) * 16 + cc;
        if (n < a.N) {
            if (FMT != kW4G32) s *= a.sw[n];
            if constexpr (PRO == 2) {
                float tot = 0.0f;
                for (int w = 0; w < nwaves; ++w) tot += s_ss[w][m];
                s *= 1.0f / sqrtf(tot / (float)a.K + a.norm_eps);
            }
            if (a.res) s += (float)a.res[(size_t)m * a.N + n];
            a.y[(size_t)m * a.N + n] = (_Float16)s;
        }
    }
}

template <int M, int PRO>
hipError_t launch_m(const Geometry &g, const GemvArgs &a, const GemvPlan &p, hipStream_t st) {
    const int waves = p.waves;
    const dim3 grid((unsigned)(a.gated_out || a.rope_per ? g.RT / 2 : (g.RT + a.row_tiles - 1) / a.row_tiles));
    const dim3 block((unsigned)(waves * 64));
    const int oct = g.fmt == kW8C || p.half ? 64 : 128;
    size_t lds = (size_t)waves * oct * M * 16;
    const size_t red = (size_t)waves * 4 * M * 16 * sizeof(float);
    if (red > lds) lds = red;
    // long-lived wavefronts (>= 3 items each) get the double-buffered variant
    const int items = ((p.units + waves - 1) / waves) * (a.gated_out || a.rope_per ? 2 : a.row_tiles);
    if constexpr (PRO == 0 && M > 4) {
        if (p.half && p.copy) {
            if (g.fmt == kW4C)
                gemv_kernel<M, kW4C, false, 0, false, true, true><<<grid, block, lds, st>>>(a);
            else
                gemv_kernel<M, kW4G32, false, 0, false, true, true><<<grid, block, lds, st>>>(a);
            return hipGetLastError();
        }
    }
    if constexpr (PRO == 0 || M <= 4) {
        if (p.half) {
            if (g.fmt == kW4C)
                gemv_kernel<M, kW4C, false, PRO, false, true><<<grid, block, lds, st>>>(a);
            else
                gemv_kernel<M, kW4G32, false, PRO, false, true><<<grid, block, lds, st>>>(a);
            return hipGetLastError();
        }
    }
    if constexpr (M <= 2 && PRO == 0) {
        if (waves > 8) {
            if (g.fmt == kW8C)
                gemv_kernel<M, kW8C, false, 0, true><<<grid, block, lds, st>>>(a);
            else if (g.fmt == kW4C)
                gemv_kernel<M, kW4C, false, 0, true><<<grid, block, lds, st>>>(a);
            else
                gemv_kernel<M, kW4G32, false, 0, true><<<grid, block, lds, st>>>(a);
            return hipGetLastError();
        }
    }
    if constexpr (M <= 2) {
        if (items >= 3) {
            if (g.fmt == kW8C)
                gemv_kernel<M, kW8C, true, PRO><<<grid, block, lds, st>>>(a);
            else if (g.fmt == kW4C)
                gemv_kernel<M, kW4C, true, PRO><<<grid, block, lds, st>>>(a);
            else
                gemv_kernel<M, kW4G32, true, PRO><<<grid, block, lds, st>>>(a);
            return hipGetLastError();
        }
    }
    if (g.fmt == kW8C)
        gemv_kernel<M, kW8C, false, PRO><<<grid, block, lds, st>>>(a);
    else if (g.fmt == kW4C)
        gemv_kernel<M, kW4C, false, PRO><<<grid, block, lds, st>>>(a);
    else
        gemv_kernel<M, kW4G32, false, PRO><<<grid, block, lds, st>>>(a);
    return hipGetLastError();
}

template <int PRO>
hipError_t launch_any_m(const Geometry &g, const GemvArgs &a, int M, const GemvPlan &waves, hipStream_t st) {
    switch (M) {
        case 1: return launch_m<1, PRO>(g, a, waves, st);
        case 2: return launch_m<2, PRO>(g, a, waves, st);
        case 3: return launch_m<3, PRO>(g, a, waves, st);
        case 4: return launch_m<4, PRO>(g, a, waves, st);
        case 5: return launch_m<5, PRO>(g, a, waves, st);
        case 6: return launch_m<6, PRO>(g, a, waves, st);
        case 7: return launch_m<7, PRO>(g, a, waves, st);
        case 8: return launch_m<8, PRO>(g, a, waves, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_gemv(const Geometry &g, const void *packed, const void *x, int M, void *y,
                       const Fusion &f, int num_cus, hipStream_t st) {
    const GemvPlan p = plan_gemv(g, M, num_cus, f.norm_gamma ? 2 : f.gate ? 1 : 0);
    GemvArgs a;
    a.packed = static_cast<const u32x4 *>(packed);
    a.x = static_cast<const u32x4 *>(x);
    a.gate = static_cast<const u32x4 *>(f.gate);
    a.res = static_cast<const _Float16 *>(f.residual);
    a.act = f.activation;
    a.y = static_cast<_Float16 *>(y);
    a.sw = reinterpret_cast<const float *>(static_cast<const char *>(packed) + g.scale_off);
    a.N = g.N;
    a.K = g.K;
    a.RT = g.RT;
    a.KT = g.KT;
    a.KU = p.units;
    a.rt_stride = g.rt_stride;
    a.row_tiles = p.row_tiles;
    a.paired = g.pair_half ? 1 : 0;
    a.rt_step = f.gated_output && !a.paired ? g.RT / 2 : 1;
    a.gated_out = f.gated_output ? 1 : 0;
    a.rope_per = 0;
    a.rope_d = a.rope_hq = a.rope_hkv = a.rope_C = a.rope_pos = 0;
    a.rope_table = nullptr;
    a.rope_q = a.rope_kc = a.rope_vc = nullptr;
    if (f.rope) {
        const RopeOut &r = *f.rope;
        a.rope_per = r.d / 32;
        a.rt_step = a.rope_per;
        a.rope_d = r.d;
        a.rope_hq = r.h_q;
        a.rope_hkv = r.h_kv;
        a.rope_C = r.C;
        a.rope_pos = r.pos;
        a.rope_table = r.table;
        a.rope_q = static_cast<_Float16 *>(r.q);
        a.rope_kc = static_cast<_Float16 *>(r.kc);
        a.rope_vc = static_cast<_Float16 *>(r.vc);
    }
    a.units_q = p.units / p.waves;
    a.units_rem = p.units % p.waves;
    a.norm_eps = f.norm_eps;
    a.norm_offset = f.norm_offset;
    if (f.norm_gamma) {
        a.gate = static_cast<const u32x4 *>(f.norm_gamma);
        return launch_any_m<2>(g, a, M, p, st);
    }
    return f.gate ? launch_any_m<1>(g, a, M, p, st) : launch_any_m<0>(g, a, M, p, st);
}

}  // namespace qfc
