// A chain of decode layers (M <= 4 token rows) in ONE persistent launch.
//
// The decode stage's fully connected layers are bound by the weight stream
// (section 3.7 of the paper), and a layer of a few MB is over before the
// memory system has reached its rate: launched one by one, every layer pays
// the start and the drain of its own kernel with the memory pipe idle.  Here a
// fixed grid of resident workgroups walks through the layers; between two
// layers all workgroups meet at a barrier in device memory (layer f + 1 reads
// what layer f wrote).  Weights do not depend on the previous layer, so every
// wavefront requests the first weight item of its NEXT piece of work (the next
// round of this layer, or its first round of the next layer) before it joins
// the reduction and the barrier: the weight stream keeps going while the
// workgroups synchronize.
//
// The arithmetic of a layer is that of the one-launch-per-layer kernel
// (same items, same order of the partial sums), so results are bit-identical
// to it.
//
// Work split of a layer with plan (P wavefronts per 16-row block group, R row
// tiles): the 8 wavefronts of a workgroup form 8 / P slots that work on
// different virtual blocks at the same time; a round is one virtual block per
// slot; workgroup g takes rounds g, g + G, ...
//
// The barrier.  The last wavefront of a workgroup writes the round's outputs,
// makes them visible to the device (release), adds one to a counter in device
// memory and polls it until all workgroups of the grid have arrived, then
// invalidates the caches (acquire); the other wavefronts wait for it at a
// workgroup barrier.  The poll is bounded by a wall-clock limit: on expiry the
// wavefront raises an error flag, which ends every later wait at once, so the
// kernel always terminates (its outputs are then meaningless and the flag tells
// the caller).  The grid never exceeds the number of workgroups that are
// resident at the same time.  The polling wavefront does not request weights
// across a layer boundary: loads return in order, so its first poll would wait
// for them.
#include <type_traits>

#include "gemv_common.h"

namespace qfc {
namespace {

using namespace gemv_detail;

struct alignas(16) SeqLayer {
    GemvArgs a;
    int fmt;
    int waves;    // P
    int slots;    // 8 / P
    int nblocks;  // virtual blocks of the layer
    int rounds;   // ceil(nblocks / slots)
};
static_assert(sizeof(SeqLayer) == kSeqLayerBytes, "layer record");

constexpr int kSeqWaves = 8;
constexpr int kPollWave = kSeqWaves - 1;

// Device-side view of a layer record.  The record is read once per layer, every dword made
// wavefront-uniform (scalar registers), and its pointers typed as global memory: what the
// compiler loads itself from a record behind a barrier lands in vector registers, and pointers
// read from memory are generic to it (flat instructions, which also occupy the LDS counter).
#define QFC_GLOBAL __attribute__((address_space(1)))
typedef const QFC_GLOBAL u32x4 *gvec_c;
struct DevLayer {
    gvec_c packed, x;
    const QFC_GLOBAL _Float16 *res;
    QFC_GLOBAL _Float16 *y;
    const QFC_GLOBAL float *sw;
    int act, N, K, RT, KT, rt_stride, row_tiles, rt_step, gated_out, units_q, units_rem;
    int fmt, waves, slots, nblocks, rounds;
};

__device__ __forceinline__ DevLayer read_layer(const SeqLayer *rec) {
    constexpr int W = sizeof(SeqLayer) / 4;
    struct Words {
        uint32_t w[W];
    } raw;
    const QFC_GLOBAL uint32_t *p = (const QFC_GLOBAL uint32_t *)(uintptr_t)rec;
#pragma unroll
    for (int i = 0; i < W; ++i) raw.w[i] = __builtin_amdgcn_readfirstlane(p[i]);
    const SeqLayer L = __builtin_bit_cast(SeqLayer, raw);
    DevLayer d;
    d.packed = (gvec_c)(uintptr_t)L.a.packed;
    d.x = (gvec_c)(uintptr_t)L.a.x;
    d.res = (const QFC_GLOBAL _Float16 *)(uintptr_t)L.a.res;
    d.y = (QFC_GLOBAL _Float16 *)(uintptr_t)L.a.y;
    d.sw = (const QFC_GLOBAL float *)(uintptr_t)L.a.sw;
    d.act = L.a.act;
    d.N = L.a.N;
    d.K = L.a.K;
    d.RT = L.a.RT;
    d.KT = L.a.KT;
    d.rt_stride = L.a.rt_stride;
    d.row_tiles = L.a.row_tiles;
    d.rt_step = L.a.rt_step;
    d.gated_out = L.a.gated_out;
    d.units_q = L.a.units_q;
    d.units_rem = L.a.units_rem;
    d.fmt = L.fmt;
    d.waves = L.waves;
    d.slots = L.slots;
    d.nblocks = L.nblocks;
    d.rounds = L.rounds;
    return d;
}

struct WavePiece {
    bool live;
    int rt0, R, u0, u1, slot;
};

// the part of round vr of layer L that belongs to this wavefront
__device__ __forceinline__ WavePiece wave_piece(const DevLayer &L, int vr, int wave) {
    WavePiece p;
    int slot = 0, lw = wave;
    while (lw >= L.waves) {
        lw -= L.waves;
        ++slot;
    }
    const int vb = vr * L.slots + slot;
    p.slot = slot;
    p.live = slot < L.slots && vb < L.nblocks;
    p.rt0 = L.gated_out ? vb : vb * L.row_tiles;
    p.R = !p.live ? 0 : L.gated_out ? 2 : min(L.row_tiles, L.RT - p.rt0);
    p.u0 = lw * L.units_q + min(lw, L.units_rem);
    p.u1 = p.u0 + L.units_q + (lw < L.units_rem ? 1 : 0);
    return p;
}

// Request the vectors of item (unit u, row tile rt) of a layer of any format.
__device__ __forceinline__ void request_item(gvec_c packed, int rt_stride, int KT, int fmt, int rt, int u, int lane,
                                             u32x4 (&buf)[12]) {
    const int nt = min(8, KT - 8 * u);
    const int pos = fmt == kW4G32 ? 9 * u : 8 * u;
    gvec_c base = packed + ((size_t)rt * rt_stride + pos) * 64;
    if (fmt == kW4G32) {
#pragma unroll
        for (int p = 0; p < 4; ++p) buf[8 + p] = __builtin_nontemporal_load(base + nt * 64 + p * 16 + (lane & 15));
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < nt) buf[t] = __builtin_nontemporal_load(base + t * 64 + lane);
}

// First item of this wavefront in round vr of layer L; false if it has none there.
__device__ __forceinline__ bool request_first(const DevLayer &L, int vr, int wave, int lane, u32x4 (&buf)[12]) {
    const WavePiece p = wave_piece(L, vr, wave);
    if (!p.live || p.u1 <= p.u0) return false;
    request_item(L.packed, L.rt_stride, L.KT, L.fmt, p.rt0, p.u0, lane, buf);
    return true;
}

__device__ __forceinline__ void grid_barrier(unsigned *sync, unsigned target, long long limit, int wave, int lane) {
    if (wave == kPollWave) {
        // release: this wavefront's stores of the layer's outputs are visible device-wide first
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        if (lane == 0) {
            __hip_atomic_fetch_add(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const long long t0 = wall_clock64();
            while (__hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (__hip_atomic_load(&sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
                if (wall_clock64() - t0 > limit) {
                    __hip_atomic_store(&sync[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

// Invariant: when a wavefront starts an item, the item's weight vectors have been requested into
// `cur` already (at the start of the kernel, after the previous item, or, for the polling
// wavefront, after the barrier).  Weights are requested at one place only, after an item's
// arithmetic has consumed `cur`: one buffer suffices, and the compiler sees one definition of it.
template <int M, int FMT>
__device__ __forceinline__ void run_layer(const DevLayer &L, const DevLayer &next, u32x4 *lds_all, float *red,
                                          u32x4 (&cur)[12], int wave, int lane) {
    constexpr int TILES = 8;
    constexpr int OCT = FMT == kW8C ? 64 : 128;
    constexpr int MI = M < 4 ? M : 4;
    const DevLayer &a = L;
    const int g = blockIdx.x, G = gridDim.x;
    const int c = lane & 15, q = lane >> 4;
    u32x4 *lds_x = lds_all + wave * (OCT * M);

    // (a workgroup without a round in this layer makes one empty pass: it only looks ahead)
    for (int vr = g; vr < L.rounds || vr == g; vr += G) {
        const WavePiece wp = wave_piece(L, vr, wave);
        const int rt0 = wp.rt0, R = wp.R;
        float acc[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[r][i] = 0.0f;

        XStage<M, FMT, 0> xs;
        const int items = wp.live ? (wp.u1 - wp.u0) * R : 0;
        int u = wp.u0, r = 0;
        auto stage = [&]() {
            xs.store(lds_x, lane, 0, 0.0f);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        };
        const int trips = items > 0 ? items : 1;
        for (int it = 0; it < trips; ++it) {
            if (it < items) {
                const int nt = min(TILES, a.KT - TILES * u);
                float accr[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                v4f accw = {0.0f, 0.0f, 0.0f, 0.0f};
                v4f accw2 = {0.0f, 0.0f, 0.0f, 0.0f};
                constexpr int XA = FMT == kW8C ? 2 : 4;
                const u32x4 *xrow = lds_x + q * M + (c % M);
                auto load_xa = [&](v8h(&xa)[XA], int t) {
#pragma unroll
                    for (int j = 0; j < XA; ++j)
                        xa[j] = __builtin_bit_cast(v8h, xrow[(FMT == kW8C ? t * 8 + j * 4 : (4 * t + j) * 4) * M]);
                };
                v4f d_prev = {0.0f, 0.0f, 0.0f, 0.0f};
                _Float16 s_prev = (_Float16)0.0f;
                auto tile_math = [&](const v8h(&xa)[XA], int t) {
                    if constexpr (FMT == kW4G32) {
                        const uint32_t wd[4] = {cur[t].x, cur[t].y, cur[t].z, cur[t].w};
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int gl = 4 * t + j;
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
                    } else if constexpr (FMT == kW4C) {
                        accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[0], dequant8(cur[t].x), accw, 0, 0, 0);
                        accw2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[1], dequant8(cur[t].y), accw2, 0, 0, 0);
                        accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[2], dequant8(cur[t].z), accw, 0, 0, 0);
                        accw2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[3], dequant8(cur[t].w), accw2, 0, 0, 0);
                    } else {
                        accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[0], dequant_i8x8(cur[t].x, cur[t].y), accw, 0, 0, 0);
                        accw = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[1], dequant_i8x8(cur[t].z, cur[t].w), accw, 0, 0, 0);
                    }
                };
                if (r == 0) {
                    // token rows of this unit: global -> registers (zeros beyond K) -> LDS
                    const int K8 = a.K / 8;
#pragma unroll
                    for (int i = 0; i < xs.XV; ++i) {
                        const int p = i * 64 + lane;
                        const int m = p / OCT, o = u * OCT + p % OCT;
                        const u32x4 zero = {0, 0, 0, 0};
                        xs.v[i] = o < K8 ? a.x[(size_t)m * K8 + o] : zero;
                    }
                    stage();
                }
                if (nt == TILES) {
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
                } else {
#pragma unroll
                    for (int t = 0; t < TILES; ++t) {
                        if (t < nt) {
                            v8h xa[XA];
                            load_xa(xa, t);
                            tile_math(xa, t);
                        }
                    }
                }
                if (FMT == kW4G32) {
#pragma unroll
                    for (int i = 0; i < MI; ++i) accr[i] = fmaf((float)s_prev, d_prev[i], accr[i]);
                }
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    if (rr == r) {
#pragma unroll
                        for (int i = 0; i < MI; ++i)
                            acc[rr][i] += FMT == kW4G32 ? accr[i] : FMT == kW4C ? accw[i] + accw2[i] : accw[i];
                    }
                if (++r == R) {
                    r = 0;
                    ++u;
                }
            }
            // the one place where weights are requested: the item this wavefront computes next
            // (its next item of this round, else its first of the workgroup's next round, else
            // its first of the workgroup's first round of the next layer)
            bool ahead = false, in_next = false;
            int nrt = 0, nu = 0;
            if (it + 1 < items) {
                ahead = true;
                nrt = rt0 + r * a.rt_step;
                nu = u;
            } else if (vr + G < L.rounds) {
                const WavePiece p = wave_piece(L, vr + G, wave);
                ahead = p.live && p.u1 > p.u0;
                nrt = p.rt0;
                nu = p.u0;
            } else if (g < next.rounds && wave != kPollWave) {
                const WavePiece p = wave_piece(next, g, wave);
                ahead = p.live && p.u1 > p.u0;
                in_next = true;
                nrt = p.rt0;
                nu = p.u0;
            }
            if (ahead)
                request_item(in_next ? next.packed : L.packed, in_next ? next.rt_stride : L.rt_stride,
                             in_next ? next.KT : L.KT, in_next ? next.fmt : L.fmt, nrt, nu, lane, cur);
        }

        // partial sums meet in LDS: red[wave][r][m][16 rows] (a region of its own: the poll
        // wavefront may still be reading it while the others stage the next round)
        __syncthreads();
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int m = 4 * q + i;
                if (rr < R && m < M) red[((wave * 4 + rr) * M + m) * 16 + c] = acc[rr][i];
            }
        __syncthreads();
        if (wave == kPollWave) {
            for (int s = 0; s < L.slots; ++s) {
                const int vb = vr * L.slots + s;
                if (vb >= L.nblocks) break;
                const int w0 = s * L.waves;
                if (a.gated_out) {
                    const GateCoeffs gc = gate_coeffs(a.act);
                    const int half = a.N / 2;
                    for (int e = lane; e < M * 16; e += 64) {
                        const int cc = e & 15, m = e >> 4;
                        float sg = 0.0f, su = 0.0f;
                        for (int w = w0; w < w0 + L.waves; ++w) {
                            sg += red[((w * 4 + 0) * M + m) * 16 + cc];
                            su += red[((w * 4 + 1) * M + m) * 16 + cc];
                        }
                        const int n = vb * 16 + cc;
                        if (n < half) {
                            if (FMT != kW4G32) {
                                sg *= a.sw[n];
                                su *= a.sw[n + half];
                            }
                            a.y[(size_t)m * half + n] = (_Float16)(gate_activation(sg, gc) * su);
                        }
                    }
                } else {
                    const int b0 = vb * a.row_tiles;
                    const int Rs = min(a.row_tiles, a.RT - b0);
                    for (int e = lane; e < Rs * M * 16; e += 64) {
                        const int cc = e & 15, m = (e >> 4) % M, rr = (e >> 4) / M;
                        float s_ = 0.0f;
                        for (int w = w0; w < w0 + L.waves; ++w) s_ += red[((w * 4 + rr) * M + m) * 16 + cc];
                        const int n = (b0 + rr) * 16 + cc;
                        if (n < a.N) {
                            if (FMT != kW4G32) s_ *= a.sw[n];
                            if (a.res) s_ += (float)a.res[(size_t)m * a.N + n];
                            a.y[(size_t)m * a.N + n] = (_Float16)s_;
                        }
                    }
                }
            }
        }
    }
}

// All layers of a launch have the weight format FMT (the host cuts a chain into such runs: with
// the three formats' code in one kernel the register allocation of each suffers).
template <int M, int FMT>
__global__ __launch_bounds__(64 * kSeqWaves, 4) void gemv_seq_kernel(const SeqLayer *__restrict__ layers, int n,
                                                                  unsigned *sync, long long spin_limit,
                                                                  int red_offset) {
    extern __shared__ u32x4 lds_all[];
    float *red = reinterpret_cast<float *>(lds_all + red_offset);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u32x4 cur[12];
    DevLayer L = read_layer(layers);
    if ((int)blockIdx.x < L.rounds) request_first(L, blockIdx.x, wave, lane, cur);
    for (int f = 0; f < n; ++f) {
        const bool last = f + 1 == n;
        DevLayer next = read_layer(layers + (last ? f : f + 1));
        if (last) next.rounds = 0;  // nothing to look ahead to
        run_layer<M, FMT>(L, next, lds_all, red, cur, wave, lane);
        if (!last) {
            grid_barrier(sync, (unsigned)(f + 1) * gridDim.x, spin_limit, wave, lane);
            // the polling wavefront asks for its first item only now
            if (wave == kPollWave && (int)blockIdx.x < next.rounds) request_first(next, blockIdx.x, wave, lane, cur);
        }
        L = next;
    }
}

// sync: two words (arrival counter, time-out flag) per run of layers, 32 runs at most
__global__ void seq_reset_kernel(unsigned *sync) { sync[threadIdx.x] = 0u; }

typedef void (*SeqKernel)(const SeqLayer *, int, unsigned *, long long, int);

template <int M>
SeqKernel seq_kernel_fmt(int fmt) {
    return fmt == kW4G32 ? gemv_seq_kernel<M, kW4G32> : fmt == kW4C ? gemv_seq_kernel<M, kW4C> : gemv_seq_kernel<M, kW8C>;
}

SeqKernel seq_kernel(int M, int fmt) {
    switch (M) {
        case 1: return seq_kernel_fmt<1>(fmt);
        case 2: return seq_kernel_fmt<2>(fmt);
        case 3: return seq_kernel_fmt<3>(fmt);
        case 4: return seq_kernel_fmt<4>(fmt);
        default: return nullptr;
    }
}

// staged token rows of 8 wavefronts (int4 unit: 128 vectors per row), then the partial sums
size_t seq_x_bytes(int M) { return (size_t)kSeqWaves * 128 * M * 16; }
size_t seq_lds_bytes(int M) { return seq_x_bytes(M) + (size_t)kSeqWaves * 4 * M * 16 * sizeof(float); }

}  // namespace

void fill_seq_layer(void *dst, const Geometry &g, const void *packed, const void *x, void *y, const Fusion &f,
                    int M, int num_cus, int *rounds) {
    const GemvPlan p = plan_gemv(g, M, num_cus);
    SeqLayer L;
    L.a = make_gemv_args(g, packed, x, y, f, p);
    L.fmt = g.fmt;
    L.waves = p.waves;
    L.slots = kSeqWaves / p.waves;
    L.nblocks = f.gated_output ? g.RT / 2 : (g.RT + p.row_tiles - 1) / p.row_tiles;
    L.rounds = (L.nblocks + L.slots - 1) / L.slots;
    *static_cast<SeqLayer *>(dst) = L;
    *rounds = L.rounds;
}

// Workgroups of the kernel for (M, fmt) that are resident at the same time.
hipError_t seq_resident_workgroups(int M, int fmt, int num_cus, int *grid) {
    const SeqKernel k = seq_kernel(M, fmt);
    if (!k) return hipErrorInvalidValue;
    int per_cu = 0;
    const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k, 64 * kSeqWaves, seq_lds_bytes(M));
    if (e != hipSuccess) return e;
    if (per_cu < 1) return hipErrorInvalidValue;
    if (per_cu > 2) per_cu = 2;
    *grid = per_cu * num_cus;
    return hipSuccess;
}

hipError_t launch_gemv_seq_reset(unsigned *sync, hipStream_t st) {
    seq_reset_kernel<<<1, 64, 0, st>>>(sync);
    return hipGetLastError();
}

// n consecutive layer records of one weight format; sync = this run's two words (zero)
hipError_t launch_gemv_seq(const void *layers, int n, int M, int fmt, unsigned *sync, int grid, hipStream_t st) {
    const SeqKernel k = seq_kernel(M, fmt);
    if (!k) return hipErrorInvalidValue;
    const long long limit = (long long)tuning().seq_spin_limit_us * 100;  // 100 MHz wall clock
    const int red_offset = (int)(seq_x_bytes(M) / 16);
    k<<<dim3((unsigned)grid), dim3(64 * kSeqWaves), seq_lds_bytes(M), st>>>(static_cast<const SeqLayer *>(layers), n,
                                                                             sync, limit, red_offset);
    return hipGetLastError();
}

}  // namespace qfc
