// Internal declarations shared by the translation units of libqfc.so.
// Physical weight layouts (the "weights conversion" of section 3.4 of the
// paper; the layouts themselves are this library's own, chosen for 64-lane
// wavefronts and 16-byte lane loads):
//
// W8C (int8 codes, fp32 scale per output channel)
//   rows are grouped in blocks of 64, K in chunks of 16 codes.  One 1 KiB tile
//   holds chunk kc of the 64 rows of row block rb: lane r owns the 16 bytes
//   (rb*64 + r, kc*16 .. kc*16+15).  Tiles are stored [rb][kc].  A wavefront
//   load of 16 B per lane is therefore one contiguous KiB, every lane works on
//   its own output row (no cross-lane reduction), and the same tile is an MFMA
//   int8 operand fragment when 16 rows x 4 chunks are read from LDS.
//   K is padded to a multiple of 256 and N to a multiple of 256 with zero
//   codes.  The fp32 scales [Np] follow the codes.
//
// W4G32 (int4 codes, binary16 scale per 32 consecutive k)
//   a unit is 64 rows x 256 k = 9 KiB: eight 1 KiB tiles (tile j = quantization
//   group j of the unit; lane r owns the 32 codes of (row r, group j) in 16
//   bytes) followed by one 1 KiB tile of scales (lane r owns the eight binary16
//   scales of its row).  Units are stored [rb][k/256].  Codes are stored biased
//   (q + 8) and nibble-interleaved so that two mask operations per byte pair
//   yield k-adjacent binary16 pairs: code e (0..7) of a dword sits in nibble
//   (e >> 1) + 4 * (e & 1).  Padding codes are 8 (zero), padding scales 0.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qfc.h"

namespace qfc {

constexpr int kRowsPerBlock = 64;
constexpr int kPadN = 256;
constexpr int kPadK = 256;
constexpr int kW4UnitVecs = 9 * 64;  // 16-byte vectors per W4G32 unit
constexpr int kMaxDecodeM = 8;

enum Format { kW8C = 0, kW4G32 = 1 };

struct Geometry {
    int N, K;    // logical
    int Np, Kp;  // padded
    int RB;      // row blocks holding real rows: ceil(N / 64)
    int RBp;     // Np / 64
    int fmt;
    size_t code_bytes;   // bytes of the code (+ group scale) region
    size_t scale_off;    // W8C: byte offset of the fp32 scales
    size_t total_bytes;
};

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

inline Geometry make_geometry(int N, int K, int fmt) {
    Geometry g;
    g.N = N; g.K = K; g.fmt = fmt;
    g.Np = round_up(N, kPadN);
    g.Kp = round_up(K, kPadK);
    g.RB = (N + kRowsPerBlock - 1) / kRowsPerBlock;
    g.RBp = g.Np / kRowsPerBlock;
    if (fmt == kW8C) {
        g.code_bytes = (size_t)g.Np * g.Kp;
        g.scale_off = g.code_bytes;
        g.total_bytes = g.code_bytes + (size_t)g.Np * 4;
    } else {
        g.code_bytes = (size_t)g.RBp * (g.Kp / 256) * kW4UnitVecs * 16;
        g.scale_off = 0;
        g.total_bytes = g.code_bytes;
    }
    return g;
}

struct GemvPlan {
    int waves;   // wavefronts per workgroup
    int splits;  // workgroups sharing one row block (K split)
    int units;   // work units along K per row block
};

// Tunables (set through qfc_tune, used by the planners).
struct Tuning {
    int gemv_target_waves = 4096;
    int gemv_max_waves_per_wg = 8;
    int gemm_variant = 0;
};
Tuning &tuning();

GemvPlan plan_gemv(const Geometry &g, int M, int num_cus);
size_t gemv_workspace_bytes(const Geometry &g, int M, int num_cus);

// Launchers.  Every one validates nothing (the C ABI layer did) and returns
// the hipError_t of the launch.
hipError_t launch_pack(const Geometry &g, const int8_t *wq, const void *scales, void *packed,
                       hipStream_t st);
hipError_t launch_unpack(const Geometry &g, const void *packed, int8_t *wq, void *scales,
                         hipStream_t st);
hipError_t launch_gemv(const Geometry &g, const void *packed, const void *x, int M, void *y,
                       void *workspace, int num_cus, hipStream_t st);
hipError_t launch_act_quant(const void *x, int M, int K, int8_t *xq, float *sx, int tiled,
                            int Mp, int Kp, hipStream_t st);
hipError_t launch_retile_xq(const int8_t *xq, int M, int K, int8_t *tiled, int Mp, int Kp,
                            hipStream_t st);
// out_mode 0: binary16 y with scales; 1: raw int32 accumulators.
hipError_t launch_gemm_i8(const Geometry &g, const void *packed, const int8_t *xq_tiled,
                          const float *sx, int M, int Mp, void *out, int out_mode,
                          hipStream_t st);
hipError_t launch_gemm_f16(const Geometry &g, const void *packed, const void *x, int M, void *y,
                           hipStream_t st);

}  // namespace qfc
