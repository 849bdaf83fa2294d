// Measurement probe, not part of the product path: a register-only loop of back-to-back MFMAs with
// no memory traffic at all, to find out what rate and what shader clock the matrix cores hold with
// constant and with random operands.  The prefill kernels' fractions of the published peak are
// read against these figures.
#include "qfc_internal.h"
#include "../../include/qfc_experimental.h"

namespace qfc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// KIND 0: v_mfma_i32_32x32x32_i8, 1: v_mfma_f32_32x32x16_f16.  Eight accumulators, eight operand pairs
// used in rotation (with random operands consecutive MFMAs see unrelated bits; with constant ones
// every operand register holds the same value).  ticks[2 b] = shader clock ticks, ticks[2 b + 1] =
// ticks of the constant 100 MHz counter, both over the loop of workgroup b's first wavefront.
template <int KIND>
__global__ __launch_bounds__(256, 2) void probe_mfma_kernel(int iters, int random, uint64_t *ticks) {
    v16i acc[8];
    v16f accf[8];
    v4i a[8], b[8];
    v8h ah[8], bh[8];
    const uint32_t id = blockIdx.x * 256 + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) { acc[i][e] = 0; accf[i][e] = 0.0f; }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[i][e] = random ? (int)mix(id * 64 + i * 8 + e) : 0x01010101;
            b[i][e] = random ? (int)mix(id * 64 + i * 8 + 4 + e) : 0x01010101;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {  // finite binary16 values in [-1, 1)
            ah[i][e] = random ? (_Float16)((int)(mix(id * 128 + i * 16 + e) & 2047) - 1024) * (_Float16)(1.0f / 1024) : (_Float16)1.0f;
            bh[i][e] = random ? (_Float16)((int)(mix(id * 128 + i * 16 + 8 + e) & 2047) - 1024) * (_Float16)(1.0f / 1024) : (_Float16)1.0f;
        }
    }
    const uint64_t c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (KIND == 0)
                    acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[(i + r) & 7], b[i], acc[i], 0, 0, 0);
                else
                    accf[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[(i + r) & 7], bh[i], accf[i], 0, 0, 0);
            }
        if (KIND == 1 && (it & 63) == 63) {  // keep the fp32 sums finite
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) accf[i][e] *= 0.5f;
        }
    }
    const uint64_t c1 = clock64(), w1 = wall_clock64();
    int s = 0;
    float fs = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            s += acc[i][e];
            fs += accf[i][e];
        }
    s += __float_as_int(fs);
    if (threadIdx.x == 0) {
        ticks[2 * blockIdx.x] = c1 - c0 + (s == 0x7fffffff ? 1 : 0);  // (the sums are used, so the loop stays)
        ticks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

}  // namespace
}  // namespace qfc

extern "C" qfc_status_t qfc_probe_mfma(int32_t kind, int32_t random_operands, int32_t iters, int32_t workgroups,
                                       uint64_t *ticks, void *stream) {
    if ((kind != 0 && kind != 1) || iters < 1 || iters > (1 << 22) || workgroups < 1 || workgroups > 4096 || !ticks)
        return QFC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(ticks) & 7u) return QFC_ERR_ALIGNMENT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (kind == 0)
        qfc::probe_mfma_kernel<0><<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, random_operands, ticks);
    else
        qfc::probe_mfma_kernel<1><<<dim3((unsigned)workgroups), 256, 0, st>>>(iters, random_operands, ticks);
    return hipGetLastError() == hipSuccess ? QFC_OK : QFC_ERR_HIP;
}
