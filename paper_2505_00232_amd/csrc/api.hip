// C ABI of libqfc.so: argument checking, handle bookkeeping and dispatch
// (decode kernel for M <= 8, prefill kernels above; section 3.7 of the paper:
// the stage decides the kernel).  All arithmetic is in the kernels' files.
#include <new>

#include "../../include/qfc_experimental.h"
#include "qfc_internal.h"

using namespace qfc;

struct qfc_weights_s {
    uint32_t magic;
    qfc_desc_t desc;
    Geometry geo;
    void *packed;
    void *workspace;
    size_t workspace_bytes;
    int num_cus;
};

namespace {

constexpr uint32_t kMagic = 0x51464331u;  // "QFC1"

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

qfc_status_t check_desc(const qfc_desc_t *d, int *fmt) {
    if (!d) return QFC_ERR_INVALID_ARG;
    if (d->N < 1 || d->K < 1 || d->K % 32 != 0) return QFC_ERR_INVALID_ARG;
    if (d->wbits != 8 && d->wbits != 4) return QFC_ERR_INVALID_ARG;
    if (d->group_size < 0) return QFC_ERR_INVALID_ARG;
    if (d->scale_dtype != QFC_SCALE_F32 && d->scale_dtype != QFC_SCALE_F16) return QFC_ERR_INVALID_ARG;
    if (d->compute_mode != QFC_COMPUTE_FP16_DEQUANT && d->compute_mode != QFC_COMPUTE_INT8_ACT &&
        d->compute_mode != QFC_COMPUTE_INT8_ACT_DECODE)
        return QFC_ERR_INVALID_ARG;
    if (d->flags != 0 && d->flags != QFC_PACK_GATED_PAIRS) return QFC_ERR_INVALID_ARG;
    if (d->flags == QFC_PACK_GATED_PAIRS && d->N % 32 != 0) return QFC_ERR_INVALID_ARG;
    // (the decode design with in-kernel quantization has no merged gating)
    if (d->flags == QFC_PACK_GATED_PAIRS && d->compute_mode == QFC_COMPUTE_INT8_ACT_DECODE) return QFC_ERR_UNSUPPORTED;
    if (d->wbits == 8 && d->group_size == 0 && d->scale_dtype == QFC_SCALE_F32) {
        *fmt = kW8C;
    } else if (d->wbits == 4 && d->group_size == 32 && d->scale_dtype == QFC_SCALE_F16) {
        *fmt = kW4G32;
        if (d->compute_mode != QFC_COMPUTE_FP16_DEQUANT) return QFC_ERR_UNSUPPORTED;
    } else if (d->wbits == 4 && d->group_size == 0 && d->scale_dtype == QFC_SCALE_F32) {
        *fmt = kW4C;
    } else {
        return QFC_ERR_UNSUPPORTED;
    }
    // int32 accumulators must hold K * 127 * 128
    if ((int64_t)d->K * 127 * 128 > INT32_MAX) return QFC_ERR_UNSUPPORTED;
    return QFC_OK;
}

bool valid(qfc_handle_t h) { return h && h->magic == kMagic; }

int prefill_rows(int M) { return round_up(M, 256); }

// Workspace: the tiled int8 activations and their scales (int8 weights only).
size_t int8_region(const Geometry &g, int M) {
    const size_t Mp = (size_t)prefill_rows(M);
    return Mp * (size_t)g.Kp + Mp * sizeof(float);
}

// Formats whose M > 8 path multiplies int8 activations: 8-bit weights unless the handle asks for the
// fp16 path, 4-bit per-channel weights when it asks for int8 activations.
bool int8_prefill(qfc_handle_t h) {
    if (h->geo.fmt == kW8C) return h->desc.compute_mode != QFC_COMPUTE_FP16_DEQUANT;
    return h->geo.fmt == kW4C && h->desc.compute_mode == QFC_COMPUTE_INT8_ACT;
}

size_t workspace_need(qfc_handle_t h, int M) {
    return h->geo.fmt == kW8C || int8_prefill(h) ? int8_region(h->geo, M) : 256;
}

qfc_status_t hip_status(hipError_t e) { return e == hipSuccess ? QFC_OK : QFC_ERR_HIP; }

// ---- scratch of the entry point that allocates nothing (qfc_forward_static)
// Device memory that is part of the library's code object: every GPU the library runs on holds its
// own copy, at its own address, until the process ends.  In host code the array's NAME is only a
// stand-in for the symbol, not a device address; the address on the current device comes from
// hipGetSymbolAddress, once per device, and only that pointer is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = QFC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// The array's address on the current device (looked up on the first call on that device).
qfc_status_t static_scratch(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return QFC_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return QFC_ERR_UNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QFC_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // (two first callers store the same address)
    }
    *out = p;
    return QFC_OK;
}

// Common checks of the int8 entry points; on success the tiled activations are in the workspace.
qfc_status_t stage_xq(qfc_handle_t h, const int8_t *xq, int M, int8_t **tiled, float **sx_ws,
                      hipStream_t st) {
    if (!valid(h) || !xq || M < 1) return QFC_ERR_INVALID_ARG;
    if (h->geo.fmt != kW8C && !int8_prefill(h)) return QFC_ERR_UNSUPPORTED;
    if (h->geo.pair_half) return QFC_ERR_UNSUPPORTED;  // a layer packed in pairs only computes the gated output
    if (!aligned16(xq)) return QFC_ERR_ALIGNMENT;
    if (!h->workspace || h->workspace_bytes < workspace_need(h, M)) return QFC_ERR_BUFFER_TOO_SMALL;
    const int Mp = prefill_rows(M);
    char *body = static_cast<char *>(h->workspace);
    *tiled = reinterpret_cast<int8_t *>(body);
    *sx_ws = reinterpret_cast<float *>(body + (size_t)Mp * h->geo.Kp);
    return hip_status(launch_retile_xq(xq, M, h->geo.K, *tiled, Mp, h->geo.Kp, h->geo.fmt == kW4C, st));
}

}  // namespace

extern "C" {

qfc_status_t qfc_packed_size(const qfc_desc_t *desc, size_t *bytes) {
    int fmt = 0;
    if (!bytes) return QFC_ERR_INVALID_ARG;
    const qfc_status_t s = check_desc(desc, &fmt);
    if (s != QFC_OK) return s;
    *bytes = make_geometry(desc->N, desc->K, fmt, desc->flags == QFC_PACK_GATED_PAIRS).total_bytes;
    return QFC_OK;
}

qfc_status_t qfc_pack_weights(const qfc_desc_t *desc, const int8_t *wq_logical, const void *scales,
                              void *packed, size_t packed_bytes, void *stream, qfc_handle_t *out) {
    int fmt = 0;
    if (!out) return QFC_ERR_INVALID_ARG;
    *out = nullptr;
    const qfc_status_t s = check_desc(desc, &fmt);
    if (s != QFC_OK) return s;
    if (!wq_logical || !scales || !packed) return QFC_ERR_INVALID_ARG;
    if (!aligned16(wq_logical) || !aligned16(scales) || !aligned16(packed)) return QFC_ERR_ALIGNMENT;
    const Geometry g = make_geometry(desc->N, desc->K, fmt, desc->flags == QFC_PACK_GATED_PAIRS);
    if (packed_bytes < g.total_bytes) return QFC_ERR_BUFFER_TOO_SMALL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return QFC_ERR_HIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return QFC_ERR_HIP;
    if (launch_pack(g, wq_logical, scales, packed, static_cast<hipStream_t>(stream)) != hipSuccess)
        return QFC_ERR_HIP;
    qfc_weights_s *h = new (std::nothrow) qfc_weights_s;
    if (!h) return QFC_ERR_HIP;
    h->magic = kMagic;
    h->desc = *desc;
    h->geo = g;
    h->packed = packed;
    h->workspace = nullptr;
    h->workspace_bytes = 0;
    h->num_cus = cus;
    *out = h;
    return QFC_OK;
}

qfc_status_t qfc_unpack_weights(qfc_handle_t h, int8_t *wq_logical, void *scales, void *stream) {
    if (!valid(h) || !wq_logical || !scales) return QFC_ERR_INVALID_ARG;
    if (!aligned16(wq_logical) || !aligned16(scales)) return QFC_ERR_ALIGNMENT;
    return hip_status(launch_unpack(h->geo, h->packed, wq_logical, scales, static_cast<hipStream_t>(stream)));
}

qfc_status_t qfc_workspace_size(qfc_handle_t h, int32_t M, size_t *bytes) {
    if (!valid(h) || !bytes || M < 1) return QFC_ERR_INVALID_ARG;
    *bytes = workspace_need(h, M);
    return QFC_OK;
}

qfc_status_t qfc_bind_workspace(qfc_handle_t h, void *workspace, size_t bytes) {
    if (!valid(h) || !workspace) return QFC_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return QFC_ERR_ALIGNMENT;
    if (bytes < 256) return QFC_ERR_BUFFER_TOO_SMALL;
    h->workspace = workspace;
    h->workspace_bytes = bytes;
    return QFC_OK;
}

qfc_status_t qfc_quantize_activations(const void *x_f16, int32_t M, int32_t K, int8_t *xq, float *sx,
                                      void *stream) {
    if (!x_f16 || !xq || !sx || M < 1 || K < 1 || K % 32 != 0) return QFC_ERR_INVALID_ARG;
    if (!aligned16(x_f16) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u)) return QFC_ERR_ALIGNMENT;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return QFC_ERR_HIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return QFC_ERR_HIP;
    return hip_status(launch_act_quant(x_f16, nullptr, 0, M, K, xq, sx, 0, M, K, cus, static_cast<hipStream_t>(stream)));
}

// Shared body of qfc_forward, qfc_forward_fused and qfc_forward_static.  `scratch` is where the
// int8 prefill path keeps the quantized activations and their scales: the handle's bound workspace,
// or the library's static array.
static qfc_status_t forward_impl(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16, const Fusion &f,
                                 void *scratch, size_t scratch_bytes, hipStream_t st) {
    if (!valid(h) || !x_f16 || !y_f16 || M < 1) return QFC_ERR_INVALID_ARG;
    if (!aligned16(x_f16) || !aligned16(y_f16)) return QFC_ERR_ALIGNMENT;
    if ((f.gate && !aligned16(f.gate)) || (f.residual && !aligned16(f.residual))) return QFC_ERR_ALIGNMENT;
    if ((f.gate || f.gated_output) && f.activation != QFC_ACT_SILU && f.activation != QFC_ACT_GELU_TANH)
        return QFC_ERR_INVALID_ARG;
    if (f.gated_output && (f.gate || f.residual || h->geo.N % 32 != 0)) return QFC_ERR_INVALID_ARG;
    if (f.norm_gamma && (f.gate || !aligned16(f.norm_gamma) || !(f.norm_eps >= 0.0f))) return QFC_ERR_INVALID_ARG;
    if (f.norm_gamma && M > kMaxDecodeM) return QFC_ERR_UNSUPPORTED;
    const bool fused = f.gate || f.residual || f.gated_output || f.norm_gamma;
    if (h->geo.pair_half && !f.gated_output) return QFC_ERR_UNSUPPORTED;  // packed in pairs: gated output only
    const int gated_act = f.gated_output ? f.activation : -1;
    if (M <= kMaxDecodeM) {
        if (h->desc.compute_mode == QFC_COMPUTE_INT8_ACT_DECODE) {
            if (fused) return QFC_ERR_UNSUPPORTED;
            return hip_status(launch_gemv_q8(h->geo, h->packed, x_f16, nullptr, 0, M, y_f16, 0, h->num_cus, st));
        }
        return hip_status(launch_gemv(h->geo, h->packed, x_f16, M, y_f16, f, h->num_cus, st));
    }
    if (!int8_prefill(h)) {
        // activations go from memory to LDS without passing registers
        if (f.gate) return QFC_ERR_UNSUPPORTED;
        // a tile holds both branches only when the layer is packed in pairs
        if (f.gated_output && !h->geo.pair_half) return QFC_ERR_UNSUPPORTED;
        const hipError_t e = launch_gemm_f16(h->geo, h->packed, x_f16, M, y_f16, f.residual, gated_act, h->num_cus, st);
        return e == hipErrorNotSupported ? QFC_ERR_UNSUPPORTED : hip_status(e);
    }
    if (f.gated_output && !h->geo.pair_half) return QFC_ERR_UNSUPPORTED;
    if (!scratch || scratch_bytes < workspace_need(h, M)) return QFC_ERR_BUFFER_TOO_SMALL;
    // int8 activations: quantize into the scratch region (tiled), multiply, rescale
    const int Mp = prefill_rows(M);
    char *body = static_cast<char *>(scratch);
    int8_t *tiled = reinterpret_cast<int8_t *>(body);
    float *sx = reinterpret_cast<float *>(body + (size_t)Mp * h->geo.Kp);
    if (launch_act_quant(x_f16, f.gate, f.activation, M, h->geo.K, tiled, sx, h->geo.fmt == kW4C ? 2 : 1, Mp, h->geo.Kp, h->num_cus, st) !=
        hipSuccess)
        return QFC_ERR_HIP;
    return hip_status(launch_gemm_i8(h->geo, h->packed, tiled, sx, M, Mp, y_f16, 0, f.residual, gated_act, h->num_cus, st));
}

qfc_status_t qfc_forward(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16, void *stream) {
    if (!valid(h)) return QFC_ERR_INVALID_ARG;
    return forward_impl(h, x_f16, M, y_f16, Fusion(), h->workspace, h->workspace_bytes, static_cast<hipStream_t>(stream));
}

qfc_status_t qfc_forward_fused(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16,
                               const qfc_fusion_t *fusion, void *stream) {
    Fusion f;
    if (fusion) {
        f.gate = fusion->gate;
        f.activation = fusion->activation;
        f.residual = fusion->residual;
        f.gated_output = fusion->gated_output != 0;
        f.norm_gamma = fusion->norm_gamma;
        f.norm_eps = fusion->norm_eps;
        f.norm_offset = fusion->norm_offset;
    }
    if (!valid(h)) return QFC_ERR_INVALID_ARG;
    return forward_impl(h, x_f16, M, y_f16, f, h->workspace, h->workspace_bytes, static_cast<hipStream_t>(stream));
}

qfc_status_t qfc_forward_static(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16, void *stream) {
    if (!valid(h) || M < 1) return QFC_ERR_INVALID_ARG;
    // Which calls need scratch at all is the dispatcher's business (M > 8 in the int8 mode); the limit
    // is checked for those only, before anything is enqueued.
    if (M > kMaxDecodeM && int8_prefill(h) && workspace_need(h, M) > kStaticScratchBytes) return QFC_ERR_SCRATCH_LIMIT;
    void *p = nullptr;
    const qfc_status_t s = static_scratch(&p);
    if (s != QFC_OK) return s;
    return forward_impl(h, x_f16, M, y_f16, Fusion(), p, kStaticScratchBytes, static_cast<hipStream_t>(stream));
}

qfc_status_t qfc_rmsnorm(const qfc_rmsnorm_t *r, int32_t M, int32_t K, void *stream) {
    if (!r || !r->x || !r->gamma || M < 1 || K < 32 || K % 32 != 0) return QFC_ERR_INVALID_ARG;
    if (!r->h_out && !r->y && !r->xq && !r->consumer) return QFC_ERR_INVALID_ARG;
    if (r->consumer) {
        qfc_handle_t c = r->consumer;
        if (!valid(c) || c->geo.K != K || M <= kMaxDecodeM) return QFC_ERR_INVALID_ARG;
        if (!int8_prefill(c) || c->geo.pair_half) return QFC_ERR_UNSUPPORTED;
        if (!c->workspace || c->workspace_bytes < workspace_need(c, M)) return QFC_ERR_BUFFER_TOO_SMALL;
    }
    if ((r->xq == nullptr) != (r->sx == nullptr)) return QFC_ERR_INVALID_ARG;
    if (!(r->eps >= 0.0f)) return QFC_ERR_INVALID_ARG;
    if (K > 14336) return QFC_ERR_UNSUPPORTED;
    if (!aligned16(r->x) || !aligned16(r->gamma) || (r->residual && !aligned16(r->residual)) ||
        (r->h_out && !aligned16(r->h_out)) || (r->y && !aligned16(r->y)) || (r->xq && !aligned16(r->xq)) ||
        (reinterpret_cast<uintptr_t>(r->sx) & 3u))
        return QFC_ERR_ALIGNMENT;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return QFC_ERR_HIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return QFC_ERR_HIP;
    RmsNormArgs a;
    a.x = r->x;
    a.residual = r->residual;
    a.gamma = r->gamma;
    a.h_out = r->h_out;
    a.y = r->y;
    a.xq = r->xq;
    a.sx = r->sx;
    a.eps = r->eps;
    a.gamma_offset = r->gamma_offset;
    if (r->consumer) {
        // the row-major outputs, if asked for, by a launch of their own; then the tiled ones
        qfc_handle_t c = r->consumer;
        if (r->xq) {
            RmsNormArgs b = a;
            b.h_out = nullptr;
            b.y = nullptr;
            if (launch_rmsnorm(b, M, K, cus, static_cast<hipStream_t>(stream)) != hipSuccess) return QFC_ERR_HIP;
        }
        const int Mp = prefill_rows(M);
        char *body = static_cast<char *>(c->workspace);
        a.xq = reinterpret_cast<int8_t *>(body);
        a.sx = reinterpret_cast<float *>(body + (size_t)Mp * c->geo.Kp);
        a.tiled = c->geo.fmt == kW4C ? 2 : 1;
        a.Mp = Mp;
        a.Kp = c->geo.Kp;
    }
    return hip_status(launch_rmsnorm(a, M, K, cus, static_cast<hipStream_t>(stream)));
}

static qfc_status_t check_attn_shape(const qfc_attn_shape_t *a, int32_t S) {
    if (!a || a->batch < 1 || a->h_q < 1 || a->h_kv < 1 || a->h_q % a->h_kv != 0 || S < 1 || a->cache_size < 64 ||
        a->cache_size % 64 != 0)
        return QFC_ERR_INVALID_ARG;
    if (a->d_head != 64 && a->d_head != 128 && a->d_head != 256) return QFC_ERR_UNSUPPORTED;
    return QFC_OK;
}

qfc_status_t qfc_rope_qkv(const void *qkv_f16, int32_t S, int32_t pos0, const qfc_attn_shape_t *a, float rope_base,
                          void *q_out, void *kcache, void *vcache, void *stream) {
    const qfc_status_t s = check_attn_shape(a, S);
    if (s != QFC_OK) return s;
    if (!qkv_f16 || !q_out || !kcache || !vcache || pos0 < 0 || !(rope_base > 1.0f)) return QFC_ERR_INVALID_ARG;
    if ((long)pos0 + S > a->cache_size) return QFC_ERR_INVALID_ARG;
    if (!aligned16(qkv_f16) || !aligned16(q_out) || !aligned16(kcache) || !aligned16(vcache)) return QFC_ERR_ALIGNMENT;
    return hip_status(launch_rope_qkv(qkv_f16, a->batch, S, a->h_q, a->h_kv, a->d_head, a->cache_size, pos0, rope_base,
                                      q_out, kcache, vcache, static_cast<hipStream_t>(stream)));
}

qfc_status_t qfc_rope_table(const qfc_attn_shape_t *a, float rope_base, int32_t positions, float *table, void *stream) {
    const qfc_status_t s = check_attn_shape(a, 1);
    if (s != QFC_OK) return s;
    if (!table || positions < 1 || !(rope_base > 1.0f)) return QFC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(table) & 7u) return QFC_ERR_ALIGNMENT;
    return hip_status(launch_rope_table(a->d_head, rope_base, positions, table, static_cast<hipStream_t>(stream)));
}

qfc_status_t qfc_forward_qkv_rope(qfc_handle_t h, const void *x_f16, const qfc_fusion_t *fusion,
                                  const qfc_attn_shape_t *a, int32_t pos0, const float *rope_table,
                                  int32_t table_positions, void *q_out, void *kcache, void *vcache, void *stream) {
    if (!valid(h)) return QFC_ERR_INVALID_ARG;
    const qfc_status_t s = check_attn_shape(a, 1);
    if (s != QFC_OK) return s;
    if (!x_f16 || !rope_table || !q_out || !kcache || !vcache || pos0 < 0 || pos0 >= a->cache_size || pos0 >= table_positions)
        return QFC_ERR_INVALID_ARG;
    if (h->geo.N != (a->h_q + 2 * a->h_kv) * a->d_head) return QFC_ERR_INVALID_ARG;
    if (!aligned16(x_f16) || !aligned16(q_out) || !aligned16(kcache) || !aligned16(vcache) ||
        (reinterpret_cast<uintptr_t>(rope_table) & 7u))
        return QFC_ERR_ALIGNMENT;
    // decode only: the batch is the layer's M token rows, one new position per sequence
    if (a->batch > kMaxDecodeM || h->geo.pair_half || h->desc.compute_mode == QFC_COMPUTE_INT8_ACT_DECODE)
        return QFC_ERR_UNSUPPORTED;
    Fusion f;
    if (fusion) {
        if (fusion->gate || fusion->residual || fusion->gated_output) return QFC_ERR_INVALID_ARG;
        f.norm_gamma = fusion->norm_gamma;
        f.norm_eps = fusion->norm_eps;
        f.norm_offset = fusion->norm_offset;
        if (f.norm_gamma && (!aligned16(f.norm_gamma) || !(f.norm_eps >= 0.0f))) return QFC_ERR_INVALID_ARG;
    }
    RopeOut r;
    r.d = a->d_head;
    r.h_q = a->h_q;
    r.h_kv = a->h_kv;
    r.C = a->cache_size;
    r.pos = pos0;
    r.table = rope_table;
    r.q = q_out;
    r.kc = kcache;
    r.vc = vcache;
    f.rope = &r;
    return hip_status(launch_gemv(h->geo, h->packed, x_f16, a->batch, nullptr, f, h->num_cus, static_cast<hipStream_t>(stream)));
}

static int device_cus() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cus;
}

static size_t attn_workspace(const qfc_attn_shape_t *a, int32_t S) {
    // many query rows: partial results only for launches of few blocks (whose walks are cut into chunks)
    if (S * (a->h_q / a->h_kv) > 16)
        return attn_prefill_workspace(a->batch * a->h_kv, S * (a->h_q / a->h_kv), a->d_head, device_cus());
    const size_t rows = (size_t)a->batch * a->h_kv * kAttnMaxSplits * (size_t)(S * (a->h_q / a->h_kv));
    return rows * (a->d_head + 2) * sizeof(float);
}

qfc_status_t qfc_attention_workspace_size(const qfc_attn_shape_t *a, int32_t S, size_t *bytes) {
    if (!bytes) return QFC_ERR_INVALID_ARG;
    const qfc_status_t s = check_attn_shape(a, S);
    if (s != QFC_OK) return s;
    *bytes = attn_workspace(a, S);
    return QFC_OK;
}

qfc_status_t qfc_attention(const void *q, const void *kcache, const void *vcache, int32_t S, int32_t n_ctx,
                           const qfc_attn_shape_t *a, void *workspace, size_t workspace_bytes, void *out_f16,
                           void *stream) {
    const qfc_status_t s = check_attn_shape(a, S);
    if (s != QFC_OK) return s;
    if (!q || !kcache || !vcache || !workspace || !out_f16 || n_ctx < S || n_ctx > a->cache_size)
        return QFC_ERR_INVALID_ARG;
    const int g = a->h_q / a->h_kv;
    if (!aligned16(q) || !aligned16(kcache) || !aligned16(vcache) || !aligned16(workspace) || !aligned16(out_f16))
        return QFC_ERR_ALIGNMENT;
    if (workspace_bytes < attn_workspace(a, S)) return QFC_ERR_BUFFER_TOO_SMALL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return QFC_ERR_HIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return QFC_ERR_HIP;
    return hip_status(launch_attention(q, kcache, vcache, a->batch * a->h_kv, S, g, a->d_head, a->cache_size, n_ctx,
                                       workspace, out_f16, cus, static_cast<hipStream_t>(stream)));
}

qfc_status_t qfc_forward_q8(qfc_handle_t h, const int8_t *xq, const float *sx, int32_t M, void *y_f16,
                            void *stream) {
    if (!xq && !sx) {
        // the activations a preceding qfc_rmsnorm with consumer == h left in the workspace
        if (!valid(h) || !y_f16 || M <= kMaxDecodeM) return QFC_ERR_INVALID_ARG;
        if (!aligned16(y_f16)) return QFC_ERR_ALIGNMENT;
        if (!int8_prefill(h) || h->geo.pair_half) return QFC_ERR_UNSUPPORTED;
        if (!h->workspace || h->workspace_bytes < workspace_need(h, M)) return QFC_ERR_BUFFER_TOO_SMALL;
        const int Mp = prefill_rows(M);
        char *body = static_cast<char *>(h->workspace);
        return hip_status(launch_gemm_i8(h->geo, h->packed, reinterpret_cast<const int8_t *>(body),
                                         reinterpret_cast<const float *>(body + (size_t)Mp * h->geo.Kp), M, Mp, y_f16, 0,
                                         nullptr, -1, h->num_cus, static_cast<hipStream_t>(stream)));
    }
    if (!sx || !y_f16) return QFC_ERR_INVALID_ARG;
    if (!aligned16(y_f16) || (reinterpret_cast<uintptr_t>(sx) & 3u)) return QFC_ERR_ALIGNMENT;
    if (valid(h) && h->geo.pair_half) return QFC_ERR_UNSUPPORTED;
    if (valid(h) && xq && M >= 1 && M <= kMaxDecodeM && (h->geo.fmt == kW8C || h->geo.fmt == kW4C)) {
        if (!aligned16(xq)) return QFC_ERR_ALIGNMENT;
        return hip_status(launch_gemv_q8(h->geo, h->packed, xq, sx, 1, M, y_f16, 0, h->num_cus,
                                         static_cast<hipStream_t>(stream)));
    }
    int8_t *tiled = nullptr;
    float *sx_ws = nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const qfc_status_t s = stage_xq(h, xq, M, &tiled, &sx_ws, st);
    if (s != QFC_OK) return s;
    return hip_status(launch_gemm_i8(h->geo, h->packed, tiled, sx, M, prefill_rows(M), y_f16, 0, nullptr, -1, h->num_cus, st));
}

qfc_status_t qfc_forward_acc_i32(qfc_handle_t h, const int8_t *xq, int32_t M, int32_t *acc, void *stream) {
    if (!acc) return QFC_ERR_INVALID_ARG;
    if (!aligned16(acc)) return QFC_ERR_ALIGNMENT;
    if (valid(h) && h->geo.pair_half) return QFC_ERR_UNSUPPORTED;
    if (valid(h) && xq && M >= 1 && M <= kMaxDecodeM && (h->geo.fmt == kW8C || h->geo.fmt == kW4C)) {
        if (!aligned16(xq)) return QFC_ERR_ALIGNMENT;
        return hip_status(launch_gemv_q8(h->geo, h->packed, xq, nullptr, 1, M, acc, 1, h->num_cus,
                                         static_cast<hipStream_t>(stream)));
    }
    int8_t *tiled = nullptr;
    float *sx_ws = nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const qfc_status_t s = stage_xq(h, xq, M, &tiled, &sx_ws, st);
    if (s != QFC_OK) return s;
    return hip_status(launch_gemm_i8(h->geo, h->packed, tiled, nullptr, M, prefill_rows(M), acc, 1, nullptr, -1, h->num_cus, st));
}

qfc_status_t qfc_embedding(qfc_handle_t h, const int32_t *ids, int32_t M, void *y_f16, void *stream) {
    if (!valid(h) || !ids || !y_f16 || M < 1) return QFC_ERR_INVALID_ARG;
    if (!aligned16(y_f16) || (reinterpret_cast<uintptr_t>(ids) & 3u)) return QFC_ERR_ALIGNMENT;
    if (M > 65535) return QFC_ERR_UNSUPPORTED;  // one grid row per token
    if (h->geo.pair_half) return QFC_ERR_UNSUPPORTED;
    return hip_status(launch_embedding(h->geo, h->packed, ids, M, y_f16, static_cast<hipStream_t>(stream)));
}

qfc_status_t qfc_forward_batch(const qfc_handle_t *handles, const void *const *xs, int32_t M,
                               void *const *ys, int32_t count, void *stream) {
    if (!handles || !xs || !ys || count < 0) return QFC_ERR_INVALID_ARG;
    for (int32_t i = 0; i < count; ++i) {
        const qfc_status_t s = qfc_forward(handles[i], xs[i], M, ys[i], stream);
        if (s != QFC_OK) return s;
    }
    return QFC_OK;
}

qfc_status_t qfc_destroy(qfc_handle_t h) {
    if (!valid(h)) return QFC_ERR_INVALID_ARG;
    h->magic = 0;
    delete h;
    return QFC_OK;
}

const char *qfc_status_string(qfc_status_t s) {
    switch (s) {
        case QFC_OK: return "ok";
        case QFC_ERR_INVALID_ARG: return "invalid argument";
        case QFC_ERR_UNSUPPORTED: return "unsupported combination";
        case QFC_ERR_BUFFER_TOO_SMALL: return "buffer too small";
        case QFC_ERR_ALIGNMENT: return "pointer not 16-byte aligned";
        case QFC_ERR_HIP: return "HIP runtime error";
        case QFC_ERR_SCRATCH_LIMIT: return "input needs more scratch than the library's static array holds";
    }
    return "unknown status";
}

// Tunables for tests and sweeps (include/qfc_experimental.h; not part of the interface).
void qfc_tune(int32_t key, int32_t value) {
    Tuning &t = tuning();
    if (key == 0) t.gemv_target_waves = value;
    if (key == 1) t.gemv_max_row_tiles = value;
    if (key == 2) t.gemm_variant = value;
    if (key == 3) t.act_quant_rows = value;
    if (key == 4) t.gemv_half = value;
    if (key == 5) t.attn_pair = value;
    if (key == 6) t.attn_chunks = value;
}

}  // extern "C"
