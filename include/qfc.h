/*
 * qfc - weight-only-quantized fully-connected layer for MI355X (gfx950).
 *
 * C ABI of the hot path of LLM inference as the paper states it (section 3.7,
 * "Stage-Aware Optimizations for LLM Inference", and the weight formats of
 * section 4.2): the same quantized weights, resident in GPU memory, serve
 *   - decode  (M <= 8 token rows): a bandwidth-bound fully connected kernel
 *     that streams the packed weights once and dequantizes them in registers;
 *   - prefill (M > 8): either a quantization kernel that turns the float
 *     activations into int8 plus one scale per token, an int8 x int8 -> int32
 *     matrix product on the matrix cores and a dequantizing epilogue, or an
 *     fp16 matrix product over weights dequantized on the fly.
 * Weights are converted once, at load time, from their logical [N, K] form to
 * a physical layout chosen for the kernels (section 3.1 weight layouts,
 * section 3.4 "weights conversion").
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     All work is enqueued on it; no call synchronizes, allocates device
 *     memory or changes the current device.
 *   - The caller owns every buffer.  A handle is a small host object that
 *     borrows `packed` and the bound workspace: keep both alive, and do not
 *     write to them, until qfc_destroy.
 *   - Every call returns a qfc_status_t.  Argument errors are detected on the
 *     host before anything is launched; a failed launch gives QFC_ERR_HIP.
 *     No exception crosses this boundary.
 *   - Device pointers must be 16-byte aligned.  K must be a multiple of 32.
 *   - Calls that share a workspace must not overlap in time (same stream, or
 *     ordered by the caller).
 */
#ifndef QFC_H
#define QFC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct qfc_weights_s *qfc_handle_t;

typedef enum {
    QFC_OK = 0,
    QFC_ERR_INVALID_ARG = 1,      /* null pointer, bad enum, non-positive size, K % 32 != 0 */
    QFC_ERR_UNSUPPORTED = 2,      /* a valid combination this library has no kernel for */
    QFC_ERR_BUFFER_TOO_SMALL = 3, /* packed buffer or workspace smaller than required */
    QFC_ERR_ALIGNMENT = 4,        /* a device pointer is not 16-byte aligned */
    QFC_ERR_HIP = 5,              /* the HIP runtime reported an error */
    QFC_ERR_SCRATCH_LIMIT = 6     /* qfc_forward_static: the call needs more scratch than QFC_STATIC_SCRATCH_BYTES */
} qfc_status_t;

enum { QFC_SCALE_F32 = 0, QFC_SCALE_F16 = 1 };
enum { QFC_COMPUTE_FP16_DEQUANT = 0, QFC_COMPUTE_INT8_ACT = 1, QFC_COMPUTE_INT8_ACT_DECODE = 2 };

/* Description of one quantized linear layer, y[M,N] = x[M,K] . W[N,K]^T.
 * Supported formats (section 4.2 per-channel schemes; group scales are the
 * sub-channel quantization the paper names as its next step):
 *   wbits 8, group_size 0,  scale_dtype F32: int8 codes, one fp32 scale per output channel;
 *   wbits 4, group_size 32, scale_dtype F16: int4 codes in [-8,7], one binary16 scale per
 *                                            32 consecutive k of a row, scales [N, K/32];
 *   wbits 4, group_size 0,  scale_dtype F32: int4 codes in [-8,7], one fp32 scale per output
 *                                            channel (the paper's per-channel 4-bit scheme).
 * Any other combination returns QFC_ERR_UNSUPPORTED.
 * compute_mode selects the M > 8 path: QFC_COMPUTE_INT8_ACT (per-channel weights, 8-bit or 4-bit:
 * the paper's "q8" and "8/4/4" schemes in its prefill stage; group scales cannot leave an integer
 * accumulator) or QFC_COMPUTE_FP16_DEQUANT (binary16 activations, weights dequantized on the
 * fly: every format); neither changes M <= 8, which keeps binary16 activations.
 * QFC_COMPUTE_INT8_ACT_DECODE (per-channel formats only) is the decode design of section 3.7
 * of the paper: for M <= 8 the kernel quantizes the activations itself (one scale per token
 * row, as qfc_quantize_activations does) and accumulates integers; for M > 8 it behaves like
 * QFC_COMPUTE_INT8_ACT with 8-bit weights and like QFC_COMPUTE_FP16_DEQUANT with 4-bit ones. */
typedef struct {
    int32_t N;
    int32_t K;
    int32_t wbits;
    int32_t group_size;
    int32_t scale_dtype;
    int32_t compute_mode;
    int32_t flags;        /* 0, or QFC_PACK_GATED_PAIRS */
} qfc_desc_t;

/* flags.  QFC_PACK_GATED_PAIRS: the layer produces the two branches of a gated feed-forward
 * block (logical rows [0, N/2) = gate, [N/2, N) = the other branch; N a multiple of 32) and is only
 * ever used with the merged element-wise operators of qfc_fusion_t.gated_output (operator fusion,
 * section 3.6 and its figure).  Its physical layout interleaves the row tiles of the two branches,
 * so that every kernel, prefill included, holds both branches of a channel in one place and
 * multiplies them in its epilogue.  The logical interface (wq_logical, scales, unpack) is
 * unchanged.  Calls without gated_output on such a handle return QFC_ERR_UNSUPPORTED. */
enum { QFC_PACK_GATED_PAIRS = 1 };

/* Bytes of the physical (packed) form of a layer, padding included.
 * `desc` and `bytes` are host pointers. */
qfc_status_t qfc_packed_size(const qfc_desc_t *desc, size_t *bytes);

/* Weights conversion (section 3.4): rearrange the logical quantized weights
 * into the physical layout and create a handle.
 *   wq_logical  int8 [N, K], row-major, one code per byte (int4 codes in [-8, 7];
 *               only the low four bits of an int4 code are kept);
 *   scales      fp32 [N] or binary16 [N, K/32] as `desc` says;
 *   packed      caller-owned destination of at least qfc_packed_size bytes, borrowed
 *               by the handle afterwards;
 *   out         host pointer receiving the handle.
 * The inputs may be freed once the stream has run the conversion. */
qfc_status_t qfc_pack_weights(const qfc_desc_t *desc, const int8_t *wq_logical,
                              const void *scales, void *packed, size_t packed_bytes,
                              void *stream, qfc_handle_t *out);

/* Inverse of the conversion (test aid): writes back the logical codes and
 * scales, bit for bit what qfc_pack_weights was given. */
qfc_status_t qfc_unpack_weights(qfc_handle_t h, int8_t *wq_logical, void *scales, void *stream);

/* Scratch a forward call with up to M token rows needs (the tiled int8
 * activations and their scales of the int8 prefill path; at least 256 bytes).
 * `bytes` is a host pointer. */
qfc_status_t qfc_workspace_size(qfc_handle_t h, int32_t M, size_t *bytes);

/* Lend a workspace to the handle (host bookkeeping only: nothing is enqueued).
 * One workspace may be bound to many handles as long as their calls do not
 * overlap. */
qfc_status_t qfc_bind_workspace(qfc_handle_t h, void *workspace, size_t bytes);

/* Activation quantization kernel of the prefill stage (section 3.7): per token
 * row m, a = max|x[m,:]|, sx[m] = a/127 (fp32), xq[m,k] = clamp(rne(x[m,k] * (127/a)), +-127);
 * an all-zero row gives sx = 0, xq = 0.
 *   x_f16 binary16 [M, K] row-major; xq int8 [M, K] row-major; sx fp32 [M]. */
qfc_status_t qfc_quantize_activations(const void *x_f16, int32_t M, int32_t K,
                                      int8_t *xq, float *sx, void *stream);

/* y[M,N] = x[M,K] . dequant(W)^T, binary16 in, fp32 accumulation, binary16 out.
 * M <= 8: decode kernel (weights dequantized in registers).  M > 8: the path
 * `compute_mode` names; QFC_COMPUTE_INT8_ACT quantizes x per token into the
 * bound workspace first: that path needs a bound workspace of
 * qfc_workspace_size(h, M) bytes; the others use none. */
qfc_status_t qfc_forward(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16, void *stream);

/* Prefill product on already quantized activations (int8 per-channel weights
 * only): y[m,n] = fp16(float(sum_k xq[m,k] Wq[n,k]) * sx[m] * sw[n]).
 *   xq int8 [M, K] row-major, sx fp32 [M], y binary16 [M, N].  Any M >= 1. */
qfc_status_t qfc_forward_q8(qfc_handle_t h, const int8_t *xq, const float *sx, int32_t M,
                            void *y_f16, void *stream);

/* (qfc_forward_q8 with xq == NULL and sx == NULL, M > 8: the activations are those a preceding
 * qfc_rmsnorm with consumer == h and the same M left in h's workspace.) */

/* The raw int32 accumulators of the same product (parity aid): acc int32 [M, N]. */
qfc_status_t qfc_forward_acc_i32(qfc_handle_t h, const int8_t *xq, int32_t M, int32_t *acc,
                                 void *stream);

/* Element-wise operators fused with the fully connected operator (operator
 * fusion, section 3.6 and its figure: element-wise operators of two branches
 * merged into a fully connected operator; residual connections merged into the
 * neighbouring operator).  Both parts are optional (null pointer = absent):
 *   gate      binary16 [M, K]: the FC input is in = fp16(act(gate) * x), computed
 *             in fp32 and rounded once to binary16 (what an unfused element-wise
 *             operator would have stored); x is the other branch ("up").
 *             act: QFC_ACT_SILU  g / (1 + exp(-g))
 *                  QFC_ACT_GELU_TANH  0.5 g (1 + tanh(sqrt(2/pi) (g + 0.044715 g^3)))
 *   residual  binary16 [M, N]: added to the fp32 result before the one rounding
 *             to binary16: y = fp16(fc(in)[m,n] + residual[m,n]).  May alias y.
 *   gated_output  nonzero: the layer produces both branches, output channels
 *             [0, N/2) the gate and [N/2, N) the other one (N a multiple of 32), and
 *             y is binary16 [M, N/2]: y[m,n] = fp16(act(fc[m,n]) * fc[m,n + N/2]) with
 *             both fp32 results taken before any rounding.  Excludes the other two.
 *   norm_gamma  binary16 [K]: the RMS normalization that precedes the layer is merged into it.
 *             The layer's input is rmsnorm(x) * (norm_offset + gamma); since the normalization
 *             scales a row by one number rs = 1 / sqrt(mean_k x^2 + norm_eps), the kernel feeds
 *             in = fp16(x * (norm_offset + gamma)) to the product and multiplies the result by rs
 *             (fp32) before the residual is added.  Decode kernels only; excludes gate.
 * Supported: the decode kernels of QFC_COMPUTE_FP16_DEQUANT / QFC_COMPUTE_INT8_ACT
 * handles (M <= 8; all parts), the int8 prefill path (gate and residual: the gate is
 * applied by the activation quantization kernel) and the fp16 prefill path
 * (residual only: its activations go from memory to LDS without passing through
 * registers).  gated_output at M > 8 needs a handle packed with QFC_PACK_GATED_PAIRS
 * (both prefill paths; the fp16 path also needs K to be a multiple of 128); at M <= 8
 * it works with either packing.  Anything else returns QFC_ERR_UNSUPPORTED. */
#define QFC_ACT_SILU 0
#define QFC_ACT_GELU_TANH 1
typedef struct qfc_fusion {
    const void *gate;      /* device, binary16 [M, K], or null */
    int32_t activation;    /* QFC_ACT_*; read when gate or gated_output is given */
    const void *residual;  /* device, binary16 [M, N], or null */
    int32_t gated_output;  /* 0 or 1 */
    const void *norm_gamma; /* device, binary16 [K], or null */
    float norm_eps;         /* read when norm_gamma is given */
    float norm_offset;      /* 0: weight gamma; 1: weight 1 + gamma */
} qfc_fusion_t;

/* qfc_forward with the fused element-wise parts `f` names (host pointer, read
 * during the call; null or all parts absent = qfc_forward). */
qfc_status_t qfc_forward_fused(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16,
                               const qfc_fusion_t *f, void *stream);

/* qfc_forward for callers that cannot allocate or lend device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It
 * computes exactly what qfc_forward computes (same kernels, same bits) and ignores
 * the handle's bound workspace: the scratch of the int8 prefill path (the quantized
 * activations and their scales, qfc_workspace_size(h, M) bytes) lives in a device
 * array of QFC_STATIC_SCRATCH_BYTES that is part of the library's code object (each
 * GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing, on the host or the device; on its first use on a
 * device it looks up that device's copy of the array.
 *   - Calls whose scratch would not fit return QFC_ERR_SCRATCH_LIMIT before anything
 *     is enqueued (16 MiB holds M = 1024 token rows at K = 14336).  Decode calls and
 *     the fp16 prefill path use no scratch and have no such limit.
 *   - Every call on a GPU shares that GPU's array, which keeps the last call's
 *     contents; a call rewrites all of the region it reads, so nothing needs
 *     clearing, but calls that overlap in time on one GPU (two streams, two
 *     threads) race: order them.
 * x_f16, y_f16, M, stream: as qfc_forward. */
#define QFC_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
qfc_status_t qfc_forward_static(qfc_handle_t h, const void *x_f16, int32_t M, void *y_f16, void *stream);

/* RMS normalization with the residual connection and the quantization of the
 * next layer's input merged into one kernel (operator fusion, section 3.6 and
 * the right half of its figure).  Per token row, in fp32:
 *   h    = fp16(x + residual)          (h = x when residual is null)
 *   y[k] = fp16(h[k] * rs * (gamma_offset + gamma[k])),  rs = 1 / sqrt(mean_k h[k]^2 + eps)
 *   (xq, sx) = qfc_quantize_activations applied to y.
 * x, residual, h_out, y: binary16 [M, K]; gamma: binary16 [K]; xq int8 [M, K]; sx fp32 [M].
 * Each of h_out, y, (xq and sx together) is written when given; at least one must be.
 * h_out may be x or residual itself; y may be x when h_out is not x.  gamma_offset is 0
 * for a plain weight and 1 for models that store weight - 1.  K: a multiple of 32, at
 * most 14336 (a row is held in registers), else QFC_ERR_UNSUPPORTED.
 * consumer (or null): a handle whose M > 8 path multiplies int8 activations and whose K is this
 * K.  The codes and scales are then (also) written into that handle's bound workspace in the
 * physical order its product kernel reads, and qfc_forward_q8(consumer, NULL, NULL, M, y, stream)
 * runs the product on them without another pass over the activations (the normalization as the
 * producer of the next layer's quantized input).  xq and sx may be null when consumer is given.
 * The workspace must hold qfc_workspace_size(consumer, M) bytes, else QFC_ERR_BUFFER_TOO_SMALL. */
typedef struct qfc_rmsnorm {
    const void *x;        /* device */
    const void *residual; /* device or null */
    const void *gamma;    /* device */
    float eps;
    float gamma_offset;
    void *h_out;          /* device or null */
    void *y;              /* device or null */
    int8_t *xq;           /* device or null */
    float *sx;            /* device or null (with xq) */
    qfc_handle_t consumer; /* host handle or null */
} qfc_rmsnorm_t;
qfc_status_t qfc_rmsnorm(const qfc_rmsnorm_t *args, int32_t M, int32_t K, void *stream);

/* Attention-side operators of the decode stage.
 *
 * Shapes: `batch` sequences, `h_q` query heads and `h_kv` key/value heads of
 * `d_head` values (h_q a multiple of h_kv, g = h_q / h_kv; d_head 64, 128 or
 * 256), a KV cache of `cache_size` positions (a multiple of 64).  G = batch * h_kv.
 * Layouts (sections 3.6 and 3.8), all binary16:
 *   queries  q      [G, S * g, d_head]   row s * g + j = query head kv * g + j of token s
 *   K cache  kcache [G, cache_size, d_head]   (the transposed operand of Q K^T, stored as weights)
 *   V cache  vcache [G, cache_size / 64, d_head, 64]   (d_head x cache position, cut into blocks of
 *                   64 positions: element (d, p) of a group is at ((p / 64) * d_head + d) * 64 + p % 64)
 *   output   out    [G, S * g, d_head]   (for S = 1 this is [batch, h_q * d_head], the next layer's input)
 */
typedef struct qfc_attn_shape {
    int32_t batch, h_q, h_kv, d_head, cache_size;
} qfc_attn_shape_t;

/* Rotary embedding fused with the layout transformation of the query, key and
 * value projections (section 3.6): qkv_f16 is the QKV layer's output
 * [batch, S, (h_q + 2 h_kv) * d_head] (query heads, key heads, value heads) for
 * the tokens at positions pos0 .. pos0 + S - 1.  Queries and keys are rotated
 * (pairs (i, i + d_head / 2) by the angle pos * rope_base^(-2 i / d_head)); the
 * queries go to q_out, the keys are written into kcache as rows pos0 + s and
 * the values into vcache as columns pos0 + s.  pos0 + S <= cache_size. */
qfc_status_t qfc_rope_qkv(const void *qkv_f16, int32_t S, int32_t pos0, const qfc_attn_shape_t *shape,
                          float rope_base, void *q_out, void *kcache, void *vcache, void *stream);

/* The rotary angles of the first `positions` positions for this shape's head size, evaluated once
 * (in fp64, like qfc_rope_qkv): table (device, 8-byte aligned, positions * d_head / 2 * 2 floats) gets
 * table[(pos * d_head / 2 + i) * 2] = cos and [.. + 1] = sin of pos * rope_base^(-2 i / d_head).
 * Errors as qfc_rope_qkv; QFC_ERR_INVALID_ARG for positions < 1. */
qfc_status_t qfc_rope_table(const qfc_attn_shape_t *shape, float rope_base, int32_t positions, float *table,
                            void *stream);

/* Decode step of the QKV layer with the rotary embedding, the layout transformation and the cache
 * append merged into its kernel (operator fusion, section 3.6): for the shape's `batch` sequences
 * (= the layer's M token rows, at most 8), each at position pos0,
 *   qkv = x W^T (optionally rmsnorm(x) first: fusion->norm_gamma, norm_eps, norm_offset; the other
 *   members of fusion must be null / 0), never stored; queries and keys rotated on the fp32 sums
 *   with the table's cos and sin and rounded once to binary16; queries to q_out [G, g, d_head],
 *   keys to row pos0 of kcache, values to column pos0 of vcache (layouts above).
 * h: a QKV layer with N = (h_q + 2 h_kv) * d_head output channels (query heads, key heads, value
 * heads), any weight format, not packed in pairs.  rope_table: from qfc_rope_table with at least
 * pos0 + 1 positions (table_positions says how many it holds).  Same result as qfc_forward followed
 * by qfc_rope_qkv up to the rounding of the intermediate qkv, in one launch instead of two.
 * Errors: QFC_ERR_INVALID_ARG (null pointers, pos0 outside the cache or the table, N not matching
 * the shape, fusion members other than the normalization), QFC_ERR_ALIGNMENT (16 bytes; the table
 * 8), QFC_ERR_UNSUPPORTED (batch > 8, a layer packed in pairs or in the 8-bit-activation decode
 * mode, head sizes other than 64, 128, 256). */
qfc_status_t qfc_forward_qkv_rope(qfc_handle_t h, const void *x_f16, const qfc_fusion_t *fusion,
                                  const qfc_attn_shape_t *shape, int32_t pos0, const float *rope_table,
                                  int32_t table_positions, void *q_out, void *kcache, void *vcache, void *stream);

/* Bytes of scratch qfc_attention needs for this shape and S (host pointer). */
qfc_status_t qfc_attention_workspace_size(const qfc_attn_shape_t *shape, int32_t S, size_t *bytes);

/* Attention with the KV cache in the role of weights (section 3.8):
 * out = softmax(q K^T / sqrt(d_head)) V per group, over the first n_ctx cache
 * positions; the S query tokens are the last S of them (token s sees positions
 * 0 .. n_ctx - S + s).  Up to 16 query rows per KV head (S * g <= 16, decode) the
 * context is split over workgroups; with more (prefill) a wavefront owns 32 query rows
 * and walks the positions they see (launches with fewer blocks of 128 query rows than
 * compute units may cut those walks into chunks whose partial results, kept in the
 * workspace, a second kernel combines).  Positions >= n_ctx of the caches are never used,
 * whatever they hold.  The scores are not materialized.
 * workspace: device scratch of at least qfc_attention_workspace_size bytes, 16-byte aligned. */
qfc_status_t qfc_attention(const void *q, const void *kcache, const void *vcache, int32_t S, int32_t n_ctx,
                           const qfc_attn_shape_t *shape, void *workspace, size_t workspace_bytes,
                           void *out_f16, void *stream);

/* Embedding lookup from a packed layer (section 4.2: the schemes quantize the
 * embedding table like the layers, and models tie it to the LM head, so the
 * table is the LM head's handle): y[m, k] = fp16(s * Wq[ids[m], k]) with the
 * row's channel scale or the group scales, the product taken in fp32.
 * ids: device, int32 [M]; an id outside [0, N) gives a row of zeros.
 * y_f16: device, binary16 [M, K], 16-byte aligned.  M <= 65535. */
qfc_status_t qfc_embedding(qfc_handle_t h, const int32_t *ids, int32_t M, void *y_f16, void *stream);

/* `count` forward calls issued in order on one stream: handles, xs and ys are
 * host arrays of `count` entries; every call uses the same M.  Stops at the
 * first error and returns it. */
qfc_status_t qfc_forward_batch(const qfc_handle_t *handles, const void *const *xs, int32_t M,
                               void *const *ys, int32_t count, void *stream);

/* Free the host object.  Device buffers stay with the caller. */
qfc_status_t qfc_destroy(qfc_handle_t h);

/* Static, host string for a status code. */
const char *qfc_status_string(qfc_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* QFC_H */
