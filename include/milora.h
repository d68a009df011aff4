/*
 * milora.h - C ABI of the MI355X routed-LoRA linear layers (MiLoRA inference hot path).
 *
 * The library implements, as HIP kernels for gfx950, the part of MiLoRA that runs for every
 * request: the prompt-aware router evaluated once per Transformer layer at prefill
 * (Sec. 3.3, Eq. 2 and Eq. 3) and the seven LoRA-carrying linears of a LLaMA-2 layer
 * (Sec. 3.1, Eq. 1), where the low-rank term is added only for the requests whose cached
 * route selected that linear, with the LoRA matrices gathered from the request's tenant.
 *
 * General rules
 *  - Every pointer marked "device" is memory of the current HIP device, owned by the caller and
 *    never freed, resized or retained by the library beyond the work it enqueues.  Pointers
 *    marked "host" are ordinary host memory read during the call only.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *    and the call returns without synchronising.  Buffers must stay valid until that work is done.
 *  - The library allocates nothing.  Calls that need scratch memory take a device `workspace`
 *    of at least the size the matching *_workspace_bytes() function returns.  A workspace must be
 *    zero-filled once before its first use: the decode kernels keep their cross-workgroup
 *    hand-over flags in it, as values that only grow from launch to launch, so nothing has to be
 *    cleared between calls; apart from that its contents are undefined.  After a call that
 *    returned an error, or when the same memory is to serve another entry point or other sizes,
 *    zero it again.  Two calls that share a workspace must be ordered on one stream.
 *  - Return value: MILORA_OK (0) or a negative milora_status.  Arguments are validated on the
 *    host before anything is enqueued; values that live in device arrays (tenant ids, routes,
 *    prompt spans) are checked by the kernels, which then skip the offending request as
 *    documented per call and never read or write out of bounds because of it.
 *  - Matrix conventions follow the paper: row vectors, x' = x W + x W^A W^B + b with
 *    W in R^{d1 x d2}, W^A in R^{d1 x r}, W^B in R^{r x d2} (Eq. 1).
 *  - Sites (the paper's N_mod = 7 modules, Sec. 3.1): 0 q, 1 k, 2 v, 3 o, 4 gate, 5 up, 6 down.
 *    For a layer with hidden size d and FFN width F, (d1, d2) is (d, d) for q, k, v, o,
 *    (d, F) for gate and up, (F, d) for down.
 */
#ifndef MILORA_H
#define MILORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MILORA_NUM_SITES 7
#define MILORA_MAX_RANK 256       /* largest LoRA rank accepted (the paper sweeps r up to 256, Sec. 4.5) */
#define MILORA_MAX_DECODE_BATCH 128 /* largest B accepted by milora_layer_decode */
#define MILORA_ROUTE_NONE 255     /* route value written for a request the router had to skip */
/* A route byte names the sites whose LoRA term a request uses: 0..6 = that one site (top-1: what the
 * paper's parameter counts fix, Sec. 4.3); MILORA_ROUTE_SET | mask with bit m of the 7-bit mask set for
 * every chosen site m (top-k with 1 < k < 7; the chosen sites' terms are added without weights: the
 * gate of Eq. 3 is not connected to Eq. 1 in the paper); MILORA_ROUTE_NONE = no LoRA term. */
#define MILORA_ROUTE_SET 0x80
#define MILORA_NOALLOC_SCRATCH_BYTES (8u << 20) /* scratch milora_layer_decode_noalloc holds on every GPU it runs on */

typedef enum {
  MILORA_OK = 0,
  MILORA_EINVAL = -1,       /* null pointer, non-positive size, unknown enum value */
  MILORA_ERANGE = -2,       /* a size beyond a documented limit */
  MILORA_EUNSUPPORTED = -3, /* a combination the kernels do not cover (stated per call) */
  MILORA_EHIP = -4,         /* a HIP call failed; see milora_last_hip_error() */
  MILORA_EWORKSPACE = -5    /* workspace missing or smaller than *_workspace_bytes() */
} milora_status;

typedef enum { MILORA_BF16 = 0, MILORA_F32 = 1 } milora_dtype;
/* Poolers of Sec. 3.3: average, last token, max, self-attention (App. C). */
typedef enum { MILORA_POOL_MEAN = 0, MILORA_POOL_LAST = 1, MILORA_POOL_MAX = 2, MILORA_POOL_SELFATTN = 3 } milora_pool;
/* Router activation g: fixed functions, or the rational form of Sec. 3.4 with the caller's coefficients. */
typedef enum {
  MILORA_ACT_IDENTITY = 0, MILORA_ACT_TANH = 1, MILORA_ACT_RELU = 2, MILORA_ACT_GELU = 3, MILORA_ACT_RATIONAL = 4
} milora_act;

/* Storage of a base weight W (math shape d1 x d2).
 *  MILORA_W_ROWMAJOR : [d2][d1], d1 contiguous (the usual linear-layer storage).
 *  MILORA_W_PACKED   : the order milora_pack_weight() produces (bf16 only, d1 % 32 == 0 and
 *                      d2 % 16 == 0): blocks of 16 output columns x 32 inputs, each block 1 KiB laid
 *                      out lane-by-lane as the 16x16x32 matrix-core operand, blocks of one column
 *                      group consecutive along d1.  Element (j, i) of the row-major array sits at
 *                      ((j/16 * (d1/32) + i/32) * 64 + (i%32)/8 * 16 + j%16) * 8 + i%8.  */
typedef enum { MILORA_W_ROWMAJOR = 0, MILORA_W_PACKED = 1 } milora_wlayout;

/* Flags of milora_layer_decode. */
#define MILORA_LAYER_RMSNORM 1u /* weightless RMS normalisation (eps 1e-5) in front of q/k/v and gate/up */

/* Per-tenant LoRA stacks of ONE layer (host struct; the arrays it points to are device memory).
 * Tenant t owns, for each site m, W^A stored [d1][r_t] row-major and W^B stored [r_t][d2]
 * row-major, exactly as Eq. 1 writes them, in the same dtype as the base weights.  The rank r_t is
 * per tenant and the same at all seven sites.  Matrices may live anywhere; the kernels use 16-byte
 * loads when a matrix is 16-byte aligned and r_t is a multiple of 8 (bf16) or 4 (fp32), scalar
 * loads otherwise. */
typedef struct {
  int32_t n_tenants;      /* T */
  int32_t r_max;          /* an upper bound of rank[t] over all tenants, 1..MILORA_MAX_RANK */
  const int32_t *rank;    /* device [T]: r_t; a tenant with r_t outside 1..r_max gets no LoRA term */
  const void *const *A;   /* device [T*7] of device pointers, entry t*7+m -> W^A of (tenant t, site m) */
  const void *const *B;   /* device [T*7] of device pointers, entry t*7+m -> W^B of (tenant t, site m) */
} milora_adapters;

/* The seven base weights of one layer (host struct of device pointers), all in `layout`. */
typedef struct {
  const void *W[MILORA_NUM_SITES]; /* W[m]: math shape d1 x d2 of site m */
  int32_t layout;                  /* milora_wlayout */
} milora_layer_weights;

const char *milora_version(void);
const char *milora_status_string(int status);
/* The hipError_t (as int) of the most recent failed HIP call made by this thread, 0 if none. */
int milora_last_hip_error(void);

/* ------------------------------------------------------------------------------------------------
 * milora_route - the prompt-aware LoRA router of one layer (Sec. 3.3):
 *   h_b = Pooler(H^l restricted to request b's prompt tokens)        (Eq. 2; last-token / average / max /
 *                                                                     self-attention: softmax_t(H w_sa)^T H, App. C)
 *   route[b] = the top_k largest of ( g(h_b) W_r^{l, tenant(b)} )_j   (Eq. 3; top_k = 1: argmax)
 * Softmax is increasing, so the experts are taken on the logits; equal logits resolve to the
 * lowest index.  Pooled state, activation and logits are kept in fp32 whatever `dtype` is.
 * Runs once per layer per prompt; decode never calls it (the decisions are reused, Sec. 3.3).
 *
 *   H          device [M_tok][d], `dtype`: hidden states entering the layer, prompts in any packing
 *   seq_start  device [B] int32: first row of request b's prompt in H
 *   seq_len    device [B] int32: number of prompt tokens (valid rows) of request b, >= 1
 *   tenant_id  device [B] int32 in [0, T)
 *   Wr         device [T][7][d], `dtype`: column j of tenant t's d x 7 router matrix is the
 *              contiguous d-vector Wr[t][j]; no bias
 *   w_sa       device [T][d], `dtype`: the self-attention pooler's query vector of each tenant for this layer;
 *              read for MILORA_POOL_SELFATTN only, NULL otherwise.  d <= 8192 for this pooler.
 *   act_coef   HOST [12] float: a_0..a_6, b_1..b_5 of Ra(x) = (sum_j a_j x^j) / (1 + |sum_i b_i x^i|)
 *              (Sec. 3.4; one set per call, i.e. per layer); read for MILORA_ACT_RATIONAL only, NULL otherwise
 *   top_k      1..6: experts per request; 1 writes the site index, more write MILORA_ROUTE_SET | mask
 *   route_out  device [B] uint8: route byte per request (row `l` of the caller's route table)
 *   logits_out device [B][7] float or NULL: the seven logits
 *   workspace  device, milora_route_workspace_bytes(B, d, M_tok) bytes, needed by every pooler; its contents
 *              before the call do not matter (the kernels mark what they hand over with a tag unique to the call
 *              and wipe the tags they have used, so a call recorded into a HIP graph can be replayed); two calls
 *              that run at the same time need a workspace each
 * A request whose span leaves [0, M_tok), whose length is < 1 or whose tenant id is out of range
 * gets route MILORA_ROUTE_NONE and NaN logits; the others are unaffected.
 * Errors: EINVAL (null pointers, B/d/T/M_tok < 1, bad enums, w_sa / act_coef missing where needed), ERANGE
 * (B > 65535; self-attention pooling with d > 8192), EWORKSPACE, EHIP.
 */
size_t milora_route_workspace_bytes(int B, int d, int64_t M_tok);
int milora_route(const void *H, int64_t M_tok, int d, int dtype, const int32_t *seq_start,
                 const int32_t *seq_len, const int32_t *tenant_id, int B, int n_tenants,
                 const void *Wr, int pool, int act, const void *w_sa, const float *act_coef,
                 int top_k, uint8_t *route_out, float *logits_out, void *workspace,
                 size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * milora_routed_linear - one LoRA-carrying linear for M rows (Eq. 1 with the layer-level gate of
 * Sec. 3.3: a request's LoRA term is present only at the site its route selected):
 *   b = row_to_req ? row_to_req[m] : m,  t = tenant_id[b]
 *   Y[m] = X[m] W + bias + [route[b] selects site] (X[m] W^A_{t,site}) W^B_{t,site}
 * Accumulation is fp32; the low-rank intermediate stays fp32 and is added to the fp32 base result
 * before the single rounding to `dtype`.
 *
 *   X           device [M][d1], `dtype`
 *   row_to_req  device [M] int32 or NULL.  NULL means row m belongs to request m and needs M == B
 *               (decode).  Prefill tokens and beams map several rows to one request.
 *   W           device, math shape d1 x d2 in `w_layout` (MILORA_W_PACKED: bf16 only)
 *   bias        device [d2] `dtype` or NULL
 *   adapters    host struct, see milora_adapters
 *   tenant_id   device [B] int32; route: device [B] uint8 (this layer's row of the route table)
 *   Y           device [M][d2], `dtype`
 *   workspace   device, milora_routed_linear_workspace_bytes(M, d1, d2, r_max) bytes
 * A row whose request index, tenant id or tenant rank is out of range gets the base term only.
 * Errors: EINVAL, ERANGE (r_max > MILORA_MAX_RANK), EUNSUPPORTED (packed layout with fp32, with
 * d1 % 32 != 0 or d2 % 16 != 0, or with X, W, bias or Y not 16-byte aligned), EWORKSPACE, EHIP.
 */
size_t milora_routed_linear_workspace_bytes(int64_t M, int d1, int d2, int r_max);
/* Which kernel milora_routed_linear runs for these sizes when its pointers are 16-byte aligned (host
 * logic only, no device work): MILORA_KERNEL_GENERIC (any shape, fp32 arithmetic), MILORA_KERNEL_STREAM
 * (packed weights, the few-row weight-streaming kernel, M above MILORA_MAX_DECODE_BATCH in slices) or
 * MILORA_KERNEL_TILES (row-major bf16 weights, M >= 64, d1 % 64 == 0, d2 % 16 == 0: 256 x 256 matrix-core
 * tiles).  Negative status for arguments milora_routed_linear itself would reject. */
#define MILORA_KERNEL_GENERIC 0
#define MILORA_KERNEL_STREAM 1
#define MILORA_KERNEL_TILES 2
int milora_routed_linear_kernel(int64_t M, int d1, int d2, int dtype, int w_layout);
int milora_routed_linear(const void *X, int64_t M, int d1, int d2, int dtype,
                         const int32_t *row_to_req, const void *W, int w_layout, const void *bias,
                         const milora_adapters *adapters, int site, const int32_t *tenant_id,
                         const uint8_t *route, int B, void *Y, void *workspace,
                         size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * milora_layer_decode - one decode step of B requests through the seven routed linears of a layer,
 * using the cached routes (Sec. 3.3: the routing decisions of the prompt are reused for every
 * generated token; nothing here reads prompts or router weights, and `route` is read-only).
 * The paper fixes the seven linears (Sec. 3.1, Fig. 1); the glue between them is the smallest that
 * chains them at their true shapes:
 *   q, k, v = L_q(n(x)), L_k(n(x)), L_v(n(x))
 *   a       = attn_out if given, else v   (what causal attention returns for a context of one token)
 *   h       = x + L_o(a)
 *   m       = silu(L_gate(n(h))) * L_up(n(h))
 *   y       = h + L_down(m)
 * where L_m is milora_routed_linear at site m without bias and n() is the identity, or
 * u / sqrt(mean(u^2) + 1e-5) when MILORA_LAYER_RMSNORM is set.  Intermediates that feed a matrix
 * product are rounded to `dtype`; the residual stream h is carried in fp32.
 *
 *   x         device [B][d] `dtype`;  y: device [B][d] `dtype` (may alias x)
 *   weights   host struct of the seven base weights
 *   attn_out  device [B][d] `dtype` or NULL
 *   qkv_out   device [B][3d] `dtype` or NULL: q | k | v of every request, for the caller's attention
 *   workspace device, milora_layer_decode_workspace_bytes(B, d, F, r_max) bytes (packed weights and B > 32:
 *             this includes the tables of fp32 partial tiles of the wide-batch kernel, tens of MB)
 * Errors: EINVAL, ERANGE (B > MILORA_MAX_DECODE_BATCH, r_max > MILORA_MAX_RANK), EUNSUPPORTED
 * (packed layout with fp32, with d or F not a multiple of 32, or with x, y, attn_out, qkv_out or a
 * weight not 16-byte aligned), EWORKSPACE, EHIP.
 */
size_t milora_layer_decode_workspace_bytes(int B, int d, int F, int r_max);
int milora_layer_decode(const void *x, int B, int d, int F, int dtype,
                        const milora_layer_weights *weights, const milora_adapters *adapters,
                        const int32_t *tenant_id, const uint8_t *route, uint32_t flags,
                        const void *attn_out, void *y, void *qkv_out, void *workspace,
                        size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * milora_layer_decode_noalloc - milora_layer_decode for callers that can neither allocate device memory nor
 * hand over a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and glue as milora_layer_decode without `workspace`; the scratch memory is an array
 * of MILORA_NOALLOC_SCRATCH_BYTES inside the library's code object, which every GPU the entry point runs on
 * holds from the library's first use there until the process ends.  The call allocates and frees nothing and
 * enqueues a small fill kernel (the control words of the scratch start from zero in every call) and the decode
 * launch on `stream`.
 * Limits: packed bf16 weights only (anything else: EUNSUPPORTED, with the alignment rules of
 * milora_layer_decode); B <= 32, and d, F, r_max such that the packed path's scratch fits the array - every
 * LLaMA-2 shape up to d = 8192, F = 28672 with r_max <= 64, and the 7B and 13B shapes with any accepted rank
 * (beyond: ERANGE).
 * All calls on one GPU share that GPU's array: they must be ordered on one stream (or otherwise not overlap),
 * calls that overlap race.  milora_packed_workspace_status(NULL, ...) reads the array's status word, which tells
 * about the most recent call only.
 * Errors: EINVAL, ERANGE, EUNSUPPORTED, EHIP.
 */
int milora_layer_decode_noalloc(const void *x, int B, int d, int F, int dtype,
                                const milora_layer_weights *weights, const milora_adapters *adapters,
                                const int32_t *tenant_id, const uint8_t *route, uint32_t flags,
                                const void *attn_out, void *y, void *qkv_out, void *stream);

/* ------------------------------------------------------------------------------------------------
 * milora_packed_workspace_status - the packed-weight kernels (milora_layer_decode and milora_routed_linear
 * with MILORA_W_PACKED) run as ONE launch of one workgroup per compute unit whose workgroups hand data to each
 * other inside the launch (the four dependent levels of a layer step) and wait for it with bounded polls.
 * That needs all workgroups of the launch resident at the same time: a packed-path launch must not overlap
 * other GPU work of the process (another stream's kernels, a second packed-path launch on another workspace)
 * that holds compute units.  When it does, or after a fault elsewhere, a wait runs out after
 * milora_set_wait_limit() polls (seconds with the default): the wave that waited sets a word in the workspace
 * to 1 and ends, the waves that depend on it run out the same way, and the launch finishes with wrong or
 * missing results instead of hanging.  This call waits for the work queued on `stream`, then copies that word
 * to *status (host): 0 = every wait ended normally since the workspace was zero-filled.  After a 1 the
 * workspace must be zero-filled again before its next use.  workspace == NULL: the word of the scratch array
 * of milora_layer_decode_noalloc on the current GPU.
 * Errors: EINVAL, EHIP.
 */
int milora_packed_workspace_status(const void *workspace, int *status, void *stream);
/* Polls after which a bounded wait of the packed-weight kernels gives up, for the launches enqueued after this
 * call by any thread; polls <= 0 restores the default (2^22, a few seconds).  Returns the previous value.  A
 * service that prefers a fast failure to a long wait lowers it; a value of a few polls makes every wait that
 * is not satisfied at once run out, which is how the error path is tested. */
int milora_set_wait_limit(int polls);

/* ------------------------------------------------------------------------------------------------
 * milora_layer_decode_profile - measurement aid, not part of the method: runs milora_layer_decode
 * `reps` times on `stream` with a HIP event recorded on that stream after every internal kernel
 * launch, synchronises, and returns the average duration in milliseconds of each launch in
 * slot_ms (host, MILORA_PROFILE_SLOTS floats; slots the path does not use stay 0).  Packed layout:
 * the whole decode step is one launch that walks q,k,v | o | gate,up | down, timed in slot 0.
 * Other layouts: EUNSUPPORTED.  Same arguments and errors as
 * milora_layer_decode otherwise; creates and destroys HIP events, allocates no device memory.
 */
#define MILORA_PROFILE_SLOTS 8
int milora_layer_decode_profile(const void *x, int B, int d, int F, int dtype,
                                const milora_layer_weights *weights, const milora_adapters *adapters,
                                const int32_t *tenant_id, const uint8_t *route, uint32_t flags,
                                const void *attn_out, void *y, void *qkv_out, void *workspace,
                                size_t workspace_bytes, void *stream, int reps, float *slot_ms);

/* ------------------------------------------------------------------------------------------------
 * milora_layer_decode_trace - measurement aid, not part of the method: one milora_layer_decode (packed weights
 * only) on an instantiation of the decode kernel in which every wave writes time stamps (the GPU's 100 MHz
 * constant clock) at the boundaries of its phases in every stage, then a synchronisation.  Same arguments, results
 * and errors as milora_layer_decode, plus:
 *   stamps        device, milora_layer_decode_trace_bytes() bytes: int64 [workgroup][dims[2]][dims[3]][dims[4]],
 *                 zero where a wave has no such phase; cleared by the call
 *   dims          HOST int32 [5]: workgroups and stages of the launch, then the three array extents above
 * Stamp slots, few-row kernel (waves 0..5 stream, 6 loader, 7 LoRA): stream 0 stage entered, 1 first input chunk
 * there, 2 matrix work done, 3 partial tiles summed; loader 0 entered, 1 grid barrier passed, 2 first chunk landed,
 * 3 all landed, 8 partial tiles swapped with the partner (o and down stages), 4 sums complete with LoRA terms,
 * 5 own outputs stored; LoRA 0 entered, 1 barrier passed, 2 shrink items done, 3 shrinks of own rows published,
 * 4 expands formed, 5 stream waves' sums there, 6 own outputs stored, 7 hand-over flag stored.  Many-row kernel: all 0
 * level entered, 4 sums begun, 5 own sums stored; stream 1 first chunk there, 2 segments stored; loader 1 barrier
 * passed, 2 copies landed, 6 shrink items done, 3 expand items done; LoRA 1 barrier passed, 2 shrink list built,
 * 8 first shrink item begun, 9 its partial flagged, 6 shrink items done, 3 expand items done.
 * Errors: those of milora_layer_decode; EUNSUPPORTED for other layouts; EWORKSPACE for a short `stamps`.
 */
size_t milora_layer_decode_trace_bytes(void);
int milora_layer_decode_trace(const void *x, int B, int d, int F, int dtype,
                              const milora_layer_weights *weights, const milora_adapters *adapters,
                              const int32_t *tenant_id, const uint8_t *route, uint32_t flags,
                              const void *attn_out, void *y, void *qkv_out, void *workspace,
                              size_t workspace_bytes, void *stream, void *stamps, size_t stamps_bytes,
                              int32_t *dims);

/* ------------------------------------------------------------------------------------------------
 * milora_pack_weight - one-time re-ordering of a bf16 base weight from MILORA_W_ROWMAJOR to
 * MILORA_W_PACKED (see milora_wlayout), so that the decode kernels stream it with fully
 * coalesced 1 KiB loads already in matrix-core operand order.  src and dst: device, d1*d2
 * elements each, must not overlap.  Errors: EINVAL, EUNSUPPORTED (d1 % 32 or d2 % 16 nonzero), EHIP.
 */
int milora_pack_weight(const void *src_rowmajor, void *dst_packed, int d1, int d2, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Measurement helpers (not part of the method; for callers that report a kernel's rate against what the
 * GPU sustains rather than against a data-sheet figure).  Both block until their kernels have finished.
 *   milora_measure_matrix_rate: per wave 2 x 32 x iters v_mfma_f32_16x16x32_bf16 (shape 0) or 4 x 8 x iters
 *     v_mfma_f32_32x32x16_bf16 (shape 1: the same flops in half the instructions and operand reads) on
 *     independent accumulators, four waves per compute unit, nothing else -> *tflops (host pointer).  Operands are
 *     small integers; shape + 2 takes operands spread over [-1, 1) with every mantissa bit in use (what weights
 *     and activations look like: the matrix cores draw more power for them and the clock gives way).
 *   milora_measure_read_rate: reads `bytes` (device, 16-byte aligned; use a buffer much larger than the
 *     caches) `reps` times with 16-byte loads -> *gbs (host pointer).
 *   workspace: device, milora_measure_workspace_bytes() bytes.
 * Errors: EINVAL, EWORKSPACE, EHIP.
 */
size_t milora_measure_workspace_bytes(void);
int milora_measure_matrix_rate(int shape, int iters, void *workspace, size_t workspace_bytes,
                             double *tflops, void *stream);
int milora_measure_read_rate(const void *buf, size_t bytes, int reps, void *workspace,
                            size_t workspace_bytes, double *gbs, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MILORA_H */
