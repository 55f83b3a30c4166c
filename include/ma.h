/*
 * ma.h -- C ABI of the MI355X optimizer-step library (libma_step.so).
 *
 * The library runs, on one GPU, the per-sub-group optimizer step that an SSD-offloaded
 * mixed-precision fine-tuning system executes once per iteration over its flat partitioned
 * buffers (MemAscend, arXiv 2505.23254):
 *
 *   1. ma_overflow_norm      one pass over the gradient: overflow flag (any +inf, -inf or NaN;
 *                            Sec. III-C, Sec. IV-D / Algorithm 1) fused with the sum of squares
 *                            needed for global-norm clipping;
 *   2. the gate              on overflow the step is skipped and every state stays bit-unchanged
 *                            (Sec. III-C: the caller then lowers the loss scale); otherwise the
 *                            clip coefficient follows from the norm;
 *   3. ma_adamw_step         unscale + clip + AdamW with bias correction and decoupled weight
 *                            decay on fp32 master p / m / v (Sec. II-A), and the low-precision
 *                            copy of the new parameter written in the same pass (Sec. III-D lists
 *                            the low-precision compute weights kept beside the fp32 masters).
 *
 * Conventions that hold for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, unless the name ends in _host.
 *     The library never allocates, frees or keeps device memory (the placement helper ma_arena_*
 *     at the end of this header is the one exception: allocating is what it is for).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; results are valid once the stream has been synchronised.  No entry point
 *     synchronises the device, except ma_multi_prepare (documented there).
 *   - Return value: MA_OK (0) or a negative ma_status.  Argument errors (MA_ERR_NULL, _DTYPE,
 *     _ALIGN, _ARG) are found before anything is launched: no buffer has been written.  After
 *     MA_ERR_HIP (the runtime refused a launch or a copy) part of the call's work may already be
 *     enqueued, and the contents of the buffers the call writes are unspecified.
 *     ma_last_error() returns a thread-local message.
 *   - n is a size_t element count; sub-groups beyond 2^31 elements are supported.
 *   - Buffers must not overlap each other: the update and accumulation calls and ma_multi_prepare
 *     check the byte ranges they are given and return MA_ERR_ARG when two of them share a byte.
 *     Pointers must be aligned to their element size; 16-byte alignment of every buffer enables the
 *     128-bit path, anything else is handled by a scalar path with the same results.
 *   - The entry points may be called from several host threads.  Work on different streams may
 *     overlap in time as long as the calls share no buffer, workspace or plan (see
 *     ma_multi_table_bytes).
 */
#ifndef MA_STEP_H_
#define MA_STEP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ma_dtype {
  MA_F32 = 0,  /* IEEE binary32 */
  MA_BF16 = 1, /* upper 16 bits of binary32 */
  MA_F16 = 2   /* IEEE binary16 */
} ma_dtype;

typedef enum ma_status {
  MA_OK = 0,
  MA_ERR_NULL = -1,  /* a required pointer is NULL */
  MA_ERR_DTYPE = -2, /* dtype not supported in this position */
  MA_ERR_ALIGN = -3, /* pointer not aligned to its element size */
  MA_ERR_ARG = -4,   /* value out of range (see each call) or workspace too small */
  MA_ERR_HIP = -5,   /* the HIP runtime reported an error; text in ma_last_error() */
  MA_ERR_FULL = -6   /* ma_pool_acquire: every buffer of the sub-pool is in use */
} ma_status;

/* Result of the gradient scan, 16 bytes, lives in device memory. */
typedef struct ma_norm_result {
  int32_t overflow; /* 1 if any element is +inf, -inf or NaN, else 0 */
  int32_t reserved; /* written as 0 */
  double sumsq;     /* sum over i of (g_i / loss_scale)^2; unspecified when overflow == 1 */
} ma_norm_result;

/* AdamW hyper-parameters (Sec. II-A: bias correction, decoupled weight decay). */
typedef struct ma_hyper {
  float lr;                /* >= 0 */
  float beta1;             /* in [0, 1) */
  float beta2;             /* in [0, 1) */
  float eps;               /* > 0 */
  float weight_decay;      /* >= 0; multiplies lr (decoupled decay) */
  int32_t bias_correction; /* non-zero: divide by 1 - beta^step */
} ma_hyper;

/* One tensor of a multi-tensor step.  All five buffers hold n elements. */
typedef struct ma_tensor {
  float* p32;       /* fp32 master parameter, updated in place */
  float* m;         /* fp32 first moment, updated in place */
  float* v;         /* fp32 second moment, updated in place */
  const void* grad; /* gradient in the list's gradient dtype, read only */
  void* p_lp;       /* low-precision parameter copy, written */
  size_t n;
} ma_tensor;

/* One tensor of a multi-tensor step with p, m, v held in bf16 (see ma_adamw_step_bf16). */
typedef struct ma_tensor_bf16 {
  void* p;          /* bf16 parameter, updated in place (it is its own low-precision copy) */
  void* m;          /* bf16 first moment, updated in place */
  void* v;          /* bf16 second moment, updated in place */
  const void* grad; /* gradient in the list's gradient dtype, read only */
  size_t n;
} ma_tensor_bf16;

/* Host-side handle of a prepared tensor list (plain data, caller-owned, copyable). */
typedef struct ma_multi_plan {
  const void* table_dev; /* device table written by ma_multi_prepare */
  uint64_t entries;      /* table rows (one per non-empty tensor) */
  uint64_t total_elems;
  uint64_t norm_chunks;  /* work items of the scan kernel */
  uint64_t step_chunks;  /* work items of the update kernel */
  int32_t gdt;
  int32_t pdt;
  uint32_t magic;
  uint32_t sdt;          /* dtype of p, m, v: MA_F32, or MA_BF16 for a list from ma_multi_prepare_bf16 */
} ma_multi_plan;

/* Dynamic loss-scale state, 24 bytes, lives in device memory (Sec. III-C: when a value overflows,
 * the scale factor is reduced and the step skipped).  Written by ma_scaler_init / ma_scaler_update,
 * read on the device by the *_auto entry points. */
typedef struct ma_scaler_state {
  float scale;        /* current loss scale */
  int32_t good_steps; /* clean steps since the scale last changed */
  int64_t step;       /* updates applied so far; the next update is number step + 1 */
  int64_t skipped;    /* iterations skipped because of an overflow */
} ma_scaler_state;

/* Policy of the dynamic loss scale (host struct). */
typedef struct ma_scaler_config {
  float backoff;   /* in (0, 1): factor applied on overflow (0.5: halve) */
  float growth;    /* >= 1: factor applied after `window` clean steps in a row */
  float min_scale; /* > 0 */
  float max_scale; /* >= min_scale, finite */
  int32_t window;  /* >= 1 */
} ma_scaler_config;

/* ---- housekeeping ---------------------------------------------------------------------- */

/* Library version, major*10000 + minor*100 + patch. */
int ma_version(void);

/* Message of the last failing call on this thread ("" if none).  Static storage. */
const char* ma_last_error(void);

/* Bytes of device workspace ma_overflow_norm / ma_multi_overflow_norm need (per-block partial
 * results of the two-level reduction).  Independent of n.  The workspace may be reused by later calls on the same stream; calls on
 * different streams need different workspaces. */
size_t ma_workspace_bytes(void);

/* Host helper: the clip coefficient of global-norm clipping,
 *   c = min(1, max_norm / (sqrt(sumsq) + 1e-6)),  evaluated in fp64, rounded once to fp32;
 * max_norm <= 0 disables clipping (c = 1). */
float ma_clip_coef(double sumsq, float max_norm);

/* Host helper: the nine fp32 scalars one AdamW step uses, in the order
 *   {beta1, beta2, 1-beta1, 1-beta2, eps, lr/(1-beta1^step), 1/sqrt(1-beta2^step), lr*wd,
 *    clip_coef/loss_scale},
 * each evaluated in fp64 from the fp32 arguments and rounded once (the update kernels receive
 * exactly these).  beta^step is an integer power by squaring carried in double-double arithmetic
 * and rounded once to fp64 (the correctly rounded power, up to near-ties beyond 2^-95).  Same argument checks as ma_adamw_step. */
int ma_step_scalars(const ma_hyper* hyper, int64_t step, float loss_scale, float clip_coef,
                    float out_host[9]);

/* Host helper: how the library splits one tensor into work items, from its pointers alone
 * (nothing is dereferenced).  norm_items / step_items: work items of the scan / update kernel;
 * norm_head: elements before the gradient's first 16-byte boundary (scalar path);
 * step_head: elements before the first 4-element group common to all buffers;
 * step_vec: 1 if the 128-bit update path applies after step_head elements, 0 if the buffers'
 * alignments disagree and the scalar path is used.  Any out pointer may be NULL. */
int ma_plan_tensor(const ma_tensor* tensor_host, ma_dtype gdt, uint64_t* norm_items,
                   uint64_t* step_items, uint32_t* norm_head, uint32_t* step_head,
                   uint32_t* step_vec);

/* ---- step 1: overflow scan fused with the sum of squares ---------------------------------- */

/* Scans grad[0..n) (dtype gdt: MA_BF16, MA_F16 or MA_F32) once.
 *   out_dev->overflow  Algorithm 1 (Sec. IV-D): 1 iff some element has an all-ones exponent
 *                      (+inf, -inf, NaN), tested on the raw stored pattern.  No early exit: the
 *                      same pass also needs the full sum.
 *   out_dev->sumsq     sum of (g_i / loss_scale)^2, accumulated in fp64 with a fixed reduction
 *                      order (bit-identical from run to run on the same device).
 * loss_scale must be finite and > 0.  n == 0 writes {0, 0.0}.
 * ws: device workspace of at least ma_workspace_bytes(). */
int ma_overflow_norm(const void* grad, ma_dtype gdt, size_t n, float loss_scale,
                     ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream);

/* ma_overflow_norm for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  The caller brings no workspace; the
 * per-block partial results go to an array of MA_STATIC_SCRATCH_BYTES bytes that the library keeps
 * in its own device image, one copy per GPU, from the first call on that GPU until the process
 * ends.  The call allocates and frees nothing (its first call on a device looks up the array's
 * address, nothing more).  Same kernels, same reduction order and so the same bits in *out_dev as
 * ma_overflow_norm with a caller workspace.
 *   - n > MA_STATIC_SCAN_MAX_ELEMS is rejected with MA_ERR_ARG before anything is launched (the
 *     scan grid, and with it the scratch, is bounded by the device and not by n; the limit is far
 *     above what the memory of one GPU can hold).
 *   - Every call on one GPU uses that GPU's one array.  Nothing in it has to start at zero (each
 *     launch overwrites the slots it later reads), so calls in sequence on one stream need no
 *     clearing; calls that overlap in time on one GPU (two streams, two threads) race on it and
 *     give wrong results.  Use ma_overflow_norm with one workspace per stream for those. */
#define MA_STATIC_SCRATCH_BYTES (8192u * 16u)
#define MA_STATIC_SCAN_MAX_ELEMS ((size_t)1 << 38)
int ma_overflow_norm_static(const void* grad, ma_dtype gdt, size_t n, float loss_scale,
                            ma_norm_result* out_dev, void* stream);

/* Adds up `count` scan results (e.g. one per sub-group streamed through the optimizer-state
 * buffer, Sec. IV-C) in index order: overflow = OR, sumsq = fp64 sum.  out_dev may be one of
 * the inputs' neighbours but not an element of parts_dev.  count >= 1. */
int ma_norm_combine(const ma_norm_result* parts_dev, size_t count, ma_norm_result* out_dev,
                    void* stream);

/* ---- step 3: unscale + clip + AdamW + low-precision copy -------------------------------------- */

/* One AdamW step (1-based `step`) over a flat sub-group of n elements, in fp32:
 *     g    = widen(grad_i) * fl32(clip_coef / loss_scale)
 *     m'   = beta1*m + (1-beta1)*g
 *     v'   = beta2*v + (1-beta2)*g*g
 *     p'   = (p - lr*wd*p) - (lr / (1-beta1^step)) * m' / (sqrt(v') / sqrt(1-beta2^step) + eps)
 *     p_lp = round-to-nearest-even(p') in dtype pdt (MA_BF16 or MA_F16)
 * p32, m, v are updated in place; p_lp is written; grad (MA_BF16, MA_F16 or MA_F32) is read.
 * p_lp may be NULL (no low-precision copy is written; pdt is ignored).
 * Requirements: step >= 1, loss_scale finite > 0, 0 < clip_coef <= 1, hyper ranges as in
 * ma_hyper.  This entry point does not look at the overflow flag: the caller gates. */
int ma_adamw_step(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                  ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step, float loss_scale,
                  float clip_coef, void* stream);

/* The same step with the gate of Sec. III-C taken on the device, so that scan and update can be
 * enqueued back to back without a host round trip: the kernel reads *gate_dev (written earlier on
 * the same stream by ma_overflow_norm / ma_norm_combine); if gate_dev->overflow != 0 it returns
 * without touching any buffer; otherwise it derives clip_coef from gate_dev->sumsq and max_norm
 * exactly as ma_clip_coef does (max_norm <= 0: no clipping). */
int ma_adamw_step_gated(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                        ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step,
                        float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                        void* stream);

/* ---- the whole step in one call ---------------------------------------------------------------------- */

/* Scan, gate and update of one flat sub-group (Sec. IV-A: the check validates the gradients, then the
 * optimizer steps) in one call and TWO launches instead of three: the scan writes its per-block
 * partial results to ws, and every block of the update launch adds them up itself, in the order
 * ma_overflow_norm's own second-level launch uses, before it touches any buffer.  *out_dev receives
 * {overflow, sumsq}, bit-identical to ma_overflow_norm's; p32, m, v, p_lp are updated exactly as by
 * ma_adamw_step_gated with this max_norm (not at all when overflow is set).  Saves about 5 us per
 * step, which matters for sub-groups of a few million elements, whose step is launch-bound.
 * Not for sub-groups that share one global norm (Sec. IV-C): those need all scans, ma_norm_combine,
 * then the gated updates.  ws as for ma_overflow_norm; it must not overlap any buffer.  n == 0 writes
 * {0, 0.0}. */
int ma_optimizer_step(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                      ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step, float loss_scale,
                      float max_norm, ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream);

/* ---- half-precision optimizer states ---------------------------------------------------------- */

/* The same step with p, m and v held in bf16 (Extended Experiments, bf16 half-precision optimizer:
 * parameters, gradients and both moments move in half precision).  Each element is widened to
 * fp32, updated exactly as in ma_adamw_step, and stored back by direct truncation (the low 16 bits
 * of the fp32 result are dropped; a NaN stays a NaN).  p, m, v: bf16 device buffers, updated in
 * place; the parameter buffer itself is the low-precision copy, so there is no p_lp.
 * 14 bytes per element instead of 28. */
int ma_adamw_step_bf16(void* p_bf16, void* m_bf16, void* v_bf16, const void* grad, ma_dtype gdt,
                       size_t n, const ma_hyper* hyper, int64_t step, float loss_scale,
                       float clip_coef, void* stream);

/* ma_adamw_step_bf16 with the device-side gate of ma_adamw_step_gated. */
int ma_adamw_step_bf16_gated(void* p_bf16, void* m_bf16, void* v_bf16, const void* grad,
                             ma_dtype gdt, size_t n, const ma_hyper* hyper, int64_t step,
                             float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                             void* stream);

/* ---- gradient accumulation --------------------------------------------------------------------- */

/* Accumulates one micro-batch gradient into the fp32 flat gradient buffer (Sec. III-C: the flat
 * buffer is kept in fp32 to support accumulation):
 *     acc32[i] = first ? widen(grad[i]) : acc32[i] + widen(grad[i])      (one fp32 addition)
 * grad: MA_BF16, MA_F16 or MA_F32, read only.  The accumulated buffer is then scanned and applied
 * with gdt = MA_F32. */
int ma_grad_accumulate(float* acc32, const void* grad, ma_dtype gdt, size_t n, int first,
                       void* stream);

/* The same accumulation fused with the scan of ma_overflow_norm over the NEW contents of acc32
 * (Algorithm 1 on fp32 values, mask 0x7F800000, and the sum of (acc_i / loss_scale)^2): for the last
 * micro-batch of an iteration, so that the check that precedes the optimizer step (Sec. IV-A) does
 * not read the flat buffer again.  Equivalent to ma_grad_accumulate followed by
 * ma_overflow_norm(acc32, MA_F32, ...).  scaler_dev: NULL, or a loss-scale state in device memory
 * whose scale replaces loss_scale.  n == 0 writes {0, 0.0}.  ws as for ma_overflow_norm. */
int ma_grad_accumulate_scan(float* acc32, const void* grad, ma_dtype gdt, size_t n, int first,
                            float loss_scale, const ma_scaler_state* scaler_dev,
                            ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream);

/* ---- dynamic loss scale on the device ------------------------------------------------------------ */

/* Writes {scale, 0, applied_steps, 0} to *scaler_dev. */
int ma_scaler_init(ma_scaler_state* scaler_dev, float scale, int64_t applied_steps, void* stream);

/* Advances the state after an iteration whose scan result is *gate_dev:
 *   overflow:  scale = max(scale * backoff, min_scale); good_steps = 0; skipped += 1
 *   otherwise: step += 1; good_steps += 1; if good_steps >= window:
 *              scale = min(scale * growth, max_scale); good_steps = 0
 * Enqueue it after the update of the same iteration. */
int ma_scaler_update(ma_scaler_state* scaler_dev, const ma_norm_result* gate_dev,
                     const ma_scaler_config* cfg, void* stream);

/* ma_overflow_norm with the loss scale read from *scaler_dev on the device. */
int ma_overflow_norm_auto(const void* grad, ma_dtype gdt, size_t n, const ma_scaler_state* scaler_dev,
                          ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream);

/* ma_adamw_step_gated with the loss scale and the update number (scaler_dev->step + 1) read on the
 * device; the bias corrections are evaluated there in fp64 by the routine the host calls use
 * (integer power by squaring in double-double arithmetic), so the step is bit-identical to
 * ma_adamw_step_gated called with the same scale and update number.  A whole iteration
 *   ma_overflow_norm_auto -> ma_adamw_step_auto -> ma_scaler_update
 * needs no host round trip, whether or not the step is skipped. */
int ma_adamw_step_auto(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                       ma_dtype pdt, size_t n, const ma_hyper* hyper,
                       const ma_scaler_state* scaler_dev, const ma_norm_result* gate_dev,
                       float max_norm, void* stream);

/* ---- multi-tensor variants (one launch over a whole tensor list) ------------------------------ */

/* Bytes of device memory ma_multi_prepare needs for a list of `count` tensors: one row per tensor
 * and a 64-byte head of counters with which the blocks of an update launch share out the last part
 * of the work.  The library writes the table in ma_multi_prepare and the head during every
 * ma_multi_adamw_step* launch (which leaves it zeroed again); the caller never touches it.
 * NEVER have two update launches of one plan in flight at once (two streams without an ordering
 * between them): they would share the counters, work items would be skipped or done twice, and they
 * write the same tensors anyway.  The library cannot detect this.  Scan launches of one plan may
 * overlap if they use different workspaces. */
size_t ma_multi_table_bytes(size_t count);

/* Validates list_host[0..count) (host array of device pointers; gradient dtype gdt, parameter
 * copy dtype pdt for the whole list), builds the work table and copies it to table_dev.  This
 * call synchronises `stream` before it returns, so list_host may be freed at once and the table
 * may be used on any stream afterwards.  Prepare once per tensor list; the plan stays valid as
 * long as the tensors do not move.  Tensors with n == 0 are allowed and skipped.  count >= 1.
 * Every non-empty tensor costs at least one work item (4096 elements' worth of a block's time), so
 * a list of thousands of tiny tensors runs far below the memory rate (measured: 20,000 tensors of
 * 0-300 elements, 3.0e6 elements in all, 327 us per step against 25 us for one flat call over the
 * same bytes; 290 tensors of up to 60,000 elements 76 against 60 us).  When such tensors are views
 * of one buffer, pass the buffer to the flat calls instead: the step is element-wise. */
int ma_multi_prepare(const ma_tensor* list_host, size_t count, ma_dtype gdt, ma_dtype pdt,
                     void* table_dev, size_t table_bytes, void* stream, ma_multi_plan* plan_out);

/* The same for a list whose p, m, v are held in bf16 and stored by truncation (Extended Experiments,
 * bf16 half-precision optimizer).  The plan is accepted by every ma_multi_* call below; the update
 * calls then run the step of ma_adamw_step_bf16 on every tensor. */
int ma_multi_prepare_bf16(const ma_tensor_bf16* list_host, size_t count, ma_dtype gdt, void* table_dev,
                          size_t table_bytes, void* stream, ma_multi_plan* plan_out);

/* ma_overflow_norm over every tensor of the plan: one flag, one sum. */
int ma_multi_overflow_norm(const ma_multi_plan* plan, float loss_scale, ma_norm_result* out_dev,
                           void* ws, size_t ws_bytes, void* stream);

/* ma_adamw_step over every tensor of the plan (same scalars for all tensors). */
int ma_multi_adamw_step(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step,
                        float loss_scale, float clip_coef, void* stream);

/* ma_adamw_step_gated over every tensor of the plan. */
int ma_multi_adamw_step_gated(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step,
                              float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                              void* stream);

/* ma_optimizer_step over every tensor of the plan: one scan launch, one update launch. */
int ma_multi_optimizer_step(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step, float loss_scale,
                            float max_norm, ma_norm_result* out_dev, void* ws, size_t ws_bytes,
                            void* stream);

/* The *_auto forms over a prepared tensor list. */
int ma_multi_overflow_norm_auto(const ma_multi_plan* plan, const ma_scaler_state* scaler_dev,
                                ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream);
int ma_multi_adamw_step_auto(const ma_multi_plan* plan, const ma_hyper* hyper,
                             const ma_scaler_state* scaler_dev, const ma_norm_result* gate_dev,
                             float max_norm, void* stream);

/* ---- host side: parameter buffer pool and pinned sizes (plain host code, no GPU needed) ---------- */

/* Shapes of the tensors that travel through the parameter buffer pool (Sec. IV-B): embedding and
 * LM head are vocab x hidden, the three feed-forward projections intermediate x hidden, K and V
 * kv_dim x hidden (kv_dim = KV heads x head size), Q and O q_dim x hidden. */
typedef struct ma_model_dims {
  uint64_t vocab, hidden, intermediate, kv_dim, q_dim;
} ma_model_dims;

enum { MA_POOL_EMBED = 0, MA_POOL_FFN = 1, MA_POOL_KV = 2, MA_POOL_QO = 3 };

/* The adaptive pool of Sec. IV-B and, for comparison, the original uniform pool of Sec. III-A.
 * Sub-pool k holds count[k] buffers of buffer_bytes[k] bytes starting at byte offset[k] of ONE
 * monolithic allocation of total_bytes. */
typedef struct ma_pool_layout {
  uint64_t count[4];             /* 2, 3N, 2N, 2N for N transformer blocks in flight */
  uint64_t buffer_bytes[4];      /* this process's shard of one tensor, rounded up to `align` */
  uint64_t offset[4];
  uint64_t total_bytes;          /* the adaptive pool */
  uint64_t uniform_count;        /* 2 + 7N buffers ... */
  uint64_t uniform_buffer_bytes; /* ... each as large as the largest of the four kinds */
  uint64_t uniform_bytes;        /* the original pool */
} ma_pool_layout;

/* Sizes both pools.  blocks_in_flight = N >= 1; elem_bytes = bytes of a low-precision parameter
 * (1, 2 or 4); partitions >= 1: number of data-parallel processes a tensor is sharded over (each
 * process buffers its own ceil(numel / partitions) elements); align: power of two every buffer size
 * is rounded up to (1 = exact sizes, 4096 = the granularity of a pinned allocation). */
int ma_pool_layout_compute(const ma_model_dims* dims, uint32_t blocks_in_flight, uint32_t elem_bytes,
                           uint32_t partitions, uint32_t align, ma_pool_layout* out_host);

/* Logical management of the monolithic allocation (Sec. IV-B): a table from the caller's key (one
 * per tensor being fetched) to the buffer it holds.  The pool hands out byte offsets; the memory
 * itself belongs to the caller.  Not thread-safe: one pool per thread, or lock around it. */
typedef struct ma_pool ma_pool;
int ma_pool_create(const ma_pool_layout* layout, ma_pool** pool_out);
void ma_pool_destroy(ma_pool* pool);
/* Takes a free buffer of sub-pool `kind` (MA_POOL_*) for `key`.  MA_ERR_ARG if the key already
 * holds a buffer, MA_ERR_FULL if the sub-pool has none left.  bytes_out may be NULL. */
int ma_pool_acquire(ma_pool* pool, uint64_t key, int kind, uint64_t* offset_out, uint64_t* bytes_out);
int ma_pool_lookup(const ma_pool* pool, uint64_t key, uint64_t* offset_out, uint64_t* bytes_out);
int ma_pool_release(ma_pool* pool, uint64_t key);
uint64_t ma_pool_in_use(const ma_pool* pool, int kind);

/* Bytes a pinned allocation of `request` bytes occupies under a size policy (Sec. III-B, Sec. IV-C):
 * MA_PINNED_PAGE rounds up to 4096 bytes, the granularity DMA needs; MA_PINNED_POW2 rounds up to the
 * next power of two, as a caching host allocator does. */
enum { MA_PINNED_PAGE = 0, MA_PINNED_POW2 = 1 };
uint64_t ma_pinned_bytes(uint64_t request, int policy);

/* Page-locked host memory of exactly ma_pinned_bytes(bytes, MA_PINNED_PAGE) bytes, usable for DMA
 * from every device context (Sec. IV-C: static, long-lived offloading buffers get their exact size).
 * The caller frees it with ma_pinned_free.  These two calls need the HIP runtime. */
int ma_pinned_alloc(size_t bytes, void** host_ptr_out);
int ma_pinned_free(void* host_ptr);

/* ---- measurement aids (not steps of the path; a benchmark runs them beside the real kernels) ------- */

/* The update kernel's stream mix with trivial arithmetic.  state_elem_bytes == 4: per element reads
 * a, b, c (4-byte elements) and d16 (2-byte), writes a, b, c and e16 (2-byte): 14 bytes in, 14 bytes
 * out.  state_elem_bytes == 2 (states held in 16 bits): reads a, b, c, d16 (all 2-byte), writes a, b,
 * c: 8 bytes in, 6 out; e16 is not used and may be NULL.  n elements (whole work items of 4096 resp.
 * 8192 elements; the rest is left untouched).  All buffers 16-byte aligned device memory,
 * overwritten with meaningless values.  What this reaches is the ceiling the memory system sustains
 * for the step's read/write mix with the buffers where they are (Sec. II-A: the step is
 * memory-bound). */
int ma_probe_update_mix(void* a, void* b, void* c, const void* d16, void* e16, size_t n,
                        int state_elem_bytes, void* stream);

/* Two write-only streams of bytes_each bytes (whole multiples of 32 KiB are written), 16-byte aligned
 * device memory.  Two streams inside one physical region of the HBM sustain less together than two
 * streams in different regions, so timing this call at chosen offsets of a large allocation shows how
 * the allocation maps onto the regions. */
int ma_probe_two_writes(void* x, void* y, size_t bytes_each, void* stream);

/* ---- placement helper: device memory for one state, stitched from blocks of known HBM regions ------ */

/* The only calls of this library that allocate device memory; they exist to do so.  Where a state
 * lies physically decides ~4 % of the update kernel's rate (Sec. II-A: the step is memory-bound): best
 * measured is p | m | v | g with half of their traffic in one 96 GiB region of the HBM and half in
 * another, and the write-only parameter copy in a third.  ma_arena_create builds such a range with
 * the virtual-memory API: it creates physical blocks of block_bytes one by one, finds each block's
 * region by timing two write streams against the first block of every region seen so far, maps
 *     [first_region_bytes of main | rest of main | side]
 * from three different regions into ONE contiguous address range, and returns every block it does
 * not need to the driver.  On a fresh device physical memory is handed out region after region, so
 * reaching a second or third region means creating blocks worth the ones before; max_transient_bytes
 * bounds what may be held at once (0: just main + side, i.e. whatever regions come first).  When the
 * wanted regions cannot be had, the parts are filled from what there is; ma_arena_get_report says
 * how many blocks of each part lie where they were wanted.
 *   main_bytes > 0; first_region_bytes <= main_bytes: where main's traffic midpoint lies (rounded to
 *   blocks); side_bytes may be 0; block_bytes: 0 = 1 GiB, else a multiple of 2 MiB >= 64 MiB (smaller
 *   blocks are timed less reliably).  Creation synchronises the device and takes a few
 *   milliseconds per block.  The arena belongs to the device current at creation.
 *   Two things measured on MI355X that a caller should know: the driver wipes the blocks that go
 *   back in the background (~26 GB/s), and until it is done every kernel on the device runs about
 *   0.5 % slower; and once blocks have been created and released this way, a later allocation of the
 *   whole device (in any process) is no longer laid out linearly over the regions. */
typedef struct ma_arena ma_arena;
typedef struct ma_arena_report {
  uint64_t main_bytes, side_bytes, first_region_bytes; /* as mapped (whole blocks) */
  uint64_t blocks_created;                              /* physical blocks created while searching */
  uint64_t first_blocks_in_place, second_blocks_in_place, side_blocks_in_place;
  uint32_t regions_seen;
  float same_region_GBps; /* this machine's rate of two write streams inside one block */
} ma_arena_report;
int ma_arena_create(size_t main_bytes, size_t first_region_bytes, size_t side_bytes, size_t block_bytes,
                    size_t max_transient_bytes, ma_arena** arena_out);
void* ma_arena_main(const ma_arena* arena); /* device address of the main part */
void* ma_arena_side(const ma_arena* arena); /* device address of the side part, NULL if side_bytes was 0 */
int ma_arena_get_report(const ma_arena* arena, ma_arena_report* out_host);
int ma_arena_destroy(ma_arena* arena);      /* synchronises the device, then unmaps and releases everything (the
                                               addresses are invalid afterwards); NULL is allowed */

#ifdef __cplusplus
}
#endif
#endif /* MA_STEP_H_ */
