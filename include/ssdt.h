/*
 * ssdt -- transformer-layer forward/backward with activation offloading, for one AMD
 * MI355X (gfx950).  C ABI of libssdt.so.
 *
 * The library has two halves that meet in ssdt_layer_fwd / ssdt_layer_bwd:
 *
 *   - the layer kernels (hand-written HIP): the forward and backward pass of one
 *     transformer layer -- an attention block followed by an MLP block; a decoder layer
 *     is an encoder layer with a causal mask; an encoder-decoder's decoder layer has a
 *     second, cross-attention block over the encoder output (paper Sec. 2.1);
 *
 *   - the tensor cache of the paper (Sec. 3.1-3.3, Algorithm 1): a registry of the tensors
 *     saved for backward, deduplicated by storage identity, and an engine that copies them
 *     to pinned host memory on a side stream once their producer has finished, releases
 *     their device memory when the copy is done, and brings them back ahead of backward.
 *
 * General rules
 *   - Every pointer is labelled HOST or DEVICE.  "DEVICE" memory is owned by the caller
 *     (normally a PyTorch allocation) unless stated otherwise and must outlive its use on
 *     the GPU.  `ssdt_stream` is a hipStream_t passed as an opaque pointer (NULL = the
 *     default stream).
 *   - Calls enqueue GPU work and return; they never synchronise the device unless stated.
 *   - Nothing is thrown across the boundary.  Every call returns SSDT_OK (0) or a negative
 *     ssdt_status; ssdt_last_error() gives a message for the last failure on that context.
 *     A failed call leaves the registry as it was before the call.
 *   - One context per GPU per process; calls on one context must not overlap in time.
 *   - With backend SSDT_BACKEND_HIP the library needs a GPU and fails with SSDT_E_HIP
 *     without one; there is no CPU execution of the layer.  SSDT_BACKEND_SIM exists for
 *     host-side tests of the registry only: "device" pointers are ordinary host memory,
 *     copies are queued and performed when the test calls ssdt_sim_complete(), and the
 *     layer entry points return SSDT_E_UNSUPPORTED.
 */
#ifndef SSDT_H
#define SSDT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ssdt_ctx ssdt_ctx;
typedef int32_t ssdt_status;
typedef uint64_t ssdt_tid;  /* storage stamp; 0 = "bypassed: keep using the pointer you have" */
typedef void *ssdt_stream;  /* hipStream_t */

enum {
  SSDT_OK = 0,
  SSDT_E_INVAL = -1,       /* bad argument (null pointer, inconsistent shape, misaligned buffer) */
  SSDT_E_NOMEM = -2,       /* device arena or workspace too small */
  SSDT_E_HIP = -3,         /* a HIP runtime call failed (message has hipGetErrorString) */
  SSDT_E_IO = -4,          /* spill-file I/O failed */
  SSDT_E_STATE = -5,       /* call not legal in the record's / context's current state */
  SSDT_E_NOTFOUND = -6,    /* unknown tid / scope */
  SSDT_E_UNSUPPORTED = -7  /* feature or shape not supported by this build / backend */
};

enum { SSDT_BACKEND_HIP = 0, SSDT_BACKEND_SIM = 1 };
enum { SSDT_FWD = 0, SSDT_BWD = 1 };
enum { SSDT_F32 = 0, SSDT_BF16 = 1 };

/* Record classes (fixed at the first save of a storage) and states. */
enum { SSDT_CLS_SMALL = 1, SSDT_CLS_KEPT = 2, SSDT_CLS_OFFLOADED = 3 };
enum {
  SSDT_ST_RESIDENT = 1,   /* on the device (never left, reloaded, or forwarded) */
  SSDT_ST_STORING = 2,    /* device-to-host copy enqueued; device copy still present */
  SSDT_ST_OFFLOADED = 3,  /* host copy complete, device memory returned to the arena */
  SSDT_ST_LOADING = 4,    /* host-to-device copy enqueued into a new device slot */
  SSDT_ST_RELEASED = 5    /* all scopes finished; device memory returned */
};

typedef struct ssdt_config {
  int32_t backend;            /* SSDT_BACKEND_* */
  int32_t keep_last;          /* the last keep_last layers of a step are never offloaded (Sec. 3.3.2);
                                 paper default 1 */
  int64_t min_offload_elems;  /* a view with fewer elements is bypassed (Alg. 1; paper: 2^20) */
  int64_t budget_bytes;       /* offload amount per step (Sec. 3.1/3.2); < 0 = unlimited; 0 = offload off */
  void *arena_base;           /* DEVICE, 256-byte aligned: activation arena the library sub-allocates */
  size_t arena_bytes;
  size_t pool_bytes;          /* pinned host pool, allocated once at create (Sec. 3.1, CPU offloader) */
  const char *spill_path;     /* HOST string or NULL.  If set (Sec. 3.1, SSD offloader): the file is created
                                 or truncated at create (SSDT_E_IO if that fails) and becomes the store,
                                 the pool its staging buffer.  The file is opened for direct I/O (O_DIRECT:
                                 pinned pool to device without the page cache) where the file system allows it,
                                 and every tensor then starts on a 4096-byte boundary of pool and file instead
                                 of a 256-byte one.  Worker threads write every offloaded
                                 tensor to the file, at its pool offset, once its copy out of the device
                                 has completed, and then overwrite the tensor's pool bytes; a prefetch
                                 reads the tensor back into the pool, and the copy into the device is
                                 enqueued by the first later call on the context that finds the read
                                 complete (ssdt_get blocks the host for it if need be).  A failed
                                 read or write makes the next ssdt_offload / ssdt_prefetch / ssdt_get /
                                 ssdt_sync_io / ssdt_step_begin return SSDT_E_IO. */
  int32_t measure_waits;      /* nonzero: bracket every wait of a compute stream on a load with timing
                                 events so that ssdt_get_stats can report exposed I/O time */
  int32_t spill_threads;      /* threads serving the spill file (each with one request of up to 8 MiB at the
                                 device at a time); 0 = 4 */
} ssdt_config;

typedef struct ssdt_stats {
  /* bookkeeping of the current step (compared bit-exactly with the CPU checker) */
  uint64_t save_calls, unique, dedup_hits, bypass_weight, bypass_small, kept, offloaded;
  uint64_t bytes_small, bytes_kept, bytes_offloaded, pool_bytes_used;
  /* backward side */
  uint64_t loads, bytes_loaded, forwarded, demand_loads, released;
  /* arena */
  uint64_t arena_in_use, arena_high_water, arena_peak_in_use, arena_allocs;
  /* time (ns) compute streams spent blocked on loads / on arena slots still being stored during the current
     step (cleared by ssdt_step_begin like the other counters); complete once the streams have been
     synchronised, 0 unless measure_waits */
  uint64_t exposed_load_wait_ns, exposed_store_wait_ns;
} ssdt_stats;

typedef struct ssdt_record {
  ssdt_tid tid;
  int32_t layer;          /* owning layer = bottom of the scope stack at first save */
  int32_t cls;            /* SSDT_CLS_* */
  int32_t state;          /* SSDT_ST_* */
  int32_t n_scopes;       /* scopes still referring to it */
  uint64_t bytes;         /* storage bytes */
  int64_t pack_offset;    /* offset in its layer's pack, -1 unless OFFLOADED class */
  int64_t pool_offset;    /* offset in the host pool (= offset in the spill file) */
  void *device_ptr;       /* current device address or NULL */
  int32_t micro_batch;    /* micro-batch that was current at its first save */
  int32_t reserved;
} ssdt_record;

const char *ssdt_last_error(const ssdt_ctx *ctx); /* HOST string owned by the context; "" if none */
const char *ssdt_version(void);

/* ---- context ---------------------------------------------------------------------------- */

/* Creates a context: pins `pool_bytes` of host memory once, creates the store and load streams
 * (the paper's two first-in-first-out pools, Sec. 3.3.2).  `cfg` is copied.  E_INVAL for a null or
 * misaligned arena, E_HIP / E_NOMEM if pinning fails. */
ssdt_status ssdt_ctx_create(const ssdt_config *cfg, ssdt_ctx **out);
/* Waits for the side streams, frees the pool, streams, events and records.  The arena stays the
 * caller's. */
ssdt_status ssdt_ctx_destroy(ssdt_ctx *ctx);

/* Starts a step of `num_layers` layers (scopes 0 .. num_layers-1 are the layers; the keep-last rule
 * refers to them).  Clears the step's records and counters; E_STATE if records of the previous step
 * have not been released. */
ssdt_status ssdt_step_begin(ssdt_ctx *ctx, int32_t num_layers);
/* Switches to the records of micro-batch `mb` (Sec. 3.1: individual records are kept for each micro-batch and
 * the cache switches to the one of the new micro-batch when the scheduler changes micro-batch).  Every scope id
 * passed afterwards (scope_begin/end, offload, prefetch, release, the layer entry points) refers to that
 * micro-batch, so the records of several micro-batches can be alive between their forward and their backward.
 * `keep_last` >= 0 overrides ssdt_config.keep_last for this micro-batch (the paper keeps the last module only
 * where its backward follows its forward immediately); < 0 keeps the configured value.  ssdt_step_begin
 * selects micro-batch 0 and forgets the overrides.  E_STATE while a scope is open or before ssdt_step_begin;
 * E_INVAL for mb outside [0, 2^20). Scope ids must be below 2^20. */
ssdt_status ssdt_micro_batch(ssdt_ctx *ctx, int32_t mb, int32_t keep_last);
/* Changes the per-step offload amount (same meaning as ssdt_config.budget_bytes). */
ssdt_status ssdt_set_budget(ssdt_ctx *ctx, int64_t budget_bytes);

/* ---- offload amount ---------------------------------------------------------------------- */

/* Inputs of ssdt_plan: per-layer figures of one training step, forward order, all HOST memory. */
typedef struct ssdt_plan_in {
  int32_t num_layers;
  int32_t keep_last;            /* trailing layers that are never offloaded (Sec. 3.3.2) */
  const uint64_t *layer_bytes;  /* [num_layers] bytes each layer saves that can be offloaded */
  const double *fwd_s;          /* [num_layers] forward time of each layer, seconds */
  const double *bwd_s;          /* [num_layers] backward time of each layer, seconds */
  double store_Bps;             /* device -> pool (or file) rate, bytes / s */
  double load_Bps;              /* pool (or file) -> device rate, bytes / s */
  double safety;                /* in (0, 1]: share of both rates the plan may count on */
} ssdt_plan_in;

typedef struct ssdt_plan_out {
  int64_t budget_bytes;         /* value for ssdt_config.budget_bytes / ssdt_set_budget */
  int32_t layers;               /* leading layers entirely within the amount */
  int32_t prefetch_distance;    /* smallest d such that loading layer l when the backward of layer l+d starts
                                   hides every load; 0 if nothing is offloaded */
  uint64_t partial_bytes;       /* bytes of layer `layers` that are also within the amount */
  double store_done_s;          /* predicted end of the last store, from the start of the step */
  double fwd_total_s;
} ssdt_plan_out;

/* Sets the offload amount of a step from the amount of computation, the activation sizes and the
 * transfer rates (Sec. 3.1, workflow; Sec. 3.2, first condition of the pack hook).  Stores form one
 * queue in forward order, a layer's tensors being available when its forward ends; a byte is counted
 * only if it leaves the device before the forward pass ends, where the activation peak is reached.
 * Loads form one queue in reverse order and each must be complete when its layer's backward starts;
 * if no prefetch distance achieves that the amount is cut back, the partial layer first.  Pure host
 * arithmetic: needs no context and no GPU.  SSDT_E_INVAL for null pointers, num_layers <= 0,
 * negative times or keep_last, rates <= 0, safety outside (0, 1]. */
ssdt_status ssdt_plan(const ssdt_plan_in *in, ssdt_plan_out *out);

/* ---- device arena ----------------------------------------------------------------------- */

/* Sub-allocates `bytes` (rounded up to 256) from the arena for use on `stream`.  Memory whose
 * store has completed is reused first; if the only room left belongs to tensors still being stored,
 * `stream` is made to wait for the oldest such store (that wait is exposed I/O).  E_NOMEM otherwise.
 * The block belongs to the caller until it is passed to ssdt_save (then the registry frees it when
 * the record is released or its store completes) or to ssdt_arena_free. */
ssdt_status ssdt_arena_alloc(ssdt_ctx *ctx, size_t bytes, ssdt_stream stream, void **out);
/* Returns a block; work already enqueued on `stream` may still use it (later users on other
 * streams are ordered after an event recorded here). */
ssdt_status ssdt_arena_free(ssdt_ctx *ctx, void *ptr, ssdt_stream stream);

/* ---- registry (the tensor cache) -------------------------------------------------------- */

/* Records a weight buffer so that saves of it, or of any view of it, are bypassed (Sec. 3.3.1). */
ssdt_status ssdt_register_weight(ssdt_ctx *ctx, const void *base, size_t bytes);

/* Forward / backward hook pairs (Sec. 3.2).  FWD begin pushes `scope` on the scope stack and FWD
 * end pops it (E_STATE if it is not on top).  BWD begin/end only bracket a layer's backward for
 * error checking; the release is explicit (ssdt_release). */
ssdt_status ssdt_scope_begin(ssdt_ctx *ctx, int32_t scope, int32_t phase);
ssdt_status ssdt_scope_end(ssdt_ctx *ctx, int32_t scope, int32_t phase);

/* The pack hook (Algorithm 1).  A tensor is a view (`view_offset` bytes into the storage,
 * `shape[ndim]`, element type `dtype`) of the storage [storage_base, +storage_bytes) (DEVICE).
 * Applied in order: registered weight -> bypass; fewer than min_offload_elems elements -> bypass
 * (the storage is still tracked, class SMALL, so that its arena block is released with its scopes);
 * otherwise the storage gets a stamp the first time it is seen (a counter starting at 1, never
 * reused, also not when a later storage has the same address) and later saves of any view of it are
 * dedup hits; the current scope is added to its scope list; at the first save it is classed KEPT
 * (layer among the last keep_last, or offloaded-so-far + bytes > budget, or the host pool is full)
 * or OFFLOADED and given its place in the layer's pack (256-byte aligned, 4096 with a spill file; first-save
 * order; packs are rounded to 4096 bytes and follow each other in the pool).  `*out` = stamp, or 0 if bypassed.
 * E_STATE outside a forward scope. */
ssdt_status ssdt_save(ssdt_ctx *ctx, const void *storage_base, size_t storage_bytes, size_t view_offset,
                      const int64_t *shape, int32_t ndim, int32_t dtype, ssdt_tid *out);

/* Enqueues the device-to-host copies of layer `scope`'s OFFLOADED-class records that are not yet
 * stored, in save order, on the store stream, after an event recorded now on `producer` (offloading
 * starts once the producing operator has finished, Sec. 3.1).  When a copy completes the record's
 * arena block becomes reusable. */
ssdt_status ssdt_offload(ssdt_ctx *ctx, int32_t scope, ssdt_stream producer);

/* Enqueues the host-to-device copies of layer `scope`'s offloaded records on the load stream, in the
 * reverse of their save order (Sec. 3.1 step 5).  A record whose store has not completed yet is not
 * loaded: its device copy is kept and handed back instead (data forwarding, Sec. 3.3.2). */
ssdt_status ssdt_prefetch(ssdt_ctx *ctx, int32_t scope);

/* The unpack hook.  Returns the device address of the storage `tid`; `consumer` is made to wait for
 * its load if one is in flight (a load is started here if none was: a demand load).  The pointer is
 * borrowed until the release of the last scope referring to the record. */
ssdt_status ssdt_get(ssdt_ctx *ctx, ssdt_tid tid, ssdt_stream consumer, void **device_ptr);

/* Backward of `scope` is enqueued on `stream`: removes the scope from every record; records left
 * without scopes are released and their arena blocks freed (ordered after `stream`'s work). */
ssdt_status ssdt_release(ssdt_ctx *ctx, int32_t scope, ssdt_stream stream);

ssdt_status ssdt_get_stats(ssdt_ctx *ctx, ssdt_stats *out);
ssdt_status ssdt_num_records(const ssdt_ctx *ctx, uint32_t *out);
ssdt_status ssdt_get_record(const ssdt_ctx *ctx, uint32_t index, ssdt_record *out); /* in first-save order */
/* Copies `bytes` of the host pool starting at `pool_offset` into `dst` (HOST); waits for the store
 * stream first.  With a spill file it waits for the pending file writes too and reads the file
 * instead.  For tests of the reload-is-bit-identical invariant. */
ssdt_status ssdt_pool_read(ssdt_ctx *ctx, size_t pool_offset, void *dst, size_t bytes);
/* SIM backend only: performs the next `n` queued copies of direction 0 (store) or 1 (load), in
 * order, and marks them complete.  `*done` = number performed. */
ssdt_status ssdt_sim_complete(ssdt_ctx *ctx, int32_t direction, int32_t n, int32_t *done);
/* Blocks the host until the store and load streams are idle and, with a spill file, until every
 * file write and read requested so far has been done. */
ssdt_status ssdt_sync_io(ssdt_ctx *ctx);
/* Bytes written to and read from the spill file since create (either pointer may be NULL, HOST).
 * SSDT_E_STATE if the context has no spill file. */
ssdt_status ssdt_spill_stats(ssdt_ctx *ctx, uint64_t *bytes_written, uint64_t *bytes_read);
/* The same with the rest of what the file tier can report (HOST struct, filled): whether direct I/O is in
 * effect, the number of threads, and the wall time during which at least one write (read) request was at the
 * device, so that bytes / busy time is the file's write (read) rate as the offload path drives it. */
typedef struct ssdt_spill_info_t {
  int32_t direct_io, threads;
  uint64_t bytes_written, bytes_read, write_busy_ns, read_busy_ns;
} ssdt_spill_info_t;
ssdt_status ssdt_spill_info(ssdt_ctx *ctx, ssdt_spill_info_t *out);

/* ---- kernel timing ------------------------------------------------------------------------ */

/* Optional per-kernel-class timing: while enabled, every kernel launch of the layer entry points is
 * bracketed with HIP events on its launch stream.  ssdt_profile_read folds the finished measurements
 * into per-class totals (call it after synchronising the stream) and copies up to `cap` classes that
 * have launches; `flops` / `bytes` are the algorithmic work the launches were given (2 M N K for a
 * matrix product; the causal half for masked attention; bytes read + written for the others). */
typedef struct ssdt_kernel_time {
  char name[48];
  uint64_t launches;
  double ms, flops, bytes;
} ssdt_kernel_time;
ssdt_status ssdt_profile(ssdt_ctx *ctx, int32_t enable);  /* enabling also clears the totals */
ssdt_status ssdt_profile_read(ssdt_ctx *ctx, ssdt_kernel_time *out, uint32_t cap, uint32_t *n);

/* ---- the layer -------------------------------------------------------------------------- */

enum { SSDT_ARCH_GPT_PRELN = 0, SSDT_ARCH_BERT_POSTLN = 1, SSDT_ARCH_T5_ENC = 2, SSDT_ARCH_T5_DEC = 3 };
enum { SSDT_ACT_GELU = 0, SSDT_ACT_RELU = 1 };         /* GELU in its erf form */
enum { SSDT_NORM_LAYERNORM = 0, SSDT_NORM_RMSNORM = 1 };
enum { SSDT_MASK_NONE = 0, SSDT_MASK_CAUSAL = 1, SSDT_MASK_KEYPAD = 2 };

typedef struct ssdt_layer_desc {
  int32_t arch, dtype, act, norm, mask, has_bias;
  int32_t B, S, S_kv, H, A, F; /* micro-batch, (query) length, encoder length (T5_DEC), hidden, heads, FFN */
  float eps;                   /* norm epsilon */
  float softmax_scale;         /* 0 = 1/sqrt(H/A) */
  int32_t checkpoint;          /* nonzero: ssdt_layer_fwd registers only the layer's inputs (x, enc_out) for
                                  backward and frees every intermediate; the caller recomputes the layer
                                  inside its backward scope before ssdt_layer_bwd (layerwise full
                                  recomputation, the comparison arm of Sec. 4.3) */
  int32_t accumulate;          /* nonzero: ssdt_layer_bwd adds the weight, bias and norm-parameter gradients to what
                                  `grads` holds instead of overwriting it (gradient accumulation over the
                                  micro-batches of a step, Sec. 1); the sum is rounded to the tensors' type once
                                  per call */
} ssdt_layer_desc;

/* DEVICE pointers, element type = desc.dtype.  Matrices are row-major [in, out] (y = x W + b);
 * NULL where the variant has none (biases when has_bias = 0, *_b of RMSNorm, the lnx and *x
 * members unless T5_DEC).  The same struct carries the gradients in ssdt_layer_bwd. */
typedef struct ssdt_layer_weights {
  void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  void *lnx_g, *lnx_b, *w_qx, *b_qx, *w_kvx, *b_kvx, *w_ox, *b_ox;
  void *ln2_g, *ln2_b, *w_1, *b_1, *w_2, *b_2;
} ssdt_layer_weights;

/* What a layer saved for its backward, in the order of this enum (unused members have bytes = 0).
 * x: layer input; mean/rstd: fp32 per-row statistics of each norm; a, ax, m: norm outputs feeding
 * the QKV, cross-Q and FC1 projections (pre-norm variants); qkv [T,3H] (Q|K|V thirds, head h =
 * columns h*d..(h+1)*d-1 of a third); o: attention output; lse: fp32 [B,A,S]; r1, r2: residual sums
 * entering the norms (post-norm variant); x1, x2: block outputs; enc: encoder output; qx, kvx
 * [T_enc,2H], ox, lsex: cross-attention; h1: FC1 output (GELU only); g: activation output. */
enum {
  SSDT_SV_X = 0, SSDT_SV_MEAN1, SSDT_SV_RSTD1, SSDT_SV_A, SSDT_SV_QKV, SSDT_SV_O, SSDT_SV_LSE, SSDT_SV_R1,
  SSDT_SV_X1, SSDT_SV_MEANX, SSDT_SV_RSTDX, SSDT_SV_AX, SSDT_SV_ENC, SSDT_SV_QX, SSDT_SV_KVX, SSDT_SV_OX,
  SSDT_SV_LSEX, SSDT_SV_X2, SSDT_SV_MEAN2, SSDT_SV_RSTD2, SSDT_SV_M, SSDT_SV_H1, SSDT_SV_G, SSDT_SV_R2,
  SSDT_SV_COUNT
};
typedef struct ssdt_saved_entry {
  ssdt_tid tid;   /* 0 if bypassed: then `ptr` stays valid until the layer's release */
  void *ptr;      /* DEVICE address at forward time */
  uint64_t bytes;
} ssdt_saved_entry;
typedef struct ssdt_layer_saved {
  int32_t scope;
  int32_t reserved;
  ssdt_saved_entry e[SSDT_SV_COUNT];
} ssdt_layer_saved;

/* Bytes of scratch (DEVICE, 256-byte aligned, contents undefined between calls) that the two calls
 * below need for `desc`.  E_INVAL / E_UNSUPPORTED for an unusable description. */
ssdt_status ssdt_layer_workspace(const ssdt_layer_desc *desc, size_t *fwd_bytes, size_t *bwd_bytes);

/* Where ssdt_layer_bwd leaves its intermediate gradients: byte offsets from `ws` (for inspection and for
 * tests that check one operator of the backward at a time; nothing else needs them).  The contents are those of
 * the last ssdt_layer_bwd with this description, once its work on the stream has finished, and stay until the
 * next call that is given the workspace.  All are [B*S, width] in desc.dtype.
 *   d_h1  [T,F]   gradient w.r.t. the FC1 output (pre-activation)
 *   d_qkv [T,3H]  gradient w.r.t. the fused Q|K|V projection
 *   t0, t1, t2 [T,H]: for the pre-norm variants without cross-attention (GPT_PRELN, T5_ENC) t1 = gradient
 *         w.r.t. x1 (the residual stream between the two blocks), t0 = gradient w.r.t. the attention output o,
 *         t2 = gradient w.r.t. the first norm's output a (it held the gradient w.r.t. the second norm's output
 *         m earlier in the call).  BERT_POSTLN: t0 = gradient w.r.t. r2 then w.r.t. o, t1 = gradient w.r.t. x1
 *         then w.r.t. the attention block's input branch, t2 = gradient w.r.t. r1.  T5_DEC reuses them once more
 *         for the cross-attention block.
 *   d_kvx [T_enc,2H] T5_DEC only (else 0): gradient w.r.t. the fused K|V projection of the encoder output
 * E_INVAL / E_UNSUPPORTED as for ssdt_layer_workspace. */
typedef struct ssdt_bwd_temporaries {
  uint64_t d_h1, t0, t1, t2, d_qkv, d_kvx;
} ssdt_bwd_temporaries;
ssdt_status ssdt_layer_bwd_temporaries(const ssdt_layer_desc *desc, ssdt_bwd_temporaries *out);

/* Forward of one layer, enqueued on `stream`, as scope `scope` of the current step.
 *   x        DEVICE [B*S, H]: an arena block (ssdt_arena_alloc, or the previous layer's *y) whose
 *            ownership passes to the registry, or caller memory (then it is never freed here)
 *   enc_out  DEVICE [B*S_kv, H], T5_DEC only (else NULL); same ownership rule as x
 *   kv_len   DEVICE int32 [B], valid key count per sequence, MASK_KEYPAD only (else NULL)
 *   *y       DEVICE [B*S, H]: allocated here from the arena; the caller owns it
 *   *saved   HOST, filled: every tensor backward needs has been allocated from the arena and passed
 *            through the pack hook (ssdt_save) inside scope `scope`
 * The caller then calls ssdt_offload(ctx, scope, stream).  E_NOMEM (arena / workspace), E_INVAL. */
ssdt_status ssdt_layer_fwd(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w,
                           int32_t scope, const void *x, const void *enc_out, const int32_t *kv_len,
                           void **y, ssdt_layer_saved *saved, void *ws, size_t ws_bytes, ssdt_stream stream);

/* Backward of one layer, enqueued on `stream`.  Saved tensors are obtained through the unpack hook
 * (ssdt_get), so `stream` waits for loads that have not arrived.
 *   dy        DEVICE [B*S, H]   gradient of the layer output
 *   dx        DEVICE [B*S, H]   overwritten with the gradient of the layer input (may not alias dy)
 *   d_enc_out DEVICE [B*S_kv,H] T5_DEC only: the encoder-output gradient is ADDED to it
 *   grads     HOST struct of DEVICE pointers shaped like the weights; every present member is
 *             OVERWRITTEN.  Reductions run in a fixed order: results do not depend on addresses,
 *             on timing, or on whether tensors were offloaded.
 * The caller then calls ssdt_release(ctx, scope, stream). */
ssdt_status ssdt_layer_bwd(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w,
                           const ssdt_layer_saved *saved, const int32_t *kv_len, const void *dy, void *dx,
                           void *d_enc_out, const ssdt_layer_weights *grads, void *ws, size_t ws_bytes,
                           ssdt_stream stream);

/* ssdt_layer_bwd for callers that cannot allocate device memory or have none to hand over as a workspace (code
 * under stream capture, tight serving or training loops, harnesses that forbid allocation): same arguments, results
 * and ordering rules as ssdt_layer_bwd, bit for bit, but the workspace is an array of SSDT_STATIC_WS_BYTES that is
 * part of the library's device code (one per GPU the library runs on, held until the process ends).  The call
 * allocates and frees no device memory.  A layer whose backward needs more workspace than that
 * (ssdt_layer_workspace says how much) is refused with SSDT_E_NOMEM and a message; nothing is enqueued then.
 * Every call on a GPU shares that GPU's array, whatever the context: calls whose GPU work can overlap in time
 * (different streams without an ordering between them, different threads) race on it; calls enqueued on one
 * stream, or ordered by events, do not.  Nothing in the array has to be cleared between calls (every part is
 * written before it is read within a call). */
#define SSDT_STATIC_WS_BYTES ((size_t)64 << 20)
ssdt_status ssdt_layer_bwd_static(ssdt_ctx *ctx, const ssdt_layer_desc *desc, const ssdt_layer_weights *w,
                                  const ssdt_layer_saved *saved, const int32_t *kv_len, const void *dy, void *dx,
                                  void *d_enc_out, const ssdt_layer_weights *grads, ssdt_stream stream);

/* Plain SGD step on one parameter tensor: w <- w - lr * g elementwise, computed in fp32 and stored in `dtype`
 * (Sec. 4.1: the evaluation uses SGD so that the optimizer adds no state).  `w`, `g`: DEVICE, `numel` elements of
 * `dtype` (SSDT_F32 / SSDT_BF16), caller-owned; enqueued on `stream`.  E_INVAL for null pointers or an unknown
 * dtype, E_UNSUPPORTED on the simulated backend. */
ssdt_status ssdt_sgd_update(ssdt_ctx *ctx, void *w, const void *g, size_t numel, int32_t dtype, float lr, ssdt_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SSDT_H */
