/*
 * moesys.h - C ABI of the MI355X (gfx950) MoE-layer library.
 *
 * The library implements the data-parallel hot path that the MoESys paper's
 * training and inference system exists to keep fed: the forward pass of a
 * sparsely-gated Mixture-of-Experts layer on one GPU (top-k softmax gate,
 * capacity-bounded dispatch, per-expert FFN, gate-weighted combine), the
 * paper's ring memory offloading of expert parameters (Section 3.3.2), an
 * expert-granular pool under its frequency-based scheduling (Algorithm 2),
 * and the layer's backward pass (the paper is a training system, Section 3.2).
 *
 * General rules of the boundary
 *  - Every pointer marked "device" is caller-owned HBM; "host" is caller-owned
 *    host memory ("pinned host" must come from hipHostMalloc / a pinned torch
 *    tensor).  The library allocates no device memory and keeps no reference
 *    to caller buffers after a call returns, except moe_ring (stated there).
 *  - Every compute call only enqueues work on the given HIP stream
 *    (hipStream_t passed as void*; NULL = the default stream) and never
 *    synchronises the device; per-expert row counts stay in HBM and are read
 *    by the kernels, never by the host (the paper's motivation for avoiding
 *    host<->device round trips in routing, Section 1 and Section 3.3.1).
 *  - Arguments are validated before any launch; errors are return codes, and
 *    moe_last_error() gives a thread-local explanation.  A call that returns
 *    an error has launched nothing.
 *  - All matrices are dense row-major.  Token activations x[T,d_model];
 *    router weight w_router[d_model,E] (input-major) in float32.
 *  - dtype = MOE_F32: x, expert weights, xd, h, yd, out are float32.
 *    dtype = MOE_BF16: they are bfloat16 (raw 16-bit), accumulated in float32
 *    on the MFMA units; h, yd and out are rounded to bfloat16 once each.
 *    The gate always produces float32 weights (softmax in fp32, Section 5.2).
 */
#ifndef MOESYS_H
#define MOESYS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = 1, /* null pointer, bad size, k > E, misaligned d ...   */
  MOE_ERR_UNSUPPORTED = 2, /* valid request this build has no kernel for         */
  MOE_ERR_WORKSPACE = 3,   /* workspace pointer null/misaligned or too small     */
  MOE_ERR_HIP = 4,         /* a HIP runtime call failed (see moe_last_error)     */
  MOE_ERR_STATE = 5        /* ring used out of order; expert cache without a free slot */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;
typedef enum { MOE_ACT_GELU = 0, MOE_ACT_SWIGLU = 1 } moe_act;

/* Expert weight layout.  OUTPUT_MAJOR ([E,out,in], the contraction index
 * contiguous) is the layout the bf16 MFMA kernels read; INPUT_MAJOR
 * ([E,in,out]) is accepted by the float32 kernels and converted once, outside
 * the hot path, with moe_transpose_expert_weights. */
typedef enum { MOE_LAYOUT_INPUT_MAJOR = 0, MOE_LAYOUT_OUTPUT_MAJOR = 1 } moe_layout;

#define MOE_MAX_EXPERTS 256
#define MOE_MAX_TOPK 8
#define MOE_DROPLESS INT32_MAX

typedef struct {
  int32_t T;        /* tokens in this call                        (>= 0)            */
  int32_t d_model;  /* multiple of 64                                               */
  int32_t d_ff;     /* multiple of 64                                               */
  int32_t E;        /* experts, 1..MOE_MAX_EXPERTS                                  */
  int32_t k;        /* experts per token, 1..min(E, MOE_MAX_TOPK)                   */
  float capacity_factor; /* <= 0: dropless; else C = ceil(k*T*CF/E), at least 1     */
  int32_t renormalize;   /* 1: top-k weights divided by their sum (GShard top-2);
                            0: weights are the softmax probabilities (Switch top-1) */
  int32_t act;      /* moe_act                                                      */
  int32_t dtype;    /* moe_dtype                                                    */
} moe_config;

/* Expert parameters, all device pointers.  GELU experts use w1,b1,w2,b2;
 * SwiGLU experts use w_gate_proj,w_up,w_down.  Biases may be NULL (= zero).
 *   INPUT_MAJOR : w1,w_gate_proj,w_up [E,d_model,d_ff];  w2,w_down [E,d_ff,d_model]
 *   OUTPUT_MAJOR: w1,w_gate_proj,w_up [E,d_ff,d_model];  w2,w_down [E,d_model,d_ff]
 * b1 [E,d_ff], b2 [E,d_model] in the activation dtype.
 * w_router [d_model,E] and b_router [E] (nullable) are float32.
 * expert_elem_offset (nullable; MOE_BF16 only): device int64 [E].  When given,
 * the experts are not one [E,...] array each: expert e's matrices and biases
 * start expert_elem_offset[e] elements after the respective base pointer (the
 * same offset for all of them), e.g. one blob per expert in a pool of slots
 * with w1 = pool, w2 = pool + d_ff*d_model, b1 = pool + 2*d_ff*d_model, ...
 * Offsets must be multiples of 8 elements.  Only experts that own rows are
 * dereferenced. */
typedef struct {
  const void* w1;
  const void* b1;
  const void* w2;
  const void* b2;
  const void* w_gate_proj;
  const void* w_up;
  const void* w_down;
  const float* w_router;
  const float* b_router;
  int32_t layout; /* moe_layout of the expert matrices */
  const int64_t* expert_elem_offset;
  const void* w_router_packed; /* nullable: w_router pre-split by moe_pack_router (MOE_BF16, E <= 64);
                                  the layer's gate then runs at the rate the tokens stream from HBM */
} moe_weights;

/* Byte offsets of every intermediate inside the workspace of moe_layer_forward
 * (so that a caller, e.g. a parity test, can read them back). */
typedef struct {
  size_t topk_idx;       /* int32 [T,k]                                   */
  size_t topk_w;         /* float [T,k]                                   */
  size_t expert_counts;  /* int32 [E]    assignments per expert before capacity */
  size_t expert_offsets; /* int32 [E+1]  first dispatched row of each expert    */
  size_t assign_to_row;  /* int32 [k*T]  row of assignment a=j*T+t, -1 dropped  */
  size_t row_to_assign;  /* int32 [k*T]  first R entries valid                  */
  size_t xd;             /* dtype [R_max,d_model] dispatched rows.  MOE_BF16: an empty
                            segment (the FFN gathers its rows from x through
                            row_to_assign), unless T*d_model*2 >= 2^31             */
  size_t h;              /* dtype [R_max,d_ff]    hidden activations            */
  size_t yd;             /* dtype [R_max,d_model] expert outputs.  MOE_BF16 with k == 1: an
                            empty segment (the second GEMM writes `out` itself)       */
  size_t scratch;        /* dispatch bookkeeping scratch                        */
  size_t tile_counters;  /* int32 [16] work counters of the two grouped GEMMs   */
  size_t total;          /* == moe_workspace_bytes(cfg, MOE_WS_LAYER)           */
  int64_t r_max;         /* min(k*T, E*C): upper bound of dispatched rows       */
} moe_ws_layout;

typedef enum { MOE_WS_LAYER = 0, MOE_WS_DISPATCH = 1, MOE_WS_FFN = 2 } moe_ws_kind;

/* ---- host-only helpers (no GPU needed) ---------------------------------- */

const char* moe_status_string(int32_t status);
/* Thread-local text describing the last error returned on this thread. */
const char* moe_last_error(void);
/* Library version as major*10000 + minor*100 + patch. */
int32_t moe_version(void);

/* Validates cfg (same checks every compute call performs). */
int32_t moe_config_check(const moe_config* cfg);

/* Expert capacity C = ceil(k*T*CF/E) in exact integer arithmetic (CF is the
 * float32 value given), at least 1; MOE_DROPLESS if capacity_factor <= 0.
 * The paper leaves capacity unspecified; this is the GShard/Switch form of the
 * gates it evaluates (Section 5.2).  Returns -1 on an invalid cfg. */
int32_t moe_capacity(const moe_config* cfg);

/* Bytes of device workspace needed by moe_layer_forward (MOE_WS_LAYER),
 * moe_dispatch (MOE_WS_DISPATCH) or moe_expert_ffn (MOE_WS_FFN).  Workspaces
 * must be 256-byte aligned.  Returns 0 on an invalid cfg. */
size_t moe_workspace_bytes(const moe_config* cfg, int32_t kind);
int32_t moe_workspace_layout(const moe_config* cfg, moe_ws_layout* out);

/* Process-wide tuning switches, for experiments and tests; every value gives the same
 * results, only the kernels that compute them differ.  Set them while no call of the
 * library is running on another thread.
 *   MOE_TUNE_GEMM_TILE_ROWS    token rows per tile of the bf16 grouped GEMM: 256 or 320;
 *                              0 (default) = chosen per call from the expected rows per expert
 *   MOE_TUNE_FEW_TOKEN_KERNELS 1 (default): steps of at most 16 tokens / assignments use the
 *                              matrix-vector expert kernels and the one-workgroup-per-token
 *                              gate; 0: the general kernels at every size
 *   MOE_TUNE_GATE_TOKENS       tokens per workgroup of the gate on a packed router: 32, 64 or 128 (where
 *                              the expert count allows; otherwise the next smaller); 0 (default) = by T
 *   MOE_TUNE_GEMM_MFMA         matrix instruction of the 256-row grouped GEMM kernels: 16 (16x16x32) or 32
 *                              (32x32x16); 0 (default) = 16 where an evenly loaded expert fills tiles.  The
 *                              results of the two are bit-identical.
 * moe_set_tuning returns MOE_ERR_INVALID_ARG for an unknown key or value. */
typedef enum { MOE_TUNE_GEMM_TILE_ROWS = 0, MOE_TUNE_FEW_TOKEN_KERNELS = 1, MOE_TUNE_GATE_TOKENS = 2,
               MOE_TUNE_GEMM_MFMA = 3, MOE_TUNE_COUNT = 4 } moe_tuning_key;
int32_t moe_set_tuning(int32_t key, int32_t value);
int32_t moe_get_tuning(int32_t key, int32_t* value);

/* ---- the hot path -------------------------------------------------------- */

/* Top-k softmax gate (the GShard top-2 / top-1 gates of Section 5.2, softmax
 * in fp32 as Section 5.2 states).
 *   z[t,e] = sum_i x[t,i]*w_router[i,e] + b_router[e];  p = softmax_e(z)
 *   topk_idx[t,0..k) = experts of the k largest z[t,.], descending, equal
 *                      logits -> lower expert index first
 *   topk_w[t,j] = p[t,topk_idx[t,j]]  (divided by their sum if renormalize)
 * Logits that decide the ranking are accumulated so that the selection equals
 * the one made on exactly computed logits (products of the stored values are
 * exact in float64; see the kernel for the fast path / exact path split).
 * x device [T,d_model] (cfg.dtype); w_router device [d_model,E] f32; b_router
 * device [E] f32 or NULL; topk_idx device int32 [T,k]; topk_w device f32
 * [T,k]; probs device f32 [T,E] or NULL. */
int32_t moe_gate(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                 int32_t* topk_idx, float* topk_w, float* probs, void* stream);

/* One-time router preparation, outside the hot path (like moe_transpose_expert_weights): every float32
 * router weight is split into three bfloat16 pieces whose sum is the weight exactly, stored in the order
 * the gate's matrix instructions read them, so that the gate's kernel only streams tokens and multiplies.
 * Nothing about the result changes: products stay exact, ranking equals that of the exactly computed
 * logits (near-ties are recomputed in float64 from w_router itself, which the gate still takes).
 * packed: device, moe_router_pack_bytes(d_model, E) bytes (0 = this shape has no packed form: E > 64),
 * 16-byte aligned.  moe_gate_packed is moe_gate on the packed router (MOE_BF16 only); moe_layer_forward
 * and moe_layer_route use moe_weights.w_router_packed when it is given. */
size_t moe_router_pack_bytes(int32_t d_model, int32_t E);
int32_t moe_pack_router(const float* w_router, void* packed, int32_t d_model, int32_t E, void* stream);
int32_t moe_gate_packed(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                        const void* w_router_packed, int32_t* topk_idx, float* topk_w, float* probs,
                        void* stream);

/* Capacity-bounded, order-preserving dispatch.  Assignment a = j*T + t
 * (choice-major: every first choice outranks every second choice; inside a
 * choice, token order).  Expert e keeps its first min(count_e, C) assignments;
 * kept rows of expert e are rows [expert_offsets[e], expert_offsets[e+1]) of
 * xd in increasing a; the rest are dropped (assign_to_row = -1).
 * expert_counts device int32 [E] (before capacity); expert_offsets device
 * int32 [E+1]; assign_to_row device int32 [k*T]; row_to_assign device int32
 * [k*T] (first R valid, rest untouched); xd device [R_max,d_model] (rows >= R
 * untouched); ws device scratch of moe_workspace_bytes(cfg, MOE_WS_DISPATCH).
 * xd may be NULL to build the routing tables only. */
int32_t moe_dispatch(const moe_config* cfg, const void* x, const int32_t* topk_idx,
                     int32_t* expert_counts, int32_t* expert_offsets, int32_t* assign_to_row,
                     int32_t* row_to_assign, void* xd, void* ws, size_t ws_bytes, void* stream);

/* moe_dispatch for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, tables and results as moe_dispatch, without ws: the bookkeeping scratch is a
 * static device array of MOE_DISPATCH_STATIC_SCRATCH_BYTES inside the library (one per GPU,
 * held until the process ends).  The call allocates nothing, frees nothing and does not
 * synchronise.  MOE_ERR_UNSUPPORTED if moe_workspace_bytes(cfg, MOE_WS_DISPATCH) exceeds
 * that size (roughly k*T*E > 64 M).  All calls on one GPU share that GPU's array: calls that
 * overlap on one GPU (different streams, or graphs replayed concurrently) race; calls on one
 * stream, and calls on different GPUs, do not. */
#define MOE_DISPATCH_STATIC_SCRATCH_BYTES ((size_t)1 << 20)
int32_t moe_dispatch_static(const moe_config* cfg, const void* x, const int32_t* topk_idx,
                            int32_t* expert_counts, int32_t* expert_offsets, int32_t* assign_to_row,
                            int32_t* row_to_assign, void* xd, void* stream);

/* Per-expert FFN (the sparsely activated "switching FFN" of Section 3.2) on
 * the dispatched rows: for r in [expert_offsets[e], expert_offsets[e+1])
 *   GELU  : yd[r] = gelu(xd[r] W1_e + b1_e) W2_e + b2_e,  gelu(u) = u*Phi(u)
 *   SwiGLU: yd[r] = (silu(xd[r] Wg_e) * (xd[r] Wu_e)) Wd_e
 * as two grouped GEMMs with the activation fused into the first one's
 * epilogue.  expert_offsets is read on the device.  xd device [R_max,d_model];
 * yd device [R_max,d_model]; ws device scratch (holds h[R_max,d_ff]) of
 * moe_workspace_bytes(cfg, MOE_WS_FFN).  MOE_BF16 needs MOE_LAYOUT_OUTPUT_MAJOR
 * weights (MOE_ERR_UNSUPPORTED otherwise). */
int32_t moe_expert_ffn(const moe_config* cfg, const moe_weights* w, const void* xd,
                       const int32_t* expert_offsets, void* yd, void* ws, size_t ws_bytes,
                       void* stream);

/* Gate-weighted combine:
 *   out[t] = residual[t] + sum_{j<k, assign_to_row[j*T+t] >= 0} topk_w[t,j] * yd[assign_to_row[j*T+t]]
 * accumulated in fp32, rounded once to cfg.dtype.  Dropped choices add nothing
 * and surviving weights are not rescaled.  residual device [T,d_model] or
 * NULL; out device [T,d_model]; out may alias residual. */
int32_t moe_combine(const moe_config* cfg, const void* yd, const int32_t* assign_to_row,
                    const float* topk_w, const void* residual, void* out, void* stream);

/* gate -> dispatch -> expert FFN -> combine on one stream with one workspace
 * (moe_workspace_bytes(cfg, MOE_WS_LAYER); layout from moe_workspace_layout).
 * The workspace need not be cleared; it serves one call at a time (calls that
 * overlap on the device need a workspace each).  Nothing is allocated and the
 * device is never synchronised, so the call can be captured in a HIP graph.
 * x device [T,d_model]; residual device [T,d_model] or NULL; out device
 * [T,d_model] (may alias residual, must not alias x unless residual == x).
 * Fusions inside the call (MOE_BF16): the first GEMM gathers its rows from x
 * through row_to_assign, so no dispatched copy xd is made; with k == 1 the
 * second GEMM scales each row by its gate weight, adds the residual in fp32
 * and stores it at its token's place in `out` (one rounding; no yd, and the
 * combine stage only fills the rows of dropped tokens) -- the kernel fusion
 * the paper asks for in Section 3.3.1. */
int32_t moe_layer_forward(const moe_config* cfg, const moe_weights* w, const void* x,
                          const void* residual, void* out, void* ws, size_t ws_bytes, void* stream);

/* The two halves of moe_layer_forward, for callers that have to look at the
 * routing before the experts run (e.g. to bring the activated experts'
 * parameters into HBM first, see moe_expert_pool_*): moe_layer_route runs
 * gate and dispatch bookkeeping into the workspace (w->w_router, w->b_router
 * are the only weights read); moe_layer_experts runs expert FFN and combine
 * from what moe_layer_route left in the same workspace.  Same arguments,
 * workspace and rules as moe_layer_forward; calling one after the other is
 * moe_layer_forward.  moe_layer_experts leaves the routing tables as it found
 * them, so it may run again on the same workspace (e.g. with other expert
 * weights, or after a failed load) without a new moe_layer_route. */
int32_t moe_layer_route(const moe_config* cfg, const moe_weights* w, const void* x, void* ws,
                        size_t ws_bytes, void* stream);
int32_t moe_layer_experts(const moe_config* cfg, const moe_weights* w, const void* x,
                          const void* residual, void* out, void* ws, size_t ws_bytes, void* stream);

/* Same as moe_layer_forward, additionally recording HIP events on `stream`
 * around every kernel so that a bench can attribute time per stage.  `timer`
 * comes from moe_timer_create.  Adds event-record overhead; not the call to
 * time end to end. */
typedef struct moe_timer moe_timer;
enum { MOE_STAGE_GATE = 0, MOE_STAGE_DISPATCH = 1, MOE_STAGE_GEMM1 = 2, MOE_STAGE_GEMM2 = 3,
       MOE_STAGE_COMBINE = 4, MOE_STAGE_COUNT = 5 };
int32_t moe_timer_create(moe_timer** out);
int32_t moe_timer_destroy(moe_timer* t);
int32_t moe_layer_forward_timed(const moe_config* cfg, const moe_weights* w, const void* x,
                                const void* residual, void* out, void* ws, size_t ws_bytes,
                                void* stream, moe_timer* timer);
/* Waits for the last timed call to finish and writes MOE_STAGE_COUNT stage
 * durations in milliseconds (host array). */
int32_t moe_timer_read(moe_timer* t, float* stage_ms);

/* One-time weight preparation, outside the hot path: dst[e,c,r] = src[e,r,c]
 * for E matrices of rows x cols elements of cfg-style dtype (device, distinct
 * buffers).  Converts INPUT_MAJOR expert matrices to OUTPUT_MAJOR. */
int32_t moe_transpose_expert_weights(const void* src, void* dst, int32_t E, int32_t rows,
                                     int32_t cols, int32_t dtype, void* stream);

/* ---- ring memory offloading (Section 3.3.2) ------------------------------ */
/*
 * The N layers' expert parameter blobs live in pinned host memory; K sections
 * of one caller-provided HBM region hold K of them.  After layer i has been
 * computed its section is released and refilled asynchronously, on a separate
 * copy stream, with the blob of the layer K positions ahead, so copies overlap
 * the following layers' compute ("calculation-released-load").  Layers must be
 * used in order 0,1,..,N-1,0,1,... (repeated inference steps wrap around); the
 * g-th use overall occupies section g mod K.
 *
 * The ring keeps the pointers it is given (dev_base, host_layers[i]) until
 * moe_ring_destroy; the caller keeps them alive.  It owns its events and, if
 * copy_stream is NULL, its own copy stream (default priority).
 */
typedef struct moe_ring moe_ring;

/* Backend of the ring: the HIP runtime by default; tests replace it to check
 * the schedule on a machine without a GPU.  All functions return 0 on success.
 * Streams and events are opaque handles. */
typedef struct {
  void* user;
  int32_t (*copy_h2d_async)(void* user, void* dst_dev, const void* src_host, size_t bytes, void* stream);
  int32_t (*event_create)(void* user, void** event);
  int32_t (*event_destroy)(void* user, void* event);
  int32_t (*event_record)(void* user, void* event, void* stream);
  int32_t (*stream_wait_event)(void* user, void* stream, void* event);
  int32_t (*event_synchronize)(void* user, void* event);
  int32_t (*event_elapsed_ms)(void* user, void* start, void* stop, float* ms);
} moe_ring_backend;

/* dev_base: device region of at least n_sections*layer_bytes bytes (256-byte
 * aligned); host_layers: host array of n_layers pinned-host blob pointers,
 * each layer_bytes long (the array itself is copied).  n_sections > n_layers
 * is clamped to n_layers (everything resident, no refills).  Enqueues the
 * initial load of layers 0..K-1 on the copy stream.  backend NULL = HIP. */
int32_t moe_ring_create(void* dev_base, size_t budget_bytes, int32_t n_sections,
                        const void* const* host_layers, int32_t n_layers, size_t layer_bytes,
                        void* copy_stream, const moe_ring_backend* backend, moe_ring** out);
/* Makes `compute_stream` wait until `layer`'s blob is in its section and
 * returns the section's device address in *dev_ptr.  MOE_ERR_STATE if `layer`
 * is not the next layer in sequence. */
int32_t moe_ring_acquire(moe_ring* r, int32_t layer, void* compute_stream, const void** dev_ptr);
/* Declares `layer`'s compute enqueued on compute_stream: the copy stream waits
 * for it and then refills the section with layer (layer+K) mod N. */
int32_t moe_ring_release(moe_ring* r, int32_t layer, void* compute_stream);
/* Waits for all enqueued copies; reports totals since creation.  copy_ms is
 * the sum of the copies' own durations from events (nullable outputs). */
int32_t moe_ring_stats(moe_ring* r, uint64_t* bytes_copied, uint64_t* copies, double* copy_ms);
int32_t moe_ring_destroy(moe_ring* r);

/* ---- backward pass -------------------------------------------------------- */
/* Backward of moe_combine for the gradient d_out [T,d_model] of its output: for every kept
 * choice (t,j) with row r = assign_to_row[j*T+t]
 *   d_yd[r] = topk_w[t,j] * d_out[t]   (cfg.dtype, one rounding)
 *   d_topk_w[t,j] = <d_out[t], yd[r]>  (float32, fp32 accumulation; 0 for a dropped choice)
 * The gradient of the residual is d_out itself.  All pointers device; yd, d_yd [R_max,d_model]
 * (rows beyond the kept ones are not touched); d_topk_w [T,k]. */
int32_t moe_combine_backward(const moe_config* cfg, const void* d_out, const void* yd,
                             const int32_t* assign_to_row, const float* topk_w, void* d_yd,
                             float* d_topk_w, void* stream);

/* Weight-gradient product of the expert FFN's backward pass (the paper is a
 * training system, Section 3.2, and leaves the kernels open): for every expert e
 *   c[e, n1, n2] = sum over r in [expert_offsets[e], expert_offsets[e+1]) of a[r, n1] * b[r, n2]
 * e.g. dW2_e = d_y_e^T h_e (a = d_y [R,d_model], b = h [R,d_ff]) and dW1_e = d_u_e^T xd_e for
 * OUTPUT_MAJOR weights.  a device bf16 [R,N1], b device bf16 [R,N2], c device [E,N1,N2] of
 * c_dtype = MOE_F32, or MOE_BF16 (the float32 sums rounded once: half the bytes written, for
 * callers that keep bf16 gradients) (overwritten; zero for an expert without rows); expert_offsets is read on
 * the device; max_rows_per_expert is the caller's bound of any expert's row count (only
 * used to check that an expert's operand block stays below 2 GiB).  N1 and N2 must be
 * multiples of 256 (MOE_ERR_UNSUPPORTED otherwise).  a_column_sums (nullable; device float32
 * [E,N1], overwritten): the sums over an expert's rows of a[r, n1], i.e. the bias gradient that
 * goes with the weight gradient (db2_e with dW2_e, db1_e with dW1_e), from the same pass. */
int32_t moe_expert_wgrad(const void* a, const void* b, const int32_t* expert_offsets, void* c,
                         int32_t c_dtype, float* a_column_sums, int32_t E, int32_t N1, int32_t N2,
                         int64_t max_rows_per_expert, void* stream);

/* Backward of moe_expert_ffn in MOE_BF16, given d_yd [R_max,d_model].  GELU experts:
 *   d_xd [R_max,d_model] (cfg.dtype), d_w1 [E,d_ff,d_model], d_b1 [E,d_ff], d_w2 [E,d_model,d_ff],
 *   d_b2 [E,d_model] (OUTPUT_MAJOR like the weights; overwritten; d_w1 and d_w2 of d_w_dtype =
 *   MOE_F32 or MOE_BF16 as in moe_expert_wgrad, the bias gradients float32 and required exactly
 *   when w has the bias).
 * w holds the OUTPUT_MAJOR weights of the forward pass; w1_input_major [E,d_model,d_ff] and
 * w2_input_major [E,d_ff,d_model] are their transposed copies (moe_transpose_expert_weights),
 * on which the input gradients are plain grouped products.
 * SwiGLU experts: the gate and up projections are treated as one stacked matrix:
 *   d_w1 [E,2*d_ff,d_model]: rows [0,d_ff) of expert e are the gradient of w_gate_proj[e], rows
 *   [d_ff,2*d_ff) that of w_up[e]; d_w2 [E,d_model,d_ff] is the gradient of w_down; d_b1, d_b2
 *   are not used; w1_input_major [E,d_model,2*d_ff] holds, for every expert and input feature,
 *   the d_ff gate weights followed by the d_ff up weights (the transposed stacked matrix);
 *   w2_input_major [E,d_ff,d_model] is the transposed w_down.
 * xd [R_max,d_model] and
 * h [R_max,d_ff] are the forward pass's dispatched rows and hidden activations (for
 * moe_layer_forward: gather xd with moe_dispatch; h is in the workspace); the
 * pre-activations are recomputed.  ws: moe_expert_ffn_backward_workspace_bytes(cfg), 256-byte
 * aligned.  d_model and d_ff must be multiples of 256.  All pointers device. */
size_t moe_expert_ffn_backward_workspace_bytes(const moe_config* cfg);
int32_t moe_expert_ffn_backward(const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                                const void* w2_input_major, const void* xd, const void* h,
                                const void* d_yd, const int32_t* expert_offsets, void* d_xd,
                                void* d_w1, float* d_b1, void* d_w2, float* d_b2, int32_t d_w_dtype,
                                void* ws, size_t ws_bytes, void* stream);

/* Load-balancing auxiliary loss.  The paper names auxiliary losses as the known remedy for
 * expert imbalance (Section 1, the computation challenge) without a formula; this is the one
 * of the work it cites there (GShard / Switch Transformer):
 *   loss = coef * E * sum_e expert_fraction[e] * mean_prob[e]
 * expert_fraction[e] = share of the T tokens whose FIRST choice topk_idx[t,0] is e (before
 * capacity), mean_prob[e] = mean over the tokens of probs[t,e]; loss == coef when the routing or
 * the probabilities are uniform.  probs [T,E] and topk_idx [T,k] as written by moe_gate; the
 * three outputs are device float arrays of E, E and 1 elements.  T == 0: MOE_ERR_INVALID_ARG.
 * Its gradient enters through moe_layer_backward's aux_loss_coef. */
int32_t moe_gate_aux_loss(const moe_config* cfg, const float* probs, const int32_t* topk_idx, float coef,
                          float* expert_fraction, float* mean_prob, float* loss, void* stream);

/* Backward of moe_layer_forward (MOE_BF16) for the gradient d_out
 * [T,d_model] of its output, with the routing of the forward pass held fixed:
 *   d_x [T,d_model] (cfg.dtype) = add_to_d_x (nullable; e.g. d_out when the layer ran with
 *       residual == x) + the experts' path (through dispatch) + the gate's path, one rounding;
 *   d_w_router [d_model,E], d_b_router [E] (float32; the latter required iff w->b_router);
 *   d_w1, d_b1, d_w2, d_b2, d_w_dtype as in moe_expert_ffn_backward.
 * aux_loss_coef != 0 adds the gradient of moe_gate_aux_loss(coef = aux_loss_coef) of this layer's
 * routing (it reaches d_x, d_w_router and d_b_router through the logits).
 * The gradient of the residual input is d_out itself.  fwd_ws is the workspace that
 * moe_layer_forward (or route + experts) left for the same cfg, x and w: its routing
 * tables and hidden activations are read; the gate is run again for the probabilities and
 * the pre-activations are recomputed.  ws: moe_layer_backward_workspace_bytes(cfg),
 * 256-byte aligned; nothing is allocated and the device is not synchronised. */
size_t moe_layer_backward_workspace_bytes(const moe_config* cfg);
int32_t moe_layer_backward(const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                           const void* w2_input_major, const void* x, const void* d_out,
                           const void* add_to_d_x, float aux_loss_coef, const void* fwd_ws,
                           size_t fwd_ws_bytes, void* d_x,
                           float* d_w_router, float* d_b_router, void* d_w1, float* d_b1,
                           void* d_w2, float* d_b2, int32_t d_w_dtype, void* ws, size_t ws_bytes,
                           void* stream);

/* ---- frequency-based expert cache (Algorithm 2, Section 3.2.2) ----------- */
/*
 * Host-side policy deciding which items (experts, numbered by the caller, e.g.
 * layer*E + e) occupy the `slots` slots of a pool in the faster memory.  It is
 * the paper's LFU-like scheduling of sparse parameters one tier up (pinned
 * host memory -> HBM instead of SSD -> CPU memory): a request of a cached item
 * adds one to its hit count; a new item takes a free slot, or with the pool
 * full the slot of the item with the lowest hit count among those whose count
 * is >= threshold (none such: the lowest count overall; ties: cached
 * earliest); after every decay_steps requests all counts are multiplied by
 * beta.  Items requested since the last moe_expert_cache_begin_batch are
 * never evicted (one layer's experts are needed together); MOE_ERR_STATE if
 * that leaves no slot.  No GPU call is made: the caller moves the data.
 */
typedef struct moe_expert_cache moe_expert_cache;
int32_t moe_expert_cache_create(moe_expert_cache** out, int32_t slots, float threshold, float beta,
                                int32_t decay_steps);
int32_t moe_expert_cache_destroy(moe_expert_cache* c);
int32_t moe_expert_cache_begin_batch(moe_expert_cache* c);
/* One request.  *slot: where `item` (>= 0) now lives; *hit (nullable): 1 if it
 * was cached already; *evicted (nullable): the item that lost its slot, or -1. */
int32_t moe_expert_cache_schedule(moe_expert_cache* c, int64_t item, int32_t* slot, int32_t* hit,
                                  int64_t* evicted);
/* *slot = -1 and *hits = 0 if `item` is not cached (nullable outputs). */
int32_t moe_expert_cache_lookup(const moe_expert_cache* c, int64_t item, int32_t* slot, double* hits);
int32_t moe_expert_cache_stats(const moe_expert_cache* c, uint64_t* hits, uint64_t* misses,
                               uint64_t* evictions);

/* ---- pool of expert slots fed from pinned host memory -------------------- */
/*
 * Offloading at expert granularity, for steps with few tokens: every expert's
 * parameter blob (any layout the caller's moe_weights base pointers and one
 * offset per expert can describe, e.g. [W1 | W2 | b1 | b2]) lives in pinned
 * host memory; dev_pool (device, 256-byte aligned) is cut into pool_bytes /
 * slot_bytes slots, managed by the frequency-based policy above with item
 * layer*E + e.  moe_expert_pool_prepare, called between moe_layer_route and
 * moe_layer_experts of `layer`:
 *   - reads the E per-expert counts from counts_dev (device; the workspace's
 *     expert_counts) and waits for compute_stream, because the host needs them;
 *   - schedules every expert with a count > 0 (ascending e, one batch), copies
 *     the blobs of the misses into their slots on the copy stream and makes
 *     compute_stream wait for those copies;
 *   - writes, through compute_stream, the table dev_offsets (device int64 [E])
 *     of slot offsets in elements of elem_bytes (0 for experts without rows),
 *     to be used as moe_weights.expert_elem_offset.
 * The pool keeps host_blobs' pointers ([n_layers*E], each blob_bytes long,
 * pinned) and dev_pool; the caller keeps them alive.  copy_stream NULL = a
 * stream of its own (default priority).  One pool serves one compute stream.
 */
typedef struct moe_expert_pool moe_expert_pool;
int32_t moe_expert_pool_create(void* dev_pool, size_t pool_bytes, size_t slot_bytes,
                               const void* const* host_blobs, int32_t n_layers, int32_t E,
                               size_t blob_bytes, float threshold, float beta, int32_t decay_steps,
                               void* copy_stream, moe_expert_pool** out);
int32_t moe_expert_pool_prepare(moe_expert_pool* p, int32_t layer, const int32_t* counts_dev,
                                int32_t elem_bytes, int64_t* dev_offsets, void* compute_stream);
/* Copies ahead of time (Section 3.2.2 uses the gate's results to prefetch; Section 3.3.2 overlaps loads with
 * compute): while the experts of one layer run, the caller routes the NEXT layer on what it has (e.g. the
 * running layer's input, on a second stream and workspace) and hands those counts over.  Every guessed expert
 * that is not resident is requested from the policy inside the current batch (so the running layer's experts are
 * never its victims) and its copy is enqueued on the copy stream; resident ones are left alone (a guess is not
 * a use).  Waits for `stream` (the one counts_dev was produced on), not for the compute stream.  The next
 * moe_expert_pool_prepare makes the compute stream wait for these copies as for its own.  A wrong guess costs
 * one copy and one slot.  *n_copied (nullable): blobs enqueued.  Stops without error when every slot holds an
 * item of the current batch. */
int32_t moe_expert_pool_prefetch(moe_expert_pool* p, int32_t layer, const int32_t* counts_dev, void* stream,
                                 int32_t* n_copied);
/* Totals since creation (nullable outputs). */
int32_t moe_expert_pool_stats(const moe_expert_pool* p, uint64_t* bytes_copied, uint64_t* copies,
                              uint64_t* hits, uint64_t* misses, uint64_t* evictions);
int32_t moe_expert_pool_destroy(moe_expert_pool* p);

#ifdef __cplusplus
}
#endif
#endif /* MOESYS_H */
