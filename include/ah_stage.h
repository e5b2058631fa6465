/*
 * ah_stage.h — C ABI of the pipeline-stage compute library (libahstage.so).
 *
 * One stage object is one GPU's share of a training iteration: the forward and
 * the backward pass of a contiguous run of decoder layers on one
 * tensor-parallel shard, executed once per micro-batch, with gradients summed
 * in fp32 over the K micro-batches of the iteration.  Its run time is the
 * quantity t_i^j of the paper's iteration-time model (Section III-A, Eq. 1)
 * and the per-layer time and memory it reports are the inputs of the layer
 * partition problem (Section III-C, Eq. 4) and of the profiling scheme
 * (Section III-D, Eq. 5).
 *
 * General rules
 *  - Plain C.  Every function returns an ah_status_t (AH_OK = 0); nothing
 *    throws or aborts.  ah_last_error() gives a thread-local message for the
 *    last non-OK status.
 *  - All *device* pointers are caller-owned HIP device memory (the library
 *    never allocates device memory); the handle owns host metadata only.
 *  - ah_stage_forward / ah_stage_backward only enqueue work on the HIP stream
 *    passed as `hip_stream` (a hipStream_t cast to void*; NULL = the default
 *    stream) and never synchronise.  ah_stage_profile synchronises.
 *    ah_stage_backward may run work that nothing downstream waits for (the
 *    per-micro-batch weight-gradient products, the bias / gain reductions)
 *    on a stream of its own (created on the first call, at the default
 *    priority); it is ordered after the work it consumes and joined back into
 *    `hip_stream` before the call returns, so callers see ordinary
 *    single-stream semantics.
 *  - Matrices are row-major.  Rows of an activation are ordered batch-major:
 *    row = b * seq_len + s.  Linear layers are y = x W + b with W[in, out].
 *  - Activations and parameters are bf16 (bit pattern in uint16_t), gradients
 *    of parameters are fp32 and laid out exactly like the parameters.
 *
 * Tensor parallelism (Section II-B): the first matrix of each two-matrix block
 * (QKV, first MLP matrix) is cut by columns, the second (output projection,
 * second MLP matrix) by rows; a shard holds n_heads/tp_degree heads and
 * ffn_hidden/tp_degree hidden units.  The library computes one shard with
 * every reduction point treated as a sum over a one-member group, so `y` of
 * ah_stage_forward and `dx` of ah_stage_backward are the addends that the
 * tensor-parallel all-reduce would sum.
 */
#ifndef AH_STAGE_H
#define AH_STAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ah_stage ah_stage_t; /* opaque */

typedef enum {
  AH_OK = 0,
  AH_EINVAL = 1,       /* bad argument (NULL pointer, size out of range, bad slot) */
  AH_ENOMEM = 2,       /* host allocation failed */
  AH_ESTATE = 3,       /* call order: forward on a busy slot, backward on an empty one */
  AH_EDEVICE = 4,      /* a HIP call failed */
  AH_EUNSUPPORTED = 5  /* a shape the kernels do not cover (reported at create, never at launch); also: ah_stage_backward /
                        * ah_stage_flush_grads with wgrad_group > 1 on a stream that is being captured into a HIP graph */
} ah_status_t;

typedef enum {
  AH_ARCH_GPT = 0,   /* LayerNorm (eps 1e-5, biased variance), biases, tanh-form GeLU, causal attention */
  AH_ARCH_LLAMA = 1, /* RMSNorm, rotary embedding (pairs i, i+d/2), SwiGLU, no biases, causal attention */
  AH_ARCH_BERT = 2   /* the GPT block and parameter set with bidirectional attention: every position attends to
                      * every position of its sequence (the third model of Section V, BERT-Large; full-length
                      * sequences, no padding mask) */
} ah_arch_t;

/* Index of a parameter tensor inside a layer, in storage order.
 * GPT, BERT: LN1_G LN1_B WQKV BQKV WO BO LN2_G LN2_B W1 B1 W2 B2   (12 tensors)
 * LLAMA: LN1_G WQKV WO LN2_G W1(=gate|up, [h, 2*F_loc]) W2(=down)  (6 tensors)
 * WQKV columns are [Q | K | V], each block head-major. */
typedef enum {
  AH_P_LN1_G = 0, AH_P_LN1_B, AH_P_WQKV, AH_P_BQKV, AH_P_WO, AH_P_BO,
  AH_P_LN2_G, AH_P_LN2_B, AH_P_W1, AH_P_B1, AH_P_W2, AH_P_B2, AH_P_COUNT
} ah_param_t;

typedef struct {
  uint32_t struct_size;     /* sizeof(ah_stage_config_t), checked */
  int32_t arch;             /* ah_arch_t */
  int32_t n_layers;         /* l_i: layers of this stage (Section III-C), >= 1 */
  int32_t hidden;           /* h, multiple of 128, <= 16384 */
  int32_t n_heads;          /* heads of the unsharded layer */
  int32_t head_dim;         /* d: 64 or 128 */
  int32_t ffn_hidden;       /* FFN width of the unsharded layer */
  int32_t tp_degree;        /* must divide n_heads and ffn_hidden; local widths must be multiples of 128 */
  int32_t tp_rank;          /* 0 <= tp_rank < tp_degree (selects nothing inside the library: the caller passes that rank's shard) */
  int32_t seq_len;          /* S, multiple of 128 */
  int32_t microbatch_size;  /* B >= 1; T = B*S rows per call (a multiple of 128, as S is) */
  int32_t n_microbatches;   /* K of Eq. 1: micro-batches accumulated per iteration (used by ah_stage_profile) */
  int32_t max_in_flight;    /* activation slots: micro-batches whose forward has run and whose backward has not (1F1B: stages - stage index) */
  int32_t recompute;        /* 0: keep every layer's activations; 1: keep layer inputs only and re-run each layer's forward inside backward */
  int32_t wgrad_group;      /* G: how the gradient sum over the K micro-batches of an iteration (Section III-A, the
                             * accumulation behind Eq. 1's K micro-batch terms) is grouped.
                             * 0 or 1: every ah_stage_backward adds its micro-batch's weight gradients at once.
                             * G > 1 (<= 16, <= max_in_flight, recompute == 0): the weight-gradient products of a
                             * layer are taken once per G micro-batches, over the concatenation of their tokens,
                             * by the G-th backward of each group (or ah_stage_flush_grads): the fp32 gradient
                             * matrices are then read and written once per group instead of once per micro-batch.
                             * The sums are the same up to fp32 rounding order.  Cost: a micro-batch's slot stays
                             * occupied until its group is taken, and the workspace holds G * n_layers blocks of
                             * output-gradient operands (2*T*(2*hidden + first-MLP width + 3*local attention width) bytes each). */
  float norm_eps;           /* 0 selects the default: 1e-5 (GPT), 1e-6 (LLaMA) */
  float rope_base;          /* 0 selects 10000 */
  int32_t residual_fp32;    /* 0: the residual stream between the blocks (layer inputs, x + attention block) is bf16 like
                             * every other activation.  1: it is carried and saved in fp32 inside the stage (x and y at the
                             * boundary stay bf16): each layer then adds its two blocks to an unrounded sum, which removes the
                             * largest single source of forward error of a deep stage (the error of a stage of l_i layers,
                             * Section III-C Eq. 4, grows with l_i) at the cost of 4*T*hidden more bytes per saved layer. */
} ah_stage_config_t;

typedef struct {
  uint64_t param_elems;               /* bf16 elements in the parameter buffer = fp32 elements in the gradient buffer */
  uint64_t param_bytes, grad_bytes;   /* 2 and 4 bytes per element */
  uint64_t activation_bytes_per_slot; /* saved for backward, per in-flight micro-batch */
  uint64_t activation_bytes_per_layer_per_slot;
  uint64_t workspace_bytes;           /* scratch shared by all slots (includes the pending blocks of wgrad_group > 1) */
} ah_stage_sizes_t;

/* Device buffers, caller-owned, 256-byte aligned, of at least the sizes
 * ah_stage_query_sizes reports (activations: max_in_flight * per-slot bytes).
 * They must stay valid until ah_stage_destroy. */
typedef struct {
  void* params;       /* bf16 */
  void* grads;        /* fp32 */
  void* activations;
  void* workspace;
} ah_stage_buffers_t;

typedef struct {
  uint32_t struct_size;  /* sizeof(ah_stage_profile_t), checked */
  int32_t n_layers;      /* capacity of fwd_ms / bwd_ms; must be >= the stage's n_layers */
  float* fwd_ms;         /* host arrays supplied by the caller: median time of one micro-batch per layer */
  float* bwd_ms;
  float stage_fwd_ms, stage_bwd_ms;  /* whole stage, one micro-batch (median) */
  float iteration_ms;                /* K x (forward + backward), grads restarted at micro-batch 0 (median) */
  uint64_t peak_activation_bytes;    /* MEM_V: max_in_flight * per-slot bytes + workspace */
  uint64_t activation_bytes_per_layer_per_slot;
  uint64_t param_bytes, grad_bytes;  /* the part of MEM_F this library holds (no optimizer state) */
} ah_stage_profile_t;

/* Sizes of the four buffers for a configuration.  Validates the configuration
 * exactly as ah_stage_create does (AH_EINVAL / AH_EUNSUPPORTED). */
int ah_stage_query_sizes(const ah_stage_config_t* cfg, ah_stage_sizes_t* out);

/* Builds a stage over the caller's buffers.  Touches no device memory. */
int ah_stage_create(const ah_stage_config_t* cfg, const ah_stage_buffers_t* bufs, ah_stage_t** out);

/* Frees host metadata and the library's own stream and events.  The caller must have synchronised the streams it used. */
int ah_stage_destroy(ah_stage_t* st);

/* Where tensor `which` (ah_param_t) of layer `layer` lives: element offset into
 * the parameter buffer (and the gradient buffer), rows and cols (vectors:
 * rows = 1).  AH_EINVAL if the architecture has no such tensor. */
int ah_stage_param_layout(const ah_stage_t* st, int layer, int which, uint64_t* elem_offset, int32_t* rows, int32_t* cols);

/* Forward of all layers for one micro-batch (the forward half of t_i^j).
 *   x : device, bf16 [B*S, hidden], read only.   y : device, bf16 [B*S, hidden], written.
 *   slot in [0, max_in_flight) must be empty; it becomes busy until its backward.
 * Micro-batches are independent until their gradients meet (Section III-A), so with recompute = 0 the forward of one
 * slot may be enqueued on another stream than, and run beside, the backward of a different slot: forward writes only
 * its slot and `y`.  The caller orders the two streams where they meet: a slot's backward after its forward, a slot's
 * next forward after the backward that freed it.  With recompute = 1 forward and backward share the stage's one
 * per-layer workspace and must be ordered against each other like calls on one stream.  The calls themselves are
 * made from one host thread at a time. */
int ah_stage_forward(ah_stage_t* st, int slot, const void* x, void* y, void* hip_stream);

/* Backward of all layers for the micro-batch held in `slot` (the backward half
 * of t_i^j).  dy: device bf16 [B*S, hidden], read only; dx: device bf16
 * [B*S, hidden], written.  Adds every parameter's gradient into the fp32
 * gradient buffer (plain sum over micro-batches, no 1/K), or overwrites it if
 * this is the first backward after ah_stage_zero_grads, and frees the slot.
 * With wgrad_group G > 1 the slot stays occupied and the gradient buffer is
 * brought up to date when the G-th micro-batch of the group has had its
 * backward (that call takes the group's gradients and frees all G slots) or
 * at ah_stage_flush_grads; in between it may hold any mixture of old and new
 * sums (small matrices are still added per micro-batch). */
int ah_stage_backward(ah_stage_t* st, int slot, const void* dy, void* dx, void* hip_stream);

/* Closes an incomplete group of the gradient accumulation over micro-batches (Section III-A; see wgrad_group).
 * Takes the gradients of the micro-batches whose backward has run but
 * whose group is incomplete (wgrad_group > 1 and a micro-batch count that is
 * not a multiple of it), on `hip_stream`, and frees their slots.  After it the
 * gradient buffer holds the full sums, in stream order.  No-op when nothing
 * is pending. */
int ah_stage_flush_grads(ah_stage_t* st, void* hip_stream);

/* The fp32 gradient buffer (device pointer into the caller's `grads`) and its
 * element count; layout per ah_stage_param_layout.  With wgrad_group > 1 the
 * sums are complete once every group has been taken (see above). */
int ah_stage_grads(ah_stage_t* st, float** dev_ptr, uint64_t* n_elems);

/* Where the stage keeps the input of layer `layer` for the micro-batch in `slot`: device, [B*S, hidden] in bf16 (fp32
 * with residual_fp32 = 1), read only, valid from that slot's ah_stage_forward until the slot's next forward.  The input of layer l + 1 is the
 * output of layer l, so this is the per-layer view of the values that Section III-D's profiler takes of the times
 * (the stage is a chain of l_i layers, Section III-C Eq. 4): tests read it to see how the error against an exact
 * evaluation grows with depth.  Kept with and without recompute. */
int ah_stage_layer_input(ah_stage_t* st, int slot, int layer, const void** dev_ptr);

/* Starts a new accumulation: the next ah_stage_backward overwrites instead of
 * adding (no memset is enqueued; until that backward has run the buffer holds
 * the previous iteration's sums).  A new stage starts in this state.
 * AH_ESTATE while weight gradients are pending. */
int ah_stage_zero_grads(ah_stage_t* st, void* hip_stream);

/* Measures the stage on synthetic activations (what the paper's profiler
 * collects, Section III-D): per-layer forward and backward time of one
 * micro-batch, whole-stage times, the time of a K-micro-batch iteration, and
 * the byte counts of the memory model.  Uses slot 0 (all slots must be empty),
 * overwrites the gradient buffer, and synchronises the device. */
int ah_stage_profile(ah_stage_t* st, int warmup, int iters, ah_stage_profile_t* out);

/* Per-call-site timing of the kernels that forward / backward enqueue, for the
 * roofline report (Section III-D's profiler only needs whole-layer times; this
 * is the finer view).  Between _begin and _end every launch site is bracketed
 * by a HIP event pair on the stream it is launched on; _end synchronises the
 * device and fills up to `capacity` entries, one per site that ran. */
typedef struct {
  char name[32];            /* e.g. "gemm_nn.fc1_fwd", "attention_bwd", "norm_fwd" */
  int64_t launches;         /* event pairs recorded for this site */
  double total_ms;          /* sum of their durations */
  double flops_per_launch;  /* algorithmic flops of one launch (0 for bandwidth-bound sites) */
  double bytes_per_launch;  /* algorithmic HBM bytes of one launch (0 for the MFMA-bound sites) */
} ah_trace_entry_t;
int ah_stage_trace_begin(ah_stage_t* st);
int ah_stage_trace_end(ah_stage_t* st, ah_trace_entry_t* out, int capacity, int* n_out);

/* Message for the calling thread's last non-OK status (never NULL). */
const char* ah_last_error(void);

/* Single-kernel entry points used by the per-kernel parity tests and the
 * roofline measurement.  All pointers are device pointers; shapes must obey
 * the tile constraints stated with each (else AH_EUNSUPPORTED). */

/* C[M,N] (bf16) = A[M,K] B[K,N] + bias[N] (bias may be NULL).  M, N and K multiples of 128. */
int ah_gemm_nn(const void* A, const void* B, const void* bias, void* C, int M, int N, int K, void* hip_stream);
/* The first product of the SwiGLU block with its activation fused (the LLaMA-style stage's MLP, first matrix cut by
 * columns as in Section II-B): B[K, 2F] holds gate | up; U[M, 2F] (bf16) = A B, Mout[M, F] (bf16) =
 * silu(U[:, :F]) * U[:, F:] evaluated on the fp32 sums before they are rounded.  M, F and K multiples of 128. */
int ah_gemm_nn_swiglu(const void* A, const void* B, void* U, void* Mout, int M, int F, int K, void* hip_stream);
/* C[M,N] (bf16) = A[M,K] B[N,K]^T.  Same constraints. */
int ah_gemm_nt(const void* A, const void* B, void* C, int M, int N, int K, void* hip_stream);
/* C[M,N] (fp32) = beta * C + A[K,M]^T B[K,N], beta in {0, 1}.  Same constraints. */
int ah_gemm_tn(const void* A, const void* B, float* C, int M, int N, int K, int beta, void* hip_stream);
/* ah_gemm_tn with the k axis given in n_seg pieces of seg_k rows each (K = n_seg * seg_k): piece i of A is
 * A_seg[i][seg_k, M], of B is B_seg[i][seg_k, N].  A_seg and B_seg are HOST arrays of device pointers, read
 * during the call.  1 <= n_seg <= 16, seg_k a multiple of 128.  This is the product the deferred weight
 * gradient (wgrad_group) runs over the micro-batches of a group. */
int ah_gemm_tn_segmented(const void* const* A_seg, const void* const* B_seg, int n_seg, float* C, int M, int N, int seg_k,
                         int beta, void* hip_stream);
/* Attention over packed qkv[B*S, 3*nh*d] (bf16, [Q|K|V], head-major): o[B*S, nh*d] bf16, lse[B, nh, S] fp32.
 * causal != 0: query i attends to keys 0..i of its sequence; causal == 0: to all S keys. */
int ah_attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int nh, int d, int causal, void* hip_stream);
/* Its backward: dqkv[B*S, 3*nh*d] from qkv, o, lse and do[B*S, nh*d]; `delta` is fp32 scratch [B, nh, S]. */
int ah_attention_bwd(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, float* delta,
                     int B, int S, int nh, int d, int causal, void* hip_stream);


/* ah_attention_bwd for callers that cannot allocate device memory or hand over scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same output, same kernels; the
 * fp32 scratch [B, nh, S] that ah_attention_bwd takes as `delta` lives in a fixed array inside the library's
 * device image instead (1 MiB per GPU, held until the process ends), so B * nh * S must not exceed
 * AH_ATTENTION_STATIC_MAX_ROWS (else AH_EINVAL, nothing is launched).  The call allocates nothing and frees
 * nothing.  The device that holds the buffers must be the calling thread's current device.  Every call on a GPU
 * uses that GPU's one array (fully rewritten by each call before it is read): calls that overlap on one GPU, on
 * different streams or from different threads, race; calls in stream order on one stream do not. */
#define AH_ATTENTION_STATIC_MAX_ROWS 262144
int ah_attention_bwd_static(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                            int B, int S, int nh, int d, int causal, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AH_STAGE_H */
