/*
 * autochunk_rt — runtime execution of AutoChunk chunk plans on one MI355X (gfx950).
 *
 * AutoChunk (arXiv 2401.10652), section 2.2: a module Y = F(X) is "chunked" by
 * splitting X along a chunk dimension into n segments, computing y_i = F(x_i) one
 * segment after another and concatenating the y_i, which bounds the intermediate
 * activation A to A/n (second activation equation) while Y stays equal to the
 * unchunked result (section 3.3, output alignment rule).  Section 3.1 writes a
 * region as Y^c = F(X^c, X^nc): chunkable inputs are sliced, non-chunkable inputs
 * (weights, attention keys/values, the second triangle operand) are seen whole by
 * every segment.  This library is that runtime step only: it takes a region list
 * with a chunk dimension and chunk length per region (or an activation budget from
 * which it sizes the lengths, section 3.2), a workspace sized from that plan, and
 * runs the plan with hand-written HIP kernels.  The compiler passes of the paper
 * (search, selection, code generation) are not part of it.
 *
 * Conventions for every call:
 *   - "dev" pointers are device (HBM) addresses owned by the caller; the library never
 *     allocates, frees or retains device memory and never synchronises the stream,
 *     except where a call says so.  "host" pointers are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Matrices are row-major.  Every weight matrix is [out_features, in_features].
 *   - Storage dtype AC_BF16: every tensor in HBM (activations, weights, biases, LayerNorm
 *     gain/shift, workspace) is bfloat16, rounded to nearest-even once per store; all sums
 *     (GEMM, LayerNorm statistics, softmax, probability-value products, residual adds)
 *     are fp32.  AC_F32: everything fp32.
 *   - Return value: AC_OK (0) or a negative ac_status.  No exception or abort crosses
 *     this boundary; ac_last_error() gives the text of the calling thread's last failure.
 */
#ifndef AUTOCHUNK_RT_H
#define AUTOCHUNK_RT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ac_status {
  AC_OK = 0,
  AC_ERR_ARG = -1,                /* null pointer, non-positive size, inconsistent descriptor */
  AC_ERR_ILLEGAL_CHUNK_DIM = -2,  /* the region reduces over / reshapes across that dim (rules 1-4, section 3.3) */
  AC_ERR_BUDGET_INFEASIBLE = -3,  /* even the smallest segment exceeds the activation budget */
  AC_ERR_WORKSPACE = -4,          /* workspace smaller than the plan needs; nothing was launched */
  AC_ERR_ALIGN = -5,              /* a device pointer is not 256-byte aligned */
  AC_ERR_HIP = -6,                /* a HIP call failed; text in ac_last_error() */
  AC_ERR_STATE = -7,              /* weights not bound, or profiling not enabled */
  AC_ERR_UNSUPPORTED = -8         /* legal, but no kernel here covers that shape or chunk dim */
} ac_status;

typedef enum ac_workload { AC_TRANSFORMER_STACK = 0, AC_PAIR_STACK = 1, AC_UNET_RES_STACK = 2 } ac_workload;
typedef enum ac_dtype { AC_F32 = 0, AC_BF16 = 1 } ac_dtype;
typedef enum ac_activation { AC_ACT_NONE = 0, AC_ACT_GELU_ERF = 1, AC_ACT_GELU_TANH = 2,
                             AC_ACT_RELU = 3, AC_ACT_SIGMOID = 4, AC_ACT_SILU = 5 } ac_activation;

/* Region kinds.  Transformer layer: QKV, ATTENTION, OUT_PROJ, FFN in this order.  Pair-stack
 * block: TRIMUL_OUT, TRIMUL_IN, TRIATT_START, TRIATT_END, PAIR_TRANSITION in this order.
 * The attention core is a region of its own (section 3.4: a chunk region should hold few
 * nodes beyond the peak node), so the projection after it need not be cut as finely. */
typedef enum ac_region_kind {
  AC_REGION_QKV = 0,            /* LayerNorm 1 + packed query/key/value projection        */
  AC_REGION_ATTENTION = 1,      /* attention of a query segment over whole keys/values;
                                   writes its rows of the whole context tensor            */
  AC_REGION_OUT_PROJ = 2,       /* output projection of the context + residual            */
  AC_REGION_FFN = 3,            /* LayerNorm 2 + up projection + activation + down + residual */
  AC_REGION_TRIMUL_OUT = 4,     /* triangle multiplicative update, outgoing edges         */
  AC_REGION_TRIMUL_IN = 5,      /* triangle multiplicative update, incoming edges         */
  AC_REGION_TRIATT_START = 6,   /* triangle self-attention around the starting node       */
  AC_REGION_TRIATT_END = 7,     /* triangle self-attention around the ending node         */
  AC_REGION_PAIR_TRANSITION = 8,
  AC_REGION_RES_BLOCK = 9,      /* UNet residual block: GroupNorm, SiLU, 3x3 convolution, time
                                   embedding, again, skip (section 4 names the family)       */
  AC_REGION_UNET_ATTN = 10,     /* UNet attention block: GroupNorm, linear in, pre-LN self-attention
                                   over the positions of an image and feed-forward, linear out, skip */
  AC_REGION_KINDS = 11
} ac_region_kind;

/* Chunk dimensions are named per workload.  Transformer regions see their tensors as
 * [batch, sequence(query), feature, head_dim, key]; pair regions as [row i, column j,
 * channel, contraction index k].  Legal (section 3.3: no node of the region reduces over
 * the dim): batch and sequence for every transformer region; row and column for every
 * pair region; feature for the attention region (whole heads) and the output projection
 * (blocks of output columns).  Otherwise feature, head_dim, key, channel and contraction
 * index are illegal.  A column chunk of a pair region gathers its positions with the two
 * indices swapped (a copy that counts as activation memory, section 3.4) and runs the module's
 * transposed form on them.  A feature chunk spans all rows: chunk_len counts features and must be
 * a multiple of head_dim for the attention region (a segment is a run of whole heads) and of 8
 * for the output projection (a block of output columns), else AC_ERR_ARG.  Regions whose
 * segments hold no tensor of their own (the fused attention core, the fused output projection,
 * LayerNorm + packed projection) run consecutive segments in one launch; ac_region_info.launches
 * says how many launches a layer's region takes. */
enum { AC_DIM_BATCH = 0, AC_DIM_SEQ = 1, AC_DIM_FEATURE = 2, AC_DIM_HEAD_DIM = 3, AC_DIM_KEY = 4 };
enum { AC_DIM_ROW = 0, AC_DIM_COL = 1, AC_DIM_CHANNEL = 2, AC_DIM_CONTRACT = 3 };

/* ac_model_desc.flags */
enum {
  AC_FLAG_UNFUSED_ELEMENTWISE = 1, /* run bias+activation and residual as standalone passes
                                      instead of GEMM epilogues (for measuring those passes) */
  AC_FLAG_TWO_SEGMENTS_IN_FLIGHT = 4, /* segments of a region alternate between the caller's stream and a
                                      second stream owned by the plan, each with its own per-segment
                                      workspace (the plan's bytes account for both); all work is joined
                                      back into the caller's stream at the end of every region */
  AC_FLAG_LISTED_REGIONS_ONLY = 2, /* pair stack only: the block consists of just the region kinds
                                      listed in ac_plan_create (each maps z to z), in canonical
                                      order; weights of the others are still bound but unused */
  AC_FLAG_MATERIALIZED_SCORES = 8, /* transformer stack only: the attention core runs as an unfused graph
                                      would (AutoChunk section 2.1): scores = q k^T per head stored in the
                                      workspace, probabilities = softmax(scores) stored beside them,
                                      context = probabilities v.  The workspace then really holds the
                                      intermediate activations the paper's equations count, mem(A) whole
                                      or mem(A)/n per segment, so the effect of chunking on memory can be
                                      measured and not only modelled.  Same result as the fused kernel up
                                      to the rounding of the stored scores and probabilities.  With a
                                      causal mask the masked half is computed and discarded;
                                      flops_per_execute counts what is executed. */
  AC_FLAG_BUDGET_PAPER_MODEL = 16, /* act_budget_bytes additionally bounds, for every region, the bytes
                                      the paper's two activation equations give for an unfused graph in
                                      which every op output is a tensor (ac_region_info.model_bytes:
                                      scores and probabilities of a segment included), as a planner that
                                      sees such a graph would size it (AutoChunk section 3.2, 3.4).
                                      Without the flag the budget bounds what this executor really
                                      holds, where the scores never reach memory. */
  AC_FLAG_GATED_FFN = 32           /* UNet attention block only: the feed-forward's first layer is 2 * d_ffn
                                      wide and its hidden rows are value * activation(gate), value from the
                                      first d_ffn output features and gate from the second */
};

typedef struct ac_model_desc {
  int32_t workload;      /* ac_workload */
  int32_t dtype;         /* ac_dtype: storage type of every tensor */
  int32_t layers;        /* transformer: number of blocks; pair stack: number of blocks (>= 1) */
  /* transformer stack: x and y are [batch * seq, d_model] */
  int32_t batch, seq, d_model, heads, head_dim, d_ffn;
  int32_t causal;        /* 1: key j visible to query i iff j <= i */
  int32_t activation;    /* ac_activation of the feed-forward / pair transition */
  /* pair stack: z is [n_res, n_res, c_z] */
  int32_t n_res, c_z, c_hidden, tri_heads, tri_head_dim, transition_factor;
  int32_t flags;
  float ln_eps;          /* LayerNorm / GroupNorm epsilon (biased variance) */
  /* UNet residual stack (bf16 only): x and y are channels-last images [batch, img_h, img_w, channels];
   * `layers` residual blocks one after another, GroupNorm over `groups` runs of consecutive channels.
   * Its one region kind is chunked along the batch (AC_DIM_BATCH): every other dim is reduced over by
   * a GroupNorm or by a convolution window (section 3.3).
   * With heads > 0 every residual block is followed by an attention block (region kind
   * AC_REGION_UNET_ATTN, also chunked along the batch: its GroupNorm and its attention reduce over the
   * positions): `heads` heads of channels / heads = 32, 64 or 128 channels each, feed-forward width
   * d_ffn (a multiple of 64) with `activation`; head_dim is ignored.  With seq > 0 the attention block
   * also has a cross-attention between its self-attention and its feed-forward: queries from the image's
   * positions, keys and values from a context of `seq` tokens of width d_model per image, which is bound
   * like a weight ("context", [batch * seq, d_model]: a whole input every segment of that image reads).
   * A layer's weights are then the nine tensors of the residual block followed by those of the attention
   * block: eighteen, plus seven with a context (names and shapes from ac_plan_weight_info). */
  int32_t img_h, img_w, channels, groups;
} ac_model_desc;

typedef struct ac_region_desc {
  int32_t kind;          /* ac_region_kind */
  int32_t chunk_dim;     /* AC_DIM_* of the workload */
  int64_t chunk_len;     /* extent of one segment along chunk_dim ("rows per segment");
                            n = ceil(extent / chunk_len), the last segment may be short.
                            0 = largest length whose planned bytes fit the budget. */
} ac_region_desc;

typedef struct ac_region_info {
  int32_t kind, chunk_dim;
  int64_t extent;            /* size of the chunk dim */
  int64_t chunk_len;         /* chosen rows per segment */
  int64_t n_segments;        /* the paper's n */
  int64_t launches;          /* segment-loop iterations that launch kernels: n_segments, except that the fused
                                attention, which keeps nothing of a segment in memory, runs consecutive
                                segments in one launch where that needs no more workspace than the plan's */
  uint64_t model_bytes;      /* paper-style sum X + Y + A/n of this region, ops unfused */
  uint64_t model_bytes_unchunked; /* the same with n = 1 (first activation equation) */
} ac_region_info;

typedef struct ac_plan_info {
  uint64_t workspace_bytes;              /* arena the caller must pass to ac_execute */
  uint64_t io_bytes;                     /* mem(X) + mem(Y) of the whole stack */
  uint64_t peak_bytes_planned;           /* io_bytes + arena high-water mark */
  uint64_t peak_bytes_unchunked_planned; /* the same plan with one segment per region */
  uint64_t peak_bytes_model;             /* max over regions of model_bytes */
  uint64_t peak_bytes_model_unchunked;   /* max over regions of model_bytes_unchunked */
  uint64_t weight_bytes;                 /* sum of all weight tensors (not activation memory) */
  double flops_per_execute;              /* algorithmic flops: causal attention counts j <= i only */
  int32_t n_weights;                     /* device pointers ac_plan_bind_weights expects */
  int32_t n_regions;                     /* regions per layer / block */
  ac_region_info regions[AC_REGION_KINDS];
} ac_plan_info;

typedef struct ac_weight_info {
  char name[48];         /* e.g. "L0.w_qkv", "tmo.w_ap" */
  int64_t rows, cols;    /* [out, in] for matrices; rows = 1 for vectors */
  int32_t dtype;         /* ac_dtype */
  int32_t index;
} ac_weight_info;

typedef struct ac_kernel_stat {
  char name[32];         /* kernel class: "gemm", "attention", "layernorm", "elementwise", "trimul" */
  int64_t launches;
  double total_ms;       /* sum of HIP-event durations of those launches */
  double flops;          /* algorithmic flops of those launches */
  double bytes;          /* algorithmic HBM bytes (each operand read once, result written once) */
} ac_kernel_stat;

typedef struct ac_plan ac_plan;

/*
 * Build a chunk plan (host only; touches no device).  Section 3.1/3.2: regions, their
 * chunk settings, and a memory budget in; a plan out.  `regions` lists at most one entry
 * per region kind of the workload; a kind not listed runs as one segment.  The same
 * settings apply to every layer.  `act_budget_bytes` (0 = none) is the paper's memory_budget
 * (section 3.2): it bounds the activation memory this executor really needs, mem(X) + mem(Y) +
 * the workspace's high-water mark (peak_bytes_planned).  Every region whose chunk_len is 0 gets
 * the largest length (its extent, else a multiple of 128 rows for bf16 / 64 for fp32 / 1 for
 * batch elements and pair rows) at which its own peak fits; regions with an explicit length are
 * checked (AC_ERR_BUDGET_INFEASIBLE).  With AC_FLAG_BUDGET_PAPER_MODEL the paper-style bytes of
 * every region are bounded as well.
 * Errors: AC_ERR_ARG, AC_ERR_ILLEGAL_CHUNK_DIM, AC_ERR_UNSUPPORTED, AC_ERR_BUDGET_INFEASIBLE.
 * On success *out owns host memory only; release it with ac_plan_destroy.
 */
int ac_plan_create(const ac_model_desc* model, const ac_region_desc* regions, int n_regions,
                   uint64_t act_budget_bytes, ac_plan** out);

/* Sizes and byte counts of a plan (host only).  `out` is host memory of the caller.  The byte
 * counts are those of section 2.1 / 2.2: mem(X) + mem(Y) + mem(A) for one segment per region,
 * mem(X) + mem(Y) + mem(A)/n for the plan, once as this executor holds them and once as the
 * unfused graph of the paper's model would. */
int ac_plan_query(const ac_plan* plan, ac_plan_info* out);

/* Name, shape and dtype of weight tensor `index` (0 <= index < n_weights), in bind order. */
int ac_plan_weight_info(const ac_plan* plan, int index, ac_weight_info* out);

/*
 * Hand the plan the device addresses of its weights, in ac_plan_weight_info order (section 3.1:
 * the weights are non-chunkable inputs X^nc, seen whole by every segment).  The pointers stay
 * owned by the caller and must outlive every ac_execute of this plan.  Each must be 256-byte
 * aligned (AC_ERR_ALIGN); n_ptrs must equal n_weights (AC_ERR_ARG).  This is the first call of a
 * plan that touches the device: a plan with AC_FLAG_TWO_SEGMENTS_IN_FLIGHT creates its second
 * stream here (AC_ERR_HIP if that fails), so that ac_execute creates nothing.
 */
int ac_plan_bind_weights(ac_plan* plan, const void* const* dev_ptrs, int n_ptrs);

/*
 * Run the plan (section 2.2; section 3.2 "runtime pass"): for each layer, for each region,
 * for each segment in order, compute the segment's slice of the region output.  Enqueues
 * kernels on `stream` and returns without waiting.  x_dev [tokens, d_model] (or
 * [n_res, n_res, c_z]) is only read; y_dev has the same shape and must not overlap x_dev;
 * workspace_dev is scratch of at least workspace_bytes (else AC_ERR_WORKSPACE, nothing
 * launched).  All three must be 256-byte aligned.  *measured_peak_bytes (host, may be NULL)
 * receives io_bytes + the highest workspace offset actually handed to a kernel during
 * this call, which the host tracks while binding buffers (no device round trip).
 */
int ac_execute(ac_plan* plan, const void* x_dev, void* y_dev, void* workspace_dev,
               uint64_t workspace_bytes, void* stream, uint64_t* measured_peak_bytes);

/* Free the plan's host memory, its second stream and its events, if any (the plan of section
 * 3.2 holds no device memory).  NULL is allowed. */
void ac_plan_destroy(ac_plan* plan);

/*
 * Per-kernel-class timing with HIP events on the execute stream.  While enabled, every
 * kernel launch of ac_execute is bracketed by two events.  ac_plan_read_profile waits for
 * the recorded events (hipEventSynchronize), accumulates into at most `max_stats` entries
 * of `out` (host), stores the count in *n_out and clears the record.
 */
int ac_plan_set_profiling(ac_plan* plan, int enabled);
int ac_plan_read_profile(ac_plan* plan, ac_kernel_stat* out, int max_stats, int* n_out);

const char* ac_status_string(int status);
const char* ac_last_error(void);   /* thread-local; valid until the thread's next failing call */

/* ------------------------------------------------------------------------------------
 * The kernels of the path, callable one at a time (what a region runs on one segment).
 * All pointers are device pointers, 16-byte aligned, with row strides (ld*, in elements)
 * that are multiples of 8 (bf16) or 4 (fp32).  They enqueue on `stream` and return.
 * ------------------------------------------------------------------------------------ */

/* y[r,:] = (x[r,:] - mean) / sqrt(var + eps) * gain + shift over `cols`; biased variance. */
int ac_op_layernorm(const void* x, int64_t ldx, const void* gain, const void* shift, void* y,
                    int64_t ldy, int64_t rows, int64_t cols, float eps, int dtype, void* stream);

/*
 * r[m,n] = epilogue(sum_k a[m,k] * w[n,k]): + bias[n] (if bias), activation (ac_activation),
 * * mul[m,n] (if mul), + residual[m,n] (if residual), in that order, rounded once on store.
 * Columns n < n_split are stored row-major, out[m * ldo + n].  Columns n >= n_split (only
 * if out_t != NULL; otherwise every column is row-major) are stored strided:
 *   out_t[(m / t_period) * t_s1 + (m % t_period) * t_s2 + (n - n_split) * t_s3],
 * which writes a transposed or channel-major copy without a separate pass (t_period <= 0
 * means "no period": the offset is m * t_s2 + (n - n_split) * t_s3).
 */
int ac_op_linear(const void* a, int64_t lda, const void* w, int64_t ldw, const void* bias,
                 const void* mul, int64_t ldmul, const void* residual, int64_t ldr,
                 void* out, int64_t ldo,
                 void* out_t, int64_t n_split, int64_t t_period, int64_t t_s1, int64_t t_s2,
                 int64_t t_s3, int64_t m, int64_t n, int64_t k, int activation, int dtype,
                 void* stream);

/*
 * LayerNorm of `rows` short rows (k = 64 or 128 columns, bf16) followed by up to 5 projections of
 * the normalised rows t = LN(x), in one kernel: t never reaches memory.  The pair-stack modules
 * project each LayerNorm output several times (gated operands a and b of the triangle update;
 * q, k, v, gate and pair bias of the triangle attention; the transition's first layer); as separate
 * launches each would re-read t.  Part p computes
 *   plain:  out = activation(t w^T + bias)                      (w [n, k], bias [n] or NULL)
 *   gated:  out = sigmoid(t w_gate^T + bias_gate) * (t w^T + bias)   (the gate stays in registers)
 * and stores it either row-major, out[row_offset(m) + col] with row_offset(m) = m * ldo or, if
 * o_period > 0, (m / o_period) * o_s1 + (m % o_period) * o_s2 (rows regrouped on the way out), or,
 * if out_t != NULL, strided like ac_op_linear's second output:
 *   out_t[(m / t_period) * t_s1 + (m % t_period) * t_s2 + col * t_s3]   (t_period <= 0: no period).
 * n must be a multiple of 4.  Shapes outside these return AC_ERR_UNSUPPORTED (use ac_op_layernorm
 * and ac_op_linear).  A row's result does not depend on which launch or block computes it.
 */
typedef struct ac_proj_part {
  const void* w; const void* bias;
  const void* w_gate; const void* bias_gate;
  int32_t gated;            /* 1: gated pair */
  int32_t activation;       /* ac_activation of a plain part */
  int64_t n;
  void* out; int64_t ldo, o_period, o_s1, o_s2;
  void* out_t; int64_t t_period, t_s1, t_s2, t_s3;
} ac_proj_part;
int ac_op_ln_linear(const void* x, int64_t ldx, const void* gain, const void* shift, float eps,
                    int64_t rows, int64_t k, const ac_proj_part* parts, int n_parts, int dtype,
                    void* stream);

/*
 * Attention of `sq` query rows over `sk` keys, `heads` heads of `head_dim`, `batch`
 * independent problems: ctx = softmax(q k^T / sqrt(head_dim) + bias [causal mask]) v
 * [* gate].  q/k/v/ctx/gate rows of one problem are ld* apart, heads are contiguous
 * head_dim-wide column blocks, and problem b starts at b * stride_*_batch elements.
 * With v_transposed != 0 the values are read as v[(h * head_dim + d) * ldv + key] (the
 * layout the matrix-core kernel needs; ac_op_linear can write it with its strided store),
 * otherwise as v[key * ldv + h * head_dim + d] (served by a slower kernel).
 * Causal: query row r stands at position q_offset + r and sees keys j <= q_offset + r.
 * bias (may be NULL) points at the bias row of query row 0: bias[h * stride_bias_head +
 * r * ld_bias + key]; it is shared by all `batch` problems.
 * The scores never leave the chip.  n_splits / split_workspace: see below.
 */
int ac_op_attention(const void* q, int64_t ldq, int64_t stride_q_batch,
                    const void* k, int64_t ldk, int64_t stride_k_batch,
                    const void* v, int64_t ldv, int64_t stride_v_batch, int v_transposed,
                    const void* bias, int64_t ld_bias, int64_t stride_bias_head,
                    const void* gate, int64_t ldg, int64_t stride_g_batch,
                    void* ctx, int64_t ldc, int64_t stride_c_batch,
                    int64_t batch, int64_t sq, int64_t sk, int heads, int head_dim,
                    int causal, int64_t q_offset,
                    int n_splits, void* split_workspace, uint64_t split_workspace_bytes,
                    int dtype, void* stream);

/*
 * Key splits.  A launch with few query rows would leave most compute units idle, so the
 * keys each block of queries sees can be cut into n_splits runs that separate blocks
 * process; their fp32 partial results (unnormalised context, running maximum and sum) go to
 * split_workspace (device, 16-byte aligned, ac_attention_split_workspace_bytes large) and a
 * second kernel merges them.  n_splits <= 1 means one pass and no workspace; at most 16.  Results for
 * different n_splits agree to rounding, not bitwise.  ac_attention_key_splits is the count
 * the executor uses for a launch shape (1 when the launch already fills the GPU).
 */
int ac_attention_key_splits(int64_t sq, int64_t sk, int heads, int64_t batch, int head_dim,
                            int dtype, int v_transposed);
uint64_t ac_attention_split_workspace_bytes(int64_t sq, int heads, int64_t batch, int head_dim,
                                            int n_splits);

/*
 * ac_op_attention for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and result as ac_op_attention; the fp32 partial results of the key splits go to a
 * device array of ac_static_scratch_bytes() (64 MiB) that is part of the library's code object,
 * so every GPU the library runs on holds one until the process ends.  n_splits = 0 takes
 * ac_attention_key_splits' count, 1 uses no scratch at all.  A launch whose partial results
 * (ac_attention_split_workspace_bytes) exceed the array is refused with AC_ERR_WORKSPACE and
 * nothing is launched.  The call allocates and frees nothing; on its first use on a device it
 * looks up that device's address of the array (the device must be current).  All calls on one
 * GPU share the array: calls that overlap on one GPU (two streams, two threads) race on it;
 * calls on one stream are ordered and need no clearing in between.
 */
int ac_op_attention_static_scratch(const void* q, int64_t ldq, int64_t stride_q_batch,
                                   const void* k, int64_t ldk, int64_t stride_k_batch,
                                   const void* v, int64_t ldv, int64_t stride_v_batch, int v_transposed,
                                   const void* bias, int64_t ld_bias, int64_t stride_bias_head,
                                   const void* gate, int64_t ldg, int64_t stride_g_batch,
                                   void* ctx, int64_t ldc, int64_t stride_c_batch,
                                   int64_t batch, int64_t sq, int64_t sk, int heads, int head_dim,
                                   int causal, int64_t q_offset, int n_splits, int dtype, void* stream);
uint64_t ac_static_scratch_bytes(void);

/* y = activation(x + bias[col]) over [rows, cols]; bias may be NULL. */
int ac_op_bias_act(const void* x, int64_t ldx, const void* bias, void* y, int64_t ldy,
                   int64_t rows, int64_t cols, int activation, int dtype, void* stream);

/* y = a + b  (op 0)  or  y = a * b  (op 1) over [rows, cols]. */
int ac_op_binary(const void* a, int64_t lda, const void* b, int64_t ldb, void* y, int64_t ldy,
                 int64_t rows, int64_t cols, int op, int dtype, void* stream);

/*
 * p = softmax(scale * s) over each of `rows` stored rows of `cols` scores (AutoChunk section
 * 2.1 names the scores and probabilities of attention as the intermediate activations that
 * dominate memory; this is the pass between them when they are stored).  Row r belongs to
 * query r mod period, which stands at position q_offset + (r mod period); with causal != 0
 * it sees columns j <= that position and the others get probability exactly 0.  s and p may
 * be the same buffer.  scale > 0.
 */
int ac_op_softmax_rows(const void* s, int64_t lds, void* p, int64_t ldp, int64_t rows, int64_t cols,
                       float scale, int causal, int64_t q_offset, int64_t period, int dtype,
                       void* stream);

/* dst[c * ldd + r] = src[r * lds + c] for a [rows, cols] matrix (e.g. values -> v_transposed). */
int ac_op_transpose(const void* src, int64_t lds, void* dst, int64_t ldd, int64_t rows,
                    int64_t cols, int dtype, void* stream);

/*
 * Triangle contraction on `ni` output rows, one product per channel c:
 *   out_c[c][i][j] = sum_k a_t[c][i][k] * b_t[c][j][k]
 * with a_t[c * stride_a_c + i * lda + k], b_t[c * stride_b_c + j * ldb + k] and
 * out_c[c * stride_o_c + i * ldo + j].  The outgoing form of the triangle multiplicative
 * update has a_t[c][i][k] = a[i,k,c]; the incoming form a_t[c][i][k] = a[k,i,c] (both operands
 * are held channel-major with the contraction index contiguous, which ac_op_linear's strided
 * store writes; ac_op_transpose_square_inplace turns one form into the other).
 */
int ac_op_triangle_contract(const void* a_t, int64_t lda, int64_t stride_a_c,
                            const void* b_t, int64_t ldb, int64_t stride_b_c,
                            void* out_c, int64_t ldo, int64_t stride_o_c,
                            int64_t ni, int64_t nj, int64_t nk, int channels, int dtype, void* stream);

/* In-place transpose of `batch` square [n, n] matrices (row stride ld, stride_batch apart). */
int ac_op_transpose_square_inplace(void* data, int64_t ld, int64_t stride_batch, int64_t n,
                                   int64_t batch, int dtype, void* stream);

/*
 * LayerNorm over the channels of a channel-major tensor, written position-major:
 * dst[p * ldd + c] = LN_c(src[c * stride_c + p]) * gain[c] + shift[c]  (what follows the
 * triangle contraction, whose output is channel-major).
 */
int ac_op_layernorm_channel_major(const void* src, int64_t stride_c, const void* gain,
                                  const void* shift, void* dst, int64_t ldd, int64_t positions,
                                  int64_t channels, float eps, int dtype, void* stream);

/*
 * GroupNorm of channels-last images x [images, positions, channels] (the UNet residual block's
 * normalisation; AutoChunk section 4 evaluates that family): per image and per run of
 * channels / groups consecutive channels, mean and biased variance over the run's channels and all
 * positions; y = act((x - mean) / sqrt(var + eps) * gain[c] + shift[c]), act = AC_ACT_NONE or
 * AC_ACT_SILU.  workspace: ac_group_norm_workspace_bytes(images, groups) bytes of device memory
 * (partial statistics), caller's.  channels a multiple of groups and of 8 (bf16) / 4 (fp32),
 * groups <= 128, images <= 65535, else AC_ERR_ARG.
 */
uint64_t ac_group_norm_workspace_bytes(int64_t images, int groups);
int ac_op_group_norm(const void* x, const void* gain, const void* shift, void* y, void* workspace,
                     uint64_t workspace_bytes, int64_t images, int64_t positions, int channels, int groups,
                     float eps, int activation, int dtype, void* stream);

/*
 * 3x3 convolution, stride 1, zero padding 1, of channels-last bf16 images:
 * out[b,h,w,o] = sum_{kh,kw,i} x[b,h+kh-1,w+kw-1,i] * weight[o,kh,kw,i] + bias[b or 0][o] (+ residual[b,h,w,o]).
 * x [images, height, width, c_in], weight [c_out, 3, 3, c_in], out and residual [images, height, width, c_out].
 * bias: one vector [c_out] (bias_per_image = 0) or one per image [images, c_out] (the block's
 * bias plus the image's time embedding), may be null.  c_in a multiple of 64, c_out of 8; images * height * width
 * below 2^31; else AC_ERR_ARG / AC_ERR_UNSUPPORTED.
 */
int ac_op_conv3x3(const void* x, const void* weight, const void* bias, int bias_per_image, const void* residual,
                  void* out, int64_t images, int height, int width, int c_in, int c_out, int dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AUTOCHUNK_RT_H */
