/*
 * turnip.h -- C ABI of the single-GPU memgraph runtime (gfx950 / MI355X).
 *
 * The calls follow the paper's statement of the problem:
 *   taskgraph in (Section 4, first paragraph: a dataflow DAG whose input vertices hold tensors
 *   and whose other vertices are kernel calls)
 *     -> BuildMemgraph (Section 6, Algorithms 1 and 2: fixed GPU location per vertex output,
 *        memory dependencies, inserted offload/reload vertices, for a given serial order V
 *        and a given amount of GPU memory)
 *     -> execution by an event loop that launches any vertex whose dependencies have completed
 *        and for which a stream is free, with no allocation calls while it runs (Section 5 and
 *        Appendix A).
 *
 * Conventions
 *   - Every function returns a tn_status (0 = TN_OK, negative = error) unless stated.  No
 *     exception and no abort crosses this boundary.  tn_last_error() returns a thread-local,
 *     NUL-terminated description of the most recent error on the calling thread.
 *   - "host" pointers are CPU memory, "device" pointers are GPU memory of the current HIP
 *     device.  The library never frees or reallocates caller memory.
 *   - Objects returned through an out-parameter belong to the caller and are released with the
 *     matching *_destroy.  A memgraph owns a copy of everything it needs from the taskgraph, so
 *     the taskgraph may be destroyed after tn_compile.  A memgraph must outlive its executors.
 *   - All tensors are dense row-major 2-D tiles [rows, cols] of fp32 or bf16 elements, each
 *     stored contiguously (leading dimension = cols).
 */
#ifndef TURNIP_H
#define TURNIP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tn_status;
typedef int32_t tn_vid; /* taskgraph vertex id, dense from 0 in insertion order */

enum {
  TN_OK = 0,
  TN_ERR_INVALID = -1,         /* bad argument, bad handle, call out of sequence */
  TN_ERR_NOT_TOPOLOGICAL = -2, /* the given serial order violates a dataflow edge */
  TN_ERR_CYCLE = -3,           /* the graph has a cycle */
  TN_ERR_CAP_TOO_SMALL = -4,   /* some vertex's inputs and output cannot be co-resident */
  TN_ERR_ARENA = -5,           /* pinned host arena exhausted */
  TN_ERR_HIP = -6,             /* a HIP call failed; the executor is poisoned afterwards */
  TN_ERR_SHAPE = -7            /* operand shapes or types do not fit the vertex kind */
};

const char* tn_last_error(void);

typedef struct tn_taskgraph tn_taskgraph;
typedef struct tn_memgraph tn_memgraph;
typedef struct tn_executor tn_executor;

enum { TN_F32 = 0, TN_BF16 = 1 };    /* element type of a tensor */
enum { TN_HOST = 0, TN_DEVICE = 1 }; /* where an input tensor lies when execution starts */

/* Vertex kinds of a taskgraph.  Each is a pure function of its operands with a fixed summation
 * order, so that every dependency-respecting execution order produces the same bits
 * (Introduction, fourth paragraph: the output is correct no matter the execution order). */
enum {
  TN_OP_INPUT = 0,        /* ()                       -> the tensor itself                        */
  TN_OP_GEMM = 1,         /* A_0..A_{nk-1}, B_0..B_{nk-1}[, ...] -> sum_k A_k B_k, k ascending, fp32 acc (+ mode) */
  TN_OP_RMS_STAT = 2,     /* X_0..X_{n-1} (one row block) -> fp32 [rows,1]: rsqrt(sum x^2 / d + eps) */
  TN_OP_RMS_APPLY = 3,    /* X, stat[rows,1] fp32, gain[1,cols] -> x * stat * gain                 */
  TN_OP_ROPE = 4,         /* X -> rotary embedding of interleaved pairs (2i, 2i+1)                 */
  TN_OP_ATTN_BLOCK = 5,   /* Q tiles, K tiles, V tiles -> fp32 partial [rows, gw + 2*hpg]          */
  TN_OP_ATTN_COMBINE = 6, /* partial_0..partial_j -> normalised attention output tile              */
  TN_OP_SILU_MUL = 7,     /* gate, up -> gate / (1 + exp(-gate)) * up                              */
  TN_OP_ADD = 8,          /* a, b -> a + b                                                          */
  /* reverse-mode counterparts, for the fine-tuning workload (Section 8, item 2) */
  TN_OP_SILU_MUL_BWD = 9,   /* dact, gate, up -> gradient of gate (mode 0) or of up (mode 1)         */
  TN_OP_RMS_BWD_STAT = 10,  /* dy tiles, x tiles, gain tiles of a row block -> fp32 [rows,1]: sum dy*gain*x */
  TN_OP_RMS_BWD_APPLY = 11, /* dy, x, stat, dot, gain[, residual gradient] -> gradient of x            */
  TN_OP_ATTN_BWD = 12,      /* Q, K, V, dO tiles[, statistics][, transposed tiles] -> statistics, dQ, dK or dV (mode) */
  TN_OP_TRANSPOSE = 13,     /* X [rows, cols] -> X^T [cols, rows]                                      */
  /* Appendix A (resources): a sum of n tensors is run as n increment kernels into an output
   * protected by a write lock.  P_0..P_{n-1}, all of the output's shape and type -> their sum.  In
   * the memgraph the vertex becomes TN_OP_ZERO, one TN_OP_SUM_INTO per operand and TN_MG_JOIN; the
   * increments run in whatever order their operands arrive, and each rounds the output to its
   * storage type, so the result is order-independent only up to that rounding. */
  TN_OP_SUM = 14,
  TN_OP_ZERO = 15,          /* memgraph only: () -> zeros, the start of a sum's output               */
  TN_OP_SUM_INTO = 16,      /* memgraph only: P, accumulator -> accumulator += P, in place           */
  /* Softmax "in portions" over materialised attention scores (Introduction, second paragraph;
   * Appendix A, hand-written kernels): the score tiles S_0..S_{n-1} of one row block, left to right
   * -> fp32 [rows, 2]: per row the maximum m of scale * s over the visible entries, then
   * l = sum exp(scale * s - m) over them.  Entry (r, c), c counted across the tiles, is visible
   * unless causal != 0 and k_pos0 + c > q_pos0 + r. */
  TN_OP_SOFTMAX_STAT = 17,
  /* S, the SOFTMAX_STAT of its row block -> exp(scale * s - m) / l where visible, else 0;
   * k_pos0 is the position of this tile's first column. */
  TN_OP_SOFTMAX_APPLY = 18
};

typedef struct {
  int32_t dtype; /* TN_F32 or TN_BF16 */
  int32_t rows;
  int32_t cols;
} tn_tensor_desc;

/* Parameters of a vertex; fields a kind does not use are ignored.
 *   GEMM         nk, trans_b            number of k tiles; operands are A_0..A_{nk-1} then B_0..B_{nk-1};
 *                                       A_k is [rows, K_k]; B_k is [K_k, cols], or, with trans_b != 0,
 *                                       stored transposed as [cols, K_k] (the usual [out, in] layout
 *                                       of linear-layer weights, which the MFMA kernel reads directly).
 *                                       trans_c != 0: the output tensor holds the product transposed,
 *                                       [cols, rows] of the logical [rows, cols] result
 *   RMS_STAT     d, eps                 d = total number of columns of the row block
 *   ROPE         pos0, col0, head_dim, rope_base
 *                                       row r has position pos0 + r; column c belongs to pair
 *                                       ((col0 + c) mod head_dim) / 2; pair i turns by
 *                                       position * rope_base^(-2i/head_dim)
 *   ATTN_BLOCK   n_q_tiles, n_kv_tiles, n_col_tiles, head_dim, q_pos0, k_pos0, causal, scale
 *                                       operands: Q tiles row-major over (row tile, column tile),
 *                                       then K tiles, then V tiles.  gw = total columns = hpg *
 *                                       head_dim.  Output row: gw unnormalised sums of
 *                                       exp(s - m) v, then hpg row maxima m, then hpg sums l.
 *                                       causal != 0 excludes keys with k_pos0 + c > q_pos0 + r.
 *                                       v_trans != 0: the V operands are tiles of V^T, each
 *                                       [columns of the tile, key rows of the tile]
 *   ATTN_COMBINE row0, col0, head_dim, hpg
 *                                       output tile = rows [row0, row0 + rows) and columns
 *                                       [col0, col0 + cols) of the merged, normalised block.
 *   GEMM         trans_a                != 0: A_k is stored transposed, [K_k, rows]
 *   GEMM         mode                   1: one more operand follows the B tiles, R of the output's shape and
 *                                       type; the result is sum_k A_k B_k + R, added in fp32 before the one
 *                                       rounding.  2: nk more operands follow the B tiles, U_0..U_{nk-1}
 *                                       shaped like them; with gate = sum_k A_k B_k and up = sum_k A_k U_k
 *                                       (both fp32) the result is gate / (1 + exp(-gate)) * up.  Both need
 *                                       trans_a == 0 and trans_c == 0.
 *   ROPE         mode                   != 0: the inverse rotation (which is also the rotation's gradient)
 *   SILU_MUL_BWD mode                   with s = 1/(1 + exp(-gate)): mode 0 -> dact * up * s * (1 + gate * (1 - s)),
 *                                       mode 1 -> dact * gate * s
 *   RMS_BWD_STAT nk                     operands: nk tiles of dy, then the nk tiles of x, then the nk gain tiles
 *   RMS_BWD_APPLY d                     stat = the forward RMS_STAT of x, dot = RMS_BWD_STAT; result
 *                                       stat * gain * dy - x * stat^3 * dot / d, plus the sixth operand if given
 *   ATTN_BWD     mode, n_q_tiles, n_kv_tiles, n_col_tiles, head_dim, q_pos0, k_pos0, causal, scale, v_trans
 *                                       operands: Q, K, V tiles as for ATTN_BLOCK, then the dO tiles (like Q), then,
 *                                       except in mode 0, one statistics tensor per Q row tile.  With
 *                                       p = exp(scale q.k - lse), dp = dO.v:
 *                                       mode 0 -> fp32 [q rows, 2*hpg]: per head lse = log sum_k exp(scale q.k)
 *                                                 over the visible keys, then D = sum_k p dp;
 *                                       mode 1 -> dQ [q rows, gw] = scale * sum_k p (dp - D) k;
 *                                       mode 2 -> dK [kv rows, gw] = scale * sum_q p (dp - D) q;
 *                                       mode 3 -> dV [kv rows, gw] = sum_q p dO.
 *                                       Sums run over keys (queries) in ascending order.
 *                                       trans_a != 0 (modes 1..3, needs v_trans == 0): one more grid of operands
 *                                       follows, the transposes the matrix units want as row-major tiles:
 *                                       mode 1 -> K^T tiles, mode 2 -> Q^T tiles, mode 3 -> dO^T tiles, each
 *                                       [columns of the tile, rows of the tile], in the order of the grid
 *                                       they mirror. */
typedef struct {
  int32_t nk;
  int32_t d;
  float eps;
  int32_t pos0;
  int32_t col0;
  int32_t head_dim;
  float rope_base;
  int32_t n_q_tiles;
  int32_t n_kv_tiles;
  int32_t n_col_tiles;
  int32_t q_pos0;
  int32_t k_pos0;
  int32_t causal;
  float scale;
  int32_t row0;
  int32_t hpg;
  int32_t trans_b;
  int32_t trans_c;
  int32_t v_trans;
  int32_t trans_a;
  int32_t mode;
} tn_op_params;

/* ------------------------------------------------------------------------------------------ */
/* Taskgraph (host only)                                                                       */
/* ------------------------------------------------------------------------------------------ */

tn_status tn_taskgraph_create(tn_taskgraph** out);
void tn_taskgraph_destroy(tn_taskgraph* tg);

/* Adds an input vertex (Section 4: a vertex without inputs is associated with an input tensor).
 * residency TN_DEVICE: the tensor is in GPU memory at its compiled location before execution
 * starts, as in the paper's examples; TN_HOST: it is copied from the caller's host buffer by a
 * load vertex when the memgraph says so. */
tn_status tn_taskgraph_add_input(tn_taskgraph* tg, const tn_tensor_desc* desc, int32_t residency,
                                 tn_vid* out);

/* Adds a kernel-call vertex reading the outputs of `inputs` (operand order matters).  Operand
 * shapes and types are validated against the kind: TN_ERR_SHAPE on mismatch. */
tn_status tn_taskgraph_add_op(tn_taskgraph* tg, int32_t kind, const tn_op_params* params,
                              const tn_vid* inputs, int32_t n_inputs, const tn_tensor_desc* out_desc,
                              tn_vid* out);

/* Marks a vertex whose tensor the caller wants back.  Output index = order of marking. */
tn_status tn_taskgraph_mark_output(tn_taskgraph* tg, tn_vid v);

typedef struct {
  int32_t kind;
  int32_t residency; /* inputs only */
  int32_t n_inputs;
  int32_t output_index; /* -1 if not a marked output */
  tn_tensor_desc desc;
  tn_op_params params;
} tn_tg_vertex;

int64_t tn_taskgraph_num_vertices(const tn_taskgraph* tg);
int64_t tn_taskgraph_num_outputs(const tn_taskgraph* tg);
tn_status tn_taskgraph_vertex(const tn_taskgraph* tg, tn_vid v, tn_tg_vertex* out);
/* Copies up to cap operand ids of v into out; returns the operand count (or a negative status). */
int32_t tn_taskgraph_inputs(const tn_taskgraph* tg, tn_vid v, tn_vid* out, int32_t cap);

/* A serial order V for tn_compile that runs the graph level by level (Section 6 takes V as given;
 * Section 8, item 3 shows how much the choice matters to an executor that must follow it): the
 * level of a kernel vertex is one more than the highest level among its operands that are kernel
 * vertices (1 if it reads inputs only); an input comes just before the first level that reads it;
 * vertices of one level keep their numbering.  Vertices of one kind end up next to each other, so
 * launches can be grouped, and every weight tile of a layer is loaded once per pass instead of once
 * per row stripe.  out receives all vertex ids; cap = room in out, at least the vertex count. */
tn_status tn_taskgraph_level_order(const tn_taskgraph* tg, tn_vid* out, int64_t cap);

/* A serial order V for caps far below the working set (Section 6 takes V as given and notes that the
 * quality of the memgraph depends on it): level by level as above, with two changes that keep the live
 * set small.  (1) A kernel vertex whose kernel operands all lie one level below it and are read by
 * nothing but vertices with the very same operand list (the combine of attention partials, the product
 * of the two gated projections, a sum of partial products, a rotation of a projection) is placed, with
 * those vertices, right after its operands, and the operands of one such group are placed together:
 * the operands die at once instead of waiting for the whole level.  (2) Within a level, vertices and
 * such groups are ordered by the first input they read, then by their numbering, so that everything
 * that reads one weight tile is adjacent and the tile is needed for one stretch of the order only.  An
 * input comes right before its first reader.  out receives all vertex ids; cap as above. */
tn_status tn_taskgraph_clustered_order(const tn_taskgraph* tg, tn_vid* out, int64_t cap);

/* A tiled LLaMA-style decoder forward pass as a taskgraph (the paper's workload, Section 8;
 * the decomposition into tiles is this library's, since the paper leaves taskgraph production
 * to an outside framework, Section 4 second paragraph). */
typedef struct {
  int32_t layers, d_model, n_heads, head_dim, ffn, seq, batch;
  int32_t dtype;      /* storage type of activations and weights */
  int32_t tile;       /* edge of a GEMM / elementwise tile */
  int32_t attn_block; /* edge of an attention block, a multiple of tile */
  float eps;
  float rope_base;
  int32_t weights_residency; /* TN_HOST (streamed) or TN_DEVICE (pre-placed) */
  int32_t x_residency;
  int32_t kv_outputs; /* != 0: post-rotary K and V tiles of every layer are marked outputs too */
  int32_t weights_transposed; /* != 0: weight tiles are stored [out, in] and GEMMs use trans_b */
  int32_t v_transposed;       /* != 0: the V projection stores V^T tiles (trans_c) and attention reads them (v_trans) */
  /* Fine-tuning workload (Section 8, item 2): low-rank adapters on the query and value
   * projections, q = a Wq + (a Aq) Bq and v = a Wv + (a Av) Bv with Aq, Av [d_model, lora_rank] and
   * Bq, Bv [lora_rank, d_model]; 0 = no adapters. */
  int32_t lora_rank;
  /* != 0 (needs lora_rank > 0 and max(tile, head_dim) == tile): after the forward pass, the reverse pass for
   * the loss sum(y * probe) through the frozen base weights; outputs, besides y: the gradients of the adapter
   * matrices of every layer and of x.  The reverse pass reads the base weights as [in, out] tiles (bindings
   * with transposed == 0), which are input vertices of their own when weights_transposed != 0. */
  int32_t train;
  /* > 1: every projection of the forward pass is cut along K into k_split partial products
   * (contiguous runs of ceil(nk / k_split) K tiles, one GEMM vertex each) joined by a TN_OP_SUM
   * vertex -- the k-split + sum-into form of a matrix product (Appendix A, resources).  0 or 1:
   * the whole K range inside one GEMM vertex. */
  int32_t k_split;
  /* != 0 (needs tile == head_dim, so that a column tile is one head, and train == 0): attention
   * with scores and probabilities as tensors of the taskgraph -- per head and pair of row tiles
   * (i, j <= i) a GEMM S = Q_i K_j^T, per head and row tile a SOFTMAX_STAT over S_i0..S_ii, a
   * SOFTMAX_APPLY per score tile, and O_i = sum_j P_ij V_j as one GEMM -- instead of the fused
   * ATTN_BLOCK / ATTN_COMBINE vertices.  attn_block is ignored. */
  int32_t materialize_scores;
  /* != 0 (needs train != 0): activation checkpointing, the setting of the paper's fine-tuning
   * experiment (Section 8).  The forward pass keeps only each layer's input for the reverse pass;
   * the reverse pass of a layer is preceded by that layer's forward vertices over again (all but
   * the second half of the feed-forward block, which nothing reads), as vertices of their own.
   * Results are bit for bit those of train without it. */
  int32_t checkpoint;
  /* != 0: the hidden state after every layer but the last (whose output is y) is a marked output
   * too, bound as TN_T_H of that layer: what a check layer by layer, or a probe, reads. */
  int32_t hidden_outputs;
  /* n > 1: kv_outputs and hidden_outputs apply only to the layers l with l mod n == 0 or n - 1, and to
   * the last two layers -- pairs of neighbouring layers through the depth of the stack, so that
   * a layer's input and output can both be read back without storing every layer.  0 or 1: all. */
  int32_t output_layer_stride;
  /* > 0 (needs batch == 1, train == 0, materialize_scores == 0): after the prefill of `seq` positions,
   * this many decode steps, fixed beforehand (Section 9, limitations: a memgraph compiled for a given
   * number of generated tokens).  Step u runs the single row at position seq + u through all layers
   * against the cached keys and values: the prefill's tiles, plus one single-row tile per generated
   * position, so the attention block over the generated positions grows by a tile per step.  The
   * row's embedding is an input, bound as row seq + u of x (there is no vocabulary to sample from);
   * its result is row seq + u of y.  kv_outputs / hidden_outputs cover the decode rows too. */
  int32_t decode_steps;
  /* != 0 (needs train == 0, materialize_scores == 0): attention of a query block as ONE vertex over all
   * keys from position 0 to the block's own end, instead of one vertex per key block of attn_block
   * positions (the tiling is the front end's choice, Section 4; the blocks remain what the kernel walks
   * through).  The online softmax then runs over the whole range inside the kernel and a query block
   * has a single partial, which the combine vertex normalises: s + 1 times less partial traffic for the
   * block in stripe s, at the price that all earlier K/V tiles of the layer are operands of one vertex
   * and must be resident together. */
  int32_t attn_whole_rows;
  /* with checkpoint != 0: only the first this many layers are checkpointed (their forward tensors are formed
   * again in the reverse pass), the later layers keep their saved activations; 0 = every layer.  The first
   * layers are the ones whose saved activations would wait longest for the reverse pass, i.e. the ones a cap
   * pushes to the host: recomputing those and saving the rest trades a little arithmetic for all of the
   * offload traffic when the rest fits. */
  int32_t checkpoint_layers;
  /* bits (need train == 0 and k_split <= 1; which steps of a layer share a vertex is the front end's
   * choice, Section 4): 1 -- the two residual additions of a layer become the last operand of the products
   * before them (GEMM, mode 1), so the projection's own output tile is never stored; 2 -- the W1 and W3
   * products and silu(gate) * up become one vertex (GEMM, mode 2), so the two [rows, ffn] intermediates
   * never exist.  A fused vertex rounds to the storage type once. */
  int32_t fuse_epilogues;
  /* != 0 (needs train != 0): the normalised layer input, which the adapter gradients read, is not kept from
   * the forward pass; the reverse pass forms it again from the layer input and its statistic, which it keeps
   * anyway (one elementwise vertex per tile, the same bits).  One [tokens, d_model] tensor per layer less to
   * hold, or to offload under a cap. */
  int32_t recompute_normed;
  /* != 0 (needs train != 0): the gate and up products of the feed-forward block, which the reverse pass of
   * SiLU*mul reads, are not kept from the forward pass; the reverse pass forms them again from h1 (normalised
   * again from h1 and its statistic, then the two products: the same kernels on the same operands, the same
   * bits).  These are the two largest saved tensors of a layer ([tokens, ffn] each): forming them again costs
   * two products per layer and the W1 and W3 tiles a second time, keeping them under a cap costs their way to
   * the host and back.  Layers that are checkpointed as a whole are not affected. */
  int32_t recompute_gate_up;
} tn_llama_config;

/* Which vertex is which piece of which tensor of the decoder. */
enum {
  TN_T_X = 0, TN_T_WQ, TN_T_WK, TN_T_WV, TN_T_WO, TN_T_W1, TN_T_W3, TN_T_W2, TN_T_G1, TN_T_G2,
  TN_T_Y, TN_T_K, TN_T_V,
  TN_T_AQ, TN_T_BQ, TN_T_AV, TN_T_BV, TN_T_PROBE,          /* adapter matrices and the probe (inputs)      */
  TN_T_DAQ, TN_T_DBQ, TN_T_DAV, TN_T_DBV, TN_T_DX,           /* their gradients and that of x (outputs)      */
  TN_T_H                                                     /* hidden state after a layer (hidden_outputs)  */
};
typedef struct {
  tn_vid vid;
  int32_t tensor; /* TN_T_* */
  int32_t layer;  /* -1 for x and y */
  int32_t row0, row1, col0, col1; /* the slice [row0,row1) x [col0,col1) of the full tensor */
  int32_t transposed; /* != 0: the vertex holds the slice transposed, [col1-col0, row1-row0] */
} tn_llama_binding;

tn_status tn_build_llama(const tn_llama_config* cfg, tn_taskgraph** out);
int64_t tn_taskgraph_num_bindings(const tn_taskgraph* tg);
tn_status tn_taskgraph_binding(const tn_taskgraph* tg, int64_t i, tn_llama_binding* out);

/* ------------------------------------------------------------------------------------------ */
/* Compile: BuildMemgraph (host only)                                                          */
/* ------------------------------------------------------------------------------------------ */

typedef struct {
  /* Run-ahead of the allocation horizon past the execution horizon (Section 6, third
   * paragraph), in bytes of not-yet-produced outputs; UINT64_MAX = greedy as in Algorithm 1,
   * 0 = allocate a vertex only when it is about to run. */
  uint64_t max_lookahead_bytes;
  /* != 0: an evicted input whose host copy is still valid is dropped instead of copied back
   * (no bytes move); its reload is a fresh load from the caller's buffer. */
  int32_t drop_clean_inputs;
  /* != 0: add dependencies that force kernels to run in the order V and transfers to run in
   * the order V (the partially deterministic variant of Section 8, item 3). */
  int32_t fix_order;
  /* != 0: leave out memory dependencies that duplicate a data dependency (Section 4 calls them
   * superfluous). */
  int32_t prune_superfluous;
  uint32_t alignment; /* location granularity in bytes, power of two; 0 = 256 */
  /* When room has to be made for a tensor, evict this many bytes more than it needs, taking the
   * resident tensors whose next use lies furthest ahead (and at least a few thousand vertices
   * ahead).  Algorithm 2 evicts exactly what one tensor needs, which under a tight cap turns the
   * run into a chain of evict-one, produce-one steps, each a round trip through the host; evicting
   * a batch lets the transfers of the batch, and then the kernels that take the freed places, go
   * together.  0 = as in Algorithm 2. */
  uint64_t evict_ahead_bytes;
  /* Where simMalloc looks for an open range (Algorithm 2 leaves it open).  0: first fit, the lowest
   * address, which packs memory tightly but hands a tensor the place that was vacated most recently
   * in that region, so that consecutive parts of the computation wait on each other's memory.
   * 1: next fit, the lowest address above the place given out last, wrapping round, so that a place
   * rests for as long as possible before it is used again. */
  int32_t next_fit;
} tn_compile_opts;

/* Compiles tg for gpu_cap_bytes of GPU memory.  order: a permutation of all vertex ids that
 * respects every edge, or NULL for insertion order with each TN_HOST input moved to just before
 * its first consumer.  TN_DEVICE inputs are placed first, in id order, whatever `order` says.
 * Errors: TN_ERR_NOT_TOPOLOGICAL, TN_ERR_CAP_TOO_SMALL (message names the vertex). */
tn_status tn_compile(const tn_taskgraph* tg, const tn_vid* order, uint64_t gpu_cap_bytes,
                     const tn_compile_opts* opts, tn_memgraph** out);
void tn_memgraph_destroy(tn_memgraph* mg);

/* Memgraph vertex kinds.  Vertices 0..n_task-1 are the taskgraph's, with the same ids. */
enum {
  TN_MG_INPUT = 0, /* TN_DEVICE input, in place before execution                     */
  TN_MG_LOAD = 1,  /* host -> GPU copy of a TN_HOST input (first load, or after a drop) */
  TN_MG_OP = 2,    /* kernel call                                                      */
  TN_MG_OFFLOAD = 3,
  TN_MG_RELOAD = 4,
  TN_MG_DROP = 5,  /* eviction without a copy                                          */
  TN_MG_STORE = 6, /* GPU -> host copy of a marked output into the caller's buffer     */
  /* A TN_OP_SUM vertex: TN_MG_OP vertices with op_kind TN_OP_ZERO (clears the output at its
   * location; the location's memory dependencies point at it) and TN_OP_SUM_INTO (one per operand;
   * operands: the tensor to add, then the TN_OP_ZERO vertex, whose location it updates in place and
   * whose offset it repeats; the executor runs at most one increment per location at a time) come
   * first; the sum vertex itself is the join: no work, runs after every increment (data edges),
   * operand: the TN_OP_ZERO vertex, and from then on stands for the tensor at that location. */
  TN_MG_JOIN = 7
};
enum { TN_EDGE_DATA = 0, TN_EDGE_MEM = 1, TN_EDGE_ORDER = 2 /* only with fix_order */ };

typedef struct {
  int32_t kind;       /* TN_MG_* */
  int32_t op_kind;    /* TN_OP_* for TN_MG_OP */
  tn_vid src;         /* taskgraph vertex whose tensor this vertex produces or moves */
  int64_t offset;     /* byte offset of its output in [0, cap), or -1 if it writes no GPU memory */
  uint64_t bytes;     /* size of the tensor */
  int32_t n_operands; /* memgraph vertices whose output it reads */
  int64_t order_pos;  /* position in the extended serial order (Section 7) */
} tn_mg_vertex;

typedef struct {
  int64_t from, to;
  int32_t kind; /* TN_EDGE_* */
} tn_mg_edge;

typedef struct {
  uint64_t cap;              /* as given */
  uint64_t high_water;       /* highest byte offset + size ever assigned */
  uint64_t peak_live_bytes;  /* peak of allocated bytes during the simulated serial run */
  uint64_t host_arena_bytes; /* sum of all offload sizes (aligned): a safe arena size */
  int64_t n_task, n_vertices, n_edges, n_mem_edges;
  int64_t n_offload, n_reload, n_drop, n_load, n_store;
  uint64_t offload_bytes, reload_bytes, load_bytes, store_bytes;
  int64_t n_revoked;     /* run-ahead allocations that had to be undone */
  int64_t n_compactions; /* times memory had to be emptied to defeat fragmentation */
  int64_t n_increment;   /* TN_OP_SUM_INTO vertices */
} tn_mg_stats;

int64_t tn_memgraph_num_vertices(const tn_memgraph* mg);
tn_status tn_memgraph_vertex(const tn_memgraph* mg, int64_t i, tn_mg_vertex* out);
int32_t tn_memgraph_operands(const tn_memgraph* mg, int64_t i, int64_t* out, int32_t cap);
int64_t tn_memgraph_num_edges(const tn_memgraph* mg);
tn_status tn_memgraph_edge(const tn_memgraph* mg, int64_t i, tn_mg_edge* out);
tn_status tn_memgraph_stats(const tn_memgraph* mg, tn_mg_stats* out);
/* Writes vertices, edges, locations and the extended order as JSON. */
tn_status tn_memgraph_dump_json(const tn_memgraph* mg, const char* path);
/* CPU dry run of `order` (n = number of memgraph vertices; NULL = the extended serial order):
 * checks that the order respects every edge, that no vertex writes over a tensor that still
 * has readers, and that every read finds the tensor it expects.  No arithmetic is done. */
tn_status tn_memgraph_simulate(const tn_memgraph* mg, const int64_t* order, int64_t n);

/* ------------------------------------------------------------------------------------------ */
/* Execute (GPU)                                                                               */
/* ------------------------------------------------------------------------------------------ */

/* IN_ORDER is the deterministic executor of the ablation in Section 8 (item 3): kernels are launched
 * strictly in the serial order the memgraph was compiled for, and so are the transfers of each
 * direction; a vertex whose turn has come but which is not ready holds back everything behind it. */
enum { TN_POLICY_FIFO = 0, TN_POLICY_LIFO = 1, TN_POLICY_RANDOM = 2, TN_POLICY_BY_ORDER = 3, TN_POLICY_IN_ORDER = 4 };
/* How transfers are carried out.  MEMCPY: one hipMemcpyAsync per tensor on the copy streams.
 * KERNEL: one grouped copy kernel per group of ready transfers, on the same streams; needs every
 * host buffer to be pinned memory the GPU can address (hipHostMalloc), else TN_ERR_INVALID.
 * KERNEL_IN: the copy kernel for host -> GPU groups only.  GPU -> host copies go to the chip's copy
 * engines: the tensors of a group are first gathered, by a copy inside GPU memory, into a staging
 * slot (8 slots of 16 MiB of GPU memory that tn_executor_create allocates beside the caller's
 * buffer) and leave with one hipMemcpyAsync per run of adjacent places in host memory: the offloads
 * of a group get adjacent arena slots; the stores of a group are taken in the order of their
 * destinations and merged where the caller's buffers follow one another without a gap -- a caller
 * who lays its output buffers out in the order the outputs are produced in (the serial order given
 * to tn_compile) gets copies of up to a whole slot instead of one per tensor, which for tensors of
 * 512 KiB is the difference between 22 and 40 GB/s.  (Stores to host memory from a kernel are accepted slowly by
 * the link and hold up the memory traffic of the kernels that run beside them.)
 * AUTO: KERNEL_IN when all host buffers of the call qualify, otherwise MEMCPY. */
enum { TN_COPY_AUTO = 0, TN_COPY_MEMCPY = 1, TN_COPY_KERNEL = 2, TN_COPY_KERNEL_IN = 3 };

typedef struct {
  int32_t policy;        /* which ready vertex the loop takes first */
  uint64_t order_seed;   /* TN_POLICY_RANDOM */
  uint64_t delay_seed;   /* transfers: completion is held back by a pseudo-random time ... */
  uint32_t max_delay_us; /* ... in [0, max_delay_us]; 0 = no injected delay */
  int32_t max_batch;     /* most same-kind ready vertices put into one kernel launch; 0 = default */
  int32_t profile;       /* != 0: time every launch with HIP events (fills the *_ms fields) */
  int32_t max_transfers; /* most ready copies of one direction put into one group; 0 = default */
  int32_t copy_engine;   /* TN_COPY_AUTO, TN_COPY_MEMCPY or TN_COPY_KERNEL */
  int32_t max_gemm_inflight; /* most GEMM groups running at once; 0 = as many as there are streams */
  int32_t queue_depth;   /* kernel groups in flight per compute stream (1..8; 0 = 1).  1: a kernel is
                            launched when its dependencies have completed.  >1: it may be enqueued once the
                            kernels it depends on are enqueued, ordered on the device by stream events;
                            dependencies on transfers are always awaited on the host. */
  int32_t transfer_depth;  /* groups of copies in flight per direction (1..8; 0 = 3): the next group is enqueued
                              while the host has not yet seen the previous one complete */
  int32_t copy_workgroups; /* TN_COPY_KERNEL: workgroups of a copy launch (each walks over 32 KiB pieces of the
                              group's tensors); 0 = default (8) */
  int32_t d2h_workgroups;  /* TN_COPY_KERNEL: workgroups of a GPU -> host copy launch; 0 = copy_workgroups */
  int32_t small_gemm_tiles; /* a group of bf16 tile products with at most this many 256x256 output tiles is launched
                               with 128x128 tiles per workgroup instead (four times the workgroups, the same bits);
                               0 = default (128), negative = never */
} tn_exec_opts;

typedef struct {
  double wall_ms;                /* host clock around the whole run */
  uint64_t h2d_bytes, d2h_bytes; /* all transfers, per direction */
  int64_t n_vertices, n_launches, n_kernel_launches;
  int64_t n_offload, n_reload;
  uint64_t arena_high_water;
  /* per kernel family (profile != 0): summed device time, launches, algorithmic work */
  double gemm_ms, attn_ms, ewise_ms, h2d_ms, d2h_ms;
  int64_t gemm_launches, attn_launches, ewise_launches;
  double gemm_flops, attn_flops;
  double ewise_bytes;
  double kernel_busy_ms; /* union of kernel intervals over all compute streams */
  double idle_frac;      /* 1 - kernel_busy_ms / (first kernel start .. last kernel end): gaps between kernels only */
  double idle_frac_wall; /* 1 - kernel_busy_ms / wall_ms: the share of the run during which no kernel ran
                            (Section 5: the GPU "sits idle"), leading loads and trailing stores included */
  int64_t untimed_launches; /* profile != 0: launches beyond the executor's pool of timing events (65536 per
                               run), left out of the *_ms fields */
} tn_exec_report;

/* device_base: device memory of at least the memgraph's cap bytes, 256-byte aligned; borrowed
 * for the executor's lifetime.  pinned_arena: pinned host memory for offloaded tensors, or NULL
 * to let the library allocate arena_bytes itself (arena_bytes 0 = the memgraph's safe bound).
 * Streams are hipStream_t values created by the caller at default priority; n_compute >= 1.
 * Creation allocates the operand tables the kernels read (GPU memory plus a pinned host image),
 * the staging slots of GPU -> host copies (8 x 16 MiB of GPU memory, see TN_COPY_KERNEL_IN) and
 * every event a run can need; nothing is allocated or created later. */
tn_status tn_executor_create(const tn_memgraph* mg, void* device_base, uint64_t device_bytes,
                             void* pinned_arena, uint64_t arena_bytes, void* const* compute_streams,
                             int32_t n_compute, void* h2d_stream, void* d2h_stream,
                             tn_executor** out);
void tn_executor_destroy(tn_executor* ex);

/* Copies every TN_DEVICE input from host_inputs[vid] (host memory, or GPU memory outside the
 * device buffer) to its compiled location and waits.  Must
 * precede each tn_execute of a graph that has such inputs (their locations are reused once they
 * are dead).  host_inputs has one entry per taskgraph vertex; entries of non-inputs are ignored. */
tn_status tn_executor_place_inputs(tn_executor* ex, const void* const* host_inputs);

/* Runs the memgraph to completion (Section 5; Appendix A).  host_inputs as above, read by load
 * vertices (pinned memory recommended); host_outputs[i] receives marked output i.  An entry of
 * either array may instead point into memory of the executor's GPU outside its device buffer (a
 * result the next step consumes on the GPU, an input another kernel left there): that transfer is
 * then a copy inside GPU memory, on the same streams; a buffer that overlaps the executor's device
 * buffer is TN_ERR_INVALID.  Synchronous:
 * returns after every vertex has completed.  Makes no hipMalloc/hipFree/hipHostMalloc call.
 * opts NULL = FIFO, no delays; report may be NULL.  Calls on one executor must not overlap. */
tn_status tn_execute(tn_executor* ex, const void* const* host_inputs, void* const* host_outputs,
                     const tn_exec_opts* opts, tn_exec_report* report);

/* For callers that cannot allocate while they run -- a serving loop that keeps one executor per
 * compiled memgraph and must not grow GPU memory per executor, a harness that forbids hipMalloc
 * after start-up, code whose surroundings are being captured into a HIP graph.  Same contract and
 * same results as tn_execute, bit for bit, but the kernels read their operand tables (descriptors,
 * operand addresses, tile sizes, rotary angles: what tn_executor_create puts into GPU memory of its
 * own) from a region of 8 MiB that is part of the loaded library on every GPU: the call copies the
 * executor's pinned table image there (one asynchronous copy on the first compute stream, awaited
 * before anything is launched) and runs.  It calls no hipMalloc, hipFree, hipHostMalloc or
 * hipEventCreate, nor anything else that allocates GPU or pinned memory.
 *   - A memgraph whose tables exceed 8 MiB (about 25 000 kernel vertices of the LLaMA graphs) is
 *     refused with TN_ERR_INVALID; tn_last_error() names both sizes.
 *   - All calls on one GPU share the one region, which keeps the last call's tables; every call
 *     rewrites all of what its own kernels read, so nothing needs clearing.  Calls that overlap
 *     in time on the same GPU (from several threads or executors) race on it: serialise them.
 *     tn_execute does not use the region and may overlap with it. */
tn_status tn_execute_static(tn_executor* ex, const void* const* host_inputs, void* const* host_outputs,
                            const tn_exec_opts* opts, tn_exec_report* report);

/* Launch order of the last run: copies up to cap memgraph vertex ids in the order the loop
 * launched them; returns the count. */
int64_t tn_executor_last_order(const tn_executor* ex, int64_t* out, int64_t cap);

/* One timed launch of the last run (Section 5: what the engine launched when, for judging how well a
 * memgraph keeps the GPU and the link busy).  family: 0 tile products, 1 attention kernels, 2 everything
 * else on the compute streams, 3 a group of host -> GPU copies, 4 a group of GPU -> host copies.
 * work: workgroups of a kernel launch, bytes of a copy group.  Times in ms from the run's first stamp,
 * taken by HIP events on the stream of the launch. */
typedef struct {
  int32_t family, n_vertices;
  int64_t work;
  double amount; /* algorithmic flops of a launch of family 0 or 1, algorithmic bytes of the others */
  float start_ms, end_ms;
} tn_launch_record;

/* The timed launches of the last tn_execute / tn_execute_static with opts.profile != 0, in launch order
 * (none if the run was not profiled).  Copies up to cap records to out (out may be NULL); returns how
 * many there are, or a negative tn_status.  The records live in memory set aside at creation. */
int64_t tn_executor_last_launches(const tn_executor* ex, tn_launch_record* out, int64_t cap);

#ifdef __cplusplus
}
#endif
#endif /* TURNIP_H */
