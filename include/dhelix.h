/*
 * libdhelix -- one GPU's share of a Strand-Interleaving (SI) layer step on MI355X (gfx950).
 *
 * Strand Interleaving (paper Sec. 3.3, 4.2) co-executes the forward pass of micro-batch strand
 * alpha with the backward pass of strand beta on one GPU.  Both strands use one copy of the
 * weights and one weight-gradient buffer (Sec. 3.3, "share model states"), and the operators of
 * the two strands are paired by a plan found offline from pairwise overlap profiling (Sec. 3.2,
 * Eq. 1) with a dynamic program (Sec. 4.2, Eq. 2).
 *
 * General rules of this interface
 *   - plain C ABI; every call returns a dh_status (0 = ok, negative = error) unless stated;
 *     dh_last_error() gives a thread-local message for the last failing call.
 *   - pointers documented "device" are raw HIP device pointers owned by the caller; the library
 *     never allocates or frees device memory (Sec. 5: all allocation stays with one owner).
 *     Handles (dh_layer, dh_plan) are host objects owned by the caller and freed by *_destroy.
 *   - streams are hipStream_t passed as void*; NULL = the null stream.  Compute calls only enqueue
 *     work and return; dh_profile_pairs and dh_plan_search run to completion on the host.
 *   - matrices are row-major; weights are stored [in, out]; activations are [tokens, features]
 *     with tokens = batch*seq laid out sequence after sequence.
 *   - dtype DH_F32: every buffer float32.  DH_BF16: activations/weights bf16, statistics
 *     (rstd, lse), weight gradients and norm-gain gradients float32, fp32 accumulation.
 *   - feature dimensions (hidden, head_dim, ffn) must be multiples of 8; head_dim must be 64 or
 *     128 for DH_BF16; the token count is arbitrary.  Violations return DH_ERR_SHAPE.
 */
#ifndef DHELIX_H
#define DHELIX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DH_OK = 0,
  DH_ERR_INVALID_ARG = -1,
  DH_ERR_SHAPE = -2,
  DH_ERR_WORKSPACE_TOO_SMALL = -3,
  DH_ERR_PLAN_INVALID = -4,
  DH_ERR_HIP = -5,
  DH_ERR_UNSUPPORTED = -6
} dh_status;

typedef enum { DH_F32 = 0, DH_BF16 = 1 } dh_dtype;
/* DH_ARCH_LLAMA: RMSNorm, RoPE, SwiGLU, tensor parallel with all-reduce (Llama models of Table 3).
 * DH_ARCH_GPT:   LayerNorm, biases, GeLU, tensor + sequence parallel (all-gather / reduce-scatter; GPT
 *                models of Table 3).
 * DH_ARCH_MOE:   Llama-style attention (not sharded) + top-2 mixture-of-experts SwiGLU FFN under expert
 *                parallelism (all-to-all dispatch / combine; MoE models of Table 3).
 * DH_ARCH_LLAMA_CP: DH_ARCH_LLAMA on one rank of a context-parallel group (Sec. 2.1): the rank holds one chunk of
 *                each sequence and collects the earlier chunks' keys/values by Send/Recv (Sec. 2.1, Sec. 2.3). */
typedef enum { DH_ARCH_LLAMA = 0, DH_ARCH_GPT = 1, DH_ARCH_MOE = 2, DH_ARCH_LLAMA_CP = 3 } dh_arch;

/* Message of the last error raised on this thread ("" if none).  Host memory owned by the library. */
const char* dh_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Layer description: one GPU's share of a pre-norm transformer layer (the models of Sec. 6.1,
 * Table 3).  DH_ARCH_LLAMA: RMSNorm, QKV GEMM, RoPE, causal grouped-query attention, output GEMM,
 * all-reduce, residual, RMSNorm, gate/up GEMM, SwiGLU, down GEMM, all-reduce, residual.
 * DH_ARCH_GPT: the layer's input, output and norms live on this rank's sequence shard of
 * Ts = T / n_ranks rows (the first Ts rows of the [T,H] row order); an all-gather precedes each
 * column-parallel GEMM, a reduce-scatter follows each row-parallel one; no RoPE.
 * DH_ARCH_MOE: no tensor parallelism; the FFN is routed: top-2 of n_experts logical experts, of which
 * this GPU holds n_local_experts (logical expert e runs on local expert e % n_local_experts, the
 * other factor of e standing for the source rank of an expert-parallel group).
 * DH_ARCH_LLAMA_CP: seq is the length of this rank's chunk; its rows sit at positions cp_rank*seq .. of each
 * sequence (contiguous chunks in rank order).  After RoPE the rank's keys/values and those of the cp_rank earlier
 * ranks are gathered into one buffer (the chunks of later ranks pass through the rank too, as on a ring, but no causal
 * query reads them); attention runs over that buffer; in the backward pass the key/value gradients of the earlier
 * chunks are sent back and the rank adds what the later ranks send for its own chunk.  bf16: cp_rank*seq must be
 * a multiple of 128.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int arch;        /* dh_arch */
  int dtype;       /* dh_dtype */
  int batch;       /* sequences per micro-batch */
  int seq;         /* tokens per sequence; tokens T = batch*seq */
  int hidden;      /* H */
  int n_q_heads;   /* local query heads */
  int n_kv_heads;  /* local key/value heads; must divide n_q_heads */
  int head_dim;    /* d */
  int ffn;         /* local FFN width F (per expert for DH_ARCH_MOE) */
  float eps;       /* RMSNorm epsilon */
  float rope_base; /* RoPE base; pair i turns by position * base^(-2i/d) */
  int n_ranks;     /* R: partials summed by each collective stand-in (1 = no peers) */
  int comm_blocks; /* thread blocks a collective stand-in may use (its "channel" count); 0 = enough
                      to cover the payload */
  int n_experts;       /* DH_ARCH_MOE: logical experts E (2..256); else 0 */
  int n_local_experts; /* DH_ARCH_MOE: experts held by this GPU, divides E; else 0 */
  int cp_ranks;        /* DH_ARCH_LLAMA_CP: ranks of the context-parallel group (1..16); else 0 */
  int cp_rank;         /* DH_ARCH_LLAMA_CP: this rank's index, 0 .. cp_ranks-1 */
  int cross_blocks;    /* DH_ARCH_LLAMA_CP: thread blocks of a Send/Recv stand-in, which set its rate (a block
                          moves 5-7 GB/s on MI355X); 0 = 8 blocks, about one 400 Gb/s network port */
  int rope_pairing;    /* dh_rope_pairing: which two elements of a head form RoPE pair i (the paper names no
                          convention); 0 = DH_ROPE_HALVES */
  int gelu_form;       /* DH_ARCH_GPT: dh_gelu_form of the MLP activation; 0 = DH_GELU_TANH */
} dh_layer_config;

/* Device pointers to the shard's weights (read only).  g1,g2: [H]; Wqkv: [H,(nq+2nkv)d] with columns
 * [q heads | k heads | v heads]; Wo: [nq*d,H]; Wgu: [H,2F] with columns [gate | up]; Wd: [F,H].
 * DH_ARCH_GPT: Wgu is the first MLP matrix [H,F], Wd the second [F,H]; b1,b2: LayerNorm shifts [H];
 * bqkv [(nq+2nkv)d], bo [H], bfc1 [F], bfc2 [H]: biases of the four linears (bo and bfc2 are added
 * after the reduce-scatter).  DH_ARCH_MOE: Wgu [n_local,H,2F], Wd [n_local,F,H].
 * Pointers an architecture does not use are ignored. */
typedef struct {
  const void *g1, *Wqkv, *Wo, *g2, *Wgu, *Wd;
  const void *b1, *bqkv, *bo, *b2, *bfc1, *bfc2;
} dh_weights;

/* Device pointers to the float32 gradient buffers, same shapes as the weights.  The backward pass
 * ADDS into them; one set is shared by both strands (Sec. 3.3). */
typedef struct {
  float *dg1, *dWqkv, *dWo, *dg2, *dWgu, *dWd;
  float *db1, *dbqkv, *dbo, *db2, *dbfc1, *dbfc2;
} dh_wgrads;

typedef struct dh_layer dh_layer;

/* Creates the host-side layer object (shapes, launch configuration, events).  Host only. */
int dh_layer_create(const dh_layer_config* cfg, dh_layer** out);
void dh_layer_destroy(dh_layer* layer);
int dh_layer_bind_weights(dh_layer* layer, const dh_weights* w);
int dh_layer_bind_wgrads(dh_layer* layer, const dh_wgrads* g);

/* Bytes of one strand's saved-activation slot (written by forward, read by backward): norm
 * statistics, h1, (rotated) qkv, o, lse, x2, h2, FFN pre-activation, a; DH_ARCH_MOE adds the routing
 * decision, its index tables and the dispatched rows. */
size_t dh_layer_saved_bytes(const dh_layer* layer);

typedef enum { DH_WS_FWD = 0, DH_WS_BWD = 1, DH_WS_SI = 2 } dh_ws_kind;
/* Bytes of transient workspace for a forward pass, a backward pass, or one SI step (a forward and a
 * backward region side by side, so the two strands never share a transient buffer). */
size_t dh_layer_workspace_bytes(const dh_layer* layer, int kind);

/* One strand's forward call.  x: device [T,H] input ([Ts,H] for DH_ARCH_GPT), must stay valid and
 * unchanged until that strand's backward has run.  out: device, same shape.  saved: device slot of
 * dh_layer_saved_bytes.
 * peers_ar1/peers_ar2: frozen contributions of the other ranks to the two forward reductions
 * (ignored when n_ranks == 1): DH_ARCH_LLAMA [R-1,T,H] partials of the all-reduces; DH_ARCH_GPT
 * [R-1,Ts,H] partials of the reduce-scatters for this rank's rows.
 * peers_ag1/peers_ag2: DH_ARCH_GPT only, [R-1,Ts,H] the other ranks' shards entering the all-gathers.
 * logits: DH_ARCH_MOE only, float32 [T,n_experts] router logits (an input of the layer).
 * peers_kv: DH_ARCH_LLAMA_CP only, [cp_ranks-1, T, 2*nkv*d]: the other ranks' key/value chunks ([k heads | v heads]
 * per row, keys rotated), ordered by source rank with this rank left out (ignored when cp_ranks == 1). */
typedef struct {
  const void* x;
  void* out;
  void* saved;
  const void* peers_ar1;
  const void* peers_ar2;
  const void* peers_ag1;
  const void* peers_ag2;
  const float* logits;
  const void* peers_kv;
} dh_fwd_args;

/* One strand's backward call.  dout: device [T,H] upstream gradient; dx: device [T,H] result;
 * x/saved: what the strand's forward call read/wrote; peers_ar3/peers_ar4: frozen partials of the
 * two backward collectives. */
typedef struct {
  const void* dout;
  void* dx;
  const void* x;
  const void* saved;
  const void* peers_ar3;
  const void* peers_ar4;
  const void* peers_ag3; /* DH_ARCH_GPT: [R-1,Ts,H] peers' gradient shards of the backward all-gathers */
  const void* peers_ag4;
  float* dlogits;        /* DH_ARCH_MOE: float32 [T,n_experts] gradient of the router logits (written) */
  const void* peers_dkv; /* DH_ARCH_LLAMA_CP: [cp_ranks-1, T, 2*nkv*d] the other ranks' gradient contributions to this
                            rank's keys/values (order of peers_kv); those of the later ranks are added */
  void* dkv_peers;       /* DH_ARCH_LLAMA_CP: [cp_rank, T, 2*nkv*d] (written) the key/value gradients this rank sends
                            back to each earlier rank */
} dh_bwd_args;

/* Forward / backward of one strand, operators in their default order, all on `stream`
 * (single-strand execution, the baseline of Sec. 6.1).  ws: device workspace of at least
 * dh_layer_workspace_bytes(layer, DH_WS_FWD / DH_WS_BWD), ws_bytes its size. */
int dh_layer_fwd(dh_layer* layer, const dh_fwd_args* a, void* ws, size_t ws_bytes, void* stream);
int dh_layer_bwd(dh_layer* layer, const dh_bwd_args* b, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Operator graphs (Sec. 4.2, "Operator Sequencing and Partitioning").  Node ids are the operator
 * ids below; an edge (src,dst) means src must run before dst within the strand.
 * ------------------------------------------------------------------------------------------ */
typedef enum {
  DH_F_NORM1 = 0, DH_F_QKV, DH_F_ROPE, DH_F_ATTN, DH_F_PROJ, DH_F_AR1, DH_F_NORM2, DH_F_FC1,
  DH_F_ACT, DH_F_FC2, DH_F_AR2, DH_F_BDA2, DH_F_NOPS
} dh_fwd_op;
typedef enum {
  DH_B_FC2_DGRAD = 0, DH_B_FC2_WGRAD, DH_B_ACT, DH_B_FC1_DGRAD, DH_B_FC1_WGRAD, DH_B_AR3,
  DH_B_NORM2, DH_B_PROJ_DGRAD, DH_B_PROJ_WGRAD, DH_B_ATTN, DH_B_ROPE, DH_B_QKV_DGRAD,
  DH_B_QKV_WGRAD, DH_B_AR4, DH_B_NORM1, DH_B_NOPS
} dh_bwd_op;

/* DH_ARCH_GPT.  Bias gradients belong to the weight-gradient operator of their linear. */
typedef enum {
  DH_GF_NORM1 = 0, DH_GF_AG1, DH_GF_QKV, DH_GF_ATTN, DH_GF_PROJ, DH_GF_RS1, DH_GF_NORM2, DH_GF_AG2,
  DH_GF_FC1, DH_GF_ACT, DH_GF_FC2, DH_GF_RS2, DH_GF_BDA2, DH_GF_NOPS
} dh_gpt_fwd_op;
typedef enum {
  DH_GB_AG3 = 0, DH_GB_FC2_DGRAD, DH_GB_FC2_WGRAD, DH_GB_ACT, DH_GB_FC1_DGRAD, DH_GB_FC1_WGRAD,
  DH_GB_RS3, DH_GB_NORM2, DH_GB_AG4, DH_GB_PROJ_DGRAD, DH_GB_PROJ_WGRAD, DH_GB_ATTN,
  DH_GB_QKV_DGRAD, DH_GB_QKV_WGRAD, DH_GB_RS4, DH_GB_NORM1, DH_GB_NOPS
} dh_gpt_bwd_op;
/* DH_ARCH_MOE. */
typedef enum {
  DH_MF_NORM1 = 0, DH_MF_QKV, DH_MF_ROPE, DH_MF_ATTN, DH_MF_PROJ, DH_MF_NORM2, DH_MF_ROUTE,
  DH_MF_PERMUTE, DH_MF_A2A_DISPATCH, DH_MF_FC1, DH_MF_ACT, DH_MF_FC2, DH_MF_A2A_COMBINE,
  DH_MF_UNPERMUTE, DH_MF_NOPS
} dh_moe_fwd_op;
typedef enum {
  DH_MB_UNPERMUTE = 0, DH_MB_ROUTE, DH_MB_A2A_DISPATCH, DH_MB_FC2_DGRAD, DH_MB_FC2_WGRAD, DH_MB_ACT,
  DH_MB_FC1_DGRAD, DH_MB_FC1_WGRAD, DH_MB_A2A_COMBINE, DH_MB_PERMUTE, DH_MB_NORM2,
  DH_MB_PROJ_DGRAD, DH_MB_PROJ_WGRAD, DH_MB_ATTN, DH_MB_ROPE, DH_MB_QKV_DGRAD, DH_MB_QKV_WGRAD,
  DH_MB_NORM1, DH_MB_NOPS
} dh_moe_bwd_op;

/* DH_ARCH_LLAMA_CP: the Llama operators plus the key/value exchange (F_CP_KV: no predecessor, only attention waits for
 * it; the rank's own keys/values are put in place by F_ROPE), the reduction of the rank's own key/value gradient with
 * what later ranks send (B_CP_DKV) and the send-back of the earlier chunks' gradients (B_CP_SEND: no successor). */
typedef enum {
  DH_CF_NORM1 = 0, DH_CF_QKV, DH_CF_ROPE, DH_CF_CP_KV, DH_CF_ATTN, DH_CF_PROJ, DH_CF_AR1, DH_CF_NORM2, DH_CF_FC1,
  DH_CF_ACT, DH_CF_FC2, DH_CF_AR2, DH_CF_BDA2, DH_CF_NOPS
} dh_cp_fwd_op;
typedef enum {
  DH_CB_FC2_DGRAD = 0, DH_CB_FC2_WGRAD, DH_CB_ACT, DH_CB_FC1_DGRAD, DH_CB_FC1_WGRAD, DH_CB_AR3, DH_CB_NORM2,
  DH_CB_PROJ_DGRAD, DH_CB_PROJ_WGRAD, DH_CB_ATTN, DH_CB_CP_DKV, DH_CB_CP_SEND, DH_CB_ROPE, DH_CB_QKV_DGRAD,
  DH_CB_QKV_WGRAD, DH_CB_AR4, DH_CB_NORM1, DH_CB_NOPS
} dh_cp_bwd_op;

#define DH_MAX_OPS 32
#define DH_MAX_DEPS 96
typedef struct {
  int n_ops;
  int is_comm[DH_MAX_OPS];   /* 1 = collective stand-in (issued on the communication stream); 2 = cross-node
                                Send/Recv stand-in (issued on the layer's cross-node stream if one is set) */
  int n_deps;
  int dep_src[DH_MAX_DEPS];
  int dep_dst[DH_MAX_DEPS];
  int side_ok[DH_MAX_OPS];   /* backward graph: 1 = the operator has no dependents and touches no buffer a later operator
                                of its strand writes, so a plan may run it beside the strand (dh_plan.bwd_side) */
  int like_other[DH_MAX_OPS]; /* 1 + id of the operator of the OTHER direction's graph that runs the same kernel on the
                                same amount of data (a backward all-reduce and a forward one; a weight-gradient GEMM and
                                the forward GEMM of its shape), 0 = none.  The pair profiler co-runs forward with backward
                                operators only; the lane model (dh_plan_cost) looks up two operators of one direction
                                through this. */
} dh_op_graph;

/* Fills the forward (direction 0) or backward (direction 1) operator graph of the layer. */
int dh_layer_op_graph(const dh_layer* layer, int direction, dh_op_graph* out);
/* Static name of an operator of an architecture ("F_QKV", "B_ATTN", ...), NULL if out of range. */
const char* dh_op_name(int arch, int direction, int op);

/* ------------------------------------------------------------------------------------------
 * Overlap table (Sec. 3.2): solo time of every operator and, for every (forward, backward)
 * operator pair started together, the progress rate of each while both are active
 * (1 = undisturbed).  From these, P(i,j) of Eq. 2 and OEF of Eq. 1 follow.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int n_fwd, n_bwd;
  double t_fwd[DH_MAX_OPS];                 /* seconds */
  double t_bwd[DH_MAX_OPS];
  double rate_fwd[DH_MAX_OPS][DH_MAX_OPS];  /* [fwd op][bwd op] */
  double rate_bwd[DH_MAX_OPS][DH_MAX_OPS];
  double p_pair[DH_MAX_OPS][DH_MAX_OPS];    /* P_ij of one instance of each, seconds, from the measured rates */
  double oef[DH_MAX_OPS][DH_MAX_OPS];       /* Eq. 1 */
} dh_overlap_table;

/* Eq. 1: (t_i + t_j - p_ij) / min(t_i, t_j).  Host only; returns the value. */
double dh_oef(double t_i, double t_j, double p_ij);

/* Co-run time of a forward segment with a backward segment under the two-queue fluid model
 * (each strand runs its operators in order; a pair of active operators progresses at the table's
 * rates; a lone operator at rate 1).  seg_f/seg_b: host arrays of operator ids.  Host only;
 * returns seconds, or a negative dh_status cast to double on bad arguments. */
double dh_segment_cost(const dh_overlap_table* t, const int* seg_f, int n_f, const int* seg_b, int n_b);

/* Measures the table on the current device: every operator alone and every forward/backward pair
 * co-started on two streams (collective stand-ins on comm_stream).  The strands' buffers must
 * already hold a completed forward (alpha, beta) and backward (beta) so every operator has valid
 * inputs.  The operators run over and over in place: the gradient buffers are added to, and alpha's
 * saved slot, alpha's out and beta's dx are overwritten (RoPE turns alpha's saved qkv again on every
 * repetition), so run the strands' forward and backward again before their results are used.  Solo
 * times are the shorter of two timed groups of reps launches (a hiccup of the machine lengthens one group, not both)
 * and have a floor of 0.1 us (an operator that launches nothing), rates lie in [0.02, 1].
 * Blocks until done.  reps: timed repetitions (>=1). */
int dh_profile_pairs(dh_layer* layer, const dh_fwd_args* alpha, const dh_bwd_args* beta, void* ws,
                     size_t ws_bytes, void* stream_alpha, void* stream_beta, void* comm_stream,
                     int reps, dh_overlap_table* out);

/* The solo times alone (Sec. 3.2, the T_i of Eq. 1): every operator launched reps times back to back (after one
 * warm-up launch; two such groups, the shorter counts) on the stream dh_si_step would issue it to, timed with events on
 * that stream.  t_fwd / t_bwd: host
 * arrays of DH_MAX_OPS doubles, seconds.  Same requirements and side effects as dh_profile_pairs.  Blocks until done. */
int dh_profile_solo(dh_layer* layer, const dh_fwd_args* alpha, const dh_bwd_args* beta, void* ws, size_t ws_bytes,
                    void* stream_alpha, void* stream_beta, void* comm_stream, int reps, double* t_fwd, double* t_bwd);

/* ------------------------------------------------------------------------------------------
 * Plans (Sec. 4.2).  A plan = one operator sequence per strand plus segment pairs: pair k
 * co-runs forward operators fwd_order[f_begin:f_end] with backward operators
 * bwd_order[b_begin:b_end]; a cross-strand barrier follows every pair.
 * bwd_side[op] != 0 lets backward operator `op` run beside its strand: it is issued on the other strand's stream
 * once the backward operators before it in bwd_order are done, so the backward strand goes on without waiting for it
 * (Sec. 4.2: a weight-gradient operator has no dependents inside the layer and may overlap its own strand).  It still
 * ends before its segment pair's barrier.  Only operators whose graph entry has side_ok set may be marked.
 * ------------------------------------------------------------------------------------------ */
typedef struct { int f_begin, f_end, b_begin, b_end; } dh_seg_pair;
typedef struct {
  int n_fwd, n_bwd, n_pairs;
  int fwd_order[DH_MAX_OPS];
  int bwd_order[DH_MAX_OPS];
  dh_seg_pair pairs[2 * DH_MAX_OPS];
  int bwd_side[DH_MAX_OPS]; /* indexed by operator id */
} dh_plan;

/* Eq. 2 for given segments: p_f[i] = P(i, none), p_b[j] = P(none, j), p_fb[i*n_b + j] = P(i,j).
 * Writes T_opt(n_f, n_b) to *t_opt; if steps != NULL writes up to n_f+n_b chosen steps as
 * (i or -1, j or -1) pairs and their count to *n_steps.  Host only. */
int dh_pair_dp(const double* p_f, int n_f, const double* p_b, int n_b, const double* p_fb,
               double* t_opt, int* steps, int* n_steps);

/* Plan search: enumerates topological orders of both graphs (at most max_orders per graph, 0 =
 * library default), and for each pair of orders places barriers optimally by Eq. 2 applied over
 * operator prefixes with dh_segment_cost (+ barrier_cost seconds per pair) as P.  Writes the best
 * plan and its predicted makespan.  Host only. */
int dh_plan_search(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table,
                   double barrier_cost, int max_orders, dh_plan* out, double* makespan);

/* Number of topological orders of an operator graph, counted up to `cap` (the count stops there): Sec. 4.2 step (1)
 * enumerates them all.  dh_plan_search tries every order when there are at most max_orders (default 20000; the Llama
 * backward graph has 5760); otherwise the first half of the depth-first enumeration plus as many orders drawn by a
 * seeded generator, so that operators without successors are tried everywhere.  Host only; negative dh_status on bad
 * arguments. */
long long dh_plan_count_orders(const dh_op_graph* g, long long cap);

/* Where dh_si_step places the stand-ins, as the lane model needs to know it. */
typedef struct {
  int comm_alpha; /* strand alpha's collectives: 0 = in alpha's stream (stream_comm == NULL), 1 = on the communication stream */
  int comm_beta;  /* strand beta's: 0 = in beta's stream, 1 = on the communication stream shared with alpha's,
                     2 = on beta's own communication stream (dh_layer_set_beta_comm_stream) */
  int cross;      /* cross-node transfers (is_comm == 2): 0 = where their strand's collectives go, 1 = on the cross-node stream */
} dh_lanes;

/* Predicted time of a plan under the lane model: the segment pairs are replayed the way dh_si_step issues them -- the
 * two strands, the communication stream(s) and the cross-node stream are lanes that run their operators in issue
 * order; a stand-in on a lane of its own starts behind what its strand has issued and holds up only the operators
 * that consume its result; bwd_side operators run in alpha's lane -- and integrated as a fluid: every active operator
 * advances at the product of its profiled pairwise rates against the other active operators (operators of one
 * direction through like_other, rate 1 where that is 0).  barrier_cost is added per segment pair.  This is P of Eq. 2
 * for three and more participants (a stand-in beside two compute kernels), which the two-queue dh_segment_cost cannot
 * express.  Host only; returns seconds, or a negative dh_status cast to double. */
double dh_plan_cost(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table, const dh_plan* plan,
                    const dh_lanes* lanes, double barrier_cost);

typedef struct {
  long long orders_fwd_total, orders_bwd_total; /* topological orders of the graphs (counted up to max_orders + 1) */
  int orders_fwd_tried, orders_bwd_tried;
  int truncated;                                /* 1 = not every order was tried */
  int refined;                                  /* order pairs that went through barrier placement */
} dh_search_info;

/* Plan search under the lane model (Sec. 4.2 with P = dh_plan_cost of a segment pair).  Step 1 ranks every pair of
 * operator orders (all orders, see dh_plan_count_orders) as one free-running segment pair.  Step 2 takes the 24 best
 * and 8 spread over the rest, tries the side_ok operators beside their strand (every subset of up to 4), and places
 * barriers by Eq. 2 over operator prefixes.  Writes the best plan (orders, segment pairs, bwd_side) and its predicted
 * time; info may be NULL.  Host only, multi-threaded. */
int dh_plan_search_lanes(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table,
                         const dh_lanes* lanes, double barrier_cost, int max_orders, dh_plan* out, double* makespan,
                         dh_search_info* info);

/* Checks that a plan's orders are permutations respecting the graphs and that its pairs tile both
 * sequences.  Returns DH_OK or DH_ERR_PLAN_INVALID. */
int dh_plan_validate(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_plan* plan);

/* The round-robin comparison schedule of Sec. 6.1 ("Wavelet+"): default operator orders, one forward
 * operator paired with one backward operator at a time, a barrier after every pair.  (The other
 * ablation of Sec. 6.4, weight gradients left in their default places, is dh_plan_search with
 * max_orders = 1.)  Host only. */
int dh_plan_round_robin(const dh_op_graph* fwd, const dh_op_graph* bwd, dh_plan* out);

/* The degenerate plan "all forward, then all backward" in default order (sequential baseline). */
int dh_plan_sequential(const dh_layer* layer, dh_plan* out);

/* One SI step (Sec. 3.3, 5): forward of strand alpha and backward of strand beta, operators issued
 * per plan on stream_alpha / stream_beta, collective stand-ins on stream_comm (NULL = issue them on
 * the strand's own stream), barriers between segment pairs by events (no host synchronisation).
 * A stand-in issued on another stream than its strand's starts after what the strand has issued so far; the strand
 * waits for it only when an operator that depends on it (operator graph) comes up, or at the end of the segment
 * pair, so operators of the same strand that do not need the result overlap the transfer (Sec. 4.2, the
 * "self-overlapping" operators of the pairing figure).
 * On return all work is enqueued; all three streams are joined back into stream_alpha.
 * ws: at least dh_layer_workspace_bytes(layer, DH_WS_SI). */
int dh_si_step(dh_layer* layer, const dh_fwd_args* alpha, const dh_bwd_args* beta,
               const dh_plan* plan, void* ws, size_t ws_bytes, void* stream_alpha,
               void* stream_beta, void* stream_comm);

/* SwiGLU inside the epilogues of the neighbouring GEMMs (dh_gemm_swiglu_fwd / _bwd below) for later calls on this
 * layer: enable != 0 (the state after dh_layer_create) uses them wherever the layer's shapes fit, 0 runs the separate
 * operators.  Results are bit-identical either way; the switch exists to measure one against the other.  Returns a
 * negative dh_status on error, else a bit mask of what is now fused: 1 = forward (F_ACT launches nothing),
 * 2 = backward (B_ACT launches nothing).  Host only. */
int dh_layer_set_fused_activation(dh_layer* layer, int enable);

/* Backward all-reduces carried by a weight-gradient GEMM of their own strand (dh_gemm_allreduce below) for later
 * calls on this layer, Llama architectures in bf16: bit 1 = B_AR3 with B_FC1_WGRAD, bit 2 = B_AR4 with B_QKV_WGRAD
 * (Sec. 4.2: the weight gradients are the operators free to move; here they move into the collective's launch).  While
 * the stand-ins run on a block budget (comm_blocks > 0) and the GEMM fits, the collective operator launches both and
 * the weight-gradient operator launches nothing; otherwise the operators run apart as before.  Default 0.  Results
 * are bit-identical either way.  Returns a negative dh_status on error, else the mask now in force.  Host only. */
int dh_layer_set_fused_collective(dh_layer* layer, int mask);

/* A communication stream of strand beta's own for later SI steps of this layer (NULL, the default: beta's collectives
 * go where alpha's go).  With one shared stream the two strands' collectives run one after the other in issue order;
 * when a collective costs what a link makes it cost, that order is the step's critical path.  Host only. */
int dh_layer_set_beta_comm_stream(dh_layer* layer, void* stream_comm_beta);

/* Thread blocks of the layer's collective stand-ins from now on (the layer configuration's comm_blocks): 0 = cover the
 * payload, n > 0 = n blocks (a link-like rate), -1 = the stand-ins launch nothing (their events and stream
 * dependencies stay): the step then computes nothing meaningful and serves only to time the schedule without its
 * communication, T_SI,no-comm of the hidden-communication measure.  Host only. */
int dh_layer_set_comm_blocks(dh_layer* layer, int comm_blocks);

/* Stream for the cross-node Send/Recv stand-ins of later SI steps of this layer (Sec. 5: computation, local-node
 * and cross-node communication each get a stream); NULL (the default) issues them where the collective stand-ins
 * go.  The stream must outlive those steps; each step joins it back into stream_alpha.  Host only. */
int dh_layer_set_cross_stream(dh_layer* layer, void* stream_cross);

/* One SI step across two layers of identical shape: forward of strand alpha through layer_alpha while
 * strand beta runs backward through layer_beta (each layer has its own weights and gradient buffers).
 * dh_si_step is the case layer_alpha == layer_beta. */
int dh_si_step_layers(dh_layer* layer_alpha, dh_layer* layer_beta, const dh_fwd_args* alpha,
                      const dh_bwd_args* beta, const dh_plan* plan, void* ws, size_t ws_bytes,
                      void* stream_alpha, void* stream_beta, void* stream_comm);

/* ------------------------------------------------------------------------------------------
 * A stack of L layers of one shape under SI on one GPU: the single-stage case of the folded
 * pipeline of Sec. 4.1.  In a phase, strand alpha (a new micro-batch) sweeps forward through layers
 * 0..L-1 while strand beta (the micro-batch of the previous phase) sweeps backward through L-1..0;
 * step k is one SI step of alpha's layer k with beta's layer L-1-k.  Activations live in a caller-owned
 * arena shared by both strands in the two-triangle arrangement of Sec. 3.3: L+1 saved-activation slots
 * and L layer-input buffers (dh_stack_arena_bytes) instead of two full sets (dh_stack_unshared_bytes).
 * DH_ARCH_LLAMA only.  Host-side objects; every operator runs through the layer calls above.
 * ------------------------------------------------------------------------------------------ */
typedef struct dh_stack dh_stack;
/* x: device [T,H] input of layer 0, must stay valid until this micro-batch's backward phase has run;
 * out: device [T,H] output of layer L-1; peers as in dh_fwd_args, the same buffers for every layer. */
typedef struct { const void* x; void* out; const void* peers_ar1; const void* peers_ar2; } dh_stack_fwd;
/* dout: device [T,H] gradient of the last layer's output; dx: device [T,H] gradient of layer 0's input. */
typedef struct { const void* dout; void* dx; const void* peers_ar3; const void* peers_ar4; } dh_stack_bwd;
int dh_stack_create(const dh_layer_config* cfg, int n_layers, dh_stack** out);
void dh_stack_destroy(dh_stack* stack);
/* Layer i of the stack (owned by the stack), to bind its weights and gradient buffers. */
dh_layer* dh_stack_layer(dh_stack* stack, int i);
size_t dh_stack_arena_bytes(const dh_stack* stack);
size_t dh_stack_unshared_bytes(const dh_stack* stack);
size_t dh_stack_workspace_bytes(const dh_stack* stack);
/* One phase.  alpha != NULL, beta == NULL: warm-up (forward sweep only); both: L SI steps with `plan`;
 * alpha == NULL: cool-down (backward sweep of the last micro-batch).  beta always refers to the
 * micro-batch that was alpha in the previous phase.  Enqueues on the given streams and returns. */
int dh_stack_phase(dh_stack* stack, const dh_stack_fwd* alpha, const dh_stack_bwd* beta,
                   const dh_plan* plan, void* arena, size_t arena_bytes, void* ws, size_t ws_bytes,
                   void* stream_alpha, void* stream_beta, void* stream_comm);

/* The same step recorded once into a HIP graph (stream capture on stream_alpha, which forks into
 * stream_beta; nothing runs) and replayed with one launch per step, which removes the per-operator
 * launch intervals (Sec. 6.3, Table 7, names them as part of the remaining loss).  The two streams must be distinct and
 * non-null.  A graph holds dependencies, not streams: every collective stand-in becomes a node in its
 * strand's chain.  All buffers named by alpha, beta, ws and the bound weights/gradients must stay where
 * they are while the graph is in use.  dh_si_graph_launch enqueues one step on `stream`. */
typedef struct dh_si_graph dh_si_graph;
int dh_si_graph_create(dh_layer* layer, const dh_fwd_args* alpha, const dh_bwd_args* beta,
                       const dh_plan* plan, void* ws, size_t ws_bytes, void* stream_alpha,
                       void* stream_beta, dh_si_graph** out);
int dh_si_graph_launch(dh_si_graph* graph, void* stream);
void dh_si_graph_destroy(dh_si_graph* graph);

/* ------------------------------------------------------------------------------------------
 * Collective stand-ins (Sec. 2.1, "Collective Communication"): memory-bound local kernels with the
 * payload of the collective they replace.  parts: host array of n_ranks device pointers, each `elems`
 * elements of `dtype`; parts[0] is this GPU's own buffer, parts[1..] the frozen peers' buffers.
 *   DH_COMM_ALLREDUCE      out[i] = sum_r parts[r][i], added in rank order in fp32; out: elems.
 *   DH_COMM_REDUCESCATTER  the same sum over this rank's slice: parts[0] points at the slice of the own
 *                          partial this rank keeps, parts[r] at peer r's partial for that slice; out: elems.
 *                          (Receive side only: the own partial's other slices, which a real
 *                          reduce-scatter sends away, are not touched.)
 *   DH_COMM_ALLGATHER      out = [parts[0] | parts[1] | ...]; out: n_ranks*elems.
 *   DH_COMM_A2A_DISPATCH,  an expert-parallel all-to-all with equal splits (fixed expert capacity, Sec. 6.1), receive
 *   DH_COMM_A2A_COMBINE    side: parts[r] = the elems elements rank r sends to this rank, out = [parts[0] | parts[1] | ...].
 *                          Dispatch and combine move the same payload in opposite directions.  (The layer's dropless
 *                          routing has data-dependent splits and uses dh_moe_gather_rows with its index maps instead.)
 * dtype must be DH_F32 or DH_BF16; out and every parts[r] must be 16-byte aligned (DH_ERR_INVALID_ARG otherwise).
 * n_blocks: 256-thread blocks the kernel may use (the analogue of a collective library's
 * channel/thread limit, Sec. 5); 0 = enough to cover the payload (at most 2048).  Enqueued on `stream`.
 * ------------------------------------------------------------------------------------------ */
typedef enum {
  DH_COMM_ALLREDUCE = 0, DH_COMM_ALLGATHER = 1, DH_COMM_REDUCESCATTER = 2, DH_COMM_A2A_DISPATCH = 3, DH_COMM_A2A_COMBINE = 4
} dh_comm_kind;
int dh_comm_standin(int kind, int n_ranks, const void* const* parts, void* out, size_t elems,
                    int dtype, int n_blocks, void* stream);

/* Context parallelism (Sec. 2.1, Sec. 2.3: CP ranks pass key/value chunks around by Send/Recv; Sec. 5: such
 * cross-node transfers get a stream of their own).  One-GPU stand-in of the exchange: n_moves (<= 16) copies, each
 * of `rows` rows of `width` elements (multiple of 8) for each of `batch` sequences.  A side of a move is a row-major
 * buffer with a row pitch of ld elements holding seq_rows rows per sequence, of which the move touches rows
 * row0 .. row0+rows-1.  Device pointers, 16-byte aligned; n_blocks as for dh_comm_standin (a handful of blocks move
 * data at about the rate of a network link, which is what the transfer is a stand-in for). */
typedef struct {
  const void* src;
  void* dst;
  int src_ld, src_seq_rows, src_row0;
  int dst_ld, dst_seq_rows, dst_row0;
} dh_cp_move;
int dh_cp_exchange(int dtype, int n_moves, const dh_cp_move* moves, int batch, int rows, int width, int n_blocks,
                   void* stream);
/* The key/value gradient a CP rank keeps: own->dst rows = own->src rows + peers[0] + peers[1] + ... (added in that
 * order in float32, rounded once); peers[k]: device [batch*rows, width] contiguous. */
int dh_cp_grad_reduce(int dtype, const dh_cp_move* own, int n_peers, const void* const* peers, int batch, int rows,
                      int width, int n_blocks, void* stream);

/* Creates a stream whose kernels may only use n_cus compute units (spread over the chip), the
 * analogue of limiting a collective's thread/channel count (Sec. 5).  Default priority. */
int dh_stream_create_masked(int n_cus, void** stream);
int dh_stream_destroy(void* stream);

/* ------------------------------------------------------------------------------------------
 * Single operators, exposed for unit parity tests and micro-benchmarks.
 * ------------------------------------------------------------------------------------------ */
/* All take device pointers, enqueue on `stream` and return a dh_status.  dtype is the storage type of
 * the activations (dh_dtype); rstd, lse, delta, dgamma are always float32. */

/* C[M,N] (+)= opA(A) * opB(B) (GEMM operator base, Table 2).  trans_a = 0: A is [M,K]; 1: A is [K,M].
 * trans_b = 0: B is [K,N]; 1: B is [N,K].  dtype = type of A and B; out_f32_accumulate = 0: C has
 * dtype and is overwritten, 1: C is float32 and is added to (weight gradients).  DH_BF16 needs N and
 * every contiguous operand dimension to be a multiple of 8 and does not build trans_a with trans_b.
 * ws: device workspace for split-K partials of dh_gemm_workspace_bytes (fewer bytes, or NULL with
 * ws_bytes 0, reduce or disable split-K; results then differ in rounding only). */
int dh_gemm(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, const void* B,
            void* C, int out_f32_accumulate, void* ws, size_t ws_bytes, void* stream);
size_t dh_gemm_workspace_bytes(int dtype, int trans_a, int trans_b, int M, int N, int K);

/* RMSNorm forward (LayerNorm operator base, Table 2, RMS form).  If residual != NULL the fused
 * bias-dropout-add residual is applied first: x_out = x + residual (stored), and the norm reads
 * x_out.  h[T,H] = gamma * x * rstd, rstd[T] = (mean x^2 + eps)^(-1/2). */
int dh_rmsnorm_fwd(int dtype, int T, int H, const void* x, const void* residual, const void* gamma,
                   float eps, void* x_out, void* h, float* rstd, void* stream);
/* RMSNorm backward: dx = rstd*(gamma*dy - xh*mean(gamma*dy*xh)) (+ dres if not NULL), xh = x*rstd;
 * dgamma[H] += sum_t dy*xh (fixed summation order).  ws: dh_rmsnorm_bwd_ws_bytes(T,H) bytes. */
int dh_rmsnorm_bwd(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                   const float* rstd, const void* dres, void* dx, float* dgamma, void* ws,
                   size_t ws_bytes, void* stream);
size_t dh_rmsnorm_bwd_ws_bytes(int T, int H);

/* dh_rmsnorm_bwd for callers that cannot allocate or carry a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments and results (bitwise) without ws: the partial rows of the gain
 * gradient go to a static device array of dh_rmsnorm_bwd_noalloc_max_bytes() (8 MiB) that every GPU the library runs on
 * holds until the process ends.  The call allocates and frees nothing; dh_rmsnorm_bwd_ws_bytes(T,H) above that limit
 * returns DH_ERR_WORKSPACE_TOO_SMALL.  All calls on one GPU share the array: calls that overlap on one GPU (two
 * streams, two threads) race; calls on one stream are safe. */
int dh_rmsnorm_bwd_noalloc(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                           const float* rstd, const void* dres, void* dx, float* dgamma, void* stream);
size_t dh_rmsnorm_bwd_noalloc_max_bytes(void);

/* RoPE pair i of a head of d elements: DH_ROPE_HALVES = elements (i, i + d/2), DH_ROPE_ADJACENT = elements
 * (2i, 2i + 1).  Attention does not care (both are the same rotation up to a fixed permutation of the head's
 * elements); what matters is that weights trained with one convention meet the same one. */
typedef enum { DH_ROPE_HALVES = 0, DH_ROPE_ADJACENT = 1 } dh_rope_pairing;
/* GeLU of the GPT-style MLP (Table 2): DH_GELU_TANH = 0.5 f (1 + tanh(sqrt(2/pi)(f + 0.044715 f^3))),
 * DH_GELU_ERF = f Phi(f) = 0.5 f (1 + erf(f / sqrt 2)). */
typedef enum { DH_GELU_TANH = 0, DH_GELU_ERF = 1 } dh_gelu_form;

/* Rotary embedding in place on n_heads heads stored side by side at the start of each row of
 * row_stride elements: pair (i, i+d/2) of a token at position p (= row % seq) turns by
 * p * base^(-2i/d); inverse != 0 turns back (the backward of the rotation). */
int dh_rope(int dtype, int T, int seq, int n_heads, int head_dim, int row_stride, float base,
            int inverse, void* t, void* stream);
/* The same with position p = pos0 + row % seq: the rows of a context-parallel rank (Sec. 2.1, "Intra-layer
 * parallelism") are a later chunk of each sequence. */
int dh_rope_at(int dtype, int T, int seq, int pos0, int n_heads, int head_dim, int row_stride, float base,
               int inverse, void* t, void* stream);
/* The same with the pairing convention given (dh_rope_pairing); dh_rope and dh_rope_at use DH_ROPE_HALVES. */
int dh_rope_pairs(int dtype, int pairing, int T, int seq, int pos0, int n_heads, int head_dim, int row_stride,
                  float base, int inverse, void* t, void* stream);

/* SwiGLU: gu[T,2F] = [gate | up]; a[T,F] = gate*sigmoid(gate)*up; backward writes dgu[T,2F]. */
int dh_swiglu_fwd(int dtype, int T, int F, const void* gu, void* a, void* stream);
int dh_swiglu_bwd(int dtype, int T, int F, const void* gu, const void* da, void* dgu, void* stream);

/* out[i] = a[i] + b[i], n elements (n multiple of 8): the residual of the bias-dropout-add operator. */
int dh_add(int dtype, size_t n, const void* a, const void* b, void* out, void* stream);

/* Causal grouped-query attention (FlashAttention operator base, Table 2).  qkv[T,(nq+2nkv)d] =
 * [q heads | k heads | v heads] (already rotated); o[T,nq*d]; lse[nq,T] natural-log sum-exp of the
 * scaled masked scores; attention is per sequence (T = batch*seq).  Backward writes dqkv (same
 * layout as qkv; dk,dv summed over the query heads of each group in head order) and uses
 * delta[nq,T] and ws (dh_attn_bwd_workspace_bytes; per-head float32 dk,dv partials when nq > nkv)
 * as scratch.  Forward: ws (dh_attn_fwd_workspace_bytes) lets long causal rows be split over several
 * blocks whose float32 partial results are merged in a fixed order; with ws == NULL (or too small) the
 * rows are not split and results differ in rounding only. */
int dh_attn_fwd(int dtype, int batch, int seq, int nq, int nkv, int d, const void* qkv, void* o,
                float* lse, void* ws, size_t ws_bytes, void* stream);
size_t dh_attn_fwd_workspace_bytes(int dtype, int batch, int seq, int nq, int nkv, int d);
int dh_attn_bwd(int dtype, int batch, int seq, int nq, int nkv, int d, const void* qkv, const void* o,
                const void* dout, const float* lse, void* dqkv, float* delta, void* ws, size_t ws_bytes,
                void* stream);
size_t dh_attn_bwd_workspace_bytes(int dtype, int batch, int seq, int nq, int nkv, int d);

/* Attention of a context-parallel rank (Sec. 2.1: the token sequence is partitioned over the CP ranks and each
 * collects the others' key/value tensors; Sec. 2.1 and 2.3: by Send/Recv, ring-attention style).  The rank's seq queries
 * per sequence sit at positions q_off .. q_off+seq-1 and read, causally, the keys/values of positions
 * 0 .. q_off+seq-1 from kv[batch*(q_off+seq), 2*nkv*d] = [k heads | v heads] per row (keys rotated), sequence-major:
 * q_off rows received from the earlier ranks, then the rank's own.  qkv, o, lse, dout, delta are as in dh_attn_fwd /
 * dh_attn_bwd with T = batch*seq; only the q columns of qkv are read and only the q columns of dqkv written; dk,dv of
 * every key row go to dkv (layout of kv): the rows of earlier chunks are what the rank sends back to their owners.
 * q_off = 0 reduces to dh_attn_fwd/bwd with keys and values held apart.  bf16: q_off must be a multiple of 128;
 * workspaces from the _ctx_ queries below.  Device pointers; nothing is allocated. */
int dh_attn_ctx_fwd(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d, const void* qkv,
                    const void* kv, void* o, float* lse, void* ws, size_t ws_bytes, void* stream);
size_t dh_attn_ctx_fwd_workspace_bytes(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d);
int dh_attn_ctx_bwd(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d, const void* qkv,
                    const void* kv, const void* o, const void* dout, const float* lse, void* dqkv, void* dkv,
                    float* delta, void* ws, size_t ws_bytes, void* stream);
size_t dh_attn_ctx_bwd_workspace_bytes(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d);

/* ------------------------------------------------------------------------------------------
 * Mixture-of-experts operators (Sec. 6.1, top-2 gating; operator bases Router, Permute, AlltoAll and
 * Group-GEMM of Table 2).  Expert parallelism on one GPU: the E logical experts are
 * e = source_rank * n_local + local_expert; this GPU holds the n_local local experts and receives
 * every source rank's rows for them.  All index work is integer and deterministic.
 * ------------------------------------------------------------------------------------------ */

/* Router: logits[T,E] float32 -> idx[T,2] (largest logit first; ties go to the lower expert id) and
 * prob[T,2] = softmax over the two kept logits.  2 <= E <= 256. */
int dh_moe_route(int T, int E, const float* logits, int32_t* idx, float* prob, void* stream);
/* dlogits[T,E] = gradient of the router given dprob[T,2]; zero outside the two kept experts. */
int dh_moe_route_bwd(int T, int E, const float* dprob, const int32_t* idx, const float* prob,
                     float* dlogits, void* stream);

/* Index tables of one routing decision, all int32 device arrays owned by the caller.  "Assignment"
 * a = 2t+k is token t's k-th expert.  Send order: assignments grouped by expert ascending, inside an
 * expert by a ascending (stable).  Receive order: [local expert][source rank], same order inside. */
typedef struct {
  int32_t* rank;         /* [2T]   scratch: position of assignment a among its expert's rows     */
  int32_t* dest;         /* [2T]   send row of assignment a                                      */
  int32_t* src_tok;      /* [2T]   token of send row r                                           */
  int32_t* send_of_recv; /* [2T]   send row copied into receive row j (all-to-all dispatch map)  */
  int32_t* recv_of_send; /* [2T]   receive row of send row r (all-to-all combine map)            */
  int32_t* counts;       /* [E]    rows per logical expert                                       */
  int32_t* offsets;      /* [E+1]  first send row of each logical expert                         */
  int32_t* recv_start;   /* [E]    first receive row of each logical expert                      */
  int32_t* group_rows;   /* [n_local] rows per local expert (dh_gemm_grouped reads it on the device)     */
} dh_moe_tables;
/* Fills every table from idx[T,2].  E % n_local must be 0. */
int dh_moe_plan(int T, int E, int n_local, const int32_t* idx, const dh_moe_tables* tables,
                void* stream);

/* out[r,:] = in[map[r],:] for r < n_rows, rows of H elements (H % 8 == 0); map must be in range of
 * `in`.  Serves as the token permute (map = src_tok) and as the all-to-all stand-in: a memory-bound
 * copy of exactly the payload (dispatch: map = send_of_recv, combine: map = recv_of_send).
 * n_blocks: 256-thread blocks it may use (0 = cover the payload, at most 4096). */
int dh_moe_gather_rows(int dtype, int n_rows, int H, const void* in, const int32_t* map, void* out,
                       int n_blocks, void* stream);

/* Un-permute: y[t,:] = prob[t,0]*yp[dest[2t],:] + prob[t,1]*yp[dest[2t+1],:] (+ residual[t,:] if not
 * NULL); prob == NULL means weights 1 (the backward of the token permute). */
int dh_moe_combine(int dtype, int T, int H, const void* yp, const int32_t* dest, const float* prob,
                   const void* residual, void* y, void* stream);
/* Backward of the weighted un-permute: dyp[dest[2t+k],:] = prob[t,k]*dy[t,:] and
 * dprob[t,k] = <dy[t,:], yp[dest[2t+k],:]> (float32). */
int dh_moe_combine_bwd(int dtype, int T, int H, const void* dy, const void* yp, const int32_t* dest,
                       const float* prob, void* dyp, float* dprob, void* stream);

/* Grouped GEMM over row groups that are stored back to back; group g has group_rows[g] rows, a DEVICE
 * int32 array (the counts come out of the routing, no host round trip); max_rows is a host-side upper
 * bound on any group's rows (e.g. the total row count) that sizes the grid.
 *   mode 0  C[rows_g, dim_b]  = A[rows_g, dim_a]   * B_g[dim_a, dim_b]          (expert forward)
 *   mode 1  C[rows_g, dim_b]  = A[rows_g, dim_a]   * B_g[dim_b, dim_a]^T        (data gradient)
 *   mode 2  C_g[dim_a, dim_b] += A[rows_g, dim_a]^T * B[rows_g, dim_b], float32 (weight gradient)
 * dim_a, dim_b multiples of 8 for DH_BF16; at most 64 groups. */
int dh_gemm_grouped(int dtype, int mode, int n_groups, const int32_t* group_rows, int max_rows,
                    int dim_a, int dim_b, const void* A, const void* B, void* C, void* stream);

/* A bf16 GEMM and an all-reduce stand-in in ONE launch (the direction the closing paragraph of the cross-node analysis
 * of Sec. 6.3 / Table 7 names: computation and communication inside one kernel, so that their shares of the machine
 * are fixed in the kernel and not by the dispatcher).  The launch's first blocks -- as many threads as n_blocks
 * 256-thread blocks of dh_comm_standin -- stream the payload and hold their compute units until it is through; the
 * GEMM's tiles take the other units.  C (+)= opA(A) opB(B) exactly as dh_gemm (bf16, no bias), ar_out = the sum of the
 * n_ranks bf16 partial buffers of ar_elems elements exactly as dh_comm_standin(DH_COMM_ALLREDUCE): both results are
 * bit-identical to the two separate calls.  The two halves are independent: the payload is NOT the GEMM's result.
 * Fits (dh_gemm_allreduce_fits = 1) when the GEMM is a single launch without workspace (no K split, no tail launch);
 * otherwise DH_ERR_UNSUPPORTED.  All pointers device, 16-byte aligned; parts is a host array of n_ranks device
 * pointers; nothing is allocated. */
int dh_gemm_allreduce_fits(int trans_a, int trans_b, int M, int N, int K);
int dh_gemm_allreduce(int trans_a, int trans_b, int M, int N, int K, const void* A, const void* B, void* C,
                      int out_f32_accumulate, int n_ranks, const void* const* parts, void* ar_out, size_t ar_elems,
                      int n_blocks, void* stream);

/* The feed-forward block's SwiGLU (operator ACT of the layer, Sec. 4.2's operator list; Table 2 bases it on an
 * element-wise kernel) run inside the epilogue of the GEMM next to it, bf16 only, so that the activation costs no
 * launch and no second pass over the gate/up tensor.  Results are bit-identical to dh_gemm followed by
 * dh_swiglu_fwd / dh_swiglu_bwd.  All pointers device, row-major, 16-byte aligned; nothing is allocated.
 *   forward : gu[T,2F] = x[T,H] * w_gate_up[H,2F] (columns [gate | up]), a[T,F] = gate * sigmoid(gate) * up.
 *             Fits (dh_gemm_swiglu_fwd_fits = 1) when T % 256 == 0, F % 128 == 0, H % 32 == 0 and the plain GEMM
 *             would be a single launch of 256x256 tiles.
 *   backward: dgu[T,2F] = (d gate | d up) from dA = dy[T,H] * w_down[F,H]^T (never stored) and gu[T,2F].
 *             Fits when the plain GEMM would be a single launch of whole tiles without a K split.
 * A shape that does not fit returns DH_ERR_UNSUPPORTED (the caller then uses the two separate operators, as the
 * layer does); null pointers DH_ERR_INVALID_ARG. */
int dh_gemm_swiglu_fwd_fits(int T, int F, int H);
int dh_gemm_swiglu_fwd(int T, int F, int H, const void* x, const void* w_gate_up, void* gu, void* a, void* stream);
int dh_gemm_swiglu_bwd_fits(int T, int F, int H);
int dh_gemm_swiglu_bwd(int T, int F, int H, const void* dy, const void* w_down, const void* gu, void* dgu, void* stream);

/* dh_gemm with a bias row: C = opA(A)*opB(B) + bias[N] (bias in the operand dtype; stored results only). */
int dh_gemm_bias(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, const void* B,
                 const void* bias, void* C, int out_f32_accumulate, void* ws, size_t ws_bytes,
                 void* stream);

/* ------------------------------------------------------------------------------------------
 * Operators of the GPT-style dense layer (Table 2: LayerNorm, GeLU activation, fused
 * bias-dropout-add with p = 0).
 * ------------------------------------------------------------------------------------------ */
/* LayerNorm forward.  If residual != NULL: x_out = x + residual (+ residual_bias[H] if not NULL) is
 * stored and normalised, else x is.  h = gamma*(x-mu)*rstd + beta; mu[T], rstd[T] float32 (biased
 * variance). */
int dh_layernorm_fwd(int dtype, int T, int H, const void* x, const void* residual,
                     const void* residual_bias, const void* gamma, const void* beta, float eps,
                     void* x_out, void* h, float* mu, float* rstd, void* stream);
/* LayerNorm backward: dx = rstd*(gh - mean(gh) - xh*mean(gh*xh)) (+ dres if not NULL), gh = gamma*dy,
 * xh = (x-mu)*rstd; dgamma[H] += sum_t dy*xh, dbeta[H] += sum_t dy (float32, fixed order). */
int dh_layernorm_bwd(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                     const float* mu, const float* rstd, const void* dres, void* dx, float* dgamma,
                     float* dbeta, void* ws, size_t ws_bytes, void* stream);
size_t dh_layernorm_bwd_ws_bytes(int T, int H);

/* GeLU, tanh form: a = 0.5 f (1 + tanh(sqrt(2/pi)(f + 0.044715 f^3))); backward df = da * gelu'(f).
 * n elements, n % 8 == 0. */
int dh_gelu_fwd(int dtype, size_t n, const void* f, void* a, void* stream);
int dh_gelu_bwd(int dtype, size_t n, const void* f, const void* da, void* df, void* stream);
/* The same with the form given (dh_gelu_form); backward of the erf form: df = da (Phi(f) + f phi(f)). */
int dh_gelu_fwd_form(int dtype, int form, size_t n, const void* f, void* a, void* stream);
int dh_gelu_bwd_form(int dtype, int form, size_t n, const void* f, const void* da, void* df, void* stream);

/* out[t,:] = a[t,:] + b[t,:] + bias[:]: bias-dropout-add with p = 0 and the residual. */
int dh_bias_residual_add(int dtype, int T, int H, const void* a, const void* b, const void* bias,
                         void* out, void* stream);

/* out[N] += sum_t x[t,:] in float32, fixed summation order (bias gradients). */
int dh_colsum(int dtype, int T, int N, const void* x, float* out, void* ws, size_t ws_bytes,
              void* stream);
size_t dh_colsum_ws_bytes(int T, int N);

#ifdef __cplusplus
}
#endif
#endif
