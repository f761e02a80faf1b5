// The layer object, its operator tables for the three architectures, single-strand forward/backward,
// the Strand-Interleaving executor (paper Sec. 3.3 and 5) and the pairwise overlap profiler (Sec. 3.2).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>
#include "common.h"

#define DH_EVENT_POOL 256

struct dh_layer {
  dh_layer_config c;
  int T;      // tokens of the micro-batch
  int Ts;     // rows of the layer's input/output (T, or T / n_ranks under sequence parallelism)
  int Tf;     // rows entering the FFN GEMMs (T, or 2T routed rows for the MoE)
  int n_qkv, n_o;
  size_t es;  // bytes per activation element
  dh_weights w;
  dh_wgrads g;
  bool have_w, have_g;
  // saved-slot offsets (bytes)
  size_t s_mu1, s_rstd1, s_h1, s_qkv, s_o, s_lse, s_x2, s_mu2, s_rstd2, s_h2, s_gu, s_a;
  size_t s_idx, s_prob, s_tab[9], s_xg, s_yp, s_kv, saved_bytes;
  int q_off, kv_w;  // context parallelism: first position of this rank's chunk; elements of a key/value row
  size_t f_kvrecv, b_dkv;
  hipStream_t cross_stream;
  hipStream_t beta_comm_stream;  // beta's collectives in SI steps (nullptr: where alpha's go)
  // SwiGLU runs in the epilogue of the gate/up projection (forward) / of the down projection's data gradient (backward)
  // where the shapes allow; the activation operator of that direction then launches nothing
  bool fuse_act_fwd, fuse_act_bwd;
  // backward all-reduces carried by a weight-gradient GEMM's launch: bit 1 = B_AR3 with B_FC1_WGRAD, bit 2 = B_AR4 with
  // B_QKV_WGRAD; in force only while the stand-ins run on a block budget (comm_blocks > 0)
  int fuse_comm;
  // forward workspace offsets
  size_t f_hs, f_part, f_red, f_xp, f_yg, f_attn, f_attn_bytes, f_gemm, f_gemm_bytes, fwd_bytes;
  // backward workspace offsets
  size_t b_dz, b_da, b_dgu, b_part, b_red, b_dx2, b_dy, b_do, b_dqkv, b_delta, b_attn, b_attn_bytes, b_norm, b_norm_bytes;
  size_t b_colsum, b_colsum_bytes, b_dyp, b_dprob, b_dyg, b_dxg, b_gemm, b_gemm_bytes, bwd_bytes;
  hipEvent_t ev[DH_EVENT_POOL];  // created on the first SI step (needs a device)
  bool have_events;
  int ev_next;
  dh_op_graph gf, gb;
};

static const char* kLlamaFwd[DH_F_NOPS] = {"F_NORM1", "F_QKV", "F_ROPE", "F_ATTN", "F_PROJ", "F_AR1",
                                           "F_NORM2", "F_FC1", "F_ACT", "F_FC2", "F_AR2", "F_BDA2"};
static const char* kLlamaBwd[DH_B_NOPS] = {"B_FC2_DGRAD", "B_FC2_WGRAD", "B_ACT", "B_FC1_DGRAD", "B_FC1_WGRAD",
                                           "B_AR3", "B_NORM2", "B_PROJ_DGRAD", "B_PROJ_WGRAD", "B_ATTN",
                                           "B_ROPE", "B_QKV_DGRAD", "B_QKV_WGRAD", "B_AR4", "B_NORM1"};
static const char* kGptFwd[DH_GF_NOPS] = {"F_NORM1", "F_AG1", "F_QKV", "F_ATTN", "F_PROJ", "F_RS1", "F_NORM2",
                                          "F_AG2", "F_FC1", "F_ACT", "F_FC2", "F_RS2", "F_BDA2"};
static const char* kGptBwd[DH_GB_NOPS] = {"B_AG3", "B_FC2_DGRAD", "B_FC2_WGRAD", "B_ACT", "B_FC1_DGRAD", "B_FC1_WGRAD",
                                          "B_RS3", "B_NORM2", "B_AG4", "B_PROJ_DGRAD", "B_PROJ_WGRAD", "B_ATTN",
                                          "B_QKV_DGRAD", "B_QKV_WGRAD", "B_RS4", "B_NORM1"};
static const char* kCpFwd[DH_CF_NOPS] = {"F_NORM1", "F_QKV", "F_ROPE", "F_CP_KV", "F_ATTN", "F_PROJ", "F_AR1",
                                         "F_NORM2", "F_FC1", "F_ACT", "F_FC2", "F_AR2", "F_BDA2"};
static const char* kCpBwd[DH_CB_NOPS] = {"B_FC2_DGRAD", "B_FC2_WGRAD", "B_ACT", "B_FC1_DGRAD", "B_FC1_WGRAD", "B_AR3",
                                         "B_NORM2", "B_PROJ_DGRAD", "B_PROJ_WGRAD", "B_ATTN", "B_CP_DKV", "B_CP_SEND", "B_ROPE",
                                         "B_QKV_DGRAD", "B_QKV_WGRAD", "B_AR4", "B_NORM1"};
static const char* kMoeFwd[DH_MF_NOPS] = {"F_NORM1", "F_QKV", "F_ROPE", "F_ATTN", "F_PROJ", "F_NORM2", "F_ROUTE",
                                          "F_PERMUTE", "F_A2A_DISPATCH", "F_FC1", "F_ACT", "F_FC2", "F_A2A_COMBINE",
                                          "F_UNPERMUTE"};
static const char* kMoeBwd[DH_MB_NOPS] = {"B_UNPERMUTE", "B_ROUTE", "B_A2A_DISPATCH", "B_FC2_DGRAD", "B_FC2_WGRAD", "B_ACT",
                                          "B_FC1_DGRAD", "B_FC1_WGRAD", "B_A2A_COMBINE", "B_PERMUTE", "B_NORM2",
                                          "B_PROJ_DGRAD", "B_PROJ_WGRAD", "B_ATTN", "B_ROPE", "B_QKV_DGRAD", "B_QKV_WGRAD",
                                          "B_NORM1"};

extern "C" const char* dh_op_name(int arch, int direction, int op) {
  if (direction != 0 && direction != 1) return nullptr;
  const char* const* names;
  int n;
  switch (arch) {
    case DH_ARCH_LLAMA: names = direction ? kLlamaBwd : kLlamaFwd; n = direction ? DH_B_NOPS : DH_F_NOPS; break;
    case DH_ARCH_GPT: names = direction ? kGptBwd : kGptFwd; n = direction ? DH_GB_NOPS : DH_GF_NOPS; break;
    case DH_ARCH_MOE: names = direction ? kMoeBwd : kMoeFwd; n = direction ? DH_MB_NOPS : DH_MF_NOPS; break;
    case DH_ARCH_LLAMA_CP: names = direction ? kCpBwd : kCpFwd; n = direction ? DH_CB_NOPS : DH_CF_NOPS; break;
    default: return nullptr;
  }
  return op >= 0 && op < n ? names[op] : nullptr;
}

static void add_dep(dh_op_graph& g, int s, int d) {
  g.dep_src[g.n_deps] = s;
  g.dep_dst[g.n_deps] = d;
  g.n_deps++;
}
static void add_chain(dh_op_graph& g, const int* chain, size_t n) {
  for (size_t i = 0; i + 1 < n; i++) add_dep(g, chain[i], chain[i + 1]);
}
#define CHAIN(g, ...)                                       \
  do {                                                      \
    const int _c[] = {__VA_ARGS__};                         \
    add_chain(g, _c, sizeof(_c) / sizeof(int));             \
  } while (0)

// Forward: a chain (the MoE router only needs the logits, so it hangs off nothing).  Backward: the
// data-gradient chain plus the weight-gradient GEMMs, each depending only on the operator that
// produces its dY (Sec. 4.2: wgrad may move in the sequence).
static void build_graphs(dh_layer* L) {
  dh_op_graph& f = L->gf;
  dh_op_graph& b = L->gb;
  memset(&f, 0, sizeof(f));
  memset(&b, 0, sizeof(b));
  if (L->c.arch == DH_ARCH_LLAMA) {
    f.n_ops = DH_F_NOPS;
    for (int i = 0; i + 1 < DH_F_NOPS; i++) add_dep(f, i, i + 1);
    f.is_comm[DH_F_AR1] = f.is_comm[DH_F_AR2] = 1;
    b.n_ops = DH_B_NOPS;
    CHAIN(b, DH_B_FC2_DGRAD, DH_B_ACT, DH_B_FC1_DGRAD, DH_B_AR3, DH_B_NORM2, DH_B_PROJ_DGRAD, DH_B_ATTN, DH_B_ROPE,
          DH_B_QKV_DGRAD, DH_B_AR4, DH_B_NORM1);
    add_dep(b, DH_B_ACT, DH_B_FC1_WGRAD);     // needs dgu
    add_dep(b, DH_B_NORM2, DH_B_PROJ_WGRAD);  // needs dx2
    add_dep(b, DH_B_ROPE, DH_B_QKV_WGRAD);    // needs dqkv
    // FC2_WGRAD needs only the upstream gradient and the saved activation: no predecessor.
    b.is_comm[DH_B_AR3] = b.is_comm[DH_B_AR4] = 1;
    b.side_ok[DH_B_FC2_WGRAD] = b.side_ok[DH_B_FC1_WGRAD] = b.side_ok[DH_B_PROJ_WGRAD] = b.side_ok[DH_B_QKV_WGRAD] = 1;
  } else if (L->c.arch == DH_ARCH_LLAMA_CP) {
    // The other ranks' key/value chunks depend on nothing this rank computes: the exchange has no predecessor and only
    // attention waits for it.  The gradient send-back has no successor.
    f.n_ops = DH_CF_NOPS;
    CHAIN(f, DH_CF_NORM1, DH_CF_QKV, DH_CF_ROPE, DH_CF_ATTN, DH_CF_PROJ, DH_CF_AR1, DH_CF_NORM2, DH_CF_FC1, DH_CF_ACT, DH_CF_FC2,
          DH_CF_AR2, DH_CF_BDA2);
    add_dep(f, DH_CF_CP_KV, DH_CF_ATTN);
    f.is_comm[DH_CF_AR1] = f.is_comm[DH_CF_AR2] = 1;
    f.is_comm[DH_CF_CP_KV] = 2;
    b.n_ops = DH_CB_NOPS;
    CHAIN(b, DH_CB_FC2_DGRAD, DH_CB_ACT, DH_CB_FC1_DGRAD, DH_CB_AR3, DH_CB_NORM2, DH_CB_PROJ_DGRAD, DH_CB_ATTN, DH_CB_CP_DKV,
          DH_CB_ROPE, DH_CB_QKV_DGRAD, DH_CB_AR4, DH_CB_NORM1);
    add_dep(b, DH_CB_ATTN, DH_CB_CP_SEND);
    b.is_comm[DH_CB_CP_SEND] = 2;
    add_dep(b, DH_CB_ACT, DH_CB_FC1_WGRAD);
    add_dep(b, DH_CB_NORM2, DH_CB_PROJ_WGRAD);
    add_dep(b, DH_CB_ROPE, DH_CB_QKV_WGRAD);
    b.is_comm[DH_CB_AR3] = b.is_comm[DH_CB_AR4] = 1;
    b.is_comm[DH_CB_CP_DKV] = 2;
    b.side_ok[DH_CB_FC2_WGRAD] = b.side_ok[DH_CB_FC1_WGRAD] = b.side_ok[DH_CB_PROJ_WGRAD] = b.side_ok[DH_CB_QKV_WGRAD] = 1;
  } else if (L->c.arch == DH_ARCH_GPT) {
    f.n_ops = DH_GF_NOPS;
    for (int i = 0; i + 1 < DH_GF_NOPS; i++) add_dep(f, i, i + 1);
    f.is_comm[DH_GF_AG1] = f.is_comm[DH_GF_RS1] = f.is_comm[DH_GF_AG2] = f.is_comm[DH_GF_RS2] = 1;
    b.n_ops = DH_GB_NOPS;
    CHAIN(b, DH_GB_AG3, DH_GB_FC2_DGRAD, DH_GB_ACT, DH_GB_FC1_DGRAD, DH_GB_RS3, DH_GB_NORM2, DH_GB_AG4, DH_GB_PROJ_DGRAD,
          DH_GB_ATTN, DH_GB_QKV_DGRAD, DH_GB_RS4, DH_GB_NORM1);
    add_dep(b, DH_GB_AG3, DH_GB_FC2_WGRAD);   // needs the gathered dz
    add_dep(b, DH_GB_ACT, DH_GB_FC1_WGRAD);   // needs df
    add_dep(b, DH_GB_AG4, DH_GB_PROJ_WGRAD);  // needs the gathered dy
    add_dep(b, DH_GB_ATTN, DH_GB_QKV_WGRAD);  // needs dqkv
    b.is_comm[DH_GB_AG3] = b.is_comm[DH_GB_RS3] = b.is_comm[DH_GB_AG4] = b.is_comm[DH_GB_RS4] = 1;
  } else {
    f.n_ops = DH_MF_NOPS;
    CHAIN(f, DH_MF_NORM1, DH_MF_QKV, DH_MF_ROPE, DH_MF_ATTN, DH_MF_PROJ, DH_MF_NORM2, DH_MF_PERMUTE, DH_MF_A2A_DISPATCH,
          DH_MF_FC1, DH_MF_ACT, DH_MF_FC2, DH_MF_A2A_COMBINE, DH_MF_UNPERMUTE);
    add_dep(f, DH_MF_ROUTE, DH_MF_PERMUTE);
    f.is_comm[DH_MF_A2A_DISPATCH] = f.is_comm[DH_MF_A2A_COMBINE] = 1;
    b.n_ops = DH_MB_NOPS;
    CHAIN(b, DH_MB_UNPERMUTE, DH_MB_A2A_DISPATCH, DH_MB_FC2_DGRAD, DH_MB_ACT, DH_MB_FC1_DGRAD, DH_MB_A2A_COMBINE,
          DH_MB_PERMUTE, DH_MB_NORM2, DH_MB_PROJ_DGRAD, DH_MB_ATTN, DH_MB_ROPE, DH_MB_QKV_DGRAD, DH_MB_NORM1);
    add_dep(b, DH_MB_UNPERMUTE, DH_MB_ROUTE);          // needs dprob
    add_dep(b, DH_MB_A2A_DISPATCH, DH_MB_FC2_WGRAD);   // needs the dispatched dy rows
    add_dep(b, DH_MB_ACT, DH_MB_FC1_WGRAD);            // needs dgu
    add_dep(b, DH_MB_NORM2, DH_MB_PROJ_WGRAD);         // needs dx2
    add_dep(b, DH_MB_ROPE, DH_MB_QKV_WGRAD);           // needs dqkv
    b.is_comm[DH_MB_A2A_DISPATCH] = b.is_comm[DH_MB_A2A_COMBINE] = 1;
    b.side_ok[DH_MB_FC2_WGRAD] = b.side_ok[DH_MB_FC1_WGRAD] = b.side_ok[DH_MB_PROJ_WGRAD] = b.side_ok[DH_MB_QKV_WGRAD] = 1;
  }
}

// like_other: pairs (forward op, backward op) that run the same kernel on the same amount of data.
static void link_like(dh_op_graph& f, dh_op_graph& b, int fop, int bop) {
  if (f.like_other[fop] == 0) f.like_other[fop] = bop + 1;
  if (b.like_other[bop] == 0) b.like_other[bop] = fop + 1;
}
static void build_likes(dh_layer* L) {
  dh_op_graph& f = L->gf;
  dh_op_graph& b = L->gb;
  switch (L->c.arch) {
    case DH_ARCH_LLAMA:
      link_like(f, b, DH_F_AR1, DH_B_AR3); link_like(f, b, DH_F_AR2, DH_B_AR4);
      link_like(f, b, DH_F_FC1, DH_B_FC1_WGRAD); link_like(f, b, DH_F_FC2, DH_B_FC2_WGRAD);
      link_like(f, b, DH_F_PROJ, DH_B_PROJ_WGRAD); link_like(f, b, DH_F_QKV, DH_B_QKV_WGRAD);
      break;
    case DH_ARCH_LLAMA_CP:
      link_like(f, b, DH_CF_AR1, DH_CB_AR3); link_like(f, b, DH_CF_AR2, DH_CB_AR4);
      link_like(f, b, DH_CF_FC1, DH_CB_FC1_WGRAD); link_like(f, b, DH_CF_FC2, DH_CB_FC2_WGRAD);
      link_like(f, b, DH_CF_PROJ, DH_CB_PROJ_WGRAD); link_like(f, b, DH_CF_QKV, DH_CB_QKV_WGRAD);
      link_like(f, b, DH_CF_CP_KV, DH_CB_CP_SEND); link_like(f, b, DH_CF_CP_KV, DH_CB_CP_DKV);
      break;
    case DH_ARCH_GPT:
      link_like(f, b, DH_GF_AG1, DH_GB_AG3); link_like(f, b, DH_GF_AG2, DH_GB_AG4);
      link_like(f, b, DH_GF_RS1, DH_GB_RS3); link_like(f, b, DH_GF_RS2, DH_GB_RS4);
      link_like(f, b, DH_GF_FC1, DH_GB_FC1_WGRAD); link_like(f, b, DH_GF_FC2, DH_GB_FC2_WGRAD);
      link_like(f, b, DH_GF_PROJ, DH_GB_PROJ_WGRAD); link_like(f, b, DH_GF_QKV, DH_GB_QKV_WGRAD);
      break;
    default:
      link_like(f, b, DH_MF_A2A_DISPATCH, DH_MB_A2A_DISPATCH); link_like(f, b, DH_MF_A2A_COMBINE, DH_MB_A2A_COMBINE);
      link_like(f, b, DH_MF_FC1, DH_MB_FC1_WGRAD); link_like(f, b, DH_MF_FC2, DH_MB_FC2_WGRAD);
      link_like(f, b, DH_MF_PROJ, DH_MB_PROJ_WGRAD); link_like(f, b, DH_MF_QKV, DH_MB_QKV_WGRAD);
      break;
  }
}

extern "C" int dh_layer_op_graph(const dh_layer* layer, int direction, dh_op_graph* out) {
  if (!layer || !out || (direction != 0 && direction != 1)) DH_FAIL(DH_ERR_INVALID_ARG, "layer_op_graph: bad arguments");
  *out = direction == 0 ? layer->gf : layer->gb;
  return DH_OK;
}

static size_t take(size_t& cur, size_t bytes) {
  size_t o = cur;
  cur += dh_align_up(bytes, 256);
  return o;
}

extern "C" int dh_layer_create(const dh_layer_config* cfg, dh_layer** out) {
  if (!cfg || !out) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: null pointer");
  const dh_layer_config& c = *cfg;
  if (c.arch != DH_ARCH_LLAMA && c.arch != DH_ARCH_GPT && c.arch != DH_ARCH_MOE && c.arch != DH_ARCH_LLAMA_CP)
    DH_FAIL(DH_ERR_UNSUPPORTED, "layer_create: arch %d not supported", c.arch);
  if (c.dtype != DH_F32 && c.dtype != DH_BF16) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: dtype %d", c.dtype);
  if (c.batch < 0 || c.seq < 0 || c.hidden <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 || c.ffn <= 0)
    DH_FAIL(DH_ERR_SHAPE, "layer_create: non-positive dimension");
  if (c.n_q_heads % c.n_kv_heads) DH_FAIL(DH_ERR_SHAPE, "layer_create: n_kv_heads %d must divide n_q_heads %d", c.n_kv_heads, c.n_q_heads);
  if (c.hidden % 8 || c.ffn % 8 || c.head_dim % 16) DH_FAIL(DH_ERR_SHAPE, "layer_create: hidden/ffn must be multiples of 8 and head_dim of 16");
  if (c.hidden > 16384) DH_FAIL(DH_ERR_SHAPE, "layer_create: hidden %d above 16384", c.hidden);
  if (c.dtype == DH_BF16 && c.head_dim != 64 && c.head_dim != 128) DH_FAIL(DH_ERR_SHAPE, "layer_create: bf16 needs head_dim 64 or 128");
  if (c.dtype == DH_F32 && c.head_dim > 256) DH_FAIL(DH_ERR_SHAPE, "layer_create: fp32 needs head_dim <= 256");
  if (c.n_ranks < 1 || c.n_ranks > 16) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: n_ranks %d outside 1..16", c.n_ranks);
  if (c.rope_pairing != DH_ROPE_HALVES && c.rope_pairing != DH_ROPE_ADJACENT)
    DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: rope_pairing %d", c.rope_pairing);
  if (c.gelu_form != DH_GELU_TANH && c.gelu_form != DH_GELU_ERF) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: gelu_form %d", c.gelu_form);
  if (c.comm_blocks < 0 || c.comm_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: comm_blocks %d outside 0..65536", c.comm_blocks);
  if ((long long)c.batch * c.seq > (1 << 24)) DH_FAIL(DH_ERR_SHAPE, "layer_create: too many tokens");
  if (c.arch == DH_ARCH_GPT && (c.batch * c.seq) % c.n_ranks)
    DH_FAIL(DH_ERR_SHAPE, "layer_create: sequence parallelism needs tokens %d divisible by n_ranks %d", c.batch * c.seq, c.n_ranks);
  if (c.arch == DH_ARCH_MOE) {
    if (c.n_experts < 2 || c.n_experts > 256 || c.n_local_experts < 1 || c.n_local_experts > 64 || c.n_experts % c.n_local_experts)
      DH_FAIL(DH_ERR_SHAPE, "layer_create: n_experts %d (2..256) must be a multiple of n_local_experts %d (1..64)", c.n_experts, c.n_local_experts);
    if (c.n_ranks != 1) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: the MoE layer has no tensor-parallel peers (n_ranks must be 1)");
  }
  const bool cp = c.arch == DH_ARCH_LLAMA_CP;
  if (cp) {
    if (c.cp_ranks < 1 || c.cp_ranks > 16 || c.cp_rank < 0 || c.cp_rank >= c.cp_ranks)
      DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: cp_rank %d / cp_ranks %d (1..16)", c.cp_rank, c.cp_ranks);
    if ((long long)c.cp_rank * c.seq > (1 << 24)) DH_FAIL(DH_ERR_SHAPE, "layer_create: context too long");
    if (c.dtype == DH_BF16 && (c.cp_rank * c.seq) % 128)
      DH_FAIL(DH_ERR_SHAPE, "layer_create: bf16 context parallelism needs cp_rank*seq = %d to be a multiple of 128", c.cp_rank * c.seq);
    if (c.cross_blocks < 0 || c.cross_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "layer_create: cross_blocks %d outside 0..65536", c.cross_blocks);
  }
  dh_layer* L = new dh_layer();
  L->c = c;
  L->cross_stream = nullptr;
  L->beta_comm_stream = nullptr;
  L->q_off = cp ? c.cp_rank * c.seq : 0;
  L->kv_w = 2 * c.n_kv_heads * c.head_dim;
  L->T = c.batch * c.seq;
  L->Ts = c.arch == DH_ARCH_GPT ? L->T / c.n_ranks : L->T;
  L->Tf = c.arch == DH_ARCH_MOE ? 2 * L->T : L->T;
  const bool glu_layer = c.dtype == DH_BF16 && (c.arch == DH_ARCH_LLAMA || c.arch == DH_ARCH_LLAMA_CP);
  L->fuse_comm = 0;
  L->fuse_act_fwd = glu_layer && dh_glu_fwd_fits(L->T, c.ffn, c.hidden);
  L->fuse_act_bwd = glu_layer && dh_glu_bwd_fits(L->T, c.ffn, c.hidden);
  L->n_qkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  L->n_o = c.n_q_heads * c.head_dim;
  L->es = dh_elem_size(c.dtype);
  L->have_w = L->have_g = false;
  const size_t T = L->T, Ts = L->Ts, Tf = L->Tf, H = c.hidden, F = c.ffn, es = L->es;
  const size_t Fin = c.arch == DH_ARCH_GPT ? F : 2 * F;  // columns of the first FFN GEMM
  const bool moe = c.arch == DH_ARCH_MOE, gpt = c.arch == DH_ARCH_GPT;
  size_t cur = 0;
  L->s_mu1 = take(cur, gpt ? Ts * 4 : 0);
  L->s_rstd1 = take(cur, Ts * 4);
  L->s_h1 = take(cur, T * H * es);
  L->s_qkv = take(cur, T * L->n_qkv * es);
  L->s_o = take(cur, T * L->n_o * es);
  L->s_lse = take(cur, (size_t)c.n_q_heads * T * 4);
  L->s_x2 = take(cur, Ts * H * es);
  L->s_mu2 = take(cur, gpt ? Ts * 4 : 0);
  L->s_rstd2 = take(cur, Ts * 4);
  L->s_h2 = take(cur, T * H * es);
  L->s_gu = take(cur, Tf * Fin * es);
  L->s_a = take(cur, Tf * F * es);
  L->s_idx = take(cur, moe ? 2 * T * 4 : 0);
  L->s_prob = take(cur, moe ? 2 * T * 4 : 0);
  const size_t tab_ints[9] = {2 * T, 2 * T, 2 * T, 2 * T, 2 * T, (size_t)c.n_experts, (size_t)c.n_experts + 1,
                              (size_t)c.n_experts, (size_t)c.n_local_experts};
  for (int i = 0; i < 9; i++) L->s_tab[i] = take(cur, moe ? tab_ints[i] * 4 : 0);
  L->s_xg = take(cur, moe ? Tf * H * es : 0);
  L->s_yp = take(cur, moe ? Tf * H * es : 0);
  const size_t kv_rows = (size_t)c.batch * (L->q_off + c.seq);  // key/value rows a context-parallel rank attends to
  L->s_kv = take(cur, cp ? kv_rows * L->kv_w * es : 0);
  L->saved_bytes = cur;
  const bool bf = c.dtype == DH_BF16;
  auto gw = [&](bool ta, bool tb, size_t M, size_t N, size_t K) {
    return bf ? dh_gemm_bf16_ws_bytes(ta, tb, (int)M, (int)N, (int)K) : (size_t)0;
  };
  cur = 0;
  L->f_hs = take(cur, gpt ? Ts * H * es : 0);
  L->f_part = take(cur, T * H * es);
  L->f_red = take(cur, moe ? 0 : Ts * H * es);
  L->f_xp = take(cur, moe ? Tf * H * es : 0);
  L->f_yg = take(cur, moe ? Tf * H * es : 0);
  L->f_kvrecv = take(cur, cp ? (size_t)(c.cp_ranks - 1 - c.cp_rank) * T * L->kv_w * es : 0);  // later ranks' chunks pass through
  L->f_attn_bytes = bf ? dh_attn_fwd_bf16_ws_bytes(c.batch, c.seq, L->q_off, c.n_q_heads, c.n_kv_heads, c.head_dim) : 0;
  L->f_attn = take(cur, L->f_attn_bytes);
  size_t fg = std::max(gw(0, 0, T, L->n_qkv, H), gw(0, 0, T, H, L->n_o));
  if (!moe) fg = std::max(fg, std::max(gw(0, 0, T, Fin, H), gw(0, 0, T, H, F)));
  if (!gpt) {  // weight-gradient GEMMs that run beside their strand borrow this workspace
    fg = std::max(fg, std::max(gw(1, 0, L->n_o, H, T), gw(1, 0, H, L->n_qkv, T)));
    if (!moe) fg = std::max(fg, std::max(gw(1, 0, F, H, T), gw(1, 0, H, Fin, T)));
  }
  L->f_gemm_bytes = fg;
  L->f_gemm = take(cur, fg);
  L->fwd_bytes = cur;
  cur = 0;
  L->b_dz = take(cur, gpt ? T * H * es : 0);
  L->b_da = take(cur, Tf * F * es);
  L->b_dgu = take(cur, Tf * Fin * es);
  L->b_part = take(cur, T * H * es);
  L->b_red = take(cur, Ts * H * es);
  L->b_dx2 = take(cur, Ts * H * es);
  L->b_dy = take(cur, gpt ? T * H * es : 0);
  L->b_do = take(cur, T * L->n_o * es);
  L->b_dqkv = take(cur, T * L->n_qkv * es);
  L->b_delta = take(cur, (size_t)c.n_q_heads * T * 4);
  L->b_dkv = take(cur, cp ? kv_rows * L->kv_w * es : 0);
  L->b_attn_bytes = bf ? dh_attn_bwd_bf16_ws_bytes(c.batch, c.seq, L->q_off, c.n_q_heads, c.n_kv_heads, c.head_dim) : 0;
  L->b_attn = take(cur, L->b_attn_bytes);
  L->b_norm_bytes = gpt ? dh_layernorm_bwd_ws_bytes(L->Ts, c.hidden) : dh_rmsnorm_bwd_ws_bytes(L->Ts, c.hidden);
  L->b_norm = take(cur, L->b_norm_bytes);
  L->b_colsum_bytes = gpt ? dh_colsum_ws_bytes(L->T, (int)std::max(std::max(H, F), (size_t)L->n_qkv)) : 0;
  L->b_colsum = take(cur, L->b_colsum_bytes);
  L->b_dyp = take(cur, moe ? Tf * H * es : 0);
  L->b_dprob = take(cur, moe ? 2 * T * 4 : 0);
  L->b_dyg = take(cur, moe ? Tf * H * es : 0);
  L->b_dxg = take(cur, moe ? Tf * H * es : 0);
  size_t gb = 0;
  if (!moe) {
    gb = std::max(gb, gw(0, 1, T, F, H));      // da = dz * Wd^T
    gb = std::max(gb, gw(1, 0, F, H, T));      // dWd
    gb = std::max(gb, gw(0, 1, T, H, Fin));    // dh2 = dgu * Wgu^T
    gb = std::max(gb, gw(1, 0, H, Fin, T));    // dWgu
  }
  gb = std::max(gb, gw(0, 1, T, L->n_o, H));      // do = dx2 * Wo^T
  gb = std::max(gb, gw(1, 0, L->n_o, H, T));      // dWo
  gb = std::max(gb, gw(0, 1, T, H, L->n_qkv));    // dh1 = dqkv * Wqkv^T
  gb = std::max(gb, gw(1, 0, H, L->n_qkv, T));    // dWqkv
  L->b_gemm_bytes = gb;
  L->b_gemm = take(cur, gb);
  L->bwd_bytes = cur;
  build_graphs(L);
  build_likes(L);
  for (int i = 0; i < DH_EVENT_POOL; i++) L->ev[i] = nullptr;
  L->have_events = false;
  L->ev_next = 0;
  *out = L;
  return DH_OK;
}

extern "C" void dh_layer_destroy(dh_layer* L) {
  if (!L) return;
  for (int i = 0; i < DH_EVENT_POOL; i++)
    if (L->ev[i]) (void)hipEventDestroy(L->ev[i]);
  delete L;
}

extern "C" int dh_layer_bind_weights(dh_layer* L, const dh_weights* w) {
  if (!L || !w) DH_FAIL(DH_ERR_INVALID_ARG, "bind_weights: null pointer");
  if (!w->g1 || !w->Wqkv || !w->Wo || !w->g2 || !w->Wgu || !w->Wd) DH_FAIL(DH_ERR_INVALID_ARG, "bind_weights: a weight pointer is null");
  if (L->c.arch == DH_ARCH_GPT && (!w->b1 || !w->bqkv || !w->bo || !w->b2 || !w->bfc1 || !w->bfc2))
    DH_FAIL(DH_ERR_INVALID_ARG, "bind_weights: a bias pointer is null");
  L->w = *w;
  L->have_w = true;
  return DH_OK;
}

extern "C" int dh_layer_bind_wgrads(dh_layer* L, const dh_wgrads* g) {
  if (!L || !g) DH_FAIL(DH_ERR_INVALID_ARG, "bind_wgrads: null pointer");
  if (!g->dg1 || !g->dWqkv || !g->dWo || !g->dg2 || !g->dWgu || !g->dWd) DH_FAIL(DH_ERR_INVALID_ARG, "bind_wgrads: a gradient pointer is null");
  if (L->c.arch == DH_ARCH_GPT && (!g->db1 || !g->dbqkv || !g->dbo || !g->db2 || !g->dbfc1 || !g->dbfc2))
    DH_FAIL(DH_ERR_INVALID_ARG, "bind_wgrads: a bias gradient pointer is null");
  L->g = *g;
  L->have_g = true;
  return DH_OK;
}

extern "C" size_t dh_layer_saved_bytes(const dh_layer* L) { return L ? L->saved_bytes : 0; }

extern "C" int dh_layer_set_cross_stream(dh_layer* L, void* stream_cross) {
  if (!L) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_cross_stream: null layer");
  L->cross_stream = (hipStream_t)stream_cross;
  return DH_OK;
}

extern "C" int dh_layer_set_fused_collective(dh_layer* L, int mask) {
  if (!L) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_fused_collective: null layer");
  if (mask < 0 || mask > 3) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_fused_collective: mask %d outside 0..3", mask);
  const dh_layer_config& c = L->c;
  const bool ok = c.dtype == DH_BF16 && (c.arch == DH_ARCH_LLAMA || c.arch == DH_ARCH_LLAMA_CP) && L->T > 0;
  int m = 0;
  if (ok && (mask & 1) && dh_gemm_ar_fits(true, false, c.hidden, 2 * c.ffn, L->T)) m |= 1;
  if (ok && (mask & 2) && dh_gemm_ar_fits(true, false, c.hidden, L->n_qkv, L->T)) m |= 2;
  L->fuse_comm = m;
  return m;
}

extern "C" int dh_layer_set_fused_activation(dh_layer* L, int enable) {
  if (!L) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_fused_activation: null layer");
  const dh_layer_config& c = L->c;
  const bool glu_layer = c.dtype == DH_BF16 && (c.arch == DH_ARCH_LLAMA || c.arch == DH_ARCH_LLAMA_CP);
  if (enable < 0 || enable > 3) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_fused_activation: mask %d outside 0..3", enable);
  L->fuse_act_fwd = (enable & 1) && glu_layer && dh_glu_fwd_fits(L->T, c.ffn, c.hidden);
  L->fuse_act_bwd = (enable & 2) && glu_layer && dh_glu_bwd_fits(L->T, c.ffn, c.hidden);
  return (L->fuse_act_fwd ? 1 : 0) | (L->fuse_act_bwd ? 2 : 0);
}

extern "C" int dh_layer_set_beta_comm_stream(dh_layer* L, void* stream_comm_beta) {
  if (!L) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_beta_comm_stream: null layer");
  L->beta_comm_stream = (hipStream_t)stream_comm_beta;
  return DH_OK;
}

extern "C" int dh_layer_set_comm_blocks(dh_layer* L, int comm_blocks) {
  if (!L) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_comm_blocks: null layer");
  if (comm_blocks < -1 || comm_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "layer_set_comm_blocks: %d outside -1..65536", comm_blocks);
  L->c.comm_blocks = comm_blocks;
  return DH_OK;
}

extern "C" size_t dh_layer_workspace_bytes(const dh_layer* L, int kind) {
  if (!L) return 0;
  if (kind == DH_WS_FWD) return L->fwd_bytes;
  if (kind == DH_WS_BWD) return L->bwd_bytes;
  if (kind == DH_WS_SI) return L->fwd_bytes + L->bwd_bytes;
  return 0;
}

// ------------------------------------------------------------------------------------ operators
static int gemm(const dh_layer* L, bool ta, bool tb, int M, int N, int K, const void* A, const void* B, void* C, bool acc,
                void* ws, size_t ws_bytes, hipStream_t s, const void* bias = nullptr) {
  if (L->c.dtype == DH_BF16)
    return dh_launch_gemm_bf16(ta, tb, M, N, K, (const bf16_t*)A, (const bf16_t*)B, C, acc, (const bf16_t*)bias, ws, ws_bytes, s);
  return dh_launch_gemm_f32(ta, tb, M, N, K, (const float*)A, (const float*)B, (float*)C, acc, (const float*)bias, s);
}

// Collective stand-in over parts = {own, peers[0], ..., peers[R-2]}, each `elems` elements.
static int collective(const dh_layer* L, int kind, const void* own, const void* peers, size_t elems, void* out, hipStream_t s) {
  const void* parts[16];
  parts[0] = own;
  for (int r = 1; r < L->c.n_ranks; r++) parts[r] = (const char*)peers + (size_t)(r - 1) * elems * L->es;
  return dh_comm_standin(kind, L->c.n_ranks, parts, out, elems, L->c.dtype, L->c.comm_blocks, (void*)s);
}

// Whether backward all-reduce `which` (1: AR3, 2: AR4) is carried by its weight-gradient GEMM right now.
static bool fused_collective(const dh_layer* L, int which) { return (L->fuse_comm & which) != 0 && L->c.comm_blocks > 0; }

// The all-reduce stand-in over {own, peers...} and an unrelated bf16 GEMM in one launch.
static int collective_with_gemm(const dh_layer* L, const void* own, const void* peers, size_t elems, void* out, bool ta, bool tb, int M,
                                int N, int K, const void* A, const void* B, void* C, bool acc, hipStream_t s) {
  const void* parts[16];
  parts[0] = own;
  for (int r = 1; r < L->c.n_ranks; r++) parts[r] = (const char*)peers + (size_t)(r - 1) * elems * L->es;
  return dh_launch_gemm_bf16_ar(ta, tb, M, N, K, (const bf16_t*)A, (const bf16_t*)B, C, acc, L->c.n_ranks, parts, (bf16_t*)out, elems,
                                L->c.comm_blocks, s);
}

static dh_moe_tables moe_tables_of(const dh_layer* L, const void* saved) {
  char* sv = (char*)saved;
  dh_moe_tables t;
  t.rank = (int32_t*)(sv + L->s_tab[0]);
  t.dest = (int32_t*)(sv + L->s_tab[1]);
  t.src_tok = (int32_t*)(sv + L->s_tab[2]);
  t.send_of_recv = (int32_t*)(sv + L->s_tab[3]);
  t.recv_of_send = (int32_t*)(sv + L->s_tab[4]);
  t.counts = (int32_t*)(sv + L->s_tab[5]);
  t.offsets = (int32_t*)(sv + L->s_tab[6]);
  t.recv_start = (int32_t*)(sv + L->s_tab[7]);
  t.group_rows = (int32_t*)(sv + L->s_tab[8]);
  return t;
}

// The attention block's operators are shared by the three architectures.
static int op_attn_fwd(dh_layer* L, char* sv, char* ws, hipStream_t s) {
  const dh_layer_config& c = L->c;
  return dh_attn_fwd(c.dtype, c.batch, c.seq, c.n_q_heads, c.n_kv_heads, c.head_dim, sv + L->s_qkv, sv + L->s_o,
                     (float*)(sv + L->s_lse), ws + L->f_attn, L->f_attn_bytes, s);
}
static int op_attn_bwd(dh_layer* L, const char* sv, char* ws, hipStream_t s) {
  const dh_layer_config& c = L->c;
  return dh_attn_bwd(c.dtype, c.batch, c.seq, c.n_q_heads, c.n_kv_heads, c.head_dim, sv + L->s_qkv, sv + L->s_o, ws + L->b_do,
                     (const float*)(sv + L->s_lse), ws + L->b_dqkv, (float*)(ws + L->b_delta), ws + L->b_attn, L->b_attn_bytes, s);
}
static int op_rope(dh_layer* L, void* qkv, int inverse, hipStream_t s) {
  const dh_layer_config& c = L->c;
  return dh_rope_pairs(c.dtype, c.rope_pairing, L->T, c.seq, 0, c.n_q_heads + c.n_kv_heads, c.head_dim, L->n_qkv, c.rope_base, inverse, qkv, s);
}

static int llama_fwd_op(dh_layer* L, int op, const dh_fwd_args& a, char* ws, hipStream_t s) {
  const dh_layer_config& c = L->c;
  const int T = L->T, H = c.hidden, F = c.ffn, dt = c.dtype;
  char* sv = (char*)a.saved;
  void* gws = ws + L->f_gemm;
  const size_t n = (size_t)T * H;
  switch (op) {
    case DH_F_NORM1:
      return dh_rmsnorm_fwd(dt, T, H, a.x, nullptr, L->w.g1, c.eps, nullptr, sv + L->s_h1, (float*)(sv + L->s_rstd1), s);
    case DH_F_QKV:
      return gemm(L, false, false, T, L->n_qkv, H, sv + L->s_h1, L->w.Wqkv, sv + L->s_qkv, false, gws, L->f_gemm_bytes, s);
    case DH_F_ROPE:
      return op_rope(L, sv + L->s_qkv, 0, s);
    case DH_F_ATTN:
      return op_attn_fwd(L, sv, ws, s);
    case DH_F_PROJ:
      return gemm(L, false, false, T, H, L->n_o, sv + L->s_o, L->w.Wo, ws + L->f_part, false, gws, L->f_gemm_bytes, s);
    case DH_F_AR1:
      return collective(L, DH_COMM_ALLREDUCE, ws + L->f_part, a.peers_ar1, n, ws + L->f_red, s);
    case DH_F_NORM2:  // x2 = x + y (residual of the bias-dropout-add operator), h2 = norm(x2)
      return dh_rmsnorm_fwd(dt, T, H, a.x, ws + L->f_red, L->w.g2, c.eps, sv + L->s_x2, sv + L->s_h2, (float*)(sv + L->s_rstd2), s);
    case DH_F_FC1:
      if (L->fuse_act_fwd)
        return dh_launch_gemm_swiglu_fwd_bf16(T, F, H, (const bf16_t*)(sv + L->s_h2), (const bf16_t*)L->w.Wgu, (bf16_t*)(sv + L->s_gu),
                                              (bf16_t*)(sv + L->s_a), s);
      return gemm(L, false, false, T, 2 * F, H, sv + L->s_h2, L->w.Wgu, sv + L->s_gu, false, gws, L->f_gemm_bytes, s);
    case DH_F_ACT:
      if (L->fuse_act_fwd) return DH_OK;  // done by F_FC1's epilogue
      return dh_swiglu_fwd(dt, T, F, sv + L->s_gu, sv + L->s_a, s);
    case DH_F_FC2:
      return gemm(L, false, false, T, H, F, sv + L->s_a, L->w.Wd, ws + L->f_part, false, gws, L->f_gemm_bytes, s);
    case DH_F_AR2:
      return collective(L, DH_COMM_ALLREDUCE, ws + L->f_part, a.peers_ar2, n, ws + L->f_red, s);
    case DH_F_BDA2:
      return dh_add(dt, n, sv + L->s_x2, ws + L->f_red, a.out, s);
  }
  DH_FAIL(DH_ERR_INVALID_ARG, "unknown forward operator %d", op);
}

// side_ws: a weight-gradient operator that runs beside its strand (on the other strand's stream) takes its GEMM
// workspace from there instead of the backward region, which the strand's own GEMMs are using meanwhile.
static int llama_bwd_op(dh_layer* L, int op, const dh_bwd_args& b, char* ws, hipStream_t s, char* side_ws = nullptr) {
  const dh_layer_config& c = L->c;
  const int T = L->T, H = c.hidden, F = c.ffn, dt = c.dtype;
  const char* sv = (const char*)b.saved;
  void* gws = side_ws ? side_ws : ws + L->b_gemm;
  const size_t gwb = side_ws ? L->f_gemm_bytes : L->b_gemm_bytes, n = (size_t)T * H;
  switch (op) {
    case DH_B_FC2_DGRAD:
      if (L->fuse_act_bwd)
        return dh_launch_gemm_swiglu_bwd_bf16(T, F, H, (const bf16_t*)b.dout, (const bf16_t*)L->w.Wd, (const bf16_t*)(sv + L->s_gu),
                                              (bf16_t*)(ws + L->b_dgu), s);
      return gemm(L, false, true, T, F, H, b.dout, L->w.Wd, ws + L->b_da, false, gws, gwb, s);
    case DH_B_FC2_WGRAD:
      return gemm(L, true, false, F, H, T, sv + L->s_a, b.dout, L->g.dWd, true, gws, gwb, s);
    case DH_B_ACT:
      if (L->fuse_act_bwd) return DH_OK;  // done by B_FC2_DGRAD's epilogue
      return dh_swiglu_bwd(dt, T, F, sv + L->s_gu, ws + L->b_da, ws + L->b_dgu, s);
    case DH_B_FC1_DGRAD:
      return gemm(L, false, true, T, H, 2 * F, ws + L->b_dgu, L->w.Wgu, ws + L->b_part, false, gws, gwb, s);
    case DH_B_FC1_WGRAD:
      if (fused_collective(L, 1)) return DH_OK;  // rides in B_AR3's launch
      return gemm(L, true, false, H, 2 * F, T, sv + L->s_h2, ws + L->b_dgu, L->g.dWgu, true, gws, gwb, s);
    case DH_B_AR3:
      if (fused_collective(L, 1))
        return collective_with_gemm(L, ws + L->b_part, b.peers_ar3, n, ws + L->b_red, true, false, H, 2 * F, T, sv + L->s_h2,
                                    ws + L->b_dgu, L->g.dWgu, true, s);
      return collective(L, DH_COMM_ALLREDUCE, ws + L->b_part, b.peers_ar3, n, ws + L->b_red, s);
    case DH_B_NORM2:  // dx2 = dout + norm2_bwd(dh2)
      return dh_rmsnorm_bwd(dt, T, H, ws + L->b_red, sv + L->s_x2, L->w.g2, (const float*)(sv + L->s_rstd2), b.dout,
                            ws + L->b_dx2, L->g.dg2, ws + L->b_norm, L->b_norm_bytes, s);
    case DH_B_PROJ_DGRAD:
      return gemm(L, false, true, T, L->n_o, H, ws + L->b_dx2, L->w.Wo, ws + L->b_do, false, gws, gwb, s);
    case DH_B_PROJ_WGRAD:
      return gemm(L, true, false, L->n_o, H, T, sv + L->s_o, ws + L->b_dx2, L->g.dWo, true, gws, gwb, s);
    case DH_B_ATTN:
      return op_attn_bwd(L, sv, ws, s);
    case DH_B_ROPE:
      return op_rope(L, ws + L->b_dqkv, 1, s);
    case DH_B_QKV_DGRAD:
      return gemm(L, false, true, T, H, L->n_qkv, ws + L->b_dqkv, L->w.Wqkv, ws + L->b_part, false, gws, gwb, s);
    case DH_B_QKV_WGRAD:
      if (fused_collective(L, 2)) return DH_OK;  // rides in B_AR4's launch
      return gemm(L, true, false, H, L->n_qkv, T, sv + L->s_h1, ws + L->b_dqkv, L->g.dWqkv, true, gws, gwb, s);
    case DH_B_AR4:
      if (fused_collective(L, 2))
        return collective_with_gemm(L, ws + L->b_part, b.peers_ar4, n, ws + L->b_red, true, false, H, L->n_qkv, T, sv + L->s_h1,
                                    ws + L->b_dqkv, L->g.dWqkv, true, s);
      return collective(L, DH_COMM_ALLREDUCE, ws + L->b_part, b.peers_ar4, n, ws + L->b_red, s);
    case DH_B_NORM1:  // dx = dx2 + norm1_bwd(dh1)
      return dh_rmsnorm_bwd(dt, T, H, ws + L->b_red, b.x, L->w.g1, (const float*)(sv + L->s_rstd1), ws + L->b_dx2, b.dx,
                            L->g.dg1, ws + L->b_norm, L->b_norm_bytes, s);
  }
  DH_FAIL(DH_ERR_INVALID_ARG, "unknown backward operator %d", op);
}

// Llama-style layer on one rank of a context-parallel group (Sec. 2.1, 2.2): the Llama operators with rotary
// positions and attention shifted to the rank's chunk, plus the key/value exchange and the gradient send-back.
static int cp_fwd_op(dh_layer* L, int op, const dh_fwd_args& a, char* ws, hipStream_t s) {
  static const int same[DH_CF_NOPS] = {DH_F_NORM1, DH_F_QKV, -1, -1, -1, DH_F_PROJ, DH_F_AR1, DH_F_NORM2, DH_F_FC1,
                                       DH_F_ACT,   DH_F_FC2, DH_F_AR2, DH_F_BDA2};
  const dh_layer_config& c = L->c;
  char* sv = (char*)a.saved;
  const int r = c.cp_rank, S = L->q_off + c.seq, W = L->kv_w, blocks = c.cross_blocks > 0 ? c.cross_blocks : 8;
  switch (op) {
    case DH_CF_ROPE: {  // rotate q and k, then put the rank's own keys/values in their place of the attention buffer
      int rc = dh_rope_pairs(c.dtype, c.rope_pairing, L->T, c.seq, L->q_off, c.n_q_heads + c.n_kv_heads, c.head_dim, L->n_qkv, c.rope_base, 0, sv + L->s_qkv, s);
      if (rc) return rc;
      dh_cp_move m;
      m.src = sv + L->s_qkv + (size_t)c.n_q_heads * c.head_dim * L->es;
      m.src_ld = L->n_qkv; m.src_seq_rows = c.seq; m.src_row0 = 0;
      m.dst = sv + L->s_kv; m.dst_ld = W; m.dst_seq_rows = S; m.dst_row0 = r * c.seq;
      return dh_cp_exchange(c.dtype, 1, &m, c.batch, c.seq, W, 0, s);  // a local copy, not a transfer: at full speed
    }
    case DH_CF_CP_KV: {  // the exchange: the chunks of earlier ranks land in the attention buffer, later ranks' pass through
      dh_cp_move mv[16];
      int n = 0;
      for (int k = 0; k < c.cp_ranks; k++) {
        if (k == r) continue;
        dh_cp_move& m = mv[n++];
        m.src = (const char*)a.peers_kv + (size_t)(k < r ? k : k - 1) * L->T * W * L->es;
        m.src_ld = W; m.src_seq_rows = c.seq; m.src_row0 = 0;
        if (k < r) { m.dst = sv + L->s_kv; m.dst_ld = W; m.dst_seq_rows = S; m.dst_row0 = k * c.seq; }
        else { m.dst = ws + L->f_kvrecv + (size_t)(k - r - 1) * L->T * W * L->es; m.dst_ld = W; m.dst_seq_rows = c.seq; m.dst_row0 = 0; }
      }
      return dh_cp_exchange(c.dtype, n, mv, c.batch, c.seq, W, blocks, s);
    }
    case DH_CF_ATTN:
      return dh_attn_ctx_fwd(c.dtype, c.batch, c.seq, L->q_off, c.n_q_heads, c.n_kv_heads, c.head_dim, sv + L->s_qkv, sv + L->s_kv,
                             sv + L->s_o, (float*)(sv + L->s_lse), ws + L->f_attn, L->f_attn_bytes, s);
  }
  if (op < 0 || op >= DH_CF_NOPS) DH_FAIL(DH_ERR_INVALID_ARG, "unknown forward operator %d", op);
  return llama_fwd_op(L, same[op], a, ws, s);
}

static int cp_bwd_op(dh_layer* L, int op, const dh_bwd_args& b, char* ws, hipStream_t s, char* side_ws = nullptr) {
  static const int same[DH_CB_NOPS] = {DH_B_FC2_DGRAD, DH_B_FC2_WGRAD, DH_B_ACT, DH_B_FC1_DGRAD, DH_B_FC1_WGRAD, DH_B_AR3,
                                       DH_B_NORM2, DH_B_PROJ_DGRAD, DH_B_PROJ_WGRAD, -1, -1, -1, -1, DH_B_QKV_DGRAD,
                                       DH_B_QKV_WGRAD, DH_B_AR4, DH_B_NORM1};
  const dh_layer_config& c = L->c;
  const char* sv = (const char*)b.saved;
  const int r = c.cp_rank, S = L->q_off + c.seq, W = L->kv_w, blocks = c.cross_blocks > 0 ? c.cross_blocks : 8;
  switch (op) {
    case DH_CB_ATTN:
      return dh_attn_ctx_bwd(c.dtype, c.batch, c.seq, L->q_off, c.n_q_heads, c.n_kv_heads, c.head_dim, sv + L->s_qkv, sv + L->s_kv,
                             sv + L->s_o, ws + L->b_do, (const float*)(sv + L->s_lse), ws + L->b_dqkv, ws + L->b_dkv,
                             (float*)(ws + L->b_delta), ws + L->b_attn, L->b_attn_bytes, s);
    case DH_CB_CP_SEND: {  // the earlier chunks' key/value gradients go back to their owners: nothing here waits for it
      dh_cp_move mv[16];
      for (int k = 0; k < r; k++) {
        dh_cp_move& m = mv[k];
        m.src = ws + L->b_dkv; m.src_ld = W; m.src_seq_rows = S; m.src_row0 = k * c.seq;
        m.dst = (char*)b.dkv_peers + (size_t)k * L->T * W * L->es; m.dst_ld = W; m.dst_seq_rows = c.seq; m.dst_row0 = 0;
      }
      return dh_cp_exchange(c.dtype, r, mv, c.batch, c.seq, W, blocks, s);
    }
    case DH_CB_CP_DKV: {  // own chunk: own contribution + what the later ranks send for it
      dh_cp_move own;
      own.src = ws + L->b_dkv; own.src_ld = W; own.src_seq_rows = S; own.src_row0 = L->q_off;
      own.dst = ws + L->b_dqkv + (size_t)c.n_q_heads * c.head_dim * L->es; own.dst_ld = L->n_qkv; own.dst_seq_rows = c.seq; own.dst_row0 = 0;
      const void* later[16];
      const int n_later = c.cp_ranks - 1 - r;
      for (int k = 0; k < n_later; k++) later[k] = (const char*)b.peers_dkv + (size_t)(r + k) * L->T * W * L->es;
      return dh_cp_grad_reduce(c.dtype, &own, n_later, later, c.batch, c.seq, W, blocks, s);
    }
    case DH_CB_ROPE:
      return dh_rope_pairs(c.dtype, c.rope_pairing, L->T, c.seq, L->q_off, c.n_q_heads + c.n_kv_heads, c.head_dim, L->n_qkv, c.rope_base, 1, ws + L->b_dqkv, s);
  }
  if (op < 0 || op >= DH_CB_NOPS) DH_FAIL(DH_ERR_INVALID_ARG, "unknown backward operator %d", op);
  return llama_bwd_op(L, same[op], b, ws, s, side_ws);
}

// GPT-style layer under tensor + sequence parallelism (Sec. 2.1).  The norms, residuals and the
// layer's input/output live on this rank's Ts = T/R rows; GEMMs and attention see all T rows.
static int gpt_fwd_op(dh_layer* L, int op, const dh_fwd_args& a, char* ws, hipStream_t s) {
  const dh_layer_config& c = L->c;
  const int T = L->T, Ts = L->Ts, H = c.hidden, F = c.ffn, dt = c.dtype;
  char* sv = (char*)a.saved;
  void* gws = ws + L->f_gemm;
  const size_t ns = (size_t)Ts * H;
  switch (op) {
    case DH_GF_NORM1:
      return dh_layernorm_fwd(dt, Ts, H, a.x, nullptr, nullptr, L->w.g1, L->w.b1, c.eps, nullptr, ws + L->f_hs,
                              (float*)(sv + L->s_mu1), (float*)(sv + L->s_rstd1), s);
    case DH_GF_AG1:
      return collective(L, DH_COMM_ALLGATHER, ws + L->f_hs, a.peers_ag1, ns, sv + L->s_h1, s);
    case DH_GF_QKV:
      return gemm(L, false, false, T, L->n_qkv, H, sv + L->s_h1, L->w.Wqkv, sv + L->s_qkv, false, gws, L->f_gemm_bytes, s, L->w.bqkv);
    case DH_GF_ATTN:
      return op_attn_fwd(L, sv, ws, s);
    case DH_GF_PROJ:
      return gemm(L, false, false, T, H, L->n_o, sv + L->s_o, L->w.Wo, ws + L->f_part, false, gws, L->f_gemm_bytes, s);
    case DH_GF_RS1:
      return collective(L, DH_COMM_REDUCESCATTER, ws + L->f_part, a.peers_ar1, ns, ws + L->f_red, s);
    case DH_GF_NORM2:  // x2 = x + y + bo, h2 = norm(x2)
      return dh_layernorm_fwd(dt, Ts, H, a.x, ws + L->f_red, L->w.bo, L->w.g2, L->w.b2, c.eps, sv + L->s_x2, ws + L->f_hs,
                              (float*)(sv + L->s_mu2), (float*)(sv + L->s_rstd2), s);
    case DH_GF_AG2:
      return collective(L, DH_COMM_ALLGATHER, ws + L->f_hs, a.peers_ag2, ns, sv + L->s_h2, s);
    case DH_GF_FC1:
      return gemm(L, false, false, T, F, H, sv + L->s_h2, L->w.Wgu, sv + L->s_gu, false, gws, L->f_gemm_bytes, s, L->w.bfc1);
    case DH_GF_ACT:
      return dh_gelu_fwd_form(dt, c.gelu_form, (size_t)T * F, sv + L->s_gu, sv + L->s_a, s);
    case DH_GF_FC2:
      return gemm(L, false, false, T, H, F, sv + L->s_a, L->w.Wd, ws + L->f_part, false, gws, L->f_gemm_bytes, s);
    case DH_GF_RS2:
      return collective(L, DH_COMM_REDUCESCATTER, ws + L->f_part, a.peers_ar2, ns, ws + L->f_red, s);
    case DH_GF_BDA2:
      return dh_bias_residual_add(dt, Ts, H, sv + L->s_x2, ws + L->f_red, L->w.bfc2, a.out, s);
  }
  DH_FAIL(DH_ERR_INVALID_ARG, "unknown forward operator %d", op);
}

static int gpt_bwd_op(dh_layer* L, int op, const dh_bwd_args& b, char* ws, hipStream_t s) {
  const dh_layer_config& c = L->c;
  const int T = L->T, Ts = L->Ts, H = c.hidden, F = c.ffn, dt = c.dtype;
  const char* sv = (const char*)b.saved;
  void* gws = ws + L->b_gemm;
  const size_t gwb = L->b_gemm_bytes, ns = (size_t)Ts * H;
  int rc;
  switch (op) {
    case DH_GB_AG3:  // the backward of a reduce-scatter gathers the gradient shards
      return collective(L, DH_COMM_ALLGATHER, b.dout, b.peers_ag3, ns, ws + L->b_dz, s);
    case DH_GB_FC2_DGRAD:
      return gemm(L, false, true, T, F, H, ws + L->b_dz, L->w.Wd, ws + L->b_da, false, gws, gwb, s);
    case DH_GB_FC2_WGRAD:
      if ((rc = gemm(L, true, false, F, H, T, sv + L->s_a, ws + L->b_dz, L->g.dWd, true, gws, gwb, s))) return rc;
      return dh_colsum(dt, Ts, H, b.dout, L->g.dbfc2, ws + L->b_colsum, L->b_colsum_bytes, s);
    case DH_GB_ACT:
      return dh_gelu_bwd_form(dt, c.gelu_form, (size_t)T * F, sv + L->s_gu, ws + L->b_da, ws + L->b_dgu, s);
    case DH_GB_FC1_DGRAD:
      return gemm(L, false, true, T, H, F, ws + L->b_dgu, L->w.Wgu, ws + L->b_part, false, gws, gwb, s);
    case DH_GB_FC1_WGRAD:
      if ((rc = gemm(L, true, false, H, F, T, sv + L->s_h2, ws + L->b_dgu, L->g.dWgu, true, gws, gwb, s))) return rc;
      return dh_colsum(dt, T, F, ws + L->b_dgu, L->g.dbfc1, ws + L->b_colsum, L->b_colsum_bytes, s);
    case DH_GB_RS3:  // the backward of an all-gather reduce-scatters
      return collective(L, DH_COMM_REDUCESCATTER, ws + L->b_part, b.peers_ar3, ns, ws + L->b_red, s);
    case DH_GB_NORM2:  // dx2 = dout + norm2_bwd(dh2)
      return dh_layernorm_bwd(dt, Ts, H, ws + L->b_red, sv + L->s_x2, L->w.g2, (const float*)(sv + L->s_mu2),
                              (const float*)(sv + L->s_rstd2), b.dout, ws + L->b_dx2, L->g.dg2, L->g.db2, ws + L->b_norm,
                              L->b_norm_bytes, s);
    case DH_GB_AG4:
      return collective(L, DH_COMM_ALLGATHER, ws + L->b_dx2, b.peers_ag4, ns, ws + L->b_dy, s);
    case DH_GB_PROJ_DGRAD:
      return gemm(L, false, true, T, L->n_o, H, ws + L->b_dy, L->w.Wo, ws + L->b_do, false, gws, gwb, s);
    case DH_GB_PROJ_WGRAD:
      if ((rc = gemm(L, true, false, L->n_o, H, T, sv + L->s_o, ws + L->b_dy, L->g.dWo, true, gws, gwb, s))) return rc;
      return dh_colsum(dt, Ts, H, ws + L->b_dx2, L->g.dbo, ws + L->b_colsum, L->b_colsum_bytes, s);
    case DH_GB_ATTN:
      return op_attn_bwd(L, sv, ws, s);
    case DH_GB_QKV_DGRAD:
      return gemm(L, false, true, T, H, L->n_qkv, ws + L->b_dqkv, L->w.Wqkv, ws + L->b_part, false, gws, gwb, s);
    case DH_GB_QKV_WGRAD:
      if ((rc = gemm(L, true, false, H, L->n_qkv, T, sv + L->s_h1, ws + L->b_dqkv, L->g.dWqkv, true, gws, gwb, s))) return rc;
      return dh_colsum(dt, T, L->n_qkv, ws + L->b_dqkv, L->g.dbqkv, ws + L->b_colsum, L->b_colsum_bytes, s);
    case DH_GB_RS4:
      return collective(L, DH_COMM_REDUCESCATTER, ws + L->b_part, b.peers_ar4, ns, ws + L->b_red, s);
    case DH_GB_NORM1:  // dx = dx2 + norm1_bwd(dh1)
      return dh_layernorm_bwd(dt, Ts, H, ws + L->b_red, b.x, L->w.g1, (const float*)(sv + L->s_mu1),
                              (const float*)(sv + L->s_rstd1), ws + L->b_dx2, b.dx, L->g.dg1, L->g.db1, ws + L->b_norm,
                              L->b_norm_bytes, s);
  }
  DH_FAIL(DH_ERR_INVALID_ARG, "unknown backward operator %d", op);
}

// MoE layer: attention as in the Llama layer without collectives; the FFN is routed (top-2), its rows
// permuted by expert, exchanged by the all-to-all stand-in and run through grouped GEMMs.
static int moe_fwd_op(dh_layer* L, int op, const dh_fwd_args& a, char* ws, hipStream_t s) {
  const dh_layer_config& c = L->c;
  const int T = L->T, Tf = L->Tf, H = c.hidden, F = c.ffn, dt = c.dtype, E = c.n_experts, nl = c.n_local_experts;
  char* sv = (char*)a.saved;
  void* gws = ws + L->f_gemm;
  const dh_moe_tables tb = moe_tables_of(L, sv);
  int32_t* idx = (int32_t*)(sv + L->s_idx);
  float* prob = (float*)(sv + L->s_prob);
  int rc;
  switch (op) {
    case DH_MF_NORM1:
      return dh_rmsnorm_fwd(dt, T, H, a.x, nullptr, L->w.g1, c.eps, nullptr, sv + L->s_h1, (float*)(sv + L->s_rstd1), s);
    case DH_MF_QKV:
      return gemm(L, false, false, T, L->n_qkv, H, sv + L->s_h1, L->w.Wqkv, sv + L->s_qkv, false, gws, L->f_gemm_bytes, s);
    case DH_MF_ROPE:
      return op_rope(L, sv + L->s_qkv, 0, s);
    case DH_MF_ATTN:
      return op_attn_fwd(L, sv, ws, s);
    case DH_MF_PROJ:
      return gemm(L, false, false, T, H, L->n_o, sv + L->s_o, L->w.Wo, ws + L->f_part, false, gws, L->f_gemm_bytes, s);
    case DH_MF_NORM2:
      return dh_rmsnorm_fwd(dt, T, H, a.x, ws + L->f_part, L->w.g2, c.eps, sv + L->s_x2, sv + L->s_h2, (float*)(sv + L->s_rstd2), s);
    case DH_MF_ROUTE:
      if ((rc = dh_moe_route(T, E, a.logits, idx, prob, s))) return rc;
      return dh_moe_plan(T, E, nl, idx, &tb, s);
    case DH_MF_PERMUTE:
      return dh_moe_gather_rows(dt, Tf, H, sv + L->s_h2, tb.src_tok, ws + L->f_xp, 0, s);
    case DH_MF_A2A_DISPATCH:
      return dh_moe_gather_rows(dt, Tf, H, ws + L->f_xp, tb.send_of_recv, sv + L->s_xg, c.comm_blocks, s);
    case DH_MF_FC1:
      return dh_gemm_grouped(dt, 0, nl, tb.group_rows, Tf, H, 2 * F, sv + L->s_xg, L->w.Wgu, sv + L->s_gu, s);
    case DH_MF_ACT:
      return dh_swiglu_fwd(dt, Tf, F, sv + L->s_gu, sv + L->s_a, s);
    case DH_MF_FC2:
      return dh_gemm_grouped(dt, 0, nl, tb.group_rows, Tf, F, H, sv + L->s_a, L->w.Wd, ws + L->f_yg, s);
    case DH_MF_A2A_COMBINE:
      return dh_moe_gather_rows(dt, Tf, H, ws + L->f_yg, tb.recv_of_send, sv + L->s_yp, c.comm_blocks, s);
    case DH_MF_UNPERMUTE:  // out = x2 + sum_k p_k * (expert output of assignment k)
      return dh_moe_combine(dt, T, H, sv + L->s_yp, tb.dest, prob, sv + L->s_x2, a.out, s);
  }
  DH_FAIL(DH_ERR_INVALID_ARG, "unknown forward operator %d", op);
}

static int moe_bwd_op(dh_layer* L, int op, const dh_bwd_args& b, char* ws, hipStream_t s, char* side_ws = nullptr) {
  const dh_layer_config& c = L->c;
  const int T = L->T, Tf = L->Tf, H = c.hidden, F = c.ffn, dt = c.dtype, E = c.n_experts, nl = c.n_local_experts;
  const char* sv = (const char*)b.saved;
  void* gws = side_ws ? side_ws : ws + L->b_gemm;
  const size_t gwb = side_ws ? L->f_gemm_bytes : L->b_gemm_bytes;
  const dh_moe_tables tb = moe_tables_of(L, sv);
  const int32_t* idx = (const int32_t*)(sv + L->s_idx);
  const float* prob = (const float*)(sv + L->s_prob);
  switch (op) {
    case DH_MB_UNPERMUTE:
      return dh_moe_combine_bwd(dt, T, H, b.dout, sv + L->s_yp, tb.dest, prob, ws + L->b_dyp, (float*)(ws + L->b_dprob), s);
    case DH_MB_ROUTE:
      return dh_moe_route_bwd(T, E, (const float*)(ws + L->b_dprob), idx, prob, b.dlogits, s);
    case DH_MB_A2A_DISPATCH:
      return dh_moe_gather_rows(dt, Tf, H, ws + L->b_dyp, tb.send_of_recv, ws + L->b_dyg, c.comm_blocks, s);
    case DH_MB_FC2_DGRAD:
      return dh_gemm_grouped(dt, 1, nl, tb.group_rows, Tf, H, F, ws + L->b_dyg, L->w.Wd, ws + L->b_da, s);
    case DH_MB_FC2_WGRAD:
      return dh_gemm_grouped(dt, 2, nl, tb.group_rows, Tf, F, H, sv + L->s_a, ws + L->b_dyg, L->g.dWd, s);
    case DH_MB_ACT:
      return dh_swiglu_bwd(dt, Tf, F, sv + L->s_gu, ws + L->b_da, ws + L->b_dgu, s);
    case DH_MB_FC1_DGRAD:
      return dh_gemm_grouped(dt, 1, nl, tb.group_rows, Tf, 2 * F, H, ws + L->b_dgu, L->w.Wgu, ws + L->b_dxg, s);
    case DH_MB_FC1_WGRAD:
      return dh_gemm_grouped(dt, 2, nl, tb.group_rows, Tf, H, 2 * F, sv + L->s_xg, ws + L->b_dgu, L->g.dWgu, s);
    case DH_MB_A2A_COMBINE:  // the un-dispatched rows reuse the buffer of the dispatched upstream gradient
      return dh_moe_gather_rows(dt, Tf, H, ws + L->b_dxg, tb.recv_of_send, ws + L->b_dyp, c.comm_blocks, s);
    case DH_MB_PERMUTE:  // dh2[t] = sum of the gradients of token t's two permuted copies
      return dh_moe_combine(dt, T, H, ws + L->b_dyp, tb.dest, nullptr, nullptr, ws + L->b_red, s);
    case DH_MB_NORM2:
      return dh_rmsnorm_bwd(dt, T, H, ws + L->b_red, sv + L->s_x2, L->w.g2, (const float*)(sv + L->s_rstd2), b.dout,
                            ws + L->b_dx2, L->g.dg2, ws + L->b_norm, L->b_norm_bytes, s);
    case DH_MB_PROJ_DGRAD:
      return gemm(L, false, true, T, L->n_o, H, ws + L->b_dx2, L->w.Wo, ws + L->b_do, false, gws, gwb, s);
    case DH_MB_PROJ_WGRAD:
      return gemm(L, true, false, L->n_o, H, T, sv + L->s_o, ws + L->b_dx2, L->g.dWo, true, gws, gwb, s);
    case DH_MB_ATTN:
      return op_attn_bwd(L, sv, ws, s);
    case DH_MB_ROPE:
      return op_rope(L, ws + L->b_dqkv, 1, s);
    case DH_MB_QKV_DGRAD:
      return gemm(L, false, true, T, H, L->n_qkv, ws + L->b_dqkv, L->w.Wqkv, ws + L->b_part, false, gws, gwb, s);
    case DH_MB_QKV_WGRAD:
      return gemm(L, true, false, H, L->n_qkv, T, sv + L->s_h1, ws + L->b_dqkv, L->g.dWqkv, true, gws, gwb, s);
    case DH_MB_NORM1:
      return dh_rmsnorm_bwd(dt, T, H, ws + L->b_part, b.x, L->w.g1, (const float*)(sv + L->s_rstd1), ws + L->b_dx2, b.dx,
                            L->g.dg1, ws + L->b_norm, L->b_norm_bytes, s);
  }
  DH_FAIL(DH_ERR_INVALID_ARG, "unknown backward operator %d", op);
}

static int run_fwd_op(dh_layer* L, int op, const dh_fwd_args& a, char* ws, hipStream_t s) {
  if (L->c.comm_blocks < 0 && L->gf.is_comm[op] != 0) return DH_OK;  // timing without communication: the stand-in launches nothing
  switch (L->c.arch) {
    case DH_ARCH_GPT: return gpt_fwd_op(L, op, a, ws, s);
    case DH_ARCH_MOE: return moe_fwd_op(L, op, a, ws, s);
    case DH_ARCH_LLAMA_CP: return cp_fwd_op(L, op, a, ws, s);
    default: return llama_fwd_op(L, op, a, ws, s);
  }
}
static int run_bwd_op(dh_layer* L, int op, const dh_bwd_args& b, char* ws, hipStream_t s, char* side_ws = nullptr) {
  if (L->c.comm_blocks < 0 && L->gb.is_comm[op] != 0) return DH_OK;
  switch (L->c.arch) {
    case DH_ARCH_GPT: return gpt_bwd_op(L, op, b, ws, s);
    case DH_ARCH_MOE: return moe_bwd_op(L, op, b, ws, s, side_ws);
    case DH_ARCH_LLAMA_CP: return cp_bwd_op(L, op, b, ws, s, side_ws);
    default: return llama_bwd_op(L, op, b, ws, s, side_ws);
  }
}

static int check_fwd_args(const dh_layer* L, const dh_fwd_args* a) {
  if (!L || !a) DH_FAIL(DH_ERR_INVALID_ARG, "forward: null pointer");
  if (!L->have_w) DH_FAIL(DH_ERR_INVALID_ARG, "forward: weights not bound");
  if (L->T == 0) return DH_OK;
  if (!a->x || !a->out || !a->saved) DH_FAIL(DH_ERR_INVALID_ARG, "forward: x/out/saved is null");
  if (L->c.n_ranks > 1 && (!a->peers_ar1 || !a->peers_ar2)) DH_FAIL(DH_ERR_INVALID_ARG, "forward: peer partials are null but n_ranks > 1");
  if (L->c.arch == DH_ARCH_GPT && L->c.n_ranks > 1 && (!a->peers_ag1 || !a->peers_ag2))
    DH_FAIL(DH_ERR_INVALID_ARG, "forward: all-gather peer shards are null but n_ranks > 1");
  if (L->c.arch == DH_ARCH_MOE && !a->logits) DH_FAIL(DH_ERR_INVALID_ARG, "forward: router logits are null");
  if (L->c.arch == DH_ARCH_LLAMA_CP && L->c.cp_ranks > 1 && !a->peers_kv)
    DH_FAIL(DH_ERR_INVALID_ARG, "forward: the peers' key/value chunks are null but cp_ranks > 1");
  return DH_OK;
}
static int check_bwd_args(const dh_layer* L, const dh_bwd_args* b) {
  if (!L || !b) DH_FAIL(DH_ERR_INVALID_ARG, "backward: null pointer");
  if (!L->have_w || !L->have_g) DH_FAIL(DH_ERR_INVALID_ARG, "backward: weights or gradient buffers not bound");
  if (L->T == 0) return DH_OK;
  if (!b->dout || !b->dx || !b->x || !b->saved) DH_FAIL(DH_ERR_INVALID_ARG, "backward: dout/dx/x/saved is null");
  if (L->c.n_ranks > 1 && (!b->peers_ar3 || !b->peers_ar4)) DH_FAIL(DH_ERR_INVALID_ARG, "backward: peer partials are null but n_ranks > 1");
  if (L->c.arch == DH_ARCH_GPT && L->c.n_ranks > 1 && (!b->peers_ag3 || !b->peers_ag4))
    DH_FAIL(DH_ERR_INVALID_ARG, "backward: all-gather peer shards are null but n_ranks > 1");
  if (L->c.arch == DH_ARCH_MOE && !b->dlogits) DH_FAIL(DH_ERR_INVALID_ARG, "backward: dlogits is null");
  if (L->c.arch == DH_ARCH_LLAMA_CP && ((L->c.cp_rank + 1 < L->c.cp_ranks && !b->peers_dkv) || (L->c.cp_rank > 0 && !b->dkv_peers)))
    DH_FAIL(DH_ERR_INVALID_ARG, "backward: a key/value gradient exchange buffer is null");
  return DH_OK;
}
static int check_ws(const dh_layer* L, int kind, const void* ws, size_t ws_bytes) {
  size_t need = dh_layer_workspace_bytes(L, kind);
  if (need > 0 && (!ws || ws_bytes < need)) DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "workspace %zu bytes, need %zu", ws_bytes, need);
  if (((uintptr_t)ws & 255) != 0) DH_FAIL(DH_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  return DH_OK;
}

// Default operator order of a strand: a topological order taking the smallest ready operator id first
// (the ids are numbered so that this is simply 0, 1, 2, ... for every architecture).
static void default_order(const dh_op_graph& g, int* order) {
  int indeg[DH_MAX_OPS] = {0};
  bool done[DH_MAX_OPS] = {false};
  for (int e = 0; e < g.n_deps; e++) indeg[g.dep_dst[e]]++;
  for (int k = 0; k < g.n_ops; k++) {
    int pick = -1;
    for (int i = 0; i < g.n_ops && pick < 0; i++)
      if (!done[i] && indeg[i] == 0) pick = i;
    order[k] = pick;
    done[pick] = true;
    for (int e = 0; e < g.n_deps; e++)
      if (g.dep_src[e] == pick) indeg[g.dep_dst[e]]--;
  }
}

extern "C" int dh_layer_fwd(dh_layer* L, const dh_fwd_args* a, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_fwd_args(L, a);
  if (rc) return rc;
  if ((rc = check_ws(L, DH_WS_FWD, ws, ws_bytes))) return rc;
  if (L->T == 0) return DH_OK;
  int order[DH_MAX_OPS];
  default_order(L->gf, order);
  for (int k = 0; k < L->gf.n_ops; k++)
    if ((rc = run_fwd_op(L, order[k], *a, (char*)ws, (hipStream_t)stream))) return rc;
  return DH_OK;
}

extern "C" int dh_layer_bwd(dh_layer* L, const dh_bwd_args* b, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_bwd_args(L, b);
  if (rc) return rc;
  if ((rc = check_ws(L, DH_WS_BWD, ws, ws_bytes))) return rc;
  if (L->T == 0) return DH_OK;
  int order[DH_MAX_OPS];
  default_order(L->gb, order);
  for (int k = 0; k < L->gb.n_ops; k++)
    if ((rc = run_bwd_op(L, order[k], *b, (char*)ws, (hipStream_t)stream))) return rc;
  return DH_OK;
}

extern "C" int dh_plan_sequential(const dh_layer* L, dh_plan* out) {
  if (!L || !out) DH_FAIL(DH_ERR_INVALID_ARG, "plan_sequential: null pointer");
  memset(out, 0, sizeof(*out));
  const int nf = L->gf.n_ops, nb = L->gb.n_ops;
  out->n_fwd = nf;
  out->n_bwd = nb;
  default_order(L->gf, out->fwd_order);
  default_order(L->gb, out->bwd_order);
  out->n_pairs = 2;
  out->pairs[0] = {0, nf, 0, 0};
  out->pairs[1] = {nf, nf, 0, nb};
  return DH_OK;
}

// ------------------------------------------------------------------------------------ SI executor
static int ensure_events(dh_layer* L) {
  if (L->have_events) return DH_OK;
  for (int i = 0; i < DH_EVENT_POOL; i++)
    if (!L->ev[i]) DH_HIP(hipEventCreateWithFlags(&L->ev[i], hipEventDisableTiming));
  L->have_events = true;
  return DH_OK;
}

static hipEvent_t next_event(dh_layer* L) {
  hipEvent_t e = L->ev[L->ev_next];
  L->ev_next = (L->ev_next + 1) % DH_EVENT_POOL;
  return e;
}

// Runs `launch` on the communication stream after the work already queued on `strand`.  *done receives the event that
// marks its completion (nullptr if it ran in the strand's own stream): the strand does not wait for it here but when
// an operator that needs the result comes up, so that operators of the same strand that do not need it (weight
// gradients, mostly) overlap the transfer -- the "self-overlapping" operators of the paper's pairing figure.
template <typename Fn>
static int on_comm_stream(dh_layer* L, hipStream_t strand, hipStream_t comm, hipEvent_t* done, Fn launch) {
  *done = nullptr;
  if (comm == nullptr || comm == strand) return launch(strand);
  hipEvent_t before = next_event(L), after = next_event(L);
  DH_HIP(hipEventRecord(before, strand));
  DH_HIP(hipStreamWaitEvent(comm, before, 0));
  int rc = launch(comm);
  if (rc) return rc;
  DH_HIP(hipEventRecord(after, comm));
  *done = after;
  return DH_OK;
}

// Completion events of the communication operators a strand has issued on another stream and not waited for yet.
struct PendingComm {
  hipEvent_t ev[DH_MAX_OPS];
};
// Before operator `op` is issued: its strand waits for the pending transfers among op's direct predecessors (everything
// issued to the strand's stream afterwards is then ordered behind them too).
static int wait_for_inputs(const dh_op_graph& g, PendingComm& pd, int op, hipStream_t strand) {
  for (int e = 0; e < g.n_deps; e++) {
    const int src = g.dep_src[e];
    if (g.dep_dst[e] == op && pd.ev[src]) {
      DH_HIP(hipStreamWaitEvent(strand, pd.ev[src], 0));
      pd.ev[src] = nullptr;
    }
  }
  return DH_OK;
}
static int wait_for_all(const dh_op_graph& g, PendingComm& pd, hipStream_t strand) {
  for (int op = 0; op < g.n_ops; op++)
    if (pd.ev[op]) {
      DH_HIP(hipStreamWaitEvent(strand, pd.ev[op], 0));
      pd.ev[op] = nullptr;
    }
  return DH_OK;
}

// Stream of a communication operator: cross-node transfers (kind 2) use the layer's cross-node stream if one is set.
static hipStream_t comm_stream_of(const dh_layer* L, int kind, hipStream_t comm) {
  return kind == 2 && L->cross_stream ? L->cross_stream : comm;
}

static int check_si_args(dh_layer* L, const dh_fwd_args* alpha, const dh_bwd_args* beta, const dh_plan* plan, const void* ws,
                         size_t ws_bytes) {
  int rc = check_fwd_args(L, alpha);
  if (rc) return rc;
  if ((rc = check_bwd_args(L, beta))) return rc;
  if (!plan) DH_FAIL(DH_ERR_INVALID_ARG, "si_step: plan is null");
  if ((rc = dh_plan_validate(&L->gf, &L->gb, plan))) return rc;
  return check_ws(L, DH_WS_SI, ws, ws_bytes);
}

// Enqueues one SI step.  Stream beta (and the communication stream, through the events around each stand-in)
// forks from stream alpha at the start and is joined back into it at the end, so the whole step is one
// fork/join region of stream alpha -- which is also what stream capture requires.
static int enqueue_si(dh_layer* L, dh_layer* LB, const dh_fwd_args* alpha, const dh_bwd_args* beta, const dh_plan* plan, void* ws,
                      hipStream_t sa, hipStream_t sb, hipStream_t sc) {  // L: alpha's layer (also the event pool), LB: beta's
  int rc;
  char* ws_f = (char*)ws;
  char* ws_b = (char*)ws + L->fwd_bytes;
  const bool two = sb != sa;
  const hipStream_t scb = sc != nullptr && L->beta_comm_stream != nullptr ? L->beta_comm_stream : sc;  // beta's collectives
  PendingComm pf, pb;
  memset(&pf, 0, sizeof(pf));
  memset(&pb, 0, sizeof(pb));
  if (two) {  // beta starts after whatever alpha's stream already holds
    hipEvent_t e = next_event(L);
    DH_HIP(hipEventRecord(e, sa));
    DH_HIP(hipStreamWaitEvent(sb, e, 0));
  }
  for (int k = 0; k < plan->n_pairs; k++) {
    const dh_seg_pair& p = plan->pairs[k];
    int fi = p.f_begin, bj = p.b_begin;
    // alternate the two strands' launches so both streams receive work early
    while (fi < p.f_end || bj < p.b_end) {
      if (fi < p.f_end) {
        const int op = plan->fwd_order[fi++];
        if ((rc = wait_for_inputs(L->gf, pf, op, sa))) return rc;
        if (L->gf.is_comm[op]) rc = on_comm_stream(L, sa, comm_stream_of(L, L->gf.is_comm[op], sc), &pf.ev[op], [&](hipStream_t s) { return run_fwd_op(L, op, *alpha, ws_f, s); });
        else rc = run_fwd_op(L, op, *alpha, ws_f, sa);
        if (rc) return rc;
      }
      if (bj < p.b_end) {
        const int op = plan->bwd_order[bj++];
        if ((rc = wait_for_inputs(L->gb, pb, op, sb))) return rc;
        if (two && plan->bwd_side[op]) {  // beside the strand: after what the strand has issued so far, on the other stream
          hipEvent_t e = next_event(L);
          DH_HIP(hipEventRecord(e, sb));
          DH_HIP(hipStreamWaitEvent(sa, e, 0));
          if ((rc = run_bwd_op(LB, op, *beta, ws_b, sa, ws_f + L->f_gemm))) return rc;
          continue;
        }
        if (L->gb.is_comm[op]) rc = on_comm_stream(L, sb, comm_stream_of(L, L->gb.is_comm[op], scb), &pb.ev[op], [&](hipStream_t s) { return run_bwd_op(LB, op, *beta, ws_b, s); });
        else rc = run_bwd_op(LB, op, *beta, ws_b, sb);
        if (rc) return rc;
      }
    }
    // a segment pair ends with all of its transfers done
    if ((rc = wait_for_all(L->gf, pf, sa)) || (rc = wait_for_all(L->gb, pb, sb))) return rc;
    if (two) {  // cross-strand barrier on the device; after the last pair beta only joins alpha
      hipEvent_t ea = next_event(L), eb = next_event(L);
      const bool last = k + 1 == plan->n_pairs;
      if (!last) DH_HIP(hipEventRecord(ea, sa));
      DH_HIP(hipEventRecord(eb, sb));
      DH_HIP(hipStreamWaitEvent(sa, eb, 0));
      if (!last) DH_HIP(hipStreamWaitEvent(sb, ea, 0));
    }
  }
  return DH_OK;
}

extern "C" int dh_si_step(dh_layer* L, const dh_fwd_args* alpha, const dh_bwd_args* beta, const dh_plan* plan, void* ws,
                          size_t ws_bytes, void* stream_alpha, void* stream_beta, void* stream_comm) {
  int rc = check_si_args(L, alpha, beta, plan, ws, ws_bytes);
  if (rc) return rc;
  if (L->T == 0) return DH_OK;
  if ((rc = ensure_events(L))) return rc;
  return enqueue_si(L, L, alpha, beta, plan, ws, (hipStream_t)stream_alpha, (hipStream_t)stream_beta, (hipStream_t)stream_comm);
}

static bool same_shape(const dh_layer_config& a, const dh_layer_config& b) {
  return a.arch == b.arch && a.dtype == b.dtype && a.batch == b.batch && a.seq == b.seq && a.hidden == b.hidden &&
         a.n_q_heads == b.n_q_heads && a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim && a.ffn == b.ffn &&
         a.n_ranks == b.n_ranks && a.n_experts == b.n_experts && a.n_local_experts == b.n_local_experts &&
         a.cp_ranks == b.cp_ranks && a.cp_rank == b.cp_rank && a.rope_pairing == b.rope_pairing && a.gelu_form == b.gelu_form;
}

extern "C" int dh_si_step_layers(dh_layer* layer_alpha, dh_layer* layer_beta, const dh_fwd_args* alpha, const dh_bwd_args* beta,
                                 const dh_plan* plan, void* ws, size_t ws_bytes, void* stream_alpha, void* stream_beta,
                                 void* stream_comm) {
  if (!layer_alpha || !layer_beta) DH_FAIL(DH_ERR_INVALID_ARG, "si_step_layers: null layer");
  if (!same_shape(layer_alpha->c, layer_beta->c)) DH_FAIL(DH_ERR_SHAPE, "si_step_layers: the two layers differ in shape");
  int rc = check_fwd_args(layer_alpha, alpha);
  if (rc) return rc;
  if ((rc = check_bwd_args(layer_beta, beta))) return rc;
  if (!plan) DH_FAIL(DH_ERR_INVALID_ARG, "si_step_layers: plan is null");
  if ((rc = dh_plan_validate(&layer_alpha->gf, &layer_beta->gb, plan))) return rc;
  if ((rc = check_ws(layer_alpha, DH_WS_SI, ws, ws_bytes))) return rc;
  if (layer_alpha->T == 0) return DH_OK;
  if ((rc = ensure_events(layer_alpha))) return rc;
  return enqueue_si(layer_alpha, layer_beta, alpha, beta, plan, ws, (hipStream_t)stream_alpha, (hipStream_t)stream_beta,
                    (hipStream_t)stream_comm);
}

// ------------------------------------------------------------------------------------ captured SI step
struct dh_si_graph {
  hipGraph_t graph;
  hipGraphExec_t exec;
};

extern "C" int dh_si_graph_create(dh_layer* L, const dh_fwd_args* alpha, const dh_bwd_args* beta, const dh_plan* plan, void* ws,
                                  size_t ws_bytes, void* stream_alpha, void* stream_beta, dh_si_graph** out) {
  if (!out) DH_FAIL(DH_ERR_INVALID_ARG, "si_graph_create: null pointer");
  *out = nullptr;
  int rc = check_si_args(L, alpha, beta, plan, ws, ws_bytes);
  if (rc) return rc;
  if (L->T == 0) DH_FAIL(DH_ERR_INVALID_ARG, "si_graph_create: empty micro-batch");
  hipStream_t sa = (hipStream_t)stream_alpha, sb = (hipStream_t)stream_beta;
  if (sa == nullptr || sb == nullptr || sb == sa)
    DH_FAIL(DH_ERR_INVALID_ARG, "si_graph_create: needs two distinct, non-null strand streams");
  if ((rc = ensure_events(L))) return rc;
  // A graph holds dependencies, not streams.  A strand never runs past its own collective (its next operator
  // consumes the result), so a stand-in is recorded as a node of its strand's chain; a separate communication
  // stream would add nothing but an order among the two strands' collectives.
  hipStream_t cross = L->cross_stream;  // the same holds for cross-node transfers: recorded in their strand's chain
  L->cross_stream = nullptr;
  hipError_t e = hipStreamBeginCapture(sa, hipStreamCaptureModeThreadLocal);
  if (e != hipSuccess) {
    L->cross_stream = cross;
    (void)hipGetLastError();
    return dh_set_error(DH_ERR_HIP, "si_graph_create: hipStreamBeginCapture failed: %s", hipGetErrorString(e));
  }
  rc = enqueue_si(L, L, alpha, beta, plan, ws, sa, sb, nullptr);
  L->cross_stream = cross;
  hipGraph_t graph = nullptr;
  e = hipStreamEndCapture(sa, &graph);  // always end the capture, also after a failed enqueue
  if (rc != DH_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipGetLastError();
    return rc;
  }
  if (e != hipSuccess || graph == nullptr) {
    (void)hipGetLastError();
    return dh_set_error(DH_ERR_HIP, "si_graph_create: stream capture failed: %s", hipGetErrorString(e));
  }
  hipGraphExec_t exec = nullptr;
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    (void)hipGraphDestroy(graph);
    (void)hipGetLastError();
    return dh_set_error(DH_ERR_HIP, "si_graph_create: hipGraphInstantiate failed: %s", hipGetErrorString(e));
  }
  dh_si_graph* g = new dh_si_graph();
  g->graph = graph;
  g->exec = exec;
  *out = g;
  return DH_OK;
}

extern "C" int dh_si_graph_launch(dh_si_graph* g, void* stream) {
  if (!g) DH_FAIL(DH_ERR_INVALID_ARG, "si_graph_launch: null graph");
  DH_HIP(hipGraphLaunch(g->exec, (hipStream_t)stream));
  return DH_OK;
}

extern "C" void dh_si_graph_destroy(dh_si_graph* g) {
  if (!g) return;
  (void)hipGraphExecDestroy(g->exec);
  (void)hipGraphDestroy(g->graph);
  delete g;
}

// ------------------------------------------------------------------------------------ profiler
struct TimedOp {
  int dir, op;
};

static int launch_op(dh_layer* L, const TimedOp& o, const dh_fwd_args& a, const dh_bwd_args& b, char* ws_f, char* ws_b,
                     hipStream_t s) {
  return o.dir == 0 ? run_fwd_op(L, o.op, a, ws_f, s) : run_bwd_op(L, o.op, b, ws_b, s);
}

// Solo time of every operator (the first half of the pair profiler), each on the stream dh_si_step would issue it to.
extern "C" int dh_profile_solo(dh_layer* L, const dh_fwd_args* alpha, const dh_bwd_args* beta, void* ws, size_t ws_bytes,
                               void* stream_alpha, void* stream_beta, void* comm_stream, int reps, double* t_fwd, double* t_bwd) {
  int rc = check_fwd_args(L, alpha);
  if (rc) return rc;
  if ((rc = check_bwd_args(L, beta))) return rc;
  if (!t_fwd || !t_bwd || reps < 1) DH_FAIL(DH_ERR_INVALID_ARG, "profile_solo: bad arguments");
  if ((rc = check_ws(L, DH_WS_SI, ws, ws_bytes))) return rc;
  hipStream_t sa = (hipStream_t)stream_alpha, sb = (hipStream_t)stream_beta, sc = (hipStream_t)comm_stream;
  char* ws_f = (char*)ws;
  char* ws_b = (char*)ws + L->fwd_bytes;
  const int NF = L->gf.n_ops, NB = L->gb.n_ops;
  for (int i = 0; i < NF; i++) t_fwd[i] = 0.0;
  for (int j = 0; j < NB; j++) t_bwd[j] = 0.0;
  if (L->T == 0) return DH_OK;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  auto cleanup = [&]() { if (e0) (void)hipEventDestroy(e0); if (e1) (void)hipEventDestroy(e1); };
  hipError_t he = hipEventCreate(&e0);
  if (he == hipSuccess) he = hipEventCreate(&e1);
  if (he != hipSuccess) { cleanup(); return dh_set_error(DH_ERR_HIP, "profile_solo: event creation failed: %s", hipGetErrorString(he)); }
  for (int dir = 0; dir < 2; dir++)
    for (int op = 0; op < (dir == 0 ? NF : NB); op++) {
      const int comm = dir == 0 ? L->gf.is_comm[op] : L->gb.is_comm[op];
      const hipStream_t base = dir == 1 && sc != nullptr && L->beta_comm_stream != nullptr ? L->beta_comm_stream : sc;
      hipStream_t s = comm ? comm_stream_of(L, comm, base) : nullptr;
      if (!s) s = dir == 0 ? sa : sb;
      // one warm-up launch, then two timed groups of reps launches; the shorter group counts (a hiccup of the machine --
      // a clock ramp, a first touch -- lengthens one group, not both)
      double best = 1e30;
      for (int grp = 0; grp < 2; grp++) {
        for (int r = (grp == 0 ? 0 : 1); r < reps + 1; r++) {
          if (r == 1) (void)hipEventRecord(e0, s);
          rc = dir == 0 ? run_fwd_op(L, op, *alpha, ws_f, s) : run_bwd_op(L, op, *beta, ws_b, s);
          if (rc) { cleanup(); return rc; }
        }
        (void)hipEventRecord(e1, s);
        he = hipEventSynchronize(e1);
        if (he != hipSuccess) { cleanup(); return dh_set_error(DH_ERR_HIP, "profile_solo: %s", hipGetErrorString(he)); }
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        best = std::min(best, (double)ms * 1e-3 / reps);
      }
      (dir == 0 ? t_fwd : t_bwd)[op] = std::max(best, 1e-7);
    }
  cleanup();
  return DH_OK;
}

extern "C" int dh_profile_pairs(dh_layer* L, const dh_fwd_args* alpha, const dh_bwd_args* beta, void* ws, size_t ws_bytes,
                                void* stream_alpha, void* stream_beta, void* comm_stream, int reps, dh_overlap_table* out) {
  int rc = check_fwd_args(L, alpha);
  if (rc) return rc;
  if ((rc = check_bwd_args(L, beta))) return rc;
  if (!out || reps < 1) DH_FAIL(DH_ERR_INVALID_ARG, "profile_pairs: bad arguments");
  if ((rc = check_ws(L, DH_WS_SI, ws, ws_bytes))) return rc;
  if (stream_alpha == stream_beta) DH_FAIL(DH_ERR_INVALID_ARG, "profile_pairs: needs two distinct strand streams");
  hipStream_t sa = (hipStream_t)stream_alpha, sb = (hipStream_t)stream_beta, sc = (hipStream_t)comm_stream;
  char* ws_f = (char*)ws;
  char* ws_b = (char*)ws + L->fwd_bytes;
  memset(out, 0, sizeof(*out));
  const int NF = L->gf.n_ops, NB = L->gb.n_ops;
  out->n_fwd = NF;
  out->n_bwd = NB;
  if (L->T == 0) return DH_OK;
  hipEvent_t e0 = nullptr, e1 = nullptr, e3 = nullptr, gate = nullptr;
  auto cleanup = [&]() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e3) (void)hipEventDestroy(e3);
    if (gate) (void)hipEventDestroy(gate);
  };
  {
    hipError_t he = hipEventCreate(&e0);
    if (he == hipSuccess) he = hipEventCreate(&e1);
    if (he == hipSuccess) he = hipEventCreate(&e3);
    if (he == hipSuccess) he = hipEventCreateWithFlags(&gate, hipEventDisableTiming);
    if (he != hipSuccess) { cleanup(); return dh_set_error(DH_ERR_HIP, "profile: event creation failed: %s", hipGetErrorString(he)); }
  }
  auto stream_of = [&](int dir, int op) {
    const int comm = dir == 0 ? L->gf.is_comm[op] : L->gb.is_comm[op];
    const hipStream_t base = dir == 1 && sc != nullptr && L->beta_comm_stream != nullptr ? L->beta_comm_stream : sc;
    hipStream_t cs = comm ? comm_stream_of(L, comm, base) : nullptr;
    if (cs) return cs;
    return dir == 0 ? sa : sb;
  };
  // solo times
  for (int dir = 0; dir < 2; dir++) {
    const int n = dir == 0 ? NF : NB;
    for (int op = 0; op < n; op++) {
      hipStream_t s = stream_of(dir, op);
      TimedOp t{dir, op};
      if ((rc = launch_op(L, t, *alpha, *beta, ws_f, ws_b, s))) { cleanup(); return rc; }  // warm-up
      // two timed groups of reps launches, the shorter one counts: a hiccup of the machine (a clock ramp, a first touch)
      // lengthens one group, not both, and every pair measurement below is sized from these times
      double best = 1e30;
      for (int grp = 0; grp < 2; grp++) {
        (void)hipEventRecord(e0, s);
        for (int r = 0; r < reps; r++)
          if ((rc = launch_op(L, t, *alpha, *beta, ws_f, ws_b, s))) { cleanup(); return rc; }
        (void)hipEventRecord(e1, s);
        hipError_t he = hipEventSynchronize(e1);
        if (he != hipSuccess) { cleanup(); return dh_set_error(DH_ERR_HIP, "profile: %s", hipGetErrorString(he)); }
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        best = std::min(best, (double)ms * 1e-3 / reps);
      }
      // an operator that launches nothing (a Send/Recv stand-in with no peer, an activation that runs in its
      // neighbour's epilogue) measures ~0: floor it, so that the repeat counts, rates and Eq. 1 below stay finite
      (dir == 0 ? out->t_fwd : out->t_bwd)[op] = std::max(best, 1e-7);
    }
  }
  // pairs: both operators repeated so that the two streams stay busy for about the same window
  for (int i = 0; i < NF; i++)
    for (int j = 0; j < NB; j++) {
      const double ta = out->t_fwd[i], tb = out->t_bwd[j];
      const double window = std::max(ta, tb) * reps;
      const int ra = (int)std::min(64.0 * reps, std::max(1.0, std::round(window / ta)));
      const int rb = (int)std::min(64.0 * reps, std::max(1.0, std::round(window / tb)));
      hipStream_t s1 = stream_of(0, i), s2 = stream_of(1, j);
      TimedOp A{0, i}, B{1, j};
      double end_a, end_b;
      if (s1 == s2) {  // both on the one communication stream: they serialise
        end_a = ta * ra;
        end_b = ta * ra + tb * rb;
      } else {
        (void)hipEventRecord(gate, s1);
        (void)hipStreamWaitEvent(s2, gate, 0);
        (void)hipEventRecord(e0, s1);
        for (int r = 0; r < std::max(ra, rb); r++) {
          if (r < ra && (rc = launch_op(L, A, *alpha, *beta, ws_f, ws_b, s1))) { cleanup(); return rc; }
          if (r < rb && (rc = launch_op(L, B, *alpha, *beta, ws_f, ws_b, s2))) { cleanup(); return rc; }
        }
        (void)hipEventRecord(e1, s1);
        (void)hipEventRecord(e3, s2);
        hipError_t he = hipEventSynchronize(e1);
        if (he == hipSuccess) he = hipEventSynchronize(e3);
        if (he != hipSuccess) { cleanup(); return dh_set_error(DH_ERR_HIP, "profile: %s", hipGetErrorString(he)); }
        float ma = 0.f, mb = 0.f;
        (void)hipEventElapsedTime(&ma, e0, e1);
        (void)hipEventElapsedTime(&mb, e0, e3);
        end_a = (double)ma * 1e-3;
        end_b = (double)mb * 1e-3;
      }
      // invert the fluid model on the aggregated operators (ra*ta, rb*tb)
      const double wa = ta * ra, wb = tb * rb, t1 = std::min(end_a, end_b);
      double qa, qb;
      if (end_a <= end_b) { qa = wa / t1; qb = (wb - (end_b - t1)) / t1; }
      else { qa = (wa - (end_a - t1)) / t1; qb = wb / t1; }
      qa = std::min(1.0, std::max(0.02, qa));
      qb = std::min(1.0, std::max(0.02, qb));
      out->rate_fwd[i][j] = qa;
      out->rate_bwd[i][j] = qb;
      const int sf[1] = {i}, sbk[1] = {j};
      out->p_pair[i][j] = dh_segment_cost(out, sf, 1, sbk, 1);
      out->oef[i][j] = dh_oef(ta, tb, out->p_pair[i][j]);
    }
  cleanup();
  return DH_OK;
}
