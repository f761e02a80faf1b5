// Several layers under Strand Interleaving on one GPU (the single-stage case of the paper's folded pipeline,
// Sec. 4.1): while micro-batch strand alpha sweeps forward through layers 0..L-1, strand beta -- the micro-batch of
// the previous phase -- sweeps backward through layers L-1..0; step k co-executes alpha's layer k with beta's layer
// L-1-k as one SI step.  Activation memory is shared in the two-triangle arrangement of Sec. 3.3: beta's backward
// frees slots from the top layer down while alpha's forward needs them from the bottom layer up, so L+1 saved-activation
// slots and L layer-input buffers serve both strands (against 2L and 2(L-1) without sharing).  Host-side orchestration
// only: every operator runs in the layer library's kernels, and all buffers belong to the caller.
#include <cstring>
#include <vector>
#include "common.h"

struct dh_stack {
  dh_layer_config c;
  int L;
  std::vector<dh_layer*> layers;
  size_t x_bytes, saved_bytes, ws_layer_bytes;
  // slots of the strand that runs backward in the next phase: saved_of[l], x_of[l] (x_of[0] unused: the caller's buffer)
  std::vector<int> saved_of, x_of;
  std::vector<int> free_saved, free_x;
  const void* x0;
  bool have_beta;
};

extern "C" int dh_stack_create(const dh_layer_config* cfg, int n_layers, dh_stack** out) {
  if (!cfg || !out) DH_FAIL(DH_ERR_INVALID_ARG, "stack_create: null pointer");
  if (n_layers < 1 || n_layers > 1024) DH_FAIL(DH_ERR_INVALID_ARG, "stack_create: n_layers %d outside 1..1024", n_layers);
  if (cfg->arch != DH_ARCH_LLAMA) DH_FAIL(DH_ERR_UNSUPPORTED, "stack_create: only DH_ARCH_LLAMA layers can be stacked");
  dh_stack* S = new dh_stack();
  S->c = *cfg;
  S->L = n_layers;
  for (int l = 0; l < n_layers; l++) {
    dh_layer* layer = nullptr;
    int rc = dh_layer_create(cfg, &layer);
    if (rc != DH_OK) {
      for (dh_layer* p : S->layers) dh_layer_destroy(p);
      delete S;
      return rc;
    }
    S->layers.push_back(layer);
  }
  const size_t T = (size_t)cfg->batch * cfg->seq;
  S->x_bytes = dh_align_up(T * cfg->hidden * dh_elem_size(cfg->dtype), 256);
  S->saved_bytes = dh_align_up(dh_layer_saved_bytes(S->layers[0]), 256);
  S->ws_layer_bytes = dh_align_up(dh_layer_workspace_bytes(S->layers[0], DH_WS_SI), 256);
  S->saved_of.assign(n_layers, -1);
  S->x_of.assign(n_layers, -1);
  for (int s = n_layers; s >= 0; s--) S->free_saved.push_back(s);   // L+1 saved slots
  for (int s = n_layers - 1; s >= 0; s--) S->free_x.push_back(s);   // L layer-input buffers
  S->x0 = nullptr;
  S->have_beta = false;
  *out = S;
  return DH_OK;
}

extern "C" void dh_stack_destroy(dh_stack* S) {
  if (!S) return;
  for (dh_layer* p : S->layers) dh_layer_destroy(p);
  delete S;
}

extern "C" dh_layer* dh_stack_layer(dh_stack* S, int i) { return S && i >= 0 && i < S->L ? S->layers[i] : nullptr; }
extern "C" size_t dh_stack_arena_bytes(const dh_stack* S) {
  return S ? (size_t)(S->L + 1) * S->saved_bytes + (size_t)S->L * S->x_bytes : 0;
}
extern "C" size_t dh_stack_unshared_bytes(const dh_stack* S) {  // two strands, each with its own full set
  return S ? 2 * ((size_t)S->L * S->saved_bytes + (size_t)(S->L - 1) * S->x_bytes) : 0;
}
extern "C" size_t dh_stack_workspace_bytes(const dh_stack* S) { return S ? S->ws_layer_bytes + 2 * S->x_bytes : 0; }

extern "C" int dh_stack_phase(dh_stack* S, const dh_stack_fwd* alpha, const dh_stack_bwd* beta, const dh_plan* plan, void* arena,
                              size_t arena_bytes, void* ws, size_t ws_bytes, void* stream_alpha, void* stream_beta,
                              void* stream_comm) {
  if (!S) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: null stack");
  if (!alpha && !beta) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: neither a forward nor a backward strand");
  if (beta && !S->have_beta) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: no micro-batch has run forward yet, nothing to run backward");
  if (!beta && S->have_beta) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: the previous micro-batch still waits for its backward pass");
  if (alpha && (!alpha->x || !alpha->out)) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: alpha x/out is null");
  if (beta && (!beta->dout || !beta->dx)) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: beta dout/dx is null");
  if (alpha && beta && !plan) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: a co-run phase needs a plan");
  if (!arena || arena_bytes < dh_stack_arena_bytes(S)) DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "stack_phase: arena %zu bytes, need %zu", arena_bytes, dh_stack_arena_bytes(S));
  if (!ws || ws_bytes < dh_stack_workspace_bytes(S)) DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "stack_phase: workspace %zu bytes, need %zu", ws_bytes, dh_stack_workspace_bytes(S));
  if (((uintptr_t)arena & 255) || ((uintptr_t)ws & 255)) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: arena and workspace must be 256-byte aligned");
  const int L = S->L;
  char* saved_pool = (char*)arena;
  char* x_pool = saved_pool + (size_t)(L + 1) * S->saved_bytes;
  char* grad[2] = {(char*)ws + S->ws_layer_bytes, (char*)ws + S->ws_layer_bytes + S->x_bytes};
  std::vector<int> new_saved(L, -1), new_x(L, -1);
  const void* layer_in = alpha ? alpha->x : nullptr;
  for (int k = 0; k < L; k++) {
    const int lb = L - 1 - k;  // beta's layer in this step
    dh_fwd_args fa;
    dh_bwd_args ba;
    memset(&fa, 0, sizeof(fa));
    memset(&ba, 0, sizeof(ba));
    if (alpha) {
      // a saved slot for layer k and, unless it is the last layer, a buffer for its output = layer k+1's input; both
      // come from what beta released in earlier steps (or the spares), never from what beta reads in this step
      if (S->free_saved.empty() || (k + 1 < L && S->free_x.empty())) DH_FAIL(DH_ERR_INVALID_ARG, "stack_phase: internal error, activation arena exhausted");
      new_saved[k] = S->free_saved.back();
      S->free_saved.pop_back();
      fa.x = layer_in;
      fa.saved = saved_pool + (size_t)new_saved[k] * S->saved_bytes;
      if (k + 1 < L) {
        new_x[k + 1] = S->free_x.back();
        S->free_x.pop_back();
        fa.out = x_pool + (size_t)new_x[k + 1] * S->x_bytes;
      } else {
        fa.out = alpha->out;
      }
      fa.peers_ar1 = alpha->peers_ar1;
      fa.peers_ar2 = alpha->peers_ar2;
    }
    if (beta) {
      ba.dout = k == 0 ? beta->dout : grad[(k - 1) & 1];
      ba.dx = lb == 0 ? beta->dx : grad[k & 1];
      ba.x = lb == 0 ? S->x0 : x_pool + (size_t)S->x_of[lb] * S->x_bytes;
      ba.saved = saved_pool + (size_t)S->saved_of[lb] * S->saved_bytes;
      ba.peers_ar3 = beta->peers_ar3;
      ba.peers_ar4 = beta->peers_ar4;
    }
    int rc;
    if (alpha && beta)
      rc = dh_si_step_layers(S->layers[k], S->layers[lb], &fa, &ba, plan, ws, S->ws_layer_bytes, stream_alpha, stream_beta, stream_comm);
    else if (alpha)
      rc = dh_layer_fwd(S->layers[k], &fa, ws, S->ws_layer_bytes, stream_alpha);
    else
      rc = dh_layer_bwd(S->layers[lb], &ba, ws, S->ws_layer_bytes, stream_alpha);
    if (rc != DH_OK) return rc;
    if (beta) {  // released for alpha's later steps: the step's end joins beta's stream into alpha's
      S->free_saved.push_back(S->saved_of[lb]);
      S->saved_of[lb] = -1;
      if (lb > 0) { S->free_x.push_back(S->x_of[lb]); S->x_of[lb] = -1; }
    }
    if (alpha) layer_in = fa.out;
  }
  if (alpha) {
    S->saved_of = new_saved;
    S->x_of = new_x;
    S->x0 = alpha->x;
    S->have_beta = true;
  } else {
    S->have_beta = false;
    S->x0 = nullptr;
  }
  return DH_OK;
}
