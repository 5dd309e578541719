// C-ABI entry points (declared in include/mlip.h): argument checks, context life cycle,
// the whole-step driver with per-phase HIP-event timing.
#include <cstring>
#include <new>

#include "common.h"

void* ctx_alloc(mlip_ctx* ctx, size_t bytes) {
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    ctx->err = std::string("hipMalloc failed: ") + hipGetErrorString(e);
    return nullptr;
  }
  ctx->allocs.push_back(p);
  ctx->bytes += (int64_t)bytes;
  return p;
}

// ---- dispatch on the model kind
#define IS_EQV(ctx) ((ctx)->cfg.model_kind == MLIP_MODEL_EQUIVARIANT)
static int model_alloc(mlip_ctx* c) { return IS_EQV(c) ? eqv_alloc(c) : inv_alloc(c); }
static void model_free(mlip_ctx* c) { if (IS_EQV(c)) eqv_free(c); else inv_free(c); }
static int model_forward_energy(mlip_ctx* c, const float* pos, const int32_t* sp, const float* th, const float* h_in, float* E, float* h_out) {
  return IS_EQV(c) ? eqv_forward_energy(c, pos, sp, th, h_in, E, h_out) : inv_forward_energy(c, pos, sp, th, h_in, E, h_out);
}
static int model_forward_force(mlip_ctx* c, const float* g_out, float* F, float* g_in) {
  return IS_EQV(c) ? eqv_forward_force(c, g_out, F, g_in) : inv_forward_force(c, g_out, F, g_in);
}
static int model_loss(mlip_ctx* c, const float* E, const float* F, const float* Er, const float* Fr, float* loss, float* Ebar, float* v) {
  return inv_loss(c, E, F, Er, Fr, loss, Ebar, v);
}
static int model_backward_force(mlip_ctx* c, const float* v, const float* hd, float* g, float* hdo) {
  return IS_EQV(c) ? eqv_backward_force(c, v, hd, g, hdo) : inv_backward_force(c, v, hd, g, hdo);
}
static int model_backward_energy(mlip_ctx* c, const float* Ebar, const float* lo, float* g, float* li) {
  return IS_EQV(c) ? eqv_backward_energy(c, Ebar, lo, g, li) : inv_backward_energy(c, Ebar, lo, g, li);
}

namespace {

struct StepBufs {
  float* Ebar = nullptr;
  float* v = nullptr;
};

int layout_params(mlip_ctx* ctx) {
  const mlip_config& c = ctx->cfg;
  const int64_t C = c.channels, H = c.edge_hidden, K = c.n_rbf;
  int64_t off = 0;
  ctx->lay.assign(c.n_layers, LayerOffsets{});
  if (c.model_kind != MLIP_MODEL_STAGE) { ctx->off_emb = off; off += (int64_t)c.n_species * C; }
  for (int l = 0; l < c.n_layers; ++l) {
    LayerOffsets& lo = ctx->lay[l];
    lo.W[0] = off; off += H * K;
    if (c.model_kind == MLIP_MODEL_EQUIVARIANT) {
      lo.W[1] = off; off += (int64_t)mlip_npath(c.l_max) * C * H;
      lo.W[2] = -1;
      const int64_t banks = c.n_experts > 0 ? c.n_experts : 1;  // expert banks [n_experts][C][C]
      for (int k = 0; k <= c.l_max; ++k) { lo.Wl[k] = off; off += banks * C * C; }
    } else {
      if (c.edge_mlp_depth == 3) { lo.W[1] = off; off += H * H; lo.W[2] = off; off += C * H; }
      else { lo.W[1] = off; off += C * H; lo.W[2] = -1; }
      const int64_t banks = c.n_experts > 0 ? c.n_experts : 1;  // expert banks [n_experts][C][C]
      lo.V1 = off; off += banks * C * C;
      lo.V2 = off; off += banks * C * C;
    }
  }
  if (c.model_kind != MLIP_MODEL_STAGE) { ctx->off_U = off; off += C * C; ctx->off_wo = off; off += C; }
  ctx->n_params = off;
  return MLIP_OK;
}

__global__ void k_copy_probe(float4* __restrict__ dst, const float4* __restrict__ src, int64_t n4) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) dst[i] = src[i];
}

const char* check_config(const mlip_config& c) {
  if (c.model_kind < 0 || c.model_kind > 2) return "model_kind must be 0, 1 or 2";
  if (c.channels < 4 || c.channels % 4 || c.channels > 1024) return "channels must be a multiple of 4 in [4, 1024]";
  if (c.edge_hidden < 4 || c.edge_hidden % 4) return "edge_hidden must be a positive multiple of 4";
  if (c.n_rbf < 4 || c.n_rbf % 4 || c.n_rbf > 1024) return "n_rbf must be a multiple of 4 in [4, 1024]";
  if (c.n_layers < 1 || c.n_layers > 64) return "n_layers must be in [1, 64]";
  if (c.edge_mlp_depth != 2 && c.edge_mlp_depth != 3) return "edge_mlp_depth must be 2 or 3";
  if (c.model_kind == MLIP_MODEL_EQUIVARIANT ? ((c.l_max != 2 && c.l_max != 3) || c.edge_mlp_depth != 2) : (c.l_max != 0))
    return "l_max must be 2 or 3 (edge_mlp_depth 2) for the equivariant model and 0 otherwise";
  if (c.model_kind != MLIP_MODEL_STAGE && c.n_species < 1) return "n_species must be positive";
  if (c.gemm_dtype != MLIP_GEMM_FP32 && c.gemm_dtype != MLIP_GEMM_BF16) return "gemm_dtype must be 0 or 1";
  if (c.n_experts < 0 || c.n_experts > 1024) return "n_experts must be in [0, 1024]";
  if (c.n_experts > 0 && c.model_kind == MLIP_MODEL_STAGE) return "expert banks are built for the whole models only";
  if (c.gate != 0 && c.gate != 1) return "gate must be 0 or 1";
  if (c.filter_fp32 != 0 && c.filter_fp32 != 1) return "filter_fp32 must be 0 or 1";
  if (c.position_grad != 0 && c.position_grad != 1) return "position_grad must be 0 or 1";
  if (c.gate == 1 && c.model_kind != MLIP_MODEL_EQUIVARIANT) return "the gated update belongs to the equivariant model";
  if (!(c.cutoff > 0.f)) return "cutoff must be positive";
  if (c.max_atoms < 1 || c.max_structs < 1 || c.max_edges < 1) return "capacities must be positive";
  if (c.max_atoms > 50000000 || c.max_edges > 2000000000LL) return "capacity too large for 32-bit indices";
  return nullptr;
}

}  // namespace

extern "C" {

int mlip_create(const mlip_config* cfg, void* hip_stream, mlip_ctx** out) {
  if (!cfg || !out) return MLIP_E_INVALID;
  *out = nullptr;
  if (check_config(*cfg)) return MLIP_E_INVALID;
  mlip_ctx* ctx = new (std::nothrow) mlip_ctx();
  if (!ctx) return MLIP_E_HIP;
  ctx->cfg = *cfg;
  ctx->stream = (hipStream_t)hip_stream;
  layout_params(ctx);
  int s = graph_alloc(ctx);
  if (s == MLIP_OK) s = model_alloc(ctx);
  if (s == MLIP_OK) {
    StepBufs* sb = new StepBufs();
    sb->Ebar = (float*)ctx_alloc(ctx, sizeof(float) * cfg->max_structs);
    sb->v = (float*)ctx_alloc(ctx, sizeof(float) * 3 * cfg->max_atoms);
    ctx->step_bufs = sb;
    if (!sb->Ebar || !sb->v) s = MLIP_E_HIP;
  }
  if (s != MLIP_OK) {
    mlip_destroy(ctx);
    return s;
  }
  *out = ctx;
  return MLIP_OK;
}

int mlip_destroy(mlip_ctx* ctx) {
  if (!ctx) return MLIP_OK;
  hipStreamSynchronize(ctx->stream);
  for (void* p : ctx->allocs) hipFree(p);
  for (hipEvent_t e : ctx->tev) hipEventDestroy(e);
  model_free(ctx);
  delete (StepBufs*)ctx->step_bufs;
  delete ctx;
  return MLIP_OK;
}

int64_t mlip_param_count(const mlip_ctx* ctx) { return ctx ? ctx->n_params : -1; }
const char* mlip_last_error(const mlip_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }
int64_t mlip_workspace_bytes(const mlip_ctx* ctx) { return ctx ? ctx->bytes : -1; }

int mlip_graph_build(mlip_ctx* ctx, int64_t n_atoms, int32_t n_structs, const float* pos, const int32_t* struct_ptr,
                     const float* cell, float cutoff, int64_t* n_edges_host) {
  if (!ctx) return MLIP_E_INVALID;
  return graph_build(ctx, n_atoms, n_structs, pos, struct_ptr, cell, cutoff, n_edges_host);
}

int mlip_set_expert_weights(mlip_ctx* ctx, const float* alpha, int32_t n_structs) {
  if (!ctx) return MLIP_E_INVALID;
  if (ctx->cfg.n_experts <= 0) MLIP_FAIL(ctx, MLIP_E_INVALID, "set_expert_weights: the context has no expert banks");
  if (!alpha || n_structs < 1 || n_structs > ctx->cfg.max_structs) MLIP_FAIL(ctx, MLIP_E_INVALID, "set_expert_weights: bad arguments");
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_alpha, alpha, sizeof(float) * (size_t)n_structs * ctx->cfg.n_experts,
                                     hipMemcpyDeviceToDevice, ctx->stream));
  ctx->alpha_structs = n_structs;
  return MLIP_OK;
}

int mlip_set_expert_weight_grad(mlip_ctx* ctx, float* grad_alpha, int32_t n_structs) {
  if (!ctx) return MLIP_E_INVALID;
  if (ctx->cfg.n_experts <= 0) MLIP_FAIL(ctx, MLIP_E_INVALID, "set_expert_weight_grad: the context has no expert banks");
  if (grad_alpha && (n_structs < 1 || n_structs > ctx->cfg.max_structs))
    MLIP_FAIL(ctx, MLIP_E_INVALID, "set_expert_weight_grad: n_structs must be in [1, max_structs]");
  ctx->d_grad_alpha = grad_alpha;
  ctx->grad_alpha_structs = grad_alpha ? n_structs : 0;
  return MLIP_OK;
}

int mlip_set_position_grad(mlip_ctx* ctx, float* grad_pos) {
  if (!ctx) return MLIP_E_INVALID;
  if (grad_pos && !ctx->cfg.position_grad)
    MLIP_FAIL(ctx, MLIP_E_INVALID, "set_position_grad: create the context with position_grad = 1 (its workspace is allocated at creation)");
  ctx->d_grad_pos = grad_pos;
  return MLIP_OK;
}

int mlip_input_status(mlip_ctx* ctx) {
  if (!ctx) return MLIP_E_INVALID;
  return input_status(ctx);
}

int mlip_graph_sizes(const mlip_ctx* ctx, int64_t* n_atoms_host, int64_t* n_structs_host, int64_t* n_edges_host) {
  if (!ctx) return MLIP_E_INVALID;
  if (ctx->phase < PH_GRAPH) return MLIP_E_STATE;
  if (n_atoms_host) *n_atoms_host = ctx->N;
  if (n_structs_host) *n_structs_host = ctx->B;
  if (n_edges_host) *n_edges_host = ctx->E;
  return MLIP_OK;
}

int mlip_copy_probe(mlip_ctx* ctx, float* dst, const float* src, int64_t n_floats) {
  if (!ctx || !dst || !src || n_floats <= 0 || (n_floats & 3)) return MLIP_E_INVALID;
  const int64_t n4 = n_floats / 4;
  hipLaunchKernelGGL(k_copy_probe, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, ctx->stream,
                     reinterpret_cast<float4*>(dst), reinterpret_cast<const float4*>(src), n4);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

int mlip_kernel_timer_select(mlip_ctx* ctx, int kernel_id) {
  if (!ctx) return MLIP_E_INVALID;
  if (kernel_id < 0 || kernel_id > MLIP_K_EDGE_FEATURES) MLIP_FAIL(ctx, MLIP_E_INVALID, "kernel_timer_select: unknown kernel id");
  MLIP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
  ctx->timed_kernel = kernel_id;
  ctx->tev_used = 0;
  return MLIP_OK;
}

int mlip_kernel_timer_read(mlip_ctx* ctx, int64_t* launches_host, float* total_ms_host) {
  if (!ctx || !launches_host || !total_ms_host) return MLIP_E_INVALID;
  MLIP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
  double total = 0.0;
  for (size_t k = 0; k + 1 < ctx->tev_used; k += 2) {
    float ms = 0.f;
    MLIP_HIP_CHECK(ctx, hipEventElapsedTime(&ms, ctx->tev[k], ctx->tev[k + 1]));
    total += ms;
  }
  *launches_host = (int64_t)(ctx->tev_used / 2);
  *total_ms_host = (float)total;
  return MLIP_OK;
}

int mlip_graph_export(mlip_ctx* ctx, int32_t* row_ptr, int32_t* sender, int32_t* shift, int32_t* rev) {
  if (!ctx) return MLIP_E_INVALID;
  return graph_export(ctx, row_ptr, sender, shift, rev);
}

int mlip_graph_export_pairs(mlip_ctx* ctx, int32_t* slot, int32_t* pair_edge) {
  if (!ctx) return MLIP_E_INVALID;
  return graph_export_pairs(ctx, slot, pair_edge);
}

int mlip_forward_energy(mlip_ctx* ctx, const float* pos, const int32_t* species, const float* params, const float* h_in,
                        float* E, float* h_out) {
  if (!ctx) return MLIP_E_INVALID;
  return model_forward_energy(ctx, pos, species, params, h_in, E, h_out);
}

int mlip_forward_force(mlip_ctx* ctx, const float* g_out, float* F, float* g_in) {
  if (!ctx) return MLIP_E_INVALID;
  return model_forward_force(ctx, g_out, F, g_in);
}

int mlip_loss(mlip_ctx* ctx, const float* E, const float* F, const float* E_ref, const float* F_ref, float* loss,
              float* Ebar, float* v) {
  if (!ctx) return MLIP_E_INVALID;
  if (ctx->cfg.model_kind == MLIP_MODEL_STAGE) MLIP_FAIL(ctx, MLIP_E_UNSUPPORTED, "loss: a stage has no loss");
  return model_loss(ctx, E, F, E_ref, F_ref, loss, Ebar, v);
}

int mlip_backward_force(mlip_ctx* ctx, const float* v, const float* hdot_in, float* grad_params, float* hdot_out) {
  if (!ctx) return MLIP_E_INVALID;
  return model_backward_force(ctx, v, hdot_in, grad_params, hdot_out);
}

int mlip_backward_energy(mlip_ctx* ctx, const float* Ebar, const float* lam_out, float* grad_params, float* lam_in) {
  if (!ctx) return MLIP_E_INVALID;
  return model_backward_energy(ctx, Ebar, lam_out, grad_params, lam_in);
}

int mlip_train_step(mlip_ctx* ctx, int64_t n_atoms, int32_t n_structs, const float* pos, const int32_t* species,
                    const int32_t* struct_ptr, const float* cell, float cutoff, const float* params, const float* E_ref,
                    const float* F_ref, float* loss, float* E, float* F, float* grad_params, float* phase_ms_host) {
  if (!ctx) return MLIP_E_INVALID;
  if (ctx->cfg.model_kind == MLIP_MODEL_STAGE) MLIP_FAIL(ctx, MLIP_E_UNSUPPORTED, "train_step: a stage is driven phase by phase");
  if (!E_ref || !F_ref || !loss || !E || !F || !grad_params) MLIP_FAIL(ctx, MLIP_E_INVALID, "train_step: null pointer");
  hipStream_t st = ctx->stream;
  StepBufs* sb = (StepBufs*)ctx->step_bufs;
  hipEvent_t ev[6];
  const bool timed = phase_ms_host != nullptr;
  if (timed) {
    for (int k = 0; k < 6; ++k)
      if (hipEventCreate(&ev[k]) != hipSuccess) {  // destroy the ones already made before reporting
        for (int q = 0; q < k; ++q) hipEventDestroy(ev[q]);
        MLIP_FAIL(ctx, MLIP_E_HIP, "train_step: hipEventCreate failed");
      }
    if (hipEventRecord(ev[0], st) != hipSuccess) {
      for (auto& e : ev) hipEventDestroy(e);
      MLIP_FAIL(ctx, MLIP_E_HIP, "train_step: hipEventRecord failed");
    }
  }
  int64_t n_edges = 0;
  int s = mlip_graph_build(ctx, n_atoms, n_structs, pos, struct_ptr, cell, cutoff, &n_edges);
  if (s == MLIP_OK && timed) hipEventRecord(ev[1], st);
  if (s == MLIP_OK) s = model_forward_energy(ctx, pos, species, params, nullptr, E, nullptr);
  if (s == MLIP_OK && timed) hipEventRecord(ev[2], st);
  if (s == MLIP_OK) s = model_forward_force(ctx, nullptr, F, nullptr);
  if (s == MLIP_OK) s = model_loss(ctx, E, F, E_ref, F_ref, loss, sb->Ebar, sb->v);
  if (s == MLIP_OK && timed) hipEventRecord(ev[3], st);
  if (s == MLIP_OK && hipMemsetAsync(grad_params, 0, sizeof(float) * ctx->n_params, st) != hipSuccess) s = MLIP_E_HIP;
  if (s == MLIP_OK && ctx->d_grad_alpha && ctx->grad_alpha_structs < ctx->B) {
    ctx->err = "train_step: the registered coefficient-gradient buffer holds fewer rows than the batch has structures";
    s = MLIP_E_CAPACITY;
  }
  if (s == MLIP_OK && ctx->d_grad_alpha &&
      hipMemsetAsync(ctx->d_grad_alpha, 0, sizeof(float) * (size_t)ctx->B * ctx->cfg.n_experts, st) != hipSuccess)
    s = MLIP_E_HIP;
  if (s == MLIP_OK) s = model_backward_force(ctx, sb->v, nullptr, grad_params, nullptr);
  if (s == MLIP_OK && timed) hipEventRecord(ev[4], st);
  if (s == MLIP_OK) s = model_backward_energy(ctx, sb->Ebar, nullptr, grad_params, nullptr);
  if (s == MLIP_OK && timed) hipEventRecord(ev[5], st);
  if (timed) {
    if (s == MLIP_OK) {
      if (hipEventSynchronize(ev[5]) != hipSuccess) s = MLIP_E_HIP;
      for (int k = 0; k < 5 && s == MLIP_OK; ++k)
        if (hipEventElapsedTime(&phase_ms_host[k], ev[k], ev[k + 1]) != hipSuccess) s = MLIP_E_HIP;
    }
    for (auto& e : ev) hipEventDestroy(e);
    if (s == MLIP_OK) s = input_status(ctx);  // the call has waited anyway: report clamped species, coincident atoms
  }
  return s;
}

}  // extern "C"
