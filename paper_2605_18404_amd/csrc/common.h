// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/mlip.h"

#define MLIP_HIP_CHECK(ctx, expr)                                                         \
  do {                                                                                    \
    hipError_t _e = (expr);                                                               \
    if (_e != hipSuccess) {                                                               \
      (ctx)->err = std::string(#expr) + ": " + hipGetErrorString(_e);                     \
      return MLIP_E_HIP;                                                                  \
    }                                                                                     \
  } while (0)

#define MLIP_FAIL(ctx, code, msg) \
  do {                            \
    (ctx)->err = (msg);           \
    return (code);                \
  } while (0)

#define MLIP_TRY(expr)          \
  do {                          \
    int _s = (expr);            \
    if (_s != MLIP_OK) return _s; \
  } while (0)

// number of coupling paths (l1, l2, l3): every degree <= l_max, triangle rule, even parity (11 for l_max 2, 23 for 3)
inline int mlip_npath(int l_max) {
  int n = 0;
  for (int a = 0; a <= l_max; ++a)
    for (int b = 0; b <= l_max; ++b)
      for (int c = (a > b ? a - b : b - a); c <= a + b && c <= l_max; ++c) n += ((a + b + c) % 2 == 0);
  return n;
}

// Per-structure record used by the graph kernels (built on the host at graph build).
enum CellKind { CELL_ORTHO = 0, CELL_TRICLINIC = 1, CELL_FREE = 2 };
struct StructMeta {
  int32_t atom_begin, atom_end;
  int32_t nb[3];     // bins per axis
  int32_t bin_base;  // first global bin of this structure
  int32_t kind;      // CellKind: diagonal cell, general lattice, or a molecule in vacuum (zero cell)
  float lat[9];      // rows = lattice vectors (all zero for a molecule)
  float inv[9];      // binning coordinate f_a = sum_b (x_b - origin_b) inv[3 b + a], in [0, 1) inside the cell / bounding box
  float origin[3];   // zero for periodic cells; corner of the bounding box of a molecule
};

struct PartialBuf {  // split-k / chunk partial sums, reduced in a fixed order
  float* buf = nullptr;
  int64_t cap = 0;  // floats
};

// bits of the deferred input-diagnostics word (mlip_input_status)
enum { INPUT_NO_REVERSE_EDGE = 1, INPUT_BAD_SPECIES = 2, INPUT_COINCIDENT = 4 };

enum Phase { PH_NONE = 0, PH_GRAPH = 1, PH_FE = 2, PH_FF = 3, PH_BF = 4, PH_BE = 5 };

struct LayerOffsets {  // offsets (in floats) into the flat parameter vector
  int64_t W[3];        // edge MLP matrices (W[2] unused for depth 2)
  int64_t V1, V2;      // invariant update
  int64_t Wl[4];       // equivariant per-l mixing (l = 0..l_max)
};

struct mlip_ctx {
  mlip_config cfg{};
  hipStream_t stream = nullptr;
  std::string err;
  std::vector<void*> allocs;
  int64_t bytes = 0;
  int phase = PH_NONE;
  // sizes of the current batch
  int64_t N = 0, E = 0;
  int64_t Eu = 0;  // edge pairs: E / 2
  int32_t B = 0;
  int64_t n_params = 0;
  int64_t off_emb = -1, off_U = -1, off_wo = -1;
  std::vector<LayerOffsets> lay;

  // ---- graph
  StructMeta* d_meta = nullptr;       // [max_structs]
  int32_t* d_atom_struct = nullptr;   // [N]
  int32_t* d_atom_bin = nullptr;      // [N]
  int32_t* d_bin_count = nullptr;     // [max_bins + 1]
  int32_t* d_bin_start = nullptr;     // [max_bins + 1]
  int32_t* d_bin_cursor = nullptr;    // [max_bins]
  int32_t* d_bin_atoms = nullptr;     // [N]
  int32_t* d_deg = nullptr;           // [N + 1]
  int32_t* d_row_ptr = nullptr;       // [N + 1]
  int32_t* d_key_tmp = nullptr;       // [max_edges] unsorted keys sender*27+code
  int32_t* d_sender = nullptr;        // [max_edges]
  int32_t* d_code = nullptr;          // [max_edges] shift code 0..26
  int32_t* d_receiver = nullptr;      // [max_edges]
  int32_t* d_rev = nullptr;           // [max_edges]
  // Edge pairs (model contexts only; null in a bare graph build).  An edge and its opposite have the same length, so all
  // that depends on the length alone -- the radial basis, the edge MLP, the filter jets and their adjoints -- is kept once
  // per pair: pair u = the rank of its lower-numbered edge among such edges, rows 2u and 2u + 1 of a per-pair jet matrix.
  int2* d_se = nullptr;               // [max_edges] (sender, slot): slot = 2 u + (0 for the pair's lower-numbered edge, 1 for the other)
  int32_t* d_und = nullptr;           // [max_edges / 2 + 1] the lower-numbered edge of each pair
  int32_t* d_pair_pre = nullptr;      // [max_edges + 1] scan work array of the pair numbering
  int32_t* d_scan_tmp = nullptr;      // block sums for the scans
  int32_t* d_flag = nullptr;          // device flags [4]: word 0 = positions outside their cell (read by the graph build);
                                      // word 1 = deferred input diagnostics (INPUT_* bits, read by input_status)
  float* d_bounds = nullptr;          // [max_structs][6] bounding boxes (min xyz, max xyz), molecules only
  int64_t max_bins = 0;
  std::vector<StructMeta> h_meta;
  std::vector<int32_t> h_struct_ptr;
  std::vector<float> h_cell;

  // ---- model workspace (see model.hip)
  float* d_pos = nullptr;      // [N,3] copy taken at FE
  float* d_params = nullptr;   // copy taken at FE
  int32_t* d_species = nullptr;
  float4* d_geo = nullptr;     // [E] unit vector and length of each edge
  void* model_ws = nullptr;    // workspace of the model kind, owned by its translation unit
  void* step_bufs = nullptr;   // cotangent buffers of mlip_train_step
  PartialBuf partial;
  // bf16 products only: weight arrays mirrored in bf16 (refreshed once per forward pass), so that
  // the matrix at f32 + k is also available, already rounded, at b16 + k
  struct Shadow { const float* f32; __bf16* b16; int64_t n; };
  std::vector<Shadow> shadows;

  // ---- mixture of linear experts (n_experts > 0)
  float* d_alpha = nullptr;        // [max_structs][n_experts] coefficients (mlip_set_expert_weights)
  int32_t alpha_structs = -1;      // how many rows of d_alpha are set
  float* d_grad_alpha = nullptr;   // caller's buffer [B][n_experts] for dL/dalpha, or null (mlip_set_expert_weight_grad)
  int32_t grad_alpha_structs = 0;  // rows the caller said that buffer holds
  int4* d_row_groups = nullptr;    // row tiles of 64 atoms that never straddle a structure: (first, end, structure, 0)
  std::vector<int4> h_row_groups;
  std::vector<int32_t> h_k_ranges;
  int32_t* d_struct_ptr = nullptr; // [copies * max_structs + 1] first row of every (copy, structure) block, then the end
  int64_t n_row_groups = 0;        // row tiles per copy of the atom rows

  // ---- optional position gradient (mlip_set_position_grad): caller's buffer [N,3] that BE fills, or null
  float* d_grad_pos = nullptr;

  // ---- kernel timer (mlip_kernel_timer_select / _read): event pairs around one kernel's launches
  int timed_kernel = 0;
  std::vector<hipEvent_t> tev;  // pool, pairs (start, stop)
  size_t tev_used = 0;
};

// Scope guard: brackets the launches made inside its lifetime with a HIP-event pair when the
// given kernel id is the one selected for timing.  Costs nothing otherwise.
struct KernelTimer {
  mlip_ctx* c;
  bool on;
  KernelTimer(mlip_ctx* ctx, int id) : c(ctx), on(ctx->timed_kernel == id && id != 0) {
    if (!on) return;
    if (c->tev_used + 2 > c->tev.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
      c->tev.push_back(a);
      c->tev.push_back(b);
    }
    hipEventRecord(c->tev[c->tev_used], c->stream);
  }
  ~KernelTimer() {
    if (!on) return;
    hipEventRecord(c->tev[c->tev_used + 1], c->stream);
    c->tev_used += 2;
  }
};

void* ctx_alloc(mlip_ctx* ctx, size_t bytes);  // returns nullptr on failure (err set)

// graph.hip
int graph_alloc(mlip_ctx* ctx);
int graph_build(mlip_ctx* ctx, int64_t n_atoms, int32_t n_structs, const float* pos, const int32_t* struct_ptr,
                const float* cell, float cutoff, int64_t* n_edges_host);
int graph_export(mlip_ctx* ctx, int32_t* row_ptr, int32_t* sender, int32_t* shift, int32_t* rev);
int input_status(mlip_ctx* ctx);
int graph_export_shift(mlip_ctx* ctx, int32_t* shift);
int graph_export_pairs(mlip_ctx* ctx, int32_t* slot, int32_t* pair_edge);
constexpr int GRAPH_SCAN_TILE = 2048;  // elements per workgroup of the graph build's scans: d_scan_tmp holds one int per tile (+ 2)

// model.hip (invariant model and pipeline stage) / equivariant.hip (l <= 2 model)
#define MLIP_DECLARE_MODEL(pfx)                                                                                       \
  int pfx##_alloc(mlip_ctx* ctx);                                                                                     \
  void pfx##_free(mlip_ctx* ctx);                                                                                     \
  int pfx##_forward_energy(mlip_ctx* ctx, const float* pos, const int32_t* species, const float* params,             \
                           const float* h_in, float* E, float* h_out);                                                \
  int pfx##_forward_force(mlip_ctx* ctx, const float* g_out, float* F, float* g_in);                                  \
  int pfx##_backward_force(mlip_ctx* ctx, const float* v, const float* hdot_in, float* grad, float* hdot_out);        \
  int pfx##_backward_energy(mlip_ctx* ctx, const float* Ebar, const float* lam_out, float* grad, float* lam_in);
MLIP_DECLARE_MODEL(inv)
MLIP_DECLARE_MODEL(eqv)
int inv_loss(mlip_ctx* ctx, const float* E, const float* F, const float* E_ref, const float* F_ref, float* loss,
             float* Ebar, float* v);
