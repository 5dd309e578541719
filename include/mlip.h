/*
 * libmlip -- the four-phase training step of a conservative message-passing interatomic
 * potential on one MI355X (gfx950), behind a C ABI.
 *
 * A training iteration of a conservative potential has four compute phases (paper, Sec. 2
 * "Training MLIPs with Four Phases"): Forward Energy (FE) predicts E, Forward Force (FF)
 * obtains F = -dE/dx by differentiating FE, Backward Force (BF) back-propagates the force
 * loss through FF (the double backward) and Backward Energy (BE) back-propagates through FE.
 * The parameter gradient is split between the last two as in Eq. 2 (Sec. 4.1, Pass 1,
 * Rule 2): BF contributes only the second-order term, BE every first-order term.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its name ends in _host.  The caller owns every
 *    buffer it passes; the library owns the context and all workspace inside it.
 *  - All floating-point tensors are float32, row-major, densely packed.  Indices are int32.
 *  - Calls enqueue work on the HIP stream given at mlip_create and return without waiting,
 *    except where "synchronous" is stated.  The library never uses atomics on floating-point
 *    data: results are bitwise reproducible from run to run.
 *  - Return value: MLIP_OK (0) or a negative mlip_status; no C++ exception crosses the
 *    boundary.  mlip_last_error gives a message for the last failure on a context.
 *  - There is no CPU fallback: every step of the path runs in the library's GPU kernels.
 *
 * Parameter vector (float32, each tensor row-major [out, in], concatenated in this order):
 *    whole model : emb[S,C]; per layer {W1[H,K], W2[C,H], V1[C,C], V2[C,C]} (edge MLP depth 2)
 *                  or {W1[H,K], W2[H,H], W3[C,H], V1, V2} (depth 3); U[C,C]; w_o[C]
 *    equivariant : emb[S,C]; per layer {W1[H,K], W2[n_paths*C,H] (row = path*C + channel; n_paths = 11 for
 *                  l_max = 2, 23 for l_max = 3), Wl0[C,C] .. Wl{l_max}[C,C]}; U[C,C]; w_o[C]
 *    stage       : the per-layer blocks only.
 *    With n_experts > 0 the node-level matrices (V1, V2; Wl0 .. Wl{l_max}) are banks
 *    [n_experts, C, C] in place of [C, C] (see mlip_set_expert_weights).
 *
 * Model (no biases anywhere; sigma = SiLU):
 *    phi_k(r) = exp(-gamma (r - k r_c/(K-1))^2), gamma = ((K-1)/r_c)^2 / 2;
 *    f_c(r) = (1 + cos(pi r / r_c)) / 2;
 *    invariant layer: w_e = W2 sigma(W1 phi(r_e))  (depth 3: W3 sigma(W2 sigma(W1 phi))),
 *        a_i = sum_{e=(i<-j)} f_c(r_e) w_e (.) h_j,   h_i <- h_i + V2 sigma(V1 a_i);
 *    equivariant layer (features h_i[c; l m], l <= l_max = 2 or 3): radial weights R_e = W2 sigma(W1 phi(r_e)) as
 *        [n_paths, C]; m_e[c; l3 m3] = f_c(r_e) sum_p R_e[p, c] sum_{m1 m2} T^p[m1 m2 m3]
 *        h_j[c; l1 m1] Y_{l2 m2}(r_e / r_e) over the even-parity paths p = (l1, l2, l3) with every degree <= l_max
 *        (triangle rule, l1 + l2 + l3 even, ordered by (l1, l2, l3): 11 paths for l_max = 2, 23 for 3) with real Gaunt
 *        tensors T^p scaled to sum T^2 = 2 l3 + 1 and component-normalised real harmonics Y;
 *        a_i = sum_e m_e;  u_i[l] = Wl^(l) a_i[l];  h_i <- h_i + u_i, or with mlip_config.gate the gated
 *        update h_i[c; 0] += sigma(u_i[c; 0]), h_i[c; l m] += sigmoid(u_i[c; 0]) u_i[c; l m];
 *        embedding into and readout from l = 0;
 *    readout: E_s = sum_{i in s} w_o . sigma(U h_i);   h^0_i = emb[species_i];
 *    loss: L = mean_s (E_s - E_ref,s)^2 + force_weight * mean_{i,alpha} (F - F_ref)^2.
 */
#ifndef MLIP_H
#define MLIP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mlip_ctx mlip_ctx;

typedef enum {
  MLIP_OK = 0,
  MLIP_E_INVALID = -1,     /* null pointer, non-positive size, cutoff <= 0 or > a cell height, singular cell, bad order of calls' arguments */
  MLIP_E_CAPACITY = -2,    /* more atoms / structures / edges than the context was created for */
  MLIP_E_UNSUPPORTED = -3, /* unsupported model shape or option; a cell too skewed for the float32 binning */
  MLIP_E_STATE = -4,       /* phase called out of order (FE -> FF -> BF -> BE) or without a graph */
  MLIP_E_HIP = -5,         /* a HIP runtime call failed */
  MLIP_E_POSITION = -6     /* a position lies outside its cell, or is not finite (found at graph build) */
} mlip_status;

enum { MLIP_MODEL_INVARIANT = 0, MLIP_MODEL_EQUIVARIANT = 1, MLIP_MODEL_STAGE = 2 };
enum { MLIP_GEMM_FP32 = 0, MLIP_GEMM_BF16 = 1 };

typedef struct {
  int32_t model_kind;       /* MLIP_MODEL_* */
  int32_t n_species;        /* S (ignored for a stage) */
  int32_t channels;         /* C, multiple of 4 */
  int32_t n_layers;
  int32_t n_rbf;            /* K: multiple of 4 in [4, 1024] */
  int32_t edge_hidden;      /* H, multiple of 4 */
  int32_t edge_mlp_depth;   /* 2 or 3 */
  int32_t l_max;            /* 0 (invariant, stage); 2 or 3 (equivariant: features up to that degree, 9 / 16 components, 11 / 23 coupling paths) */
  int32_t gemm_dtype;       /* MLIP_GEMM_FP32, or MLIP_GEMM_BF16: both operands of every matrix
                               product rounded to bf16 (nearest even), fp32 accumulation; the
                               radial-filter jets (outputs of such a product) are also kept in
                               bf16 unless filter_fp32 is set, and with them (equivariant model, l_max = 2)
                               the sender rows that the tensor product gathers per edge are read from bf16
                               copies of the node tables; node features, pre-activations and all sums stay fp32 */
  int32_t n_experts;        /* 0: dense.  > 0 (whole models only): the node-level matrices of every layer
                               (invariant: the update MLP's two; equivariant: the three per-l mixing
                               matrices) are banks [n_experts][C][C] in the parameter vector, merged
                               per structure with mlip_set_expert_weights' coefficients */
  int32_t gate;             /* 0: the equivariant node update is linear, h += W^(l) a.  1 (equivariant model
                               only): gated nonlinearity, with u = W^(l) a per channel
                               h_0 += silu(u_0), h_lm += sigmoid(u_0) u_lm for l = 1, 2 */
  int32_t filter_fp32;      /* bf16 mode only (ignored otherwise).  0: the radial-filter jets f_c w(r) -- outputs of a
                               bf16 product, consumed element-wise by the message kernels -- are stored in bf16, as a
                               mixed-precision linear layer returns them (half the bytes of the largest edge tensor).
                               1: they are stored in fp32 and the tensor product gathers fp32 sender rows, so that bf16
                               rounding touches matrix-product operands only */
  int32_t position_grad;    /* 1: also allocate the workspace for the position gradient dL/dx (mlip_set_position_grad);
                               0: none, and that call is refused */
  float cutoff;             /* r_c, Angstrom */
  float force_weight;       /* weight of the force term of the loss */
  int64_t max_atoms;        /* capacities the workspace is sized for */
  int64_t max_structs;
  int64_t max_edges;
} mlip_config;

/* Synchronous.  Allocates the context and all device workspace for the given capacities.
 * hip_stream is a hipStream_t (NULL = the default stream); it must outlive the context. */
int mlip_create(const mlip_config* cfg, void* hip_stream, mlip_ctx** out);
/* Synchronous.  Waits for the stream, frees everything.  NULL is accepted. */
int mlip_destroy(mlip_ctx* ctx);
/* Length of the flat parameter vector for this context's model. */
int64_t mlip_param_count(const mlip_ctx* ctx);
/* Message of the last failing call on this context (host string owned by the context). */
const char* mlip_last_error(const mlip_ctx* ctx);
/* Bytes of device memory held by the context. */
int64_t mlip_workspace_bytes(const mlip_ctx* ctx);

/* Radius graph of a batch of structures (cell-list binning, receiver-sorted CSR).
 * Edge e = (i <- j, S) exists iff |x_j + S.cell - x_i|^2 < cutoff^2 in float32 (differences
 * first, then the shift S.cell = (Sx a1 + Sy a2) + Sz a3 rounded after every operation, then the
 * three squares summed left to right, no fused multiply-add) and (j, S) != (i, 0); i, j in the
 * same structure.  Rows are receivers in global atom order; inside a row edges are ordered by
 * (sender, then (Sx+1)*9 + (Sy+1)*3 + (Sz+1)).
 *   pos[N,3], struct_ptr[B+1] (atom ranges of the structures), cell[B,3,3] (rows = lattice
 *   vectors a1, a2, a3 of each structure).  Per structure the cell is one of
 *   - diagonal (orthorhombic): positions in [0, L_a) exactly, cutoff <= every edge L_a;
 *   - a general non-singular lattice (triclinic, either handedness): fractional coordinates
 *     x . cell^-1 in [0, 1] (evaluated in float32, 1e-5 slack), cutoff (1 + 1e-4) <= every
 *     perpendicular height V / |a_b x a_c| (so that S in {-1, 0, 1}^3 covers the cutoff sphere),
 *     and the longest edge at most 50 times the smallest height (MLIP_E_UNSUPPORTED otherwise:
 *     reduce the lattice first);
 *   - all zeros: a molecule in vacuum, no images (S = 0), positions anywhere (finite).
 *   A cell with some but not all lattice vectors zero (a slab or wire) is refused as singular.
 * cutoff must equal mlip_config.cutoff (MLIP_E_INVALID otherwise): the radial basis and the envelope
 * of the context's model live on [0, mlip_config.cutoff], so the edge set has to end there too.
 * Synchronous: reads struct_ptr and cell back to validate them and returns the edge count in
 * *n_edges_host.  On MLIP_E_CAPACITY *n_edges_host holds the count that was needed.
 * The graph stays in the context until the next build. */
int mlip_graph_build(mlip_ctx* ctx, int64_t n_atoms, int32_t n_structs, const float* pos,
                     const int32_t* struct_ptr, const float* cell, float cutoff,
                     int64_t* n_edges_host);
/* Sizes of the current graph, written to host integers (any may be NULL).  Does not wait. */
int mlip_graph_sizes(const mlip_ctx* ctx, int64_t* n_atoms_host, int64_t* n_structs_host, int64_t* n_edges_host);
/* Copies the current graph into caller buffers (any may be NULL): row_ptr[N+1], sender[E],
 * shift[E,3] (int32 components in {-1,0,1}), rev[E] (index of the opposite edge j <- i, -S).
 * Asking for rev makes the call synchronous (it checks mlip_input_status first). */
int mlip_graph_export(mlip_ctx* ctx, int32_t* row_ptr, int32_t* sender, int32_t* shift, int32_t* rev);
/* The pairing of opposite edges that the model phases work with (an edge and its opposite have the same length, so
 * the radial network of the model is evaluated once per pair): slot[E] (device, int32) = 2 u + d, where u in
 * [0, E/2) is the edge's pair -- pairs are numbered in the order of their lower-numbered edges -- and d = 0 for the
 * pair's lower-numbered edge, 1 for the other; pair_edge[E/2] (device, int32, may be NULL) = the lower-numbered edge
 * of each pair.  Synchronous (checks mlip_input_status first: an edge without an opposite has no pair). */
int mlip_graph_export_pairs(mlip_ctx* ctx, int32_t* slot, int32_t* pair_edge);

/* For callers that cannot allocate device memory at this point -- code under HIP graph capture set-up,
 * tight serving loops that rebuild the neighbour list every step, harnesses that forbid hipMalloc: the
 * radius graph of mlip_graph_build without a context and without any device allocation.  Same edge rule,
 * same row and in-row order, same kernels; their work arrays live in a file-scope device array of the
 * library (about 13 MB per GPU, held from the first use on that GPU until the process ends).
 *   Inputs (device): pos[N,3], struct_ptr[B+1], cell[B,3,3]; hip_stream = the hipStream_t to run on.
 *   Outputs (device, caller-allocated): row_ptr[N+1], sender[edge_capacity], shift[edge_capacity,3],
 *   rev[edge_capacity]; *n_edges_host = the edge count E (entries beyond E are not written).
 * Limits: N <= 16384 atoms, B <= 1024 structures, E <= min(edge_capacity, 1048576); beyond them
 * MLIP_E_CAPACITY (*n_edges_host then holds the count that was needed if it was the edges), other errors
 * as mlip_graph_build; mlip_graph_build_static_error() returns the calling thread's last message.
 * Synchronous like mlip_graph_build (it reads struct_ptr, cell and the edge count back), so it cannot be
 * recorded into a HIP graph itself.  Calls no hipMalloc / hipFree.  All calls on one GPU share that GPU's
 * work array: two calls that overlap in time on one GPU (other threads, other streams) race; calls on
 * different GPUs do not.  Nothing is kept between calls that a later call relies on. */
int mlip_graph_build_static(int64_t n_atoms, int32_t n_structs, const float* pos, const int32_t* struct_ptr,
                            const float* cell, float cutoff, void* hip_stream, int64_t edge_capacity,
                            int32_t* row_ptr, int32_t* sender, int32_t* shift, int32_t* rev, int64_t* n_edges_host);
const char* mlip_graph_build_static_error(void);

/* Deferred input diagnostics.  Bad inputs that only a kernel can see, after the graph build's own
 * read-back, never fault the GPU and cannot fail the asynchronous call that met them: the kernel keeps
 * its accesses in bounds and raises a device flag.  This call waits for the stream (synchronous) and
 * reports, for the work enqueued since the last graph build:
 *   MLIP_E_INVALID   a species index outside [0, n_species) (it was clamped into range);
 *   MLIP_E_POSITION  two atoms of one structure at the same place (an edge of length zero, whose
 *                    direction was set to zero), or an edge without its opposite edge;
 * MLIP_OK otherwise.  Results of a step that reports an error here are not meaningful.
 * mlip_train_step with phase timing (already synchronous) ends with this check. */
int mlip_input_status(mlip_ctx* ctx);

/* Mixture of linear experts (Sec. 5.1 "Models": expert weight matrices combined by weighted
 * averaging into a temporary linear map).  alpha: device pointer [n_structs][n_experts], row s =
 * the coefficients of structure s, copied into the context asynchronously on the stream.  The
 * next mlip_forward_energy merges every bank per structure, W_s = sum_k alpha[s][k] W_k, and all
 * four phases use W_s for the atoms of s; BF and BE add alpha[s][k] * dL/dW_s into expert k's
 * slice of grad_params.  Required before mlip_forward_energy / mlip_train_step when the context
 * has n_experts > 0 (MLIP_E_STATE otherwise), with n_structs equal to the graph's; MLIP_E_INVALID
 * for a dense context.  The gradient with respect to alpha is not produced. */
int mlip_set_expert_weights(mlip_ctx* ctx, const float* alpha, int32_t n_structs);
/* Optional gradient with respect to those coefficients (what a router producing them would be
 * trained with): dL/dalpha[s][k] = sum over the banks of <dL/dW_s, W_k>.  grad_alpha: device pointer
 * [n_structs][n_experts] float32, or NULL to switch it off again (the default; nothing is computed
 * then).  While set, mlip_backward_force and mlip_backward_energy ADD their shares to it, as they do
 * for grad_params (the caller zeroes it), and mlip_train_step zeroes it itself before its two
 * backward phases.  n_structs = the number of rows the buffer holds (1 .. max_structs, MLIP_E_INVALID
 * otherwise; ignored with NULL): a later batch with more structures than that makes the backward
 * phases return MLIP_E_CAPACITY instead of writing past the buffer.  The caller keeps it alive. */
int mlip_set_expert_weight_grad(mlip_ctx* ctx, float* grad_alpha, int32_t n_structs);

/* FE.  Whole model: h^0 = emb[species], E[B] written.  Stage: h_in[N,C] read, h_out[N,C]
 * written, species and E may be NULL.  pos and params are copied into the context, so the
 * caller may reuse them at once.  Needs a graph built from the same positions. */
int mlip_forward_energy(mlip_ctx* ctx, const float* pos, const int32_t* species, const float* params,
                        const float* h_in, float* E, float* h_out);
/* FF.  Whole model: F[N,3] = -dE_total/dx.  Stage: g_out[N,C] = dE/dh_out read; g_in[N,C] =
 * dE/dh_in and F[N,3] = +(dH/dx)^T g_out (this stage's additive contribution to dE/dx) written. */
int mlip_forward_force(mlip_ctx* ctx, const float* g_out, float* F, float* g_in);
/* Loss and its cotangents (whole model): loss[1], Ebar[B] = dL/dE, v[N,3] = -dL/dF. */
int mlip_loss(mlip_ctx* ctx, const float* E, const float* F, const float* E_ref, const float* F_ref,
              float* loss, float* Ebar, float* v);
/* BF.  v[N,3] = -dL/dF.  Adds the second-order share of the parameter gradient (Eq. 2) to
 * grad_params.  Stage: hdot_in[N,C] = dL_F/d(dE/dh_in) read (NULL = zero), hdot_out written. */
int mlip_backward_force(mlip_ctx* ctx, const float* v, const float* hdot_in, float* grad_params,
                        float* hdot_out);
/* BE.  Adds the merged first-order share (Eq. 2) to grad_params.  Whole model: Ebar[B] = dL/dE.
 * Stage: lam_out[N,C] = dL/dh_out read, lam_in[N,C] = dL/dh_in written. */
int mlip_backward_energy(mlip_ctx* ctx, const float* Ebar, const float* lam_out, float* grad_params,
                         float* lam_in);
/* Optional position gradient of the loss, dL/dx.  It differentiates the forces once more in the positions, so
 * it is where the second derivatives of the edge features enter (d2 phi/dr2, f_c'', the second r-derivative of
 * the edge MLP; for the equivariant model also the second derivatives of the harmonics); the parameter gradient
 * never needs them, and nothing of this runs unless a buffer is registered here.
 *   grad_pos: device pointer [N,3] float32 that every later mlip_backward_energy (and mlip_train_step) OVERWRITES:
 *   whole model: dL/dx for the loss of mlip_loss's cotangents, i.e. d/dx [sum_s Ebar_s E_s + D_v E] with Ebar and
 *   v = -dL/dF held fixed; stage: this stage's additive share d/dx [<lam_out, h_out> + <hdot_in, g_in> + <v, p>].
 *   NULL switches it off again (the default).  Needs mlip_config.position_grad = 1 (MLIP_E_INVALID otherwise).
 * The caller keeps the buffer alive and sized for the batches it builds. */
int mlip_set_position_grad(mlip_ctx* ctx, float* grad_pos);

/* Whole step for a whole model: graph build, FE, FF, loss, BF, BE.  grad_params is overwritten.
 * phase_ms_host[5] (graph, FE, FF+loss, BF, BE; milliseconds from HIP events) makes the call
 * synchronous; NULL skips timing.  The graph build inside is synchronous in any case. */
int mlip_train_step(mlip_ctx* ctx, int64_t n_atoms, int32_t n_structs, const float* pos,
                    const int32_t* species, const int32_t* struct_ptr, const float* cell, float cutoff,
                    const float* params, const float* E_ref, const float* F_ref, float* loss, float* E,
                    float* F, float* grad_params, float* phase_ms_host);

/* Measurement aid (Appendix "Four Phase Profiler" times whole phases; this times one kernel).
 * Selecting a kernel id makes the library record a HIP-event pair, on the context's stream,
 * around every later launch of that kernel; 0 switches it off.  Selecting resets the counters.
 * mlip_kernel_timer_read is synchronous: it waits for the recorded events and returns the
 * number of launches and the sum of their durations in milliseconds. */
enum {
  MLIP_K_NONE = 0,
  MLIP_K_FE_HIDDEN_GEMM = 1,  /* jets of the first hidden layer: [2P,K] x [K,H]; P = E/2 pairs of opposite edges (equal
                                 lengths: the edge MLP and its adjoints are evaluated once per pair) */
  MLIP_K_FE_FILTER_GEMM = 2,  /* last edge-MLP product with the envelope epilogue: [2P,H] x [H,C] */
  MLIP_K_MSG_FE = 3,          /* gather * filter, segmented sum into receivers */
  MLIP_K_MSG_FF = 4,
  MLIP_K_MSG_BF = 5,
  MLIP_K_MSG_BE = 6,
  MLIP_K_BF_DGRAD = 7,        /* [P,C] x [C,H] data gradient with the activation-derivative epilogue */
  MLIP_K_BE_DGRAD = 8,
  MLIP_K_BF_WGRAD = 9,        /* [C,P] x [P,H] weight gradient of the last edge-MLP matrix (split-k) */
  MLIP_K_BE_WGRAD = 10,
  MLIP_K_GRAPH_NEIGHBOURS = 11,
  MLIP_K_EDGE_FEATURES = 12
};
int mlip_kernel_timer_select(mlip_ctx* ctx, int kernel_id);
/* Plain copy kernel of known size (dst[i] = src[i], n_floats a multiple of 4; reads and writes
 * 4*n_floats bytes each): the reference that hardware byte counters are scaled against. */
int mlip_copy_probe(mlip_ctx* ctx, float* dst, const float* src, int64_t n_floats);
int mlip_kernel_timer_read(mlip_ctx* ctx, int64_t* launches_host, float* total_ms_host);

/* Optimizer step (Table 2, runtime-control instruction "OS"; it follows the summation of the BF
 * and BE parameter gradients, Sec. 3).  The paper names no optimizer: this is AdamW.  In place,
 * asynchronous on the context's stream, float32 arithmetic:
 *   g = grad_scale * grad;  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *   params <- params - lr * ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *                             + weight_decay * params )
 * params, grad, m, v: device float32 [n] (m and v zero before step 1; the four arrays must not
 * overlap); step counts from 1; hyper_host is a host pointer, read before the call returns.
 * grad_scale folds a gradient average (e.g. 1 / number of accumulated micro-batches) into the pass.
 * MLIP_E_INVALID: null pointer, n < 0, step < 1, beta outside [0, 1), negative eps or weight_decay,
 * non-finite values.  n = 0 is a no-op.  Needs no graph and does not touch the context's state. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay, grad_scale;
} mlip_adamw;
int mlip_optimizer_step(mlip_ctx* ctx, int64_t n, float* params, const float* grad, float* m, float* v,
                        int32_t step, const mlip_adamw* hyper_host);

/* Graph-aware rescheduling (Appendix A.2, Algorithm 1): HOST routine, host pointers only.
 * Repacks the n_graphs graphs of a global batch (sizes_host[g] = atom count) into n_mb
 * micro-batches: graphs sorted by size descending (ties: lower index first), each placed into
 * the micro-batch of currently smallest total size (ties: lowest micro-batch index); every
 * micro-batch is then shuffled (Fisher-Yates from the last position down, draw t of micro-batch
 * j = splitmix64-finaliser(key(seed, stream j) + (t+1) * 0x9E3779B97F4A7C15) mod (t+1), key =
 * finaliser(seed xor j * 0x9E3779B97F4A7C15)) and tagged MLIP_GARS_COMM_FREE iff its largest
 * graph is at most (total size) / d_gp, else MLIP_GARS_DIST.
 * Outputs: mb_ptr_host[n_mb+1], order_host[n_graphs] (graph indices, grouped by micro-batch in
 * shuffled order), type_host[n_mb].  Returns MLIP_E_INVALID on null pointers, negative sizes,
 * n_mb < 1 or d_gp < 1. */
enum { MLIP_GARS_COMM_FREE = 0, MLIP_GARS_DIST = 1 };
int mlip_gars_pack(const int32_t* sizes_host, int64_t n_graphs, int32_t n_mb, int32_t d_gp, uint64_t seed,
                   int32_t* mb_ptr_host, int32_t* order_host, int32_t* type_host);

#ifdef __cplusplus
}
#endif
#endif /* MLIP_H */
