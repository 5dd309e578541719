// Equivariant message-passing potential (features up to degree l_max = 2 or 3): FE / FF / BF / BE with
// hand-derived adjoints.  Everything that depends on l_max -- component and path counts, coupling
// tables, the harmonics -- comes from G = gaunt::Tab<l_max>; kernels and phases are templates on G.
//
// Node features h[m][n][c], m = 0..NM-1 the real spherical-harmonic component (l=0 | y,z,x | five
// l=2 | seven l=3), stored component-major so every l block is a plain [(2l+1) N, C] matrix for the per-l
// channel mixing.  Messages:  m_e = B(rho_e, h_j, Y_e),  B(rho, x, y)[m3] = sum_p rho_p
// sum_{m1 m2} T^p[m1 m2 m3] x[m1] y[m2]  (T = scaled real Gaunt couplings, gaunt_table.h),
// rho_e = f_c(r) R(r) in R^{NPATH x C} the radial filter, carried with its r-derivative rho'_e as
// a jet.  B is trilinear, so every derivative pass is B or one of its partial contractions:
//   FE  a_i      = sum_e B(rho, h_j, Y)
//   FF  mu_h[i] += sum_e B_x^T(rho, PY; mu_a[j])          (P = parity (-1)^l: the opposite edge
//       F_i      = sum_e s_e rhat_e + J_e^T nu_e            has Y -> PY, Ydot -> P Ydot, same r, rdot)
//         s_e  = sum_c <mu_a,i , B(rho', h_j, Y)> + <mu_a,j , B(rho', h_i, PY)>
//         nu_e = sum_c B_y^T(rho, h_j; mu_a,i) + P B_y^T(rho, h_i; mu_a,j),  J = dY/dr_vec
//   BF  adot_i   = sum_e B(rdot rho', h_j, Y) + B(rho, hdot_j, Y) + B(rho, h_j, Ydot)
//   BE  lam_h[i]+= sum_e B_x^T(rho, PY; lam_a[j]) + B_x^T(rdot rho', PY; mu_a[j]) + B_x^T(rho, P Ydot; mu_a[j])
// with the radial adjoints  X_bf[p,c] = rdot f_c t_p(h_j, Y, mu_a,i)  (derivative rows -> BF) and
// X_be[p,c] = f_c (t_p(h_j,Y,lam_a,i) + t_p(hdot_j,Y,mu_a,i) + t_p(h_j,Ydot,mu_a,i)) + f_c' rdot t_p(h_j,Y,mu_a,i)
// (value rows -> BE), t_p = the path-p trilinear form; they feed the same GEMM chains as the
// invariant model's edge MLP.
#include <algorithm>
#include <cmath>

#include "gaunt_table.h"
#include "shared_kernels.h"

// This file is compiled nine times (side by side).  With MLIP_EQV_LMAX = 2 or 3 and MLIP_EQV_PHASE = 0..3 (FE, FF, BF, BE)
// an object instantiates the kernels of one phase for one set of coupling tables and defines eqv_phase_l<l_max>_<phase>;
// with MLIP_EQV_PHASE = -1 it holds the model's interface functions (workspace, the four calls), which pick one of those
// eight by the context's l_max.
#ifndef MLIP_EQV_LMAX
#define MLIP_EQV_LMAX 2
#endif
#ifndef MLIP_EQV_PHASE
#define MLIP_EQV_PHASE -1
#endif
#define MLIP_EQV_DECLARE(l, ph) int eqv_phase_l##l##_##ph(mlip_ctx* ctx, float* out);
MLIP_EQV_DECLARE(2, 0) MLIP_EQV_DECLARE(2, 1) MLIP_EQV_DECLARE(2, 2) MLIP_EQV_DECLARE(2, 3)
MLIP_EQV_DECLARE(3, 0) MLIP_EQV_DECLARE(3, 1) MLIP_EQV_DECLARE(3, 2) MLIP_EQV_DECLARE(3, 3)

namespace {

struct EqvWs {
  float* paramsT = nullptr;
  // Opposite edges have the same length: what depends on the length alone is kept once per edge PAIR (Eu = E / 2 rows or
  // jets; pair u of an edge = slot >> 1, mlip_ctx::d_se), and the two edges' adjoint rows of X lie side by side (row = slot).
  float* jphi = nullptr;  // [Eu][2][K]
  float2* env = nullptr;  // [E]
  float2* env_u = nullptr;  // [Eu] the same per pair (rows of the filter product)
  std::vector<float*> U;    // [Eu][2][H]
  std::vector<__bf16*> SJ;  // bf16 GEMMs only: activated jets [Eu][2][H]
  std::vector<float*> Rho;  // [Eu][2][C][NPP]: per channel the NPATH path filters + padding, operand precision (fp32 or bf16)
  std::vector<float*> Wp;   // per layer: filter weights with rows regrouped to that order, [NPP C][H]
  std::vector<float*> WpT;  // and their transpose [H][NPP C]
  float* gWp = nullptr;     // [NPP C][H] weight gradient in the regrouped row order
  float* Wp0 = nullptr;     // first layer: the rows of its live paths only, [4 C][H], and the transpose [H][4 C]
  float* WpT0 = nullptr;
  float* WpZ = nullptr;     // last layer: the same for its live paths
  float* WpTZ = nullptr;
  std::vector<float*> Wm[4], WmT[4];  // expert banks of the per-l mixing matrices merged per structure: [B][C][C], and transposed
  float* cy = nullptr;      // [E][CY_LD] coupling coefficient x harmonic of the edge direction
  float* cyd = nullptr;     // [E][CY_LD] the same with the directional derivative of the harmonics (BF, BE)
  std::vector<float*> Y1;   // [Eu][H]  BF -> BE
  float* X = nullptr;       // [Eu][2][C][NPP] (the two edges of a pair), operand precision
  float* X2 = nullptr;      // [Eu][H]
  std::vector<float*> h, a, mu_h, mu_a, hd, ad;  // [NM][N][C]
  // bf16 filter jets only: packed bf16 copies [N][C][NMP] of the tables gathered per edge from the sender (per layer: features,
  // their tangents, the cotangent mu_a; one for the adjoint lam_a)
  std::vector<__bf16*> gh, ghd, gmu;
  __bf16* glam = nullptr;
  std::vector<float*> u, mu_u, ud;  // gated update only, [NM][N][C]: pre-activations W a, their FF cotangents, their BF tangents
  float* lam_u = nullptr;           // gated update only: BE adjoint of the pre-activations
  float* lam_h[2] = {nullptr, nullptr};
  float* lam_a = nullptr;
  float* y = nullptr;
  float* yd = nullptr;
  float* lam_y = nullptr;
  float* lam0 = nullptr;  // [N][C] scratch for the readout's adjoint
  float* eps = nullptr;
  float* Facc = nullptr;
  float* Fp = nullptr;      // [L][Eu][C / 64][3] force terms per layer, edge pair and block of 64 channels (C a multiple of 64)
  float* v = nullptr;
  float* Ebar = nullptr;
  // optional position gradient dL/dx (mlip_config.position_grad)
  float* U2 = nullptr;      // [Eu][H] second-derivative row of the hidden level
  float* Rj = nullptr;      // [Eu][2][C][12] radial weights R and dR/dr (before the envelope), fp32
  float* Rpp = nullptr;     // [Eu][C][12] d2R/dr2
  float* gp_acc = nullptr;  // [N,3]
};
inline EqvWs* ws_of(mlip_ctx* ctx) { return (EqvWs*)ctx->model_ws; }

// ------------------------------------------------------------------------------ geometry helpers
// Degree-3 harmonics (component normalisation, m = -3..3):  c35 y(3x^2 - y^2), c105 xyz, c21 y(5z^2 - 1), c7 z(5z^2 - 3),
// c21 x(5z^2 - 1), (c105/2) z(x^2 - y^2), c35 x(x^2 - 3y^2).  Gradients below are those of these forms as polynomials;
// every use projects them onto the tangent plane of the unit sphere, where the choice of form does not matter.
constexpr float S3 = 1.7320508075688772f, S15 = 3.872983346207417f, S5 = 2.23606797749979f;
constexpr float C35 = 2.0916500663351889f, C105 = 10.246950765959598f, C21 = 1.6201851746019651f, C7 = 1.3228756555322954f;

template <int NM>
__device__ __forceinline__ void sph_harm(float x, float y, float z, float (&Y)[NM]) {
  Y[0] = 1.f;
  Y[1] = S3 * y; Y[2] = S3 * z; Y[3] = S3 * x;
  Y[4] = S15 * x * y; Y[5] = S15 * y * z; Y[6] = 0.5f * S5 * (3.f * z * z - 1.f); Y[7] = S15 * x * z;
  Y[8] = 0.5f * S15 * (x * x - y * y);
  if constexpr (NM == 16) {
    const float f = 5.f * z * z - 1.f;
    Y[9] = C35 * y * (3.f * x * x - y * y);
    Y[10] = C105 * x * y * z;
    Y[11] = C21 * y * f;
    Y[12] = C7 * z * (f - 2.f);
    Y[13] = C21 * x * f;
    Y[14] = 0.5f * C105 * z * (x * x - y * y);
    Y[15] = C35 * x * (x * x - 3.f * y * y);
  }
}
// w = sum_m nu[m] grad_u Y_m  (polynomial gradient at the unit vector u)
template <int NM>
__device__ __forceinline__ float3 sph_grad_T(float x, float y, float z, const float (&nu)[NM]) {
  float3 w;
  w.x = S3 * nu[3] + S15 * (y * nu[4] + z * nu[7] + x * nu[8]);
  w.y = S3 * nu[1] + S15 * (x * nu[4] + z * nu[5] - y * nu[8]);
  w.z = S3 * nu[2] + S15 * (y * nu[5] + x * nu[7]) + 3.f * S5 * z * nu[6];
  if constexpr (NM == 16) {
    const float f = 5.f * z * z - 1.f, q = x * x - y * y;
    w.x += C35 * (6.f * x * y * nu[9] + 3.f * q * nu[15]) + C105 * (y * z * nu[10] + x * z * nu[14]) + C21 * f * nu[13];
    w.y += C35 * (3.f * q * nu[9] - 6.f * x * y * nu[15]) + C105 * (x * z * nu[10] - y * z * nu[14]) + C21 * f * nu[11];
    w.z += C105 * (x * y * nu[10] + 0.5f * q * nu[14]) + 10.f * C21 * z * (y * nu[11] + x * nu[13]) + C7 * (15.f * z * z - 3.f) * nu[12];
  }
  return w;
}
// Ydot = (dY/dr_vec) d = grad_u Y . d_perp / r,  d_perp = d - u (u.d)
template <int NM>
__device__ __forceinline__ void sph_dot(float x, float y, float z, float r, float3 d, float (&Yd)[NM]) {
  float ud = x * d.x + y * d.y + z * d.z;
  float inv = 1.f / r;
  float px = (d.x - x * ud) * inv, py = (d.y - y * ud) * inv, pz = (d.z - z * ud) * inv;
  Yd[0] = 0.f;
  Yd[1] = S3 * py; Yd[2] = S3 * pz; Yd[3] = S3 * px;
  Yd[4] = S15 * (y * px + x * py);
  Yd[5] = S15 * (z * py + y * pz);
  Yd[6] = 3.f * S5 * z * pz;
  Yd[7] = S15 * (z * px + x * pz);
  Yd[8] = S15 * (x * px - y * py);
  if constexpr (NM == 16) {
    const float f = 5.f * z * z - 1.f, q = x * x - y * y;
    Yd[9] = C35 * (6.f * x * y * px + 3.f * q * py);
    Yd[10] = C105 * (y * z * px + x * z * py + x * y * pz);
    Yd[11] = C21 * (f * py + 10.f * y * z * pz);
    Yd[12] = C7 * (15.f * z * z - 3.f) * pz;
    Yd[13] = C21 * (f * px + 10.f * x * z * pz);
    Yd[14] = C105 * (x * z * px - y * z * py + 0.5f * q * pz);
    Yd[15] = C35 * (3.f * q * px - 6.f * x * y * py);
  }
}
template <int NM>
__device__ __forceinline__ void loadm(const float* __restrict__ t, int64_t NC, int64_t off, float (&x)[NM]) {
#pragma unroll
  for (int m = 0; m < NM; ++m) x[m] = t[m * NC + off];
}
// The filter jets and their adjoints are stored per edge as [C][NPP]: the NPATH path values of one channel are
// contiguous (padded to a multiple of four), so a thread moves them with a few wide accesses instead of NPATH narrow ones.
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ uint32_t bf_pack(float lo, float hi) {
  __bf16 a = (__bf16)lo, b = (__bf16)hi;
  return (uint32_t)__builtin_bit_cast(unsigned short, a) | ((uint32_t)__builtin_bit_cast(unsigned short, b) << 16);
}
template <int NPATH>
__device__ __forceinline__ void load_rho(const float* __restrict__ row, int c, float (&rho)[NPATH]) {
  constexpr int NPP = (NPATH + 3) / 4 * 4;
  const float4* q = reinterpret_cast<const float4*>(row + c * NPP);
#pragma unroll
  for (int k = 0; k < NPP / 4; ++k) {
    const float4 a = q[k];
    const float v[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (4 * k + j < NPATH) rho[4 * k + j] = v[j];
  }
}
template <int NPATH>
__device__ __forceinline__ void load_rho(const __bf16* __restrict__ row, int c, float (&rho)[NPATH]) {
  constexpr int NPP = (NPATH + 3) / 4 * 4;
  const uint2* q = reinterpret_cast<const uint2*>(row + c * NPP);
#pragma unroll
  for (int k = 0; k < NPP / 4; ++k) {
    const uint2 a = q[k];
    const float v[4] = {bf_lo(a.x), bf_hi(a.x), bf_lo(a.y), bf_hi(a.y)};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (4 * k + j < NPATH) rho[4 * k + j] = v[j];
  }
}
template <int NPATH>
__device__ __forceinline__ void store_paths(float* __restrict__ row, int c, const float (&x)[NPATH]) {
  constexpr int NPP = (NPATH + 3) / 4 * 4;
  float4* q = reinterpret_cast<float4*>(row + c * NPP);
#pragma unroll
  for (int k = 0; k < NPP / 4; ++k)
    q[k] = make_float4(x[4 * k], 4 * k + 1 < NPATH ? x[4 * k + 1 < NPATH ? 4 * k + 1 : 0] : 0.f, 4 * k + 2 < NPATH ? x[4 * k + 2 < NPATH ? 4 * k + 2 : 0] : 0.f,
                       4 * k + 3 < NPATH ? x[4 * k + 3 < NPATH ? 4 * k + 3 : 0] : 0.f);
}
template <int NPATH>
__device__ __forceinline__ void store_paths(__bf16* __restrict__ row, int c, const float (&x)[NPATH]) {
  constexpr int NPP = (NPATH + 3) / 4 * 4;
  uint2* q = reinterpret_cast<uint2*>(row + c * NPP);
#pragma unroll
  for (int k = 0; k < NPP / 4; ++k) {
    const float b1 = 4 * k + 1 < NPATH ? x[4 * k + 1 < NPATH ? 4 * k + 1 : 0] : 0.f, b2 = 4 * k + 2 < NPATH ? x[4 * k + 2 < NPATH ? 4 * k + 2 : 0] : 0.f,
                b3 = 4 * k + 3 < NPATH ? x[4 * k + 3 < NPATH ? 4 * k + 3 : 0] : 0.f;
    q[k] = make_uint2(bf_pack(x[4 * k], b1), bf_pack(b2, b3));
  }
}

// Packed sender rows.  When the filter jets are stored in bf16, the node tables a kernel gathers per edge from the
// SENDER (features, their tangents, the two cotangents) are read from bf16 copies laid out [N][C][NMP]: the NM components
// of one (atom, channel) are contiguous (NMP = 10 for 9 components, 16 for 16), so a lane fetches its sender row with two
// wide loads instead of NM four-byte ones, and the gathers -- most of these kernels' memory traffic -- move 20 (32) bytes
// per table, lane and edge instead of 36 (64).  Both operands of the tensor product are then in the matrix products'
// operand precision; the receiver's own rows, all sums and every table itself stay fp32.
// (Used for l_max = 2 only: at l_max = 3 the kernels are bound by instruction issue, not by the gathers, and the
// conversions made them 3 % slower.)
template <int NM> struct PackedRow { static constexpr int NMP = NM == 9 ? 10 : 16; };
template <typename TF, typename G>
__host__ __device__ constexpr bool packed_rows() { return std::is_same<TF, __bf16>::value && G::LMAX == 2; }
struct __attribute__((aligned(4))) Words4 { uint32_t x, y, z, w; };
template <int NM>
__device__ __forceinline__ void load_packed(const __bf16* __restrict__ g, int64_t row, float (&x)[NM]) {
  static_assert(NM == 9 || NM == 16, "packed rows exist for l_max = 2 and 3");
  const uint32_t* p = reinterpret_cast<const uint32_t*>(g + row * PackedRow<NM>::NMP);
  const Words4 a = *reinterpret_cast<const Words4*>(p);
  const uint32_t lo[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) { x[2 * k] = bf_lo(lo[k]); x[2 * k + 1] = bf_hi(lo[k]); }
  if constexpr (NM == 9) {
    x[8] = bf_lo(p[4]);
  } else {
    const Words4 b = *reinterpret_cast<const Words4*>(p + 4);
    const uint32_t hi[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) { x[8 + 2 * k] = bf_lo(hi[k]); x[9 + 2 * k] = bf_hi(hi[k]); }
  }
}
// a single live component comes from the fp32 table; a full row from the packed copy when there is one
template <bool PACK, int NX>
__device__ __forceinline__ void gather_row(const float* __restrict__ tab, const __bf16* __restrict__ packed, int64_t NC, int64_t row,
                                           float (&x)[NX]) {
  if constexpr (PACK && NX > 1) load_packed(packed, row, x);
  else loadm(tab, NC, row, x);
}
// tab [NM][N][C] fp32 -> packed [N][C][NMP] bf16 (pad = 0)
template <int NM>
__global__ void k_pack_rows(const float* __restrict__ tab, int64_t NC, __bf16* __restrict__ packed) {
  constexpr int NMP = PackedRow<NM>::NMP;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NC) return;
  float x[NMP];
#pragma unroll
  for (int m = 0; m < NMP; ++m) x[m] = m < NM ? tab[m * NC + idx] : 0.f;
  uint32_t* q = reinterpret_cast<uint32_t*>(packed + idx * NMP);
#pragma unroll
  for (int k = 0; k < NMP / 2; ++k) q[k] = bf_pack(x[2 * k], x[2 * k + 1]);
}

struct RowChan {
  int row, c;
  bool active;
};
__device__ __forceinline__ RowChan row_chan(int N, int C) {
  int rpb = 256 / C;
  int rl = threadIdx.x / C;
  RowChan t;
  t.c = threadIdx.x % C;
  t.row = xcd_block() * rpb + rl;
  t.active = (rl < rpb) && (t.row < N);
  return t;
}

// ------------------------------------------------------------------------------ edge kernels
// One thread per (receiver row, channel); a row's edges are walked in order.  Every coupling term
// T^p[m1,m2,m3] Y[m2] is the same for all channels of an edge, so the products cy[n] =
// T_n Y[m2_n] (and cyd[n] with the directional derivative of Y) are tabulated once per edge and
// each term costs one multiply-add here.  With UNI (C a multiple of 64) all lanes of a wave
// share the row: the edge index is made wave-uniform, and the per-edge tables, indices and
// geometry then arrive through scalar loads.
template <bool UNI>
__device__ __forceinline__ int uni(int x) { return UNI ? __builtin_amdgcn_readfirstlane(x) : x; }

// UNI: the 64 lanes fetch the edge's table with TAB_LOADS coalesced loads and publish it in the
// wave's own LDS slot, from where every lane reads the entries it needs as broadcasts.  (LDS
// operations of one wave execute in order, so the next edge's copy cannot overtake the reads.)
template <typename G>
struct TabRegs { float v[G::TAB_LOADS]; };
template <typename G>
__device__ __forceinline__ TabRegs<G> tab_fetch(const float* __restrict__ src, int lane) {
  TabRegs<G> r;
#pragma unroll
  for (int k = 0; k < G::TAB_LOADS; ++k) r.v[k] = src[64 * k + lane];  // runs into the next edge's table (the allocation is padded): no branch
  return r;
}
template <typename G>
__device__ __forceinline__ void tab_publish(const TabRegs<G>& r, float* slot, int lane) {
#pragma unroll
  for (int k = 0; k < G::TAB_LOADS; ++k) slot[64 * k + lane] = r.v[k];
  __builtin_amdgcn_wave_barrier();
}

// The coupling entries n = (p; m1, m2, m3) are ordered by slot (p, m3), so a slot's entries are consecutive: sums over a
// slot's entries are kept in one register and handed on at the slot's last entry (ENT_SFIRST / ENT_SLAST), and a value that
// belongs to the slot is formed at its first entry.  No array over the slots is ever held.
// L0 (the model's first layer): the features entering it have their l = 0 component only (the embedding) and no tangent
// (the embedding does not depend on the positions), so of the coupling entries n = (p; m1, m2, m3) only those with m1 = 0
// contribute -- the paths (0, l, l), one entry per slot -- and one sender value per edge is gathered instead of a row of
// NM; FF needs no adjoint of the embedding, BE only the l = 0 component of it (the embedding's gradient).  Those paths
// are the first l_max + 1 in the path order, so the first layer's filter jets and their adjoints are computed, stored and
// multiplied for these paths alone: rows of 4 values per channel instead of NPP, a filter product of 4 C columns.
// LZ (the model's last layer, if it is not also the first): the readout takes the l = 0 component of its output only, so
// only the entries with m3 = 0 contribute -- the paths (l, l, 0), G::LAST_PATHS, whose filter rows are regrouped to the
// same rows of 4 -- and the cotangents mu_a, lam_a of that layer have their l = 0 component only: FE and BF produce one
// component, FF and BE gather one component of each adjoint instead of NM.
enum { LS_ANY = 0, LS_FIRST = 1, LS_LAST = 2 };  // which layer a tensor-product kernel is specialised for
// position of path p in a layer's stored filter rows
template <typename G, int LS>
__host__ __device__ constexpr int path_row(int p) { return LS == LS_LAST ? G::LAST_K[p] : p; }
template <int N>
__device__ __forceinline__ void zero(float (&x)[N]) {
#pragma unroll
  for (int k = 0; k < N; ++k) x[k] = 0.f;
}
// f(integral_constant<int, k>) for k = B..E-1, in order: the loops over the coupling entries index register arrays through
// tables, so every index must be a constant -- a loop the compiler leaves rolled would turn those arrays into scratch memory.
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (E - B == 1) {
    f(std::integral_constant<int, B>{});
  } else if constexpr (E - B > 1) {
    static_for<B, (B + E) / 2>(f);
    static_for<(B + E) / 2, E>(f);
  }
}

// Sum of v over the 64 lanes of a wave, delivered in lane 63 (other lanes hold partial sums): an inclusive scan inside each
// row of 16 lanes by shifts of 1, 2, 4, 8 (lanes shifted in from outside the row read zero), then lane 15 of a row added
// to the next row (rows 1 and 3), then lane 31 to rows 2 and 3.  Register-to-register: no LDS round trips.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_shifted(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, true));
}
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v += dpp_shifted<0x111, 0xf>(v);  // row_shr:1
  v += dpp_shifted<0x112, 0xf>(v);  // row_shr:2
  v += dpp_shifted<0x114, 0xf>(v);  // row_shr:4
  v += dpp_shifted<0x118, 0xf>(v);  // row_shr:8
  v += dpp_shifted<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
  v += dpp_shifted<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
  return v;
}

template <typename G, typename TF, bool UNI, int LS>
__global__ void __launch_bounds__(256) k_tp_fe(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                               const TF* __restrict__ Rho, const float* __restrict__ cyt,
                                               const float* __restrict__ h, const __bf16* __restrict__ gh, int N, int C,
                                               float* __restrict__ a) {
  constexpr bool PACK = packed_rows<TF, G>();  // sender rows from the packed bf16 copies
  constexpr bool L0 = LS == LS_FIRST, LZ = LS == LS_LAST;
  constexpr int NM = G::NM, NPATH = LS ? G::LMAX + 1 : G::NPATH, NPP = LS ? 4 : G::NPP, CY_LD = G::CY_LD;  // paths and row width of this layer
  constexpr int NA = LZ ? 1 : NM;  // components of the output that anything reads
  RowChan t = row_chan(N, C);
  if (!t.active) return;  // no workgroup barrier below
  const int64_t NC = (int64_t)N * C;
  float acc[NA];
  zero(acc);
  __shared__ float tabs[4][64 * G::TAB_LOADS];
  float* slot = tabs[threadIdx.x >> 6];
  const int lane = threadIdx.x & 63;
  const int e0 = uni<UNI>(row_ptr[t.row]), e1 = uni<UNI>(row_ptr[t.row + 1]);
  int2 sn = e0 < e1 ? se[e0] : make_int2(0, 0);
  for (int e = e0; e < e1; ++e) {
    const int j = sn.x, es = sn.y;  // sender; pair row 2u + (0 | 1) of the edge
    sn = se[e + 1 < e1 ? e + 1 : e];  // next edge's sender: its gathers need not wait for an index
    float x[L0 ? 1 : NM], rho[NPATH];
    const float* cy = cyt + (int64_t)e * CY_LD;
    TabRegs<G> tr;
    if constexpr (UNI) tr = tab_fetch<G>(cy, lane);
    gather_row<PACK>(h, gh, NC, (int64_t)j * C + t.c, x);
    load_rho(Rho + (int64_t)(es & ~1) * NPP * C, t.c, rho);
    if constexpr (UNI) { tab_publish<G>(tr, slot, lane); cy = slot; }
    float S = 0.f;  // sum_n cy[n] x[m1_n] over the entries of one slot
    static_for<0, G::NNZ>([&](auto n_) {
      constexpr int n = decltype(n_)::value;
      constexpr int sl = G::ENT_SLOT[n];
      if constexpr (L0) {
        if constexpr (G::ENT_M1[n] == 0) acc[G::SLOT_M3[sl]] = fmaf(rho[G::SLOT_P[sl]], cy[n] * x[0], acc[G::SLOT_M3[sl]]);
      } else if constexpr (!LZ || G::SLOT_M3[sl] == 0) {
        S = G::ENT_SFIRST[n] ? cy[n] * x[G::ENT_M1[n]] : fmaf(cy[n], x[G::ENT_M1[n]], S);
        if (G::ENT_SLAST[n]) acc[G::SLOT_M3[sl]] = fmaf(rho[path_row<G, LS>(G::SLOT_P[sl])], S, acc[G::SLOT_M3[sl]]);
      }
    });
  }
#pragma unroll
  for (int m = 0; m < NA; ++m) a[m * NC + (int64_t)t.row * C + t.c] = acc[m];
}

template <typename G, typename TF, bool UNI, int LS>
__global__ void __launch_bounds__(256, 2) k_tp_ff(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                  const float4* __restrict__ geo, const TF* __restrict__ Rho,
                                                  const float* __restrict__ cyt, const float* __restrict__ h,
                                                  const float* __restrict__ mu_a, const __bf16* __restrict__ gh,
                                                  const __bf16* __restrict__ gmu, const float* __restrict__ mu_h_next, int N,
                                                  int C, float* __restrict__ mu_h, float* __restrict__ Facc,
                                                  float* __restrict__ Fp) {
  // Two jobs per edge: the message this atom sends back along the reversed edge (cotangent of the layer's input features),
  // and the force terms.  The force that an edge pair exerts on its two atoms is equal and opposite (shown below), so with
  // UNI (a wave holds channels of one receiver row: its branches are uniform) only the pair's lower-numbered edge evaluates
  // it, in a second walk over the row's edges: the wave sums the term over its channels and stores it per (pair, channel
  // block of 64) in Fp [Eu][C / 64][3]; the rows' forces are collected from Fp afterwards (k_force_rows).  Without UNI
  // every edge evaluates its term, in one walk, into the row's Facc.
  constexpr bool PACK = packed_rows<TF, G>();  // sender rows from the packed bf16 copies
  constexpr bool L0 = LS == LS_FIRST, LZ = LS == LS_LAST;
  constexpr int NM = G::NM, NPATH = LS ? G::LMAX + 1 : G::NPATH, NPP = LS ? 4 : G::NPP, CY_LD = G::CY_LD, NNZ = G::NNZ;
  constexpr int NX = L0 ? 1 : NM;  // live components of the layer's input features
  constexpr int NU = LZ ? 1 : NM;  // live components of the cotangent of the layer's messages
  __shared__ float3 red[UNI ? 1 : 256];
  __shared__ float tabs[4][64 * G::TAB_LOADS];
  RowChan t = row_chan(N, C);
  float3 f = make_float3(0.f, 0.f, 0.f);
  if (t.active) {
    const int64_t NC = (int64_t)N * C;
    const int64_t io = (int64_t)t.row * C + t.c;
    float xi[NX], mi[NU];
    loadm(h, NC, io, xi);
    loadm(mu_a, NC, io, mi);
    float* slot = tabs[threadIdx.x >> 6];
    const int lane = threadIdx.x & 63;
    const int e0 = uni<UNI>(row_ptr[t.row]), e1 = uni<UNI>(row_ptr[t.row + 1]);

    // acc += the reversed edge's message: couplings of -u, i.e. the path's parity sign
    auto back_message = [&](const float* cy, const float (&rho)[NPATH], const float (&mj)[NU], float (&acc)[NM]) {
      float R = 0.f;
      static_for<0, G::NNZ>([&](auto n_) {
        constexpr int n = decltype(n_)::value;
        constexpr int sl = G::ENT_SLOT[n];
        if constexpr (!LZ || G::SLOT_M3[sl] == 0) {
          if (G::ENT_SFIRST[n]) R = G::PATH_SIGN[G::SLOT_P[sl]] * rho[path_row<G, LS>(G::SLOT_P[sl])] * mj[G::SLOT_M3[sl]];
          acc[G::ENT_M1[n]] = fmaf(cy[n], R, acc[G::ENT_M1[n]]);
        }
      });
    };
    // Force terms.  With W_n = x_j[m1] mu_i[m3] + sign_p x_i[m1] mu_j[m3] per coupling entry n = (p; m1, m2, m3), formed
    // once, both directions of the edge pair give
    //   radial:  s = sum_p rho'_p sum_{n in p} (T_n Y[m2]) W_n,      angular:  nu[m2] = sum_p rho_p sum_{n in (p, m2)} T_n W_n
    // (the opposite edge sees the harmonics of -u, i.e. the path's parity sign).  Seen from the opposite edge, W_n and
    // the coupling each change by the path's sign, so s is the same and nu[m2] changes by the parity of m2's degree, which
    // the gradient of the harmonics at -u turns into an overall minus: the term on the sender is minus this one.
    auto force_term = [&](const float* cy, const float (&xj)[NX], const float (&mj)[NU], const float (&rho)[NPATH],
                          const float (&rhop)[NPATH], const float4 g) -> float3 {
      float s = 0.f;
      float nu[NM];
      zero(nu);
      if constexpr (L0 || LZ) {  // few live entries (m1 = 0, or m3 = 0): each adds to both sums directly
        static_for<0, G::NNZ>([&](auto n_) {
          constexpr int n = decltype(n_)::value;
          constexpr int sl = G::ENT_SLOT[n], p = G::SLOT_P[sl], m3 = G::SLOT_M3[sl], m1 = G::ENT_M1[n], m2 = G::ENT_M2[n];
          if constexpr (L0 ? m1 == 0 : m3 == 0) {
            constexpr int pr = path_row<G, LS>(p);
            const float W = fmaf(G::PATH_SIGN[p] * xi[m1], mj[m3], xj[m1] * mi[m3]);
            s = fmaf(rhop[pr] * cy[n], W, s);
            nu[m2] = fmaf(rho[pr] * G::ENT_COEF[n], W, nu[m2]);
          }
        });
      } else if constexpr (G::LMAX == 2) {
        // few entries: the per-path and per-(path, m2) sums are kept side by side while the entries are walked in table order
        float sp[NPATH], Gy[G::NYSLOT];
        static_for<0, G::NNZ>([&](auto n_) {
          constexpr int n = decltype(n_)::value;
          constexpr int sl = G::ENT_SLOT[n], p = G::SLOT_P[sl], m3 = G::SLOT_M3[sl], m1 = G::ENT_M1[n], ys = G::ENT_YSLOT[n];
          const float W = fmaf(G::PATH_SIGN[p] * xi[m1], mj[m3], xj[m1] * mi[m3]);
          sp[p] = G::ENT_PFIRST[n] ? cy[n] * W : fmaf(cy[n], W, sp[p]);
          Gy[ys] = G::ENT_YFIRST[n] ? G::ENT_COEF[n] * W : fmaf(G::ENT_COEF[n], W, Gy[ys]);
        });
#pragma unroll
        for (int p = 0; p < NPATH; ++p) s = fmaf(rhop[p], sp[p], s);
#pragma unroll
        for (int ys = 0; ys < G::NYSLOT; ++ys) nu[G::YSLOT_M2[ys]] = fmaf(rho[G::YSLOT_P[ys]], Gy[ys], nu[G::YSLOT_M2[ys]]);
      } else {
        // many entries: they are walked in the order (path, m2), in which the runs of one (path, m2) pair and of one path are
        // consecutive, so both sums stay in one register each
        float sp = 0.f, gy = 0.f;
        static_for<0, G::NNZ>([&](auto k_) {
          constexpr int k = decltype(k_)::value;
          constexpr int n = G::YORD[k];
          constexpr int sl = G::ENT_SLOT[n], p = G::SLOT_P[sl], m3 = G::SLOT_M3[sl], m1 = G::ENT_M1[n], m2 = G::ENT_M2[n];
          const float W = fmaf(G::PATH_SIGN[p] * xi[m1], mj[m3], xj[m1] * mi[m3]);
          sp = G::YORD_PFIRST[k] ? cy[n] * W : fmaf(cy[n], W, sp);
          gy = G::YORD_YFIRST[k] ? G::ENT_COEF[n] * W : fmaf(G::ENT_COEF[n], W, gy);
          if (G::YORD_YLAST[k]) nu[m2] = fmaf(rho[p], gy, nu[m2]);
          if (G::YORD_PLAST[k]) s = fmaf(rhop[p], sp, s);
        });
      }
      const float3 w = sph_grad_T(g.x, g.y, g.z, nu);
      const float uw = g.x * w.x + g.y * w.y + g.z * w.z;
      const float inv = 1.f / g.w;
      return make_float3(s * g.x + (w.x - g.x * uw) * inv, s * g.y + (w.y - g.y * uw) * inv, s * g.z + (w.z - g.z * uw) * inv);
    };

    float acc[NM];
    if constexpr (LZ) {  // the readout's cotangent has its l = 0 component only
      zero(acc);
      acc[0] = mu_h_next[io];
    } else if constexpr (!L0) {
      loadm(mu_h_next, NC, io, acc);
    }
    if constexpr (!UNI || !L0) {  // (the first layer's input is the embedding: no cotangent to send back)
      int2 sn = e0 < e1 ? se[e0] : make_int2(0, 0);
      for (int e = e0; e < e1; ++e) {
        const int j = sn.x, es = sn.y;
        sn = se[e + 1 < e1 ? e + 1 : e];
        const float* cy = cyt + (int64_t)e * CY_LD;
        TabRegs<G> tr;
        if constexpr (UNI) tr = tab_fetch<G>(cy, lane);
        float mj[NU], rho[NPATH];
        const int64_t jo = (int64_t)j * C + t.c;
        gather_row<PACK>(mu_a, gmu, NC, jo, mj);
        const TF* rrow = Rho + (int64_t)(es & ~1) * NPP * C;
        load_rho(rrow, t.c, rho);
        if constexpr (!UNI) {  // one walk: the force term of every edge too
          const float4 g = geo[e];
          float xj[NX], rhop[NPATH];
          gather_row<PACK>(h, gh, NC, jo, xj);
          load_rho(rrow + NPP * C, t.c, rhop);
          if constexpr (!L0) back_message(cy, rho, mj, acc);
          if constexpr (G::LMAX == 3 && LS == LS_ANY) asm volatile("" ::: "memory");  // the table is read again rather than kept
          const float3 fe = force_term(cy, xj, mj, rho, rhop, g);
          f.x += fe.x; f.y += fe.y; f.z += fe.z;
        } else {
          tab_publish<G>(tr, slot, lane);
          back_message(slot, rho, mj, acc);
        }
      }
    }
    if constexpr (!L0) {
#pragma unroll
      for (int m = 0; m < NM; ++m) mu_h[m * NC + io] = acc[m];
    }
    if constexpr (UNI) {  // second walk: the force terms of the pairs whose lower-numbered edge this row receives
      int2 sn = e0 < e1 ? se[e0] : make_int2(0, 0);
      for (int e = e0; e < e1; ++e) {
        const int j = sn.x, es = sn.y;
        sn = se[e + 1 < e1 ? e + 1 : e];
        if (es & 1) continue;
        const float4 g = geo[e];
        const TabRegs<G> tr = tab_fetch<G>(cyt + (int64_t)e * CY_LD, lane);
        float xj[NX], mj[NU], rho[NPATH], rhop[NPATH];
        const int64_t jo = (int64_t)j * C + t.c;
        gather_row<PACK>(h, gh, NC, jo, xj);
        gather_row<PACK>(mu_a, gmu, NC, jo, mj);
        const TF* rrow = Rho + (int64_t)es * NPP * C;
        load_rho(rrow, t.c, rho);
        load_rho(rrow + NPP * C, t.c, rhop);
        tab_publish<G>(tr, slot, lane);
        float3 fe = force_term(slot, xj, mj, rho, rhop, g);
        fe.x = wave_sum_to_lane63(fe.x);  // over the wave's 64 channels
        fe.y = wave_sum_to_lane63(fe.y);
        fe.z = wave_sum_to_lane63(fe.z);
        if (lane == 63) {
          float* q = Fp + ((int64_t)(es >> 1) * (C >> 6) + (t.c >> 6)) * 3;
          q[0] = fe.x; q[1] = fe.y; q[2] = fe.z;
        }
      }
    }
  }
  if constexpr (!UNI) {
    red[threadIdx.x] = f;
    __syncthreads();
    if (t.active && t.c == 0) {
      float3 s = make_float3(0.f, 0.f, 0.f);
      for (int k = 0; k < C; ++k) {
        float3 x = red[threadIdx.x + k];
        s.x += x.x; s.y += x.y; s.z += x.z;
      }
      Facc[3 * t.row] += s.x;
      Facc[3 * t.row + 1] += s.y;
      Facc[3 * t.row + 2] += s.z;
    }
  }
}

// Forces of the rows from the per-pair terms of all layers: Fp [L][Eu][NW][3] (layer, pair, channel block).  An atom takes
// the term of every edge it receives with + if that edge is its pair's lower-numbered one (the one that evaluated it) and
// with - otherwise.  One wave per atom, lanes over its edges; sums in a fixed order.
__global__ void __launch_bounds__(256) k_force_rows(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                    const float* __restrict__ Fp, int L, int64_t Eu, int NW, int N,
                                                    float* __restrict__ F) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= N) return;  // whole waves leave; no workgroup barrier below
  float3 f = make_float3(0.f, 0.f, 0.f);
  for (int e = row_ptr[row] + lane; e < row_ptr[row + 1]; e += 64) {
    const int es = se[e].y;
    float3 g = make_float3(0.f, 0.f, 0.f);
    for (int l = 0; l < L; ++l)
      for (int w = 0; w < NW; ++w) {
        const float* q = Fp + (((int64_t)l * Eu + (es >> 1)) * NW + w) * 3;
        g.x += q[0]; g.y += q[1]; g.z += q[2];
      }
    const float sg = (es & 1) ? -1.f : 1.f;
    f.x += sg * g.x; f.y += sg * g.y; f.z += sg * g.z;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    f.x += __shfl_xor(f.x, o, 64);
    f.y += __shfl_xor(f.y, o, 64);
    f.z += __shfl_xor(f.z, o, 64);
  }
  if (lane == 0) { F[3 * row] = f.x; F[3 * row + 1] = f.y; F[3 * row + 2] = f.z; }
}

template <typename G, typename TX, typename TF, bool UNI, int LS>
__global__ void __launch_bounds__(256, 2) k_tp_bf(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                  const float2* __restrict__ env,
                                                  const TF* __restrict__ Rho, const float* __restrict__ cyt,
                                                  const float* __restrict__ cydt, const float* __restrict__ h,
                                                  const float* __restrict__ hd, const float* __restrict__ mu_a,
                                                  const __bf16* __restrict__ gh, const __bf16* __restrict__ ghd, int N, int C,
                                                  float* __restrict__ ad,
                                                  TX* __restrict__ X) {
  constexpr bool PACK = packed_rows<TF, G>();  // sender rows from the packed bf16 copies
  constexpr bool L0 = LS == LS_FIRST, LZ = LS == LS_LAST;
  constexpr int NM = G::NM, NPATH = LS ? G::LMAX + 1 : G::NPATH, NPP = LS ? 4 : G::NPP, CY_LD = G::CY_LD, NNZ = G::NNZ;
  constexpr int NU = LZ ? 1 : NM;  // live components of the messages' cotangent, and components of the output that anything reads
  RowChan t = row_chan(N, C);
  if (!t.active) return;
  const int64_t NC = (int64_t)N * C;
  const int64_t io = (int64_t)t.row * C + t.c;
  float mi[NU];
  loadm(mu_a, NC, io, mi);
  float acc[NU];
  zero(acc);
  __shared__ float tabs[4][2][64 * G::TAB_LOADS];
  float* slot = tabs[threadIdx.x >> 6][0];
  float* slotd = tabs[threadIdx.x >> 6][1];
  const int lane = threadIdx.x & 63;
  const int e0 = uni<UNI>(row_ptr[t.row]), e1 = uni<UNI>(row_ptr[t.row + 1]);
  int2 sn = e0 < e1 ? se[e0] : make_int2(0, 0);
  for (int e = e0; e < e1; ++e) {
    const int j = sn.x, es = sn.y;
    sn = se[e + 1 < e1 ? e + 1 : e];
    const float* cy = cyt + (int64_t)e * CY_LD;
    const float* cyd = cydt + (int64_t)e * CY_LD;
    TabRegs<G> tr, trd;
    if constexpr (UNI) { tr = tab_fetch<G>(cy, lane); trd = tab_fetch<G>(cyd, lane); }
    constexpr int NX = L0 ? 1 : NM;  // live components of the layer's input features (their tangent vanishes in the first layer)
    float xj[NX], xdj[NX], rho[NPATH], rr[NPATH];
    const int64_t jo = (int64_t)j * C + t.c;
    gather_row<PACK>(h, gh, NC, jo, xj);
    if constexpr (!L0) gather_row<PACK>(hd, ghd, NC, jo, xdj);
    const TF* rrow = Rho + (int64_t)(es & ~1) * NPP * C;
    load_rho(rrow, t.c, rho);
    load_rho(rrow + NPP * C, t.c, rr);
    if constexpr (UNI) { tab_publish<G>(tr, slot, lane); tab_publish<G>(trd, slotd, lane); cy = slot; cyd = slotd; }
    const float rd = cyd[NNZ];  // u . (v_sender - v_receiver), stored behind the table
#pragma unroll
    for (int p = 0; p < NPATH; ++p) rr[p] *= rd;
    // d/dt of the message: (rdot rho') T x Y + rho T xdot Y + rho T x Ydot; per slot S1 = sum cy x, S23 = sum cy xdot + cyd x
    float tp[NPATH];
    zero(tp);
    float S1 = 0.f, S23 = 0.f;
    static_for<0, G::NNZ>([&](auto n_) {
      constexpr int n = decltype(n_)::value;
      constexpr int sl = G::ENT_SLOT[n], p = G::SLOT_P[sl], m3 = G::SLOT_M3[sl], m1 = G::ENT_M1[n];
      if constexpr (L0) {
        if constexpr (m1 == 0) {  // the slot's only live entry
          const float s1 = cy[n] * xj[0];
          acc[m3] = fmaf(rr[p], s1, acc[m3]);
          if constexpr (G::ENT_M2[n] != 0) acc[m3] = fmaf(rho[p] * cyd[n], xj[0], acc[m3]);
          tp[p] = fmaf(mi[m3], s1, tp[p]);
        }
      } else if constexpr (!LZ || m3 == 0) {
        constexpr int pr = path_row<G, LS>(p);
        S1 = G::ENT_SFIRST[n] ? cy[n] * xj[m1] : fmaf(cy[n], xj[m1], S1);
        S23 = G::ENT_SFIRST[n] ? cy[n] * xdj[m1] : fmaf(cy[n], xdj[m1], S23);
        if constexpr (G::ENT_M2[n] != 0) S23 = fmaf(cyd[n], xj[m1], S23);  // the constant harmonic has no rate of change: cyd[n] = 0
        if (G::ENT_SLAST[n]) {
          acc[m3] = fmaf(rr[pr], S1, fmaf(rho[pr], S23, acc[m3]));
          tp[pr] = fmaf(mi[m3], S1, tp[pr]);
        }
      }
    });
    const float s = rd * env[e].x;
#pragma unroll
    for (int p = 0; p < NPATH; ++p) tp[p] *= s;
    store_paths(X + (int64_t)es * NPP * C, t.c, tp);
  }
#pragma unroll
  for (int m = 0; m < NU; ++m) ad[m * NC + io] = acc[m];
}

// BE gathers only the sender's cotangents lam_a[j], mu_a[j] (its own lam_h needs them).  The adjoint of the filter jet
// that it writes is that of the OPPOSITE edge (i -> j), the pair's other row of X: its path-wise forms need the features
// of that edge's sender -- this row's own x_i, xdot_i, loaded once per row -- and the cotangents of its receiver j, which
// are the two gathered tables; r, rdot, the envelope and the filter jet are equal on opposite edges, and the couplings of
// -u are those of u times the path's parity sign.  Every edge is some edge's opposite, so each row of X is still written
// exactly once, and half the gathers are gone.  (Before the filter jets were kept per edge pair this form was slower: the
// rows of X were then written in sequence by the direct form and scattered by this one.  Holding an edge's row of X back
// for one trip of the loop, so that its stores follow the next edge's loads, changed nothing.)
template <typename G, typename TX, typename TF, bool UNI, int LS>
__global__ void __launch_bounds__(256, 2) k_tp_be(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                  const float2* __restrict__ env,
                                                  const TF* __restrict__ Rho, const float* __restrict__ cyt,
                                                  const float* __restrict__ cydt, const float* __restrict__ h,
                                                  const float* __restrict__ hd, const float* __restrict__ mu_a,
                                                  const float* __restrict__ lam_a, const __bf16* __restrict__ gmu,
                                                  const __bf16* __restrict__ glam, const float* __restrict__ lam_h_next, int N, int C,
                                                  float* __restrict__ lam_h, TX* __restrict__ X) {
  constexpr bool PACK = packed_rows<TF, G>();  // sender rows from the packed bf16 copies
  constexpr bool L0 = LS == LS_FIRST, LZ = LS == LS_LAST;
  constexpr int NM = G::NM, NPATH = LS ? G::LMAX + 1 : G::NPATH, NPP = LS ? 4 : G::NPP, CY_LD = G::CY_LD, NNZ = G::NNZ;
  RowChan t = row_chan(N, C);
  if (!t.active) return;
  const int64_t NC = (int64_t)N * C;
  const int64_t io = (int64_t)t.row * C + t.c;
  constexpr int NX = L0 ? 1 : NM;  // live components of the layer's input features, and needed ones of their adjoint
  constexpr int NU = LZ ? 1 : NM;  // live components of the cotangents of the layer's messages
  float xi[NX], xdi[NX], acc[NX];
  loadm(h, NC, io, xi);
  if constexpr (!L0) loadm(hd, NC, io, xdi);  // the first layer's input has no tangent
  if constexpr (LZ) {  // the readout's adjoint has its l = 0 component only
    zero(acc);
    acc[0] = lam_h_next[io];
  } else {
    loadm(lam_h_next, NC, io, acc);
  }
  __shared__ float tabs[4][2][64 * G::TAB_LOADS];
  float* slot = tabs[threadIdx.x >> 6][0];
  float* slotd = tabs[threadIdx.x >> 6][1];
  const int lane = threadIdx.x & 63;
  const int e0 = uni<UNI>(row_ptr[t.row]), e1 = uni<UNI>(row_ptr[t.row + 1]);
  int2 sn = e0 < e1 ? se[e0] : make_int2(0, 0);
  for (int e = e0; e < e1; ++e) {
    const int j = sn.x, es = sn.y;
    sn = se[e + 1 < e1 ? e + 1 : e];
    const float* cy = cyt + (int64_t)e * CY_LD;
    const float* cyd = cydt + (int64_t)e * CY_LD;
    TabRegs<G> tr, trd;
    if constexpr (UNI) { tr = tab_fetch<G>(cy, lane); trd = tab_fetch<G>(cyd, lane); }
    float lj[NU], mj[NU], rho[NPATH], rr[NPATH];
    const int64_t jo = (int64_t)j * C + t.c;
    gather_row<PACK>(lam_a, glam, NC, jo, lj);
    gather_row<PACK>(mu_a, gmu, NC, jo, mj);
    const TF* rrow = Rho + (int64_t)(es & ~1) * NPP * C;
    load_rho(rrow, t.c, rho);
    load_rho(rrow + NPP * C, t.c, rr);
    if constexpr (UNI) { tab_publish<G>(tr, slot, lane); tab_publish<G>(trd, slotd, lane); cy = slot; cyd = slotd; }
    const float rd = cyd[NNZ];  // u . (v_sender - v_receiver), stored behind the table
#pragma unroll
    for (int p = 0; p < NPATH; ++p) rr[p] *= rd;
    // Per slot: R1, R2 = what the reversed edge (couplings of -u) hands back to this atom's features through cy and cyd;
    // S1 = sum cy x_i, S23 = sum cy xdot_i + cyd x_i feed the adjoint of the opposite edge's filter jet (up to the path's sign):
    // value row  c (t(x,Y,lam) + t(xdot,Y,mu) + t(x,Ydot,mu)) + c' rdot t(x,Y,mu)
    float ta[NPATH], t4[NPATH];
    zero(ta);
    zero(t4);
    float R1 = 0.f, R2 = 0.f, S1 = 0.f, S23 = 0.f;
    static_for<0, G::NNZ>([&](auto n_) {
      constexpr int n = decltype(n_)::value;
      constexpr int sl = G::ENT_SLOT[n], p = G::SLOT_P[sl], m3 = G::SLOT_M3[sl], m1 = G::ENT_M1[n];
      if constexpr (L0) {
        if constexpr (m1 == 0) {  // the slot's only live entry
          const float r2 = G::PATH_SIGN[p] * rho[p] * mj[m3];
          const float r1 = G::PATH_SIGN[p] * fmaf(rho[p], lj[m3], rr[p] * mj[m3]);
          acc[0] = fmaf(cy[n], r1, acc[0]);
          const float s1 = cy[n] * xi[0];
          ta[p] = fmaf(lj[m3], s1, ta[p]);
          if constexpr (G::ENT_M2[n] != 0) {
            acc[0] = fmaf(cyd[n], r2, acc[0]);
            ta[p] = fmaf(mj[m3] * cyd[n], xi[0], ta[p]);
          }
          t4[p] = fmaf(mj[m3], s1, t4[p]);
        }
      } else if constexpr (!LZ || m3 == 0) {
        constexpr int pr = path_row<G, LS>(p);
        if (G::ENT_SFIRST[n]) {
          R2 = G::PATH_SIGN[p] * rho[pr] * mj[m3];
          R1 = G::PATH_SIGN[p] * fmaf(rho[pr], lj[m3], rr[pr] * mj[m3]);
        }
        acc[m1] = fmaf(cy[n], R1, acc[m1]);
        if constexpr (G::ENT_M2[n] != 0) acc[m1] = fmaf(cyd[n], R2, acc[m1]);
        S1 = G::ENT_SFIRST[n] ? cy[n] * xi[m1] : fmaf(cy[n], xi[m1], S1);
        S23 = G::ENT_SFIRST[n] ? cy[n] * xdi[m1] : fmaf(cy[n], xdi[m1], S23);
        if constexpr (G::ENT_M2[n] != 0) S23 = fmaf(cyd[n], xi[m1], S23);  // the constant harmonic has no rate of change: cyd[n] = 0
        if (G::ENT_SLAST[n]) {
          ta[pr] = fmaf(lj[m3], S1, fmaf(mj[m3], S23, ta[pr]));
          t4[pr] = fmaf(mj[m3], S1, t4[pr]);
        }
      }
    });
    const float2 cc = env[e];
    const float s = cc.y * rd;
    static_for<0, NPATH>([&](auto k_) {  // the opposite edge sees the harmonics of -u: the path's parity sign
      constexpr int k = decltype(k_)::value;
      constexpr float sg = G::PATH_SIGN[LZ ? G::LAST_PATHS[k] : k];
      ta[k] = sg * fmaf(cc.x, ta[k], s * t4[k]);
    });
    store_paths(X + (int64_t)(es ^ 1) * NPP * C, t.c, ta);
  }
#pragma unroll
  for (int m = 0; m < NX; ++m) lam_h[m * NC + io] = acc[m];  // first layer: only the l = 0 component is needed (the embedding's gradient)
}


// ------------------------------------------------------------------------------ position gradient (optional)
// d/dr_vec of F(r_vec) = sum_m nu[m] Y_m(r_vec / |r_vec|), differentiated once more along d:
// with u = r_vec / r, Q(u) = sum_m nu[m] P_m(u) the harmonics' polynomials (the forms sph_grad_T differentiates),
// g = grad Q(u), H = Hessian of Q at u (constant for l <= 2, linear in u for the degree-3 terms), Pi = I - u u^T,
// delta = Pi d / r:
//   grad F = Pi g / r,    D_d grad F = [H delta - delta (u.g) - u (delta.g + u.H delta)] / r - Pi g (u.d) / r^2.
template <int NM>
__device__ __forceinline__ float3 sph_hess_apply(float x, float y, float z, float r, const float (&nu)[NM], float3 d) {
  const float3 g = sph_grad_T(x, y, z, nu);
  const float inv = r > 0.f ? 1.f / r : 0.f;
  const float ud = x * d.x + y * d.y + z * d.z;
  const float3 dl = make_float3((d.x - x * ud) * inv, (d.y - y * ud) * inv, (d.z - z * ud) * inv);
  // H: xx = s15 nu8, yy = -s15 nu8, zz = 3 s5 nu6, xy = s15 nu4, yz = s15 nu5, xz = s15 nu7
  float hxx = S15 * nu[8], hyy = -S15 * nu[8], hzz = 3.f * S5 * nu[6], hxy = S15 * nu[4], hyz = S15 * nu[5], hxz = S15 * nu[7];
  if constexpr (NM == 16) {
    // second derivatives of  c35 y(3x^2 - y^2), c105 xyz, c21 y(5z^2 - 1), c7 z(5z^2 - 3), c21 x(5z^2 - 1), (c105/2) z(x^2 - y^2), c35 x(x^2 - 3y^2)
    hxx += 6.f * C35 * (y * nu[9] + x * nu[15]) + C105 * z * nu[14];
    hyy += -6.f * C35 * (y * nu[9] + x * nu[15]) - C105 * z * nu[14];
    hzz += 10.f * C21 * (y * nu[11] + x * nu[13]) + 30.f * C7 * z * nu[12];
    hxy += 6.f * C35 * (x * nu[9] - y * nu[15]) + C105 * z * nu[10];
    hyz += C105 * (x * nu[10] - y * nu[14]) + 10.f * C21 * z * nu[11];
    hxz += C105 * (y * nu[10] + x * nu[14]) + 10.f * C21 * z * nu[13];
  }
  const float3 hd = make_float3(hxx * dl.x + hxy * dl.y + hxz * dl.z, hxy * dl.x + hyy * dl.y + hyz * dl.z, hxz * dl.x + hyz * dl.y + hzz * dl.z);
  const float ug = x * g.x + y * g.y + z * g.z;
  const float dg = dl.x * g.x + dl.y * g.y + dl.z * g.z;
  const float uh = x * hd.x + y * hd.y + z * hd.z;
  const float k = ud * inv * inv;
  float3 o;
  o.x = (hd.x - dl.x * ug - x * (dg + uh)) * inv - (g.x - x * ug) * k;
  o.y = (hd.y - dl.y * ug - y * (dg + uh)) * inv - (g.y - y * ug) * k;
  o.z = (hd.z - dl.z * ug - z * (dg + uh)) * inv - (g.z - z * ug) * k;
  return o;
}

// One layer's share of dPsi/dx, Psi = sum_s Ebar_s E_s + D_v E.  An edge's geometry enters through rho(r) = f_c R(r),
// rhodot = rdot rho'(r) with rdot = u.(v_j - v_i), Y(u) and Ydot = (dY/dr_vec)(v_j - v_i):
//   dPsi/dr_vec = [lam_rho.rho' + rdot lam_rhodot.rho''] u + (lam_rhodot.rho') (dv - u rdot)/r + J^T lam_Y + K^T lam_Ydot,
//   lam_rho = t(h_j, Y; lam_a,i) + t(hdot_j, Y; mu_a,i) + t(h_j, Ydot; mu_a,i),   lam_rhodot = t(h_j, Y; mu_a,i),
//   lam_Y = B_y^T(rho, h_j; lam_a,i) + B_y^T(rdot rho', h_j; mu_a,i) + B_y^T(rho, hdot_j; mu_a,i),  lam_Ydot = B_y^T(rho, h_j; mu_a,i),
//   J = dY/dr_vec, K = d(Ydot)/dr_vec (second derivatives of the harmonics, sph_hess_apply).
// Atom i takes -dPsi/dr_vec of the edges it receives and +dPsi/dr_vec of those it sends; the opposite edge (same r, rdot;
// u, dv negated; Y -> PY) is formed here too, from the row's own node values and the gathered sender's.
// One thread per (receiver row, channel), couplings straight from the entry tables; off the timed path.
template <typename G>
__global__ void __launch_bounds__(256) k_tp_gp(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                               const float4* __restrict__ geo, const float2* __restrict__ env,
                                               const float* __restrict__ Rj, const float* __restrict__ Rpp,
                                               const float* __restrict__ h, const float* __restrict__ hd,
                                               const float* __restrict__ mu_a, const float* __restrict__ lam_a,
                                               const float* __restrict__ v, float k2, int N, int C, float* __restrict__ gp) {
  constexpr int NM = G::NM, NPATH = G::NPATH, NPP = G::NPP;
  __shared__ float3 red[256];
  RowChan t = row_chan(N, C);
  float3 f = make_float3(0.f, 0.f, 0.f);
  if (t.active) {
    const int64_t NC = (int64_t)N * C;
    const int64_t io = (int64_t)t.row * C + t.c;
    float xi[NM], xdi[NM], li[NM], mi[NM];
    loadm(h, NC, io, xi);
    loadm(hd, NC, io, xdi);
    loadm(lam_a, NC, io, li);
    loadm(mu_a, NC, io, mi);
    const float vi0 = v[3 * t.row], vi1 = v[3 * t.row + 1], vi2 = v[3 * t.row + 2];
    for (int e = row_ptr[t.row]; e < row_ptr[t.row + 1]; ++e) {
      const int j = se[e].x, es = se[e].y;
      const float4 g = geo[e];
      const float2 cc = env[e];
      const float3 d = make_float3(v[3 * j] - vi0, v[3 * j + 1] - vi1, v[3 * j + 2] - vi2);
      const float rd = g.x * d.x + g.y * d.y + g.z * d.z;
      float xj[NM], xdj[NM], lj[NM], mj[NM], R[NPATH], Rp[NPATH], Rq[NPATH];
      const int64_t jo = (int64_t)j * C + t.c;
      loadm(h, NC, jo, xj);
      loadm(hd, NC, jo, xdj);
      loadm(lam_a, NC, jo, lj);
      loadm(mu_a, NC, jo, mj);
      load_rho(Rj + (int64_t)(es & ~1) * NPP * C, t.c, R);
      load_rho(Rj + (int64_t)(es | 1) * NPP * C, t.c, Rp);
      load_rho(Rpp + (int64_t)(es >> 1) * NPP * C, t.c, Rq);
      const float c = cc.x, cp = cc.y, cq = -k2 * (c - 0.5f);
      float rho[NPATH], rr[NPATH], r1[NPATH], r2[NPATH];  // rho, rdot rho', rho', rho''
#pragma unroll
      for (int p = 0; p < NPATH; ++p) {
        rho[p] = c * R[p];
        r1[p] = cp * R[p] + c * Rp[p];
        r2[p] = cq * R[p] + 2.f * cp * Rp[p] + c * Rq[p];
        rr[p] = rd * r1[p];
      }
      float Y[NM], Yd[NM], PY[NM], PYd[NM];
      sph_harm(g.x, g.y, g.z, Y);
      sph_dot(g.x, g.y, g.z, g.w, d, Yd);
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        PY[m] = G::M_SIGN[m] * Y[m];
        PYd[m] = G::M_SIGN[m] * Yd[m];
      }
      // One walk over the coupling entries n = (p; m1, m2, m3) forms the path-wise trilinear forms t_p and the adjoints of the
      // harmonics B_y^T of this edge and of the opposite edge (own features, the sender's adjoints, harmonics of -u):
      //   lr = lam_rho, lrd = lam_rhodot (both edges summed);  LY, LYd = lam_Y, lam_Ydot of this edge, QY, QYd of the opposite one
      float lr[NPATH], lrd[NPATH], LY[NM], LYd[NM], QY[NM], QYd[NM];
      zero(lr); zero(lrd); zero(LY); zero(LYd); zero(QY); zero(QYd);
      static_for<0, G::NNZ>([&](auto n_) {
        constexpr int n = decltype(n_)::value;
        constexpr int sl = G::ENT_SLOT[n], p = G::SLOT_P[sl], m3 = G::SLOT_M3[sl], m1 = G::ENT_M1[n], m2 = G::ENT_M2[n];
        const float co = G::ENT_COEF[n];
        const float a_l = xj[m1] * li[m3] + xdj[m1] * mi[m3], a_m = xj[m1] * mi[m3];  // this edge
        const float b_l = xi[m1] * lj[m3] + xdi[m1] * mj[m3], b_m = xi[m1] * mj[m3];  // the opposite edge
        lr[p] += co * (a_l * Y[m2] + a_m * Yd[m2] + b_l * PY[m2] + b_m * PYd[m2]);
        lrd[p] += co * (a_m * Y[m2] + b_m * PY[m2]);
        const float q = rho[p] * co, qr = rr[p] * co;
        LY[m2] += q * a_l + qr * a_m;
        LYd[m2] += q * a_m;
        QY[m2] += q * b_l + qr * b_m;
        QYd[m2] += q * b_m;
      });
      float rad = 0.f, gg = 0.f;
#pragma unroll
      for (int p = 0; p < NPATH; ++p) {
        rad += lr[p] * r1[p] + lrd[p] * rd * r2[p];
        gg += lrd[p] * r1[p];
      }
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        LY[m] += G::M_SIGN[m] * QY[m];
        LYd[m] += G::M_SIGN[m] * QYd[m];
      }
      const float inv = g.w > 0.f ? 1.f / g.w : 0.f;
      const float3 w = sph_grad_T(g.x, g.y, g.z, LY);
      const float uw = g.x * w.x + g.y * w.y + g.z * w.z;
      const float3 hs = sph_hess_apply(g.x, g.y, g.z, g.w, LYd, d);
      f.x -= rad * g.x + gg * (d.x - g.x * rd) * inv + (w.x - g.x * uw) * inv + hs.x;
      f.y -= rad * g.y + gg * (d.y - g.y * rd) * inv + (w.y - g.y * uw) * inv + hs.y;
      f.z -= rad * g.z + gg * (d.z - g.z * rd) * inv + (w.z - g.z * uw) * inv + hs.z;
    }
  }
  red[threadIdx.x] = f;
  __syncthreads();
  if (t.active && t.c == 0) {
    float3 s = make_float3(0.f, 0.f, 0.f);
    for (int k = 0; k < C; ++k) {
      float3 x = red[threadIdx.x + k];
      s.x += x.x; s.y += x.y; s.z += x.z;
    }
    gp[3 * t.row] += s.x;
    gp[3 * t.row + 1] += s.y;
    gp[3 * t.row + 2] += s.z;
  }
}

// Per-edge tables of coupling coefficient x harmonic: cy[e][n] = T_n Y_{m2_n}(u_e), and, with
// WITH_DOT, cyd[e][n] = T_n Ydot_{m2_n} for the displacement rate v_sender - v_receiver,
// followed (entry NNZ) by the rate of change of the edge length, u . (v_sender - v_receiver).
// A workgroup takes 64 edges: 64 of its threads evaluate the harmonics (or their rates of change) of one edge each into
// LDS, then all threads write the edges' tables in order (coalesced), one multiplication per entry.
template <typename G, bool WITH_DOT>
__global__ void __launch_bounds__(256) k_edge_cy(const float4* __restrict__ geo, const int32_t* __restrict__ sender,
                                                 const int32_t* __restrict__ receiver, const float* __restrict__ v, int64_t E,
                                                 float* __restrict__ out) {
  constexpr int NM = G::NM, NNZ = G::NNZ, CY_LD = G::CY_LD, EB = 64;
  __shared__ float ys[EB][NM + 2];  // harmonics of an edge, then the rate of change of its length; odd pitch
  const int64_t eb = (int64_t)blockIdx.x * EB;
  if (threadIdx.x < EB && eb + threadIdx.x < E) {
    const int64_t e = eb + threadIdx.x;
    const float4 g = geo[e];
    float Y[NM];
    float rd = 0.f;
    if (WITH_DOT) {
      const int j = sender[e], i = receiver[e];
      const float3 dv = make_float3(v[3 * j] - v[3 * i], v[3 * j + 1] - v[3 * i + 1], v[3 * j + 2] - v[3 * i + 2]);
      sph_dot(g.x, g.y, g.z, g.w, dv, Y);
      rd = g.x * dv.x + g.y * dv.y + g.z * dv.z;
    } else {
      sph_harm(g.x, g.y, g.z, Y);
    }
#pragma unroll
    for (int m = 0; m < NM; ++m) ys[threadIdx.x][m] = Y[m];
    ys[threadIdx.x][NM] = rd;
  }
  __syncthreads();
  const int64_t n_out = (E - eb < EB ? E - eb : EB) * CY_LD;
  for (int k = threadIdx.x; k < n_out; k += 256) {
    const int el = k / CY_LD, n = k % CY_LD;
    float val = 0.f;
    if (n < NNZ) val = gaunt::ent_coef_dev<G::LMAX>(n) * ys[el][gaunt::ent_m2_dev<G::LMAX>(n)];
    else if (n == NNZ) val = ys[el][NM];
    out[eb * CY_LD + k] = val;
  }
}


// The paths a layer stores filter rows for: all NPATH in order (x < 0), or up to four listed ones (a specialised layer).
struct PathList {
  int n, x, y, z, w;  // n stored paths; which path each of the first four is, unless x < 0
  __host__ __device__ int path(int k) const { return x < 0 ? k : (k == 0 ? x : k == 1 ? y : k == 2 ? z : w); }
};
template <typename G>
PathList path_list(int ls) {
  if (ls == LS_FIRST) return PathList{G::LMAX + 1, 0, 1, 2, 3};  // (0, l, l): the first LMAX + 1 paths
  if (ls == LS_LAST) return PathList{G::LMAX + 1, G::LAST_PATHS[0], G::LAST_PATHS[1], G::LAST_PATHS[2], G::LAST_PATHS[G::LMAX]};
  return PathList{G::NPATH, -1, 0, 0, 0};
}
// Filter weights W [NPATH C][H] (row p C + c) regrouped to the stored order of the filter jets:
// Wp [(c NPP + k)][H] for the k-th stored path, zero rows for the pad, and the transpose WpT [H][NPP C].
__global__ void k_regroup_filter(const float* __restrict__ W, int C, int H, PathList pl, int NPP, float* __restrict__ Wp, float* __restrict__ WpT) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)NPP * C * H) return;
  const int r = (int)(idx / H), hh = (int)(idx % H), c = r / NPP, k = r % NPP;
  const float val = k < pl.n ? W[((int64_t)pl.path(k) * C + c) * H + hh] : 0.f;
  Wp[idx] = val;
  WpT[(int64_t)hh * NPP * C + r] = val;
}
// grad[(p C + c)][H] += g[(c NPP + k)][H] for the k-th stored path p
__global__ void k_regroup_add(const float* __restrict__ g, int C, int H, PathList pl, int NPP, float* __restrict__ grad) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)NPP * C * H) return;
  const int r = (int)(idx / H), hh = (int)(idx % H), c = r / NPP, k = r % NPP;
  if (k < pl.n) grad[((int64_t)pl.path(k) * C + c) * H + hh] += g[idx];
}
// Which specialisation layer l of L runs as.  The position gradient's kernel reads every component of the last layer's
// cotangents, so that layer stays general when the gradient is wanted.
inline int layer_spec(int l, int L, bool position_grad) {
  if (l == 0) return LS_FIRST;
  return (l == L - 1 && !position_grad) ? LS_LAST : LS_ANY;
}
// the tensor-product kernel instance for a layer: KERN(k_tp_fe, ls, uni, G, TF) -> k_tp_fe<G, TF, uni, ls>
#define TP_KERNEL(name, ls, uni, ...)                                                                                         \
  ((ls) == LS_FIRST ? ((uni) ? name<__VA_ARGS__, true, LS_FIRST> : name<__VA_ARGS__, false, LS_FIRST>)                          \
   : (ls) == LS_LAST ? ((uni) ? name<__VA_ARGS__, true, LS_LAST> : name<__VA_ARGS__, false, LS_LAST>)                           \
                     : ((uni) ? name<__VA_ARGS__, true, LS_ANY> : name<__VA_ARGS__, false, LS_ANY>))

// h0[m=0] = emb[species], other components zero
__global__ void k_embed_l0(const float* __restrict__ emb, const int32_t* __restrict__ species, int64_t N, int C, int NM,
                           float* __restrict__ h) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NM * N * C) return;
  int64_t m = idx / (N * C), r = idx % (N * C);
  h[idx] = (m == 0) ? emb[(int64_t)species[r / C] * C + (r % C)] : 0.f;
}

// The mixing matrix of degree k in layer l acting on the [(2k+1) N, C] block at offset o: dense, or
// merged per structure from an expert bank (then every product is structure-wise).
template <typename P, typename LdA, typename Epi>
void mix_mm(mlip_ctx* ctx, int l, int k, bool transposed, const LdA& a, const Epi& epi) {
  EqvWs* w = ws_of(ctx);
  const int C = ctx->cfg.channels;
  const int64_t rows = (2 * k + 1) * ctx->N;
  if (ctx->cfg.n_experts > 0)
    gemm_nt_grouped<P>(ctx, a, (transposed ? w->WmT : w->Wm)[k][l], rows, C, C, epi, 2 * k + 1);
  else
    gemm_nt<P>(ctx, a, (transposed ? w->paramsT : ctx->d_params) + ctx->lay[l].Wl[k], rows, C, C, epi);
}
template <typename P, typename LdA, typename LdB>
int mix_wgrad(mlip_ctx* ctx, int l, int k, const LdA& a, const LdB& b, float* grad) {
  const int C = ctx->cfg.channels;
  const int64_t rows = (2 * k + 1) * ctx->N;
  float* g = grad + ctx->lay[l].Wl[k];
  if (ctx->cfg.n_experts > 0) return gemm_wgrad_experts<P>(ctx, a, b, rows, C, C, g, ctx->d_params + ctx->lay[l].Wl[k], 2 * k + 1);
  return gemm_wgrad<P>(ctx, a, b, rows, C, C, g);
}

// ------------------------------------------------------------------------------ gated node update
// cfg.gate: with u = W a (per l) the update is z_0 = silu(u_0), z_m = sigmoid(u_0) u_m for the NM - 1
// l >= 1 components m of the same channel, h' = h + z.  One thread per (atom, channel); arrays are
// [NM][N][C], component-major.  The four kernels are the map itself, its transpose applied to a
// cotangent (FF), its tangent map (BF), and for BE the transpose applied to lambda plus the derivative
// with respect to u of <ud, J(u)^T mu> (ud: BF's tangent of u, mu: FF's cotangent of z).
struct GateFn {
  float s, ds, dds, f1, f2;  // sigmoid, its first and second derivative; silu', silu''
};
__device__ __forceinline__ GateFn gate_fn(float u0) {
  GateFn g;
  g.s = sigm(u0);
  g.ds = g.s * (1.f - g.s);
  g.dds = g.ds * (1.f - 2.f * g.s);
  g.f1 = g.s + u0 * g.ds;
  g.f2 = 2.f * g.ds + u0 * g.dds;
  return g;
}

__global__ void k_gate_fe(const float* __restrict__ u, const float* __restrict__ h_in, float* __restrict__ h_out, int64_t NC, int NM) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NC) return;
  const float u0 = u[idx];
  const float s = sigm(u0);
  h_out[idx] = h_in[idx] + u0 * s;
  for (int m = 1; m < NM; ++m) h_out[m * NC + idx] = h_in[m * NC + idx] + s * u[m * NC + idx];
}

__global__ void k_gate_ff(const float* __restrict__ u, const float* __restrict__ mu, float* __restrict__ mu_u, int64_t NC, int NM) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NC) return;
  const GateFn g = gate_fn(u[idx]);
  float dot = 0.f;
  for (int m = 1; m < NM; ++m) {
    const float mm = mu[m * NC + idx];
    dot += u[m * NC + idx] * mm;
    mu_u[m * NC + idx] = g.s * mm;
  }
  mu_u[idx] = g.f1 * mu[idx] + g.ds * dot;
}

__global__ void k_gate_bf(const float* __restrict__ u, const float* __restrict__ ud, const float* __restrict__ hd_in,
                          float* __restrict__ hd_out, int64_t NC, int NM) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NC) return;
  const GateFn g = gate_fn(u[idx]);
  const float ud0 = ud[idx];
  hd_out[idx] = hd_in[idx] + g.f1 * ud0;
  for (int m = 1; m < NM; ++m)
    hd_out[m * NC + idx] = hd_in[m * NC + idx] + (g.ds * ud0 * u[m * NC + idx] + g.s * ud[m * NC + idx]);
}

__global__ void k_gate_be(const float* __restrict__ u, const float* __restrict__ ud, const float* __restrict__ mu,
                          const float* __restrict__ lam, float* __restrict__ lam_u, int64_t NC, int NM) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NC) return;
  const GateFn g = gate_fn(u[idx]);
  const float ud0 = ud[idx];
  float u_lam = 0.f, u_mu = 0.f, ud_mu = 0.f;
  for (int m = 1; m < NM; ++m) {
    const float um = u[m * NC + idx], mm = mu[m * NC + idx], lm = lam[m * NC + idx];
    u_lam += um * lm;
    u_mu += um * mm;
    ud_mu += ud[m * NC + idx] * mm;
    lam_u[m * NC + idx] = g.s * lm + ud0 * g.ds * mm;
  }
  lam_u[idx] = g.f1 * lam[idx] + g.ds * u_lam + ud0 * (g.f2 * mu[idx] + g.dds * u_mu) + g.ds * ud_mu;
}

// packed bf16 copy of a node table for the sender gathers (only when the filter jets are bf16)
template <typename TF, typename G>
void pack_rows(mlip_ctx* ctx, const float* tab, __bf16* packed) {
  if constexpr (packed_rows<TF, G>()) {
    const int64_t NC = ctx->N * ctx->cfg.channels;
    hipLaunchKernelGGL(k_pack_rows<G::NM>, dim3(nblk(NC)), dim3(256), 0, ctx->stream, tab, NC, packed);
  }
}

// ------------------------------------------------------------------------------ phases
template <typename P, typename TF, typename G>
int fe_impl(mlip_ctx* ctx, float* E_out) {
  EqvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  static_assert(sizeof(typename Act<P>::xop_t) == (P::IS_BF16 ? 2 : 4), "the workspace is sized for 2-byte operand-precision tensors in bf16 mode and 4-byte ones otherwise");
  const int64_t N = ctx->N, E = ctx->E, Eu = ctx->Eu, NC = N * cf.channels;  // atoms, edges, edge pairs (rows of the edge MLP's products)
  constexpr int NM = G::NM, NPATH = G::NPATH, NPP = G::NPP, CY_LD = G::CY_LD, LMAX = G::LMAX;
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, PC = NPP * C;
  const float* th = ctx->d_params;
  const bool gate = cf.gate != 0;
  auto tr = [&](int64_t off, int rows, int cols) {
    hipLaunchKernelGGL(k_transpose, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(32, 8), 0, st, th + off, w->paramsT + off, rows, cols);
  };
  for (int l = 0; l < L; ++l) {
    // the first and the last layer multiply by their live paths only (rows of 4 per channel); the position gradient's
    // products need all paths everywhere
    const int ls = layer_spec(l, L, cf.position_grad);
    if (ls != LS_ANY)
      hipLaunchKernelGGL(k_regroup_filter, dim3(nblk((int64_t)4 * C * H)), dim3(256), 0, st, th + ctx->lay[l].W[1], C, H, path_list<G>(ls), 4,
                         ls == LS_FIRST ? w->Wp0 : w->WpZ, ls == LS_FIRST ? w->WpT0 : w->WpTZ);
    if (ls == LS_ANY || cf.position_grad)
      hipLaunchKernelGGL(k_regroup_filter, dim3(nblk((int64_t)PC * H)), dim3(256), 0, st, th + ctx->lay[l].W[1], C, H, path_list<G>(LS_ANY), NPP, w->Wp[l], w->WpT[l]);
    for (int k = 0; k <= LMAX; ++k) {
      if (cf.n_experts > 0)
        hipLaunchKernelGGL(k_merge_experts, dim3(nblk((int64_t)C * C, 64), (unsigned)((ctx->B + 15) / 16)), dim3(256), 0, st, ctx->d_alpha,
                           th + ctx->lay[l].Wl[k], ctx->B, cf.n_experts, C, w->Wm[k][l], w->WmT[k][l]);
      else
        tr(ctx->lay[l].Wl[k], C, C);
    }
  }
  tr(ctx->off_U, C, C);
  if (P::IS_BF16) refresh_shadows(ctx);  // bf16 mirrors of the weights, their transposes and the regrouped filters
  if (E > 0)
    launch_edge_features(ctx, E, K, cf.cutoff, w->env, w->env_u, w->jphi);
  if (E > 0)
    hipLaunchKernelGGL((k_edge_cy<G, false>), dim3(nblk(E, 64)), dim3(256), 0, st, ctx->d_geo, ctx->d_sender, ctx->d_receiver, nullptr, E, w->cy);
  hipLaunchKernelGGL(k_embed_l0, dim3(nblk(NM * NC)), dim3(256), 0, st, th + ctx->off_emb, ctx->d_species, N, C, NM, w->h[0]);
  const int rpb = 256 / C;
  const bool uni = C % 64 == 0;  // a wave then holds channels of one receiver row only
  for (int l = 0; l < L; ++l) {
    const LayerOffsets& lo = ctx->lay[l];
    const int ls = layer_spec(l, L, cf.position_grad);
    if (Eu > 0) {
      {
        KernelTimer kt(ctx, MLIP_K_FE_HIDDEN_GEMM);
        gemm_nt<P>(ctx, LdPlain{w->jphi, K}, th + lo.W[0], 2 * Eu, H, K, Act<P>::store(w->U[l], w->SJ[l], H, 2 * Eu));
      }
      KernelTimer kt(ctx, MLIP_K_FE_FILTER_GEMM);
      const int PCl = ls != LS_ANY ? 4 * C : PC;  // filter width of this layer
      gemm_nt<P>(ctx, Act<P>::jet(w->U[l], w->SJ[l], H), ls == LS_FIRST ? w->Wp0 : ls == LS_LAST ? w->WpZ : w->Wp[l], 2 * Eu, PCl, H,
                 EpiOmega<TF>{reinterpret_cast<TF*>(w->Rho[l]), w->env_u, PCl, 2 * Eu});
    }
    {
      KernelTimer kt(ctx, MLIP_K_MSG_FE);
      auto kern = TP_KERNEL(k_tp_fe, ls, uni, G, TF);
      hipLaunchKernelGGL(kern, dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, reinterpret_cast<const TF*>(w->Rho[l]),
                         w->cy, w->h[l], w->gh[l], (int)N, C, w->a[l]);
    }
    const int kmax = ls == LS_LAST ? 0 : LMAX;  // the readout takes the last layer's l = 0 output only
    for (int k = 0; k <= kmax; ++k) {
      const int64_t o = G::L_OFF[k] * NC, rows = (2 * k + 1) * N;
      if (gate)
        mix_mm<P>(ctx, l, k, false, LdPlain{w->a[l] + o, C}, EpiStore{w->u[l] + o, C, rows});
      else
        mix_mm<P>(ctx, l, k, false, LdPlain{w->a[l] + o, C}, EpiAddStore{w->h[l + 1] + o, w->h[l] + o, C, rows});
    }
    if (gate) hipLaunchKernelGGL(k_gate_fe, dim3(nblk(NC)), dim3(256), 0, st, w->u[l], w->h[l], w->h[l + 1], NC, ls == LS_LAST ? 1 : NM);
    if (l + 1 < L) pack_rows<TF, G>(ctx, w->h[l + 1], w->gh[l + 1]);  // the next layer gathers these rows in all four phases
  }
  gemm_nt<P>(ctx, LdPlain{w->h[L], C}, th + ctx->off_U, N, C, C, EpiStore{w->y, C, N});
  hipLaunchKernelGGL(k_atom_energy, dim3(nblk(N, 4)), dim3(256), 0, st, w->y, th + ctx->off_wo, (int)N, C, w->eps);
  hipLaunchKernelGGL(k_struct_sum, dim3(ctx->B), dim3(256), 0, st, w->eps, ctx->d_meta, E_out);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

template <typename P, typename TF, typename G>
int ff_impl(mlip_ctx* ctx, float* F) {
  EqvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  constexpr int NM = G::NM, LMAX = G::LMAX;
  const int64_t N = ctx->N, NC = N * cf.channels;
  const int C = cf.channels, L = cf.n_layers;
  const float* th = ctx->d_params;
  const bool gate = cf.gate != 0;
  const float* tT = w->paramsT;
  // mu_h^L: l = 0 block from the readout, zero elsewhere
  hipLaunchKernelGGL(k_fill, dim3(nblk((NM - 1) * NC)), dim3(256), 0, st, w->mu_h[L] + NC, 0.f, (NM - 1) * NC);
  gemm_nt<P>(ctx, LdMuY{w->y, th + ctx->off_wo, C}, tT + ctx->off_U, N, C, C, EpiStore{w->mu_h[L], C, N});
  hipLaunchKernelGGL(k_fill, dim3(nblk(3 * N)), dim3(256), 0, st, w->Facc, 0.f, 3 * N);
  const int rpb = 256 / C;
  const bool uni = C % 64 == 0;  // a wave then holds channels of one receiver row only
  for (int l = L - 1; l >= 0; --l) {
    const LayerOffsets& lo = ctx->lay[l];
    const int ls = layer_spec(l, L, cf.position_grad);
    const int kmax = ls == LS_LAST ? 0 : LMAX;  // the last layer's cotangents have their l = 0 component only
    const float* mu_z = w->mu_h[l + 1];  // cotangent of the update's output; through the gate it becomes that of W a
    if (gate) {
      hipLaunchKernelGGL(k_gate_ff, dim3(nblk(NC)), dim3(256), 0, st, w->u[l], w->mu_h[l + 1], w->mu_u[l], NC, ls == LS_LAST ? 1 : NM);
      mu_z = w->mu_u[l];
    }
    for (int k = 0; k <= kmax; ++k) {
      const int64_t o = G::L_OFF[k] * NC, rows = (2 * k + 1) * N;
      mix_mm<P>(ctx, l, k, true, LdPlain{mu_z + o, C}, EpiStore{w->mu_a[l] + o, C, rows});
    }
    if (ls != LS_LAST) pack_rows<TF, G>(ctx, w->mu_a[l], w->gmu[l]);  // gathered by this phase and by BE (one component in the last layer)
    KernelTimer kt(ctx, MLIP_K_MSG_FF);
    auto kern = TP_KERNEL(k_tp_ff, ls, uni, G, TF);
    hipLaunchKernelGGL(kern, dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, ctx->d_geo, reinterpret_cast<const TF*>(w->Rho[l]),
                       w->cy, w->h[l], w->mu_a[l], w->gh[l], w->gmu[l], w->mu_h[l + 1], (int)N, C, w->mu_h[l], w->Facc,
                       uni ? w->Fp + (int64_t)l * ctx->Eu * (C / 64) * 3 : nullptr);
  }
  if (uni)  // the per-pair force terms of all layers, with their signs, summed per atom
    hipLaunchKernelGGL(k_force_rows, dim3(nblk(N, 4)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, w->Fp, L, ctx->Eu, C / 64, (int)N, F);
  else
    hipLaunchKernelGGL(k_scale3, dim3(nblk(3 * N)), dim3(256), 0, st, w->Facc, 1.f, 3 * N, F);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

template <typename P, typename TF, typename G>
int bf_impl(mlip_ctx* ctx, float* grad) {
  EqvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  const int64_t N = ctx->N, E = ctx->E, Eu = ctx->Eu, NC = N * cf.channels;  // atoms, edges, edge pairs (rows of the edge MLP's products)
  constexpr int NM = G::NM, NPATH = G::NPATH, NPP = G::NPP, CY_LD = G::CY_LD, LMAX = G::LMAX;
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, PC = NPP * C;
  const float* th = ctx->d_params;
  const bool gate = cf.gate != 0;
  const float* tT = w->paramsT;
  typedef typename Act<P>::xop_t TX;  // X and X2 only feed matrix products: stored in the operand precision
  TX* X = reinterpret_cast<TX*>(w->X);
  TX* X2 = reinterpret_cast<TX*>(w->X2);
  hipLaunchKernelGGL(k_fill, dim3(nblk(NM * NC)), dim3(256), 0, st, w->hd[0], 0.f, NM * NC);
  if (E > 0)  // harmonics' rate of change under the displacement rate v: used by this phase and by BE
    hipLaunchKernelGGL((k_edge_cy<G, true>), dim3(nblk(E, 64)), dim3(256), 0, st, ctx->d_geo, ctx->d_sender, ctx->d_receiver, w->v, E, w->cyd);
  const int rpb = 256 / C;
  const bool uni = C % 64 == 0;  // a wave then holds channels of one receiver row only
  for (int l = 0; l < L; ++l) {
    const LayerOffsets& lo = ctx->lay[l];
    const int ls = layer_spec(l, L, cf.position_grad);
    const int PCl = ls != LS_ANY ? 4 * C : PC;  // width of this layer's filter jets and adjoints
    const int kmax = ls == LS_LAST ? 0 : LMAX;  // the readout takes the last layer's l = 0 output only
    {
      KernelTimer kt(ctx, MLIP_K_MSG_BF);
      auto kern = TP_KERNEL(k_tp_bf, ls, uni, G, TX, TF);
      hipLaunchKernelGGL(kern, dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, w->env,
                         reinterpret_cast<const TF*>(w->Rho[l]), w->cy, w->cyd, w->h[l], w->hd[l], w->mu_a[l], w->gh[l], w->ghd[l], (int)N, C, w->ad[l], X);
    }
    for (int k = 0; k <= kmax; ++k) {
      const int64_t o = G::L_OFF[k] * NC, rows = (2 * k + 1) * N;
      if (gate)
        mix_mm<P>(ctx, l, k, false, LdPlain{w->ad[l] + o, C}, EpiStore{w->ud[l] + o, C, rows});
      else
        mix_mm<P>(ctx, l, k, false, LdPlain{w->ad[l] + o, C}, EpiAddStore{w->hd[l + 1] + o, w->hd[l] + o, C, rows});
      MLIP_TRY((mix_wgrad<P>(ctx, l, k, LdPlain{(gate ? w->mu_u[l] : w->mu_h[l + 1]) + o, C}, LdPlain{w->ad[l] + o, C}, grad)));
    }
    if (gate) hipLaunchKernelGGL(k_gate_bf, dim3(nblk(NC)), dim3(256), 0, st, w->u[l], w->ud[l], w->hd[l], w->hd[l + 1], NC, ls == LS_LAST ? 1 : NM);
    if (l + 1 < L) pack_rows<TF, G>(ctx, w->hd[l + 1], w->ghd[l + 1]);  // gathered by the next layer here and in BE
    if (Eu > 0) {
      {
        KernelTimer kt(ctx, MLIP_K_BF_WGRAD);
        hipLaunchKernelGGL(k_fill, dim3(nblk((int64_t)PCl * H)), dim3(256), 0, st, w->gWp, 0.f, (int64_t)PCl * H);
        MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xpair(X, PCl), Act<P>::odd(w->U[l], w->SJ[l], H), Eu, PCl, H, w->gWp)));
        hipLaunchKernelGGL(k_regroup_add, dim3(nblk((int64_t)PCl * H)), dim3(256), 0, st, w->gWp, C, H, path_list<G>(ls), ls != LS_ANY ? 4 : NPP, grad + lo.W[1]);
      }
      {
        KernelTimer kt(ctx, MLIP_K_BF_DGRAD);
        gemm_nt<P>(ctx, Act<P>::xpair(X, PCl), ls == LS_FIRST ? w->WpT0 : ls == LS_LAST ? w->WpTZ : w->WpT[l], Eu, H, PCl, EpiYZ<TX>{w->Y1[l], X2, w->U[l], H, Eu});
      }
      MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xld(X2, H), LdPlain{w->jphi + K, 2 * K}, Eu, H, K, grad + lo.W[0])));
    }
  }
  gemm_nt<P>(ctx, LdPlain{w->hd[L], C}, th + ctx->off_U, N, C, C, EpiStore{w->yd, C, N});
  MLIP_TRY((gemm_wgrad<P>(ctx, LdMuY{w->y, th + ctx->off_wo, C}, LdPlain{w->hd[L], C}, N, C, C, grad + ctx->off_U)));
  {
    const int chunks = atom_chunks(N), len = (int)((N + chunks - 1) / chunks);
    hipLaunchKernelGGL(k_wo_grad<0>, dim3((C + 63) / 64, chunks), dim3(256), 0, st, w->y, w->yd, nullptr, nullptr, (int)N, C, len, ctx->partial.buf);
    hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(C, 64)), dim3(256), 0, st, ctx->partial.buf, chunks, (int64_t)C, grad + ctx->off_wo);
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

template <typename P, typename TF, typename G>
int be_impl(mlip_ctx* ctx, float* grad) {
  EqvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  const int64_t N = ctx->N, E = ctx->E, Eu = ctx->Eu, NC = N * cf.channels;  // atoms, edges, edge pairs (rows of the edge MLP's products)
  constexpr int NM = G::NM, NPATH = G::NPATH, NPP = G::NPP, CY_LD = G::CY_LD, LMAX = G::LMAX;
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, PC = NPP * C;
  const float* th = ctx->d_params;
  const bool gate = cf.gate != 0;
  const float* tT = w->paramsT;
  typedef typename Act<P>::xop_t TX;  // X and X2 only feed matrix products: stored in the operand precision
  TX* X = reinterpret_cast<TX*>(w->X);
  TX* X2 = reinterpret_cast<TX*>(w->X2);
  int cur = 0;
  hipLaunchKernelGGL(k_lam_y, dim3(nblk(NC)), dim3(256), 0, st, w->y, w->yd, th + ctx->off_wo, w->Ebar, ctx->d_atom_struct, N, C, w->lam_y);
  {
    const int chunks = atom_chunks(N), len = (int)((N + chunks - 1) / chunks);
    hipLaunchKernelGGL(k_wo_grad<1>, dim3((C + 63) / 64, chunks), dim3(256), 0, st, w->y, nullptr, w->Ebar, ctx->d_atom_struct, (int)N, C, len, ctx->partial.buf);
    hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(C, 64)), dim3(256), 0, st, ctx->partial.buf, chunks, (int64_t)C, grad + ctx->off_wo);
  }
  MLIP_TRY((gemm_wgrad<P>(ctx, LdPlain{w->lam_y, C}, LdPlain{w->h[L], C}, N, C, C, grad + ctx->off_U)));
  hipLaunchKernelGGL(k_fill, dim3(nblk((NM - 1) * NC)), dim3(256), 0, st, w->lam_h[cur] + NC, 0.f, (NM - 1) * NC);
  gemm_nt<P>(ctx, LdPlain{w->lam_y, C}, tT + ctx->off_U, N, C, C, EpiStore{w->lam_h[cur], C, N});
  const int rpb = 256 / C;
  const bool uni = C % 64 == 0;  // a wave then holds channels of one receiver row only
  const bool want_gp = ctx->d_grad_pos != nullptr;
  if (want_gp) hipLaunchKernelGGL(k_fill, dim3(nblk(3 * N)), dim3(256), 0, st, w->gp_acc, 0.f, 3 * N);
  for (int l = L - 1; l >= 0; --l) {
    const LayerOffsets& lo = ctx->lay[l];
    const int ls = layer_spec(l, L, cf.position_grad);
    const int PCl = ls != LS_ANY ? 4 * C : PC;  // width of this layer's filter jets and adjoints
    const int kmax = ls == LS_LAST ? 0 : LMAX;  // the last layer's adjoints have their l = 0 component only
    float* lh_next = w->lam_h[cur];
    float* lh = w->lam_h[cur ^ 1];
    const float* lam_z = lh_next;  // adjoint of the update's output; through the gate it becomes that of W a
    if (gate) {
      hipLaunchKernelGGL(k_gate_be, dim3(nblk(NC)), dim3(256), 0, st, w->u[l], w->ud[l], w->mu_h[l + 1], lh_next, w->lam_u, NC, ls == LS_LAST ? 1 : NM);
      lam_z = w->lam_u;
    }
    for (int k = 0; k <= kmax; ++k) {
      const int64_t o = G::L_OFF[k] * NC, rows = (2 * k + 1) * N;
      mix_mm<P>(ctx, l, k, true, LdPlain{lam_z + o, C}, EpiStore{w->lam_a + o, C, rows});
      MLIP_TRY((mix_wgrad<P>(ctx, l, k, LdPlain{lam_z + o, C}, LdPlain{w->a[l] + o, C}, grad)));
    }
    if (ls != LS_LAST) pack_rows<TF, G>(ctx, w->lam_a, w->glam);
    {
      KernelTimer kt(ctx, MLIP_K_MSG_BE);
      auto kern = TP_KERNEL(k_tp_be, ls, uni, G, TX, TF);
      hipLaunchKernelGGL(kern, dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, w->env,
                         reinterpret_cast<const TF*>(w->Rho[l]), w->cy, w->cyd, w->h[l], w->hd[l], w->mu_a[l], w->lam_a, w->gmu[l], w->glam, lh_next,
                         (int)N, C, lh, X);
    }
    if (want_gp && Eu > 0) {
      // dL/dx (optional, off the timed path): radial weights with their first and second r-derivative, then this layer's share
      const float dmu = cf.cutoff / (float)(K - 1), gamma = 0.5f / (dmu * dmu);
      gemm_nt<P>(ctx, LdPhi2{ctx->d_geo, ctx->d_und, dmu, gamma}, th + lo.W[0], Eu, H, K, EpiStore{w->U2, H, Eu});
      gemm_nt<P>(ctx, Act<P>::jet(w->U[l], w->SJ[l], H), w->Wp[l], 2 * Eu, PC, H, EpiStore{w->Rj, PC, 2 * Eu});
      gemm_nt<P>(ctx, LdJetSecond{w->U[l], w->U2, H}, w->Wp[l], Eu, PC, H, EpiStore{w->Rpp, PC, Eu});
      const float kk = 3.14159265358979323846f / cf.cutoff;
      hipLaunchKernelGGL(k_tp_gp<G>, dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, ctx->d_geo, w->env, w->Rj, w->Rpp,
                         w->h[l], w->hd[l], w->mu_a[l], w->lam_a, w->v, kk * kk, (int)N, C, w->gp_acc);
    }
    if (Eu > 0) {
      {
        KernelTimer kt(ctx, MLIP_K_BE_WGRAD);
        hipLaunchKernelGGL(k_fill, dim3(nblk((int64_t)PCl * H)), dim3(256), 0, st, w->gWp, 0.f, (int64_t)PCl * H);
        MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xpair(X, PCl), Act<P>::even(w->U[l], w->SJ[l], H), Eu, PCl, H, w->gWp)));
        hipLaunchKernelGGL(k_regroup_add, dim3(nblk((int64_t)PCl * H)), dim3(256), 0, st, w->gWp, C, H, path_list<G>(ls), ls != LS_ANY ? 4 : NPP, grad + lo.W[1]);
      }
      {
        KernelTimer kt(ctx, MLIP_K_BE_DGRAD);
        gemm_nt<P>(ctx, Act<P>::xpair(X, PCl), ls == LS_FIRST ? w->WpT0 : ls == LS_LAST ? w->WpTZ : w->WpT[l], Eu, H, PCl, EpiLamU<TX>{X2, w->U[l], w->Y1[l], H, Eu});
      }
      MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xld(X2, H), LdPlain{w->jphi, 2 * K}, Eu, H, K, grad + lo.W[0])));
    }
    cur ^= 1;
  }
  if (want_gp) hipLaunchKernelGGL(k_scale3, dim3(nblk(3 * N)), dim3(256), 0, st, w->gp_acc, 1.f, 3 * N, ctx->d_grad_pos);
  {
    const int chunks = atom_chunks(N), len = (int)((N + chunks - 1) / chunks), S = cf.n_species;
    hipLaunchKernelGGL(k_emb_grad, dim3((C + 63) / 64, chunks, S), dim3(256), 0, st, w->lam_h[cur], ctx->d_species, (int)N, C, S, len, ctx->partial.buf);
    hipLaunchKernelGGL(k_reduce_partials, dim3(nblk((int64_t)S * C, 64)), dim3(256), 0, st, ctx->partial.buf, chunks, (int64_t)S * C, grad + ctx->off_emb);
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

}  // namespace

#if MLIP_EQV_PHASE >= 0
// One phase for a context whose l_max is this object's.  TF = storage type of the radial-filter jets: float, or bf16 in
// bf16 mode unless the context asks for fp32 filters; G = the coupling tables.
#define MLIP_EQV_CAT2(l, ph) eqv_phase_l##l##_##ph
#define MLIP_EQV_CAT(l, ph) MLIP_EQV_CAT2(l, ph)
int MLIP_EQV_CAT(MLIP_EQV_LMAX, MLIP_EQV_PHASE)(mlip_ctx* ctx, float* out) {
  typedef gaunt::Tab<MLIP_EQV_LMAX> G;
#define EQV_RUN(fn)                                                                                         \
  (ctx->cfg.gemm_dtype == MLIP_GEMM_BF16                                                                    \
       ? (ctx->cfg.filter_fp32 ? fn<gemm::Bf16, float, G>(ctx, out) : fn<gemm::Bf16, __bf16, G>(ctx, out))  \
       : fn<gemm::Fp32, float, G>(ctx, out))
#if MLIP_EQV_PHASE == 0
  return EQV_RUN(fe_impl);
#elif MLIP_EQV_PHASE == 1
  return EQV_RUN(ff_impl);
#elif MLIP_EQV_PHASE == 2
  return EQV_RUN(bf_impl);
#else
  return EQV_RUN(be_impl);
#endif
#undef EQV_RUN
}
#else
// =================================================================================== interface
int eqv_alloc(mlip_ctx* ctx) {
  const mlip_config& cf = ctx->cfg;
  const int64_t N = cf.max_atoms, E = cf.max_edges, B = cf.max_structs;
  const int lmax = cf.l_max;
  const int NM = (lmax + 1) * (lmax + 1);
  const int NPP = lmax == 3 ? gaunt::Tab<3>::NPP : gaunt::Tab<2>::NPP;
  const int CY_LD = lmax == 3 ? gaunt::Tab<3>::CY_LD : gaunt::Tab<2>::CY_LD;
  const int TAB = 64 * (lmax == 3 ? gaunt::Tab<3>::TAB_LOADS : gaunt::Tab<2>::TAB_LOADS);
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, PC = NPP * C;
  if (C > 256) MLIP_FAIL(ctx, MLIP_E_UNSUPPORTED, "equivariant model: channels must not exceed 256");
  EqvWs* w = new EqvWs();
  ctx->model_ws = w;
  bool ok = true;
  auto A = [&](int64_t n) { float* p = alloc_n<float>(ctx, n); ok &= (p != nullptr); return p; };
  ok &= (ctx->d_pos = alloc_n<float>(ctx, 3 * N)) != nullptr;
  ok &= (ctx->d_params = alloc_n<float>(ctx, ctx->n_params)) != nullptr;
  ok &= (ctx->d_species = alloc_n<int32_t>(ctx, N)) != nullptr;
  ok &= (ctx->d_geo = alloc_n<float4>(ctx, E)) != nullptr;
  w->paramsT = A(ctx->n_params);
  if (cf.gemm_dtype == MLIP_GEMM_BF16) ok &= add_shadow(ctx, ctx->d_params, ctx->n_params) && add_shadow(ctx, w->paramsT, ctx->n_params);
  const int64_t Eu = E / 2 + 1;  // edge pairs
  w->jphi = A(2 * Eu * K);
  ok &= (w->env = alloc_n<float2>(ctx, E)) != nullptr;
  ok &= (w->env_u = alloc_n<float2>(ctx, Eu)) != nullptr;
  const bool b16 = cf.gemm_dtype == MLIP_GEMM_BF16;
  // tensors held in the operand precision: half the floats when that is bf16
  auto AH = [&](int64_t n) { return A(b16 ? (n + 1) / 2 : n); };
  w->X = AH(2 * Eu * PC);
  w->gWp = A((int64_t)PC * H);
  w->Wp0 = A((int64_t)4 * C * H);
  w->WpT0 = A((int64_t)4 * C * H);
  w->WpZ = A((int64_t)4 * C * H);
  w->WpTZ = A((int64_t)4 * C * H);
  if (cf.gemm_dtype == MLIP_GEMM_BF16 && ok)
    ok &= add_shadow(ctx, w->Wp0, (int64_t)4 * C * H) && add_shadow(ctx, w->WpT0, (int64_t)4 * C * H) && add_shadow(ctx, w->WpZ, (int64_t)4 * C * H) &&
          add_shadow(ctx, w->WpTZ, (int64_t)4 * C * H);
  w->cy = A(E * CY_LD + TAB);  // + TAB: the cooperative fetch of the last edge's table reads TAB floats from its start
  w->cyd = A(E * CY_LD + TAB);
  w->X2 = AH(Eu * H);
  const int64_t NC9 = (int64_t)NM * N * C;  // a node table: all components
  const bool packed = b16 && !cf.filter_fp32 && lmax == 2;  // packed bf16 sender rows [N][C][10]: 5 floats per (atom, channel)
  const int64_t NCP = N * C * 5;
  for (int l = 0; l < L; ++l) {
    w->U.push_back(A(2 * Eu * H));
    w->SJ.push_back(b16 ? (__bf16*)A(Eu * H) : nullptr);
    w->Rho.push_back(cf.filter_fp32 ? A(2 * Eu * PC) : AH(2 * Eu * PC));
    w->Wp.push_back(A((int64_t)PC * H));
    w->WpT.push_back(A((int64_t)PC * H));
    if (b16 && ok) ok &= add_shadow(ctx, w->Wp[l], (int64_t)PC * H) && add_shadow(ctx, w->WpT[l], (int64_t)PC * H);
    w->Y1.push_back(A(Eu * H));
    w->a.push_back(A(NC9)); w->mu_a.push_back(A(NC9)); w->ad.push_back(A(NC9));
    if (packed) { w->gh.push_back((__bf16*)A(NCP)); w->ghd.push_back((__bf16*)A(NCP)); w->gmu.push_back((__bf16*)A(NCP)); }
    else { w->gh.push_back(nullptr); w->ghd.push_back(nullptr); w->gmu.push_back(nullptr); }
    if (cf.gate) { w->u.push_back(A(NC9)); w->mu_u.push_back(A(NC9)); w->ud.push_back(A(NC9)); }
    if (cf.n_experts > 0)
      for (int k = 0; k <= lmax; ++k) { w->Wm[k].push_back(A(B * C * C)); w->WmT[k].push_back(A(B * C * C)); }
  }
  for (int l = 0; l <= L; ++l) { w->h.push_back(A(NC9)); w->mu_h.push_back(A(NC9)); w->hd.push_back(A(NC9)); }
  w->lam_h[0] = A(NC9); w->lam_h[1] = A(NC9); w->lam_a = A(NC9);
  if (cf.gate) w->lam_u = A(NC9);
  if (packed) w->glam = (__bf16*)A(NCP);
  w->y = A(N * C); w->yd = A(N * C); w->lam_y = A(N * C);
  w->eps = A(N); w->Facc = A(3 * N); w->v = A(3 * N); w->Ebar = A(B);
  if (C % 64 == 0) w->Fp = A((int64_t)L * Eu * (C / 64) * 3);
  if (cf.position_grad) {
    w->U2 = A(Eu * H);
    w->Rj = A(2 * Eu * PC);
    w->Rpp = A(Eu * PC);
    w->gp_acc = A(3 * N);
  }
  int64_t cap = 0;
  auto need = [&](int64_t rows, int cols, int64_t R) {
    const bool narrow = cols <= 32;
    int bm = narrow ? 128 : (rows > 64 ? 128 : 64), bn = narrow ? 32 : (rows > 64 ? 128 : 64);
    cap = std::max<int64_t>(cap, (int64_t)pick_splits(rows, cols, R, bm, bn) * rows * cols);
  };
  need(PC, H, E); need(H, K, E); need(C, C, (2 * lmax + 1) * N);
  cap = std::max<int64_t>(cap, (int64_t)128 * std::max(1, cf.n_species) * C);
  if (cf.n_experts > 0)  // one weight-gradient partial per (component, structure), plus the split products of the coefficient gradient
    cap = std::max<int64_t>(cap, (2 * lmax + 1) * B * ((int64_t)C * C + 256 * (int64_t)((cf.n_experts + 3) / 4 * 4)));
  ctx->partial.cap = cap;
  ctx->partial.buf = A(cap);
  return ok ? MLIP_OK : MLIP_E_HIP;
}

void eqv_free(mlip_ctx* ctx) {
  delete ws_of(ctx);
  ctx->model_ws = nullptr;
}

// the phase's object for the context's l_max
#define DISPATCH(ph, out) (ctx->cfg.l_max == 3 ? eqv_phase_l3_##ph(ctx, out) : eqv_phase_l2_##ph(ctx, out))

int eqv_forward_energy(mlip_ctx* ctx, const float* pos, const int32_t* species, const float* params, const float*,
                       float* E, float*) {
  if (ctx->phase < PH_GRAPH) MLIP_FAIL(ctx, MLIP_E_STATE, "forward_energy: build the graph first");
  if (!pos || !params || !species || !E) MLIP_FAIL(ctx, MLIP_E_INVALID, "forward_energy: null pointer");
  if (ctx->cfg.n_experts > 0 && ctx->alpha_structs != ctx->B)
    MLIP_FAIL(ctx, MLIP_E_STATE, "forward_energy: set the expert coefficients of this batch's structures first (mlip_set_expert_weights)");
  hipStream_t st = ctx->stream;
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_pos, pos, sizeof(float) * 3 * ctx->N, hipMemcpyDeviceToDevice, st));
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_params, params, sizeof(float) * ctx->n_params, hipMemcpyDeviceToDevice, st));
  hipLaunchKernelGGL(k_copy_species, dim3(nblk(ctx->N)), dim3(256), 0, st, species, ctx->N, ctx->cfg.n_species, ctx->d_species, ctx->d_flag);
  MLIP_TRY(DISPATCH(0, E));
  ctx->phase = PH_FE;
  return MLIP_OK;
}

int eqv_forward_force(mlip_ctx* ctx, const float*, float* F, float*) {
  if (ctx->phase < PH_FE) MLIP_FAIL(ctx, MLIP_E_STATE, "forward_force: run forward_energy first");
  if (!F) MLIP_FAIL(ctx, MLIP_E_INVALID, "forward_force: null pointer");
  MLIP_TRY(DISPATCH(1, F));
  ctx->phase = PH_FF;
  return MLIP_OK;
}

int eqv_backward_force(mlip_ctx* ctx, const float* v, const float*, float* grad, float*) {
  if (ctx->phase < PH_FF) MLIP_FAIL(ctx, MLIP_E_STATE, "backward_force: run forward_force first");
  if (!v || !grad) MLIP_FAIL(ctx, MLIP_E_INVALID, "backward_force: null pointer");
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ws_of(ctx)->v, v, sizeof(float) * 3 * ctx->N, hipMemcpyDeviceToDevice, ctx->stream));
  MLIP_TRY(DISPATCH(2, grad));
  ctx->phase = PH_BF;
  return MLIP_OK;
}

int eqv_backward_energy(mlip_ctx* ctx, const float* Ebar, const float*, float* grad, float*) {
  if (ctx->phase < PH_BF) MLIP_FAIL(ctx, MLIP_E_STATE, "backward_energy: run backward_force first");
  if (!Ebar || !grad) MLIP_FAIL(ctx, MLIP_E_INVALID, "backward_energy: null pointer");
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ws_of(ctx)->Ebar, Ebar, sizeof(float) * ctx->B, hipMemcpyDeviceToDevice, ctx->stream));
  MLIP_TRY(DISPATCH(3, grad));
  ctx->phase = PH_BE;
  return MLIP_OK;
}
#endif  // MLIP_EQV_PHASE
