// Invariant message-passing potential and its pipeline-stage variant: the four phases
// FE / FF / BF / BE (paper, Sec. 2) with hand-derived adjoints, no autograd.
//
// Derivation used throughout.  The edge MLP depends on the geometry only through the edge
// length r, so each layer's radial filter omega(r) = f_c(r) w(r) in R^C is carried together
// with its derivative omega'(r) as a "jet" (two rows per edge).  With m_e = omega_e (.) h_j:
//   FE  a_i = sum_e omega_e (.) h_j
//   FF  mu_h[i] += sum_e omega_e (.) mu_a[j]          (the graph is symmetric and omega, r are
//       F_i  = sum_e rhat_e sum_c omega'_e (h_j mu_a_i + h_i mu_a_j)   equal on opposite edges)
//   BF  adot_i = sum_e rdot_e omega'_e (.) h_j + omega_e (.) hdot_j,  rdot_e = rhat_e.(v_j - v_i)
//   BE  lam_h[i] += sum_e omega_e (.) lam_a[j] + rdot_e omega'_e (.) mu_a[j]
// where mu = dE/d(.) (FF's activation gradients), dotted quantities are tangents along
// v = -dL/dF, and lam = dPsi/d(.) with Psi = sum_s Ebar_s E_s + D_v E, whose parameter
// gradient is dL/dtheta.  Weight gradients: products that involve a derivative row of a jet
// (or a tangent) are the second-order term of Eq. 2 and are added by BF; products with value
// rows are the merged first-order term and are added by BE.
//
// Opposite edges have the same length, so the radial basis, the edge MLP and the filter jets are evaluated once per
// edge PAIR (half the rows of every edge matrix product): pair u owns rows 2u, 2u + 1 of the jet matrices, and an
// edge's slot = 2u + (0 | 1) says which pair it belongs to and which of the pair's two adjoint rows (X) it writes.
// The adjoint of a pair's filter jet is the sum of its two edges' rows, formed when X is staged for a product.
#include <algorithm>
#include <cmath>

#include "shared_kernels.h"

namespace {

using namespace fx;

struct InvWs {
  int L = 0, depth = 2;
  float* paramsT = nullptr;
  float* jphi = nullptr;   // [Eu][2][K]; every edge tensor below marked Eu has one row (or jet) per edge pair
  float2* env = nullptr;   // [E] (f_c, f_c')
  float2* env_u = nullptr; // [Eu] the same per edge pair (rows of the filter product)
  float4* erd = nullptr;   // [E] (rdot, f_c, f_c', 0), written by BF for itself and BE
  std::vector<float*> U[2];   // hidden pre-activations, jets [Eu][2][H]; U[0] level 1, U[1] level 2 (depth 3)
  std::vector<__bf16*> SJ[2];  // bf16 GEMMs only: activated jets of each hidden level, [Eu][2][H]
  std::vector<float*> Om;     // [Eu][2][C], in the operand precision (fp32 or bf16)
  std::vector<float*> Y[2];   // [Eu][H]  BF -> BE
  std::vector<float*> Vm[2], VmT[2];  // expert banks merged per structure: [B][C][C] of V1 / V2 per layer, and transposed
  float* X = nullptr;         // [Eu][2][C] adjoint rows of the two edges of each pair, then [Eu][max(C,H)] scratch; operand precision
  float* X2 = nullptr;
  std::vector<float*> h, a, q, mu_h, mu_a, mu_q, mu_t, hd, ad, qd;
  float* lam_h[2] = {nullptr, nullptr};
  float* lam_q = nullptr;
  float* lam_a = nullptr;
  float* y = nullptr;
  float* yd = nullptr;
  float* lam_y = nullptr;
  float* eps = nullptr;     // [N]
  float* Facc = nullptr;    // [N,3]
  float* v = nullptr;       // [N,3] copy taken at BF
  float* Ebar = nullptr;    // [B]
  // optional position gradient dL/dx (mlip_config.position_grad): second-derivative rows of the hidden levels,
  // the last edge matrix's output with its first and second r-derivative, and the per-atom accumulator
  float* U2[2] = {nullptr, nullptr};  // [Eu][H]
  float* Wj = nullptr;                // [Eu][2][C] (w, w')
  float* Wpp = nullptr;               // [Eu][C]   w''
  float* gp_acc = nullptr;            // [N,3]
};

inline InvWs* ws_of(mlip_ctx* ctx) { return (InvWs*)ctx->model_ws; }

// ------------------------------------------------------------------------------ small kernels
// Row-parallel gather kernels.  A row (receiver atom) is handled by TPR = C/4 threads, one
// float4 of channels each; a block of 256 threads holds 256/TPR rows.
struct RowThread {
  int row, cq;
  bool active;
};
__device__ __forceinline__ RowThread row_thread(int N, int CQ) {
  int rpb = 256 / CQ;
  int rl = threadIdx.x / CQ;
  RowThread t;
  t.cq = threadIdx.x % CQ;
  t.row = xcd_block() * rpb + rl;
  t.active = (rl < rpb) && (t.row < N);
  return t;
}
__device__ __forceinline__ void fma4(float4& acc, float4 a, float4 b) {
  acc.x += a.x * b.x; acc.y += a.y * b.y; acc.z += a.z * b.z; acc.w += a.w * b.w;
}
__device__ __forceinline__ void fma4s(float4& acc, float s, float4 a, float4 b) {
  acc.x += s * a.x * b.x; acc.y += s * a.y * b.y; acc.z += s * a.z * b.z; acc.w += s * a.w * b.w;
}

// The four message kernels walk a receiver row's edges in order.  An edge needs its sender index
// before it can gather the sender's node rows: two dependent memory round trips per edge if done
// naively (counters showed the waves waiting 92 % of the time).  So the loops are software
// pipelined in blocks of D edges: the sender indices are fetched two blocks ahead and all operands
// of the next block are requested before the current block's arithmetic.  Indices past the row's
// end are clamped to its last edge (a valid, redundant load), so no branch surrounds a load; only
// the arithmetic and the stores of the tail are guarded.
template <int D, typename In, typename Fetch, typename Use>
__device__ __forceinline__ void walk_row(const int2* __restrict__ se, int e0, int e1, Fetch fetch, Use use) {
  if (e0 >= e1) return;
  const int last = e1 - 1;
  auto clamp = [&](int e) { return e < last ? e : last; };
  In cur[D];
  int2 jn[D];  // (sender, slot) of an edge
#pragma unroll
  for (int k = 0; k < D; ++k) {
    const int2 x = se[clamp(e0 + k)];
    cur[k] = fetch(clamp(e0 + k), x.x, x.y);
  }
#pragma unroll
  for (int k = 0; k < D; ++k) jn[k] = se[clamp(e0 + D + k)];
  for (int e = e0; e < e1; e += D) {
    In nxt[D];
#pragma unroll
    for (int k = 0; k < D; ++k) nxt[k] = fetch(clamp(e + D + k), jn[k].x, jn[k].y);
#pragma unroll
    for (int k = 0; k < D; ++k) jn[k] = se[clamp(e + 2 * D + k)];
#pragma unroll
    for (int k = 0; k < D; ++k)
      if (e + k < e1) use(e + k, cur[k]);
#pragma unroll
    for (int k = 0; k < D; ++k) cur[k] = nxt[k];
  }
}

// UNI: a row's C/4 threads fill whole waves (C a multiple of 256), so the row's edge range is the same in every lane of a
// wave: taken from the first lane, it lets the edge indices, the (sender, slot) pairs and the per-edge values be fetched
// by scalar loads, which leaves the vector memory pipeline -- what bounds these loops -- to the rows of Om and the gathers.
template <bool UNI>
__device__ __forceinline__ int uni_row(int x) { return UNI ? __builtin_amdgcn_readfirstlane(x) : x; }

struct InFe { float4 w, hj; };
template <typename TF, bool UNI>
__global__ void __launch_bounds__(256) k_msg_fe(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                const TF* __restrict__ Om, const float* __restrict__ h, int N, int C,
                                                float* __restrict__ a) {
  RowThread t = row_thread(N, C / 4);
  if (!t.active) return;
  const int c0 = 4 * t.cq;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  walk_row<4, InFe>(
      se, uni_row<UNI>(row_ptr[t.row]), uni_row<UNI>(row_ptr[t.row + 1]),
      [&](int, int j, int slot) { return InFe{ld4(Om + (int64_t)(slot & ~1) * C + c0), ld4(h + (int64_t)j * C + c0)}; },
      [&](int, const InFe& c) { fma4(acc, c.w, c.hj); });
  *reinterpret_cast<float4*>(a + (int64_t)t.row * C + c0) = acc;
}

struct InFf { float4 w, wp, hj, maj, ge; };
template <typename TF, bool UNI>
__global__ void __launch_bounds__(256) k_msg_ff(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                const float4* __restrict__ geo, const TF* __restrict__ Om,
                                                const float* __restrict__ h, const float* __restrict__ mu_a,
                                                const float* __restrict__ mu_h_next, int N, int C,
                                                float* __restrict__ mu_h, float* __restrict__ Facc) {
  __shared__ float3 red[256];
  const int CQ = C / 4;
  RowThread t = row_thread(N, CQ);
  float3 f = make_float3(0.f, 0.f, 0.f);
  if (t.active) {
    const int c0 = 4 * t.cq;
    const int64_t ro = (int64_t)t.row * C + c0;
    float4 acc = ld4(mu_h_next + ro);
    const float4 hi = ld4(h + ro), mai = ld4(mu_a + ro);
    walk_row<2, InFf>(
        se, uni_row<UNI>(row_ptr[t.row]), uni_row<UNI>(row_ptr[t.row + 1]),
        [&](int e, int j, int slot) {
          InFf x;
          x.w = ld4(Om + (int64_t)(slot & ~1) * C + c0);
          x.wp = ld4(Om + (int64_t)(slot | 1) * C + c0);
          x.hj = ld4(h + (int64_t)j * C + c0);
          x.maj = ld4(mu_a + (int64_t)j * C + c0);
          x.ge = geo[e];
          return x;
        },
        [&](int, const InFf& c) {
          fma4(acc, c.w, c.maj);
          const float g = c.wp.x * (c.hj.x * mai.x + hi.x * c.maj.x) + c.wp.y * (c.hj.y * mai.y + hi.y * c.maj.y) +
                          c.wp.z * (c.hj.z * mai.z + hi.z * c.maj.z) + c.wp.w * (c.hj.w * mai.w + hi.w * c.maj.w);
          f.x += g * c.ge.x; f.y += g * c.ge.y; f.z += g * c.ge.z;
        });
    *reinterpret_cast<float4*>(mu_h + ro) = acc;
  }
  red[threadIdx.x] = f;
  __syncthreads();
  if (t.active && t.cq == 0) {
    float3 s = make_float3(0.f, 0.f, 0.f);
    for (int k = 0; k < CQ; ++k) {
      float3 x = red[threadIdx.x + k];
      s.x += x.x; s.y += x.y; s.z += x.z;
    }
    Facc[3 * t.row] += s.x;
    Facc[3 * t.row + 1] += s.y;
    Facc[3 * t.row + 2] += s.z;
  }
}

// Per edge (rdot, f_c, f_c', 0) with rdot = rhat . (v_sender - v_receiver): what BF and BE need of the geometry, the
// envelope and the displacement rate, in one 16-byte value per edge (their loops are bound by the number of loads they
// issue per edge, and every lane of a row would otherwise fetch the unit vector, the envelope and three rate components).
__global__ void k_edge_rdot(const float4* __restrict__ geo, const float2* __restrict__ env, const int32_t* __restrict__ sender,
                            const int32_t* __restrict__ receiver, const float* __restrict__ v, int64_t E,
                            float4* __restrict__ out) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const int j = sender[e], i = receiver[e];
  const float4 g = geo[e];
  const float2 c = env[e];
  const float rd = g.x * (v[3 * j] - v[3 * i]) + g.y * (v[3 * j + 1] - v[3 * i + 1]) + g.z * (v[3 * j + 2] - v[3 * i + 2]);
  out[e] = make_float4(rd, c.x, c.y, 0.f);
}

struct InBf { float4 w, wp, hj, hdj, q; int slot; };
template <typename TX, typename TF, bool UNI>
__global__ void __launch_bounds__(256) k_msg_bf(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                const float4* __restrict__ erd,
                                                const TF* __restrict__ Om, const float* __restrict__ h,
                                                const float* __restrict__ hd, const float* __restrict__ mu_a,
                                                int N, int C, float* __restrict__ ad,
                                                TX* __restrict__ X) {
  RowThread t = row_thread(N, C / 4);
  if (!t.active) return;
  const int c0 = 4 * t.cq;
  const int64_t ro = (int64_t)t.row * C + c0;
  const float4 mai = ld4(mu_a + ro);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  walk_row<2, InBf>(
      se, uni_row<UNI>(row_ptr[t.row]), uni_row<UNI>(row_ptr[t.row + 1]),
      [&](int e, int j, int slot) {
        InBf x;
        x.slot = slot;
        x.w = ld4(Om + (int64_t)(slot & ~1) * C + c0);
        x.wp = ld4(Om + (int64_t)(slot | 1) * C + c0);
        x.hj = ld4(h + (int64_t)j * C + c0);
        x.hdj = ld4(hd + (int64_t)j * C + c0);
        x.q = erd[e];
        return x;
      },
      [&](int, const InBf& c) {
        const float rd = c.q.x;
        fma4s(acc, rd, c.wp, c.hj);
        fma4(acc, c.w, c.hdj);
        const float s = rd * c.q.y;
        st4(X + (int64_t)c.slot * C + c0, make_float4(s * c.hj.x * mai.x, s * c.hj.y * mai.y, s * c.hj.z * mai.z, s * c.hj.w * mai.w));
      });
  *reinterpret_cast<float4*>(ad + ro) = acc;
}

// BE gathers only the sender's adjoints lam_a[j], mu_a[j] (its own lam_h needs them).  The edge-MLP adjoint it writes is
// that of the OPPOSITE edge (j <- i), the pair's other row (slot ^ 1): c (h_i lam_a,j + hdot_i mu_a,j) + c' rdot h_i mu_a,j
// needs this row's own features and the same two gathered tables; r, rdot and the envelope are equal on opposite edges.
// Every edge is some edge's opposite, so each X row is written exactly once, and half the gathers are gone.
struct InBe { float4 w, wp, laj, maj, q; int slot; };
template <typename TX, typename TF, bool UNI>
__global__ void __launch_bounds__(256) k_msg_be(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                const float4* __restrict__ erd,
                                                const TF* __restrict__ Om, const float* __restrict__ h,
                                                const float* __restrict__ hd, const float* __restrict__ mu_a,
                                                const float* __restrict__ lam_a,
                                                const float* __restrict__ lam_h_next, int N, int C,
                                                float* __restrict__ lam_h, TX* __restrict__ X) {
  RowThread t = row_thread(N, C / 4);
  if (!t.active) return;
  const int c0 = 4 * t.cq;
  const int64_t ro = (int64_t)t.row * C + c0;
  const float4 hi = ld4(h + ro), hdi = ld4(hd + ro);
  float4 acc = ld4(lam_h_next + ro);
  walk_row<2, InBe>(
      se, uni_row<UNI>(row_ptr[t.row]), uni_row<UNI>(row_ptr[t.row + 1]),
      [&](int e, int j, int slot) {
        InBe x;
        x.slot = slot;
        x.w = ld4(Om + (int64_t)(slot & ~1) * C + c0);
        x.wp = ld4(Om + (int64_t)(slot | 1) * C + c0);
        const int64_t jo = (int64_t)j * C + c0;
        x.laj = ld4(lam_a + jo); x.maj = ld4(mu_a + jo);
        x.q = erd[e];
        return x;
      },
      [&](int, const InBe& c) {
        const float rd = c.q.x, fc = c.q.y;
        fma4(acc, c.w, c.laj);
        fma4s(acc, rd, c.wp, c.maj);
        const float s = c.q.z * rd;
        float4 x;
        x.x = fc * (hi.x * c.laj.x + hdi.x * c.maj.x) + s * hi.x * c.maj.x;
        x.y = fc * (hi.y * c.laj.y + hdi.y * c.maj.y) + s * hi.y * c.maj.y;
        x.z = fc * (hi.z * c.laj.z + hdi.z * c.maj.z) + s * hi.z * c.maj.z;
        x.w = fc * (hi.w * c.laj.w + hdi.w * c.maj.w) + s * hi.w * c.maj.w;
        st4(X + (int64_t)(c.slot ^ 1) * C + c0, x);
      });
  *reinterpret_cast<float4*>(lam_h + ro) = acc;
}

// Position gradient of one layer.  With Psi = sum_s Ebar_s E_s + D_v E (whose x-derivative is dL/dx), an edge's
// geometry enters through the filter omega(r) = f_c w and through omegadot = rdot omega'(r), rdot = rhat.(v_j - v_i):
//   dPsi/dr_vec_e = [A_e . omega' + rdot B_e . omega''] rhat + (B_e . omega') (dv - rhat rdot) / r,
//   A_e = h_j lam_a,i + hdot_j mu_a,i  (adjoint of omega_e),   B_e = h_j mu_a,i  (adjoint of omegadot_e),
// and atom i collects -dPsi/dr_vec over the edges it receives and +dPsi/dr_vec over those it sends; the opposite
// edge has the same r, omega, rdot and the opposite rhat, dv, so both are formed here from the row's own and the
// gathered sender's node values.  omega' = c' w + c w', omega'' = c'' w + 2 c' w' + c w'', c'' = -(pi/r_c)^2 (c - 1/2).
struct InGp { float4 w, wp, wpp, hj, hdj, laj, maj, ge; float2 cc; float v0, v1, v2; };
__global__ void __launch_bounds__(256) k_msg_gp(const int32_t* __restrict__ row_ptr, const int2* __restrict__ se,
                                                const float4* __restrict__ geo, const float2* __restrict__ env,
                                                const float* __restrict__ Wj, const float* __restrict__ Wpp,
                                                const float* __restrict__ h, const float* __restrict__ hd,
                                                const float* __restrict__ mu_a, const float* __restrict__ lam_a,
                                                const float* __restrict__ v, float k2, int N, int C, float* __restrict__ gp) {
  __shared__ float3 red[256];
  const int CQ = C / 4;
  RowThread t = row_thread(N, CQ);
  float3 f = make_float3(0.f, 0.f, 0.f);
  if (t.active) {
    const int c0 = 4 * t.cq;
    const int64_t ro = (int64_t)t.row * C + c0;
    const float4 hi = ld4(h + ro), hdi = ld4(hd + ro), mai = ld4(mu_a + ro), lai = ld4(lam_a + ro);
    const float vi0 = v[3 * t.row], vi1 = v[3 * t.row + 1], vi2 = v[3 * t.row + 2];
    walk_row<2, InGp>(
        se, row_ptr[t.row], row_ptr[t.row + 1],
        [&](int e, int j, int slot) {
          InGp x;
          x.w = ld4(Wj + (int64_t)(slot & ~1) * C + c0);
          x.wp = ld4(Wj + (int64_t)(slot | 1) * C + c0);
          x.wpp = ld4(Wpp + (int64_t)(slot >> 1) * C + c0);
          const int64_t jo = (int64_t)j * C + c0;
          x.hj = ld4(h + jo); x.hdj = ld4(hd + jo); x.laj = ld4(lam_a + jo); x.maj = ld4(mu_a + jo);
          x.ge = geo[e];
          x.cc = env[e];
          x.v0 = v[3 * j]; x.v1 = v[3 * j + 1]; x.v2 = v[3 * j + 2];
          return x;
        },
        [&](int, const InGp& q) {
          const float d0 = q.v0 - vi0, d1 = q.v1 - vi1, d2 = q.v2 - vi2;
          const float rd = q.ge.x * d0 + q.ge.y * d1 + q.ge.z * d2;
          const float c = q.cc.x, cp = q.cc.y, cpp = -k2 * (c - 0.5f);
          const float w[4] = {q.w.x, q.w.y, q.w.z, q.w.w}, wp[4] = {q.wp.x, q.wp.y, q.wp.z, q.wp.w}, wpp[4] = {q.wpp.x, q.wpp.y, q.wpp.z, q.wpp.w};
          const float hj[4] = {q.hj.x, q.hj.y, q.hj.z, q.hj.w}, hdj[4] = {q.hdj.x, q.hdj.y, q.hdj.z, q.hdj.w};
          const float laj[4] = {q.laj.x, q.laj.y, q.laj.z, q.laj.w}, maj[4] = {q.maj.x, q.maj.y, q.maj.z, q.maj.w};
          const float hi4[4] = {hi.x, hi.y, hi.z, hi.w}, hdi4[4] = {hdi.x, hdi.y, hdi.z, hdi.w};
          const float lai4[4] = {lai.x, lai.y, lai.z, lai.w}, mai4[4] = {mai.x, mai.y, mai.z, mai.w};
          float G = 0.f, g = 0.f;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float op = cp * w[u] + c * wp[u];
            const float opp = cpp * w[u] + 2.f * cp * wp[u] + c * wpp[u];
            const float A = hj[u] * lai4[u] + hdj[u] * mai4[u] + hi4[u] * laj[u] + hdi4[u] * maj[u];
            const float Bm = hj[u] * mai4[u] + hi4[u] * maj[u];
            G += A * op + rd * Bm * opp;
            g += Bm * op;
          }
          const float gr = q.ge.w > 0.f ? g / q.ge.w : 0.f;
          f.x -= G * q.ge.x + gr * (d0 - q.ge.x * rd);
          f.y -= G * q.ge.y + gr * (d1 - q.ge.y * rd);
          f.z -= G * q.ge.z + gr * (d2 - q.ge.z * rd);
        });
  }
  red[threadIdx.x] = f;
  __syncthreads();
  if (t.active && t.cq == 0) {
    float3 s = make_float3(0.f, 0.f, 0.f);
    for (int k = 0; k < CQ; ++k) {
      float3 x = red[threadIdx.x + k];
      s.x += x.x; s.y += x.y; s.z += x.z;
    }
    gp[3 * t.row] += s.x;
    gp[3 * t.row + 1] += s.y;
    gp[3 * t.row + 2] += s.z;
  }
}

// The update MLP's matrices V1 (which = 0) / V2 (which = 1) of layer l: dense, or merged per
// structure from expert banks (then every product is structure-wise).
template <typename P, typename LdA, typename Epi>
void node_mm(mlip_ctx* ctx, int l, int which, bool transposed, const LdA& a, const Epi& epi) {
  InvWs* w = ws_of(ctx);
  const int C = ctx->cfg.channels;
  const int64_t off = which ? ctx->lay[l].V2 : ctx->lay[l].V1;
  if (ctx->cfg.n_experts > 0)
    gemm_nt_grouped<P>(ctx, a, (transposed ? w->VmT : w->Vm)[which][l], ctx->N, C, C, epi);
  else
    gemm_nt<P>(ctx, a, (transposed ? w->paramsT : ctx->d_params) + off, ctx->N, C, C, epi);
}
template <typename P, typename LdA, typename LdB>
int node_wgrad(mlip_ctx* ctx, int l, int which, const LdA& a, const LdB& b, float* grad) {
  const int C = ctx->cfg.channels;
  const int64_t off = which ? ctx->lay[l].V2 : ctx->lay[l].V1;
  float* g = grad + off;
  if (ctx->cfg.n_experts > 0) return gemm_wgrad_experts<P>(ctx, a, b, ctx->N, C, C, g, ctx->d_params + off);
  return gemm_wgrad<P>(ctx, a, b, ctx->N, C, C, g);
}

// ------------------------------------------------------------------------------ phases
template <typename P, typename TF>
int fe_impl(mlip_ctx* ctx, const float* h_in, float* E_out, float* h_out) {
  InvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  static_assert(sizeof(typename Act<P>::xop_t) == (P::IS_BF16 ? 2 : 4), "the workspace is sized for 2-byte operand-precision tensors in bf16 mode and 4-byte ones otherwise");
  const int64_t N = ctx->N, E = ctx->E, Eu = ctx->Eu;  // atoms, edges, edge pairs (rows of the edge MLP)
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, d = cf.edge_mlp_depth;
  const float* th = ctx->d_params;
  const bool stage = cf.model_kind == MLIP_MODEL_STAGE;

  // transposed copies of every matrix, for the data-gradient products of the later phases
  auto tr = [&](int64_t off, int rows, int cols) {
    hipLaunchKernelGGL(k_transpose, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(32, 8), 0, st, th + off, w->paramsT + off, rows, cols);
  };
  for (int l = 0; l < L; ++l) {
    const LayerOffsets& lo = ctx->lay[l];
    if (d == 3) { tr(lo.W[1], H, H); tr(lo.W[2], C, H); } else { tr(lo.W[1], C, H); }
    if (cf.n_experts > 0) {
      const dim3 grid(nblk((int64_t)C * C, 64), (unsigned)((ctx->B + 15) / 16));
      hipLaunchKernelGGL(k_merge_experts, grid, dim3(256), 0, st, ctx->d_alpha, th + lo.V1, ctx->B, cf.n_experts, C, w->Vm[0][l], w->VmT[0][l]);
      hipLaunchKernelGGL(k_merge_experts, grid, dim3(256), 0, st, ctx->d_alpha, th + lo.V2, ctx->B, cf.n_experts, C, w->Vm[1][l], w->VmT[1][l]);
    } else {
      tr(lo.V1, C, C);
      tr(lo.V2, C, C);
    }
  }
  if (!stage) tr(ctx->off_U, C, C);
  if (P::IS_BF16) refresh_shadows(ctx);  // bf16 mirrors of the weights and of their transposes

  if (E > 0)
    launch_edge_features(ctx, E, K, cf.cutoff, w->env, w->env_u, w->jphi);
  if (stage)
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(w->h[0], h_in, sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  else
    hipLaunchKernelGGL(k_embed, dim3(nblk(N * C)), dim3(256), 0, st, th + ctx->off_emb, ctx->d_species, N, C, w->h[0]);

  const int rpb = 256 / (C / 4);
  const bool uni = C % 256 == 0;  // a row's threads then fill whole waves
  for (int l = 0; l < L; ++l) {
    const LayerOffsets& lo = ctx->lay[l];
    if (Eu > 0) {
      {
        KernelTimer kt(ctx, MLIP_K_FE_HIDDEN_GEMM);
        gemm_nt<P>(ctx, LdPlain{w->jphi, K}, th + lo.W[0], 2 * Eu, H, K, Act<P>::store(w->U[0][l], w->SJ[0][l], H, 2 * Eu));
      }
      const float* ulast = w->U[0][l];
      const __bf16* sjlast = w->SJ[0][l];
      if (d == 3) {
        gemm_nt<P>(ctx, Act<P>::jet(w->U[0][l], w->SJ[0][l], H), th + lo.W[1], 2 * Eu, H, H, Act<P>::store(w->U[1][l], w->SJ[1][l], H, 2 * Eu));
        ulast = w->U[1][l];
        sjlast = w->SJ[1][l];
      }
      {
        KernelTimer kt(ctx, MLIP_K_FE_FILTER_GEMM);
        gemm_nt<P>(ctx, Act<P>::jet(ulast, sjlast, H), th + lo.W[d - 1], 2 * Eu, C, H, EpiOmega<TF>{reinterpret_cast<TF*>(w->Om[l]), w->env_u, C, 2 * Eu});
      }
    }
    {
      KernelTimer kt(ctx, MLIP_K_MSG_FE);
      hipLaunchKernelGGL((uni ? k_msg_fe<TF, true> : k_msg_fe<TF, false>), dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, reinterpret_cast<const TF*>(w->Om[l]), w->h[l],
                         (int)N, C, w->a[l]);
    }
    node_mm<P>(ctx, l, 0, false, LdPlain{w->a[l], C}, EpiStore{w->q[l], C, N});
    node_mm<P>(ctx, l, 1, false, LdSilu{w->q[l], C}, EpiAddStore{w->h[l + 1], w->h[l], C, N});
  }
  if (stage) {
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(h_out, w->h[L], sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  } else {
    gemm_nt<P>(ctx, LdPlain{w->h[L], C}, th + ctx->off_U, N, C, C, EpiStore{w->y, C, N});
    hipLaunchKernelGGL(k_atom_energy, dim3(nblk(N, 4)), dim3(256), 0, st, w->y, th + ctx->off_wo, (int)N, C, w->eps);
    hipLaunchKernelGGL(k_struct_sum, dim3(ctx->B), dim3(256), 0, st, w->eps, ctx->d_meta, E_out);
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

template <typename P, typename TF>
int ff_impl(mlip_ctx* ctx, const float* g_out, float* F, float* g_in) {
  InvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  const int64_t N = ctx->N;
  const int C = cf.channels, L = cf.n_layers;
  const float* th = ctx->d_params;
  const float* tT = w->paramsT;
  const bool stage = cf.model_kind == MLIP_MODEL_STAGE;
  if (stage)
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(w->mu_h[L], g_out, sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  else  // mu_y = w_o silu'(y);  mu_h^L = mu_y U
    gemm_nt<P>(ctx, LdMuY{w->y, th + ctx->off_wo, C}, tT + ctx->off_U, N, C, C, EpiStore{w->mu_h[L], C, N});
  hipLaunchKernelGGL(k_fill, dim3(nblk(3 * N)), dim3(256), 0, st, w->Facc, 0.f, 3 * N);
  const int rpb = 256 / (C / 4);
  const bool uni = C % 256 == 0;  // a row's threads then fill whole waves
  for (int l = L - 1; l >= 0; --l) {
    const LayerOffsets& lo = ctx->lay[l];
    node_mm<P>(ctx, l, 1, true, LdPlain{w->mu_h[l + 1], C}, EpiMuT{w->mu_t[l], w->mu_q[l], w->q[l], C, N});
    node_mm<P>(ctx, l, 0, true, LdPlain{w->mu_q[l], C}, EpiStore{w->mu_a[l], C, N});
    {
      KernelTimer kt(ctx, MLIP_K_MSG_FF);
      hipLaunchKernelGGL((uni ? k_msg_ff<TF, true> : k_msg_ff<TF, false>), dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, ctx->d_geo, reinterpret_cast<const TF*>(w->Om[l]),
                         w->h[l], w->mu_a[l], w->mu_h[l + 1], (int)N, C, w->mu_h[l], w->Facc);
    }
  }
  // F_i = + sum_e g_e rhat_e = -dE/dx_i ; a stage reports its contribution to +dE/dx
  hipLaunchKernelGGL(k_scale3, dim3(nblk(3 * N)), dim3(256), 0, st, w->Facc, stage ? -1.f : 1.f, 3 * N, F);
  if (stage) MLIP_HIP_CHECK(ctx, hipMemcpyAsync(g_in, w->mu_h[0], sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

template <typename P, typename TF>
int bf_impl(mlip_ctx* ctx, const float* hdot_in, float* grad, float* hdot_out) {
  InvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  const int64_t N = ctx->N, Eu = ctx->Eu;  // atoms, edge pairs (rows of the edge MLP's products)
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, d = cf.edge_mlp_depth;
  const float* th = ctx->d_params;
  const float* tT = w->paramsT;
  typedef typename Act<P>::xop_t TX;  // X and X2 only feed matrix products: stored in the operand precision
  TX* X = reinterpret_cast<TX*>(w->X);
  TX* X2 = reinterpret_cast<TX*>(w->X2);
  const bool stage = cf.model_kind == MLIP_MODEL_STAGE;
  if (stage && hdot_in)
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(w->hd[0], hdot_in, sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  else
    hipLaunchKernelGGL(k_fill, dim3(nblk(N * C)), dim3(256), 0, st, w->hd[0], 0.f, N * C);
  const int rpb = 256 / (C / 4);
  const bool uni = C % 256 == 0;  // a row's threads then fill whole waves
  if (ctx->E > 0)
    hipLaunchKernelGGL(k_edge_rdot, dim3(nblk(ctx->E)), dim3(256), 0, st, ctx->d_geo, w->env, ctx->d_sender, ctx->d_receiver, w->v, ctx->E, w->erd);
  for (int l = 0; l < L; ++l) {
    const LayerOffsets& lo = ctx->lay[l];
    {
      KernelTimer kt(ctx, MLIP_K_MSG_BF);
      hipLaunchKernelGGL((uni ? k_msg_bf<TX, TF, true> : k_msg_bf<TX, TF, false>), dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, w->erd,
                         reinterpret_cast<const TF*>(w->Om[l]), w->h[l], w->hd[l], w->mu_a[l], (int)N, C, w->ad[l], X);
    }
    node_mm<P>(ctx, l, 0, false, LdPlain{w->ad[l], C}, EpiStore{w->qd[l], C, N});
    node_mm<P>(ctx, l, 1, false, LdDsiluMul{w->q[l], w->qd[l], C}, EpiAddStore{w->hd[l + 1], w->hd[l], C, N});
    // second-order weight gradients of the update MLP: mu_{h'}^T tdot, mu_q^T adot
    MLIP_TRY((node_wgrad<P>(ctx, l, 1, LdPlain{w->mu_h[l + 1], C}, LdDsiluMul{w->q[l], w->qd[l], C}, grad)));
    MLIP_TRY((node_wgrad<P>(ctx, l, 0, LdPlain{w->mu_q[l], C}, LdPlain{w->ad[l], C}, grad)));
    if (Eu > 0) {
      // X = rdot * mu_w (adjoint of the derivative row w').  Chain back through the jets' derivative rows.
      const float* ulast = w->U[d - 2][l];
      {
        KernelTimer kt(ctx, MLIP_K_BF_WGRAD);
        MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xpair(X, C), Act<P>::odd(ulast, w->SJ[d - 2][l], H), Eu, C, H, grad + lo.W[d - 1])));
      }
      // The last data-gradient product of the chain feeds only the gradient of the first edge
      // matrix, Z^T phi' (K columns): fp32 folds that product into the epilogue (Z never reaches HBM).
      const bool fold = !P::IS_BF16 && fold_ok(ctx, Eu, H, K);
      const FoldB fb{w->jphi + K, 2 * K, K, nullptr};
      if (d == 2) {
        KernelTimer kt(ctx, MLIP_K_BF_DGRAD);
        if constexpr (!P::IS_BF16) {
          if (fold) gemm_nt_fold<P>(ctx, Act<P>::xpair(X, C), tT + lo.W[1], Eu, H, C, EpiYZFold<TX>{w->Y[0][l], ulast, H, Eu, fb}, grad + lo.W[0]);
        }
        if (!fold) gemm_nt<P>(ctx, Act<P>::xpair(X, C), tT + lo.W[1], Eu, H, C, EpiYZ<TX>{w->Y[0][l], X2, ulast, H, Eu});
      } else {
        {
          KernelTimer kt(ctx, MLIP_K_BF_DGRAD);
          gemm_nt<P>(ctx, Act<P>::xpair(X, C), tT + lo.W[2], Eu, H, C, EpiYZ<TX>{w->Y[1][l], X2, ulast, H, Eu});
        }
        MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xld(X2, H), Act<P>::odd(w->U[0][l], w->SJ[0][l], H), Eu, H, H, grad + lo.W[1])));
        if constexpr (!P::IS_BF16) {
          if (fold) gemm_nt_fold<P>(ctx, Act<P>::xld(X2, H), tT + lo.W[1], Eu, H, H, EpiYZFold<TX>{w->Y[0][l], w->U[0][l], H, Eu, fb}, grad + lo.W[0]);
        }
        if (!fold) gemm_nt<P>(ctx, Act<P>::xld(X2, H), tT + lo.W[1], Eu, H, H, EpiYZ<TX>{w->Y[0][l], X, w->U[0][l], H, Eu});
      }
      if (!fold) MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xld(d == 3 ? X : X2, H), LdPlain{w->jphi + K, 2 * K}, Eu, H, K, grad + lo.W[0])));
    }
  }
  if (stage) {
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(hdot_out, w->hd[L], sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  } else {
    gemm_nt<P>(ctx, LdPlain{w->hd[L], C}, th + ctx->off_U, N, C, C, EpiStore{w->yd, C, N});
    MLIP_TRY((gemm_wgrad<P>(ctx, LdMuY{w->y, th + ctx->off_wo, C}, LdPlain{w->hd[L], C}, N, C, C, grad + ctx->off_U)));
    {
      const int chunks = atom_chunks(N), len = (int)((N + chunks - 1) / chunks);
      hipLaunchKernelGGL(k_wo_grad<0>, dim3((C + 63) / 64, chunks), dim3(256), 0, st, w->y, w->yd, nullptr, nullptr, (int)N, C, len, ctx->partial.buf);
      hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(C, 64)), dim3(256), 0, st, ctx->partial.buf, chunks, (int64_t)C, grad + ctx->off_wo);
    }
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

template <typename P, typename TF>
int be_impl(mlip_ctx* ctx, const float* lam_out, float* grad, float* lam_in) {
  InvWs* w = ws_of(ctx);
  const mlip_config& cf = ctx->cfg;
  hipStream_t st = ctx->stream;
  const int64_t N = ctx->N, Eu = ctx->Eu;  // atoms, edge pairs (rows of the edge MLP's products)
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, d = cf.edge_mlp_depth;
  const float* th = ctx->d_params;
  const float* tT = w->paramsT;
  typedef typename Act<P>::xop_t TX;  // X and X2 only feed matrix products: stored in the operand precision
  TX* X = reinterpret_cast<TX*>(w->X);
  TX* X2 = reinterpret_cast<TX*>(w->X2);
  const bool stage = cf.model_kind == MLIP_MODEL_STAGE;
  int cur = 0;
  if (stage) {
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(w->lam_h[cur], lam_out, sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  } else {
    hipLaunchKernelGGL(k_lam_y, dim3(nblk(N * C)), dim3(256), 0, st, w->y, w->yd, th + ctx->off_wo, w->Ebar, ctx->d_atom_struct, N, C, w->lam_y);
    {
      const int chunks = atom_chunks(N), len = (int)((N + chunks - 1) / chunks);
      hipLaunchKernelGGL(k_wo_grad<1>, dim3((C + 63) / 64, chunks), dim3(256), 0, st, w->y, nullptr, w->Ebar, ctx->d_atom_struct, (int)N, C, len, ctx->partial.buf);
      hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(C, 64)), dim3(256), 0, st, ctx->partial.buf, chunks, (int64_t)C, grad + ctx->off_wo);
    }
    MLIP_TRY((gemm_wgrad<P>(ctx, LdPlain{w->lam_y, C}, LdPlain{w->h[L], C}, N, C, C, grad + ctx->off_U)));
    gemm_nt<P>(ctx, LdPlain{w->lam_y, C}, tT + ctx->off_U, N, C, C, EpiStore{w->lam_h[cur], C, N});
  }
  const int rpb = 256 / (C / 4);
  const bool uni = C % 256 == 0;  // a row's threads then fill whole waves
  const bool want_gp = ctx->d_grad_pos != nullptr;
  if (want_gp) hipLaunchKernelGGL(k_fill, dim3(nblk(3 * N)), dim3(256), 0, st, w->gp_acc, 0.f, 3 * N);
  for (int l = L - 1; l >= 0; --l) {
    const LayerOffsets& lo = ctx->lay[l];
    float* lh_next = w->lam_h[cur];
    float* lh = w->lam_h[cur ^ 1];
    node_mm<P>(ctx, l, 1, true, LdPlain{lh_next, C}, EpiLamQ{w->lam_q, w->q[l], w->qd[l], w->mu_t[l], C, N});
    MLIP_TRY((node_wgrad<P>(ctx, l, 1, LdPlain{lh_next, C}, LdSilu{w->q[l], C}, grad)));
    MLIP_TRY((node_wgrad<P>(ctx, l, 0, LdPlain{w->lam_q, C}, LdPlain{w->a[l], C}, grad)));
    node_mm<P>(ctx, l, 0, true, LdPlain{w->lam_q, C}, EpiStore{w->lam_a, C, N});
    {
      KernelTimer kt(ctx, MLIP_K_MSG_BE);
      hipLaunchKernelGGL((uni ? k_msg_be<TX, TF, true> : k_msg_be<TX, TF, false>), dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, w->erd,
                         reinterpret_cast<const TF*>(w->Om[l]), w->h[l], w->hd[l], w->mu_a[l], w->lam_a, lh_next, (int)N, C, lh, X);
    }
    if (want_gp && Eu > 0) {
      // dL/dx (optional, off the timed path): the edge MLP's output with its first and second r-derivative
      // (second-derivative rows chained through the hidden levels), then this layer's share per atom
      const float dmu = cf.cutoff / (float)(K - 1), gamma = 0.5f / (dmu * dmu);
      gemm_nt<P>(ctx, LdPhi2{ctx->d_geo, ctx->d_und, dmu, gamma}, th + lo.W[0], Eu, H, K, EpiStore{w->U2[0], H, Eu});
      const float* u2last = w->U2[0];
      if (d == 3) {
        gemm_nt<P>(ctx, LdJetSecond{w->U[0][l], w->U2[0], H}, th + lo.W[1], Eu, H, H, EpiStore{w->U2[1], H, Eu});
        u2last = w->U2[1];
      }
      const float* ul = w->U[d - 2][l];
      gemm_nt<P>(ctx, Act<P>::jet(ul, w->SJ[d - 2][l], H), th + lo.W[d - 1], 2 * Eu, C, H, EpiStore{w->Wj, C, 2 * Eu});
      gemm_nt<P>(ctx, LdJetSecond{ul, u2last, H}, th + lo.W[d - 1], Eu, C, H, EpiStore{w->Wpp, C, Eu});
      const float kk = 3.14159265358979323846f / cf.cutoff;
      hipLaunchKernelGGL(k_msg_gp, dim3(nblk8(N, rpb)), dim3(256), 0, st, ctx->d_row_ptr, ctx->d_se, ctx->d_geo, w->env, w->Wj, w->Wpp,
                         w->h[l], w->hd[l], w->mu_a[l], w->lam_a, w->v, kk * kk, (int)N, C, w->gp_acc);
    }
    if (Eu > 0) {
      const float* ulast = w->U[d - 2][l];
      {
        KernelTimer kt(ctx, MLIP_K_BE_WGRAD);
        MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xpair(X, C), Act<P>::even(ulast, w->SJ[d - 2][l], H), Eu, C, H, grad + lo.W[d - 1])));
      }
      // as in BF: the last product of the chain is folded with phi (value rows) in fp32
      const bool fold = !P::IS_BF16 && fold_ok(ctx, Eu, H, K);
      const FoldB fb{w->jphi, 2 * K, K, nullptr};
      if (d == 2) {
        KernelTimer kt(ctx, MLIP_K_BE_DGRAD);
        if constexpr (!P::IS_BF16) {
          if (fold) gemm_nt_fold<P>(ctx, Act<P>::xpair(X, C), tT + lo.W[1], Eu, H, C, EpiLamUFold<TX>{ulast, w->Y[0][l], H, Eu, fb}, grad + lo.W[0]);
        }
        if (!fold) gemm_nt<P>(ctx, Act<P>::xpair(X, C), tT + lo.W[1], Eu, H, C, EpiLamU<TX>{X2, ulast, w->Y[0][l], H, Eu});
      } else {
        {
          KernelTimer kt(ctx, MLIP_K_BE_DGRAD);
          gemm_nt<P>(ctx, Act<P>::xpair(X, C), tT + lo.W[2], Eu, H, C, EpiLamU<TX>{X2, ulast, w->Y[1][l], H, Eu});
        }
        MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xld(X2, H), Act<P>::even(w->U[0][l], w->SJ[0][l], H), Eu, H, H, grad + lo.W[1])));
        if constexpr (!P::IS_BF16) {
          if (fold) gemm_nt_fold<P>(ctx, Act<P>::xld(X2, H), tT + lo.W[1], Eu, H, H, EpiLamUFold<TX>{w->U[0][l], w->Y[0][l], H, Eu, fb}, grad + lo.W[0]);
        }
        if (!fold) gemm_nt<P>(ctx, Act<P>::xld(X2, H), tT + lo.W[1], Eu, H, H, EpiLamU<TX>{X, w->U[0][l], w->Y[0][l], H, Eu});
      }
      if (!fold) MLIP_TRY((gemm_wgrad<P>(ctx, Act<P>::xld(d == 3 ? X : X2, H), LdPlain{w->jphi, 2 * K}, Eu, H, K, grad + lo.W[0])));
    }
    cur ^= 1;
  }
  if (want_gp) hipLaunchKernelGGL(k_scale3, dim3(nblk(3 * N)), dim3(256), 0, st, w->gp_acc, 1.f, 3 * N, ctx->d_grad_pos);
  if (stage)
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(lam_in, w->lam_h[cur], sizeof(float) * N * C, hipMemcpyDeviceToDevice, st));
  else {
    const int chunks = atom_chunks(N), len = (int)((N + chunks - 1) / chunks), S = cf.n_species;
    hipLaunchKernelGGL(k_emb_grad, dim3((C + 63) / 64, chunks, S), dim3(256), 0, st, w->lam_h[cur], ctx->d_species, (int)N, C, S, len, ctx->partial.buf);
    hipLaunchKernelGGL(k_reduce_partials, dim3(nblk((int64_t)S * C, 64)), dim3(256), 0, st, ctx->partial.buf, chunks, (int64_t)S * C, grad + ctx->off_emb);
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

}  // namespace

// =================================================================================== interface
int inv_alloc(mlip_ctx* ctx) {
  const mlip_config& cf = ctx->cfg;
  const int64_t N = cf.max_atoms, E = cf.max_edges, B = cf.max_structs;
  const int C = cf.channels, H = cf.edge_hidden, K = cf.n_rbf, L = cf.n_layers, d = cf.edge_mlp_depth;
  InvWs* w = new InvWs();
  ctx->model_ws = w;
  w->L = L;
  w->depth = d;
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
  ok &= (w->erd = alloc_n<float4>(ctx, E)) != nullptr;
  const int64_t Wmax = std::max(C, H);
  const bool b16 = cf.gemm_dtype == MLIP_GEMM_BF16;
  // tensors held in the operand precision: half the floats when that is bf16
  auto AH = [&](int64_t n) { return A(b16 ? (n + 1) / 2 : n); };
  w->X = AH(std::max(2 * Eu * C, Eu * Wmax));
  w->X2 = AH(Eu * Wmax);
  for (int l = 0; l < L; ++l) {
    w->U[0].push_back(A(2 * Eu * H));
    w->U[1].push_back(d == 3 ? A(2 * Eu * H) : nullptr);
    w->SJ[0].push_back(b16 ? (__bf16*)A(Eu * H) : nullptr);  // 2 Eu H bf16 = Eu H floats
    w->SJ[1].push_back(b16 && d == 3 ? (__bf16*)A(Eu * H) : nullptr);
    w->Om.push_back(cf.filter_fp32 ? A(2 * Eu * C) : AH(2 * Eu * C));
    w->Y[0].push_back(A(Eu * H));
    w->Y[1].push_back(d == 3 ? A(Eu * H) : nullptr);
    if (cf.n_experts > 0)
      for (int k = 0; k < 2; ++k) { w->Vm[k].push_back(A(B * C * C)); w->VmT[k].push_back(A(B * C * C)); }
    w->a.push_back(A(N * C)); w->q.push_back(A(N * C));
    w->mu_a.push_back(A(N * C)); w->mu_q.push_back(A(N * C)); w->mu_t.push_back(A(N * C));
    w->ad.push_back(A(N * C)); w->qd.push_back(A(N * C));
  }
  for (int l = 0; l <= L; ++l) {
    w->h.push_back(A(N * C)); w->mu_h.push_back(A(N * C)); w->hd.push_back(A(N * C));
  }
  w->lam_h[0] = A(N * C); w->lam_h[1] = A(N * C); w->lam_q = A(N * C); w->lam_a = A(N * C);
  w->y = A(N * C); w->yd = A(N * C); w->lam_y = A(N * C);
  w->eps = A(N); w->Facc = A(3 * N); w->v = A(3 * N); w->Ebar = A(B);
  if (cf.position_grad) {
    w->U2[0] = A(Eu * H);
    if (d == 3) w->U2[1] = A(Eu * H);
    w->Wj = A(2 * Eu * C);
    w->Wpp = A(Eu * C);
    w->gp_acc = A(3 * N);
  }
  // split-k partial sums: the largest weight matrix times its split count
  int64_t cap = 0;
  auto need = [&](int64_t rows, int cols, int64_t R) {
    const bool narrow = cols <= 32;
    int bm = narrow ? 128 : (rows > 64 ? 128 : 64), bn = narrow ? 32 : (rows > 64 ? 128 : 64);
    cap = std::max<int64_t>(cap, (int64_t)pick_splits(rows, cols, R, bm, bn) * rows * cols);
  };
  need(C, H, E); need(H, H, E); need(H, K, E); need(C, C, N);
  cap = std::max<int64_t>(cap, (int64_t)128 * std::max(1, cf.n_species) * C);  // atom-chunk partials
  if (cf.n_experts > 0)  // one weight-gradient partial per structure, plus the split products of the coefficient gradient
    cap = std::max<int64_t>(cap, B * ((int64_t)C * C + 256 * (int64_t)((cf.n_experts + 3) / 4 * 4)));
  if (cf.gemm_dtype == MLIP_GEMM_FP32 && K <= 32) cap = std::max<int64_t>(cap, fold_partial_floats(E, H, K));  // folded first-matrix gradient
  ctx->partial.cap = cap;
  ctx->partial.buf = A(cap);
  if (!ok) return MLIP_E_HIP;
  return MLIP_OK;
}

void inv_free(mlip_ctx* ctx) {
  delete ws_of(ctx);
  ctx->model_ws = nullptr;
}

// TF = storage type of the radial-filter jets: float, or bf16 in bf16 mode unless the context asks for fp32 filters
#define DISPATCH(fn, ...)                                                                                        \
  (ctx->cfg.gemm_dtype == MLIP_GEMM_BF16                                                                         \
       ? (ctx->cfg.filter_fp32 ? fn<gemm::Bf16, float>(__VA_ARGS__) : fn<gemm::Bf16, __bf16>(__VA_ARGS__))       \
       : fn<gemm::Fp32, float>(__VA_ARGS__))

int inv_forward_energy(mlip_ctx* ctx, const float* pos, const int32_t* species, const float* params, const float* h_in,
                         float* E, float* h_out) {
  const bool stage = ctx->cfg.model_kind == MLIP_MODEL_STAGE;
  if (ctx->phase < PH_GRAPH) MLIP_FAIL(ctx, MLIP_E_STATE, "forward_energy: build the graph first");
  if (!pos || !params) MLIP_FAIL(ctx, MLIP_E_INVALID, "forward_energy: null pos or params");
  if (stage ? (!h_in || !h_out) : (!species || !E)) MLIP_FAIL(ctx, MLIP_E_INVALID, "forward_energy: missing tensor for this model kind");
  if (ctx->cfg.n_experts > 0 && ctx->alpha_structs != ctx->B)
    MLIP_FAIL(ctx, MLIP_E_STATE, "forward_energy: set the expert coefficients of this batch's structures first (mlip_set_expert_weights)");
  hipStream_t st = ctx->stream;
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_pos, pos, sizeof(float) * 3 * ctx->N, hipMemcpyDeviceToDevice, st));
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_params, params, sizeof(float) * ctx->n_params, hipMemcpyDeviceToDevice, st));
  if (!stage)
    hipLaunchKernelGGL(k_copy_species, dim3(nblk(ctx->N)), dim3(256), 0, st, species, ctx->N, ctx->cfg.n_species, ctx->d_species, ctx->d_flag);
  MLIP_TRY(DISPATCH(fe_impl, ctx, h_in, E, h_out));
  ctx->phase = PH_FE;
  return MLIP_OK;
}

int inv_forward_force(mlip_ctx* ctx, const float* g_out, float* F, float* g_in) {
  const bool stage = ctx->cfg.model_kind == MLIP_MODEL_STAGE;
  if (ctx->phase < PH_FE) MLIP_FAIL(ctx, MLIP_E_STATE, "forward_force: run forward_energy first");
  if (!F || (stage && (!g_out || !g_in))) MLIP_FAIL(ctx, MLIP_E_INVALID, "forward_force: missing tensor for this model kind");
  MLIP_TRY(DISPATCH(ff_impl, ctx, g_out, F, g_in));
  ctx->phase = PH_FF;
  return MLIP_OK;
}

int inv_loss(mlip_ctx* ctx, const float* E, const float* F, const float* E_ref, const float* F_ref, float* loss,
               float* Ebar, float* v) {
  if (ctx->phase < PH_GRAPH) MLIP_FAIL(ctx, MLIP_E_STATE, "loss: no batch");
  if (!E || !F || !E_ref || !F_ref || !loss || !Ebar || !v) MLIP_FAIL(ctx, MLIP_E_INVALID, "loss: null pointer");
  const int64_t n3 = 3 * ctx->N;
  hipLaunchKernelGGL(k_loss, dim3(1), dim3(1024), 0, ctx->stream, E, E_ref, ctx->B, F, F_ref, n3, ctx->cfg.force_weight, loss);
  hipLaunchKernelGGL(k_loss_cotangents, dim3(nblk(std::max<int64_t>(n3, ctx->B))), dim3(256), 0, ctx->stream, E, E_ref, ctx->B, F,
                     F_ref, n3, ctx->cfg.force_weight, Ebar, v);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

int inv_backward_force(mlip_ctx* ctx, const float* v, const float* hdot_in, float* grad, float* hdot_out) {
  const bool stage = ctx->cfg.model_kind == MLIP_MODEL_STAGE;
  if (ctx->phase < PH_FF) MLIP_FAIL(ctx, MLIP_E_STATE, "backward_force: run forward_force first");
  if (!v || !grad || (stage && !hdot_out)) MLIP_FAIL(ctx, MLIP_E_INVALID, "backward_force: missing tensor for this model kind");
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ws_of(ctx)->v, v, sizeof(float) * 3 * ctx->N, hipMemcpyDeviceToDevice, ctx->stream));
  MLIP_TRY(DISPATCH(bf_impl, ctx, hdot_in, grad, hdot_out));
  ctx->phase = PH_BF;
  return MLIP_OK;
}

int inv_backward_energy(mlip_ctx* ctx, const float* Ebar, const float* lam_out, float* grad, float* lam_in) {
  const bool stage = ctx->cfg.model_kind == MLIP_MODEL_STAGE;
  if (ctx->phase < PH_BF) MLIP_FAIL(ctx, MLIP_E_STATE, "backward_energy: run backward_force first");
  if (!grad || (stage ? (!lam_out || !lam_in) : !Ebar)) MLIP_FAIL(ctx, MLIP_E_INVALID, "backward_energy: missing tensor for this model kind");
  if (!stage) MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ws_of(ctx)->Ebar, Ebar, sizeof(float) * ctx->B, hipMemcpyDeviceToDevice, ctx->stream));
  MLIP_TRY(DISPATCH(be_impl, ctx, lam_out, grad, lam_in));
  ctx->phase = PH_BE;
  return MLIP_OK;
}
