// Kernels and GEMM wrappers shared by the invariant and the equivariant model code.
// Included inside each translation unit's anonymous namespace users: everything here has
// internal linkage.
#pragma once
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "functors.h"
#include "gemm.h"

namespace {

using namespace fx;

__global__ void k_transpose(const float* __restrict__ src, float* __restrict__ dst, int rows, int cols) {
  __shared__ float tile[32][33];
  int c = blockIdx.x * 32 + threadIdx.x;
  for (int r = blockIdx.y * 32 + threadIdx.y; r < min(rows, (int)(blockIdx.y + 1) * 32); r += 8)
    if (c < cols) tile[r - blockIdx.y * 32][threadIdx.x] = src[(int64_t)r * cols + c];
  __syncthreads();
  int r2 = blockIdx.y * 32 + threadIdx.x;
  for (int c2 = blockIdx.x * 32 + threadIdx.y; c2 < min(cols, (int)(blockIdx.x + 1) * 32); c2 += 8)
    if (r2 < rows) dst[(int64_t)c2 * rows + r2] = tile[threadIdx.x][c2 - blockIdx.x * 32];
}

// The context's copy of the species indices, clamped into [0, S): an index outside that range is a
// caller error that must neither read past the embedding table nor pass silently, so it raises a bit
// of the deferred input-diagnostics word.
__global__ void k_copy_species(const int32_t* __restrict__ src, int64_t N, int S, int32_t* __restrict__ dst,
                               int32_t* __restrict__ flag) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  int z = src[i];
  if (z < 0 || z >= S) {
    atomicOr(flag + 1, INPUT_BAD_SPECIES);
    z = z < 0 ? 0 : S - 1;
  }
  dst[i] = z;
}

__global__ void k_embed(const float* __restrict__ emb, const int32_t* __restrict__ species, int64_t N, int C,
                        float* __restrict__ h) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= N * C) return;
  int64_t i = idx / C;
  h[idx] = emb[(int64_t)species[i] * C + (idx % C)];
}

// eps_i = sum_c w_o[c] silu(y[i,c]); one wave per atom, fixed reduction order.
__global__ void __launch_bounds__(256) k_atom_energy(const float* __restrict__ y, const float* __restrict__ wo, int N,
                                                     int C, float* __restrict__ eps) {
  int lane = threadIdx.x & 63;
  int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= N) return;
  float s = 0.f;
  for (int c = lane; c < C; c += 64) s += wo[c] * silu(y[(int64_t)i * C + c]);
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  if (lane == 0) eps[i] = s;
}

__global__ void __launch_bounds__(256) k_struct_sum(const float* __restrict__ eps, const StructMeta* __restrict__ meta,
                                                    float* __restrict__ E) {
  __shared__ float red[256];
  const StructMeta& m = meta[blockIdx.x];
  float s = 0.f;
  for (int i = m.atom_begin + threadIdx.x; i < m.atom_end; i += 256) s += eps[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) E[blockIdx.x] = red[0];
}

// Column sums over atoms in two deterministic stages: part[chunk][c] = sum over the chunk's
// atoms of f(i, c) (64 channels x 4 atom lanes per block), then k_reduce_partials.
// MODE 0: silu'(y) * yd     MODE 1: Ebar[struct(i)] * silu(y)
template <int MODE>
__global__ void __launch_bounds__(256) k_wo_grad(const float* __restrict__ y, const float* __restrict__ yd,
                                                 const float* __restrict__ Ebar, const int32_t* __restrict__ atom_struct,
                                                 int N, int C, int chunk_len, float* __restrict__ part) {
  __shared__ float red[4][64];
  int c = blockIdx.x * 64 + (threadIdx.x & 63);
  int al = threadIdx.x >> 6;
  int i0 = blockIdx.y * chunk_len, i1 = min(N, i0 + chunk_len);
  float s = 0.f;
  if (c < C)
    for (int i = i0 + al; i < i1; i += 4) {
      float yy = y[(int64_t)i * C + c];
      s += (MODE == 0) ? dsilu(yy) * yd[(int64_t)i * C + c] : Ebar[atom_struct[i]] * silu(yy);
    }
  red[al][threadIdx.x & 63] = s;
  __syncthreads();
  if (al == 0 && c < C)
    part[(int64_t)blockIdx.y * C + c] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

__global__ void k_lam_y(const float* __restrict__ y, const float* __restrict__ yd, const float* __restrict__ wo,
                        const float* __restrict__ Ebar, const int32_t* __restrict__ atom_struct, int64_t N, int C,
                        float* __restrict__ lam_y) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= N * C) return;
  int64_t i = idx / C;
  int c = (int)(idx % C);
  float d1, d2;
  dsilu12(y[idx], d1, d2);
  lam_y[idx] = wo[c] * (Ebar[atom_struct[i]] * d1 + d2 * yd[idx]);
}

// part[chunk][z][c] = sum over the chunk's atoms of species z of lam_h0[i][c].
__global__ void __launch_bounds__(256) k_emb_grad(const float* __restrict__ lam_h0, const int32_t* __restrict__ species,
                                                  int N, int C, int S, int chunk_len, float* __restrict__ part) {
  __shared__ float red[4][64];
  int z = blockIdx.z;
  int c = blockIdx.x * 64 + (threadIdx.x & 63);
  int al = threadIdx.x >> 6;
  int i0 = blockIdx.y * chunk_len, i1 = min(N, i0 + chunk_len);
  float s = 0.f;
  if (c < C)
    for (int i = i0 + al; i < i1; i += 4)
      if (species[i] == z) s += lam_h0[(int64_t)i * C + c];
  red[al][threadIdx.x & 63] = s;
  __syncthreads();
  if (al == 0 && c < C)
    part[((int64_t)blockIdx.y * S + z) * C + c] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

__global__ void k_scale3(const float* __restrict__ src, float s, int64_t n, float* __restrict__ dst) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) dst[idx] = s * src[idx];
}

__global__ void k_fill(float* __restrict__ p, float val, int64_t n) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) p[idx] = val;
}

// grad[i] += sum_z part[z][i]: 64 elements x 4 split groups per block, fixed summation order.
__global__ void __launch_bounds__(256) k_reduce_partials(const float* __restrict__ part, int splits, int64_t n,
                                                         float* __restrict__ grad) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, zg = threadIdx.x >> 6;
  const int64_t idx = (int64_t)blockIdx.x * 64 + lane;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (idx < n) {
    int z = zg;
    for (; z + 12 < splits; z += 16) {
      s0 += part[(int64_t)z * n + idx];
      s1 += part[(int64_t)(z + 4) * n + idx];
      s2 += part[(int64_t)(z + 8) * n + idx];
      s3 += part[(int64_t)(z + 12) * n + idx];
    }
    for (; z < splits; z += 4) s0 += part[(int64_t)z * n + idx];
  }
  red[zg][lane] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (zg == 0 && idx < n) grad[idx] += (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

// Loss, one block: deterministic tree.  loss = mean_s (E-Eref)^2 + fw * mean (F-Fref)^2.
__global__ void __launch_bounds__(1024) k_loss(const float* __restrict__ E, const float* __restrict__ Eref, int B,
                                               const float* __restrict__ F, const float* __restrict__ Fref, int64_t n3,
                                               float fw, float* __restrict__ loss) {
  __shared__ float red[1024];
  float se = 0.f, sf = 0.f;
  for (int s = threadIdx.x; s < B; s += 1024) {
    float d = E[s] - Eref[s];
    se += d * d;
  }
  for (int64_t k = threadIdx.x; k < n3; k += 1024) {
    float d = F[k] - Fref[k];
    sf += d * d;
  }
  red[threadIdx.x] = se / (float)B + fw * sf / (float)n3;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = red[0];
}

__global__ void k_loss_cotangents(const float* __restrict__ E, const float* __restrict__ Eref, int B,
                                  const float* __restrict__ F, const float* __restrict__ Fref, int64_t n3, float fw,
                                  float* __restrict__ Ebar, float* __restrict__ v) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < B) Ebar[idx] = 2.f * (E[idx] - Eref[idx]) / (float)B;
  if (idx < n3) v[idx] = -2.f * fw * (F[idx] - Fref[idx]) / (float)n3;
}

// How the activated jets (silu(u), silu'(u) u') of a hidden level reach the GEMMs that consume
// them.  fp32: recomputed from the stored pre-activations while a tile is staged (saves HBM
// traffic; the fp32 matrix cores leave the ALUs idle anyway).  bf16: the producing GEMM's
// epilogue stores them once, already rounded, and the consumers read bf16 (the bf16 matrix cores
// are too fast to hide per-element transcendental work in the operand path).
template <typename P>
struct Act;
template <>
struct Act<gemm::Fp32> {
  typedef LdJetSilu Jet;
  typedef LdJetSiluEven Even;
  typedef LdJetSiluOdd Odd;
  typedef EpiStore Store;
  typedef float xop_t;  // element type of the edge tensors that only feed matrix products
  typedef LdPlain XLd;
  static XLd xld(const xop_t* x, int64_t ld) { return XLd{x, ld}; }
  static LdPairSum xpair(const xop_t* x, int64_t ld) { return LdPairSum{x, ld}; }  // rows 2u, 2u + 1 summed
  static Jet jet(const float* u, const __bf16*, int H) { return Jet{u, H}; }
  static Even even(const float* u, const __bf16*, int H) { return Even{u, H}; }
  static Odd odd(const float* u, const __bf16*, int H) { return Odd{u, H}; }
  static Store store(float* u, __bf16*, int H, int64_t M) { return Store{u, H, M}; }
};
template <>
struct Act<gemm::Bf16> {
  typedef LdBf16 Jet;
  typedef LdBf16 Even;
  typedef LdBf16 Odd;
  typedef EpiStoreJetAct Store;
  typedef __bf16 xop_t;  // rounded once by the producer: half the bytes, no conversion in the operand path
  typedef LdBf16 XLd;
  static XLd xld(const xop_t* x, int64_t ld) { return XLd{x, ld}; }
  static LdBf16Pair xpair(const xop_t* x, int64_t ld) { return LdBf16Pair{x, ld}; }  // rows 2u, 2u + 1 summed
  static Jet jet(const float*, const __bf16* sj, int H) { return Jet{sj, H}; }
  static Even even(const float*, const __bf16* sj, int H) { return Even{sj, 2 * (int64_t)H}; }
  static Odd odd(const float*, const __bf16* sj, int H) { return Odd{sj + H, 2 * (int64_t)H}; }
  static Store store(float* u, __bf16* sj, int H, int64_t M) { return Store{u, sj, H, M}; }
};

// Row-parallel gather kernels: workgroups are dealt round-robin to the 8 XCDs, so XCD x takes
// the x-th contiguous eighth of the row blocks -- consecutive receivers (atoms of one structure,
// spatial neighbours) share senders, and their node-table rows then stay in one XCD's L2.
__device__ __forceinline__ int xcd_block() {
  const int per_xcd = gridDim.x >> 3;  // the grid is a multiple of 8
  return (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
}
inline unsigned nblk8(int64_t n, int b) { return (unsigned)(((n + b - 1) / b + 7) / 8 * 8); }

inline unsigned nblk(int64_t n, int b = 256) { return (unsigned)((n + b - 1) / b); }
inline int atom_chunks(int64_t N) { return (int)std::max<int64_t>(1, std::min<int64_t>(128, N / 32)); }

template <typename T>
T* alloc_n(mlip_ctx* ctx, int64_t n) {
  return (T*)ctx_alloc(ctx, (size_t)std::max<int64_t>(n, 1) * sizeof(T));
}

// ------------------------------------------------------------------------------ GEMM wrappers
// D[M][N] = A[M][K] * W[N][K]^T with loader / epilogue functors; tile chosen from N.
// ---- bf16 mirrors of the weights
__global__ void k_to_bf16(const float* __restrict__ src, __bf16* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (__bf16)src[i];
}
inline bool add_shadow(mlip_ctx* ctx, const float* f32, int64_t n) {
  __bf16* b = (__bf16*)ctx_alloc(ctx, (size_t)std::max<int64_t>(n, 1) * sizeof(__bf16));
  if (!b) return false;
  ctx->shadows.push_back({f32, b, n});
  return true;
}
inline void refresh_shadows(mlip_ctx* ctx) {
  for (const auto& sh : ctx->shadows)
    hipLaunchKernelGGL(k_to_bf16, dim3((unsigned)((sh.n + 255) / 256)), dim3(256), 0, ctx->stream, sh.f32, sh.b16, sh.n);
}
inline const __bf16* shadow_of(const mlip_ctx* ctx, const float* p) {
  for (const auto& sh : ctx->shadows)
    if (p >= sh.f32 && p < sh.f32 + sh.n) return sh.b16 + (p - sh.f32);
  return nullptr;
}

template <typename P, typename LdA, typename LdB, typename Epi>
void gemm_nt_as(hipStream_t st, const LdA& a, const LdB& b, int64_t M, int N, int K, const Epi& epi) {
  const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128);
  // long reductions over raw bf16 operands: 256 x 128 tiles (128 x 64 per wave) stage a third fewer bytes through LDS per
  // matrix instruction (LDS takes 64 bytes per clock in, 256 out, and is what bounds these kernels)
  // (not with a pair-summing A loader: its two raw rows per item do not fit the register budget of that tile)
  if constexpr (P::IS_BF16 && LdA::WIDTH == 8 && LdB::WIDTH == 8 && !std::is_same<LdA, LdBf16x8Pair>::value) {
    if (N % 128 == 0 && K >= 256 && tiles128 >= 2048) return (void)gemm::launch<P, 4, 2, 2, 2, true>(st, a, b, epi, M, N, K, 1);
  }
  if (N > 64 && tiles128 >= 512)
    gemm::launch<P, 2, 2, 2, 2, true>(st, a, b, epi, M, N, K, 1);
  else
    gemm::launch<P, 1, 1, 2, 2, true>(st, a, b, epi, M, N, K, 1);
}
// A bf16 operand is fetched 16 bytes at a time when its leading dimension, its extent along the
// contiguous index and its base address allow it.
template <typename L>
inline bool wide_ok(const L& l, int64_t extent) {
  return l.ld % 8 == 0 && extent % 8 == 0 && (reinterpret_cast<uintptr_t>(l.p) & 15) == 0;
}
// the 16-byte form of a bf16 loader
template <typename L> struct WideOf { static constexpr bool has = false; typedef L type; };
template <> struct WideOf<LdBf16> { static constexpr bool has = true; typedef LdBf16x8 type; };
template <> struct WideOf<LdBf16Pair> { static constexpr bool has = true; typedef LdBf16x8Pair type; };
// D[M][N] = A[M][K] W[N][K]^T through the epilogue.  In bf16 mode the weights come from their
// bf16 mirror when one is registered.
template <typename P, typename LdA, typename Epi>
void gemm_nt(mlip_ctx* ctx, const LdA& a, const float* W, int64_t M, int N, int K, const Epi& epi) {
  hipStream_t st = ctx->stream;
  if constexpr (P::IS_BF16) {
    const __bf16* W16 = shadow_of(ctx, W);
    const bool wb = W16 && wide_ok(LdBf16{W16, K}, K);
    if constexpr (WideOf<LdA>::has) {
      typedef typename WideOf<LdA>::type LdA8;
      if (wide_ok(a, K)) {
        // short reduction, many column tiles: the row-stripe kernel (A staged once per 128 rows)
        if constexpr (std::is_same<LdA, LdBf16>::value) {
          if (wb && (K == 64 || K == 128) && N % 128 == 0 && N >= 256 && M >= 128 * 256 && M % 2 == 0) {
            if (K == 64) return gemm::launch_stripe<64>(st, LdBf16x8{a.p, a.ld}, LdBf16x8{W16, K}, epi, M, N);
            return gemm::launch_stripe<128>(st, LdBf16x8{a.p, a.ld}, LdBf16x8{W16, K}, epi, M, N);
          }
        }
        if (wb) return gemm_nt_as<P>(st, LdA8{a.p, a.ld}, LdBf16x8{W16, K}, M, N, K, epi);
        return gemm_nt_as<P>(st, LdA8{a.p, a.ld}, LdPlain{W, K}, M, N, K, epi);
      }
    }
    if (wb) return gemm_nt_as<P>(st, a, LdBf16x8{W16, K}, M, N, K, epi);
  }
  gemm_nt_as<P>(st, a, LdPlain{W, K}, M, N, K, epi);
}

// part2[g][i] = sum of part[z][i] over the g-th of G contiguous ranges of z (fixed order)
__global__ void __launch_bounds__(256) k_reduce_ranges(const float* __restrict__ part, int splits, int64_t n, int G,
                                                       float* __restrict__ part2) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int gi = blockIdx.y;
  if (idx >= n) return;
  const int per = (splits + G - 1) / G;
  const int z0 = gi * per, z1 = min(splits, z0 + per);
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int z = z0;
  for (; z + 3 < z1; z += 4) {
    s0 += part[(int64_t)z * n + idx];
    s1 += part[(int64_t)(z + 1) * n + idx];
    s2 += part[(int64_t)(z + 2) * n + idx];
    s3 += part[(int64_t)(z + 3) * n + idx];
  }
  for (; z < z1; ++z) s0 += part[(int64_t)z * n + idx];
  part2[(int64_t)gi * n + idx] = (s0 + s1) + (s2 + s3);
}

// Floats of partial-sum space a folded product over R rows with N x Kb outputs needs (row tiles of
// 64 in the worst case, plus the second reduction stage).
constexpr int FOLD_GROUPS = 64;
inline int64_t fold_partial_floats(int64_t R, int N, int Kb) { return ((R + 63) / 64 + FOLD_GROUPS) * (int64_t)N * Kb; }
inline bool fold_ok(const mlip_ctx* ctx, int64_t R, int N, int Kb) {
  return Kb <= 32 && fold_partial_floats(R, N, Kb) <= ctx->partial.cap;
}

// D = A W^T through a folding epilogue (fp32 products): besides D's element-wise consumers, the
// product Z^T B of the epilogue's tile values with the narrow matrix B is accumulated per row tile
// and added to gradB[N][Kb].  The functor's FoldB.part is pointed at the context's partial buffer.
template <typename P, typename LdA, typename Epi>
void gemm_nt_fold(mlip_ctx* ctx, const LdA& a, const float* W, int64_t M, int N, int K, Epi epi, float* gradB) {
  static_assert(!P::IS_BF16, "folding epilogues are fp32 products");
  hipStream_t st = ctx->stream;
  epi.f.part = ctx->partial.buf;
  const int Kb = epi.f.K;
  const int64_t tiles128 = ((M + 127) / 128) * ((N + 127) / 128);
  int64_t tiles_m;
  if (N > 64 && tiles128 >= 512) {
    gemm::launch<P, 2, 2, 2, 2, true>(st, a, LdPlain{W, K}, epi, M, N, K, 1);
    tiles_m = (M + 127) / 128;
  } else {
    gemm::launch<P, 1, 1, 2, 2, true>(st, a, LdPlain{W, K}, epi, M, N, K, 1);
    tiles_m = (M + 63) / 64;
  }
  const int64_t n = (int64_t)N * Kb;
  if (tiles_m > 4 * FOLD_GROUPS) {  // two stages, so that the reduction has enough workgroups
    float* part2 = ctx->partial.buf + tiles_m * n;
    hipLaunchKernelGGL(k_reduce_ranges, dim3(nblk(n), FOLD_GROUPS), dim3(256), 0, st, ctx->partial.buf, (int)tiles_m, n, FOLD_GROUPS, part2);
    hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(n, 64)), dim3(256), 0, st, part2, FOLD_GROUPS, n, gradB);
  } else {
    hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(n, 64)), dim3(256), 0, st, ctx->partial.buf, (int)tiles_m, n, gradB);
  }
}

int pick_splits(int64_t rows_out, int cols_out, int64_t K, int bm, int bn) {
  int64_t tiles = ((rows_out + bm - 1) / bm) * ((cols_out + bn - 1) / bn);
  // 512 workgroups = one resident round of this kernel (two per compute unit); more leave a partly filled second round
  int64_t s = std::max<int64_t>(1, 512 / tiles);
  s = std::min<int64_t>(s, std::max<int64_t>(1, K / 64));
  return (int)std::min<int64_t>(s, 512);
}

// grad[Nout][Kout] += A^T B, A [R][Nout], B [R][Kout] given by loaders (reduction over R rows).
template <typename P, typename LdA, typename LdB>
int gemm_wgrad_as(mlip_ctx* ctx, const LdA& a, const LdB& b, int64_t R, int Nout, int Kout, float* grad) {
  const PartialBuf* w = &ctx->partial;
  hipStream_t st = ctx->stream;
  if (R <= 0) return MLIP_OK;
  const bool narrow = Kout <= 32;
  const int bm = narrow ? 128 : (Nout > 64 ? 128 : 64), bn = narrow ? 32 : (Nout > 64 ? 128 : 64);
  int splits = pick_splits(Nout, Kout, R, bm, bn);
  while ((int64_t)splits * Nout * Kout > w->cap && splits > 1) --splits;
  EpiPartial epi{w->buf, Kout, Nout};
  if (narrow)
    splits = gemm::launch<P, 1, 1, 4, 1, false>(st, a, b, epi, Nout, Kout, R, splits);
  else if (Nout > 64)
    splits = gemm::launch<P, 2, 2, 2, 2, false>(st, a, b, epi, Nout, Kout, R, splits);
  else
    splits = gemm::launch<P, 1, 1, 2, 2, false>(st, a, b, epi, Nout, Kout, R, splits);
  int64_t n = (int64_t)Nout * Kout;
  hipLaunchKernelGGL(k_reduce_partials, dim3(nblk(n, 64)), dim3(256), 0, st, w->buf, splits, n, grad);
  return MLIP_OK;
}


template <typename P, typename LdA, typename LdB>
int gemm_wgrad(mlip_ctx* ctx, const LdA& a, const LdB& b, int64_t R, int Nout, int Kout, float* grad) {
  constexpr bool A16 = WideOf<LdA>::has, B16 = WideOf<LdB>::has;
  typedef typename WideOf<LdA>::type LdA8;
  typedef typename WideOf<LdB>::type LdB8;
  bool wa = false, wb = false;
  if constexpr (A16) wa = wide_ok(a, Nout);
  if constexpr (B16) wb = wide_ok(b, Kout);
  if constexpr (A16 && B16) {
    if (wa && wb) return gemm_wgrad_as<P>(ctx, LdA8{a.p, a.ld}, LdB8{b.p, b.ld}, R, Nout, Kout, grad);
  }
  if constexpr (A16) {
    if (wa) return gemm_wgrad_as<P>(ctx, LdA8{a.p, a.ld}, b, R, Nout, Kout, grad);
  }
  if constexpr (B16) {
    if (wb) return gemm_wgrad_as<P>(ctx, a, LdB8{b.p, b.ld}, R, Nout, Kout, grad);
  }
  return gemm_wgrad_as<P>(ctx, a, b, R, Nout, Kout, grad);
}

// ---- mixture of linear experts (Sec. 5.1 "Models"): the expert matrices of a bank are averaged
// per structure into one temporary matrix, W_s = sum_k alpha[s][k] W_k, which is then used like
// any dense matrix on the atoms of s.
// Wm[s][i] and its transpose WmT[s][(i % C) * C + i / C], i < C*C.  Block: 64 entries x 16 structures;
// the experts are dealt to four groups of 64 threads (independent load streams), whose sums are
// combined in a fixed order.
__global__ void __launch_bounds__(256) k_merge_experts(const float* __restrict__ alpha, const float* __restrict__ bank,
                                                       int B, int Ke, int C, float* __restrict__ Wm,
                                                       float* __restrict__ WmT) {
  __shared__ float al[16][64];
  __shared__ float red[3][16][64];
  const int lane = threadIdx.x & 63, kg = threadIdx.x >> 6;
  const int64_t n = (int64_t)C * C, i = (int64_t)blockIdx.x * 64 + lane;
  const int s0 = blockIdx.y * 16;
  float acc[16];
#pragma unroll
  for (int ss = 0; ss < 16; ++ss) acc[ss] = 0.f;
  for (int k0 = 0; k0 < Ke; k0 += 64) {
    __syncthreads();
    for (int q = threadIdx.x; q < 16 * 64; q += 256) {
      const int ss = q / 64, kk = q % 64;
      al[ss][kk] = (s0 + ss < B && k0 + kk < Ke) ? alpha[(int64_t)(s0 + ss) * Ke + k0 + kk] : 0.f;
    }
    __syncthreads();
    if (i < n) {
      const int kn = min(64, Ke - k0);
#pragma unroll 4
      for (int kk = kg; kk < kn; kk += 4) {
        const float v = bank[(int64_t)(k0 + kk) * n + i];
#pragma unroll
        for (int ss = 0; ss < 16; ++ss) acc[ss] = fmaf(al[ss][kk], v, acc[ss]);
      }
    }
  }
  if (kg > 0) {
#pragma unroll
    for (int ss = 0; ss < 16; ++ss) red[kg - 1][ss][lane] = acc[ss];
  }
  __syncthreads();
  if (kg == 0 && i < n) {
    const int64_t it = (i % C) * C + i / C;
#pragma unroll
    for (int ss = 0; ss < 16; ++ss)
      if (s0 + ss < B) {
        const float v = (acc[ss] + red[0][ss][lane]) + (red[1][ss][lane] + red[2][ss][lane]);
        Wm[(int64_t)(s0 + ss) * n + i] = v;
        WmT[(int64_t)(s0 + ss) * n + it] = v;
      }
  }
}

// grad_bank[k][i] += sum_s alpha[s][k] part[s][i]  (structures in order: deterministic).
// Block: 256 entries x 16 experts.
// part holds `copies` blocks of B partials (block m = component copy m of the atom rows); partial
// z belongs to structure z % B.
__global__ void __launch_bounds__(256) k_expert_grad(const float* __restrict__ alpha, const float* __restrict__ part, int B,
                                                     int copies, int Ke, int64_t n, float* __restrict__ grad_bank) {
  __shared__ float al[64][16];
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int k0 = blockIdx.y * 16;
  float acc[16];
#pragma unroll
  for (int kk = 0; kk < 16; ++kk) acc[kk] = 0.f;
  const int Z = B * copies;
  for (int s0 = 0; s0 < Z; s0 += 64) {
    __syncthreads();
    for (int q = threadIdx.x; q < 64 * 16; q += 256) {
      const int ss = q / 16, kk = q % 16;
      al[ss][kk] = (s0 + ss < Z && k0 + kk < Ke) ? alpha[(int64_t)((s0 + ss) % B) * Ke + k0 + kk] : 0.f;
    }
    __syncthreads();
    if (i < n) {
      const int sn = min(64, Z - s0);
      for (int ss = 0; ss < sn; ++ss) {
        const float p = part[(int64_t)(s0 + ss) * n + i];
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) acc[kk] = fmaf(al[ss][kk], p, acc[kk]);
      }
    }
  }
  if (i < n) {
#pragma unroll
    for (int kk = 0; kk < 16; ++kk)
      if (k0 + kk < Ke) grad_bank[(int64_t)(k0 + kk) * n + i] += acc[kk];
  }
}

// Coefficient gradient, last step: grad_alpha[s][k] += sum_z part2[z][s][k] (z runs over k-splits and
// component copies); part2 rows are padded to ldp columns.  64 entries x 4 groups of z per block, four
// independent running sums per thread, combined in a fixed order.
__global__ void __launch_bounds__(256) k_alpha_reduce(const float* __restrict__ part2, int Z, int B, int Ke, int ldp,
                                                      float* __restrict__ grad_alpha) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, zg = threadIdx.x >> 6;
  const int idx = blockIdx.x * 64 + lane;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (idx < B * Ke) {
    const int64_t base = (int64_t)(idx / Ke) * ldp + idx % Ke, stride = (int64_t)B * ldp;
    int z = zg;
    for (; z + 12 < Z; z += 16) {
      s0 += part2[z * stride + base];
      s1 += part2[(z + 4) * stride + base];
      s2 += part2[(z + 8) * stride + base];
      s3 += part2[(z + 12) * stride + base];
    }
    for (; z < Z; z += 4) s0 += part2[z * stride + base];
  }
  red[zg][lane] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (zg == 0 && idx < B * Ke) grad_alpha[idx] += (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

// D = A W_s^T with the merged matrix of each row's structure (Wm [B][N*K]); 64-row tiles that end
// with their structure (the context's row-group table).  copies: A stacks that many copies of the
// atom rows (the 2l+1 components of an equivariant block), M = copies * N_atoms.
template <typename P, typename LdA, typename Epi>
void gemm_nt_grouped(mlip_ctx* ctx, const LdA& a, const float* Wm, int64_t M, int N, int K, const Epi& epi, int copies = 1) {
  gemm::Groups g;
  g.row_groups = ctx->d_row_groups;
  g.n_row_tiles = ctx->n_row_groups * copies;
  g.b_stride = (int64_t)N * K;
  gemm::launch<P, 1, 1, 2, 2, true>(ctx->stream, a, LdPlain{Wm, K}, epi, M, N, K, 1, g);
}
// Expert-bank gradient: one weight-gradient partial per structure (split z = structure z's
// atoms), then grad_bank[k] += sum_s alpha[s][k] partial[s].
// bank: the expert matrices themselves (for the coefficient gradient, when the caller asked for it).
template <typename P, typename LdA, typename LdB>
int gemm_wgrad_experts(mlip_ctx* ctx, const LdA& a, const LdB& b, int64_t R, int Nout, int Kout, float* grad_bank,
                       const float* bank, int copies = 1) {
  const int B = ctx->B, Ke = ctx->cfg.n_experts;
  const int64_t n = (int64_t)Nout * Kout;
  if (R <= 0 || B <= 0) return MLIP_OK;
  if ((int64_t)B * copies * n > ctx->partial.cap) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "expert gradient: partial buffer too small");
  gemm::Groups g;
  g.k_ranges = ctx->d_struct_ptr;
  EpiPartial epi{ctx->partial.buf, Kout, Nout};
  if (Nout > 64)
    gemm::launch<P, 2, 2, 2, 2, false>(ctx->stream, a, b, epi, Nout, Kout, R, B * copies, g);
  else
    gemm::launch<P, 1, 1, 2, 2, false>(ctx->stream, a, b, epi, Nout, Kout, R, B * copies, g);
  hipLaunchKernelGGL(k_expert_grad, dim3(nblk(n), (Ke + 15) / 16), dim3(256), 0, ctx->stream, ctx->d_alpha, ctx->partial.buf, B,
                     copies, Ke, n, grad_bank);
  if (ctx->d_grad_alpha) {
    if (ctx->grad_alpha_structs < B) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "coefficient gradient: the registered buffer holds fewer rows than the batch has structures");
    // dL/dalpha[s][k] = sum over copies of <partial[m B + s], W_k>: the product [B copies, n] x [Ke, n]^T over
    // the n matrix entries, split along n; always in fp32 (it is tiny)
    const int ldp = (Ke + 3) / 4 * 4;
    const int64_t rows = (int64_t)B * copies;
    const int splits = (int)std::min<int64_t>(128, std::max<int64_t>(1, n / 64));
    float* part2 = ctx->partial.buf + rows * n;
    if (rows * n + (int64_t)splits * rows * ldp > ctx->partial.cap) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "coefficient gradient: partial buffer too small");
    const int used = gemm::launch<gemm::Fp32, 1, 1, 2, 2, true>(ctx->stream, LdPlain{ctx->partial.buf, n}, LdPlain{bank, n},
                                                                EpiPartial{part2, ldp, rows}, rows, Ke, n, splits);
    // part2 is [split][copy][structure][ldp]: splits and copies are summed together
    hipLaunchKernelGGL(k_alpha_reduce, dim3(nblk((int64_t)B * Ke, 64)), dim3(256), 0, ctx->stream, part2, used * copies, B, Ke, ldp, ctx->d_grad_alpha);
  }
  return MLIP_OK;
}

// Edge geometry and featurisation: unit vector, length, Gaussian basis jets, envelope jet.
// A thread writes four consecutive basis functions of one edge (16-byte stores); an edge takes
// 2^qshift >= K/4 threads, so edge and quad indices come from shifts, not divisions.
__global__ void __launch_bounds__(256) k_edge_features(const float* __restrict__ pos, const int32_t* __restrict__ sender,
                                                       const int32_t* __restrict__ receiver, const int32_t* __restrict__ code,
                                                       const int32_t* __restrict__ atom_struct, const StructMeta* __restrict__ meta,
                                                       const int2* __restrict__ se,
                                                       int64_t E, int K, int qshift, float rc, float4* __restrict__ geo,
                                                       float2* __restrict__ env, float2* __restrict__ env_u, float* __restrict__ jphi,
                                                       int32_t* __restrict__ flag) {
  const int q = threadIdx.x & ((1 << qshift) - 1);
  const int64_t e = (int64_t)blockIdx.x * (256 >> qshift) + (threadIdx.x >> qshift);
  if (e >= E || 4 * q >= K) return;
  int i = receiver[e], j = sender[e], c = code[e];
  const StructMeta& m = meta[atom_struct[i]];
  // image shift S . cell (rows = lattice vectors); zero for a molecule, S_a L_a for a diagonal cell
  const float Sx = (float)(c / 9 - 1), Sy = (float)((c / 3) % 3 - 1), Sz = (float)(c % 3 - 1);
  float sx = (Sx * m.lat[0] + Sy * m.lat[3]) + Sz * m.lat[6];
  float sy = (Sx * m.lat[1] + Sy * m.lat[4]) + Sz * m.lat[7];
  float sz = (Sx * m.lat[2] + Sy * m.lat[5]) + Sz * m.lat[8];
  float dx = (pos[3 * j] - pos[3 * i]) + sx;
  float dy = (pos[3 * j + 1] - pos[3 * i + 1]) + sy;
  float dz = (pos[3 * j + 2] - pos[3 * i + 2]) + sz;
  float r = sqrtf(dx * dx + dy * dy + dz * dz);
  float dmu = rc / (float)(K - 1);
  float gamma = 0.5f / (dmu * dmu);
  float p[4], d[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    float t = r - (float)(4 * q + u) * dmu;
    p[u] = expf(-gamma * t * t);
    d[u] = -2.f * gamma * t * p[u];
  }
  // the radial basis is kept once per edge pair (both edges have the same length, bit for bit: the opposite edge's
  // difference vector is the exact negative): the pair's lower-numbered edge writes rows 2u, 2u + 1
  const int slot = se[e].y;
  if (!(slot & 1)) {
    *reinterpret_cast<float4*>(jphi + (int64_t)slot * K + 4 * q) = make_float4(p[0], p[1], p[2], p[3]);
    *reinterpret_cast<float4*>(jphi + (int64_t)(slot + 1) * K + 4 * q) = make_float4(d[0], d[1], d[2], d[3]);
  }
  if (q == 0) {
    // two atoms at one place have no direction: report it (deferred input diagnostics) and keep the numbers finite
    if (!(r > 0.f)) atomicOr(flag + 1, INPUT_COINCIDENT);
    float inv = r > 0.f ? 1.f / r : 0.f;
    geo[e] = make_float4(dx * inv, dy * inv, dz * inv, r);
    float w = 3.14159265358979323846f / rc;
    float sn, cs;
    sincosf(w * r, &sn, &cs);
    env[e] = make_float2(0.5f * (1.f + cs), -0.5f * w * sn);
    if (!(slot & 1)) env_u[slot >> 1] = make_float2(0.5f * (1.f + cs), -0.5f * w * sn);
  }
}

// geo[E], env[E] per edge; env_u[Eu], jphi[Eu][2][K] per edge pair
inline void launch_edge_features(mlip_ctx* ctx, int64_t E, int K, float rc, float2* env, float2* env_u, float* jphi) {
  int qshift = 0;
  while ((4 << qshift) < K) ++qshift;  // 2^qshift threads per edge, K <= 1024
  const int64_t per_block = 256 >> qshift;
  hipLaunchKernelGGL(k_edge_features, dim3((unsigned)((E + per_block - 1) / per_block)), dim3(256), 0, ctx->stream, ctx->d_pos,
                     ctx->d_sender, ctx->d_receiver, ctx->d_code, ctx->d_atom_struct, ctx->d_meta, ctx->d_se, E, K, qshift, rc, ctx->d_geo, env, env_u, jphi, ctx->d_flag);
}


}  // namespace
