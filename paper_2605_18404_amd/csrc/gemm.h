// MFMA GEMM template for gfx950 with functor operand loaders and epilogues.
//
//   D(m, n) = sum_k A(m, k) * B(n, k)
//
// The operands are not plain arrays but functors, so element-wise producers (activation, jets,
// products with saved tensors) are evaluated while a tile is staged into LDS and never written
// to HBM.  A loader has two halves:  Raw fetch(row, col4)  issues the loads of four consecutive
// values only, and  float4 finish(raw)  applies the element-wise function when the stage is
// written to LDS -- so the loads of the next stage stay in flight during the matrix products.
// Two orientations exist per operand:
//   k-contiguous (KC): fetch(row, k4) -> A(row, k4 .. k4+3)     -- forward / data-gradient
//   k-strided    (KS): fetch(k, row4) -> A(row4 .. row4+3, k)   -- weight gradients, where the
//                      reduction index is the row (edge or atom) of both stored operands.
// Precision policies:
//   Fp32: v_mfma_f32_32x32x2_f32; LDS stage k-major [BK][rows+4] (fragment = one float).
//   Bf16: v_mfma_f32_32x32x16_bf16; operands rounded to bf16 (nearest even) while staged, fp32
//         accumulate.  KC: LDS stage row-major [rows][BK+8] (fragment = one 16-byte read of 8
//         consecutive k).  KS: k-major [BK][rows+16], fragment = two transposing 8-byte reads.
//
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace gemm {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// ds_read_b64_tr_b16: 8 bytes per lane, exchanged inside groups of 16 lanes (see its use below).
__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)p);
}

struct Fp32 {
  typedef float lds_t;
  static constexpr bool IS_BF16 = false;
  static constexpr int BK_BIG = 16;
  static constexpr int WAVES = 3;  // workgroups (= waves per SIMD) the register budget is set for
};
struct Bf16 {
  typedef __bf16 lds_t;
  static constexpr bool IS_BF16 = true;
  static constexpr int BK_BIG = 32;
  static constexpr int WAVES = 3;
};

template <typename P, int ROWS, int BK, bool KC>
struct Tile {
  // k-major unless bf16 with k-contiguous operands
  static constexpr bool K_MAJOR = !(P::IS_BF16 && KC);
  // bf16 k-major: the row pitch is 8 dwords more than a multiple of 32, so the four k rows that one
  // transposed read touches (16 lanes x 8 bytes) fall into 16 distinct pairs of banks
  static constexpr int PAD = P::IS_BF16 ? (K_MAJOR ? 16 : 8) : 4;
  static constexpr int LD = K_MAJOR ? (ROWS + PAD) : (BK + PAD);
  static constexpr int SIZE = K_MAJOR ? (BK * LD) : (ROWS * LD);
};

// ---- staging: global (through the loader functor) -> registers -> LDS ------------------------
// A loader has WIDTH = 4 (float4 items, converted while staged) or 8 (raw bf16, copied as is).
// A loader with PAIRED = true (k-contiguous only) produces rows 2e and 2e+1 of a jet together:
// Raw fetch(row_even, col4), void finish(raw, float4& even, float4& odd) -- one set of loads and
// one evaluation of the shared sub-expressions for both rows.
template <typename P, int ROWS, int BK, bool KC, typename Ld>
struct Stager {
  typedef Tile<P, ROWS, BK, KC> TL;
  static constexpr bool PR = Ld::PAIRED;
  static_assert(!PR || KC, "paired loaders are k-contiguous");
  static constexpr int RPI = PR ? 2 : 1;             // rows per item
  static constexpr int VW = Ld::WIDTH;               // values per item along the contiguous index
  static_assert(VW == 4 || (VW == 8 && P::IS_BF16 && !PR), "eight-wide items are raw bf16");
  static constexpr int NVT = ROWS / RPI * BK / VW;   // items per stage (two rows each if paired)
  static constexpr int NV = (NVT + 255) / 256;       // per thread
  static constexpr int Q = KC ? (BK / VW) : (ROWS / VW);
  typename Ld::Raw v[NV];
  unsigned ok = 0;

  // KC: a row holds Q = BK/4 float4;     idx -> (row = RPI * (idx / Q), kq = idx % Q)
  // KS: a k-row holds Q = ROWS/4 float4; idx -> (k = idx / Q,  rq = idx % Q)
  // Loads are unconditional: out-of-range coordinates are clamped to a valid element and the
  // value is discarded when the stage is written (no divergent branches around memory ops).
  // FULL: the caller guarantees that the whole stage lies inside the matrix (interior tile, reduction
  // length a multiple of BK): no clamping, no validity mask -- vector instructions saved here are
  // issue slots returned to the matrix pipeline.
  template <bool FULL>
  __device__ __forceinline__ void load(const Ld& ld, int64_t row0, int64_t n_rows, int64_t k0, int64_t k_end, int t) {
    ok = 0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = t + it * 256;
      if (NVT % 256 == 0 || idx < NVT) {
        int64_t r, c;
        bool in = true;
        if (KC) {
          r = row0 + RPI * (idx / Q); c = k0 + VW * (idx % Q);
          if (!FULL) {
            in = r < n_rows && c < k_end;
            r = r < n_rows ? r : n_rows - RPI;  // paired: the row count is even
            c = c < k_end ? c : k_end - VW;
          }
        } else {
          r = k0 + idx / Q; c = row0 + VW * (idx % Q);
          if (!FULL) {
            in = c < n_rows && r < k_end;
            r = r < k_end ? r : k_end - 1;
            c = c < n_rows ? c : n_rows - VW;
          }
        }
        v[it] = ld.fetch(r, c);
        if (!FULL) ok |= (in ? 1u : 0u) << it;
      }
    }
  }

  template <bool FULL>
  __device__ __forceinline__ void store(const Ld& ld, typename P::lds_t* s, int t) const {
    constexpr int LD = TL::LD;
    typedef typename P::lds_t T;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const int idx = t + it * 256;
      if (NVT % 256 != 0 && idx >= NVT) continue;
      const int a = idx / Q, b = idx % Q;  // KC: (row or row pair, kq); KS: (k, rq)
      if constexpr (VW == 8) {  // raw bf16, KC [row][k] or KS [k][row]: one 16-byte store, no conversion
        bf16x8 x = ld.finish(v[it]);
        if (!FULL && !((ok >> it) & 1u)) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        *reinterpret_cast<bf16x8*>(reinterpret_cast<__bf16*>(s) + a * LD + 8 * b) = x;
      } else if constexpr (PR) {
        float4 x, y;
        ld.finish(v[it], x, y);
        if (!FULL && !((ok >> it) & 1u)) x = y = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (TL::K_MAJOR) {  // fp32 [k][row]: rows 2a, 2a+1 are neighbours -> 8-byte stores
          float* f = reinterpret_cast<float*>(s);
          *reinterpret_cast<float2*>(f + (4 * b + 0) * LD + 2 * a) = make_float2(x.x, y.x);
          *reinterpret_cast<float2*>(f + (4 * b + 1) * LD + 2 * a) = make_float2(x.y, y.y);
          *reinterpret_cast<float2*>(f + (4 * b + 2) * LD + 2 * a) = make_float2(x.z, y.z);
          *reinterpret_cast<float2*>(f + (4 * b + 3) * LD + 2 * a) = make_float2(x.w, y.w);
        } else {  // bf16 [row][k]
          bf16x4 p0 = {(__bf16)x.x, (__bf16)x.y, (__bf16)x.z, (__bf16)x.w};
          bf16x4 p1 = {(__bf16)y.x, (__bf16)y.y, (__bf16)y.z, (__bf16)y.w};
          *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(s) + (2 * a) * LD + 4 * b) = p0;
          *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(s) + (2 * a + 1) * LD + 4 * b) = p1;
        }
      } else {
        float4 x = ld.finish(v[it]);
        if (!FULL && !((ok >> it) & 1u)) x = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (KC && TL::K_MAJOR) {  // fp32: transpose into [k][row]
          s[(4 * b + 0) * LD + a] = (T)x.x;
          s[(4 * b + 1) * LD + a] = (T)x.y;
          s[(4 * b + 2) * LD + a] = (T)x.z;
          s[(4 * b + 3) * LD + a] = (T)x.w;
        } else if constexpr (P::IS_BF16) {  // KC [row][k] or KS [k][row]: 4 values = one 8-byte store
          bf16x4 p = {(__bf16)x.x, (__bf16)x.y, (__bf16)x.z, (__bf16)x.w};
          *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(s) + a * LD + 4 * b) = p;
        } else {  // KS fp32 [k][row]: one 16-byte store
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(s) + a * LD + 4 * b) = x;
        }
      }
    }
  }
};

// Epilogue functors with loads declare them apart from their stores: a type In, fetch<FULL>(row, col) returning the
// values rows row, row + 1 need (FULL: row + 1 exists) and apply<FULL>(row, col, a, b, z, in).  Functors without loads
// are called as they are.
template <typename Epi, typename = void>
struct EpiIO {
  struct In {};
  template <bool FULL>
  __device__ static __forceinline__ In fetch(const Epi&, int64_t, int) { return In{}; }
  template <bool FULL>
  __device__ static __forceinline__ void apply(const Epi& e, int64_t r, int col, const float4& a, const float4& b, int z, const In&) { e(r, col, a, b, z); }
};
template <typename Epi>
struct EpiIO<Epi, std::void_t<typename Epi::In>> {
  typedef typename Epi::In In;
  template <bool FULL>
  __device__ static __forceinline__ In fetch(const Epi& e, int64_t r, int col) { return e.template fetch<FULL>(r, col); }
  template <bool FULL>
  __device__ static __forceinline__ void apply(const Epi& e, int64_t r, int col, const float4& a, const float4& b, int z, const In& in) { e.template apply<FULL>(r, col, a, b, z, in); }
};

// ---- the kernel -----------------------------------------------------------------------------
// Epi: void operator()(int64_t row, int col, float4 a, float4 b, int z) const  -- columns col..col+3
// of rows row (even, < M) and row + 1 (the functor checks row + 1 < M), z = split index.
//
// One output tile per workgroup, LDS double buffer, one barrier per k-tile; several workgroups
// per compute unit hide each other's global-load latency.  Workgroups are dealt round-robin to
// the 8 XCDs (each with its own L2): a group is one (row tile, k split), its column tiles go to
// the same XCD one after the other, so the A rows are fetched into one L2 only.
// Optional structure-wise variants (all pointers null = plain product):
//   row_groups  (k-contiguous products): row tile t covers rows [row_groups[t].x, row_groups[t].y) of
//               one group (a structure) and multiplies by that group's own B matrix, found
//               b_stride elements further per group index row_groups[t].z; n_row_tiles entries.
//   k_ranges    (k-strided products, one split per group): split z reduces over rows
//               [k_ranges[z], k_ranges[z+1]); an empty range yields a zero partial.
struct Groups {
  const int4* row_groups = nullptr;
  int64_t n_row_tiles = 0;
  int64_t b_stride = 0;
  const int32_t* k_ranges = nullptr;
};

template <typename P, int TM, int TN, int WM, int WN, bool KC, int BK, typename LdA, typename LdB, typename Epi>
__global__ void __launch_bounds__(256, (TM * TN >= 8 ? 2 : P::WAVES))
k_gemm(LdA lda, LdB ldb, Epi epi, int64_t M_all, int N, int64_t K, int64_t k_chunk, int splits, Groups grp) {
  static_assert(WM * WN == 4, "four waves per workgroup");
  constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
  typedef typename P::lds_t lds_t;
  typedef Tile<P, BM, BK, KC> TA;
  typedef Tile<P, BN, BK, KC> TB;
  constexpr int LDA = TA::LD, LDB = TB::LD;
  // operand stages (two of each) and, after the k loop, the per-wave output slabs share one array
  constexpr int EW = 32 * TN, ELD = EW + 4;  // a wave's output slab: 32 rows x EW columns, padded
  constexpr int STAGE_BYTES = 2 * (TA::SIZE + TB::SIZE) * (int)sizeof(lds_t);
  constexpr int SLAB_BYTES = 4 * 32 * ELD * (int)sizeof(float);
  __shared__ __attribute__((aligned(16))) char smem[STAGE_BYTES > SLAB_BYTES ? STAGE_BYTES : SLAB_BYTES];
  lds_t(*sA)[TA::SIZE] = reinterpret_cast<lds_t(*)[TA::SIZE]>(smem);
  lds_t(*sB)[TB::SIZE] = reinterpret_cast<lds_t(*)[TB::SIZE]>(smem + 2 * TA::SIZE * sizeof(lds_t));

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int li = lane & 31, g = lane >> 5;
  const int tiles_n = (N + BN - 1) / BN;
  const int64_t tiles_m = grp.row_groups ? grp.n_row_tiles : (M_all + BM - 1) / BM;
  const int64_t local = blockIdx.x >> 3;
  const int64_t group = (local / tiles_n) * 8 + (blockIdx.x & 7);
  if (group >= tiles_m * splits) return;  // uniform for the workgroup, before any barrier
  const int z = (int)(group / tiles_m);
  int64_t m0 = (group % tiles_m) * BM, M = M_all;
  if (grp.row_groups) {  // this tile's rows end with its structure; its B matrix is the structure's
    const int4 rg = grp.row_groups[group % tiles_m];
    m0 = rg.x;
    M = rg.y;
    epi.M = M;  // the functor's own bound for the second row of a pair is the tile's, too
    ldb.shift((int64_t)rg.z * grp.b_stride);
  }
  const int n0 = (int)(local % tiles_n) * BN;
  int64_t kb = (int64_t)z * k_chunk;
  int64_t ke = (kb + k_chunk < K) ? kb + k_chunk : K;
  if (grp.k_ranges) {
    kb = grp.k_ranges[z];
    ke = grp.k_ranges[z + 1];
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  Stager<P, BM, BK, KC, LdA> stA;
  Stager<P, BN, BK, KC, LdB> stB;
  const int64_t nk = (ke - kb + BK - 1) / BK;  // >= 1 except for an empty k range (then the tile is zero)
  // interior tile with whole k-tiles: the stages need neither clamping nor masking (uniform choice)
  const bool full = (m0 + BM <= M) && (n0 + BN <= N) && ((ke - kb) % BK == 0);
  auto fetch_stage = [&](int64_t k0) {
    if (full) {
      stA.template load<true>(lda, m0, M, k0, ke, t);
      stB.template load<true>(ldb, n0, N, k0, ke, t);
    } else {
      stA.template load<false>(lda, m0, M, k0, ke, t);
      stB.template load<false>(ldb, n0, N, k0, ke, t);
    }
  };
  auto write_stage = [&](int buf) {
    if (full) {
      stA.template store<true>(lda, sA[buf], t);
      stB.template store<true>(ldb, sB[buf], t);
    } else {
      stA.template store<false>(lda, sA[buf], t);
      stB.template store<false>(ldb, sB[buf], t);
    }
  };
  if (nk > 0) {  // uniform for the workgroup
    fetch_stage(kb);
    write_stage(0);
  }
  __syncthreads();
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int cur = (int)(kt & 1);
    if (kt + 1 < nk) fetch_stage(kb + (kt + 1) * BK);
    const lds_t* a_s = sA[cur];
    const lds_t* b_s = sB[cur];
    if constexpr (!P::IS_BF16) {
      // fragments of step kk+1 are read from LDS before the products of step kk are issued, so the
      // LDS latency hides behind the matrix pipeline instead of stalling the wave every step
      float af[2][TM], bf[2][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[0][i] = a_s[g * LDA + (wm * TM + i) * 32 + li];
#pragma unroll
      for (int j = 0; j < TN; ++j) bf[0][j] = b_s[g * LDB + (wn * TN + j) * 32 + li];
#pragma unroll
      for (int kk = 0; kk < BK / 2; ++kk) {
        const int c = kk & 1, nx = c ^ 1;
        if (kk + 1 < BK / 2) {
#pragma unroll
          for (int i = 0; i < TM; ++i) af[nx][i] = a_s[(2 * kk + 2 + g) * LDA + (wm * TM + i) * 32 + li];
#pragma unroll
          for (int j = 0; j < TN; ++j) bf[nx][j] = b_s[(2 * kk + 2 + g) * LDB + (wn * TN + j) * 32 + li];
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the reads above the products (the scheduler would sink them)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[c][i], bf[c][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 af[TM], bf[TN];
        if constexpr (KC) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
            af[i] = *reinterpret_cast<const bf16x8*>(&a_s[((wm * TM + i) * 32 + li) * LDA + 16 * kk + 8 * g]);
#pragma unroll
          for (int j = 0; j < TN; ++j)
            bf[j] = *reinterpret_cast<const bf16x8*>(&b_s[((wn * TN + j) * 32 + li) * LDB + 16 * kk + 8 * g]);
        } else {
          // k-major stage [k][row]: a lane needs eight consecutive k of ONE row.  The transposing LDS read
          // (ds_read_b64_tr_b16) does that exchange inside groups of 16 lanes: lane s of a group supplies
          // the address of four consecutive rows at k0 + s/4, starting at row 4 (s % 4), and lane i of the
          // group receives the values of row i for k0 .. k0+3.  Two such reads make a fragment.
          const int s16 = lane & 15, rq = ((lane >> 4) & 1) * 16 + 4 * (s16 & 3), kq = 8 * g + (s16 >> 2);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
              const bf16x4 v = lds_read_tr(&a_s[(16 * kk + kq + 4 * hf) * LDA + (wm * TM + i) * 32 + rq]);
#pragma unroll
              for (int r = 0; r < 4; ++r) af[i][4 * hf + r] = v[r];
            }
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
              const bf16x4 v = lds_read_tr(&b_s[(16 * kk + kq + 4 * hf) * LDB + (wn * TN + j) * 32 + rq]);
#pragma unroll
              for (int r = 0; r < 4; ++r) bf[j][4 * hf + r] = v[r];
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
      }
    }
    if (kt + 1 < nk) write_stage(cur ^ 1);
    __syncthreads();
  }
  // Epilogue through LDS.  Accumulator q of a 32x32 block is row 8*(q/4) + 4*g + q%4, column
  // lane % 32: one value per row per lane.  Each wave writes a 32-row slab of its sub-tile to its
  // own LDS region and reads it back so that a lane holds two consecutive rows x four consecutive
  // columns -- the functor then moves 16 bytes per access and a row's lanes cover whole lines.
  // (Every wave has passed the k loop's last barrier, so the operand stages are dead.)
  // A folding functor (Epi::FOLD, fp32 products) returns a tile Z instead of storing it; Z goes
  // back into the slab and Z^T B (B: <= 32 columns, one row per output row) is accumulated with
  // MFMA over the slab's 32 rows: the slab is exactly the k-major operand layout for that product.
  float* eb = reinterpret_cast<float*>(smem) + wave * (32 * ELD);
  constexpr int LPR = EW / 4;     // lanes across the slab's columns
  constexpr int PPP = 64 / LPR;   // row pairs per pass
  const int ecol = 4 * (lane % LPR), epair = lane / LPR;
  constexpr bool FOLD = Epi::FOLD;
  static_assert(!FOLD || !P::IS_BF16, "folding epilogues are fp32 products");
  floatx16 gacc[FOLD ? TN : 1];
  if constexpr (FOLD) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) gacc[j][q] = 0.f;
  }
  if constexpr (!FOLD) {
    // Plain epilogues.  A functor's loads (EpiIO::fetch) run two passes ahead of its stores (EpiIO::apply): vector
    // memory operations retire in issue order, so a wait for loads issued behind a pass's stores would also wait for
    // those stores' acknowledgements -- a store round trip per pass.  Interior tiles take a branch-free body, in which
    // the compiler can count exactly which operations a wait has to cover.
    auto run = [&](auto full_tag) {
      constexpr bool FULLT = decltype(full_tag)::value;
      constexpr int NPI = 16 / PPP, NP = TM * NPI, AHEAD = NP < 2 ? NP : 2;
      typedef EpiIO<Epi> IO;
      typename IO::In in[NP];
      auto fetch = [&](int pz) {
        const int rl = 2 * ((pz % NPI) * PPP + epair);
        const int64_t row = m0 + (wm * TM + pz / NPI) * 32 + rl;
        const int col = n0 + wn * EW + ecol;
        if (FULLT || (row < M && col < N)) in[pz] = IO::template fetch<FULLT>(epi, row, col);
      };
#pragma unroll
      for (int pz = 0; pz < AHEAD; ++pz) fetch(pz);
#pragma unroll
      for (int pz = 0; pz < NP; ++pz) {
        const int i = pz / NPI, ps = pz % NPI;
        if (ps == 0) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) eb[(8 * (q / 4) + 4 * g + q % 4) * ELD + j * 32 + li] = acc[i][j][q];
          __builtin_amdgcn_wave_barrier();
        }
        if (pz + AHEAD < NP) fetch(pz + AHEAD);
        const int rl = 2 * (ps * PPP + epair);
        const float4 a = *reinterpret_cast<const float4*>(&eb[rl * ELD + ecol]);
        const float4 b = *reinterpret_cast<const float4*>(&eb[(rl + 1) * ELD + ecol]);
        const int64_t row = m0 + (wm * TM + i) * 32 + rl;
        const int col = n0 + wn * EW + ecol;
        if (FULLT || (row < M && col < N)) IO::template apply<FULLT>(epi, row, col, a, b, z, in[pz]);
        if (ps == NPI - 1) __builtin_amdgcn_wave_barrier();
      }
    };
    if ((m0 + BM <= M) && (n0 + BN <= N)) run(std::true_type());
    else run(std::false_type());
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    float bv[FOLD ? 16 : 1];  // FOLD: this lane's B values for the slab's 32 rows, requested early
    if constexpr (FOLD) {
      const int64_t rbase = m0 + (wm * TM + i) * 32;
#pragma unroll
      for (int kk = 0; kk < 16; ++kk) bv[kk] = epi.fold_b(rbase + 2 * kk + g, li);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) eb[(8 * (q / 4) + 4 * g + q % 4) * ELD + j * 32 + li] = acc[i][j][q];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int ps = 0; ps < 16 / PPP; ++ps) {
      const int rl = 2 * (ps * PPP + epair);
      const float4 a = *reinterpret_cast<const float4*>(&eb[rl * ELD + ecol]);
      const float4 b = *reinterpret_cast<const float4*>(&eb[(rl + 1) * ELD + ecol]);
      const int64_t row = m0 + (wm * TM + i) * 32 + rl;
      const int col = n0 + wn * EW + ecol;
      if constexpr (FOLD) {
        float4 za = make_float4(0.f, 0.f, 0.f, 0.f), zb = za;  // rows / columns outside the matrix contribute nothing
        if (row < M && col < N) epi(row, col, a, b, z, za, zb);
        *reinterpret_cast<float4*>(&eb[rl * ELD + ecol]) = za;  // the lane's own 2 x 4 patch
        *reinterpret_cast<float4*>(&eb[(rl + 1) * ELD + ecol]) = zb;
      } else {
        if (row < M && col < N) epi(row, col, a, b, z);
      }
    }
    if constexpr (FOLD) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int kk = 0; kk < 16; ++kk)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          gacc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(eb[(2 * kk + g) * ELD + j * 32 + li], bv[kk], gacc[j], 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
  }
  if constexpr (FOLD) {
    // the WM waves that own the same columns add their blocks (fixed order), then one partial per
    // workgroup: part[row tile][n0 + column][k]
    static_assert(WM == 2 || WM == 1, "fold: one or two waves along the rows");
    float* red = reinterpret_cast<float*>(smem);
    __syncthreads();
    if (WM == 2 && wm == 1) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) red[((wn * TN + j) * 16 + q) * 64 + lane] = gacc[j][q];
    }
    __syncthreads();
    if (wm == 0) {
      const int64_t tile = m0 / BM;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          float v = gacc[j][q];
          if (WM == 2) v += red[((wn * TN + j) * 16 + q) * 64 + lane];
          const int c = n0 + wn * EW + j * 32 + 8 * (q / 4) + 4 * g + q % 4;
          if (c < N && li < epi.f.K) epi.f.part[(tile * N + c) * epi.f.K + li] = v;
        }
    }
  }
}

// Returns the number of k splits actually used (every split is non-empty).
template <typename P, int TM, int TN, int WM, int WN, bool KC, int BK, typename LdA, typename LdB, typename Epi>
inline int launch_bk(hipStream_t st, const LdA& a, const LdB& b, const Epi& e, int64_t M, int N, int64_t K, int splits,
                     const Groups& grp = Groups()) {
  constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
  if (M <= 0 || N <= 0 || K <= 0) return 0;
  if (splits < 1) splits = 1;
  int64_t k_chunk = (K + splits - 1) / splits;
  k_chunk = (k_chunk + BK - 1) / BK * BK;
  if (!grp.k_ranges) splits = (int)((K + k_chunk - 1) / k_chunk);  // with k ranges: one split per range, as given
  const int64_t tiles_n = (N + BN - 1) / BN, tiles_m = grp.row_groups ? grp.n_row_tiles : (M + BM - 1) / BM;
  if (tiles_m <= 0) return 0;
  dim3 grid((unsigned)(((tiles_m * splits + 7) / 8) * 8 * tiles_n), 1, 1);
  hipLaunchKernelGGL((k_gemm<P, TM, TN, WM, WN, KC, BK, LdA, LdB, Epi>), grid, dim3(256), 0, st, a, b, e, M, N, K, k_chunk,
                     splits, grp);
  return splits;
}

// Stage depth by reduction length: short reductions (the radial basis) use a shallow stage.
template <typename P, int TM, int TN, int WM, int WN, bool KC, typename LdA, typename LdB, typename Epi>
inline int launch(hipStream_t st, const LdA& a, const LdB& b, const Epi& e, int64_t M, int N, int64_t K, int splits,
                  const Groups& grp = Groups()) {
  return launch_bk<P, TM, TN, WM, WN, KC, P::BK_BIG>(st, a, b, e, M, N, K, splits, grp);
}

// ---- row-stripe variant for short reductions (bf16, k-contiguous operands, K = 64 or 128) ---------------
// D(m, n) = sum_k A(m, k) B(n, k) with a reduction so short (the edge MLP's hidden width) that the k loop of
// the tiled kernel is a handful of iterations and each output tile re-reads its A rows: there the matrix
// cores wait for operands from the L2.  Here a workgroup owns a stripe of 128 rows: the stripe's A operand
// (all of K) is staged into LDS once, and the workgroup then walks the column tiles -- per column tile it
// stages only the B tile (prefetched into registers during the previous tile's products), so the L2 traffic
// per product halves and the stores of one column tile overlap the products of the next.
// Both loaders must be raw-bf16 loaders of width 8; N a multiple of 128; K a template constant.
//
// Vector memory operations retire through one in-order counter, so a wait for a load also waits for every store
// issued before it, and a wait the compiler cannot count exactly (a store under a branch, a loop header that
// joins two paths) becomes a wait for everything.  The walk over the column tiles is therefore straight-line
// code per tile (K and the trip counts are template constants, the ragged last stripe has a body of its own),
// and the only wait for the prefetched B tile sits at the end of the tile, behind a fixed number of stores:
// it covers the loads and the previous tile's stores, not this tile's.

// Workgroup barrier for LDS hand-overs only: waits for this wave's LDS operations, then s_barrier
// (__syncthreads() also fences global memory, i.e. waits for the acknowledgement of every outstanding store).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// An epilogue functor may declare row-wise inputs (type RowIn, row_in(row), apply(row, col, a, b, in)) that a kernel
// can fetch ahead of its stores; functors without them are called as they are.
template <typename Epi, typename = void>
struct RowInputs {
  struct type {};
  __device__ static __forceinline__ type get(const Epi&, int64_t) { return type{}; }
  __device__ static __forceinline__ void arrived(const type&) {}
  __device__ static __forceinline__ void apply(const Epi& e, int64_t r, int col, const float4& a, const float4& b, const type&) { e(r, col, a, b, 0); }
};
template <typename Epi>
struct RowInputs<Epi, std::void_t<typename Epi::RowIn>> {
  typedef typename Epi::RowIn type;
  __device__ static __forceinline__ type get(const Epi& e, int64_t r) { return e.row_in(r); }
  // a use the compiler must wait for: placed ahead of a loop it keeps the wait for these loads out of the loop
  __device__ static __forceinline__ void arrived(const type& in) { Epi::row_in_arrived(in); }
  __device__ static __forceinline__ void apply(const Epi& e, int64_t r, int col, const float4& a, const float4& b, const type& in) { e.apply(r, col, a, b, in); }
};

template <int K, typename LdA, typename LdB, typename Epi>
struct Stripe {
  static constexpr int LD = K + 8;          // row pitch in bf16: 16-byte fragment reads of 16 lanes fall into distinct banks
  static constexpr int ELD = 64 + 8;        // a wave's output slab: 32 rows x 64 columns; the pitch puts the two
                                            // half-waves of an accumulator write (four rows apart) on disjoint banks
  static constexpr int A_BYTES = 128 * LD * 2, B_BYTES = 128 * LD * 2, SLAB_BYTES = 4 * 32 * ELD * 4;
  static constexpr int BS_BYTES = B_BYTES > SLAB_BYTES ? B_BYTES : SLAB_BYTES;
  static constexpr int Q = K / 8;           // 16-byte items per row
  static constexpr int NV = 128 * Q / 256;  // items per thread and operand tile
  static constexpr int LPR = 16, PPP = 4;   // lanes across a slab's 64 columns, row pairs per pass
  typedef typename RowInputs<Epi>::type RowIn;

  // FULL: all 128 rows of the stripe exist (no row guards, hence no branches around the stores)
  template <bool FULL>
  __device__ static __forceinline__ void tiles(const LdB& ldb, const Epi& epi, int64_t M, int N, int64_t m0,
                                              const __bf16* sA, char* sBraw) {
    __bf16* sB = reinterpret_cast<__bf16*>(sBraw);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, g = lane >> 5;
    float* eb = reinterpret_cast<float*>(sBraw) + wave * (32 * ELD);
    const int ecol = 4 * (lane % LPR), epair = lane / LPR;
    // the epilogue's row-wise inputs of the eight row pairs this lane finishes, fetched once for all column tiles
    RowIn rin[2][16 / PPP];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int ps = 0; ps < 16 / PPP; ++ps) {
        const int64_t row = m0 + (wm * 2 + i) * 32 + 2 * (ps * PPP + epair);
        rin[i][ps] = RowInputs<Epi>::get(epi, FULL || row < M ? row : M - 2);
      }
    typename LdB::Raw vb[NV];
#pragma unroll
    for (int it = 0; it < NV; ++it) vb[it] = ldb.fetch((t + it * 256) / Q, 8 * ((t + it * 256) % Q));
#pragma unroll
    for (int it = 0; it < NV; ++it)
      *reinterpret_cast<bf16x8*>(&sB[((t + it * 256) / Q) * LD + 8 * ((t + it * 256) % Q)]) = ldb.finish(vb[it]);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int ps = 0; ps < 16 / PPP; ++ps) RowInputs<Epi>::arrived(rin[i][ps]);
    const int tiles_n = N / 128;
    for (int jt = 0; jt < tiles_n; ++jt) {
      const int n0 = jt * 128;
      lds_barrier();                          // the B tile (and, the first time, the A stripe) is in LDS
      const int nn = jt + 1 < tiles_n ? n0 + 128 : n0;  // the last tile re-fetches itself: same instruction count on every trip
#pragma unroll
      for (int it = 0; it < NV; ++it) vb[it] = ldb.fetch(nn + (t + it * 256) / Q, 8 * ((t + it * 256) % Q));
      floatx16 acc[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
#pragma unroll
      for (int kk = 0; kk < K / 16; ++kk) {
        bf16x8 af[2], bf[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) af[i] = *reinterpret_cast<const bf16x8*>(&sA[((wm * 2 + i) * 32 + li) * LD + 16 * kk + 8 * g]);
#pragma unroll
        for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const bf16x8*>(&sB[((wn * 2 + j) * 32 + li) * LD + 16 * kk + 8 * g]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
      }
      lds_barrier();  // every wave has read its B fragments: the B region now serves as the output slabs
#pragma unroll
      for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 16; ++q) eb[(8 * (q / 4) + 4 * g + q % 4) * ELD + j * 32 + li] = acc[i][j][q];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ps = 0; ps < 16 / PPP; ++ps) {
          const int rl = 2 * (ps * PPP + epair);
          const float4 a = *reinterpret_cast<const float4*>(&eb[rl * ELD + ecol]);
          const float4 b = *reinterpret_cast<const float4*>(&eb[(rl + 1) * ELD + ecol]);
          const int64_t row = m0 + (wm * 2 + i) * 32 + rl;
          const int col = n0 + wn * 64 + ecol;
          if (FULL || row < M) RowInputs<Epi>::apply(epi, row, col, a, b, rin[i][ps]);
        }
        __builtin_amdgcn_wave_barrier();
      }
      lds_barrier();  // slabs read back: the next B tile goes over them
#pragma unroll
      for (int it = 0; it < NV; ++it)
        *reinterpret_cast<bf16x8*>(&sB[((t + it * 256) / Q) * LD + 8 * ((t + it * 256) % Q)]) = ldb.finish(vb[it]);
    }
  }
};

template <int K, typename LdA, typename LdB, typename Epi>
__global__ void __launch_bounds__(256, 2)
k_gemm_stripe(LdA lda, LdB ldb, Epi epi, int64_t M, int N) {
  static_assert(LdA::WIDTH == 8 && LdB::WIDTH == 8, "raw bf16 operands");
  static_assert(K % 16 == 0 && (128 * (K / 8)) % 256 == 0, "whole k steps, whole staging passes");
  typedef Stripe<K, LdA, LdB, Epi> S;
  __shared__ __attribute__((aligned(16))) __bf16 sA[128 * S::LD];
  __shared__ __attribute__((aligned(16))) char sBraw[S::BS_BYTES];  // B tile, then the slabs
  const int t = threadIdx.x;
  const int64_t m0 = (int64_t)blockIdx.x * 128;
  // A stripe: rows beyond M are clamped (their outputs are never stored)
#pragma unroll
  for (int it = 0; it < S::NV; ++it) {
    const int idx = t + it * 256;
    const int r = idx / S::Q, q = idx % S::Q;
    int64_t row = m0 + r;
    row = row < M ? row : M - 1;
    *reinterpret_cast<bf16x8*>(&sA[r * S::LD + 8 * q]) = lda.finish(lda.fetch(row, 8 * q));
  }
  if (m0 + 128 <= M) S::template tiles<true>(ldb, epi, M, N, m0, sA, sBraw);
  else S::template tiles<false>(ldb, epi, M, N, m0, sA, sBraw);
}

// K must equal the template constant, N be a multiple of 128 and M even (rows come in pairs).
template <int K, typename LdA, typename LdB, typename Epi>
inline void launch_stripe(hipStream_t st, const LdA& a, const LdB& b, const Epi& e, int64_t M, int N) {
  if (M <= 0) return;
  hipLaunchKernelGGL((k_gemm_stripe<K, LdA, LdB, Epi>), dim3((unsigned)((M + 127) / 128)), dim3(256), 0, st, a, b, e, M, N);
}

}  // namespace gemm
