// Operand loaders and epilogues plugged into the GEMM template, and SiLU derivatives.
// Every loader maps (matrix row, first of four consecutive columns) -> float4.
// "Jets" are pairs (value, derivative with respect to the edge length r) stored as two
// consecutive rows: row 2e holds the value, row 2e+1 the derivative.  The index e below counts
// pairs of opposite edges (equal lengths, one jet per pair), E their number.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fx {

typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

// hardware reciprocal (1 ulp): an IEEE division would expand into about ten more instructions, and vector
// instructions in the matrix-product loops take issue slots away from the matrix pipeline
__device__ __forceinline__ float sigm(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }
__device__ __forceinline__ float silu(float x) { return x * sigm(x); }
__device__ __forceinline__ float dsilu(float x) {
  float s = sigm(x);
  return s * (1.f + x * (1.f - s));
}
__device__ __forceinline__ float d2silu(float x) {
  float s = sigm(x);
  return s * (1.f - s) * (2.f + x * (1.f - 2.f * s));
}
// silu', silu'' together (one exponential)
__device__ __forceinline__ void dsilu12(float x, float& d1, float& d2) {
  float s = sigm(x);
  d1 = s * (1.f + x * (1.f - s));
  d2 = s * (1.f - s) * (2.f + x * (1.f - 2.f * s));
}

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 ld4(const __bf16* p) {
  bf16x4_t b = *reinterpret_cast<const bf16x4_t*>(p);
  return make_float4((float)b[0], (float)b[1], (float)b[2], (float)b[3]);
}
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void st4(__bf16* p, float4 v) {
  bf16x4_t b = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
  *reinterpret_cast<bf16x4_t*>(p) = b;
}
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float4 mul4(float4 a, float4 b) { return make_float4(a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w); }
__device__ __forceinline__ float4 silu4(float4 a) { return make_float4(silu(a.x), silu(a.y), silu(a.z), silu(a.w)); }
__device__ __forceinline__ float4 dsilu4(float4 a) { return make_float4(dsilu(a.x), dsilu(a.y), dsilu(a.z), dsilu(a.w)); }

// ---------------------------------------------------------------------------- loaders
// fetch() only issues loads (so they overlap the matrix products of the current tile),
// finish() applies the element-wise function when the tile is staged.
struct Raw2 { float4 a, b; };

struct LdPlain {  // p[row * ld + col]
  static constexpr bool PAIRED = false;
  static constexpr int WIDTH = 4;
  __device__ __forceinline__ void shift(int64_t elems) { p += elems; }  // another matrix of a stack
  typedef float4 Raw;
  const float* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const { return ld4(p + r * ld + c); }
  __device__ __forceinline__ float4 finish(const Raw& x) const { return x; }
};
struct LdSilu {  // silu(p[row * ld + col])
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef float4 Raw;
  const float* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const { return ld4(p + r * ld + c); }
  __device__ __forceinline__ float4 finish(const Raw& x) const { return silu4(x); }
};
struct LdJetSilu {  // jet matrix u [2E][W]: row 2e -> silu(u[2e]), row 2e+1 -> silu'(u[2e]) * u[2e+1], both at once
  static constexpr bool PAIRED = true;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef Raw2 Raw;
  const float* u;
  int64_t W;
  __device__ __forceinline__ Raw fetch(int64_t r_even, int64_t c) const {
    const float* pe = u + r_even * W + c;
    return Raw{ld4(pe), ld4(pe + W)};
  }
  __device__ __forceinline__ void finish(const Raw& x, float4& val, float4& der) const {
    const float a[4] = {x.a.x, x.a.y, x.a.z, x.a.w}, b[4] = {x.b.x, x.b.y, x.b.z, x.b.w};
    float v[4], d[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float s = sigm(a[j]);
      v[j] = a[j] * s;
      d[j] = s * (1.f + a[j] * (1.f - s)) * b[j];
    }
    val = make_float4(v[0], v[1], v[2], v[3]);
    der = make_float4(d[0], d[1], d[2], d[3]);
  }
};
struct LdJetSiluEven {  // row e -> silu(u[2e])
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef float4 Raw;
  const float* u;
  int64_t W;
  __device__ __forceinline__ Raw fetch(int64_t e, int64_t c) const { return ld4(u + 2 * e * W + c); }
  __device__ __forceinline__ float4 finish(const Raw& x) const { return silu4(x); }
};
struct LdJetSiluOdd {  // row e -> silu'(u[2e]) * u[2e+1]
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef Raw2 Raw;
  const float* u;
  int64_t W;
  __device__ __forceinline__ Raw fetch(int64_t e, int64_t c) const {
    const float* pe = u + 2 * e * W + c;
    return Raw{ld4(pe), ld4(pe + W)};
  }
  __device__ __forceinline__ float4 finish(const Raw& x) const { return mul4(dsilu4(x.a), x.b); }
};
struct LdDsiluMul {  // silu'(q[row]) * x[row]
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef Raw2 Raw;
  const float* q;
  const float* x;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const { return Raw{ld4(q + r * ld + c), ld4(x + r * ld + c)}; }
  __device__ __forceinline__ float4 finish(const Raw& v) const { return mul4(dsilu4(v.a), v.b); }
};
struct LdMuY {  // w_o[col] * silu'(y[row, col])
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef Raw2 Raw;
  const float* y;
  const float* wo;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const { return Raw{ld4(y + r * ld + c), ld4(wo + c)}; }
  __device__ __forceinline__ float4 finish(const Raw& v) const { return mul4(dsilu4(v.a), v.b); }
};

// ---- second-derivative rows, used only for the optional position gradient dL/dx
struct LdPhi2 {  // row u (edge pair), columns k..k+3 -> d^2 phi_k / dr^2 at r_e = (-2 gamma + 4 gamma^2 t^2) exp(-gamma t^2), t = r_e - k dmu
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  struct Raw { float r; int k; };
  const float4* geo;   // [E] (unit vector, length)
  const int32_t* und;  // [Eu] an edge of each pair: rows are edge pairs
  float dmu, gamma;
  __device__ __forceinline__ Raw fetch(int64_t u, int64_t c) const { return Raw{geo[und[u]].w, (int)c}; }
  __device__ __forceinline__ float4 finish(const Raw& x) const {
    float o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float t = x.r - (float)(x.k + u) * dmu;
      o[u] = (4.f * gamma * gamma * t * t - 2.f * gamma) * __expf(-gamma * t * t);
    }
    return make_float4(o[0], o[1], o[2], o[3]);
  }
};
struct LdJetSecond {  // row e -> d^2 silu(u)/dr^2 = silu''(u) u'^2 + silu'(u) u'',  u = uj[2e], u' = uj[2e+1], u'' = u2[e]
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  struct Raw { float4 a, b, c; };
  const float* uj;
  const float* u2;
  int64_t W;
  __device__ __forceinline__ Raw fetch(int64_t e, int64_t c) const {
    const float* pe = uj + 2 * e * W + c;
    return Raw{ld4(pe), ld4(pe + W), ld4(u2 + e * W + c)};
  }
  __device__ __forceinline__ float4 finish(const Raw& x) const {
    const float a[4] = {x.a.x, x.a.y, x.a.z, x.a.w}, b[4] = {x.b.x, x.b.y, x.b.z, x.b.w}, c[4] = {x.c.x, x.c.y, x.c.z, x.c.w};
    float o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float d1, d2;
      dsilu12(a[j], d1, d2);
      o[j] = d2 * b[j] * b[j] + d1 * c[j];
    }
    return make_float4(o[0], o[1], o[2], o[3]);
  }
};

struct LdBf16 {  // bf16 matrix p[row * ld + col] (values already rounded by their producer)
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef bf16x4_t Raw;
  const __bf16* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const { return *reinterpret_cast<const bf16x4_t*>(p + r * ld + c); }
  __device__ __forceinline__ float4 finish(const Raw& x) const {
    return make_float4((float)x[0], (float)x[1], (float)x[2], (float)x[3]);
  }
};

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
struct LdBf16x8 {  // the same matrix fetched eight values (16 bytes) at a time and staged without conversion;
                   // needs ld, the extent along the contiguous index and the base address in multiples of 8 values
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 8;
  typedef bf16x8_t Raw;
  const __bf16* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const { return *reinterpret_cast<const bf16x8_t*>(p + r * ld + c); }
  __device__ __forceinline__ Raw finish(const Raw& x) const { return x; }
};

// ---- adjoints of per-pair quantities.  The two edges of a pair write their adjoint rows side by side (rows 2u and 2u + 1);
// what reaches the per-pair edge MLP is their sum, formed while the operand is staged.
struct LdPairSum {  // p[2 row][col] + p[2 row + 1][col]
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  typedef Raw2 Raw;
  const float* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const {
    const float* pe = p + 2 * r * ld + c;
    return Raw{ld4(pe), ld4(pe + ld)};
  }
  __device__ __forceinline__ float4 finish(const Raw& x) const { return add4(x.a, x.b); }
};
struct LdBf16Pair {  // the same for a bf16 matrix
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 4;
  struct Raw { bf16x4_t a, b; };
  const __bf16* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const {
    const __bf16* pe = p + 2 * r * ld + c;
    return Raw{*reinterpret_cast<const bf16x4_t*>(pe), *reinterpret_cast<const bf16x4_t*>(pe + ld)};
  }
  __device__ __forceinline__ float4 finish(const Raw& x) const {
    return make_float4((float)x.a[0] + (float)x.b[0], (float)x.a[1] + (float)x.b[1], (float)x.a[2] + (float)x.b[2], (float)x.a[3] + (float)x.b[3]);
  }
};
struct LdBf16x8Pair {  // ... fetched 16 bytes at a time (same conditions as LdBf16x8), summed in fp32 and rounded once
  static constexpr bool PAIRED = false;
  __device__ __forceinline__ void shift(int64_t) {}
  static constexpr int WIDTH = 8;
  struct Raw { bf16x8_t a, b; };
  const __bf16* p;
  int64_t ld;
  __device__ __forceinline__ Raw fetch(int64_t r, int64_t c) const {
    const __bf16* pe = p + 2 * r * ld + c;
    return Raw{*reinterpret_cast<const bf16x8_t*>(pe), *reinterpret_cast<const bf16x8_t*>(pe + ld)};
  }
  __device__ __forceinline__ bf16x8_t finish(const Raw& x) const {
    bf16x8_t o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (__bf16)((float)x.a[i] + (float)x.b[i]);
    return o;
  }
};

// ---------------------------------------------------------------------------- epilogues
// operator()(r, col, a, b, z): a holds columns col..col+3 of output row r (even, in range) and b
// the same columns of row r + 1, which the functor must skip when r + 1 == M unless the rows
// come in pairs (jets: M = 2E).  z is the k-split index.
__device__ __forceinline__ float4 scale4(float s, float4 a) { return make_float4(s * a.x, s * a.y, s * a.z, s * a.w); }

struct EpiStoreJetAct {  // u = v (fp32 jets) and the activated jets silu(u), silu'(u) u' rounded to bf16
  static constexpr bool FOLD = false;
  float* u;
  __bf16* sj;
  int64_t ld, M;  // M = 2E
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    const int64_t o = r * ld + col;
    st4(u + o, a);
    st4(u + o + ld, b);
    const float x[4] = {a.x, a.y, a.z, a.w}, xd[4] = {b.x, b.y, b.z, b.w};
    float val[4], der[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float s = sigm(x[j]);
      val[j] = x[j] * s;
      der[j] = s * (1.f + x[j] * (1.f - s)) * xd[j];
    }
    st4(sj + o, make_float4(val[0], val[1], val[2], val[3]));
    st4(sj + o + ld, make_float4(der[0], der[1], der[2], der[3]));
  }
};
struct EpiStore {
  static constexpr bool FOLD = false;
  float* p;
  int64_t ld, M;
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    const int64_t o = r * ld + col;
    st4(p + o, a);
    if (r + 1 < M) st4(p + o + ld, b);
  }
};
struct EpiAddStore {  // p = add + v
  static constexpr bool FOLD = false;
  float* p;
  const float* add;
  int64_t ld, M;
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    const int64_t o = r * ld + col;
    st4(p + o, add4(ld4(add + o), a));
    if (r + 1 < M) st4(p + o + ld, add4(ld4(add + o + ld), b));
  }
  struct In { float4 a, b; };
  template <bool FULL>
  __device__ __forceinline__ In fetch(int64_t r, int col) const {
    const int64_t o = r * ld + col;
    In in;
    in.a = ld4(add + o);
    in.b = (FULL || r + 1 < M) ? ld4(add + o + ld) : in.a;
    return in;
  }
  template <bool FULL>
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, int, const In& in) const {
    const int64_t o = r * ld + col;
    st4(p + o, add4(in.a, a));
    if (FULL || r + 1 < M) st4(p + o + ld, add4(in.b, b));
  }
};
template <typename TO>
struct EpiOmega {  // jets (w, w') -> radial filter jets (c w, c' w + c w'),  env[e] = (c, c')
  static constexpr bool FOLD = false;
  TO* out;
  const float2* env;
  int64_t ld, M;  // M = 2E
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    apply(r, col, a, b, env[r >> 1]);
  }
  // The functor's only load depends on the row alone.  A kernel that keeps its rows while it walks the columns
  // fetches it once, ahead of all stores: a load issued after stores cannot be waited for without waiting for
  // those stores' acknowledgements too (one in-order counter for vector memory operations), which would put a
  // store round trip into every pass of the epilogue.
  typedef float2 RowIn;
  typedef float2 In;
  template <bool FULL>
  __device__ __forceinline__ In fetch(int64_t r, int) const { return env[r >> 1]; }
  template <bool FULL>
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, int, const In& c) const { apply(r, col, a, b, c); }
  __device__ __forceinline__ RowIn row_in(int64_t r) const { return env[r >> 1]; }
  __device__ static __forceinline__ void row_in_arrived(const RowIn& c) { asm volatile("" ::"v"(c.x), "v"(c.y)); }
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, const RowIn& c) const {
    const int64_t o = r * ld + col;
    st4(out + o, scale4(c.x, a));
    st4(out + o + ld, add4(scale4(c.y, a), scale4(c.x, b)));
  }
};
struct EpiMuT {  // mu_t = v, mu_q = silu'(q) v
  static constexpr bool FOLD = false;
  float* mu_t;
  float* mu_q;
  const float* q;
  int64_t ld, M;
  __device__ __forceinline__ void one(int64_t o, const float4& v) const {
    st4(mu_t + o, v);
    st4(mu_q + o, mul4(dsilu4(ld4(q + o)), v));
  }
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    one(r * ld + col, a);
    if (r + 1 < M) one((r + 1) * ld + col, b);
  }
  struct In { float4 a, b; };
  template <bool FULL>
  __device__ __forceinline__ In fetch(int64_t r, int col) const {
    const int64_t o = r * ld + col;
    In in;
    in.a = ld4(q + o);
    in.b = (FULL || r + 1 < M) ? ld4(q + o + ld) : in.a;
    return in;
  }
  template <bool FULL>
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, int, const In& in) const {
    const int64_t o = r * ld + col;
    st4(mu_t + o, a);
    st4(mu_q + o, mul4(dsilu4(in.a), a));
    if (FULL || r + 1 < M) {
      st4(mu_t + o + ld, b);
      st4(mu_q + o + ld, mul4(dsilu4(in.b), b));
    }
  }
};
template <typename TZ>
struct EpiYZ {  // Y = v, Z = silu'(u[2e]) v   (u jets [2E][ld]); Z only ever feeds matrix products
  static constexpr bool FOLD = false;
  float* Y;
  TZ* Z;
  const float* u;
  int64_t ld, M;
  __device__ __forceinline__ void one(int64_t r, int col, const float4& v) const {
    const int64_t o = r * ld + col;
    st4(Y + o, v);
    st4(Z + o, mul4(dsilu4(ld4(u + 2 * o - col)), v));  // u row 2r: 2 r ld + col
  }
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    one(r, col, a);
    if (r + 1 < M) one(r + 1, col, b);
  }
  struct In { float4 a, b; };
  template <bool FULL>
  __device__ __forceinline__ In fetch(int64_t r, int col) const {
    const float* pu = u + 2 * r * ld + col;  // u rows 2r and 2(r + 1)
    In in;
    in.a = ld4(pu);
    in.b = (FULL || r + 1 < M) ? ld4(pu + 2 * ld) : in.a;
    return in;
  }
  template <bool FULL>
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, int, const In& in) const {
    const int64_t o = r * ld + col;
    st4(Y + o, a);
    st4(Z + o, mul4(dsilu4(in.a), a));
    if (FULL || r + 1 < M) {
      st4(Y + o + ld, b);
      st4(Z + o + ld, mul4(dsilu4(in.b), b));
    }
  }
};
__device__ __forceinline__ float4 lam4(float4 u0, float4 u1, float4 y, float4 v) {  // silu'(u0) v + silu''(u0) u1 y
  const float a0[4] = {u0.x, u0.y, u0.z, u0.w}, a1[4] = {u1.x, u1.y, u1.z, u1.w}, yy[4] = {y.x, y.y, y.z, y.w},
              vv[4] = {v.x, v.y, v.z, v.w};
  float a[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float d1, d2;
    dsilu12(a0[j], d1, d2);
    a[j] = d1 * vv[j] + d2 * a1[j] * yy[j];
  }
  return make_float4(a[0], a[1], a[2], a[3]);
}
template <typename TZ>
struct EpiLamU {  // out = silu'(u) v + silu''(u) u' Y; out only ever feeds matrix products
  static constexpr bool FOLD = false;
  TZ* out;
  const float* u;
  const float* Y;
  int64_t ld, M;
  __device__ __forceinline__ void one(int64_t r, int col, const float4& v) const {
    const int64_t o = r * ld + col;
    const float* pu = u + 2 * r * ld + col;
    st4(out + o, lam4(ld4(pu), ld4(pu + ld), ld4(Y + o), v));
  }
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    one(r, col, a);
    if (r + 1 < M) one(r + 1, col, b);
  }
  struct In { float4 u0[2], u1[2], y[2]; };
  template <bool FULL>
  __device__ __forceinline__ In fetch(int64_t r, int col) const {
    const float* pu = u + 2 * r * ld + col;
    const float* py = Y + r * ld + col;
    const bool two = FULL || r + 1 < M;
    In in;
    in.u0[0] = ld4(pu);
    in.u1[0] = ld4(pu + ld);
    in.y[0] = ld4(py);
    in.u0[1] = two ? ld4(pu + 2 * ld) : in.u0[0];
    in.u1[1] = two ? ld4(pu + 3 * ld) : in.u1[0];
    in.y[1] = two ? ld4(py + ld) : in.y[0];
    return in;
  }
  template <bool FULL>
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, int, const In& in) const {
    const int64_t o = r * ld + col;
    st4(out + o, lam4(in.u0[0], in.u1[0], in.y[0], a));
    if (FULL || r + 1 < M) st4(out + o + ld, lam4(in.u0[1], in.u1[1], in.y[1], b));
  }
};
struct EpiLamQ {  // out = silu'(q) v + silu''(q) qd mu_t
  static constexpr bool FOLD = false;
  float* out;
  const float* q;
  const float* qd;
  const float* mu_t;
  int64_t ld, M;
  __device__ __forceinline__ void one(int64_t o, const float4& v) const {
    st4(out + o, lam4(ld4(q + o), ld4(qd + o), ld4(mu_t + o), v));
  }
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int) const {
    one(r * ld + col, a);
    if (r + 1 < M) one((r + 1) * ld + col, b);
  }
  struct In { float4 q[2], qd[2], mt[2]; };
  template <bool FULL>
  __device__ __forceinline__ In fetch(int64_t r, int col) const {
    const int64_t o = r * ld + col, o2 = (FULL || r + 1 < M) ? o + ld : o;
    In in;
    in.q[0] = ld4(q + o); in.qd[0] = ld4(qd + o); in.mt[0] = ld4(mu_t + o);
    in.q[1] = ld4(q + o2); in.qd[1] = ld4(qd + o2); in.mt[1] = ld4(mu_t + o2);
    return in;
  }
  template <bool FULL>
  __device__ __forceinline__ void apply(int64_t r, int col, const float4& a, const float4& b, int, const In& in) const {
    const int64_t o = r * ld + col;
    st4(out + o, lam4(in.q[0], in.qd[0], in.mt[0], a));
    if (FULL || r + 1 < M) st4(out + o + ld, lam4(in.q[1], in.qd[1], in.mt[1], b));
  }
};
struct EpiPartial {  // split-k partial sums: part[z][row][col]
  static constexpr bool FOLD = false;
  float* part;
  int64_t ld, M;
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int z) const {
    const int64_t o = ((int64_t)z * M + r) * ld + col;
    st4(part + o, a);
    if (r + 1 < M) st4(part + o + ld, b);
  }
};

// ---- folding epilogues: besides their element-wise work they hand the kernel a tile Z of values
// (columns col..col+3 of rows r, r+1) whose product with a narrow per-row matrix B (<= 32 columns)
// the kernel accumulates on the fly:  part[tile][c][k] = sum_{rows of the tile} Z[row][c] B[row][k].
// This replaces a separate weight-gradient pass that would re-read Z from HBM (and, for Z that
// nothing else needs, its store).  fold_b(row, k) returns B[row][k], zero outside the matrix.
struct FoldB {
  const float* b;  // B[row * ldb + k]
  int ldb, K;      // K <= 32
  float* part;     // [row tiles][N][K]
};
template <typename TZ>
struct EpiYZFold {  // Y = v stored; Z = silu'(u[2e]) v folded with B
  static constexpr bool FOLD = true;
  float* Y;
  const float* u;
  int64_t ld, M;
  FoldB f;
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int, float4& za, float4& zb) const {
    const int64_t o = r * ld + col;
    st4(Y + o, a);
    za = mul4(dsilu4(ld4(u + 2 * o - col)), a);
    if (r + 1 < M) {
      st4(Y + o + ld, b);
      zb = mul4(dsilu4(ld4(u + 2 * (o + ld) - col)), b);
    }
  }
  __device__ __forceinline__ float fold_b(int64_t row, int k) const { return (row < M && k < f.K) ? f.b[row * f.ldb + k] : 0.f; }
};
template <typename TZ>
struct EpiLamUFold {  // silu'(u) v + silu''(u) u' Y folded with B, not stored
  static constexpr bool FOLD = true;
  const float* u;
  const float* Y;
  int64_t ld, M;
  FoldB f;
  __device__ __forceinline__ void operator()(int64_t r, int col, const float4& a, const float4& b, int, float4& za, float4& zb) const {
    const int64_t o = r * ld + col;
    const float* pu = u + 2 * r * ld + col;
    za = lam4(ld4(pu), ld4(pu + ld), ld4(Y + o), a);
    if (r + 1 < M) zb = lam4(ld4(pu + 2 * ld), ld4(pu + 3 * ld), ld4(Y + o + ld), b);
  }
  __device__ __forceinline__ float fold_b(int64_t row, int k) const { return (row < M && k < f.K) ? f.b[row * f.ldb + k] : 0.f; }
};

}  // namespace fx
