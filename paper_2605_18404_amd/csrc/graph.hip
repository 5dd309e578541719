// Periodic radius graph on the GPU: cell-list binning, receiver-sorted CSR with a canonical
// in-row order, and the reverse-edge map.  Integer work throughout; the only floating-point
// decision is r^2 < r_c^2, taken in float32 with a fixed operation order (see mlip.h).
#include <algorithm>
#include <cmath>
#include <cstring>

#include "common.h"

namespace {

constexpr int SCAN_BLOCK = 256;
constexpr int SCAN_ITEMS = 8;  // per thread
constexpr int SCAN_TILE = SCAN_BLOCK * SCAN_ITEMS;
static_assert(SCAN_TILE == GRAPH_SCAN_TILE, "common.h states the scan tile for those who size the scan's work array");

// ------------------------------------------------------------------ exclusive scan (int32)
__global__ void k_scan_block_sums(const int32_t* __restrict__ in, int32_t* __restrict__ block_sums, int64_t n) {
  __shared__ int32_t red[SCAN_BLOCK];
  int64_t base = (int64_t)blockIdx.x * SCAN_TILE + threadIdx.x * SCAN_ITEMS;
  int32_t s = 0;
  for (int k = 0; k < SCAN_ITEMS; ++k)
    if (base + k < n) s += in[base + k];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = SCAN_BLOCK / 2; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) block_sums[blockIdx.x] = red[0];
}

__global__ void k_scan_sums_serial(int32_t* block_sums, int n_blocks) {
  // one thread: n_blocks is at most a few thousand
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int32_t run = 0;
    for (int b = 0; b < n_blocks; ++b) {
      int32_t t = block_sums[b];
      block_sums[b] = run;
      run += t;
    }
  }
}

// out[i] = sum_{k<i} in[k] for i in [0, n]; out has n+1 entries (last = total).
__global__ void k_scan_apply(const int32_t* __restrict__ in, const int32_t* __restrict__ block_sums,
                             int32_t* __restrict__ out, int64_t n) {
  __shared__ int32_t part[SCAN_BLOCK];
  int64_t base = (int64_t)blockIdx.x * SCAN_TILE + threadIdx.x * SCAN_ITEMS;
  int32_t v[SCAN_ITEMS];
  int32_t s = 0;
  for (int k = 0; k < SCAN_ITEMS; ++k) {
    v[k] = (base + k < n) ? in[base + k] : 0;
    s += v[k];
  }
  part[threadIdx.x] = s;
  __syncthreads();
  // Hillis-Steele inclusive scan of the per-thread sums
  for (int off = 1; off < SCAN_BLOCK; off <<= 1) {
    int32_t t = (threadIdx.x >= off) ? part[threadIdx.x - off] : 0;
    __syncthreads();
    part[threadIdx.x] += t;
    __syncthreads();
  }
  int32_t run = block_sums[blockIdx.x] + part[threadIdx.x] - s;
  for (int k = 0; k < SCAN_ITEMS; ++k) {
    if (base + k < n) out[base + k] = run;
    run += v[k];
    if (base + k == n - 1) out[n] = run;
  }
}

int scan_exclusive(mlip_ctx* ctx, const int32_t* in, int32_t* out, int64_t n) {
  int n_blocks = (int)((n + SCAN_TILE - 1) / SCAN_TILE);
  hipLaunchKernelGGL(k_scan_block_sums, dim3(n_blocks), dim3(SCAN_BLOCK), 0, ctx->stream, in, ctx->d_scan_tmp, n);
  hipLaunchKernelGGL(k_scan_sums_serial, dim3(1), dim3(64), 0, ctx->stream, ctx->d_scan_tmp, n_blocks);
  hipLaunchKernelGGL(k_scan_apply, dim3(n_blocks), dim3(SCAN_BLOCK), 0, ctx->stream, in, ctx->d_scan_tmp, out, n);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

// ------------------------------------------------------------------ binning
__device__ __forceinline__ int struct_of_atom(const StructMeta* meta, int B, int i) {
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (meta[mid].atom_begin <= i) lo = mid; else hi = mid - 1;
  }
  // skip empty structures that share atom_begin
  while (lo + 1 < B && meta[lo].atom_end <= i) ++lo;
  return lo;
}

__device__ __forceinline__ int bin_coord(float x, float L, int nb) {
  int b = (int)(x / L * (float)nb);
  return b < 0 ? 0 : (b >= nb ? nb - 1 : b);
}

__device__ __forceinline__ int bin_of_fraction(float f, int nb) {
  int b = (int)floorf(f * (float)nb);
  return b < 0 ? 0 : (b >= nb ? nb - 1 : b);
}

// Fractional coordinates may leave [0, 1] by this much before a position counts as outside its
// (general) cell; the bins are wide enough to absorb it.
constexpr float FRAC_TOL = 1e-5f;

// Bounding box of every structure's atoms (one block per structure); used for molecules, whose
// bins are laid over the box.  NaNs are skipped here and reported by the binning kernel.
__global__ void __launch_bounds__(256) k_bounds(const float* __restrict__ pos, const int32_t* __restrict__ struct_ptr,
                                                float* __restrict__ bounds) {
  __shared__ float red[6][256];
  const int s = blockIdx.x, t = threadIdx.x;
  const int a = struct_ptr[s], b = struct_ptr[s + 1];
  float lo[3] = {INFINITY, INFINITY, INFINITY}, hi[3] = {-INFINITY, -INFINITY, -INFINITY};
  for (int i = a + t; i < b; i += 256)
    for (int c = 0; c < 3; ++c) {
      float x = pos[3 * (int64_t)i + c];
      lo[c] = fminf(lo[c], x);
      hi[c] = fmaxf(hi[c], x);
    }
  for (int c = 0; c < 3; ++c) {
    red[c][t] = lo[c];
    red[3 + c][t] = hi[c];
  }
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (t < off)
      for (int c = 0; c < 3; ++c) {
        red[c][t] = fminf(red[c][t], red[c][t + off]);
        red[3 + c][t] = fmaxf(red[3 + c][t], red[3 + c][t + off]);
      }
    __syncthreads();
  }
  if (t < 6) bounds[6 * s + t] = red[t][0];
}

__global__ void k_bin_count(const float* __restrict__ pos, const StructMeta* __restrict__ meta, int B, int N,
                            int32_t* __restrict__ atom_struct, int32_t* __restrict__ atom_bin,
                            int32_t* __restrict__ bin_count, int32_t* __restrict__ flag) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  int s = struct_of_atom(meta, B, i);
  StructMeta m = meta[s];
  float x = pos[3 * i], y = pos[3 * i + 1], z = pos[3 * i + 2];
  bool ok;
  int bx, by, bz;
  if (m.kind == CELL_ORTHO) {
    const float Lx = m.lat[0], Ly = m.lat[4], Lz = m.lat[8];
    ok = (x >= 0.f) && (x < Lx) && (y >= 0.f) && (y < Ly) && (z >= 0.f) && (z < Lz);  // also catches NaN
    bx = ok ? bin_coord(x, Lx, m.nb[0]) : 0;
    by = ok ? bin_coord(y, Ly, m.nb[1]) : 0;
    bz = ok ? bin_coord(z, Lz, m.nb[2]) : 0;
  } else {
    const float rx = x - m.origin[0], ry = y - m.origin[1], rz = z - m.origin[2];
    const float f0 = (rx * m.inv[0] + ry * m.inv[3]) + rz * m.inv[6];
    const float f1 = (rx * m.inv[1] + ry * m.inv[4]) + rz * m.inv[7];
    const float f2 = (rx * m.inv[2] + ry * m.inv[5]) + rz * m.inv[8];
    if (m.kind == CELL_TRICLINIC)
      ok = (f0 >= -FRAC_TOL) && (f0 <= 1.f + FRAC_TOL) && (f1 >= -FRAC_TOL) && (f1 <= 1.f + FRAC_TOL) &&
           (f2 >= -FRAC_TOL) && (f2 <= 1.f + FRAC_TOL);
    else  // a molecule may sit anywhere; its bins cover its bounding box
      ok = (fabsf(x) <= 3.0e38f) && (fabsf(y) <= 3.0e38f) && (fabsf(z) <= 3.0e38f) && (fabsf(f0) <= 2.f) &&
           (fabsf(f1) <= 2.f) && (fabsf(f2) <= 2.f);
    bx = ok ? bin_of_fraction(f0, m.nb[0]) : 0;
    by = ok ? bin_of_fraction(f1, m.nb[1]) : 0;
    bz = ok ? bin_of_fraction(f2, m.nb[2]) : 0;
  }
  if (!ok) atomicOr(flag, 1);
  int g = m.bin_base + (bz * m.nb[1] + by) * m.nb[0] + bx;
  atom_struct[i] = s;
  atom_bin[i] = g;
  atomicAdd(&bin_count[g], 1);
}

__global__ void k_bin_fill(const int32_t* __restrict__ atom_bin, const int32_t* __restrict__ bin_start,
                           int32_t* __restrict__ bin_cursor, int32_t* __restrict__ bin_atoms, int N) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  int g = atom_bin[i];
  int slot = atomicAdd(&bin_cursor[g], 1);  // order inside a bin is arbitrary; rows are sorted later
  bin_atoms[bin_start[g] + slot] = i;
}

// The float32 neighbour test, in the documented operation order, without contraction.
__device__ __forceinline__ bool within(float xi, float yi, float zi, float xj, float yj, float zj, float sx,
                                       float sy, float sz, float rc2) {
  float dx = __fadd_rn(__fsub_rn(xj, xi), sx);
  float dy = __fadd_rn(__fsub_rn(yj, yi), sy);
  float dz = __fadd_rn(__fsub_rn(zj, zi), sz);
  float r2 = __fadd_rn(__fadd_rn(__fmul_rn(dx, dx), __fmul_rn(dy, dy)), __fmul_rn(dz, dz));
  return r2 < rc2;
}

// One 64-lane wave per receiver atom.  FILL = false: count neighbours; true: write keys.
template <bool FILL>
__global__ void __launch_bounds__(256) k_neighbours(const float* __restrict__ pos, const StructMeta* __restrict__ meta,
                                                    const int32_t* __restrict__ atom_struct,
                                                    const int32_t* __restrict__ atom_bin,
                                                    const int32_t* __restrict__ bin_start,
                                                    const int32_t* __restrict__ bin_atoms, int N, float rc2,
                                                    int32_t* __restrict__ deg, const int32_t* __restrict__ row_ptr,
                                                    int32_t* __restrict__ key_tmp) {
  int lane = threadIdx.x & 63;
  int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= N) return;
  StructMeta m = meta[atom_struct[i]];
  float xi = pos[3 * i], yi = pos[3 * i + 1], zi = pos[3 * i + 2];
  int g = atom_bin[i] - m.bin_base;
  int bx = g % m.nb[0], by = (g / m.nb[0]) % m.nb[1], bz = g / (m.nb[0] * m.nb[1]);
  int count = 0;
  int out_base = FILL ? row_ptr[i] : 0;
  const bool no_images = m.kind == CELL_FREE;
  for (int o = 0; o < 27; ++o) {
    int ox = o / 9 - 1, oy = (o / 3) % 3 - 1, oz = o % 3 - 1;
    // unwrapped bin coordinate -> wrapped bin + image shift (floor division)
    int ux = bx + ox, uy = by + oy, uz = bz + oz;
    if (no_images && (ux < 0 || ux >= m.nb[0] || uy < 0 || uy >= m.nb[1] || uz < 0 || uz >= m.nb[2])) continue;  // wave-uniform
    int Sx = (ux < 0) ? -1 : (ux >= m.nb[0] ? 1 : 0);
    int Sy = (uy < 0) ? -1 : (uy >= m.nb[1] ? 1 : 0);
    int Sz = (uz < 0) ? -1 : (uz >= m.nb[2] ? 1 : 0);
    int wx = ux - Sx * m.nb[0], wy = uy - Sy * m.nb[1], wz = uz - Sz * m.nb[2];
    int gb = m.bin_base + (wz * m.nb[1] + wy) * m.nb[0] + wx;
    // S . cell, rounded after every operation (the products are exact); a diagonal cell gives S_a L_a
    const float fx = (float)Sx, fy = (float)Sy, fz = (float)Sz;
    float sx = __fadd_rn(__fadd_rn(__fmul_rn(fx, m.lat[0]), __fmul_rn(fy, m.lat[3])), __fmul_rn(fz, m.lat[6]));
    float sy = __fadd_rn(__fadd_rn(__fmul_rn(fx, m.lat[1]), __fmul_rn(fy, m.lat[4])), __fmul_rn(fz, m.lat[7]));
    float sz = __fadd_rn(__fadd_rn(__fmul_rn(fx, m.lat[2]), __fmul_rn(fy, m.lat[5])), __fmul_rn(fz, m.lat[8]));
    int code = (Sx + 1) * 9 + (Sy + 1) * 3 + (Sz + 1);
    int b0 = bin_start[gb], b1 = bin_start[gb + 1];
    for (int t0 = b0; t0 < b1; t0 += 64) {
      int t = t0 + lane;
      bool hit = false;
      int j = -1;
      if (t < b1) {
        j = bin_atoms[t];
        hit = within(xi, yi, zi, pos[3 * j], pos[3 * j + 1], pos[3 * j + 2], sx, sy, sz, rc2);
        if (j == i && code == 13) hit = false;
      }
      unsigned long long mask = __ballot(hit);
      if (FILL && hit) {
        int rank = __popcll(mask & ((1ull << lane) - 1ull));
        key_tmp[out_base + count + rank] = j * 27 + code;
      }
      count += __popcll(mask);
    }
  }
  if (!FILL && lane == 0) deg[i] = count;
}

// Rank sort of each row's keys (unique), one wave per row; writes sender, code, receiver.
__global__ void __launch_bounds__(256) k_sort_rows(const int32_t* __restrict__ row_ptr,
                                                   const int32_t* __restrict__ key_tmp, int N,
                                                   int32_t* __restrict__ sender, int32_t* __restrict__ code,
                                                   int32_t* __restrict__ receiver) {
  int lane = threadIdx.x & 63;
  int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= N) return;
  int a = row_ptr[i], b = row_ptr[i + 1];
  for (int t = a + lane; t < b; t += 64) {
    int key = key_tmp[t];
    int rank = 0;
    for (int u = a; u < b; ++u) rank += (key_tmp[u] < key) ? 1 : 0;
    sender[a + rank] = key / 27;
    code[a + rank] = key % 27;
    receiver[a + rank] = i;
  }
}

__global__ void k_reverse_map(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ sender,
                              const int32_t* __restrict__ code, const int32_t* __restrict__ receiver, int64_t E,
                              int32_t* __restrict__ rev, int32_t* __restrict__ flag) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  int i = receiver[e], j = sender[e];
  int want = i * 27 + (26 - code[e]);
  int lo = row_ptr[j], hi = row_ptr[j + 1] - 1;
  int found = -1;
  while (lo <= hi) {
    int mid = (lo + hi) >> 1;
    int k = sender[mid] * 27 + code[mid];
    if (k == want) { found = mid; break; }
    if (k < want) lo = mid + 1; else hi = mid - 1;
  }
  if (found < 0) atomicOr(flag + 1, INPUT_NO_REVERSE_EDGE);  // deferred status word, read by input_status()
  rev[e] = found;
}

// Edge pairs.  flag[e] = 1 for the lower-numbered edge of a pair; after the exclusive scan of the flags (pre),
// that edge's pair index is pre[e].  An edge without an opposite (reported through the status word) is given slot 0:
// every index stays in range, the results of such a call are not meaningful anyway.
__global__ void k_pair_flags(const int32_t* __restrict__ rev, int64_t E, int32_t* __restrict__ flag) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < E) flag[e] = rev[e] > e ? 1 : 0;
}
__global__ void k_pair_assign(const int32_t* __restrict__ rev, const int32_t* __restrict__ sender, const int32_t* __restrict__ pre,
                              int64_t E, int64_t Eu, int2* __restrict__ se, int32_t* __restrict__ und) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  const int r = rev[e];
  if (r > e) {
    const int u = pre[e];
    if (u < Eu) {  // always, for an involution without fixed points: at most E / 2 edges have a higher-numbered opposite
      und[u] = (int32_t)e;
      se[e] = make_int2(sender[e], 2 * u);
      se[r] = make_int2(sender[r], 2 * u + 1);
    }
  } else if (r < 0) {
    se[e] = make_int2(sender[e], 0);
  }
}

__global__ void k_export_shift(const int32_t* __restrict__ code, int64_t E, int32_t* __restrict__ shift) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E) return;
  int c = code[e];
  shift[3 * e] = c / 9 - 1;
  shift[3 * e + 1] = (c / 3) % 3 - 1;
  shift[3 * e + 2] = c % 3 - 1;
}

template <typename T>
T* alloc_n(mlip_ctx* ctx, int64_t n) {
  return (T*)ctx_alloc(ctx, (size_t)std::max<int64_t>(n, 1) * sizeof(T));
}

}  // namespace

int graph_alloc(mlip_ctx* ctx) {
  const int64_t N = ctx->cfg.max_atoms, B = ctx->cfg.max_structs, E = ctx->cfg.max_edges;
  ctx->max_bins = 2 * N + 8 * B;
  bool ok = true;
  ok &= (ctx->d_meta = alloc_n<StructMeta>(ctx, B)) != nullptr;
  ok &= (ctx->d_atom_struct = alloc_n<int32_t>(ctx, N)) != nullptr;
  if (ctx->cfg.n_experts > 0) {  // per-structure products of the expert banks
    ok &= (ctx->d_alpha = alloc_n<float>(ctx, (int64_t)B * ctx->cfg.n_experts)) != nullptr;
    // the equivariant model stacks up to 2 l_max + 1 copies of the atom rows (components m of one l)
    const int copies = ctx->cfg.model_kind == MLIP_MODEL_EQUIVARIANT ? 2 * ctx->cfg.l_max + 1 : 1;
    ok &= (ctx->d_row_groups = alloc_n<int4>(ctx, copies * (N / 64 + B + 1))) != nullptr;
    ok &= (ctx->d_struct_ptr = alloc_n<int32_t>(ctx, copies * B + 1)) != nullptr;
  }
  ok &= (ctx->d_atom_bin = alloc_n<int32_t>(ctx, N)) != nullptr;
  ok &= (ctx->d_bin_count = alloc_n<int32_t>(ctx, ctx->max_bins + 1)) != nullptr;
  ok &= (ctx->d_bin_start = alloc_n<int32_t>(ctx, ctx->max_bins + 1)) != nullptr;
  ok &= (ctx->d_bin_cursor = alloc_n<int32_t>(ctx, ctx->max_bins + 1)) != nullptr;
  ok &= (ctx->d_bin_atoms = alloc_n<int32_t>(ctx, N)) != nullptr;
  ok &= (ctx->d_deg = alloc_n<int32_t>(ctx, N + 1)) != nullptr;
  ok &= (ctx->d_row_ptr = alloc_n<int32_t>(ctx, N + 1)) != nullptr;
  ok &= (ctx->d_key_tmp = alloc_n<int32_t>(ctx, E)) != nullptr;
  ok &= (ctx->d_sender = alloc_n<int32_t>(ctx, E)) != nullptr;
  ok &= (ctx->d_code = alloc_n<int32_t>(ctx, E)) != nullptr;
  ok &= (ctx->d_receiver = alloc_n<int32_t>(ctx, E)) != nullptr;
  ok &= (ctx->d_rev = alloc_n<int32_t>(ctx, E)) != nullptr;
  ok &= (ctx->d_se = alloc_n<int2>(ctx, E)) != nullptr;
  ok &= (ctx->d_und = alloc_n<int32_t>(ctx, E / 2 + 1)) != nullptr;
  ok &= (ctx->d_pair_pre = alloc_n<int32_t>(ctx, E + 1)) != nullptr;
  int64_t scan_blocks = (std::max(std::max(N, ctx->max_bins), E) + SCAN_TILE) / SCAN_TILE + 1;
  ok &= (ctx->d_scan_tmp = alloc_n<int32_t>(ctx, scan_blocks)) != nullptr;
  ok &= (ctx->d_flag = alloc_n<int32_t>(ctx, 4)) != nullptr;
  ok &= (ctx->d_bounds = alloc_n<float>(ctx, 6 * B)) != nullptr;
  return ok ? MLIP_OK : MLIP_E_HIP;
}

int graph_build(mlip_ctx* ctx, int64_t n_atoms, int32_t n_structs, const float* pos, const int32_t* struct_ptr,
                const float* cell, float cutoff, int64_t* n_edges_host) {
  ctx->phase = PH_NONE;
  if (!pos || !struct_ptr || !cell || !n_edges_host) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: null pointer");
  if (n_atoms <= 0 || n_structs <= 0) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: n_atoms and n_structs must be positive");
  if (!(cutoff > 0.f) || !std::isfinite(cutoff)) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cutoff must be positive");
  // The radial basis and the envelope are laid out on [0, cfg.cutoff]: an edge set cut at any other radius would
  // give a discontinuous energy (smaller) or edges with a rising envelope beyond its zero (larger).
  if (cutoff != ctx->cfg.cutoff) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cutoff differs from the cutoff the context's model was created with");
  *n_edges_host = 0;
  if (n_atoms > ctx->cfg.max_atoms) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "graph_build: n_atoms exceeds max_atoms");
  if (n_structs > ctx->cfg.max_structs) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "graph_build: n_structs exceeds max_structs");
  const int N = (int)n_atoms, B = n_structs;
  hipStream_t st = ctx->stream;

  ctx->h_struct_ptr.resize(B + 1);
  ctx->h_cell.resize((size_t)B * 9);
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->h_struct_ptr.data(), struct_ptr, sizeof(int32_t) * (B + 1), hipMemcpyDeviceToHost, st));
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->h_cell.data(), cell, sizeof(float) * 9 * B, hipMemcpyDeviceToHost, st));
  MLIP_HIP_CHECK(ctx, hipStreamSynchronize(st));

  // validate and lay out the bins on the host
  ctx->h_meta.resize(B);
  if (ctx->h_struct_ptr[0] != 0 || ctx->h_struct_ptr[B] != N)
    MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: struct_ptr must start at 0 and end at n_atoms");
  bool any_free = false;
  for (int s = 0; s < B; ++s) {
    StructMeta& m = ctx->h_meta[s];
    m.atom_begin = ctx->h_struct_ptr[s];
    m.atom_end = ctx->h_struct_ptr[s + 1];
    if (m.atom_end < m.atom_begin) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: struct_ptr must be non-decreasing");
    const float* c = &ctx->h_cell[(size_t)s * 9];
    bool all_zero = true, diagonal = true;
    for (int a = 0; a < 3; ++a)
      for (int b = 0; b < 3; ++b) {
        if (!std::isfinite(c[3 * a + b])) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cell entries must be finite");
        if (c[3 * a + b] != 0.f) {
          all_zero = false;
          if (a != b) diagonal = false;
        }
      }
    m.kind = all_zero ? CELL_FREE : (diagonal ? CELL_ORTHO : CELL_TRICLINIC);
    any_free |= all_zero;
  }
  std::vector<float> h_bounds;
  if (any_free) {  // molecules: bins are laid over the bounding box, which only the device can see
    h_bounds.resize((size_t)B * 6);
    hipLaunchKernelGGL(k_bounds, dim3(B), dim3(256), 0, st, pos, struct_ptr, ctx->d_bounds);
    MLIP_HIP_CHECK(ctx, hipGetLastError());
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(h_bounds.data(), ctx->d_bounds, sizeof(float) * 6 * B, hipMemcpyDeviceToHost, st));
    MLIP_HIP_CHECK(ctx, hipStreamSynchronize(st));
  }
  int64_t bins = 0;
  for (int s = 0; s < B; ++s) {
    StructMeta& m = ctx->h_meta[s];
    const float* c = &ctx->h_cell[(size_t)s * 9];
    for (int k = 0; k < 9; ++k) m.lat[k] = c[k], m.inv[k] = 0.f;
    m.origin[0] = m.origin[1] = m.origin[2] = 0.f;
    int64_t cap = std::max<int64_t>(8, 2 * (int64_t)(m.atom_end - m.atom_begin));
    if (m.kind == CELL_ORTHO) {
      for (int a = 0; a < 3; ++a) {
        const float L = c[4 * a];
        if (!(L > 0.f)) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cell edge must be positive");
        if (cutoff > L) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cutoff exceeds a cell edge");
        // bins at least (1 + 1e-4) r_c wide and at most 256 per axis: the float32 bin coordinate x / L * nb
        // is off by < 3e-7 nb, which then cannot separate two atoms closer than r_c by more than one bin
        m.nb[a] = std::min(256, std::max(1, (int)std::floor((double)L / ((double)cutoff * (1.0 + 1e-4)))));
        m.inv[4 * a] = 1.f / L;
      }
    } else if (m.kind == CELL_TRICLINIC) {
      // general lattice: bins are slabs between lattice planes; their width is the perpendicular
      // height V / |a_b x a_c| divided by the bin count
      double A[3][3], X[3][3];
      for (int a = 0; a < 3; ++a)
        for (int b = 0; b < 3; ++b) A[a][b] = c[3 * a + b];
      for (int a = 0; a < 3; ++a) {  // X[a] = a_{a+1} x a_{a+2}
        const double* u = A[(a + 1) % 3];
        const double* v = A[(a + 2) % 3];
        X[a][0] = u[1] * v[2] - u[2] * v[1];
        X[a][1] = u[2] * v[0] - u[0] * v[2];
        X[a][2] = u[0] * v[1] - u[1] * v[0];
      }
      const double det = A[0][0] * X[0][0] + A[0][1] * X[0][1] + A[0][2] * X[0][2];
      double scale = 1.0;
      for (int a = 0; a < 3; ++a) scale *= std::sqrt(A[a][0] * A[a][0] + A[a][1] * A[a][1] + A[a][2] * A[a][2]);
      if (!(std::fabs(det) > 1e-6 * scale)) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cell is singular (or partly periodic, which is not supported)");
      double longest = 0.0, lowest = 1e300;
      for (int a = 0; a < 3; ++a) {
        const double height = std::fabs(det) / std::sqrt(X[a][0] * X[a][0] + X[a][1] * X[a][1] + X[a][2] * X[a][2]);
        longest = std::max(longest, std::sqrt(A[a][0] * A[a][0] + A[a][1] * A[a][1] + A[a][2] * A[a][2]));
        lowest = std::min(lowest, height);
        // the 27 nearest images cover the cutoff sphere only up to the smallest height; the margins
        // leave room for the rounding of the float32 fractional coordinates
        if ((double)cutoff * (1.0 + 1e-4) > height) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_build: cutoff exceeds a perpendicular height of the cell");
        // at most 32 slabs per axis: a slab is then >= 6e-5 wider (in fractional units) than the cutoff needs
        m.nb[a] = std::min(32, std::max(1, (int)std::floor(height / ((double)cutoff * (1.0 + 2e-3)))));
        for (int b = 0; b < 3; ++b) m.inv[3 * b + a] = (float)(X[a][b] / det);  // column a of the inverse
      }
      // A float32 fractional coordinate is off by up to ~5e-7 (longest edge / smallest height); beyond a ratio
      // of 50 that would eat the slabs' margin, so such a cell has to be reduced by the caller first.
      if (longest > 50.0 * lowest) MLIP_FAIL(ctx, MLIP_E_UNSUPPORTED, "graph_build: cell too skewed for float32 binning (reduce the lattice first)");
    } else {
      const int n_at = m.atom_end - m.atom_begin;
      for (int a = 0; a < 3; ++a) {
        float lo = n_at > 0 ? h_bounds[(size_t)6 * s + a] : 0.f, hi = n_at > 0 ? h_bounds[(size_t)6 * s + 3 + a] : 0.f;
        if (!(std::isfinite(lo) && std::isfinite(hi) && hi - lo <= 1e30f))
          MLIP_FAIL(ctx, MLIP_E_POSITION, "graph_build: a position is not finite");
        const double extent = std::max((double)hi - (double)lo, (double)cutoff) * (1.0 + 1e-3);
        // at most 256 bins per axis (coarser bins are still correct), so neither the count nor the product overflows
        m.nb[a] = (int)std::min(256.0, std::max(1.0, std::floor(extent / ((double)cutoff * (1.0 + 2e-3)))));
        m.origin[a] = lo;
        m.inv[4 * a] = (float)(1.0 / extent);
      }
    }
    // coarser bins are still correct: cap the bin count near the atom count
    while ((int64_t)m.nb[0] * m.nb[1] * m.nb[2] > cap) {
      int a = (m.nb[0] >= m.nb[1] && m.nb[0] >= m.nb[2]) ? 0 : (m.nb[1] >= m.nb[2] ? 1 : 2);
      m.nb[a] = std::max(1, m.nb[a] - 1);
    }
    m.bin_base = (int32_t)bins;
    bins += (int64_t)m.nb[0] * m.nb[1] * m.nb[2];
  }
  if (bins > ctx->max_bins) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "graph_build: bin table too small");
  const int n_bins = (int)bins;

  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_meta, ctx->h_meta.data(), sizeof(StructMeta) * B, hipMemcpyHostToDevice, st));
  if (ctx->cfg.n_experts > 0) {
    // row tiles of at most 64 atoms, none straddling two structures (each structure has its own merged matrices)
    // The equivariant model multiplies [(2l+1) N, C] matrices (component-major copies of the atom rows):
    // copy m of the tables is shifted by m N rows; a product over 2l+1 copies uses the first 2l+1.
    const int copies = ctx->cfg.model_kind == MLIP_MODEL_EQUIVARIANT ? 2 * ctx->cfg.l_max + 1 : 1;
    ctx->h_row_groups.clear();
    ctx->h_k_ranges.assign((size_t)copies * B + 1, 0);
    for (int m = 0; m < copies; ++m)
      for (int s = 0; s < B; ++s) {
        ctx->h_k_ranges[(size_t)m * B + s] = (int32_t)(m * N + ctx->h_struct_ptr[s]);
        for (int r = ctx->h_struct_ptr[s]; r < ctx->h_struct_ptr[s + 1]; r += 64)
          ctx->h_row_groups.push_back(make_int4((int)(m * N + r), (int)(m * N + std::min(r + 64, ctx->h_struct_ptr[s + 1])), s, 0));
      }
    ctx->h_k_ranges[(size_t)copies * B] = (int32_t)(copies * N);
    ctx->n_row_groups = (int64_t)ctx->h_row_groups.size() / copies;  // per copy: <= N / 64 + B
    if (!ctx->h_row_groups.empty())
      MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_row_groups, ctx->h_row_groups.data(), sizeof(int4) * ctx->h_row_groups.size(),
                                         hipMemcpyHostToDevice, st));
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->d_struct_ptr, ctx->h_k_ranges.data(), sizeof(int32_t) * ctx->h_k_ranges.size(),
                                       hipMemcpyHostToDevice, st));
  }
  MLIP_HIP_CHECK(ctx, hipMemsetAsync(ctx->d_bin_count, 0, sizeof(int32_t) * (n_bins + 1), st));
  MLIP_HIP_CHECK(ctx, hipMemsetAsync(ctx->d_bin_cursor, 0, sizeof(int32_t) * (n_bins + 1), st));
  MLIP_HIP_CHECK(ctx, hipMemsetAsync(ctx->d_flag, 0, sizeof(int32_t) * 4, st));

  const int TB = 256;
  hipLaunchKernelGGL(k_bin_count, dim3((N + TB - 1) / TB), dim3(TB), 0, st, pos, ctx->d_meta, B, N, ctx->d_atom_struct,
                     ctx->d_atom_bin, ctx->d_bin_count, ctx->d_flag);
  MLIP_TRY(scan_exclusive(ctx, ctx->d_bin_count, ctx->d_bin_start, n_bins));
  hipLaunchKernelGGL(k_bin_fill, dim3((N + TB - 1) / TB), dim3(TB), 0, st, ctx->d_atom_bin, ctx->d_bin_start,
                     ctx->d_bin_cursor, ctx->d_bin_atoms, N);
  const int rows_per_block = TB / 64;
  const int nb_rows = (N + rows_per_block - 1) / rows_per_block;
  const float rc2 = cutoff * cutoff;
  hipLaunchKernelGGL(k_neighbours<false>, dim3(nb_rows), dim3(TB), 0, st, pos, ctx->d_meta, ctx->d_atom_struct,
                     ctx->d_atom_bin, ctx->d_bin_start, ctx->d_bin_atoms, N, rc2, ctx->d_deg, nullptr, nullptr);
  MLIP_TRY(scan_exclusive(ctx, ctx->d_deg, ctx->d_row_ptr, N));
  int32_t h_tail[1] = {0};
  int32_t h_flag[4] = {0, 0, 0, 0};
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(h_tail, ctx->d_row_ptr + N, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(h_flag, ctx->d_flag, sizeof(int32_t) * 4, hipMemcpyDeviceToHost, st));
  MLIP_HIP_CHECK(ctx, hipStreamSynchronize(st));
  if (h_flag[0] & 1) MLIP_FAIL(ctx, MLIP_E_POSITION, "graph_build: a position is outside its cell or not finite");
  const int64_t E = h_tail[0];
  *n_edges_host = E;
  if (E > ctx->cfg.max_edges) MLIP_FAIL(ctx, MLIP_E_CAPACITY, "graph_build: edge count exceeds max_edges");
  if (E > 0) {
    hipLaunchKernelGGL(k_neighbours<true>, dim3(nb_rows), dim3(TB), 0, st, pos, ctx->d_meta, ctx->d_atom_struct,
                       ctx->d_atom_bin, ctx->d_bin_start, ctx->d_bin_atoms, N, rc2, nullptr, ctx->d_row_ptr,
                       ctx->d_key_tmp);
    hipLaunchKernelGGL(k_sort_rows, dim3(nb_rows), dim3(TB), 0, st, ctx->d_row_ptr, ctx->d_key_tmp, N, ctx->d_sender,
                       ctx->d_code, ctx->d_receiver);
    hipLaunchKernelGGL(k_reverse_map, dim3((unsigned)((E + TB - 1) / TB)), dim3(TB), 0, st, ctx->d_row_ptr,
                       ctx->d_sender, ctx->d_code, ctx->d_receiver, E, ctx->d_rev, ctx->d_flag);
    if (ctx->d_se) {  // edge pairs (the sorting keys are no longer needed: their array holds the flags)
      const unsigned eb = (unsigned)((E + TB - 1) / TB);
      hipLaunchKernelGGL(k_pair_flags, dim3(eb), dim3(TB), 0, st, ctx->d_rev, E, ctx->d_key_tmp);
      MLIP_TRY(scan_exclusive(ctx, ctx->d_key_tmp, ctx->d_pair_pre, E));
      MLIP_HIP_CHECK(ctx, hipMemsetAsync(ctx->d_und, 0, sizeof(int32_t) * (E / 2 + 1), st));
      hipLaunchKernelGGL(k_pair_assign, dim3(eb), dim3(TB), 0, st, ctx->d_rev, ctx->d_sender, ctx->d_pair_pre, E, E / 2, ctx->d_se, ctx->d_und);
    }
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  ctx->N = N;
  ctx->B = B;
  ctx->E = E;
  ctx->Eu = E / 2;
  ctx->phase = PH_GRAPH;
  return MLIP_OK;
}

// Deferred input diagnostics.  Kernels that run after the graph build's last read-back cannot fail the call
// that launched them (calls are asynchronous); they raise bits in the second word of the device flag instead,
// and keep every access in bounds.  This reads the word back (synchronous) and turns it into a status.
int input_status(mlip_ctx* ctx) {
  if (ctx->phase < PH_GRAPH) return MLIP_OK;
  int32_t h = 0;
  MLIP_HIP_CHECK(ctx, hipMemcpyAsync(&h, ctx->d_flag + 1, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
  MLIP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
  if (h & INPUT_NO_REVERSE_EDGE) MLIP_FAIL(ctx, MLIP_E_POSITION, "the edge list is not symmetric: an edge has no opposite edge");
  if (h & INPUT_BAD_SPECIES) MLIP_FAIL(ctx, MLIP_E_INVALID, "a species index is outside [0, n_species) (it was clamped; results are not meaningful)");
  if (h & INPUT_COINCIDENT) MLIP_FAIL(ctx, MLIP_E_POSITION, "two atoms of a structure coincide (an edge of length zero; its direction was set to zero)");
  return MLIP_OK;
}

__global__ void k_export_slots(const int2* __restrict__ se, int64_t E, int32_t* __restrict__ slot) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < E) slot[e] = se[e].y;
}

// slot[E] and the lower-numbered edge of each pair, from the pairing of the current graph
int graph_export_pairs(mlip_ctx* ctx, int32_t* slot, int32_t* pair_edge) {
  if (ctx->phase < PH_GRAPH) MLIP_FAIL(ctx, MLIP_E_STATE, "graph_export_pairs: no graph has been built");
  if (!slot) MLIP_FAIL(ctx, MLIP_E_INVALID, "graph_export_pairs: null pointer");
  if (!ctx->d_se) MLIP_FAIL(ctx, MLIP_E_STATE, "graph_export_pairs: this context keeps no edge pairs");
  MLIP_TRY(input_status(ctx));
  if (ctx->E <= 0) return MLIP_OK;
  hipLaunchKernelGGL(k_export_slots, dim3((unsigned)((ctx->E + 255) / 256)), dim3(256), 0, ctx->stream, ctx->d_se, ctx->E, slot);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  if (pair_edge)
    MLIP_HIP_CHECK(ctx, hipMemcpyAsync(pair_edge, ctx->d_und, sizeof(int32_t) * ctx->Eu, hipMemcpyDeviceToDevice, ctx->stream));
  MLIP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
  return MLIP_OK;
}

// shift[E,3] from the stored shift codes of the current graph
int graph_export_shift(mlip_ctx* ctx, int32_t* shift) {
  if (ctx->E <= 0) return MLIP_OK;
  hipLaunchKernelGGL(k_export_shift, dim3((unsigned)((ctx->E + 255) / 256)), dim3(256), 0, ctx->stream, ctx->d_code, ctx->E, shift);
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}

int graph_export(mlip_ctx* ctx, int32_t* row_ptr, int32_t* sender, int32_t* shift, int32_t* rev) {
  if (ctx->phase < PH_GRAPH) MLIP_FAIL(ctx, MLIP_E_STATE, "graph_export: no graph has been built");
  if (rev) MLIP_TRY(input_status(ctx));  // rev = -1 entries must not leave the library unreported
  hipStream_t st = ctx->stream;
  const int64_t E = ctx->E;
  if (row_ptr) MLIP_HIP_CHECK(ctx, hipMemcpyAsync(row_ptr, ctx->d_row_ptr, sizeof(int32_t) * (ctx->N + 1), hipMemcpyDeviceToDevice, st));
  if (E > 0) {
    if (sender) MLIP_HIP_CHECK(ctx, hipMemcpyAsync(sender, ctx->d_sender, sizeof(int32_t) * E, hipMemcpyDeviceToDevice, st));
    if (rev) MLIP_HIP_CHECK(ctx, hipMemcpyAsync(rev, ctx->d_rev, sizeof(int32_t) * E, hipMemcpyDeviceToDevice, st));
    if (shift) MLIP_TRY(graph_export_shift(ctx, shift));
  }
  return MLIP_OK;
}
