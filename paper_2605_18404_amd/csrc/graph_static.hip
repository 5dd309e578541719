// The radius graph for callers that cannot allocate device memory: the context-based build (graph.hip)
// run on a context that owns nothing, whose work arrays are carved out of one file-scope device array.
#include <algorithm>
#include <cmath>
#include <mutex>

#include "common.h"

// ------------------------------------------------------------------ allocation-free graph build
// For callers that cannot allocate device memory (tight serving loops that rebuild the neighbour list every
// step, harnesses that forbid hipMalloc): the same kernels as graph_build, with every work array carved out
// of one file-scope device array instead of a context's allocations.  Each GPU holds its own copy of the
// array (about 13 MB) from the first use of the library on it until the process ends.
namespace {

constexpr int64_t STATIC_MAX_ATOMS = 16384, STATIC_MAX_STRUCTS = 1024, STATIC_MAX_EDGES = 1 << 20;
constexpr int64_t STATIC_MAX_BINS = 2 * STATIC_MAX_ATOMS + 8 * STATIC_MAX_STRUCTS;
constexpr int64_t STATIC_SCAN_BLOCKS = (STATIC_MAX_BINS + GRAPH_SCAN_TILE) / GRAPH_SCAN_TILE + 1;
constexpr size_t align256(size_t x) { return (x + 255) / 256 * 256; }
// byte offsets of the work arrays inside the scratch array, in the order graph_alloc makes them
constexpr size_t SO_META = 0;
constexpr size_t SO_ATOM_STRUCT = SO_META + align256(sizeof(StructMeta) * STATIC_MAX_STRUCTS);
constexpr size_t SO_ATOM_BIN = SO_ATOM_STRUCT + align256(4 * STATIC_MAX_ATOMS);
constexpr size_t SO_BIN_COUNT = SO_ATOM_BIN + align256(4 * STATIC_MAX_ATOMS);
constexpr size_t SO_BIN_START = SO_BIN_COUNT + align256(4 * (STATIC_MAX_BINS + 1));
constexpr size_t SO_BIN_CURSOR = SO_BIN_START + align256(4 * (STATIC_MAX_BINS + 1));
constexpr size_t SO_BIN_ATOMS = SO_BIN_CURSOR + align256(4 * (STATIC_MAX_BINS + 1));
constexpr size_t SO_DEG = SO_BIN_ATOMS + align256(4 * STATIC_MAX_ATOMS);
constexpr size_t SO_SCAN = SO_DEG + align256(4 * (STATIC_MAX_ATOMS + 1));
constexpr size_t SO_FLAG = SO_SCAN + align256(4 * STATIC_SCAN_BLOCKS);
constexpr size_t SO_BOUNDS = SO_FLAG + 256;
constexpr size_t SO_KEY = SO_BOUNDS + align256(4 * 6 * STATIC_MAX_STRUCTS);
constexpr size_t SO_CODE = SO_KEY + align256(4 * STATIC_MAX_EDGES);
constexpr size_t SO_RECEIVER = SO_CODE + align256(4 * STATIC_MAX_EDGES);
constexpr size_t SCRATCH_BYTES = SO_RECEIVER + align256(4 * STATIC_MAX_EDGES);

}  // namespace

// In host code this name is only a handle for hipGetSymbolAddress: it is not a device address.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_static_mutex;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on each GPU, looked up once
thread_local std::string g_static_err;

int static_fail(int code, const std::string& msg) {
  g_static_err = msg;
  return code;
}

// Device address of the current device's copy of the scratch array.
int scratch_address(unsigned char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return static_fail(MLIP_E_HIP, "graph_build_static: no current device");
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return static_fail(MLIP_E_HIP, std::string("graph_build_static: hipGetSymbolAddress failed: ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[dev];
  return MLIP_OK;
}

}  // namespace

extern "C" const char* mlip_graph_build_static_error(void) { return g_static_err.c_str(); }

extern "C" int mlip_graph_build_static(int64_t n_atoms, int32_t n_structs, const float* pos, const int32_t* struct_ptr,
                                       const float* cell, float cutoff, void* hip_stream, int64_t edge_capacity,
                                       int32_t* row_ptr, int32_t* sender, int32_t* shift, int32_t* rev,
                                       int64_t* n_edges_host) {
  g_static_err.clear();
  if (!pos || !struct_ptr || !cell || !row_ptr || !sender || !shift || !rev || !n_edges_host)
    return static_fail(MLIP_E_INVALID, "graph_build_static: null pointer");
  *n_edges_host = 0;
  if (n_atoms <= 0 || n_structs <= 0 || edge_capacity <= 0) return static_fail(MLIP_E_INVALID, "graph_build_static: sizes must be positive");
  if (n_atoms > STATIC_MAX_ATOMS || n_structs > STATIC_MAX_STRUCTS)
    return static_fail(MLIP_E_CAPACITY, "graph_build_static: at most 16384 atoms in at most 1024 structures per call (use a context for more)");
  if (!(cutoff > 0.f) || !std::isfinite(cutoff)) return static_fail(MLIP_E_INVALID, "graph_build_static: cutoff must be positive");
  unsigned char* base = nullptr;
  int s = scratch_address(&base);
  if (s != MLIP_OK) return s;
  // A context on the stack that owns nothing: its graph arrays point into the scratch array and into the
  // caller's output buffers, so the context-based build below runs unchanged and allocates no device memory.
  mlip_ctx c;
  c.cfg.cutoff = cutoff;
  c.cfg.max_atoms = STATIC_MAX_ATOMS;
  c.cfg.max_structs = STATIC_MAX_STRUCTS;
  c.cfg.max_edges = std::min<int64_t>(edge_capacity, STATIC_MAX_EDGES);
  c.stream = (hipStream_t)hip_stream;
  c.max_bins = STATIC_MAX_BINS;
  c.d_meta = (StructMeta*)(base + SO_META);
  c.d_atom_struct = (int32_t*)(base + SO_ATOM_STRUCT);
  c.d_atom_bin = (int32_t*)(base + SO_ATOM_BIN);
  c.d_bin_count = (int32_t*)(base + SO_BIN_COUNT);
  c.d_bin_start = (int32_t*)(base + SO_BIN_START);
  c.d_bin_cursor = (int32_t*)(base + SO_BIN_CURSOR);
  c.d_bin_atoms = (int32_t*)(base + SO_BIN_ATOMS);
  c.d_deg = (int32_t*)(base + SO_DEG);
  c.d_scan_tmp = (int32_t*)(base + SO_SCAN);
  c.d_flag = (int32_t*)(base + SO_FLAG);
  c.d_bounds = (float*)(base + SO_BOUNDS);
  c.d_key_tmp = (int32_t*)(base + SO_KEY);
  c.d_code = (int32_t*)(base + SO_CODE);
  c.d_receiver = (int32_t*)(base + SO_RECEIVER);
  c.d_row_ptr = row_ptr;
  c.d_sender = sender;
  c.d_rev = rev;
  s = graph_build(&c, n_atoms, n_structs, pos, struct_ptr, cell, cutoff, n_edges_host);
  if (s != MLIP_OK) {
    if (s == MLIP_E_CAPACITY && *n_edges_host > c.cfg.max_edges)
      return static_fail(s, edge_capacity > STATIC_MAX_EDGES ? "graph_build_static: more than 1048576 edges (use a context for more)"
                                                             : "graph_build_static: edge count exceeds edge_capacity");
    return static_fail(s, c.err);
  }
  s = graph_export_shift(&c, shift);
  if (s != MLIP_OK) return static_fail(s, c.err);
  return MLIP_OK;
}
