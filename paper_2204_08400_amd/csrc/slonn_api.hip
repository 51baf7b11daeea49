// Host side of libslonn: argument validation, handles, the table blob, workspace
// carving and the per-layer launch sequence.  No arithmetic of the method lives here.
#include <algorithm>
#include <cstring>
#include <new>
#include <string>

#include "slonn_internal.h"

// Scratch memory of slonn_sparse_forward_static: one array per device, placed by the loader when the
// code object reaches that device and held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the address kernels may use is what that call returns,
// looked up once per device with that device current.
static __device__ __align__(256) unsigned char scratch[SLONN_STATIC_SCRATCH_BYTES];

namespace slonn {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

namespace {
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> start, stop;
  std::vector<int> kind;
  size_t used = 0;
} g_prof;
}  // namespace

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};
}  // namespace

// Device address of the current device's scratch array (looked up on first use per device).
int static_scratch(void** out) {
  int dev = 0;
  SLONN_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) SLONN_FAIL(SLONN_EUNSUPPORTED, "device ordinal %d beyond %d", dev, MAX_DEVICES);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    SLONN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) SLONN_FAIL(SLONN_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SLONN_OK;
}

ProfScope::ProfScope(int kind, hipStream_t s) : slot(-1), stream(s) {
  if (!g_prof.on || g_prof.used >= g_prof.start.size()) return;
  slot = (int)g_prof.used++;
  g_prof.kind[slot] = kind;
  (void)hipEventRecord(g_prof.start[slot], stream);
}
ProfScope::~ProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], stream);
}

namespace {

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// from this batch on the hash projections run on the int8 matrix cores (below it the fp64 kernels
// are latency-bound anyway and the slicing pass does not pay; C3 hash per step, fp64 against int8:
// batch 128 49 / 88 us, 192 60 / 91, 256 118 / 94, 384 120 / 105)
constexpr int HASH_INT_MIN_BATCH = 256;
// ... and from batch 64 on where the projection is large (C5, 768 hash rows of 8192 elements, at
// batch 128: 64 us per layer on the fp64 cores)
constexpr int HASH_INT_MIN_BATCH_LARGE = 64;
constexpr long long HASH_INT_LARGE_WORK = 1ll << 29;      // batch x hash rows x row length
inline bool hash_int_pays(int B, int H, int d) {
  return B >= HASH_INT_MIN_BATCH || (B >= HASH_INT_MIN_BATCH_LARGE && (long long)B * H * d >= HASH_INT_LARGE_WORK);
}

// up to GATHER_ROW_MAX_BATCH queries the selected rows are fetched by one workgroup each
// (launch_gather_forward); beyond it large layers are walked in row blocks shared between the
// queries (C3 keep .25, whole step: batch 2 71 against 97 us, batch 4 86 against 103, batch 6 107
// against 112, batch 8 122 against 114)
constexpr int ROW_BLOCK_MIN_BATCH = GATHER_ROW_MAX_BATCH + 1;

// Carves the caller's workspace into the per-batch buffers of the forward pass.
struct Workspace {
  float* act[2] = {nullptr, nullptr};   // ping-pong layer outputs [B][max_n]
  float* z = nullptr;                   // [B][max_H]
  int32_t* active = nullptr;            // [B][max_n_activated]
  int32_t* cnt = nullptr;               // [B]
  int32_t* order = nullptr;             // [B] queries by descending budget
  int32_t* part_idx = nullptr;          // [B][max_n_activated] lists regrouped by row block
  int32_t* part_pos = nullptr;          // [B][max_n_activated]
  int32_t* blk_off = nullptr;           // [B][MAX_ROW_BLOCKS + 1]
  void* grouped = nullptr;              // union lists of the grouped evaluation
  void* tiles = nullptr;                // pair masks and split activations of the masked tiles
  size_t tiles_bytes = 0;
  void* hash_int = nullptr;             // digits of the activations and partial sums of the integer hash
  void* hash_split = nullptr;           // partial sums of the split hash projection
  void* dense_split = nullptr;          // partial sums of a skinny dense layer's split reduction
  size_t bytes = 0;
  int max_n = 0, max_H = 0, max_na = 0;
};

void plan_workspace(const slonn_model* m, int B, char* base, Workspace* w) {
  int max_n = 0, max_H = 0, max_na = 0, d_bf16 = 0;
  for (const Layer& l : m->layers) {
    max_n = std::max(max_n, l.d_out);
    if (l.activated()) {
      max_H = std::max(max_H, l.H());
      max_na = std::max(max_na, l.d_out);
      if (l.w_dtype == SLONN_BF16) d_bf16 = std::max(d_bf16, l.d_in);
    }
  }
  w->max_n = max_n; w->max_H = max_H; w->max_na = max_na;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return p;
  };
  w->act[0] = reinterpret_cast<float*>(take((size_t)B * max_n * 4));
  w->act[1] = reinterpret_cast<float*>(take((size_t)B * max_n * 4));
  w->z = reinterpret_cast<float*>(take((size_t)B * std::max(max_H, 1) * 4));
  w->active = reinterpret_cast<int32_t*>(take((size_t)B * std::max(max_na, 1) * 4));
  w->cnt = reinterpret_cast<int32_t*>(take((size_t)B * 4));
  w->order = reinterpret_cast<int32_t*>(take((size_t)B * 4));
  w->part_idx = reinterpret_cast<int32_t*>(take((size_t)B * std::max(max_na, 1) * 4));
  w->part_pos = reinterpret_cast<int32_t*>(take((size_t)B * std::max(max_na, 1) * 4));
  w->blk_off = reinterpret_cast<int32_t*>(take((size_t)B * (MAX_ROW_BLOCKS + 1) * 4));
  w->grouped = take(grouped_workspace_bytes(B, std::max(max_na, 1), d_bf16));
  size_t tiles_bytes = 0;
  for (const Layer& l : m->layers)
    if (l.Wt && (l.activated() || B >= 256))   // (a layer computed in full goes through the tiles from batch 256)
      tiles_bytes = std::max(tiles_bytes, masked_tiles_workspace_bytes(B, l.d_out, l.d_in));
  w->tiles = tiles_bytes ? take(tiles_bytes) : nullptr;
  w->tiles_bytes = tiles_bytes;
  w->hash_split = take(hash_split_workspace_bytes());
  size_t dsplit = 0;
  for (const Layer& l : m->layers) dsplit = std::max(dsplit, dense_split_workspace_bytes(B, l.d_out, l.d_in));
  w->dense_split = dsplit ? take(dsplit) : nullptr;
  size_t hint = 0;
  if (B >= HASH_INT_MIN_BATCH_LARGE)
    for (const Layer& l : m->layers)
      if (l.Whd) hint = std::max(hint, hash_int_workspace_bytes(B, l.H(), l.d_in));
  w->hash_int = hint ? take(hint) : nullptr;
  w->bytes = off;
}

int check_input(const slonn_model* m, const slonn_input* X) {
  if (!X) SLONN_FAIL(SLONN_EINVAL, "input descriptor is null");
  if (X->format == SLONN_DENSE) {
    if (!X->x) SLONN_FAIL(SLONN_EINVAL, "dense input pointer is null");
    if (m->layers[0].w_layout != SLONN_ROWS_ARE_NODES)
      SLONN_FAIL(SLONN_EUNSUPPORTED, "dense input needs a node-major first layer");
  } else if (X->format == SLONN_ELL) {
    if (!X->idx || !X->val || !X->nnz || X->ell_stride <= 0)
      SLONN_FAIL(SLONN_EINVAL, "ELL input needs idx, val, nnz and a positive ell_stride");
    if (m->layers[0].activated())
      SLONN_FAIL(SLONN_EUNSUPPORTED, "a Node Activator on a sparse-input first layer is not supported");
  } else {
    SLONN_FAIL(SLONN_EINVAL, "unknown input format %d", X->format);
  }
  return SLONN_OK;
}

}  // namespace
}  // namespace slonn

using namespace slonn;

extern "C" {

const char* slonn_last_error(void) { return g_err; }

int slonn_profile_begin(int max_launches) {
  if (max_launches <= 0) SLONN_FAIL(SLONN_EINVAL, "max_launches must be positive");
  if (g_prof.on) SLONN_FAIL(SLONN_EINVAL, "profiling is already on");
  g_prof.start.assign(max_launches, nullptr);
  g_prof.stop.assign(max_launches, nullptr);
  g_prof.kind.assign(max_launches, 0);
  g_prof.used = 0;
  for (int i = 0; i < max_launches; ++i) {
    SLONN_HIP(hipEventCreate(&g_prof.start[i]));
    SLONN_HIP(hipEventCreate(&g_prof.stop[i]));
  }
  g_prof.on = true;
  return SLONN_OK;
}

int slonn_profile_end(double* ms_per_kind, int64_t* launches_per_kind) {
  if (!ms_per_kind || !launches_per_kind) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (!g_prof.on) SLONN_FAIL(SLONN_EINVAL, "profiling is not on");
  g_prof.on = false;
  for (int k = 0; k < SLONN_PROF_KINDS; ++k) { ms_per_kind[k] = 0.0; launches_per_kind[k] = 0; }
  int rc = SLONN_OK;
  if (hipDeviceSynchronize() != hipSuccess) { set_error("device synchronisation failed"); rc = SLONN_EHIP; }
  for (size_t i = 0; i < g_prof.start.size(); ++i) {
    if (rc == SLONN_OK && i < g_prof.used) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) == hipSuccess) {
        ms_per_kind[g_prof.kind[i]] += ms;
        launches_per_kind[g_prof.kind[i]] += 1;
      }
    }
    if (g_prof.start[i]) (void)hipEventDestroy(g_prof.start[i]);
    if (g_prof.stop[i]) (void)hipEventDestroy(g_prof.stop[i]);
  }
  g_prof.start.clear(); g_prof.stop.clear(); g_prof.kind.clear(); g_prof.used = 0;
  return rc;
}

int slonn_probe_mfma_rate(void* scratch, size_t scratch_bytes, void* stream, double* tflops) {
  if (!scratch || !tflops) SLONN_FAIL(SLONN_EINVAL, "null argument");
  int dev = 0, n_cu = 256;
  SLONN_HIP(hipGetDevice(&dev));
  (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  const int wgs = 2 * n_cu, iters = 4000;
  if (scratch_bytes < (size_t)wgs * 512 * 4) SLONN_FAIL(SLONN_ENOMEM, "scratch holds %zu bytes, %zu needed", scratch_bytes, (size_t)wgs * 512 * 4);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  SLONN_HIP(hipEventCreate(&e0));
  SLONN_HIP(hipEventCreate(&e1));
  (void)launch_mfma_rate_probe(static_cast<float*>(scratch), wgs, 200, s);       // warm-up
  SLONN_HIP(hipEventRecord(e0, s));
  const double flops = launch_mfma_rate_probe(static_cast<float*>(scratch), wgs, iters, s);
  SLONN_HIP(hipEventRecord(e1, s));
  SLONN_HIP(hipEventSynchronize(e1));
  float ms = 0.0f;
  SLONN_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  SLONN_HIP(hipGetLastError());
  *tflops = ms > 0.0f ? flops / (ms * 1e-3) / 1e12 : 0.0;
  return SLONN_OK;
}

int slonn_probe_l_two_read_rate(void* scratch, size_t scratch_bytes, void* stream, double* gbps_all_units,
                                double* gbps_one_unit) {
  if (!scratch || !gbps_all_units || !gbps_one_unit) SLONN_FAIL(SLONN_EINVAL, "null argument");
  int dev = 0, n_cu = 256;
  SLONN_HIP(hipGetDevice(&dev));
  (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  const size_t need = ((size_t)2 << 20) + (size_t)n_cu * 4096;
  if (scratch_bytes < need) SLONN_FAIL(SLONN_ENOMEM, "scratch holds %zu bytes, %zu needed", scratch_bytes, need);
  if (reinterpret_cast<uintptr_t>(scratch) % 16 != 0) SLONN_FAIL(SLONN_EINVAL, "scratch must be 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  SLONN_HIP(hipEventCreate(&e0));
  SLONN_HIP(hipEventCreate(&e1));
  double* outs[2] = {gbps_all_units, gbps_one_unit};
  const int grids[2] = {n_cu, 1};
  for (int k = 0; k < 2; ++k) {
    (void)launch_l2_read_probe(scratch, grids[k], 4, s);            // warm-up: the window into L2
    SLONN_HIP(hipEventRecord(e0, s));
    const double bytes = launch_l2_read_probe(scratch, grids[k], 200, s);
    SLONN_HIP(hipEventRecord(e1, s));
    SLONN_HIP(hipEventSynchronize(e1));
    float ms = 0.0f;
    SLONN_HIP(hipEventElapsedTime(&ms, e0, e1));
    *outs[k] = ms > 0.0f ? bytes / (ms * 1e-3) / 1e9 : 0.0;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int slonn_version(char* buf, size_t cap) {
  if (!buf || cap == 0) SLONN_FAIL(SLONN_EINVAL, "null buffer");
  int dev = 0, lds = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess) {
    (void)hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  }
  snprintf(buf, cap, "slonn 0.1 (gfx950, wave64, HIP %d.%d; device: %d CUs, %d bytes LDS per workgroup)",
           HIP_VERSION_MAJOR, HIP_VERSION_MINOR, cus, lds);
  return SLONN_OK;
}

int slonn_model_create(const slonn_layer_desc* layers, int n_layers, slonn_model** out) {
  if (!out) SLONN_FAIL(SLONN_EINVAL, "out is null");
  *out = nullptr;
  if (!layers || n_layers <= 0) SLONN_FAIL(SLONN_EINVAL, "no layers");
  for (int l = 0; l < n_layers; ++l) {
    const slonn_layer_desc& d = layers[l];
    if (d.d_in <= 0 || d.d_out <= 0) SLONN_FAIL(SLONN_EINVAL, "layer %d: non-positive size", l);
    if (l > 0 && d.d_in != layers[l - 1].d_out)
      SLONN_FAIL(SLONN_EINVAL, "layer %d: d_in %d does not match previous d_out %d", l, d.d_in,
                 layers[l - 1].d_out);
    if (!d.W || !d.bias) SLONN_FAIL(SLONN_EINVAL, "layer %d: null weights or bias", l);
    if (d.w_dtype != SLONN_F32 && d.w_dtype != SLONN_BF16)
      SLONN_FAIL(SLONN_EINVAL, "layer %d: unknown weight type %d", l, d.w_dtype);
    if (d.act != SLONN_ACT_NONE && d.act != SLONN_ACT_RELU && d.act != SLONN_ACT_SOFTMAX)
      SLONN_FAIL(SLONN_EINVAL, "layer %d: unknown activation %d", l, d.act);
    if (d.act == SLONN_ACT_SOFTMAX && l != n_layers - 1)
      SLONN_FAIL(SLONN_EINVAL, "layer %d: softmax is only supported on the last layer", l);
    if (d.w_layout != SLONN_ROWS_ARE_NODES && d.w_layout != SLONN_ROWS_ARE_INPUTS)
      SLONN_FAIL(SLONN_EINVAL, "layer %d: unknown weight layout %d", l, d.w_layout);
    if (d.w_layout == SLONN_ROWS_ARE_INPUTS && (l != 0 || d.K > 0 || d.L > 0))
      SLONN_FAIL(SLONN_EUNSUPPORTED,
                 "layer %d: input-major weights are only supported on a first layer without a Node Activator", l);
    if ((d.K > 0) != (d.L > 0) || d.K < 0 || d.L < 0)
      SLONN_FAIL(SLONN_EINVAL, "layer %d: K and L must both be positive or both zero", l);
    if (d.K > SLONN_MAX_K) SLONN_FAIL(SLONN_EINVAL, "layer %d: K %d exceeds %d", l, d.K, SLONN_MAX_K);
    if (d.L > SLONN_MAX_L) SLONN_FAIL(SLONN_EINVAL, "layer %d: L %d exceeds %d", l, d.L, SLONN_MAX_L);
    if (d.K > 0) {
      const long H = (long)d.K * d.L;
      if (H > d.d_out) SLONN_FAIL(SLONN_EINVAL, "layer %d: K*L = %ld exceeds its %d nodes", l, H, d.d_out);
      if (!d.hash_nodes) SLONN_FAIL(SLONN_EINVAL, "layer %d: hash_nodes is null", l);
      if (d.list_cap <= 0) SLONN_FAIL(SLONN_EINVAL, "layer %d: list_cap must be positive", l);
      std::vector<int32_t> s(d.hash_nodes, d.hash_nodes + H);
      for (int32_t v : s)
        if (v < 0 || v >= d.d_out) SLONN_FAIL(SLONN_EINVAL, "layer %d: hash node %d out of range", l, v);
      std::sort(s.begin(), s.end());
      if (std::adjacent_find(s.begin(), s.end()) != s.end())
        SLONN_FAIL(SLONN_EINVAL, "layer %d: hash nodes are not distinct", l);
    }
  }

  slonn_model* m = new (std::nothrow) slonn_model;
  if (!m) SLONN_FAIL(SLONN_ENOMEM, "out of host memory");
  m->layers.resize(n_layers);
  for (int l = 0; l < n_layers; ++l) {
    const slonn_layer_desc& d = layers[l];
    Layer& L = m->layers[l];
    L.d_in = d.d_in; L.d_out = d.d_out; L.w_dtype = d.w_dtype; L.w_layout = d.w_layout;
    L.act = d.act; L.K = d.K; L.L = d.L; L.list_cap = d.K > 0 ? d.list_cap : 0;
    L.W = d.W; L.bias = d.bias;
    if (d.K > 0) L.hash_nodes.assign(d.hash_nodes, d.hash_nodes + (size_t)d.K * d.L);
  }

  auto fail = [&](int code) {
    slonn_model_destroy(m);
    return code;
  };
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    set_error("hipGetDevice failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  int v = 0;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0)
    m->max_lds_bytes = v;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
    m->n_cu = v;

  // The caller may have filled W and bias on any stream; the set-up kernels below run on the default
  // stream.  One device-wide synchronisation first, so that they read what the caller wrote.
  if ((e = hipDeviceSynchronize()) != hipSuccess) {
    set_error("hipDeviceSynchronize failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  // the scratch array of the allocation-free entry point: its address on this device, looked up now
  // so that the entry point itself has nothing left to set up
  {
    void* sp = nullptr;
    if (static_scratch(&sp) != SLONN_OK) return fail(SLONN_EHIP);
  }
  // library-owned fp32 copies of the FreeHash rows, gathered once (on the device)
  for (Layer& L : m->layers) {
    if (!L.activated()) continue;
    const int H = L.H();
    if ((e = hipMalloc(&L.Wh, (size_t)H * L.d_in * 4)) != hipSuccess ||
        (e = hipMalloc(&L.bh, (size_t)H * 4)) != hipSuccess ||
        (e = hipMalloc(&L.hnodes, (size_t)H * 4)) != hipSuccess ||
        (e = hipMemcpy(L.hnodes, L.hash_nodes.data(), (size_t)H * 4, hipMemcpyHostToDevice)) != hipSuccess) {
      set_error("allocating the FreeHash rows failed: %s", hipGetErrorString(e));
      return fail(SLONN_EHIP);
    }
    if (launch_gather_hash_rows(L.W, L.w_dtype, L.bias, L.hnodes, H, L.d_in, L.Wh, L.bh, nullptr) != SLONN_OK ||
        (e = hipStreamSynchronize(nullptr)) != hipSuccess) {
      if (e != hipSuccess) set_error("copying FreeHash rows failed: %s", hipGetErrorString(e));
      return fail(SLONN_EHIP);
    }
    // the rows once more input-major, for the whole-network kernels (which serve models whose hash
    // rows are a few megabytes at most)
    if ((size_t)L.d_in * H * 4 <= ((size_t)16 << 20)) {
      const int Hp = (H + 3) & ~3;
      if ((e = hipMalloc(&L.WhT, (size_t)L.d_in * Hp * 4)) != hipSuccess) {
        set_error("allocating the input-major FreeHash rows failed: %s", hipGetErrorString(e));
        return fail(SLONN_EHIP);
      }
      if (launch_transpose_hash_rows(L.Wh, H, L.d_in, Hp, L.WhT, nullptr) != SLONN_OK ||
          (e = hipStreamSynchronize(nullptr)) != hipSuccess) {
        if (e != hipSuccess) set_error("transposing the FreeHash rows failed: %s", hipGetErrorString(e));
        return fail(SLONN_EHIP);
      }
    }
    // node -> hash row (K*L <= 1024 fits 16 bits): lets the forward pass take a selected hash
    // node's output from its projection instead of fetching the row again
    std::vector<int16_t> hslot((size_t)L.d_out, (int16_t)-1);
    for (int h = 0; h < H; ++h) hslot[L.hash_nodes[h]] = (int16_t)h;
    if ((e = hipMalloc(&L.hslot, hslot.size() * 2)) != hipSuccess ||
        (e = hipMemcpy(L.hslot, hslot.data(), hslot.size() * 2, hipMemcpyHostToDevice)) != hipSuccess) {
      set_error("uploading the hash-node map failed: %s", hipGetErrorString(e));
      return fail(SLONN_EHIP);
    }
    // the hash rows once more as fixed-point digits for the int8 matrix cores (large batches)
    if (hash_int_supported(L.d_in, m->max_lds_bytes)) {
      if (hipMalloc(&L.Whd, (size_t)H * hash_int_digits() * L.d_in) != hipSuccess ||
          hipMalloc(&L.ewh, (size_t)H * 4) != hipSuccess) {
        (void)hipGetLastError();
        if (L.Whd) (void)hipFree(L.Whd);
        L.Whd = nullptr;
      } else if (launch_slice_digits(L.Wh, L.d_in, H, L.d_in, L.Whd, L.ewh, nullptr, nullptr) != SLONN_OK ||
                 (e = hipStreamSynchronize(nullptr)) != hipSuccess) {
        if (e != hipSuccess) set_error("slicing the FreeHash rows failed: %s", hipGetErrorString(e));
        return fail(SLONN_EHIP);
      }
    }
  }
  // Large layers: the weights once more as scaled fp16 parts (fp32 weights: two, bf16 weights:
  // one, the same bytes again) for the tiles that serve large batches on the fp16 matrix cores --
  // activated fp32 layers of the size the forward pass walks in row blocks, and bf16 layers.
  // Without the memory for it large batches stay on the other paths.
  for (Layer& L : m->layers) {
    const size_t row_bytes = (size_t)L.d_in * (L.w_dtype == SLONN_F32 ? 4 : 2);
    const bool wanted = L.w_dtype == SLONN_F32 ? (L.activated() && row_bytes >= 2048 && row_bytes * L.d_out > ((size_t)3 << 20))
                                               : true;
    if (!wanted || !masked_tiles_supported(L.d_in, L.d_out, m->max_lds_bytes) ||
        reinterpret_cast<uintptr_t>(L.W) % 16 != 0 || L.w_layout != SLONN_ROWS_ARE_NODES)
      continue;
    if (hipMalloc(&L.Wt, tile_weights_bytes(L.w_dtype, L.d_out, L.d_in)) != hipSuccess ||
        hipMalloc(&L.wt_exp, (size_t)L.d_out * 4) != hipSuccess) {
      (void)hipGetLastError();
      if (L.Wt) (void)hipFree(L.Wt);
      L.Wt = nullptr;
    } else if (launch_split_weights(L.W, L.w_dtype, L.d_out, L.d_in, L.Wt, L.wt_exp, nullptr) != SLONN_OK ||
               (e = hipStreamSynchronize(nullptr)) != hipSuccess) {
      if (e != hipSuccess) set_error("splitting the weights failed: %s", hipGetErrorString(e));
      return fail(SLONN_EHIP);
    } else {
      L.wt_parts = L.w_dtype == SLONN_F32 ? 2 : 1;
    }
  }
  *out = m;
  return SLONN_OK;
}

namespace slonn {
namespace {

// Can the whole-network kernel serve this model?  (reason != nullptr receives why not)
bool fused_eligible(const slonn_model* m, const char** reason) {
  const char* why = nullptr;
  const int nl = (int)m->layers.size();
  if (nl > FUSED_MAX_LAYERS) why = "too many layers";
  for (int l = 0; l < nl && !why; ++l) {
    const Layer& L = m->layers[l];
    const int esz = L.w_dtype == SLONN_F32 ? 4 : 2;
    if (L.w_layout != SLONN_ROWS_ARE_NODES) why = "input-major first layer";
    else if ((size_t)L.d_in * L.d_out * esz > ((size_t)8 << 20)) why = "a weight matrix exceeds 8 MiB";
    else if (((size_t)L.d_in * esz) % 16 != 0 || L.d_in % 4 != 0) why = "row length is not a multiple of 16 bytes";
    else if (reinterpret_cast<uintptr_t>(L.W) % 16 != 0) why = "weights are not 16-byte aligned";
    else if (l == nl - 1 && L.activated()) why = "Node Activator on the last layer";
    else if (L.activated() && !L.WhT) why = "no input-major FreeHash rows";
  }
  if (!why) {
    FusedArgs a{};
    for (const Layer& L : m->layers) {
      a.max_dim = std::max(a.max_dim, std::max(L.d_in, L.d_out));
      if (L.activated()) { a.max_H = std::max(a.max_H, L.H()); a.max_na = std::max(a.max_na, L.d_out); }
    }
    a.max_dim = (a.max_dim + 7) & ~7;
    if (fused_lds_bytes(a) > (size_t)m->max_lds_bytes) why = "activations do not fit in LDS";
  }
  if (reason) *reason = why;
  return why == nullptr;
}

// Can the whole-network kernel for wide sparse-input models serve this model?  (two layers:
// a small hidden layer stored input-major without a Node Activator, an activated output layer)
bool fused_wide_eligible(const slonn_model* m, int ell_stride, const char** reason) {
  const char* why = nullptr;
  if (m->layers.size() != 2) why = "not a two-layer model";
  else {
    const Layer& A = m->layers[0];
    const Layer& Bl = m->layers[1];
    const int e0 = A.w_dtype == SLONN_F32 ? 4 : 8, e1 = Bl.w_dtype == SLONN_F32 ? 4 : 8;
    if (A.activated() || A.w_layout != SLONN_ROWS_ARE_INPUTS) why = "first layer is not a plain input-major layer";
    else if (!Bl.activated()) why = "output layer has no Node Activator";
    else if (A.d_out > 4096 || A.d_out % e0 != 0 || A.d_out % e1 != 0 || A.d_out % 4 != 0)
      why = "hidden width is above 4096 or not a multiple of 16 bytes";
    else if (reinterpret_cast<uintptr_t>(A.W) % 16 != 0 || reinterpret_cast<uintptr_t>(Bl.W) % 16 != 0)
      why = "weights are not 16-byte aligned";
    else if (!Bl.WhT) why = "no input-major FreeHash rows";
    else if ((unsigned long long)Bl.d_out * (unsigned long long)(A.d_out / 4) > 0xFFFFFFFFull)
      why = "output weight matrix too large for 32-bit row offsets";
    else {
      FusedWideArgs a{};
      a.n1p = (A.d_out + 3) & ~3; a.Hp = (Bl.H() + 3) & ~3; a.ellp = (std::max(ell_stride, 1) + 3) & ~3;
      a.n2 = Bl.d_out;
      if (fused_wide_lds_bytes(a) > (size_t)m->max_lds_bytes) why = "the query's state does not fit in LDS";
    }
  }
  if (reason) *reason = why;
  return why == nullptr;
}

}  // namespace
}  // namespace slonn

int slonn_model_set_path(slonn_model* m, int path) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "model is null");
  if (path != SLONN_PATH_AUTO && path != SLONN_PATH_LAYERS && path != SLONN_PATH_FUSED)
    SLONN_FAIL(SLONN_EINVAL, "unknown path %d", path);
  if (path == SLONN_PATH_FUSED) {
    const char* why = nullptr;
    if (!fused_eligible(m, &why) && !fused_wide_eligible(m, 1, nullptr))
      SLONN_FAIL(SLONN_EUNSUPPORTED, "fused path unavailable: %s", why);
  }
  m->path = path;
  return SLONN_OK;
}

int slonn_model_set_hash_margin(slonn_model* m, double margin) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "model is null");
  if (!(margin >= 1.0)) SLONN_FAIL(SLONN_EINVAL, "margin must be at least 1");
  m->hash_margin = margin;
  return SLONN_OK;
}

int slonn_model_set_batches_in_flight(slonn_model* m, int n) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "model is null");
  if (n < 1) SLONN_FAIL(SLONN_EINVAL, "batches in flight must be at least 1");
  m->batches_in_flight = n;
  return SLONN_OK;
}

int slonn_model_set_tables_refreshable(slonn_model* m, int on) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "model is null");
  m->tables_refreshable = on != 0;
  return SLONN_OK;
}

int slonn_model_set_dense_arithmetic(slonn_model* m, int mode) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "model is null");
  if (mode != SLONN_DENSE_FP32_MFMA && mode != SLONN_DENSE_F16_PARTS)
    SLONN_FAIL(SLONN_EINVAL, "unknown dense arithmetic %d", mode);
  m->dense_arith = mode;
  return SLONN_OK;
}

int slonn_model_set_hash_nodes_always_active(slonn_model* m, int on) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "model is null");
  m->hash_first = on != 0;
  return SLONN_OK;
}

int slonn_model_destroy(slonn_model* m) {
  if (!m) return SLONN_OK;
  for (Layer& L : m->layers) {
    if (L.Wh) (void)hipFree(L.Wh);
    if (L.WhT) (void)hipFree(L.WhT);
    if (L.bh) (void)hipFree(L.bh);
    if (L.hslot) (void)hipFree(L.hslot);
    if (L.hnodes) (void)hipFree(L.hnodes);
    if (L.Wt) (void)hipFree(L.Wt);
    if (L.wt_exp) (void)hipFree(L.wt_exp);
    if (L.Whd) (void)hipFree(L.Whd);
    if (L.ewh) (void)hipFree(L.ewh);
  }
  delete m;
  return SLONN_OK;
}

int slonn_workspace_bytes(const slonn_model* m, int B_max, size_t* out) {
  if (!m || !out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (B_max <= 0 || B_max > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B_max must be in 1 .. %d", SLONN_MAX_BATCH);
  Workspace w;
  plan_workspace(m, B_max, nullptr, &w);
  *out = w.bytes;
  return SLONN_OK;
}

// ------------------------------------------------------------------------------------ //
// tables
// ------------------------------------------------------------------------------------ //
int slonn_tables_destroy(slonn_tables* t) {
  if (!t) return SLONN_OK;
  for (TableSet& s : t->sets) free_table_set(&s);
  delete t;
  return SLONN_OK;
}

int slonn_tables_export(const slonn_tables* t, void* host_buf, size_t* bytes) {
  if (!t || !bytes) SLONN_FAIL(SLONN_EINVAL, "null argument");
  size_t need = 16;
  for (const TableSet& s : t->sets)
    need += 32 + 4 * ((size_t)s.K * s.L + s.dir.size() + s.n_ids + s.global_rank.size());
  if (!host_buf) {
    *bytes = need;
    return SLONN_OK;
  }
  if (*bytes < need) SLONN_FAIL(SLONN_ENOMEM, "export buffer holds %zu bytes, %zu needed", *bytes, need);
  char* p = static_cast<char*>(host_buf);
  auto put = [&](const void* src, size_t n) {
    std::memcpy(p, src, n);
    p += n;
  };
  const uint32_t head[4] = {SLONN_TABLE_BLOB_MAGIC, SLONN_TABLE_BLOB_VERSION, (uint32_t)t->sets.size(), 0};
  put(head, 16);
  for (const TableSet& s : t->sets) {
    const uint32_t h[8] = {(uint32_t)s.layer, (uint32_t)s.K, (uint32_t)s.L, (uint32_t)s.n,
                           (uint32_t)s.list_cap, (uint32_t)s.n_ids, 0, 0};
    put(h, 32);
    const Layer& L = t->model->layers[s.layer];
    put(L.hash_nodes.data(), 4 * L.hash_nodes.size());
    put(s.dir.data(), 4 * s.dir.size());
    if (s.n_ids) {                              // the lists are held on the device only
      const int rc = download_ids(&s, reinterpret_cast<int32_t*>(p));
      if (rc) return rc;
      p += 4 * s.n_ids;
    }
    put(s.global_rank.data(), 4 * s.global_rank.size());
  }
  *bytes = need;
  return SLONN_OK;
}

int slonn_tables_import(const slonn_model* m, const void* host_buf, size_t bytes, slonn_tables** out) {
  if (!out) SLONN_FAIL(SLONN_EINVAL, "out is null");
  *out = nullptr;
  if (!m || !host_buf) SLONN_FAIL(SLONN_EINVAL, "null argument");
  const char* p = static_cast<const char*>(host_buf);
  const char* end = p + bytes;
  auto have = [&](size_t n) { return (size_t)(end - p) >= n; };
  uint32_t head[4];
  if (!have(16)) SLONN_FAIL(SLONN_EINVAL, "blob shorter than its header");
  std::memcpy(head, p, 16);
  p += 16;
  if (head[0] != SLONN_TABLE_BLOB_MAGIC || head[1] != SLONN_TABLE_BLOB_VERSION)
    SLONN_FAIL(SLONN_EINVAL, "not a table blob (magic %08x version %u)", head[0], head[1]);
  slonn_tables* t = new (std::nothrow) slonn_tables;
  if (!t) SLONN_FAIL(SLONN_ENOMEM, "out of host memory");
  t->model = m;
  auto fail = [&](int code) {
    slonn_tables_destroy(t);
    return code;
  };
  for (uint32_t i = 0; i < head[2]; ++i) {
    uint32_t h[8];
    if (!have(32)) { set_error("blob truncated in set %u header", i); return fail(SLONN_EINVAL); }
    std::memcpy(h, p, 32);
    p += 32;
    TableSet s;
    s.layer = (int)h[0]; s.K = (int)h[1]; s.L = (int)h[2]; s.n = (int)h[3]; s.list_cap = (int)h[4];
    const size_t total = h[5];
    if (s.layer < 0 || s.layer >= (int)m->layers.size()) {
      set_error("set %u names layer %d", i, s.layer);
      return fail(SLONN_EINVAL);
    }
    const Layer& L = m->layers[s.layer];
    if (!L.activated() || L.K != s.K || L.L != s.L || L.d_out != s.n) {
      set_error("set %u (layer %d, K %d, L %d, n %d) does not match the model", i, s.layer, s.K, s.L, s.n);
      return fail(SLONN_EINVAL);
    }
    if (t->for_layer(s.layer)) { set_error("layer %d appears twice", s.layer); return fail(SLONN_EINVAL); }
    const size_t H = (size_t)s.K * s.L, nd = (size_t)s.L * (((size_t)1 << s.K) + 1);
    if (!have(4 * (H + nd + total + (size_t)s.n))) {
      set_error("blob truncated in set %u body", i);
      return fail(SLONN_EINVAL);
    }
    if (std::memcmp(p, L.hash_nodes.data(), 4 * H) != 0) {
      set_error("set %u was built with different hash nodes", i);
      return fail(SLONN_EINVAL);
    }
    p += 4 * H;
    s.dir.resize(nd);
    std::memcpy(s.dir.data(), p, 4 * nd);
    p += 4 * nd;
    s.ids.resize(total);
    std::memcpy(s.ids.data(), p, 4 * total);
    p += 4 * total;
    s.global_rank.resize(s.n);
    std::memcpy(s.global_rank.data(), p, 4 * (size_t)s.n);
    p += 4 * (size_t)s.n;
    // structural checks: offsets monotone and inside ids, ids and ranking in range, ranking a permutation
    uint32_t prev = 0;
    for (uint32_t v : s.dir) {
      if (v < prev || v > total) { set_error("set %u: bucket offsets not monotone", i); return fail(SLONN_EINVAL); }
      prev = v;
    }
    for (int32_t v : s.ids)
      if (v < 0 || v >= s.n) { set_error("set %u: node id %d out of range", i, v); return fail(SLONN_EINVAL); }
    std::vector<char> seen(s.n, 0);
    for (int32_t v : s.global_rank) {
      if (v < 0 || v >= s.n || seen[v]) { set_error("set %u: ranking is not a permutation", i); return fail(SLONN_EINVAL); }
      seen[v] = 1;
    }
    int rc = upload_table_set(&s);
    if (rc != SLONN_OK) {
      free_table_set(&s);
      return fail(rc);
    }
    t->sets.push_back(std::move(s));
  }
  for (size_t l = 0; l < m->layers.size(); ++l)
    if (m->layers[l].activated() && !t->for_layer((int)l)) {
      set_error("blob has no tables for activated layer %zu", l);
      return fail(SLONN_EINVAL);
    }
  *out = t;
  return SLONN_OK;
}

// ------------------------------------------------------------------------------------ //
// select / forward
// ------------------------------------------------------------------------------------ //
int slonn_select(const slonn_model* m, const slonn_tables* t, int layer, const float* X_l, int B,
                 const float* keep, int keep_stride, uint32_t* codes_out, float* z_out,
                 int32_t* active_idx, int32_t* active_cnt, int idx_stride, void* workspace,
                 size_t ws_bytes, void* stream) {
  if (!m || !t || !X_l || !keep || !active_idx || !active_cnt) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (t->model != m) SLONN_FAIL(SLONN_EINVAL, "tables belong to another model");
  if (B <= 0 || B > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B must be in 1 .. %d", SLONN_MAX_BATCH);
  if (layer < 0 || layer >= (int)m->layers.size()) SLONN_FAIL(SLONN_EINVAL, "no layer %d", layer);
  if (keep_stride < 0) SLONN_FAIL(SLONN_EINVAL, "negative keep stride");
  const Layer& L = m->layers[layer];
  const TableSet* ts = t->for_layer(layer);
  if (!L.activated() || !ts) SLONN_FAIL(SLONN_EINVAL, "layer %d has no Node Activator", layer);
  if (idx_stride < L.d_out)
    SLONN_FAIL(SLONN_ECAP, "idx_stride %d is below the layer's %d nodes", idx_stride, L.d_out);
  float* z = z_out;
  if (!z) {
    const size_t need = (size_t)B * L.H() * 4;
    if (!workspace || ws_bytes < need)
      SLONN_FAIL(SLONN_ENOMEM, "workspace holds %zu bytes, %zu needed", ws_bytes, need);
    z = static_cast<float*>(workspace);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  int rc = launch_hash_project(X_l, L.d_in, L.Wh, L.bh, z, B, L.H(), L.d_in, nullptr, nullptr, s);
  if (rc) return rc;
  HashFirst hf;
  if (m->hash_first) { hf.hnodes = L.hnodes; hf.hslot = L.hslot; }
  return launch_select(z, L.K, L.L, L.d_out, ts->d_dir, ts->d_ids, ts->narrow, ts->d_global_rank, keep, keep_stride,
                       B, codes_out, active_idx, active_cnt, idx_stride, nullptr, 0, m->max_lds_bytes,
                       nullptr, m->hash_first ? &hf : nullptr, nullptr, nullptr, s);
}

namespace slonn {
namespace {

// ACLO inside the forward pass: k is chosen from the first activated layer's projections
// (the Confidence LSH tables share that layer's hash functions) and serves every layer.
// Masked tiles serve 128 queries when their mean list is at least this share of the layer
// (below it the per-query gather, whose cost grows with batch x budget, is cheaper than the
// tiles, whose cost per layer is about constant while they fit the chip once: measured
// break-even on 4096-wide fp32 layers, ms per 8192 queries, gather at keep .02 / .04 / .06 / .08
// against tiles: batch 256 4.4 / 5.4 / 6.4 / 7.7 against 5.9-6.1, batch 512 3.6 / 4.6 / 5.5 / 6.4
// against 5.0, batch 1024 2.9 / 3.8 / 4.7 / 5.5 against 3.5-3.7; at batch 128 the two launches
// that find nothing to serve cost every smaller budget 13 us per step: the tiles start at batch
// 160, where three rows of 64 x 64 tiles cost what they cost at batch 192 and the per-query gather
// has lost the XCD-aware placement of its row blocks).
// bf16 weights (two MFMAs per block; the alternative is the union of 16 queries' rows on the
// bf16 cores, whose cost follows the union's size)
constexpr int BF16_TILES_MIN_KEEP_PERMILLE = 100;
int masked_tiles_min_keep_permille(int B) { return B >= 1024 ? 35 : (B >= 512 ? 50 : (B >= 256 ? 55 : 80)); }

struct PolicyHook {
  const slonn_policy* p = nullptr;
  const float* thr = nullptr;
  int thr_stride = 0;
  float* keep_out = nullptr;     // [B] device, receives the chosen keep fractions
  int layer = -1;                // first activated layer
};

int forward_impl(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                 const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                 const slonn_debug_taps* taps, void* workspace, size_t ws_bytes, void* stream,
                 const PolicyHook* hook) {
  if (!m || !X || !keep || !Y) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (B <= 0 || B > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B must be in 1 .. %d", SLONN_MAX_BATCH);
  if (keep_qstride < 0 || keep_lstride < 0) SLONN_FAIL(SLONN_EINVAL, "negative keep stride");
  int rc = check_input(m, X);
  if (rc) return rc;
  bool any_activated = false;
  for (const Layer& L : m->layers) any_activated |= L.activated();
  if (any_activated) {
    if (!t) SLONN_FAIL(SLONN_EINVAL, "tables are null but the model has activated layers");
    if (t->model != m) SLONN_FAIL(SLONN_EINVAL, "tables belong to another model");
  }
  const int nl = (int)m->layers.size();
  const Layer& last = m->layers[nl - 1];
  if ((Y->idx || Y->val) && last.activated()) {
    if (!Y->cnt) SLONN_FAIL(SLONN_EINVAL, "compact output needs cnt");
    if (Y->stride < last.d_out)
      SLONN_FAIL(SLONN_ECAP, "compact output stride %d is below the last layer's %d nodes", Y->stride,
                 last.d_out);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);

  // ---- whole-network kernel for wide sparse-input models ----
  // (one workgroup per query: ahead of the per-layer path, whose hash projection is a batch-wide
  // MFMA contraction, up to about two queries per compute unit -- C4: 30 vs 44 us at batch 128,
  // 116 vs 82 us at batch 1024)
  if (m->path != SLONN_PATH_LAYERS && X->format == SLONN_ELL && !hook &&
      (m->path == SLONN_PATH_FUSED || B <= 2 * m->n_cu) && fused_wide_eligible(m, X->ell_stride, nullptr)) {
    Workspace w;
    plan_workspace(m, B, static_cast<char*>(workspace), &w);
    if (!workspace || ws_bytes < w.bytes)
      SLONN_FAIL(SLONN_ENOMEM, "workspace holds %zu bytes, %zu needed", ws_bytes, w.bytes);
    const Layer& A = m->layers[0];
    const Layer& O = m->layers[1];
    const TableSet* ts = t->for_layer(1);
    FusedWideArgs a{};
    a.W0 = A.W; a.b0 = A.bias; a.w0_dtype = A.w_dtype; a.act0 = A.act; a.d0 = A.d_in; a.n1 = A.d_out;
    a.n1p = (A.d_out + 3) & ~3;
    a.ccp = 1;
    while (a.ccp * 4 < A.d_out) a.ccp *= 2;
    a.idx = X->idx; a.val = X->val; a.nnz = X->nnz; a.ell_stride = X->ell_stride;
    a.ellp = (X->ell_stride + 3) & ~3;
    a.W1 = O.W; a.b1 = O.bias; a.w1_dtype = O.w_dtype; a.act1 = O.act; a.n2 = O.d_out;
    a.WhT = O.WhT; a.bh = O.bh; a.K = O.K; a.L = O.L; a.Hp = (O.H() + 3) & ~3;
    a.dir = ts->d_dir; a.ids = ts->d_ids; a.ids_narrow = ts->narrow ? 1 : 0; a.global_rank = ts->d_global_rank;
    a.hnodes = O.hnodes; a.hslot = O.hslot; a.hash_first = m->hash_first ? 1 : 0;
    a.keep = keep + (size_t)1 * keep_lstride; a.keep_qstride = keep_qstride;
    int32_t* tap_idx = taps && taps->active_idx ? taps->active_idx[1] : nullptr;
    int32_t* tap_cnt = taps && taps->active_cnt ? taps->active_cnt[1] : nullptr;
    float* tap_out1 = taps && taps->layer_out ? taps->layer_out[1] : nullptr;
    a.list = Y->idx ? Y->idx : (tap_idx ? tap_idx : w.active);
    a.list_stride = Y->idx ? Y->stride : O.d_out;
    a.cnt = Y->cnt ? Y->cnt : (tap_cnt ? tap_cnt : w.cnt);
    a.vals = Y->val ? Y->val : w.act[0];
    a.vals_stride = Y->val ? Y->stride : w.max_n;
    a.dense = Y->dense ? Y->dense : tap_out1;
    a.argmax = Y->argmax;
    a.tap_codes = taps && taps->codes ? taps->codes[1] : nullptr;
    a.tap_z = taps && taps->z ? taps->z[1] : nullptr;
    a.tap_out0 = taps && taps->layer_out ? taps->layer_out[0] : nullptr;
    rc = launch_fused_wide(a, B, m->batches_in_flight, m->n_cu, m->max_lds_bytes, s);
    if (rc) return rc;
    if (tap_idx && a.list != tap_idx)
      SLONN_HIP(hipMemcpy2DAsync(tap_idx, (size_t)O.d_out * 4, a.list, (size_t)a.list_stride * 4,
                                 (size_t)O.d_out * 4, B, hipMemcpyDeviceToDevice, s));
    if (tap_cnt && a.cnt != tap_cnt)
      SLONN_HIP(hipMemcpyAsync(tap_cnt, a.cnt, (size_t)B * 4, hipMemcpyDeviceToDevice, s));
    if (tap_out1 && a.dense != tap_out1)
      SLONN_HIP(hipMemcpyAsync(tap_out1, a.dense, (size_t)B * O.d_out * 4, hipMemcpyDeviceToDevice, s));
    return SLONN_OK;
  }

  // ---- whole-network kernel ----
  const bool wants_compact = Y->idx || Y->val || Y->cnt;
  bool fused = false;
  if (m->path != SLONN_PATH_LAYERS) {
    const char* why = nullptr;
    fused = fused_eligible(m, &why) && X->format == SLONN_DENSE && !wants_compact &&
            reinterpret_cast<uintptr_t>(X->x) % 16 == 0;
    if (!fused && m->path == SLONN_PATH_FUSED)
      SLONN_FAIL(SLONN_EUNSUPPORTED, "fused path unavailable for this call: %s",
                 why ? why : "needs dense 16-byte aligned input and no compact output");
  }
  if (fused) {
    FusedArgs a{};
    a.n_layers = nl;
    for (int l = 0; l < nl; ++l) {
      const Layer& L = m->layers[l];
      FusedLayer& f = a.layer[l];
      f.W = L.W; f.bias = L.bias; f.WhT = L.WhT; f.bh = L.bh; f.hslot = L.hslot; f.hnodes = L.hnodes;
      f.d_in = L.d_in; f.d_out = L.d_out; f.act = L.act; f.w_dtype = L.w_dtype; f.K = L.K; f.L = L.L;
      if (L.activated()) {
        const TableSet* ts = t->for_layer(l);
        f.dir = ts->d_dir; f.ids = ts->d_ids; f.ids_narrow = ts->narrow ? 1 : 0; f.global_rank = ts->d_global_rank;
        a.max_H = std::max(a.max_H, L.H());
        a.max_na = std::max(a.max_na, L.d_out);
      }
      a.max_dim = std::max(a.max_dim, std::max(L.d_in, L.d_out));
      if (taps) {
        f.tap_codes = taps->codes ? taps->codes[l] : nullptr;
        f.tap_z = taps->z ? taps->z[l] : nullptr;
        f.tap_idx = taps->active_idx ? taps->active_idx[l] : nullptr;
        f.tap_cnt = taps->active_cnt ? taps->active_cnt[l] : nullptr;
        f.tap_out = taps->layer_out ? taps->layer_out[l] : nullptr;
      }
    }
    a.max_dim = (a.max_dim + 7) & ~7;
    a.X = X->x; a.ldx = m->layers[0].d_in;
    a.keep = keep; a.keep_qstride = keep_qstride; a.keep_lstride = keep_lstride;
    a.hash_first = m->hash_first ? 1 : 0;
    if (hook) {
      policy_fused_args(hook->p, &a.pol);
      a.pol.thr = hook->thr; a.pol.thr_stride = hook->thr_stride; a.pol.keep_out = hook->keep_out;
      a.pol.layer = hook->layer;
    }
    a.Y = Y->dense; a.argmax = Y->argmax;
    return launch_fused_forward(a, B, m->batches_in_flight, m->n_cu, m->max_lds_bytes, s);
  }

  Workspace w;
  plan_workspace(m, B, static_cast<char*>(workspace), &w);
  if (!workspace || ws_bytes < w.bytes)
    SLONN_FAIL(SLONN_ENOMEM, "workspace holds %zu bytes, %zu needed", ws_bytes, w.bytes);

  const float* cur = X->x;
  int ldcur = m->layers[0].d_in;
  bool order_ready = false;
  for (int l = 0; l < nl; ++l) {
    const Layer& L = m->layers[l];
    const bool is_last = (l == nl - 1);
    float* tap_out = taps && taps->layer_out ? taps->layer_out[l] : nullptr;
    // write straight into the caller's buffer when one exists for this layer
    float* out = is_last && Y->dense ? Y->dense : (tap_out ? tap_out : w.act[l & 1]);
    // a last layer whose result is only wanted in compact form never materialises the dense row
    if (is_last && L.activated() && !Y->dense && !tap_out && Y->val && Y->idx) out = nullptr;
    const int ldo = L.d_out;
    const int act = L.act;
    const int32_t* act_list = nullptr;
    const int32_t* act_cnt = nullptr;
    int act_stride = 0;
    float* yc = nullptr;
    if (L.activated()) {
      const TableSet* ts = t->for_layer(l);
      float* z = taps && taps->z && taps->z[l] ? taps->z[l] : w.z;
      uint32_t* codes = taps && taps->codes ? taps->codes[l] : nullptr;
      int32_t* aidx = taps && taps->active_idx && taps->active_idx[l] ? taps->active_idx[l] : w.active;
      int32_t* acnt = taps && taps->active_cnt && taps->active_cnt[l] ? taps->active_cnt[l] : w.cnt;
      int astride = L.d_out;
      // the caller's compact output doubles as the active list unless a tap already does
      const bool tap_idx = taps && taps->active_idx && taps->active_idx[l];
      const bool tap_cnt = taps && taps->active_cnt && taps->active_cnt[l];
      if (is_last && Y->idx && !tap_idx) { aidx = Y->idx; astride = Y->stride; }
      if (is_last && Y->cnt && !tap_cnt) acnt = Y->cnt;
      // (a medium batch leaves the projection's reduction split; the select kernel finishes it,
      // unless the policy kernel needs the projections first)
      HashSplit split;
      const bool policy_here = hook && l == hook->layer;
      const int32_t* cur_exp = nullptr;    // exponents of the rows of cur, where the hash has found them
      if (L.Whd && w.hash_int && hash_int_pays(B, L.H(), L.d_in)) {
        rc = launch_hash_project_int(cur, ldcur, L.Wh, L.Whd, L.ewh, L.bh, z, B, L.H(), L.d_in, m->hash_margin,
                                     w.hash_int, s);
        cur_exp = hash_int_row_exponents(w.hash_int, B, L.d_in);
      } else
        rc = launch_hash_project(cur, ldcur, L.Wh, L.bh, z, B, L.H(), L.d_in, w.hash_split,
                                 policy_here ? nullptr : &split, s);
      if (rc) return rc;
      if (policy_here) {
        // the budget of this and of every later layer comes from the confidence tables
        rc = launch_policy_aclo(hook->p, nullptr, z, B, hook->thr, hook->thr_stride, hook->keep_out, nullptr,
                                nullptr, s);
        if (rc) return rc;
        keep = hook->keep_out; keep_qstride = 1; keep_lstride = 0;
      }
      // Weight matrices well beyond an L2 slice (with rows long enough to occupy a wavefront)
      // are walked in blocks of rows of about 2 MiB so that concurrently running workgroups
      // share them; the others are read as listed.
      RowBlocking rb;
      const size_t esz = L.w_dtype == SLONN_F32 ? 4 : 2;
      const size_t row_bytes = (size_t)L.d_in * esz;
      const bool rows_vec = row_bytes % 16 == 0 && L.d_in % 4 == 0 && ldcur % 4 == 0 &&
                            reinterpret_cast<uintptr_t>(L.W) % 16 == 0 && reinterpret_cast<uintptr_t>(cur) % 16 == 0;
      // Large batches of a bf16-weight layer: every group of 16 queries is evaluated on the bf16
      // matrix cores; no per-query gather runs, so the lists are not regrouped by row block.
      // (C5 per step, row-block gather against tiles + unions: batch 64 866 / 2677 us, batch 128
      // 1391 / 1383, batch 192 1873 / 1441: from batch 160.)
      const long gtiles = (long)((B + 15) / 16) * ((L.d_out + 127) / 128);
      const bool all_grouped = B >= 160 && gtiles >= 640 && out && !(is_last && Y->val) && m->path_grouped && rows_vec &&
                               grouped_supported(L.d_out, m->max_lds_bytes) &&
                               grouped_uses_bf16_cores(L.W, L.w_dtype, L.d_in);
      // (the row-block gather stages a query's activations in LDS: up to 40 952 inputs)
      if (!all_grouped && B >= ROW_BLOCK_MIN_BATCH && rows_vec && row_bytes >= 2048 && row_bytes * L.d_out > ((size_t)3 << 20) &&
          ((size_t)L.d_in + 8) * 4 <= ((size_t)160 << 10) && select_fills_row_blocks(L.d_out, m->max_lds_bytes)) {
        int rpb = 16;
        while ((size_t)rpb * 2 * row_bytes <= ((size_t)2 << 20)) rpb *= 2;
        while ((L.d_out + rpb - 1) / rpb > MAX_ROW_BLOCKS) rpb *= 2;
        rb.rows_per_block = rpb;
        rb.nblk = (L.d_out + rpb - 1) / rpb;
        rb.stride = w.max_na;
        rb.part_idx = w.part_idx; rb.part_pos = w.part_pos; rb.blk_off = w.blk_off;
        // selected hash nodes take their output from z (the hash is "free", Section 3.4)
        rb.hslot = L.hslot;
        rb.y = out; rb.ldy = ldo;
        rb.yc = is_last ? Y->val : nullptr; rb.ldc = Y->stride;
        rb.relu = act == SLONN_ACT_RELU;
      }
      // fp32 layer with split weights at a batch that fills the tile kernel: masked tiles follow the
      // select kernel, which then leaves the queries they will serve out of the regrouping
      const long mtiles = (long)((B + 63) / 64) * ((L.d_out + 127) / 128);   // workgroups of the tile kernel
      const bool f32_tiles = rb.part_idx && L.w_dtype == SLONN_F32 && L.Wt && w.tiles && B >= 160 && mtiles >= 64 && out &&
                             !(is_last && Y->val) && m->path_grouped;
      // (bf16-weight layers: tiles of 128 queries with large budgets go to the masked tiles, the others
      // to the unions of 16)
      const bool bf16_tiles = all_grouped && L.Wt && w.tiles && mtiles >= 128;
      if (f32_tiles || bf16_tiles) {
        // the select kernel decides per tile of 128 queries and writes the pair masks of the served ones
        const int permille = f32_tiles ? masked_tiles_min_keep_permille(B) : BF16_TILES_MIN_KEEP_PERMILLE;
        rb.served_min_per_query = (long long)L.d_out * permille / 1000;
        rb.B = B;
        masked_tiles_buffers(w.tiles, B, L.d_out, &rb.mask, &rb.flags);
      }
      HashFirst hf;
      if (m->hash_first) { hf.hnodes = L.hnodes; hf.hslot = L.hslot; }
      // a batch beyond what the device holds at once starts its longest merges first; with one
      // keep fraction per query for all layers the order is found once per call
      const int32_t* order = nullptr;
      if (select_wants_order(L.d_out, B, m->max_lds_bytes, m->n_cu)) {
        if (!order_ready || keep_lstride != 0) {
          rc = launch_order_by_budget(keep + (size_t)l * keep_lstride, keep_qstride, B, w.order, s);
          if (rc) return rc;
          order_ready = true;
        }
        order = w.order;
      }
      rc = launch_select(z, L.K, L.L, L.d_out, ts->d_dir, ts->d_ids, ts->narrow, ts->d_global_rank,
                         keep + (size_t)l * keep_lstride, keep_qstride, B, codes, aidx, acnt, astride, out,
                         ldo, m->max_lds_bytes, (rb.part_idx || rb.mask) ? &rb : nullptr, m->hash_first ? &hf : nullptr,
                         split.part ? &split : nullptr, order, s);
      if (rc) return rc;
      act_list = aidx; act_cnt = acnt; act_stride = astride;
      if (is_last && Y->val) yc = Y->val;
      if (all_grouped) {
        GroupedReuse reuse;
        reuse.hslot = L.hslot; reuse.Z = z; reuse.H = L.H(); reuse.relu = act == SLONN_ACT_RELU;
        // tiles of 128 queries with large budgets: masked dense tiles; the others: unions of 16
        const int32_t* served = nullptr;
        if (bf16_tiles) {
          int32_t* tflags = nullptr;
          rc = launch_masked_tiles(L.Wt, L.wt_parts, L.wt_exp, L.bias, cur, ldcur, cur_exp, out, ldo, B, L.d_in,
                                   L.d_out, act, w.tiles, &tflags, s);
          if (rc) return rc;
          served = tflags;
        }
        int32_t* flags = nullptr;
        rc = launch_gather_grouped(L.W, L.w_dtype, L.bias, cur, ldcur, aidx, acnt, astride, out, ldo, B,
                                   L.d_in, L.d_out, act, &reuse, served, w.grouped, m->max_lds_bytes, &flags, s);
      } else if (rb.part_idx) {
        // Large batches: groups of 16 queries whose lists overlap enough are evaluated together
        // on the matrix cores (decided per group on the device); the rest is gathered per query.
        const int32_t* gflag = nullptr;
        if (f32_tiles) {
          // masked tiles on the fp16 matrix cores (a selected hash node of a served query is computed
          // there like any other pair; the regrouping step reuses the projections for the others)
          int32_t* flags = nullptr;
          rc = launch_masked_tiles(L.Wt, L.wt_parts, L.wt_exp, L.bias, cur, ldcur, cur_exp, out, ldo, B, L.d_in, L.d_out,
                                   act, w.tiles, &flags, s);
          if (rc) return rc;
          gflag = flags;
        } else if (gtiles >= 1024 && out && !yc && m->path_grouped && grouped_supported(L.d_out, m->max_lds_bytes)) {
          int32_t* flags = nullptr;
          GroupedReuse reuse;
          reuse.hslot = rb.hslot;        // outputs of selected hash nodes were written by the regrouping step
          rc = launch_gather_grouped(L.W, L.w_dtype, L.bias, cur, ldcur, aidx, acnt, astride, out, ldo, B,
                                     L.d_in, L.d_out, act, &reuse, nullptr, w.grouped, m->max_lds_bytes, &flags, s);
          if (rc) return rc;
          gflag = flags;
        }
        rc = launch_gather_blocked(L.W, L.w_dtype, L.bias, cur, ldcur, rb, out, ldo, yc, Y->stride, B, L.d_in,
                                   L.d_out, act, gflag, s);
      } else
        rc = launch_gather_forward(L.W, L.w_dtype, L.bias, cur, ldcur, aidx, acnt, astride, L.d_out, out, ldo,
                                   yc, Y->stride, B, L.d_in, L.d_out, act, s);
      if (rc) return rc;
      if (is_last && Y->idx && tap_idx)
        SLONN_HIP(hipMemcpy2DAsync(Y->idx, (size_t)Y->stride * 4, aidx, (size_t)astride * 4,
                                   (size_t)L.d_out * 4, B, hipMemcpyDeviceToDevice, s));
      if (is_last && Y->cnt && tap_cnt)
        SLONN_HIP(hipMemcpyAsync(Y->cnt, acnt, (size_t)B * 4, hipMemcpyDeviceToDevice, s));
    } else if (l == 0 && X->format == SLONN_ELL) {
      rc = launch_ell_layer(L.W, L.w_dtype, L.w_layout, L.bias, X->idx, X->val, X->nnz, X->ell_stride, out,
                            ldo, B, L.d_in, L.d_out, act, s);
      if (rc) return rc;
    } else if (w.tiles && L.w_dtype == SLONN_BF16 && L.Wt && (long)((B + 63) / 64) * ((L.d_out + 127) / 128) >= 128 &&
               masked_tiles_workspace_bytes(B, L.d_out, L.d_in) <= w.tiles_bytes) {
      // a bf16-weight layer computed in full for a large batch: the tiles of the masked evaluation
      // without a mask, on the fp16 matrix cores (two parts of the activations, fp32 accuracy)
      rc = launch_dense_tiles(L.Wt, L.wt_parts, L.wt_exp, L.bias, cur, ldcur, out, ldo, B, L.d_in, L.d_out, act, w.tiles,
                              s);
      if (rc) return rc;
    } else if ((size_t)((B + 63) / 64) * ((L.d_out + 63) / 64) >= 256 ||
               ((size_t)((B + 31) / 32) * ((L.d_out + 31) / 32) >= 64 &&
                dense_small_supported(L.W, L.w_dtype, cur, ldcur, L.d_in))) {
      // a layer computed in full for a real batch is a dense contraction: matrix cores
      rc = launch_dense_layer(L.W, L.w_dtype, L.bias, cur, ldcur, out, ldo, B, L.d_in, L.d_out, act, w.dense_split, s);
      if (rc) return rc;
    } else {
      rc = launch_gather_forward(L.W, L.w_dtype, L.bias, cur, ldcur, nullptr, nullptr, 0, L.d_out, out, ldo,
                                 nullptr, 0, B, L.d_in, L.d_out, act, s);
      if (rc) return rc;
    }
    if (is_last) {
      if (!L.activated() && Y->cnt) {
        if (Y->idx && Y->stride < L.d_out)
          SLONN_FAIL(SLONN_ECAP, "compact output stride %d is below the last layer's %d nodes", Y->stride,
                     L.d_out);
        rc = launch_fill_iota(Y->idx, Y->stride, Y->cnt, L.d_out, B, s);
        if (rc) return rc;
      }
      rc = launch_finalize(out, ldo, L.d_out, act_list, act_cnt, act_stride, yc, Y->stride,
                           act == SLONN_ACT_SOFTMAX, Y->argmax, B, s);
      if (rc) return rc;
      if (tap_out && tap_out != out)
        SLONN_HIP(hipMemcpyAsync(tap_out, out, (size_t)B * L.d_out * 4, hipMemcpyDeviceToDevice, s));
    }
    cur = out;
    ldcur = ldo;
  }
  return SLONN_OK;
}

}  // namespace
}  // namespace slonn

int slonn_sparse_forward(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                         const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                         const slonn_debug_taps* taps, void* workspace, size_t ws_bytes,
                         void* stream) {
  return forward_impl(m, t, X, B, keep, keep_qstride, keep_lstride, Y, taps, workspace, ws_bytes, stream,
                      nullptr);
}

int slonn_sparse_forward_static(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                                const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                                const slonn_debug_taps* taps, void* stream) {
  if (!m) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (B <= 0 || B > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B must be in 1 .. %d", SLONN_MAX_BATCH);
  Workspace w;
  plan_workspace(m, B, nullptr, &w);
  if (w.bytes > (size_t)SLONN_STATIC_SCRATCH_BYTES)
    SLONN_FAIL(SLONN_ECAP, "a batch of %d needs %zu bytes of scratch memory, the static array holds %zu: use "
               "slonn_sparse_forward with a caller-provided workspace", B, w.bytes, (size_t)SLONN_STATIC_SCRATCH_BYTES);
  void* sp = nullptr;
  int rc = static_scratch(&sp);
  if (rc) return rc;
  return forward_impl(m, t, X, B, keep, keep_qstride, keep_lstride, Y, taps, sp, SLONN_STATIC_SCRATCH_BYTES, stream,
                      nullptr);
}

int slonn_sparse_forward_aclo(const slonn_model* m, const slonn_tables* t, const slonn_policy* p,
                              const slonn_input* X, int B, const float* thr, int thr_stride, float* keep_out,
                              slonn_output* Y, const slonn_debug_taps* taps, void* workspace, size_t ws_bytes,
                              void* stream) {
  if (!m || !p || !thr || !keep_out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (thr_stride < 0) SLONN_FAIL(SLONN_EINVAL, "negative stride");
  PolicyHook hook;
  hook.p = p; hook.thr = thr; hook.thr_stride = thr_stride; hook.keep_out = keep_out;
  for (int l = 0; l < (int)m->layers.size() && hook.layer < 0; ++l)
    if (m->layers[l].activated()) hook.layer = l;
  if (hook.layer < 0) SLONN_FAIL(SLONN_EINVAL, "the model has no activated layer to take keys from");
  const slonn::Layer& L0 = m->layers[hook.layer];
  if (!policy_matches(p, L0.K, L0.L))
    SLONN_FAIL(SLONN_EINVAL, "the policy's K and L differ from those of layer %d", hook.layer);
  if (!policy_trained(p)) SLONN_FAIL(SLONN_EINVAL, "the confidence tables have not been trained");
  // keep_out doubles as the keep array of the pass; it is written before it is first read
  return forward_impl(m, t, X, B, keep_out, 1, 0, Y, taps, workspace, ws_bytes, stream, &hook);
}

// ---- a recorded forward pass for launch-bound batches ----
struct slonn_graph {
  hipStream_t capture_stream = nullptr;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

int slonn_forward_graph_destroy(slonn_graph* g) {
  if (!g) return SLONN_OK;
  if (g->exec) (void)hipGraphExecDestroy(g->exec);
  if (g->graph) (void)hipGraphDestroy(g->graph);
  if (g->capture_stream) (void)hipStreamDestroy(g->capture_stream);
  delete g;
  return SLONN_OK;
}

int slonn_forward_graph_create(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                               const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                               void* workspace, size_t ws_bytes, slonn_graph** out) {
  if (!out) SLONN_FAIL(SLONN_EINVAL, "out is null");
  *out = nullptr;
  if (g_prof.on) SLONN_FAIL(SLONN_EINVAL, "switch per-kernel timing off before recording a graph");
  slonn_graph* g = new (std::nothrow) slonn_graph;
  if (!g) SLONN_FAIL(SLONN_ENOMEM, "out of host memory");
  auto fail = [&](int code) {
    slonn_forward_graph_destroy(g);
    return code;
  };
  hipError_t e = hipStreamCreateWithFlags(&g->capture_stream, hipStreamNonBlocking);
  if (e != hipSuccess) {
    set_error("creating the capture stream failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  // one eager pass first: it validates the arguments and sets the kernels' LDS attributes
  int rc = forward_impl(m, t, X, B, keep, keep_qstride, keep_lstride, Y, nullptr, workspace, ws_bytes,
                        g->capture_stream, nullptr);
  if (rc != SLONN_OK) return fail(rc);
  if ((e = hipStreamSynchronize(g->capture_stream)) != hipSuccess) {
    set_error("the eager pass before recording failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  if ((e = hipStreamBeginCapture(g->capture_stream, hipStreamCaptureModeThreadLocal)) != hipSuccess) {
    set_error("hipStreamBeginCapture failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  rc = forward_impl(m, t, X, B, keep, keep_qstride, keep_lstride, Y, nullptr, workspace, ws_bytes,
                    g->capture_stream, nullptr);
  e = hipStreamEndCapture(g->capture_stream, &g->graph);      // always end the capture, also after an error
  if (rc != SLONN_OK) return fail(rc);
  if (e != hipSuccess || !g->graph) {
    set_error("hipStreamEndCapture failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  if ((e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0)) != hipSuccess) {
    set_error("hipGraphInstantiate failed: %s", hipGetErrorString(e));
    return fail(SLONN_EHIP);
  }
  // the stream was only needed for the recording: a serving loop holds one graph per input buffer,
  // and hundreds of idle streams slow every later launch of the process down
  (void)hipStreamDestroy(g->capture_stream);
  g->capture_stream = nullptr;
  *out = g;
  return SLONN_OK;
}

int slonn_forward_graph_launch(slonn_graph* g, void* stream) {
  if (!g || !g->exec) SLONN_FAIL(SLONN_EINVAL, "graph is null");
  SLONN_HIP(hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)));
  return SLONN_OK;
}

int slonn_dense_forward(const slonn_model* m, const slonn_input* X, int B, float* Y, int32_t* argmax,
                        float** layer_out, void* workspace, size_t ws_bytes, void* stream) {
  if (!m || !X || !Y) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (B <= 0 || B > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B must be in 1 .. %d", SLONN_MAX_BATCH);
  int rc = check_input(m, X);
  if (rc) return rc;
  Workspace w;
  plan_workspace(m, B, static_cast<char*>(workspace), &w);
  if (!workspace || ws_bytes < w.bytes)
    SLONN_FAIL(SLONN_ENOMEM, "workspace holds %zu bytes, %zu needed", ws_bytes, w.bytes);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nl = (int)m->layers.size();
  const float* cur = X->x;
  int ldcur = m->layers[0].d_in;
  for (int l = 0; l < nl; ++l) {
    const Layer& L = m->layers[l];
    const bool is_last = (l == nl - 1);
    float* out = is_last ? Y : (layer_out && layer_out[l] ? layer_out[l] : w.act[l & 1]);
    if (l == 0 && X->format == SLONN_ELL)
      rc = launch_ell_layer(L.W, L.w_dtype, L.w_layout, L.bias, X->idx, X->val, X->nnz, X->ell_stride, out,
                            L.d_out, B, L.d_in, L.d_out, L.act, s);
    else if (m->dense_arith == SLONN_DENSE_F16_PARTS && w.tiles && L.Wt &&
             (long)((B + 63) / 64) * ((L.d_out + 127) / 128) >= 64 &&
             masked_tiles_workspace_bytes(B, L.d_out, L.d_in) <= w.tiles_bytes)
      // the arithmetic of the masked tiles without a mask: activations (and fp32 weights) as two fp16
      // parts on the fp16 matrix cores, fp32 accumulation
      rc = launch_dense_tiles(L.Wt, L.wt_parts, L.wt_exp, L.bias, cur, ldcur, out, L.d_out, B, L.d_in, L.d_out, L.act,
                              w.tiles, s);
    else
      rc = launch_dense_layer(L.W, L.w_dtype, L.bias, cur, ldcur, out, L.d_out, B, L.d_in, L.d_out, L.act,
                              w.dense_split, s);
    if (rc) return rc;
    if (is_last) {
      rc = launch_finalize(out, L.d_out, L.d_out, nullptr, nullptr, 0, nullptr, 0, L.act == SLONN_ACT_SOFTMAX,
                           argmax, B, s);
      if (rc) return rc;
      if (layer_out && layer_out[l] && layer_out[l] != out)
        SLONN_HIP(hipMemcpyAsync(layer_out[l], out, (size_t)B * L.d_out * 4, hipMemcpyDeviceToDevice, s));
    }
    cur = out;
    ldcur = L.d_out;
  }
  return SLONN_OK;
}

}  // extern "C"
