// C-ABI entry points of the wave-index library: planning, argument checks,
// dispatch to the build and decode launch code, the host-side seed-point hook
// and the event profiler.
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "wave_common.h"

namespace wave {

// ----------------------------------------------------------------------------
// Profiler: brackets every launch with HIP events on the launch's own stream.
// ----------------------------------------------------------------------------
bool g_profile_on = false;

namespace {
constexpr int kMaxPending = 8192;
constexpr int kMaxNames = 64;
struct Pending {
  const char* name;
  hipEvent_t start, stop;
};
Pending g_pending[kMaxPending];
int g_npending = 0;
int g_pool_ready = 0;
hipEvent_t g_pool[2 * kMaxPending];
const char* g_names[kMaxNames];
float g_ms[kMaxNames];
int g_count[kMaxNames];
int g_nnames = 0;
bool g_profile_error = false;

void drain() {
  for (int i = 0; i < g_npending; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(g_pending[i].stop) != hipSuccess ||
        hipEventElapsedTime(&ms, g_pending[i].start, g_pending[i].stop) != hipSuccess) {
      g_profile_error = true;
      continue;
    }
    int k = 0;
    while (k < g_nnames && g_names[k] != g_pending[i].name && strcmp(g_names[k], g_pending[i].name)) ++k;
    if (k == g_nnames) {
      if (g_nnames == kMaxNames) continue;
      g_names[g_nnames] = g_pending[i].name;
      g_ms[g_nnames] = 0.f;
      g_count[g_nnames] = 0;
      ++g_nnames;
    }
    g_ms[k] += ms;
    g_count[k] += 1;
  }
  g_npending = 0;
}
}  // namespace

void profile_before(const char* name, hipStream_t st) {
  if (g_npending == kMaxPending) drain();
  Pending& p = g_pending[g_npending];
  p.name = name;
  p.start = g_pool[2 * g_npending];
  p.stop = g_pool[2 * g_npending + 1];
  if (hipEventRecord(p.start, st) != hipSuccess) g_profile_error = true;
}
void profile_after(hipStream_t st) {
  if (hipEventRecord(g_pending[g_npending].stop, st) != hipSuccess) g_profile_error = true;
  ++g_npending;
}

// ----------------------------------------------------------------------------
// Calibration kernels: plain streaming of a buffer of known size.  Profiler
// counters read for them give the factor between counter units and bytes, and
// their rate is the bandwidth a simple kernel reaches on this machine.
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void calib_copy_kernel(uint4* __restrict__ dst,
                                                         const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void calib_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                         uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t acc = 0;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive; practically never true
}

// ----------------------------------------------------------------------------
// Planning
// ----------------------------------------------------------------------------
static wave_status check_dims(const wave_index* ix) {
  if (!ix) return WAVE_ERR_ARG;
  if (ix->dtype != WAVE_F32 && ix->dtype != WAVE_BF16) return WAVE_ERR_DTYPE;
  if (ix->B < 1 || ix->Hkv < 1 || ix->N < 1 || ix->n_sink < 0 || ix->n_local < 0) return WAVE_ERR_ARG;
  if (ix->segment_len < 1 || ix->clusters_per_segment < 1) return WAVE_ERR_ARG;
  if (ix->d != 64 && ix->d != 128) return WAVE_ERR_SHAPE;
  if (ix->clusters_per_segment > WAVE_MAX_CLUSTERS_PER_SEGMENT) return WAVE_ERR_SHAPE;
  if (ix->appended_segments < 0 || ix->row_capacity < 0 || ix->steady_capacity < 0) return WAVE_ERR_ARG;
  if (ix->cluster_capacity < 0) return WAVE_ERR_ARG;
  if (ix->appended_segments > 0) {
    if (ix->update_segment_len < 1 || ix->update_clusters < 1) return WAVE_ERR_ARG;
    if (ix->update_clusters > WAVE_MAX_CLUSTERS_PER_SEGMENT) return WAVE_ERR_SHAPE;
  }
  return WAVE_OK;
}

struct Derived {
  int ns, local_start, N_idx, S, m, p;
};
static Derived derive(const wave_index& ix) {
  Derived d;
  d.ns = ix.n_sink < ix.N ? ix.n_sink : ix.N;
  const long long ls = (long long)ix.N - ix.n_local;
  d.local_start = ls > d.ns ? (int)ls : d.ns;
  d.N_idx = d.local_start - d.ns;
  d.p = d.ns + (ix.N - d.local_start);
  const int L = ix.segment_len, k = ix.clusters_per_segment;
  // the build's segments tile the indexed range without the update segments behind them
  const int A = ix.appended_segments, U = ix.update_segment_len;
  const int ku = ix.update_clusters < U ? ix.update_clusters : U;
  long long built = (long long)d.N_idx - (long long)A * U;
  if (A == 0) built = d.N_idx;
  if (built < 0) built = -1;  // inconsistent: no plan matches
  const int nb = (int)built;
  d.S = (nb + L - 1) / L + A;
  const int full = nb / L, tail = nb - full * L;
  d.m = full * (k < L ? k : L) + (tail > 0 ? (k < tail ? k : tail) : 0) + (A > 0 ? A * ku : 0);
  if (built < 0) d.m = -1;
  return d;
}

static bool planned_fields_match(const wave_index& ix) {
  const Derived d = derive(ix);
  if (ix.row_capacity > 0 && ix.row_capacity < d.N_idx) return false;
  if (ix.steady_capacity > 0 && ix.steady_capacity < d.p) return false;
  if (ix.cluster_capacity > 0 && ix.cluster_capacity < d.m) return false;
  return ix.S == d.S && ix.m == d.m && ix.N_idx == d.N_idx && ix.p == d.p;
}

BuildGeom build_geometry(const wave_index& ix);  // wave_build.hip

}  // namespace wave

using namespace wave;

extern "C" {

wave_status wave_index_plan(wave_index* ix, size_t bytes[WAVE_INDEX_BUFFERS],
                            size_t* build_workspace_bytes, int Hq, int topk_clusters,
                            size_t* decode_workspace_bytes) {
  wave_status st = check_dims(ix);
  if (st != WAVE_OK) return st;
  if (!bytes) return WAVE_ERR_ARG;
  const Derived d = derive(*ix);
  if (d.m < 0 || (ix->row_capacity > 0 && ix->row_capacity < d.N_idx)) return WAVE_ERR_SHAPE;
  if (ix->cluster_capacity > 0 && ix->cluster_capacity < d.m) return WAVE_ERR_SHAPE;
  const size_t mcap = ix->cluster_capacity > 0 ? (size_t)ix->cluster_capacity : (size_t)d.m;
  if ((long long)ix->B * ix->Hkv * ((long long)mcap + 1) >= (1ll << 31)) return WAVE_ERR_SHAPE;
  if (ix->steady_capacity > 0 && ix->steady_capacity < d.p) return WAVE_ERR_SHAPE;
  ix->S = d.S;
  ix->m = d.m;
  ix->N_idx = d.N_idx;
  ix->p = d.p;
  const size_t es = ix->dtype == WAVE_BF16 ? 2 : 4;
  const size_t units = (size_t)ix->B * ix->Hkv;
  bytes[0] = units * mcap * ix->d * es;
  bytes[1] = units * mcap * ix->d * es;
  bytes[2] = units * mcap * sizeof(int32_t);
  bytes[3] = units * (mcap + 1) * sizeof(int32_t);
  const size_t rows = ix->row_capacity > 0 ? (size_t)ix->row_capacity : (size_t)d.N_idx;
  bytes[4] = units * rows * sizeof(int32_t);
  bytes[5] = units * rows * ix->d * es;
  bytes[6] = bytes[5];
  bytes[7] = units * (ix->steady_capacity > 0 ? (size_t)ix->steady_capacity : (size_t)d.p) * ix->d * es;
  bytes[8] = bytes[7];
  if (build_workspace_bytes) *build_workspace_bytes = build_geometry(*ix).total;
  if (decode_workspace_bytes) {
    if (Hq < ix->Hkv || Hq % ix->Hkv != 0 || Hq / ix->Hkv > 8) return WAVE_ERR_SHAPE;
    if (topk_clusters < 0) return WAVE_ERR_ARG;
    *decode_workspace_bytes = decode_geometry(*ix, Hq, topk_clusters).total;
  }
  return WAVE_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static wave_status check_index_buffers(const wave_index& ix) {
  if (ix.m > 0) {
    if (!ix.centroids || !ix.vsum || !ix.sizes || !ix.offsets) return WAVE_ERR_ARG;
    if (!ix.perm || !ix.k_perm || !ix.v_perm) return WAVE_ERR_ARG;
    if (!aligned16(ix.centroids) || !aligned16(ix.vsum) || !aligned16(ix.k_perm) || !aligned16(ix.v_perm))
      return WAVE_ERR_ARG;
  }
  if (ix.p > 0) {
    if (!ix.k_steady || !ix.v_steady) return WAVE_ERR_ARG;
    if (!aligned16(ix.k_steady) || !aligned16(ix.v_steady)) return WAVE_ERR_ARG;
  }
  return WAVE_OK;
}

wave_status wave_index_build(const void* K, const void* V, wave_index* ix, int iters, uint64_t seed,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  wave_status st = check_dims(ix);
  if (st != WAVE_OK) return st;
  if (!K || !V || iters < 1) return WAVE_ERR_ARG;
  if (!aligned16(K) || !aligned16(V)) return WAVE_ERR_ARG;
  if (ix->appended_segments != 0) return WAVE_ERR_SHAPE;  // the build tiles the whole range with L
  if (!planned_fields_match(*ix)) return WAVE_ERR_SHAPE;
  st = check_index_buffers(*ix);
  if (st != WAVE_OK) return st;
  const BuildGeom g = build_geometry(*ix);
  if (g.total > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < g.total))
    return WAVE_ERR_WORKSPACE;
  return launch_build(K, V, *ix, iters, seed, workspace, static_cast<hipStream_t>(hip_stream));
}

// ----------------------------------------------------------------------------
// Incremental update
// ----------------------------------------------------------------------------
extern "C++" {
namespace wave {
AppendGeom append_geometry(const wave_index& old_ix, int n_new, int n_local_min, int U, int k_u) {
  AppendGeom g{};
  const Derived d = derive(old_ix);
  g.lc_old = old_ix.N - d.local_start;
  const long long window = (long long)g.lc_old + n_new - n_local_min;
  g.F = window > 0 ? (int)(window / U) : 0;
  g.ks = k_u < U ? k_u : U;
  wave_index& mi = g.mini;
  mi = wave_index{};
  mi.dtype = old_ix.dtype;
  mi.B = old_ix.B;
  mi.Hkv = old_ix.Hkv;
  mi.d = old_ix.d;
  mi.N = g.F * U;
  mi.segment_len = U;
  mi.clusters_per_segment = k_u;
  mi.S = g.F;
  mi.m = g.F * g.ks;
  mi.N_idx = g.F * U;
  const size_t es = old_ix.dtype == WAVE_BF16 ? 2 : 4, units = (size_t)old_ix.B * old_ix.Hkv;
  const size_t rows = units * (size_t)mi.N_idx * old_ix.d * es;
  size_t o = 0;
  g.off_k = o;       o = align_up(o + rows);
  g.off_v = o;       o = align_up(o + rows);
  g.off_build = o;
  if (g.F > 0) o = align_up(o + build_geometry(mi).total);
  g.total = g.F > 0 ? o : 0;
  return g;
}
}  // namespace wave
}  // extern "C++"

static wave_status plan_append(const wave_index* old_ix, int n_new, int n_local_min, int U, int k_u,
                               wave_index* out) {
  wave_status st = check_dims(old_ix);
  if (st != WAVE_OK) return st;
  if (!out || n_new < 0 || n_local_min < 0 || U < 1 || k_u < 1) return WAVE_ERR_ARG;
  if (k_u > WAVE_MAX_CLUSTERS_PER_SEGMENT) return WAVE_ERR_SHAPE;
  if (!planned_fields_match(*old_ix)) return WAVE_ERR_SHAPE;
  if (old_ix->N < old_ix->n_sink) return WAVE_ERR_SHAPE;  // the sink zone itself is still filling
  if (old_ix->appended_segments > 0 &&
      (U != old_ix->update_segment_len || k_u != old_ix->update_clusters))
    return WAVE_ERR_SHAPE;
  if ((long long)old_ix->N + n_new >= (1ll << 31)) return WAVE_ERR_SHAPE;
  const AppendGeom g = append_geometry(*old_ix, n_new, n_local_min, U, k_u);
  wave_index nw = *old_ix;
  nw.centroids = nw.vsum = nullptr;
  nw.sizes = nw.offsets = nw.perm = nullptr;
  nw.k_perm = nw.v_perm = nw.k_steady = nw.v_steady = nullptr;
  nw.N = old_ix->N + n_new;
  nw.n_local = g.lc_old + n_new - g.F * U;
  nw.appended_segments = old_ix->appended_segments + g.F;
  nw.update_segment_len = U;
  nw.update_clusters = k_u;
  if ((long long)old_ix->N_idx + (long long)g.F * U > old_ix->row_capacity) nw.row_capacity = 0;
  if (old_ix->n_sink + nw.n_local > old_ix->steady_capacity) nw.steady_capacity = 0;
  if ((long long)old_ix->m + (long long)g.F * g.ks > old_ix->cluster_capacity) nw.cluster_capacity = 0;
  *out = nw;
  return WAVE_OK;
}

wave_status wave_index_append_plan(const wave_index* old_ix, int n_new, int n_local_min,
                                   int update_segment_len, int update_clusters, wave_index* new_ix,
                                   size_t bytes[WAVE_INDEX_BUFFERS], size_t* workspace_bytes) {
  wave_index nw;
  wave_status st = plan_append(old_ix, n_new, n_local_min, update_segment_len, update_clusters, &nw);
  if (st != WAVE_OK) return st;
  if (!new_ix || !bytes) return WAVE_ERR_ARG;
  st = wave_index_plan(&nw, bytes, nullptr, 0, 0, nullptr);
  if (st != WAVE_OK) return st;
  *new_ix = nw;
  if (workspace_bytes)
    *workspace_bytes = append_geometry(*old_ix, n_new, n_local_min, update_segment_len, update_clusters).total;
  return WAVE_OK;
}

wave_status wave_index_append(const wave_index* old_ix, const void* K_new, const void* V_new,
                              int n_new, int n_local_min, int update_segment_len,
                              int update_clusters, int iters, uint64_t seed, wave_index* new_ix,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  wave_index want;
  wave_status st = plan_append(old_ix, n_new, n_local_min, update_segment_len, update_clusters, &want);
  if (st != WAVE_OK) return st;
  if (!new_ix || iters < 1) return WAVE_ERR_ARG;
  if (n_new > 0 && (!K_new || !V_new || !aligned16(K_new) || !aligned16(V_new))) return WAVE_ERR_ARG;
  st = check_dims(new_ix);
  if (st != WAVE_OK) return st;
  if (new_ix->dtype != want.dtype || new_ix->B != want.B || new_ix->Hkv != want.Hkv ||
      new_ix->d != want.d || new_ix->N != want.N || new_ix->n_sink != want.n_sink ||
      new_ix->n_local != want.n_local || new_ix->segment_len != want.segment_len ||
      new_ix->clusters_per_segment != want.clusters_per_segment ||
      new_ix->appended_segments != want.appended_segments ||
      new_ix->update_segment_len != want.update_segment_len ||
      new_ix->update_clusters != want.update_clusters || !planned_fields_match(*new_ix))
    return WAVE_ERR_SHAPE;  // (row_capacity of new_ix is the caller's choice, checked against its N_idx)
  st = check_index_buffers(*old_ix);
  if (st != WAVE_OK) return st;
  st = check_index_buffers(*new_ix);
  if (st != WAVE_OK) return st;
  const AppendGeom g = append_geometry(*old_ix, n_new, n_local_min, update_segment_len, update_clusters);
  {  // the seven arrays of the clustered part may be the old ones only if nothing is appended to them
    const void* a[7] = {old_ix->centroids, old_ix->vsum, old_ix->sizes, old_ix->offsets, old_ix->perm,
                        old_ix->k_perm, old_ix->v_perm};
    const void* b[7] = {new_ix->centroids, new_ix->vsum, new_ix->sizes, new_ix->offsets, new_ix->perm,
                        new_ix->k_perm, new_ix->v_perm};
    const bool in_place = new_ix->row_capacity > 0 && new_ix->row_capacity == old_ix->row_capacity;
    const bool meta_in_place = new_ix->cluster_capacity > 0 && new_ix->cluster_capacity == old_ix->cluster_capacity;
    for (int i = 0; i < 7; ++i) {
      if (g.F > 0 && a[i] && a[i] == b[i] && !(i >= 4 ? in_place : meta_in_place)) return WAVE_ERR_ARG;
      // an array both indexes name is read with one stride per unit
      if (a[i] && a[i] == b[i] &&
          (i >= 4 ? row_stride(*old_ix) != row_stride(*new_ix) : cluster_stride(*old_ix) != cluster_stride(*new_ix)))
        return WAVE_ERR_ARG;
    }
    const bool steady_in_place = g.F == 0 && new_ix->steady_capacity > 0 &&
                                 new_ix->steady_capacity == old_ix->steady_capacity;
    if (old_ix->k_steady && !steady_in_place &&
        (old_ix->k_steady == new_ix->k_steady || old_ix->v_steady == new_ix->v_steady))
      return WAVE_ERR_ARG;
    if (steady_in_place && (old_ix->k_steady == new_ix->k_steady) != (old_ix->v_steady == new_ix->v_steady))
      return WAVE_ERR_ARG;
  }
  if (g.total > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < g.total))
    return WAVE_ERR_WORKSPACE;
  return launch_append(*old_ix, K_new, V_new, n_new, iters, seed, *new_ix, g, workspace,
                       static_cast<hipStream_t>(hip_stream));
}

wave_status wave_attention_decode(const void* q, const wave_index* ix, int Hq, int topk_clusters,
                                  int n_sink, int n_local, float* out, float* lse, int32_t* selected,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  wave_status st = check_dims(ix);
  if (st != WAVE_OK) return st;
  if (!q || !out || !lse || topk_clusters < 0) return WAVE_ERR_ARG;
  if (!aligned16(q)) return WAVE_ERR_ARG;
  if (Hq < ix->Hkv || Hq % ix->Hkv != 0 || Hq / ix->Hkv > 8) return WAVE_ERR_SHAPE;
  if (!planned_fields_match(*ix)) return WAVE_ERR_SHAPE;
  if (n_sink != ix->n_sink || n_local != ix->n_local) return WAVE_ERR_STEADY_MISMATCH;
  st = check_index_buffers(*ix);
  if (st != WAVE_OK) return st;
  const DecodeGeom g = decode_geometry(*ix, Hq, topk_clusters);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < g.total)
    return WAVE_ERR_WORKSPACE;
  return launch_decode(q, *ix, Hq, topk_clusters, out, lse, selected, workspace,
                       static_cast<hipStream_t>(hip_stream));
}

// ----------------------------------------------------------------------------
// Decode without a caller workspace: the scratch memory is a static device array.
// Every GPU the library runs on holds its own copy at its own address, found once
// per device with hipGetSymbolAddress; after that only that address is used (the
// array's name is a host-side stand-in, not a device address).
// ----------------------------------------------------------------------------
}  // extern "C"

namespace {
constexpr size_t kStaticScratchBytes = (size_t)WAVE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// The device-side address of `scratch` on the current device (nullptr on error).
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  void* addr = nullptr;
  if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) return nullptr;
  if (reinterpret_cast<uintptr_t>(addr) & 255u) return nullptr;
  g_scratch_ptr[dev].store(addr, std::memory_order_release);
  return addr;
}
}  // namespace

extern "C" {

size_t wave_attention_decode_static_capacity(void) { return kStaticScratchBytes; }

wave_status wave_attention_decode_static(const void* q, const wave_index* ix, int Hq, int topk_clusters,
                                         int n_sink, int n_local, float* out, float* lse,
                                         int32_t* selected, void* hip_stream) {
  wave_status st = check_dims(ix);
  if (st != WAVE_OK) return st;
  if (!q || !out || !lse || topk_clusters < 0) return WAVE_ERR_ARG;
  if (!aligned16(q)) return WAVE_ERR_ARG;
  if (Hq < ix->Hkv || Hq % ix->Hkv != 0 || Hq / ix->Hkv > 8) return WAVE_ERR_SHAPE;
  if (!planned_fields_match(*ix)) return WAVE_ERR_SHAPE;
  if (n_sink != ix->n_sink || n_local != ix->n_local) return WAVE_ERR_STEADY_MISMATCH;
  st = check_index_buffers(*ix);
  if (st != WAVE_OK) return st;
  // The step's scratch layout is the one of wave_attention_decode; a step that needs more
  // than the static array holds is refused here, before anything is launched.
  const DecodeGeom g = decode_geometry(*ix, Hq, topk_clusters);
  if (g.total > kStaticScratchBytes) return WAVE_ERR_WORKSPACE;
  void* ws = static_scratch();
  if (!ws) return WAVE_ERR_HIP;
  return launch_decode(q, *ix, Hq, topk_clusters, out, lse, selected, ws,
                       static_cast<hipStream_t>(hip_stream));
}

static wave_status check_decode_args(const void* q, const wave_index* ix, int Hq, int topk_clusters,
                                     int n_sink, int n_local, const float* out, const float* lse) {
  wave_status st = check_dims(ix);
  if (st != WAVE_OK) return st;
  if (!q || !out || !lse || topk_clusters < 0) return WAVE_ERR_ARG;
  if (!aligned16(q)) return WAVE_ERR_ARG;
  if (Hq < ix->Hkv || Hq % ix->Hkv != 0 || Hq / ix->Hkv > 8) return WAVE_ERR_SHAPE;
  if (!planned_fields_match(*ix)) return WAVE_ERR_SHAPE;
  if (n_sink != ix->n_sink || n_local != ix->n_local) return WAVE_ERR_STEADY_MISMATCH;
  return check_index_buffers(*ix);
}

size_t wave_attention_decode_budget_workspace(const wave_index* ix, int Hq, int topk_clusters,
                                              int est_clusters) {
  if (check_dims(ix) != WAVE_OK || !planned_fields_match(*ix) || topk_clusters < 0) return 0;
  if (Hq < ix->Hkv || Hq % ix->Hkv != 0 || Hq / ix->Hkv > 8) return 0;
  return budget_geometry(*ix, Hq, topk_clusters, est_clusters).total;
}

wave_status wave_attention_decode_budget(const void* q, const wave_index* ix, int Hq, int topk_clusters,
                                         int est_clusters, int n_sink, int n_local, float* out,
                                         float* lse, int32_t* selected, void* workspace,
                                         size_t workspace_bytes, void* hip_stream) {
  const wave_status st = check_decode_args(q, ix, Hq, topk_clusters, n_sink, n_local, out, lse);
  if (st != WAVE_OK) return st;
  const size_t need = budget_geometry(*ix, Hq, topk_clusters, est_clusters).total;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
    return WAVE_ERR_WORKSPACE;
  return launch_decode_budget(q, *ix, Hq, topk_clusters, est_clusters, out, lse, selected, workspace,
                              static_cast<hipStream_t>(hip_stream));
}

size_t wave_full_attention_workspace(int B, int Hq, int N, int d) {
  if (B < 1 || Hq < 1 || N < 1 || (d != 64 && d != 128)) return 0;
  return align_up(sizeof(float) * (size_t)B * Hq * full_attention_chunks(N) * (d + 2));
}

wave_status wave_full_attention_decode(const void* q, const void* K, const void* V, int dtype, int B,
                                       int Hq, int Hkv, int N, int d, float* out, float* lse,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (dtype != WAVE_F32 && dtype != WAVE_BF16) return WAVE_ERR_DTYPE;
  if (!q || !K || !V || !out || !lse || B < 1 || Hkv < 1 || N < 1) return WAVE_ERR_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V)) return WAVE_ERR_ARG;
  if (d != 64 && d != 128) return WAVE_ERR_SHAPE;
  if (Hq < Hkv || Hq % Hkv != 0 || Hq / Hkv > 8) return WAVE_ERR_SHAPE;
  if ((long long)B * Hkv * full_attention_chunks(N) >= (1ll << 31)) return WAVE_ERR_SHAPE;
  const size_t need = wave_full_attention_workspace(B, Hq, N, d);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
    return WAVE_ERR_WORKSPACE;
  return launch_full_attention(q, K, V, dtype, B, Hq, Hkv, N, d, out, lse, workspace,
                               static_cast<hipStream_t>(hip_stream));
}

wave_status wave_init_indices(uint64_t seed, int b, int h, int s, int L_s, int k_s, int32_t* out) {
  if (!out || L_s < 1 || k_s < 1 || k_s > L_s) return WAVE_ERR_ARG;
  // Fisher-Yates on a sparse image of the array: only positions that were
  // swapped differ from the identity, and at most k_s of them exist.
  struct Moved { int pos, val; };
  Moved* moved = new Moved[k_s];
  int nmoved = 0;
  uint64_t st = init_stream_state(seed, b, h, s);
  for (int i = 0; i < k_s; ++i) {
    const uint64_t draw = splitmix64_next(st);
    const int j = i + (int)(draw % (uint64_t)(L_s - i));
    // value currently at j and at i
    int vj = j, vi = i, at_j = -1;
    for (int t = 0; t < nmoved; ++t) {
      if (moved[t].pos == j) { vj = moved[t].val; at_j = t; }
      if (moved[t].pos == i) vi = moved[t].val;
    }
    out[i] = vj;
    if (j != i) {
      if (at_j >= 0) moved[at_j].val = vi;
      else { moved[nmoved].pos = j; moved[nmoved].val = vi; ++nmoved; }
    }
  }
  delete[] moved;
  return WAVE_OK;
}

wave_status wave_kmeans_assign_step(const void* xhat, const void* chat, int dtype, int L_s, int k_s,
                                    int d, int32_t* assign, void* workspace, size_t workspace_bytes,
                                    void* hip_stream) {
  if (!xhat || !chat || !assign) return WAVE_ERR_ARG;
  if (dtype != WAVE_F32 && dtype != WAVE_BF16) return WAVE_ERR_DTYPE;
  if (d != 64 && d != 128) return WAVE_ERR_SHAPE;
  if (L_s < 1 || k_s < 1 || k_s > WAVE_MAX_CLUSTERS_PER_SEGMENT || k_s > L_s) return WAVE_ERR_SHAPE;
  if (!aligned16(xhat) || !aligned16(chat)) return WAVE_ERR_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) ||
      workspace_bytes < (size_t)4 * L_s + 1024)
    return WAVE_ERR_WORKSPACE;
  return launch_assign_step(xhat, chat, dtype, L_s, k_s, d, assign, workspace,
                            static_cast<hipStream_t>(hip_stream));
}

wave_status wave_calibration_copy(void* dst, const void* src, size_t bytes, int workgroups,
                                  void* hip_stream) {
  if (!dst || !src || bytes == 0 || (bytes & 15u) || workgroups < 1) return WAVE_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return WAVE_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  WAVE_LAUNCH("calib_copy", calib_copy_kernel, workgroups, 256, 0, st, static_cast<uint4*>(dst),
              static_cast<const uint4*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

wave_status wave_calibration_read(const void* src, size_t bytes, void* sink, int workgroups,
                                  void* hip_stream) {
  if (!sink || !src || bytes == 0 || (bytes & 15u) || workgroups < 1) return WAVE_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(src) & 15u) return WAVE_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  WAVE_LAUNCH("calib_read", calib_read_kernel, workgroups, 256, 0, st, static_cast<const uint4*>(src),
              bytes / 16, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

wave_status wave_profile_enable(int on) {
  if (on && !g_pool_ready) {
    for (int i = 0; i < 2 * kMaxPending; ++i)
      if (hipEventCreate(&g_pool[i]) != hipSuccess) return WAVE_ERR_HIP;
    g_pool_ready = 1;
  }
  if (!on && g_profile_on) drain();
  g_profile_on = on != 0;
  return WAVE_OK;
}

int wave_profile_read(const char** names, float* total_ms, int* launches, int cap) {
  drain();
  if (g_profile_error) {
    g_profile_error = false;
    g_nnames = 0;
    return -1;
  }
  const int n = g_nnames;
  for (int i = 0; i < n && i < cap; ++i) {
    if (names) names[i] = g_names[i];
    if (total_ms) total_ms[i] = g_ms[i];
    if (launches) launches[i] = g_count[i];
  }
  g_nnames = 0;
  return n;
}

const char* wave_status_string(wave_status st) {
  switch (st) {
    case WAVE_OK: return "ok";
    case WAVE_ERR_ARG: return "invalid argument";
    case WAVE_ERR_SHAPE: return "unsupported or inconsistent shape";
    case WAVE_ERR_DTYPE: return "unsupported dtype";
    case WAVE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case WAVE_ERR_STEADY_MISMATCH: return "n_sink/n_local differ from the index";
    case WAVE_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

}  // extern "C"
