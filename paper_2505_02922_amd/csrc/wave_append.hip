// Index update during decoding ("Lightweight Index Construction", last
// paragraph): new tokens join the local window; whole update segments of the
// window's oldest tokens are clustered on their own, as segments of the build,
// and their clusters are appended to the index.
//
// The index arrays are dense per (sequence, KV head) unit, so an index with
// more clusters has other strides: the result is written as a new index.  The
// steps: (1) the old arrays are copied to the new strides; (2) the window (old
// local rows, then the new tokens) is routed row by row, its flushed prefix to a
// scratch key/value tensor and the rest to the new steady rows; (3) the flushed
// tokens are clustered by the build's kernels, with their segments numbered
// after the old ones for the seeding rule, and the build's last step writes
// their clusters and rows straight behind the old ones in the new index's
// arrays (offsets continued from the old row count, positions from the window's
// first position).  When arrays of both indexes are the same buffers with room
// left (row_capacity for perm, k_perm, v_perm; cluster_capacity for the meta
// index), step (1) skips them: the update then writes only what is new.
#include "wave_common.h"

namespace wave {

// dst[u * dst_stride + dst_off + i] = src[u * src_stride + i] (+ add), i < n, for every unit u.
template <typename C>
__global__ __launch_bounds__(256) void copy_units_kernel(C* __restrict__ dst, const C* __restrict__ src,
                                                         size_t n, size_t dst_stride, size_t src_stride,
                                                         size_t dst_off, int units) {
  const size_t total = n * (size_t)units, step = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += step) {
    const size_t u = i / n, j = i - u * n;
    dst[u * dst_stride + dst_off + j] = src[u * src_stride + j];
  }
}
__global__ __launch_bounds__(256) void set_first_kernel(int32_t* __restrict__ dst, size_t stride, int units) {
  const int u = blockIdx.x * 256 + threadIdx.x;
  if (u < units) dst[(size_t)u * stride] = 0;
}

// Row j of a unit's sink + window (ns sink rows of the old steady buffer, lc_old
// old local rows, n_new new tokens) goes to: the new steady buffer as it is
// (sink), the scratch tensor (window rows before `flush`), or the new steady
// buffer behind the sink rows.  One thread per 16-byte chunk of a row.
template <int ROWB>
__global__ __launch_bounds__(256) void route_window_kernel(
    const char* __restrict__ ks_old, const char* __restrict__ vs_old, const char* __restrict__ k_new,
    const char* __restrict__ v_new, char* __restrict__ k_flush, char* __restrict__ v_flush,
    char* __restrict__ ks_out, char* __restrict__ vs_out, int ns, int lc_old, int n_new, int flush,
    int p_old, int p_out, int units, int first) {
  // p_old, p_out: rows per unit of the old and the new steady buffers; first: rows before it are
  // already in place (the new buffers are the old ones and nothing is flushed)
  constexpr int CPR = ROWB / 16;
  const size_t rows_u = (size_t)ns + lc_old + n_new - first;
  const size_t total = rows_u * units * CPR, step = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += step) {
    const size_t row = i / CPR, ch = i - row * CPR;
    const size_t u = row / rows_u;
    const int j = (int)(row - u * rows_u) + first;
    const char *sk, *sv;
    if (j < ns + lc_old) {
      sk = ks_old + ((size_t)u * p_old + j) * ROWB;
      sv = vs_old + ((size_t)u * p_old + j) * ROWB;
    } else {
      sk = k_new + ((size_t)u * n_new + (j - ns - lc_old)) * ROWB;
      sv = v_new + ((size_t)u * n_new + (j - ns - lc_old)) * ROWB;
    }
    char *dk, *dv;
    const int w = j - ns;  // position in the window; negative for sink rows
    if (w >= 0 && w < flush) {
      dk = k_flush + ((size_t)u * flush + w) * ROWB;
      dv = v_flush + ((size_t)u * flush + w) * ROWB;
    } else {
      const int r = w < 0 ? j : ns + (w - flush);
      dk = ks_out + ((size_t)u * p_out + r) * ROWB;
      dv = vs_out + ((size_t)u * p_out + r) * ROWB;
    }
    *reinterpret_cast<uint4*>(dk + ch * 16) = *reinterpret_cast<const uint4*>(sk + ch * 16);
    *reinterpret_cast<uint4*>(dv + ch * 16) = *reinterpret_cast<const uint4*>(sv + ch * 16);
  }
}

static int grid_for(size_t items) {
  const size_t g = (items + 255) / 256;
  return (int)(g < 1 ? 1 : (g > 65536 ? 65536 : g));
}

template <typename C>
static void copy_units(void* dst, const void* src, size_t n, size_t dst_stride, size_t src_stride,
                       size_t dst_off, int units, hipStream_t st) {
  if (n == 0 || dst == src) return;  // (an update that flushes nothing may keep the old arrays)
  WAVE_LAUNCH("append_copy", (copy_units_kernel<C>), grid_for(n * units), 256, 0, st,
              static_cast<C*>(dst), static_cast<const C*>(src), n, dst_stride, src_stride, dst_off, units);
}

wave_status launch_append(const wave_index& o, const void* K_new, const void* V_new, int n_new,
                          int iters, uint64_t seed, const wave_index& nw, const AppendGeom& g, void* ws,
                          hipStream_t st) {
  const int units = o.B * o.Hkv, D = o.d;
  const size_t es = o.dtype == WAVE_BF16 ? 2 : 4;
  const size_t rowc = (size_t)D * es / 16;  // 16-byte chunks per row
  const int U = nw.update_segment_len, flush = g.F * U;
  const int ns = o.n_sink;                  // old N >= n_sink was checked
  char* w = static_cast<char*>(ws);

  // (1) the old index at the new strides (arrays that are the old ones stay as they are)
  const size_t cs_new = (size_t)cluster_stride(nw), cs_old = (size_t)cluster_stride(o);  // clusters per unit
  copy_units<uint4>(nw.centroids, o.centroids, (size_t)o.m * rowc, cs_new * rowc, cs_old * rowc, 0, units, st);
  copy_units<uint4>(nw.vsum, o.vsum, (size_t)o.m * rowc, cs_new * rowc, cs_old * rowc, 0, units, st);
  copy_units<int32_t>(nw.sizes, o.sizes, (size_t)o.m, cs_new, cs_old, 0, units, st);
  if (o.offsets)
    copy_units<int32_t>(nw.offsets, o.offsets, (size_t)o.m + 1, cs_new + 1, cs_old + 1, 0, units, st);
  else if (nw.offsets)  // no clusters before and no array for them: the first offset of every unit is 0
    WAVE_LAUNCH("append_copy", set_first_kernel, grid_for(units), 256, 0, st, nw.offsets, cs_new + 1, units);
  const size_t rs_new = (size_t)row_stride(nw), rs_old = (size_t)row_stride(o);  // rows per unit
  copy_units<int32_t>(nw.perm, o.perm, (size_t)o.N_idx, rs_new, rs_old, 0, units, st);
  copy_units<uint4>(nw.k_perm, o.k_perm, (size_t)o.N_idx * rowc, rs_new * rowc, rs_old * rowc, 0, units, st);
  copy_units<uint4>(nw.v_perm, o.v_perm, (size_t)o.N_idx * rowc, rs_new * rowc, rs_old * rowc, 0, units, st);

  // (2) sink rows and the window
  {
    // with the old steady buffers as the new ones (no flush, room left) only the new tokens move
    const int first = nw.k_steady == o.k_steady ? ns + g.lc_old : 0;
    const size_t chunks = ((size_t)ns + g.lc_old + n_new - first) * units * rowc;
    if (chunks > 0) {
#define WAVE_ROUTE(ROWB)                                                                              \
  WAVE_LAUNCH("append_window", (route_window_kernel<ROWB>), grid_for(chunks), 256, 0, st,             \
              static_cast<const char*>(o.k_steady), static_cast<const char*>(o.v_steady),             \
              static_cast<const char*>(K_new), static_cast<const char*>(V_new), w + g.off_k,          \
              w + g.off_v, static_cast<char*>(nw.k_steady), static_cast<char*>(nw.v_steady), ns,      \
              g.lc_old, n_new, flush, steady_stride(o), steady_stride(nw), units, first)
      const size_t rowb = (size_t)D * es;
      if (rowb == 128) WAVE_ROUTE(128);
      else if (rowb == 256) WAVE_ROUTE(256);
      else if (rowb == 512) WAVE_ROUTE(512);
      else return WAVE_ERR_SHAPE;
#undef WAVE_ROUTE
    }
  }
  if (g.F == 0) return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;

  // (3) the flushed tokens are built as an index whose arrays are the new index's own, from
  // the old clusters' and rows' end onwards and at the new index's strides: segments numbered
  // after the old ones, offsets continued from the old row count, positions from the window's
  // first token (window row w is token old N - old local count + w)
  wave_index mi = g.mini;
  const size_t rowb = (size_t)D * es;
  mi.centroids = static_cast<char*>(nw.centroids) + (size_t)o.m * rowb;
  mi.vsum = static_cast<char*>(nw.vsum) + (size_t)o.m * rowb;
  mi.sizes = nw.sizes + o.m;
  mi.offsets = nw.offsets + o.m;
  mi.cluster_capacity = cluster_stride(nw);
  mi.perm = nw.perm + o.N_idx;
  mi.k_perm = static_cast<char*>(nw.k_perm) + (size_t)o.N_idx * rowb;
  mi.v_perm = static_cast<char*>(nw.v_perm) + (size_t)o.N_idx * rowb;
  mi.row_capacity = row_stride(nw);
  return launch_build(w + g.off_k, w + g.off_v, mi, iters, seed, w + g.off_build, st, o.S, o.N_idx,
                      o.N - g.lc_old);
}

}  // namespace wave
