// Shared device helpers and host-side launch plumbing of the wave-index library.
// gfx950 only: 64-lane wavefronts, DPP cross-lane operations, 16-byte vector loads.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/wave.h"

namespace wave {

// ----------------------------------------------------------------------------
// Storage types.  A row of d elements is read as 16-byte chunks, one per lane:
// EPC elements per chunk, LPR = d / EPC lanes per row, 64 / LPR rows per
// wavefront load instruction (a wave-wide load covers 1 KiB of contiguous rows).
// ----------------------------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int EPC = 4;
};
template <>
struct Elem<bf16_t> {
  static constexpr int EPC = 8;
};

__device__ __forceinline__ uint4 load16(const void* p) {
  return *reinterpret_cast<const uint4*>(p);
}
// For rows that are read once per step and never again: keeps them from
// displacing the reusable lines (scores, partial results) in the caches.
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16(void* p, uint4 v) { *reinterpret_cast<uint4*>(p) = v; }

template <typename T>
__device__ __forceinline__ void unpack(const uint4& v, float (&f)[Elem<T>::EPC]);

template <>
__device__ __forceinline__ void unpack<float>(const uint4& v, float (&f)[4]) {
  f[0] = __uint_as_float(v.x);
  f[1] = __uint_as_float(v.y);
  f[2] = __uint_as_float(v.z);
  f[3] = __uint_as_float(v.w);
}
template <>
__device__ __forceinline__ void unpack<bf16_t>(const uint4& v, float (&f)[8]) {
  f[0] = __uint_as_float(v.x << 16);
  f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16);
  f[3] = __uint_as_float(v.y & 0xffff0000u);
  f[4] = __uint_as_float(v.z << 16);
  f[5] = __uint_as_float(v.z & 0xffff0000u);
  f[6] = __uint_as_float(v.w << 16);
  f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// Round an fp64 value to bfloat16, nearest even, in ONE rounding: first to
// fp32 with round-to-odd (truncate, then set the last bit if anything was
// lost), which keeps enough information for the final nearest-even step.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
  float f = (float)x;  // nearest-even fp32
  const double back = (double)f;
  uint32_t u = __float_as_uint(f);
  if (back != x && (u & 0x7f800000u) != 0x7f800000u) {
    // make f the truncation of x towards zero, then force the sticky bit
    if ((back > x) == (x > 0.0)) u -= 1;  // rounded away from zero: step back
    u |= 1u;
  }
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  const uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return (uint16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ T quant_store(double x);
template <>
__device__ __forceinline__ float quant_store<float>(double x) {
  return (float)x;
}
template <>
__device__ __forceinline__ bf16_t quant_store<bf16_t>(double x) {
  bf16_t r;
  r.bits = f64_to_bf16_rne(x);
  return r;
}

__device__ __forceinline__ double to_f64(float x) { return (double)x; }
__device__ __forceinline__ double to_f64(bf16_t x) {
  return (double)__uint_as_float(((uint32_t)x.bits) << 16);
}
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

// ----------------------------------------------------------------------------
// Cross-lane reductions over the LPR lanes that share a row, with DPP.
// ----------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // reverse within 8 lanes
constexpr int DPP_MIRROR = 0x140;      // reverse within 16 lanes

template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "lanes per row");
  x += dpp<DPP_XOR1>(x);
  x += dpp<DPP_XOR2>(x);
  x += dpp<DPP_HALF_MIRROR>(x);
  if (LPR >= 16) x += dpp<DPP_MIRROR>(x);
  if (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

template <int LPR>
__device__ __forceinline__ double group_sum_f64(double x) {
  for (int off = 1; off < LPR; off <<= 1) x += __shfl_xor(x, off);
  return x;
}

__device__ __forceinline__ float wave_max(float x) {
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ __forceinline__ int wave_sum_i(int x) {
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ __forceinline__ float wave_sum_f(float x) {
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ __forceinline__ double wave_sum_d(double x) {
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// Workgroups are handed to the 8 XCDs round-robin by their id; each XCD has its
// own L2.  This maps the hardware id to a logical id such that consecutive
// logical ids (which share data: one sequence/head, one segment) sit on one XCD.
__device__ __forceinline__ int xcd_logical_block(int bid, int nblocks) {
  const int per = nblocks >> 3;
  if (bid >= (per << 3)) return bid;
  return (bid & 7) * per + (bid >> 3);
}

// ----------------------------------------------------------------------------
// Host side
// ----------------------------------------------------------------------------
inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
// rows per unit in perm / k_perm / v_perm
inline int row_stride(const wave_index& ix) { return ix.row_capacity > 0 ? ix.row_capacity : ix.N_idx; }
// clusters per unit in centroids / vsum / sizes (and + 1 entries in offsets)
inline int cluster_stride(const wave_index& ix) { return ix.cluster_capacity > 0 ? ix.cluster_capacity : ix.m; }
// rows per unit in k_steady / v_steady
inline int steady_stride(const wave_index& ix) { return ix.steady_capacity > 0 ? ix.steady_capacity : ix.p; }

// Profiler hooks (implemented in wave_api.hip).
void profile_before(const char* name, hipStream_t st);
void profile_after(hipStream_t st);
extern bool g_profile_on;

#define WAVE_LAUNCH(name, kernel, grid, block, shmem, stream, ...)                     \
  do {                                                                                 \
    if (::wave::g_profile_on) ::wave::profile_before(name, stream);                    \
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), shmem, stream, __VA_ARGS__);   \
    if (::wave::g_profile_on) ::wave::profile_after(stream);                           \
  } while (0)

// Launch geometry of one decode step; shared by wave_index_plan (workspace
// size) and wave_attention_decode (launches) so the two always agree.
struct DecodeGeom {
  int score_rows, score_chunks;    // clusters per workgroup / workgroups per unit (scoring)
  int gather_chunks;               // workgroups per query head over the retrieved tokens
  int steady_rows, steady_chunks;  // steady tokens per workgroup / workgroups per unit
  int est_rows, est_chunks;        // clusters per workgroup / workgroups per unit (estimation)
  int slots;                       // partial results per query head
  int mwords;                      // 32-bit words of the selection bitmap per query head
  int rcap;                        // entries of the selected-id list per query head
  int fused;                       // selection and retrieval fused into one workgroup per head
  int neg_in_gather, neg_slots;    // selected clusters' estimation terms: taken out by the retrieval kernel / a partial of their own
  int sliced, nslices, slice_len;  // selection cut into slices ranked by workgroups of their own
  int est_with_slices_pct;         // sliced path: share of the estimation work in the slices' launch
  int listed, list_filtered;       // selection launch + retrieval from one work list of token ranges;
                                   // with more clusters than fit in LDS: filtered by the tile maxima
  int chunk_tokens, wmain, wtotal, gather_wgs, stage;  // work list: tokens per range, entries, launch size
  size_t off_z, off_cn2, off_sel, off_pref, off_srow, off_bitmap, off_nsel, off_part,
      off_slice_ids, off_slice_z, off_tile_max, off_chunk_first, off_head_info, off_work,
      off_work_count, off_part_g, total;
};
DecodeGeom decode_geometry(const wave_index& ix, int Hq, int topk);

struct BuildGeom {
  size_t off_xhat, off_chat, off_assign, off_order, off_prev, off_count, off_flag, off_nflag, off_init, total;
  int units, segs;                 // B*Hkv, units * S
};
BuildGeom build_geometry(const wave_index& ix);

wave_status launch_decode(const void* q, const wave_index& ix, int Hq, int topk, float* out,
                          float* lse, int32_t* selected, void* ws, hipStream_t st);
// Decode with a budget for the estimation zone (the e best-ranked clusters after
// the r retrieved ones are estimated, the rest ignored): launch geometry and
// workspace layout.  delegate: the budget covers every cluster, the plain decode runs.
struct BudgetGeom {
  int delegate;
  int r, k2;                        // retrieved clusters, retrieved + estimated clusters
  int rcap1, rcap2, mwords;
  int sliced1, sliced2, nslices, slice_len;
  int score_chunks, steady_rows, steady_chunks, gather_chunks, est_chunks, slots;
  size_t off_z, off_cn2, off_ids1, off_ids2, off_nsel1, off_nsel2, off_pref, off_srow, off_bitmap,
      off_slice_ids, off_slice_z, off_part, total;
};
BudgetGeom budget_geometry(const wave_index& ix, int Hq, int topk, int est_clusters);
wave_status launch_decode_budget(const void* q, const wave_index& ix, int Hq, int topk, int est_clusters,
                                 float* out, float* lse, int32_t* selected, void* ws, hipStream_t st);

// Full attention over all N tokens: chunks of FULL_ATTN_ROWS tokens per workgroup.
constexpr int FULL_ATTN_ROWS = 1024;
inline int full_attention_chunks(int N) { return (N + FULL_ATTN_ROWS - 1) / FULL_ATTN_ROWS; }
wave_status launch_full_attention(const void* q, const void* K, const void* V, int dtype, int B, int Hq,
                                  int Hkv, int N, int d, float* out, float* lse, void* ws,
                                  hipStream_t st);
wave_status launch_build(const void* K, const void* V, const wave_index& ix, int iters,
                         uint64_t seed, void* ws, hipStream_t st, int seg_id_base = 0, int row_base = 0,
                         int pos_base = 0);
// Incremental update: geometry of its workspace and the launches (wave_append.hip).
struct AppendGeom {
  int F, ks, lc_old;              // flushed segments, clusters per update segment, old local count
  wave_index mini;                // the flushed tokens as an index of their own (pointers unset)
  size_t off_k, off_v, off_build, total;  // the flushed keys and values, the build's workspace
};
AppendGeom append_geometry(const wave_index& old_ix, int n_new, int n_local_min, int U, int k_u);
wave_status launch_append(const wave_index& old_ix, const void* K_new, const void* V_new, int n_new,
                          int iters, uint64_t seed, const wave_index& new_ix, const AppendGeom& g,
                          void* ws, hipStream_t st);
wave_status launch_assign_step(const void* xhat, const void* chat, int dtype, int L_s, int k_s, int d,
                               int32_t* assign, void* ws, hipStream_t st);

// splitmix64-keyed Fisher-Yates seed points, shared by the host hook and the device kernel.
__host__ __device__ inline uint64_t splitmix64_next(uint64_t& state) {
  state += 0x9E3779B97F4A7C15ull;
  uint64_t z = state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__host__ __device__ inline uint64_t init_stream_state(uint64_t seed, int b, int h, int s) {
  uint64_t st = 0;
  const uint64_t v[4] = {seed, (uint64_t)(int64_t)b, (uint64_t)(int64_t)h, (uint64_t)(int64_t)s};
  for (int i = 0; i < 4; ++i) {
    st ^= v[i];
    st = splitmix64_next(st);
  }
  return st;
}

}  // namespace wave
