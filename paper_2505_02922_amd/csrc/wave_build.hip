// Index construction of the wave index: segmented spherical k-means over the
// keys of every (sequence, KV head) unit and the meta index / cluster-contiguous
// KV layout that results (paper: "Index Organization", "Lightweight Index
// Construction and Updates"; value sums and sizes from the estimation section).
//
// Per segment of L tokens:
//   mean        fp64 mean of the segment's keys
//   normalise   xhat = quant((K - mean) / |K - mean|)             (fp64, one rounding)
//   init        k seeded distinct points of the segment become the first centroids
//   T times:    assign  (bf16 MFMA similarities, fp32 accumulate; running best and
//                        second best per point; near-ties flagged)
//               refine  (flagged points re-decided with fp64 similarities)
//               sort    (stable counting sort of the segment's points by cluster)
//               update  (centroid = quant(member sum / |member sum|), fp64)
//   finalize    sizes, offsets, mean of raw keys, value sums, permuted K/V rows
#include <stdlib.h>

#include "wave_common.h"

namespace wave {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr float kNegHuge = -3.0e38f;
// Two similarities closer than this are re-decided in fp64.  It covers the fp32
// accumulation error of a unit-vector dot product (<= (d + 1) * 2^-24 < 8e-6; in the
// MFMA path the sums run near 2, so 8 steps of 2^-23) on both values plus the 5 low
// mantissa bits the MFMA path overwrites with the row code (<= 2^-18 relative each).
constexpr float kAssignGuard = 4.0e-5f;

struct SegInfo {
  int unit, s, seg_start, L_s, k_s;
};
__device__ __forceinline__ SegInfo seg_info(int sg, int S, int L, int kk, int N_idx) {
  SegInfo r;
  r.unit = sg / S;
  r.s = sg - r.unit * S;
  r.seg_start = r.s * L;
  r.L_s = min(L, N_idx - r.seg_start);
  r.k_s = min(kk, r.L_s);
  return r;
}

// a / b for many a and one b: with r the correctly rounded 1 / b, one multiply
// and one fused residual correction give the correctly rounded quotient (the
// classic Newton step on the quotient), three instructions instead of a full
// division each.
__device__ __forceinline__ double div_shared(double a, double b, double r) {
  const double q = a * r;
  return fma(fma(-q, b, a), r, q);
}

// ============================================================================
// Segment mean (fp64).  One workgroup per segment; fixed summation order.
// ============================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void seg_mean_kernel(const T* __restrict__ K, double* __restrict__ mean,
                                                       int32_t* __restrict__ flag_count, int S, int L,
                                                       int kk, int N, int N_idx, int n_sink) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  const int sg = blockIdx.x;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  if (sg == 0 && threadIdx.x == 0) *flag_count = 0;
  const T* Ku = K + ((size_t)si.unit * N + n_sink + si.seg_start) * D + sub * EPC;
  double acc[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) acc[e] = 0.0;
  int i = grp;
  for (; i + 3 * GROUPS < si.L_s; i += 4 * GROUPS) {  // four rows in flight, added in row order
    uint4 raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) raw[u] = load16(Ku + (size_t)(i + u * GROUPS) * D);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float f[EPC];
      unpack<T>(raw[u], f);
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[e] += (double)f[e];
    }
  }
  for (; i < si.L_s; i += GROUPS) {
    float f[EPC];
    unpack<T>(load16(Ku + (size_t)i * D), f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] += (double)f[e];
  }
  __shared__ double red[GROUPS][D];
#pragma unroll
  for (int e = 0; e < EPC; ++e) red[grp][sub * EPC + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    double s = 0.0;
    for (int g = 0; g < GROUPS; ++g) s += red[g][threadIdx.x];
    mean[(size_t)sg * D + threadIdx.x] = s / (double)si.L_s;
  }
}

// ============================================================================
// Centre, normalise, round to the storage type.
// ============================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void normalise_kernel(const T* __restrict__ K,
                                                        const double* __restrict__ mean,
                                                        T* __restrict__ xhat, int S, int L, int N,
                                                        int N_idx, int n_sink, int rows_total) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  for (int row = blockIdx.x * GROUPS + grp; row < rows_total; row += gridDim.x * GROUPS) {
    const int unit = row / N_idx, pos = row - unit * N_idx;
    const int s = pos / L;
    const double* mu = mean + ((size_t)unit * S + s) * D + sub * EPC;
    float f[EPC];
    unpack<T>(load16(K + ((size_t)unit * N + n_sink + pos) * D + sub * EPC), f);
    double x[EPC], n2 = 0.0;
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      x[e] = (double)f[e] - mu[e];
      n2 = fma(x[e], x[e], n2);
    }
    n2 = group_sum_f64<LPR>(n2);
    const double nrm = sqrt(n2);
    const double dv = nrm > 0.0 ? nrm : 1.0;
    const double rdv = 1.0 / dv;
    T o[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) o[e] = quant_store<T>(div_shared(x[e], dv, rdv));
    store16(xhat + (size_t)row * D + sub * EPC, *reinterpret_cast<uint4*>(o));
  }
}

// ============================================================================
// Seeded initial centroids: the first k entries of a Fisher-Yates shuffle of the
// segment's positions, without running the shuffle.  The generator's state
// advances by a constant per draw, so draw i is a function of i alone, and so is
// its target j_i = i + draw_i mod (L_s - i).  Step i picks the value found at
// position j_i and leaves position i's value there.  The value at position p
// just before step b (p >= b) is p itself unless an earlier step targeted p; if
// t < b is the latest such step, it is the value position t held before step t.
// Every thread follows that chain for its own i (chains are short: k << L).
// ============================================================================

template <typename T, int D>
__global__ __launch_bounds__(256) void init_kernel(const T* __restrict__ xhat, T* __restrict__ chat,
                                                   int S, int L, int kk, int N_idx, int Hkv,
                                                   uint64_t seed, int seg_id_base) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  const int sg = blockIdx.x;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  extern __shared__ int init_lds[];  // 2 * kk ints
  int* target = init_lds;
  int* chosen = init_lds + kk;
  // (seg_id_base: the segments of an index update continue the numbering of the build)
  const uint64_t st0 = init_stream_state(seed, si.unit / Hkv, si.unit % Hkv, si.s + seg_id_base);
  for (int i = threadIdx.x; i < si.k_s; i += 256) {
    uint64_t st = st0 + (uint64_t)i * 0x9E3779B97F4A7C15ull;  // state before draw i
    const uint64_t draw = splitmix64_next(st);
    target[i] = i + (int)(draw % (uint64_t)(si.L_s - i));
  }
  __syncthreads();
  for (int i = threadIdx.x; i < si.k_s; i += 256) {
    int cur = target[i], bound = i;
    while (true) {
      int t = -1;
      for (int u = 0; u < bound; ++u) t = target[u] == cur ? u : t;  // latest earlier step onto cur
      if (t < 0) break;
      cur = t;
      bound = t;
    }
    chosen[i] = cur;
  }
  __syncthreads();
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const T* X = xhat + ((size_t)si.unit * N_idx + si.seg_start) * D + sub * EPC;
  T* Cs = chat + (size_t)sg * kk * D + sub * EPC;
  for (int c = grp; c < si.k_s; c += GROUPS) store16(Cs + (size_t)c * D, load16(X + (size_t)chosen[c] * D));
}

// ============================================================================
// Assign, MFMA path (bf16).  A workgroup of NW waves takes NW * 32 * NF points
// of one segment.  Each wave keeps its points as B operands (K x N = 16 x 32 per
// instruction) in registers for the whole kernel and streams the centroids,
// 32 at a time, through a padded LDS tile as A operands (M x K = 32 x 16), so
// D[centroid][point] accumulates in v_mfma_f32_32x32x16_bf16 and a lane holds
// 16 centroid rows of ONE point: the running best / second best never leave the
// lane.  Four of the five bits of the centroid's row inside the tile are written
// over low mantissa bits of the similarity (the fifth is the lane's half), so
// one v_med3 pair carries value and index: 3 VALU instructions per similarity.
// ============================================================================
// Similarities of unit vectors lie in [-1, 1]; the accumulators start at
// kAssignBias so every value is a positive float, whose bit pattern orders like
// a signed integer: max and median then run on the integer pipes, free of the
// NaN handling a float max drags in.
constexpr float kAssignBias = 2.0f;

__device__ __forceinline__ int med3_i32(int a, int b, int c) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

template <int NF, bool TAIL>
__device__ __forceinline__ void assign_epilogue(const floatx16 (&acc)[NF], int (&best)[NF],
                                                int (&second)[NF], int (&btile)[NF], int t, int half,
                                                int k_s) {
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    const int before = best[f];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      constexpr uint32_t kClear = ~27u;               // bits 0,1,3,4 carry the row code
      const uint32_t code = 8u * (v / 4) + (v % 4);   // row = code | 4 * half
      int key = (int)((__float_as_uint(acc[f][v]) & kClear) | code);
      if (TAIL && 32 * t + (int)code + 4 * half >= k_s) key = 0;
      second[f] = med3_i32(best[f], second[f], key);
      best[f] = max(best[f], key);
    }
    btile[f] = (best[f] != before) ? t : btile[f];
  }
}

template <int D, int NF, int NW>
__global__ __launch_bounds__(64 * NW) void assign_mfma_kernel(
    const bf16_t* __restrict__ xhat, const bf16_t* __restrict__ chat, int32_t* __restrict__ assign,
    int32_t* __restrict__ flag_list, int32_t* __restrict__ flag_count, int S, int L, int kk, int N_idx,
    int wgs_per_seg) {
  constexpr int KS = D / 16;            // MFMA k-steps per tile
  constexpr int PW = 32 * NF;           // points per wave
  constexpr int PWG = NW * PW;          // points per workgroup
  constexpr int NT = 64 * NW;           // threads
  constexpr int ROWB = D * 2 + 16;      // LDS row pitch: 16 B pad keeps 16 lanes on 64 distinct banks
  constexpr int CPR = D / 8;            // 16-byte chunks per centroid row
  constexpr int CHUNKS = 32 * CPR;      // chunks per tile
  constexpr int CPT = (CHUNKS + NT - 1) / NT;  // chunks each thread moves per tile
  __shared__ __attribute__((aligned(16))) char lds[2][32 * ROWB];

  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int sg = wg / wgs_per_seg, piece = wg - sg * wgs_per_seg;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  const int p0 = piece * PWG;
  if (p0 >= si.L_s) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const bf16_t* X = xhat + ((size_t)si.unit * N_idx + si.seg_start) * D;
  const bf16_t* Cs = chat + (size_t)sg * kk * D;

  uint4 bfrag[NF][KS];
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    const int row = min(p0 + wave * PW + 32 * f + col, si.L_s - 1);
#pragma unroll
    for (int s = 0; s < KS; ++s) bfrag[f][s] = load16(X + (size_t)row * D + (2 * s + half) * 8);
  }
  int best[NF], second[NF], btile[NF];  // biased similarities as integers; 0 is below all of them
#pragma unroll
  for (int f = 0; f < NF; ++f) best[f] = second[f] = btile[f] = 0;

  const int ntiles = (si.k_s + 31) / 32;
  // Centroid tiles travel global -> registers -> LDS.  Two register stages keep
  // the loads two tiles ahead of the MFMAs that consume them.
  uint4 stage[2][CPT];
  auto gload = [&](int t, uint4 (&st)[CPT]) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int id = tid + NT * i, row = id / CPR, ch = id - row * CPR;
      if (CHUNKS % NT == 0 || id < CHUNKS) {
        const int crow = min(32 * t + row, si.k_s - 1);
        st[i] = load16(Cs + (size_t)crow * D + ch * 8);
      }
    }
  };
  auto sstore = [&](int buf, const uint4 (&st)[CPT]) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int id = tid + NT * i, row = id / CPR, ch = id - row * CPR;
      if (CHUNKS % NT == 0 || id < CHUNKS) store16(&lds[buf][row * ROWB + ch * 16], st[i]);
    }
  };
  auto tile_step = [&](int t, uint4 (&st_next)[CPT], uint4 (&st_load)[CPT]) {
    // st_next holds tile t + 1 (requested one step ago); st_load receives tile t + 2
    if (t + 2 < ntiles) gload(t + 2, st_load);
    floatx16 acc[NF];
    const char* tile = lds[t & 1];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, load16(tile + col * ROWB + (2 * s + half) * 16));
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const bf16x8 bv = __builtin_bit_cast(bf16x8, bfrag[f][s]);
        if (s == 0) {
          constexpr float B0 = kAssignBias;
          const floatx16 bias = {B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0};
          acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bv, bias, 0, 0, 0);
        } else {
          acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bv, acc[f], 0, 0, 0);
        }
      }
    }
    if (32 * t + 32 > si.k_s)
      assign_epilogue<NF, true>(acc, best, second, btile, t, half, si.k_s);
    else
      assign_epilogue<NF, false>(acc, best, second, btile, t, half, si.k_s);
    if (t + 1 < ntiles) sstore((t + 1) & 1, st_next);
    __syncthreads();
  };
  gload(0, stage[0]);
  if (ntiles > 1) gload(1, stage[1]);
  sstore(0, stage[0]);
  __syncthreads();
  for (int t = 0; t < ntiles; t += 2) {
    tile_step(t, stage[1], stage[0]);
    if (t + 1 < ntiles) tile_step(t + 1, stage[0], stage[1]);
  }

  // lanes l and l ^ 32 hold the same points over disjoint centroid rows
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    int brow = (best[f] & 27) | (4 * half);
    const int ob = __shfl_xor(best[f], 32), os = __shfl_xor(second[f], 32);
    const int ot = __shfl_xor(btile[f], 32), orow = __shfl_xor(brow, 32);
    const int nsec = max(min(best[f], ob), max(second[f], os));
    if (ob > best[f]) {
      best[f] = ob;
      btile[f] = ot;
      brow = orow;
    }
    const int point = p0 + wave * PW + 32 * f + col;
    if (half == 0 && point < si.L_s) {
      const size_t gp = (size_t)si.unit * N_idx + si.seg_start + point;
      assign[gp] = btile[f] * 32 + brow;
      const float gap = __int_as_float(best[f]) - (nsec > 0 ? __int_as_float(nsec) : 0.f);
      if (gap < kAssignGuard) flag_list[atomicAdd(flag_count, 1)] = (int32_t)gp;
    }
  }
}

// ============================================================================
// Assign, MFMA path with the segment's centroids resident in LDS: one workgroup
// of 16 waves copies all k_s centroid rows into LDS once (padded rows, at most
// ~136 KiB) and then every wave works through fragments of 32 * NF points on
// its own: no barrier and no global centroid traffic inside the loop.
// ============================================================================
template <int D>
struct ResidentTile {
  static constexpr int KS = D / 16;        // MFMA k-steps per tile
  static constexpr int ROWB = D * 2 + 16;  // LDS row pitch: 16 B pad keeps 16 lanes on 64 distinct banks
  static constexpr int CPR = D / 8;        // 16-byte chunks per centroid row
};

// The segment's k_s centroid rows into the padded LDS tiles (rows beyond k_s repeat the
// last one; the epilogue ignores them).  All NT threads call this; the caller's barrier follows.
template <int D, int NT>
__device__ __forceinline__ void resident_load_centroids(const bf16_t* Cs, int k_s, char* cent) {
  using RT = ResidentTile<D>;
  const int ntiles = (k_s + 31) / 32;
  for (int id = threadIdx.x; id < 32 * ntiles * RT::CPR; id += NT) {
    const int row = id / RT::CPR, ch = id - row * RT::CPR;
    store16(cent + row * RT::ROWB + ch * 16, load16(Cs + (size_t)min(row, k_s - 1) * D + ch * 8));
  }
}

// Wave `wave` of NW takes the fragments f_lo + wave * NF, + NW * NF, ... below f_hi of the
// segment's points X against the centroids in `cent`; emit(point, cluster, near_tie) is
// called once per point by the lane that holds it.
template <int D, int NF, int NW, typename Emit>
__device__ __forceinline__ void resident_assign_fragments(const bf16_t* X, const char* cent, int L_s, int k_s,
                                                          int f_lo, int f_hi, Emit&& emit) {
  using RT = ResidentTile<D>;
  constexpr int KS = RT::KS, ROWB = RT::ROWB;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int ntiles = (k_s + 31) / 32;
  const int nfull = k_s / 32;  // tiles without rows beyond k_s
  constexpr float B0 = kAssignBias;
  floatx16 bias = {B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0};
  asm volatile("" : "+v"(bias));  // kept in registers: one accumulator-start operand for every tile
  for (int fb = f_lo + wave * NF; fb < f_hi; fb += NW * NF) {
    uint4 bfrag[NF][KS];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const int row = min(32 * (fb + f) + col, L_s - 1);
#pragma unroll
      for (int s = 0; s < KS; ++s) bfrag[f][s] = load16(X + (size_t)row * D + (2 * s + half) * 8);
    }
    int best[NF], second[NF], btile[NF];  // biased similarities as integers; 0 is below all of them
#pragma unroll
    for (int f = 0; f < NF; ++f) best[f] = second[f] = btile[f] = 0;
    auto mfma_tile = [&](int t, floatx16 (&acc)[NF]) {
      const char* tile = cent + (size_t)(32 * t + col) * ROWB + half * 16;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, load16(tile + s * 32));
#pragma unroll
        for (int f = 0; f < NF; ++f) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, bfrag[f][s]);
          acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bv, s == 0 ? bias : acc[f], 0, 0, 0);
        }
      }
    };
    // One tile's MFMAs are issued between the integer epilogue instructions of
    // the tile before it (two accumulator sets): the matrix pipe works while the
    // vector ALU ranks the previous results.
    auto interleave = [&]() {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // the first two LDS reads
#pragma unroll
      for (int i = 0; i < KS * NF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // the LDS read two MFMAs ahead
        __builtin_amdgcn_sched_group_barrier(0x002, 48 / KS, 0);  // a share of the epilogue
      }
    };
    floatx16 accA[NF], accB[NF];
    if (nfull > 0) {
      mfma_tile(0, accA);
      int t = 1;
      for (; t + 1 < nfull; t += 2) {
        mfma_tile(t, accB);
        assign_epilogue<NF, false>(accA, best, second, btile, t - 1, half, k_s);
        interleave();
        mfma_tile(t + 1, accA);
        assign_epilogue<NF, false>(accB, best, second, btile, t, half, k_s);
        interleave();
      }
      if (t < nfull) {
        mfma_tile(t, accB);
        assign_epilogue<NF, false>(accA, best, second, btile, t - 1, half, k_s);
        interleave();
        assign_epilogue<NF, false>(accB, best, second, btile, t, half, k_s);
      } else {
        assign_epilogue<NF, false>(accA, best, second, btile, t - 1, half, k_s);
      }
    }
    if (nfull < ntiles) {  // the last tile has rows beyond k_s
      mfma_tile(nfull, accA);
      assign_epilogue<NF, true>(accA, best, second, btile, nfull, half, k_s);
    }
    // lanes l and l ^ 32 hold the same points over disjoint centroid rows
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      int brow = (best[f] & 27) | (4 * half);
      const int ob = __shfl_xor(best[f], 32), os = __shfl_xor(second[f], 32);
      const int ot = __shfl_xor(btile[f], 32), orow = __shfl_xor(brow, 32);
      const int nsec = max(min(best[f], ob), max(second[f], os));
      if (ob > best[f]) {
        best[f] = ob;
        btile[f] = ot;
        brow = orow;
      }
      const int point = 32 * (fb + f) + col;
      if (half == 0 && fb + f < f_hi && point < L_s) {
        const float gap = __int_as_float(best[f]) - (nsec > 0 ? __int_as_float(nsec) : 0.f);
        emit(point, btile[f] * 32 + brow, gap < kAssignGuard);
      }
    }
  }
}

// The same step for few centroid tiles (short segments): one accumulator set and no
// instruction interleaving, the next fragment's rows requested before the current one is
// worked on.  Same similarities, same epilogue, same emit.
template <int D, int NW, typename Emit>
__device__ __forceinline__ void lean_assign_fragments(const bf16_t* X, const char* cent, int L_s, int k_s,
                                                      int f_hi, Emit&& emit) {
  using RT = ResidentTile<D>;
  constexpr int KS = RT::KS, ROWB = RT::ROWB;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int ntiles = (k_s + 31) / 32, nfull = k_s / 32;
  constexpr float B0 = kAssignBias;
  const floatx16 bias = {B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0, B0};
  auto load_frag = [&](int fb, uint4 (&dst)[KS]) {
    const int row = min(32 * fb + col, L_s - 1);
#pragma unroll
    for (int s = 0; s < KS; ++s) dst[s] = load16(X + (size_t)row * D + (2 * s + half) * 8);
  };
  uint4 cur[KS], nxt[KS];
  if (wave < f_hi) load_frag(wave, cur);
  for (int fb = wave; fb < f_hi; fb += NW) {
    if (fb + NW < f_hi) load_frag(fb + NW, nxt);
    int best[1] = {0}, second[1] = {0}, btile[1] = {0};
    for (int t = 0; t < ntiles; ++t) {
      const char* tile = cent + (size_t)(32 * t + col) * ROWB + half * 16;
      floatx16 acc[1];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, load16(tile + s * 32));
        const bf16x8 bv = __builtin_bit_cast(bf16x8, cur[s]);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bv, s == 0 ? bias : acc[0], 0, 0, 0);
      }
      if (t < nfull) assign_epilogue<1, false>(acc, best, second, btile, t, half, k_s);
      else assign_epilogue<1, true>(acc, best, second, btile, t, half, k_s);
    }
    // lanes l and l ^ 32 hold the same points over disjoint centroid rows
    int brow = (best[0] & 27) | (4 * half);
    const int ob = __shfl_xor(best[0], 32), os = __shfl_xor(second[0], 32);
    const int ot = __shfl_xor(btile[0], 32), orow = __shfl_xor(brow, 32);
    const int nsec = max(min(best[0], ob), max(second[0], os));
    if (ob > best[0]) {
      best[0] = ob;
      btile[0] = ot;
      brow = orow;
    }
    const int point = 32 * fb + col;
    if (half == 0 && point < L_s) {
      const float gap = __int_as_float(best[0]) - (nsec > 0 ? __int_as_float(nsec) : 0.f);
      emit(point, btile[0] * 32 + brow, gap < kAssignGuard);
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) cur[s] = nxt[s];
  }
}

template <int D, int NF, int NW>
__global__ __launch_bounds__(64 * NW) void assign_resident_kernel(
    const bf16_t* __restrict__ xhat, const bf16_t* __restrict__ chat, int32_t* __restrict__ assign,
    int32_t* __restrict__ flag_list, int32_t* __restrict__ flag_count, int S, int L, int kk, int N_idx,
    int pieces_per_seg) {
  extern __shared__ __attribute__((aligned(16))) char cent[];  // 32 * ceil(k_s / 32) rows

  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int sg = wg / pieces_per_seg, piece = wg - sg * pieces_per_seg;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  const int nfrag = (si.L_s + 31) / 32;
  const int per = ((nfrag + pieces_per_seg - 1) / pieces_per_seg + NF - 1) / NF * NF;
  const int f_lo = piece * per, f_hi = min(nfrag, f_lo + per);
  if (f_lo >= f_hi) return;
  const bf16_t* X = xhat + ((size_t)si.unit * N_idx + si.seg_start) * D;
  resident_load_centroids<D, 64 * NW>(chat + (size_t)sg * kk * D, si.k_s, cent);
  __syncthreads();
  const size_t gp0 = (size_t)si.unit * N_idx + si.seg_start;
  resident_assign_fragments<D, NF, NW>(X, cent, si.L_s, si.k_s, f_lo, f_hi,
                                       [&](int point, int cluster, bool near_tie) {
                                         assign[gp0 + point] = cluster;
                                         if (near_tie) flag_list[atomicAdd(flag_count, 1)] = (int32_t)(gp0 + point);
                                       });
}

// ============================================================================
// Assign, plain path (any storage type): one point per thread, fp32 FMA chain,
// centroids broadcast from LDS.
// ============================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void assign_plain_kernel(
    const T* __restrict__ xhat, const T* __restrict__ chat, int32_t* __restrict__ assign,
    int32_t* __restrict__ flag_list, int32_t* __restrict__ flag_count, int S, int L, int kk, int N_idx,
    int wgs_per_seg) {
  constexpr int CT = 16;  // centroids per LDS tile
  __shared__ __attribute__((aligned(16))) float cs[CT][D];
  const int sg = blockIdx.x / wgs_per_seg, piece = blockIdx.x - sg * wgs_per_seg;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  const int p0 = piece * 256;
  if (p0 >= si.L_s) return;
  const int point = p0 + threadIdx.x;
  const T* xr = xhat + ((size_t)si.unit * N_idx + si.seg_start + min(point, si.L_s - 1)) * D;
  const T* Cs = chat + (size_t)sg * kk * D;
  float x[D];
#pragma unroll
  for (int e = 0; e < D; ++e) x[e] = to_f32(xr[e]);
  float best = kNegHuge, second = kNegHuge;
  int bidx = 0;
  for (int c0 = 0; c0 < si.k_s; c0 += CT) {
    __syncthreads();
    for (int i = threadIdx.x; i < CT * D; i += 256) {
      const int r = i / D, e = i - r * D;
      cs[r][e] = to_f32(Cs[(size_t)min(c0 + r, si.k_s - 1) * D + e]);
    }
    __syncthreads();
    const int nc = min(CT, si.k_s - c0);
    for (int r = 0; r < nc; ++r) {
      float a = 0.f;
#pragma unroll
      for (int e = 0; e < D; ++e) a = fmaf(x[e], cs[r][e], a);
      if (a > best) {
        second = best;
        best = a;
        bidx = c0 + r;
      } else {
        second = fmaxf(second, a);
      }
    }
  }
  if (point < si.L_s) {
    const size_t gp = (size_t)si.unit * N_idx + si.seg_start + point;
    assign[gp] = bidx;
    if (best - second < kAssignGuard) flag_list[atomicAdd(flag_count, 1)] = (int32_t)gp;
  }
}

// ============================================================================
// Refine: every flagged point gets its argmax from fp64 similarities (exact for
// the stored operands up to fp64 rounding), ties to the lowest centroid.
// ============================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void refine_kernel(const T* __restrict__ xhat, const T* __restrict__ chat,
                                                     int32_t* __restrict__ assign,
                                                     const int32_t* __restrict__ flag_list,
                                                     const int32_t* __restrict__ flag_count, int S,
                                                     int L, int kk, int N_idx) {
  __shared__ double xs[D];
  __shared__ double bval[4];
  __shared__ int bidx[4];
  const int n = *flag_count;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int it = blockIdx.x; it < n; it += gridDim.x) {
    const int gp = flag_list[it];
    const int unit = gp / N_idx, pos = gp - unit * N_idx;
    const int s = pos / L;
    const int L_s = min(L, N_idx - s * L), k_s = min(kk, L_s);
    const T* Cs = chat + ((size_t)unit * S + s) * kk * D;
    __syncthreads();
    if (threadIdx.x < D) xs[threadIdx.x] = to_f64(xhat[(size_t)gp * D + threadIdx.x]);
    __syncthreads();
    double bv = -1.0e300;
    int bi = 0x7fffffff;
    for (int c = threadIdx.x; c < k_s; c += 256) {
      const T* row = Cs + (size_t)c * D;
      double a = 0.0;
      constexpr int EPC = Elem<T>::EPC;
      for (int e0 = 0; e0 < D; e0 += 4 * EPC) {  // four 16-byte chunks in flight, summed in index order
        uint4 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) raw[u] = load16(row + e0 + u * EPC);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          float f[EPC];
          unpack<T>(raw[u], f);
#pragma unroll
          for (int e = 0; e < EPC; ++e) a = fma(xs[e0 + u * EPC + e], (double)f[e], a);
        }
      }
      if (a > bv) {  // c ascends within a thread, so strict > keeps the lowest index
        bv = a;
        bi = c;
      }
    }
    for (int off = 32; off >= 1; off >>= 1) {
      const double ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ov > bv || (ov == bv && oi < bi)) {
        bv = ov;
        bi = oi;
      }
    }
    if (lane == 0) {
      bval[wave] = bv;
      bidx[wave] = bi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < 4; ++w)
        if (bval[w] > bv || (bval[w] == bv && bidx[w] < bi)) {
          bv = bval[w];
          bi = bidx[w];
        }
      assign[gp] = bi;
    }
  }
}

// ============================================================================
// Stable counting sort of one segment's points by cluster.  Wave w owns the
// w-th contiguous stripe of the segment and a private row of counters, so the
// scatter keeps positions ascending inside every cluster.
// ============================================================================
constexpr int SORT_HIST_INTS = 11264;  // LDS budget for the per-wave counters

// One segment's points a[0, L_s) sorted into ord[] by the calling workgroup of W waves;
// per-cluster counts and first positions to cnt[] / first[] (kk entries each).
// prev (may be null): the clusters of the round before, replaced by this round's on the way; when
// a point's cluster differs from it (and `compare` is set: not in the first round), both clusters
// are marked in changed[] (plain stores of 1: who wins does not matter).  The update step
// recomputes only marked clusters: a cluster nobody entered or left keeps its member sum and with
// it, bit for bit, its centroid.
__device__ __forceinline__ void sort_segment(const int32_t* a, int32_t* ord, int32_t* cnt, int32_t* first,
                                             int L_s, int kk, int key_bits, int* hist, int32_t* prev = nullptr,
                                             int32_t* changed = nullptr, bool compare = false) {
  const int W = blockDim.x >> 6;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int* tot = hist + W * kk;
  for (int i = tid; i < W * kk; i += blockDim.x) hist[i] = 0;
  __syncthreads();
  const int stripe = (L_s + W - 1) / W;
  const int s0 = min(L_s, wave * stripe), s1 = min(L_s, s0 + stripe);
  for (int i = s0 + lane; i < s1; i += 64) {
    const int c = a[i];
    atomicAdd(&hist[wave * kk + c], 1);
    if (prev) {
      const int before = prev[i];
      if (compare && before != c) {
        changed[before] = 1;
        changed[c] = 1;
      }
      prev[i] = c;
    }
  }
  __syncthreads();
  // per cluster: exclusive scan over the waves, total into tot[]
  for (int c = tid; c < kk; c += blockDim.x) {
    int run = 0;
    for (int w = 0; w < W; ++w) {
      const int t = hist[w * kk + c];
      hist[w * kk + c] = run;
      run += t;
    }
    tot[c] = run;
  }
  __syncthreads();
  // exclusive scan of the totals over clusters (one wave, chunks of 64)
  if (wave == 0) {
    int carry = 0;
    for (int c0 = 0; c0 < kk; c0 += 64) {
      const int c = c0 + lane;
      const int v = c < kk ? tot[c] : 0;
      int inc = v;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
      }
      if (c < kk) {
        cnt[c] = v;
        first[c] = carry + inc - v;
        tot[c] = carry + inc - v;
      }
      carry += __shfl(inc, 63);
    }
  }
  __syncthreads();
  for (int i = tid; i < W * kk; i += blockDim.x) hist[i] += tot[i % kk];
  __syncthreads();
  // scatter, 64 points of the stripe at a time
  for (int i0 = s0; i0 < s1; i0 += 64) {
    const int i = i0 + lane;
    const bool on = i < s1;
    const int key = on ? a[i] : -1;
    // lanes holding the same key
    uint64_t peers = __ballot(on);
    for (int bit = 0; bit < key_bits; ++bit) {
      const uint64_t bal = __ballot((key >> bit) & 1);
      peers &= ((key >> bit) & 1) ? bal : ~bal;
    }
    const uint64_t below = peers & ((1ull << lane) - 1ull);
    const int rank = __popcll(below), cnt_l = __popcll(peers);
    if (on) {
      const int base = hist[wave * kk + key];
      ord[base + rank] = i;
      __builtin_amdgcn_wave_barrier();
      if (rank == cnt_l - 1) hist[wave * kk + key] = base + cnt_l;
    }
    __threadfence_block();
    __builtin_amdgcn_wave_barrier();
  }
}

__global__ __launch_bounds__(1024) void sort_kernel(const int32_t* __restrict__ assign,
                                                    int32_t* __restrict__ order,
                                                    int32_t* __restrict__ count,
                                                    int32_t* __restrict__ start,
                                                    int32_t* __restrict__ flag_count,
                                                    int32_t* __restrict__ prev,
                                                    int32_t* __restrict__ changed, int first_round, int S,
                                                    int L, int kk, int N_idx, int key_bits) {
  extern __shared__ int hist[];  // [W][kk], then kk ints of scan space
  const int sg = blockIdx.x;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  if (sg == 0 && threadIdx.x == 0) {
    flag_count[0] = 0;  // the refine pass before this one has consumed it
    flag_count[1] = 0;  // the list of large clusters the update step of this round fills
  }
  sort_segment(assign + (size_t)si.unit * N_idx + si.seg_start, order + (size_t)si.unit * N_idx + si.seg_start,
               count + (size_t)sg * kk, start + (size_t)sg * kk, si.L_s, kk, key_bits, hist,
               prev + (size_t)si.unit * N_idx + si.seg_start, changed + (size_t)sg * kk, !first_round);
}

// ============================================================================
// Update: one group of LPR lanes per cluster sums its members' xhat in fp64.
// ============================================================================
// Exponent fields of the nonzero elements of a 16-byte chunk: their smallest and largest
// (a subnormal counts as exponent field 1, which has the same unit in the last place).
template <typename T>
__device__ __forceinline__ void exponent_range(const uint4& raw, int& emin, int& emax);
template <>
__device__ __forceinline__ void exponent_range<bf16_t>(const uint4& raw, int& emin, int& emax) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t v = h ? w[i] >> 16 : w[i] & 0xffffu;
      if (v & 0x7fffu) {
        const int e = max(1, (int)((v >> 7) & 0xffu));
        emin = min(emin, e);
        emax = max(emax, e);
      }
    }
  }
}
template <>
__device__ __forceinline__ void exponent_range<float>(const uint4& raw, int& emin, int& emax) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (w[i] & 0x7fffffffu) {
      const int e = max(1, (int)((w[i] >> 23) & 0xffu));
      emin = min(emin, e);
      emax = max(emax, e);
    }
}
template <typename T>
struct MantissaBits;
template <>
struct MantissaBits<bf16_t> {
  static constexpr int value = 7;
};
template <>
struct MantissaBits<float> {
  static constexpr int value = 23;
};

// The member rows ord[0, n) of the segment's points X (already offset to the lane's chunk)
// added to acc in fp64 in that order, U loads in flight.  STATS: also the exponent range of
// what was added.  (STREAM: the rows are read once per launch and should not displace other
// lines in the caches.)
template <typename T, int D, int U, bool STREAM, bool STATS>
__device__ __forceinline__ void sum_members(const T* X, const int32_t* ord, int n,
                                            double (&acc)[Elem<T>::EPC], int& emin, int& emax) {
  auto load_row = [](const T* p) { return STREAM ? load16_stream(p) : load16(p); };
  constexpr int EPC = Elem<T>::EPC;
  auto add = [&](const uint4& raw) {
    float f[EPC];
    unpack<T>(raw, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] += (double)f[e];
    if (STATS) exponent_range<T>(raw, emin, emax);
  };
  int i = 0;
  for (; i + U <= n; i += U) {
    uint4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) raw[u] = load_row(X + (size_t)ord[i + u] * D);
#pragma unroll
    for (int u = 0; u < U; ++u) add(raw[u]);
  }
  if (U > 4 && i + 4 <= n) {
    uint4 raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) raw[u] = load_row(X + (size_t)ord[i + u] * D);
#pragma unroll
    for (int u = 0; u < 4; ++u) add(raw[u]);
    i += 4;
  }
  for (; i < n; ++i) add(load16(X + (size_t)ord[i] * D));
}

// The member sum of a cluster, normalised and rounded, to dst (the lane's 16-byte chunk of the
// centroid row); members that cancel keep the centroid.
template <typename T, int D>
__device__ __forceinline__ void finish_centroid(const double (&acc)[Elem<T>::EPC], T* dst) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC;
  double n2 = 0.0;
#pragma unroll
  for (int e = 0; e < EPC; ++e) n2 = fma(acc[e], acc[e], n2);
  n2 = group_sum_f64<LPR>(n2);
  const double nrm = sqrt(n2);
  if (!(nrm > 0.0)) return;
  T o[EPC];
  const double rn = 1.0 / nrm;
#pragma unroll
  for (int e = 0; e < EPC; ++e) o[e] = quant_store<T>(div_shared(acc[e], nrm, rn));
  store16(dst, *reinterpret_cast<uint4*>(o));
}

// One cluster's update by the calling group of LPR lanes (lane `sub` of it): the n member
// rows ord[0, n) of the segment's points X are summed in fp64 in that order, U loads in
// flight, and the normalised sum goes to dst.
template <typename T, int D, int U, bool STREAM>
__device__ __forceinline__ void update_cluster(const T* X, const int32_t* ord, int n, T* dst, int sub) {
  constexpr int EPC = Elem<T>::EPC;
  if (n == 0) return;  // an empty cluster keeps its centroid
  double acc[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) acc[e] = 0.0;
  int emin = 0, emax = 0;
  sum_members<T, D, U, STREAM, false>(X + sub * EPC, ord, n, acc, emin, emax);
  finish_centroid<T, D>(acc, dst);
}

// Clusters of more than UPD_BIG members (heavy-tailed data: a thousand tokens in one cluster)
// are summed by all groups of the workgroup, a contiguous run of members each, and the
// partial sums are added in run order.  The reference sum adds the members one by one, and
// the two agree bit for bit when no addition rounds, in either order.  That is certain when
// every partial sum of any subset of the addends is representable: all addends are multiples of
// 2^q, q the unit in the last place of the smallest exponent present, and n of them below
// 2^(emax + 1) in magnitude sum to less than n 2^(emax + 1); fp64 holds every multiple of 2^q
// below 2^(q + 53), so  emax - emin + ceil(log2 n) <= 52 - (mantissa bits of the storage type)
// suffices.  The exponent range is gathered on the way; a cluster that fails the test (a
// component spread over more than 2^34 at bf16) is summed again one by one by one group.
constexpr int UPD_BIG = 128;

template <typename T, int D>
__global__ __launch_bounds__(256) void update_big_kernel(const T* __restrict__ xhat, T* __restrict__ chat,
                                                         const int32_t* __restrict__ order,
                                                         const int32_t* __restrict__ count,
                                                         const int32_t* __restrict__ start,
                                                         const int32_t* __restrict__ big_list,
                                                         const int32_t* __restrict__ big_count, int S, int L,
                                                         int kk, int N_idx) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  __shared__ double part[GROUPS * D];
  __shared__ int erange[2 * GROUPS];
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const int nbig = *big_count;
#pragma unroll 1
  for (int b = blockIdx.x; b < nbig; b += gridDim.x) {  // (the same for every thread of the workgroup)
    const int gc = big_list[b];
    const int sg = gc / kk;
    const SegInfo si = seg_info(sg, S, L, kk, N_idx);
    const size_t p0 = (size_t)si.unit * N_idx + si.seg_start;
    const int n = count[gc];
    const int32_t* ord = order + p0 + start[gc];
    const T* X = xhat + p0 * D + sub * EPC;
    const int per = (n + GROUPS - 1) / GROUPS;
    const int i0 = min(n, grp * per), i1 = min(n, i0 + per);
    double acc[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] = 0.0;
    int emin = 255, emax = 0;
    sum_members<T, D, 4, true, true>(X, ord + i0, i1 - i0, acc, emin, emax);
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) {
      emin = min(emin, __shfl_xor(emin, off));
      emax = max(emax, __shfl_xor(emax, off));
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) part[grp * D + sub * EPC + e] = acc[e];
    if (sub == 0) {
      erange[2 * grp] = emin;
      erange[2 * grp + 1] = emax;
    }
    __syncthreads();
    if (grp == 0) {
      double tot[EPC];
#pragma unroll
      for (int e = 0; e < EPC; ++e) tot[e] = part[sub * EPC + e];
      int lo = erange[0], hi = erange[1];
#pragma unroll 1
      for (int g = 1; g < GROUPS; ++g) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) tot[e] += part[g * D + sub * EPC + e];
        lo = min(lo, erange[2 * g]);
        hi = max(hi, erange[2 * g + 1]);
      }
      const int lg = 32 - __clz(n - 1);  // ceil(log2 n), n > UPD_BIG
      T* dst = chat + (size_t)gc * D + sub * EPC;
      if (hi < lo || hi - lo + lg <= 52 - MantissaBits<T>::value)  // (hi < lo: every addend is zero)
        finish_centroid<T, D>(tot, dst);
      else
        update_cluster<T, D, 4, true>(xhat + p0 * D, ord, n, dst, sub);
    }
    __syncthreads();
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void update_kernel(const T* __restrict__ xhat, T* __restrict__ chat,
                                                     const int32_t* __restrict__ order,
                                                     const int32_t* __restrict__ count,
                                                     const int32_t* __restrict__ start,
                                                     int32_t* __restrict__ changed, int all,
                                                     int32_t* __restrict__ big_list,
                                                     int32_t* __restrict__ big_count, int S, int L, int kk,
                                                     int N_idx, int nclusters) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const int gc = blockIdx.x * GROUPS + grp;  // sg * kk + c
  if (gc >= nclusters) return;
  const int sg = gc / kk, c = gc - sg * kk;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  if (c >= si.k_s) return;
  // Only clusters that a point entered or left in this round (marked by the sort step) are
  // summed again; `all`: the first round, every cluster.  The mark is consumed here.
  const int touched = changed[gc];
  if (sub == 0) changed[gc] = 0;
  if (!all && !touched) return;
  const int n = count[gc];
  if (n > UPD_BIG) {  // left to update_big_kernel
    if (sub == 0) big_list[atomicAdd(big_count, 1)] = gc;
    return;
  }
  const size_t p0 = (size_t)si.unit * N_idx + si.seg_start;
  update_cluster<T, D, 4, true>(xhat + p0 * D, order + p0 + start[gc], n, chat + (size_t)gc * D + sub * EPC, sub);
}

// The update of the later rounds, when most clusters are untouched: a workgroup reads the marks
// of 256 consecutive clusters at once, lists the marked ones in LDS and its 16-lane groups take
// them from the list (one mark per group and workgroup, as in update_kernel, is a round trip and
// a workgroup launch per 16 clusters even when none of them changed).
template <typename T, int D>
__global__ __launch_bounds__(256) void update_touched_kernel(const T* __restrict__ xhat, T* __restrict__ chat,
                                                             const int32_t* __restrict__ order,
                                                             const int32_t* __restrict__ count,
                                                             const int32_t* __restrict__ start,
                                                             int32_t* __restrict__ changed,
                                                             int32_t* __restrict__ big_list,
                                                             int32_t* __restrict__ big_count, int S, int L,
                                                             int kk, int N_idx, int nclusters) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  __shared__ int list[256];
  __shared__ int wave_n[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int gc_mine = blockIdx.x * 256 + tid;
  const bool on = gc_mine < nclusters && changed[gc_mine] != 0;
  if (on) changed[gc_mine] = 0;
  const uint64_t mk = __ballot(on);
  if (lane == 0) wave_n[wave] = __popcll(mk);
  __syncthreads();
  int base = 0, n = 0;
  for (int w = 0; w < 4; ++w) {
    base += w < wave ? wave_n[w] : 0;
    n += wave_n[w];
  }
  if (on) list[base + __popcll(mk & ((1ull << lane) - 1ull))] = gc_mine;
  __syncthreads();
  const int sub = tid % LPR;
  for (int j = tid / LPR; j < n; j += GROUPS) {
    const int gc = list[j];
    const int sg = gc / kk, c = gc - sg * kk;
    const SegInfo si = seg_info(sg, S, L, kk, N_idx);
    if (c >= si.k_s) continue;
    const int members = count[gc];
    if (members > UPD_BIG) {  // left to update_big_kernel
      if (sub == 0) big_list[atomicAdd(big_count, 1)] = gc;
      continue;
    }
    const size_t p0 = (size_t)si.unit * N_idx + si.seg_start;
    update_cluster<T, D, 4, true>(xhat + p0 * D, order + p0 + start[gc], members,
                                  chat + (size_t)gc * D + sub * EPC, sub);
  }
}

// ============================================================================
// Short segments (an index update's 1K tokens into 64 clusters; small builds): all T
// iterations of one segment in ONE workgroup of 16 waves, with the centroids, the
// assignments, the sorted order and the cluster counts in LDS from the first
// iteration to the last.  Per iteration: assign (the resident MFMA form), near-ties
// re-decided with fp64 similarities by one wave each, the counting sort, the update
// straight into the LDS centroid rows; the steps are those of the kernels above,
// separated by workgroup barriers instead of launches.  Only the normalised keys are
// read from global memory; the last iteration's order, counts and first positions
// are written there for the finalize step.  Launches per build: 5 instead of 4 T + 3.
// ============================================================================
constexpr int SMALL_L_MAX = 2048;   // points per segment
constexpr int SMALL_K_MAX = 128;    // clusters per segment
constexpr int SMALL_NW = 16;

template <int D>
inline size_t small_kmeans_lds(int kk) {
  return (size_t)32 * ((kk + 31) / 32) * ResidentTile<D>::ROWB +
         sizeof(int) * ((size_t)SMALL_NW * kk + kk + 2 * SMALL_L_MAX + 2 * (size_t)kk);
}

template <int D>
__global__ __launch_bounds__(64 * SMALL_NW) void kmeans_small_kernel(
    const bf16_t* __restrict__ xhat, const bf16_t* __restrict__ chat, int32_t* __restrict__ order,
    int32_t* __restrict__ count, int32_t* __restrict__ start, int S, int L, int kk, int N_idx, int iters,
    int key_bits) {
  using RT = ResidentTile<D>;
  constexpr int NT = 64 * SMALL_NW, LPR = D / 8, GROUPS = NT / LPR;
  extern __shared__ __attribute__((aligned(16))) char small_lds[];
  char* cent = small_lds;
  int* hist = reinterpret_cast<int*>(small_lds + (size_t)32 * ((kk + 31) / 32) * RT::ROWB);  // sort_segment's
  int* a_s = hist + SMALL_NW * kk + kk;   // cluster of every point
  int* ord_s = a_s + SMALL_L_MAX;         // points by cluster; before the sort: the near-tie list
  int* cnt_s = ord_s + SMALL_L_MAX;
  int* first_s = cnt_s + kk;
  int* flags = ord_s;
  __shared__ int nflag;
  const int sg = blockIdx.x;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t p0 = (size_t)si.unit * N_idx + si.seg_start;
  const bf16_t* X = xhat + p0 * D;
  const int nfrag = (si.L_s + 31) / 32;
  resident_load_centroids<D, NT>(chat + (size_t)sg * kk * D, si.k_s, cent);
#ifdef WAVE_TRACE  // phase times of workgroup 0 (100 MHz clock), printed at the end
  unsigned long long tp[5] = {0, 0, 0, 0, 0}, tl = wall_clock64();
  int nf_total = 0;
#define WAVE_PHASE(k) do { const unsigned long long now_ = wall_clock64(); tp[k] += now_ - tl; tl = now_; } while (0)
#else
#define WAVE_PHASE(k) do { } while (0)
#endif
  for (int t = 0; t < iters; ++t) {
    if (tid == 0) nflag = 0;
    __syncthreads();
    WAVE_PHASE(0);
    lean_assign_fragments<D, SMALL_NW>(X, cent, si.L_s, si.k_s, nfrag,
                                       [&](int point, int cluster, bool near_tie) {
                                         a_s[point] = cluster;
                                         if (near_tie) flags[atomicAdd(&nflag, 1)] = point;
                                       });
    __syncthreads();
    WAVE_PHASE(1);
    // near-ties: fp64 similarities in index order against the LDS copy of the centroids,
    // ties to the lowest centroid (the arithmetic of refine_kernel)
    const int nf = nflag;
#ifdef WAVE_TRACE
    nf_total += nf;
#endif
    for (int it = wave; it < nf; it += SMALL_NW) {
      const int point = flags[it];
      const bf16_t* xr = X + (size_t)point * D;
      double bv = -1.0e300;
      int bi = 0x7fffffff;
      for (int c = lane; c < si.k_s; c += 64) {
        const char* row = cent + (size_t)c * RT::ROWB;
        double acc = 0.0;
#pragma unroll 4
        for (int e0 = 0; e0 < D; e0 += 8) {
          float xf[8], cf[8];
          unpack<bf16_t>(load16(xr + e0), xf);
          unpack<bf16_t>(load16(row + e0 * 2), cf);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc = fma((double)xf[e], (double)cf[e], acc);
        }
        if (acc > bv) {  // c ascends within a lane, so strict > keeps the lowest index
          bv = acc;
          bi = c;
        }
      }
      for (int off = 32; off >= 1; off >>= 1) {
        const double ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (ov > bv || (ov == bv && oi < bi)) {
          bv = ov;
          bi = oi;
        }
      }
      if (lane == 0) a_s[point] = bi;
    }
    __syncthreads();
    WAVE_PHASE(2);
    sort_segment(a_s, ord_s, cnt_s, first_s, si.L_s, kk, key_bits, hist);
    __syncthreads();
    WAVE_PHASE(3);
    if (t + 1 < iters)
      for (int c = tid / LPR; c < si.k_s; c += GROUPS)
        update_cluster<bf16_t, D, 8, false>(X, ord_s + first_s[c], cnt_s[c],
                                     reinterpret_cast<bf16_t*>(cent + (size_t)c * RT::ROWB) + (tid % LPR) * 8,
                                     tid % LPR);
    WAVE_PHASE(4);
  }
#ifdef WAVE_TRACE
  if (blockIdx.x == 0 && (tid == 0 || tid == 1023))
    printf("kmeans_small tid %d (x10 ns): top %llu assign %llu refine %llu sort %llu update %llu; near-ties %d\n", tid,
           tp[0], tp[1], tp[2], tp[3], tp[4], nf_total);
#endif
#undef WAVE_PHASE
  for (int i = tid; i < si.L_s; i += NT) order[p0 + i] = ord_s[i];
  for (int c = tid; c < kk; c += NT) {
    count[(size_t)sg * kk + c] = cnt_s[c];
    start[(size_t)sg * kk + c] = first_s[c];
  }
}

// ============================================================================
// Finalize: sizes, offsets, mean of raw keys, value sums, permuted rows.
// ============================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void finalize_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const int32_t* __restrict__ order,
    const int32_t* __restrict__ count, const int32_t* __restrict__ start, T* __restrict__ centroids,
    T* __restrict__ vsum, int32_t* __restrict__ sizes, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, T* __restrict__ k_perm, T* __restrict__ v_perm, int S, int L, int kk,
    int N, int N_idx, int n_sink, int m, int mc, int nclusters, int row_stride, int row_base, int pos_base) {
  // row_base, pos_base: added to the offsets and to the positions (an update's clusters continue
  // the rows and the token positions of the index they are written behind)
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const int gc = blockIdx.x * GROUPS + grp;
  if (gc >= nclusters) return;
  const int sg = gc / kk, c = gc - sg * kk;
  const SegInfo si = seg_info(sg, S, L, kk, N_idx);
  if (c >= si.k_s) return;
  const int n = count[gc], st = start[gc];
  const int cid = si.s * kk + c;  // only the last segment can have fewer than kk clusters
  const size_t urow = (size_t)si.unit * N_idx;
  const size_t orow = (size_t)si.unit * row_stride;  // rows per unit in perm / k_perm / v_perm
  const int row0 = si.seg_start + st;
  if (sub == 0) {
    sizes[(size_t)si.unit * mc + cid] = n;  // mc: clusters per unit in the meta-index arrays
    offsets[(size_t)si.unit * (mc + 1) + cid] = row0 + row_base;
    if (cid == m - 1) offsets[(size_t)si.unit * (mc + 1) + m] = N_idx + row_base;
  }
  const int32_t* ord = order + urow + si.seg_start + st;
  const T* Ku = K + ((size_t)si.unit * N + n_sink + si.seg_start) * D + sub * EPC;
  const T* Vu = V + ((size_t)si.unit * N + n_sink + si.seg_start) * D + sub * EPC;
  double ka[EPC], va[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) ka[e] = va[e] = 0.0;
  for (int i = 0; i < n; i += 2) {
    const int i1 = min(i + 1, n - 1);
    const int pa = ord[i], pb = ord[i1];
    const uint4 k0 = load16(Ku + (size_t)pa * D), v0 = load16(Vu + (size_t)pa * D);
    const uint4 k1 = load16(Ku + (size_t)pb * D), v1 = load16(Vu + (size_t)pb * D);
    float f[EPC];
    store16(k_perm + (orow + row0 + i) * D + sub * EPC, k0);
    store16(v_perm + (orow + row0 + i) * D + sub * EPC, v0);
    if (sub == 0) perm[orow + row0 + i] = n_sink + si.seg_start + pa + pos_base;
    unpack<T>(k0, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) ka[e] += (double)f[e];
    unpack<T>(v0, f);
#pragma unroll
    for (int e = 0; e < EPC; ++e) va[e] += (double)f[e];
    if (i + 1 < n) {
      store16(k_perm + (orow + row0 + i + 1) * D + sub * EPC, k1);
      store16(v_perm + (orow + row0 + i + 1) * D + sub * EPC, v1);
      if (sub == 0) perm[orow + row0 + i + 1] = n_sink + si.seg_start + pb + pos_base;
      unpack<T>(k1, f);
#pragma unroll
      for (int e = 0; e < EPC; ++e) ka[e] += (double)f[e];
      unpack<T>(v1, f);
#pragma unroll
      for (int e = 0; e < EPC; ++e) va[e] += (double)f[e];
    }
  }
  T oc[EPC], ov[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) {
    oc[e] = quant_store<T>(n > 0 ? ka[e] / (double)n : 0.0);
    ov[e] = quant_store<T>(va[e]);
  }
  store16(centroids + ((size_t)si.unit * mc + cid) * D + sub * EPC, *reinterpret_cast<uint4*>(oc));
  store16(vsum + ((size_t)si.unit * mc + cid) * D + sub * EPC, *reinterpret_cast<uint4*>(ov));
}

// Steady rows: the first ns and the last (N - local_start) tokens of every unit.
template <typename T, int D>
__global__ __launch_bounds__(256) void steady_copy_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                          T* __restrict__ ks, T* __restrict__ vs, int N,
                                                          int ns, int local_start, int p,
                                                          int p_stride, int rows_total) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, GROUPS = 256 / LPR;
  const int sub = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  for (int row = blockIdx.x * GROUPS + grp; row < rows_total; row += gridDim.x * GROUPS) {
    const int unit = row / p, i = row - unit * p;
    const int src = i < ns ? i : local_start + (i - ns);
    const size_t dst = (size_t)unit * p_stride + i;  // p_stride: rows per unit in the steady buffers
    store16(ks + dst * D + sub * EPC, load16(K + ((size_t)unit * N + src) * D + sub * EPC));
    store16(vs + dst * D + sub * EPC, load16(V + ((size_t)unit * N + src) * D + sub * EPC));
  }
}

__global__ void zero_int_kernel(int32_t* p) { *p = 0; }
// p[i * stride] = v for i < n
__global__ void fill_int_kernel(int32_t* p, int n, size_t stride, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[(size_t)i * stride] = v;
}

// ============================================================================
// Host
// ============================================================================
static int min_kL(const wave_index& ix) {
  return ix.clusters_per_segment < ix.segment_len ? ix.clusters_per_segment : ix.segment_len;
}

BuildGeom build_geometry(const wave_index& ix) {
  BuildGeom g{};
  g.units = ix.B * ix.Hkv;
  g.segs = g.units * ix.S;
  if (ix.m == 0) {
    g.total = 0;
    return g;
  }
  const size_t es = ix.dtype == WAVE_BF16 ? 2 : 4;
  const size_t pts = (size_t)g.units * ix.N_idx;
  const size_t ncl = (size_t)g.segs * min_kL(ix);
  size_t o = 0;
  g.off_xhat = o;   o = align_up(o + pts * ix.d * es);
  g.off_chat = o;   o = align_up(o + ncl * ix.d * es);
  g.off_assign = o; o = align_up(o + pts * sizeof(int32_t));
  g.off_order = o;  o = align_up(o + pts * sizeof(int32_t));
  g.off_prev = o;   o = align_up(o + pts * sizeof(int32_t));
  g.off_count = o;  o = align_up(o + 3 * ncl * sizeof(int32_t));   // count, start, changed marks
  g.off_flag = o;   o = align_up(o + pts * sizeof(int32_t));
  g.off_nflag = o;  o = align_up(o + 256);
  g.off_init = o;   o = align_up(o + (size_t)g.segs * ix.d * sizeof(double));  // segment means
  g.total = o;
  return g;
}

// WAVE_NO_SMALL_KMEANS=1 in the environment keeps short segments on the one-launch-per-step
// kernels (the tests run both forms against the oracle).
static bool no_small_kmeans() {
  const char* e = getenv("WAVE_NO_SMALL_KMEANS");
  return e && e[0] == '1';
}

static int key_bits_for(int kk) {
  int b = 1;
  while ((1 << b) < kk) ++b;
  return b;
}

template <typename T, int D>
static void launch_assign(const T* xhat, const T* chat, int32_t* assign, int32_t* flag, int32_t* nflag,
                          int S, int L, int kk, int N_idx, int segs, hipStream_t st) {
  const int Lmax = L < N_idx ? L : N_idx;
  if constexpr (sizeof(T) == 2) {
    // Centroids resident in LDS when a segment's padded rows fit (k = 512 at d = 128 is
    // 136 KiB of the 160 KiB); two workgroups per segment keep the last round of
    // workgroups short.  Otherwise the centroids are staged through LDS tile by tile.
    const int kmax = kk < Lmax ? kk : Lmax;
    const size_t resident_lds = (size_t)32 * ((kmax + 31) / 32) * (D * 2 + 16);
    if (resident_lds <= 144 * 1024) {
      const int pieces = Lmax > 2048 ? 2 : 1;
      WAVE_LAUNCH("assign_mfma", (assign_resident_kernel<D, 1, 16>), segs * pieces, 1024, resident_lds, st,
                  xhat, chat, assign, flag, nflag, S, L, kk, N_idx, pieces);
    } else {
      constexpr int PWG = 8 * 32;
      const int wps = (Lmax + PWG - 1) / PWG;
      WAVE_LAUNCH("assign_mfma", (assign_mfma_kernel<D, 1, 8>), segs * wps, 64 * 8, 0, st, xhat, chat,
                  assign, flag, nflag, S, L, kk, N_idx, wps);
    }
  } else {
    const int wps = (Lmax + 255) / 256;
    WAVE_LAUNCH("assign_plain", (assign_plain_kernel<T, D>), segs * wps, 256, 0, st, xhat, chat,
                assign, flag, nflag, S, L, kk, N_idx, wps);
  }
}

template <typename T, int D>
static wave_status build_td(const void* K_, const void* V_, const wave_index& ix, int iters,
                            uint64_t seed, void* ws, hipStream_t st, int seg_id_base, int row_base,
                            int pos_base) {
  const T* K = static_cast<const T*>(K_);
  const T* V = static_cast<const T*>(V_);
  const int units = ix.B * ix.Hkv;
  const int ns = ix.n_sink < ix.N ? ix.n_sink : ix.N;
  const int local_start = ns + ix.N_idx;
  if (ix.p > 0) {
    const int rows = units * ix.p;
    const int grid = (rows + 15) / 16 < 65536 ? (rows + 15) / 16 : 65536;
    WAVE_LAUNCH("steady_copy", (steady_copy_kernel<T, D>), grid, 256, 0, st, K, V,
                static_cast<T*>(ix.k_steady), static_cast<T*>(ix.v_steady), ix.N, ns, local_start, ix.p,
                steady_stride(ix), rows);
  }
  if (ix.m == 0) {
    // nothing to cluster: offsets[0] = 0 in every unit (units are cluster_stride + 1 entries apart)
    if (ix.offsets)
      WAVE_LAUNCH("fill", fill_int_kernel, (units + 255) / 256, 256, 0, st, ix.offsets, units,
                  (size_t)cluster_stride(ix) + 1, 0);
    return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
  }

  const BuildGeom g = build_geometry(ix);
  char* w = static_cast<char*>(ws);
  T* xhat = reinterpret_cast<T*>(w + g.off_xhat);
  T* chat = reinterpret_cast<T*>(w + g.off_chat);
  int32_t* assign = reinterpret_cast<int32_t*>(w + g.off_assign);
  int32_t* order = reinterpret_cast<int32_t*>(w + g.off_order);
  const int kk = min_kL(ix);
  const int ncl = g.segs * kk;
  int32_t* count = reinterpret_cast<int32_t*>(w + g.off_count);
  int32_t* start = count + ncl;
  int32_t* changed = start + ncl;  // per cluster: a point entered or left it in the current round
  int32_t* prev = reinterpret_cast<int32_t*>(w + g.off_prev);  // every point's cluster of the round before
  int32_t* flag = reinterpret_cast<int32_t*>(w + g.off_flag);
  int32_t* nflag = reinterpret_cast<int32_t*>(w + g.off_nflag);
  double* mean = reinterpret_cast<double*>(w + g.off_init);
  const int S = ix.S, L = ix.segment_len, N_idx = ix.N_idx;
  constexpr int GROUPS = 256 / (D / Elem<T>::EPC);

  WAVE_LAUNCH("seg_mean", (seg_mean_kernel<T, D>), g.segs, 256, 0, st, K, mean, nflag, S, L, kk, ix.N,
              N_idx, ns);
  {
    const long long rows = (long long)units * N_idx;
    const long long want = (rows + GROUPS - 1) / GROUPS;
    const int grid = (int)(want < 262144 ? want : 262144);
    WAVE_LAUNCH("normalise", (normalise_kernel<T, D>), grid, 256, 0, st, K, mean, xhat, S, L, ix.N,
                N_idx, ns, (int)rows);
  }
  WAVE_LAUNCH("init", (init_kernel<T, D>), g.segs, 256, 2 * sizeof(int) * (size_t)kk, st, xhat, chat, S, L,
              kk, N_idx, ix.Hkv, seed, seg_id_base);

  int W = SORT_HIST_INTS / kk;
  if (W > 16) W = 16;
  if (W < 1) W = 1;
  const size_t sort_lds = ((size_t)W * kk + kk) * sizeof(int);
  const int kb = key_bits_for(kk);
  const int cl_grid = (ncl + GROUPS - 1) / GROUPS;
  bool small = false;
  if constexpr (sizeof(T) == 2) {
    const int Lmax = L < N_idx ? L : N_idx;
    small = Lmax <= SMALL_L_MAX && kk <= SMALL_K_MAX && !no_small_kmeans();
    if (small)
      WAVE_LAUNCH("kmeans_small", (kmeans_small_kernel<D>), g.segs, 64 * SMALL_NW, small_kmeans_lds<D>(kk), st,
                  xhat, chat, order, count, start, S, L, kk, N_idx, iters, kb);
  }
  for (int t = 0; t < iters && !small; ++t) {
    launch_assign<T, D>(xhat, chat, assign, flag, nflag, S, L, kk, N_idx, g.segs, st);
    WAVE_LAUNCH("refine", (refine_kernel<T, D>), 1024, 256, 0, st, xhat, chat, assign, flag, nflag, S,
                L, kk, N_idx);
    // (first round: nothing to compare with, every cluster is updated and every mark cleared)
    WAVE_LAUNCH("sort", sort_kernel, g.segs, 64 * W, sort_lds, st, assign, order, count, start, nflag,
                prev, changed, t == 0 ? 1 : 0, S, L, kk, N_idx, kb);
    if (t + 1 < iters) {
      // (large clusters go onto a list, which the third kernel takes: nflag[1] counts them and
      // the flagged-point list, consumed by refine, is free to hold them)
      if (t == 0) {
        WAVE_LAUNCH("update", (update_kernel<T, D>), cl_grid, 256, 0, st, xhat, chat, order, count,
                    start, changed, 1, flag, nflag + 1, S, L, kk, N_idx, ncl);
      } else {
        WAVE_LAUNCH("update", (update_touched_kernel<T, D>), (ncl + 255) / 256, 256, 0, st, xhat, chat,
                    order, count, start, changed, flag, nflag + 1, S, L, kk, N_idx, ncl);
      }
      const int big_grid = ncl / UPD_BIG + 1 < 2048 ? ncl / UPD_BIG + 1 : 2048;
      WAVE_LAUNCH("update", (update_big_kernel<T, D>), big_grid, 256, 0, st, xhat, chat, order, count,
                  start, flag, nflag + 1, S, L, kk, N_idx);
    }
  }
  WAVE_LAUNCH("finalize", (finalize_kernel<T, D>), cl_grid, 256, 0, st, K, V, order, count, start,
              static_cast<T*>(ix.centroids), static_cast<T*>(ix.vsum), ix.sizes, ix.offsets, ix.perm,
              static_cast<T*>(ix.k_perm), static_cast<T*>(ix.v_perm), S, L, kk, ix.N, N_idx, ns, ix.m,
              cluster_stride(ix), ncl, row_stride(ix), row_base, pos_base);
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

wave_status launch_build(const void* K, const void* V, const wave_index& ix, int iters, uint64_t seed,
                         void* ws, hipStream_t st, int seg_id_base, int row_base, int pos_base) {
  if (ix.dtype == WAVE_BF16) {
    if (ix.d == 128) return build_td<bf16_t, 128>(K, V, ix, iters, seed, ws, st, seg_id_base, row_base, pos_base);
    if (ix.d == 64) return build_td<bf16_t, 64>(K, V, ix, iters, seed, ws, st, seg_id_base, row_base, pos_base);
  } else {
    if (ix.d == 128) return build_td<float, 128>(K, V, ix, iters, seed, ws, st, seg_id_base, row_base, pos_base);
    if (ix.d == 64) return build_td<float, 64>(K, V, ix, iters, seed, ws, st, seg_id_base, row_base, pos_base);
  }
  return WAVE_ERR_SHAPE;
}

template <typename T, int D>
static wave_status assign_step_td(const void* xhat, const void* chat, int L_s, int k_s, int32_t* assign,
                                  void* ws, hipStream_t st) {
  int32_t* nflag = static_cast<int32_t*>(ws);
  int32_t* flag = nflag + 64;
  hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, nflag);
  // one unit, one segment: S = 1, L = N_idx = L_s, kk = k_s
  launch_assign<T, D>(static_cast<const T*>(xhat), static_cast<const T*>(chat), assign, flag, nflag, 1,
                      L_s, k_s, L_s, 1, st);
  WAVE_LAUNCH("refine", (refine_kernel<T, D>), 256, 256, 0, st, static_cast<const T*>(xhat),
              static_cast<const T*>(chat), assign, flag, nflag, 1, L_s, k_s, L_s);
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

wave_status launch_assign_step(const void* xhat, const void* chat, int dtype, int L_s, int k_s, int d,
                               int32_t* assign, void* ws, hipStream_t st) {
  if (dtype == WAVE_BF16) {
    if (d == 128) return assign_step_td<bf16_t, 128>(xhat, chat, L_s, k_s, assign, ws, st);
    if (d == 64) return assign_step_td<bf16_t, 64>(xhat, chat, L_s, k_s, assign, ws, st);
  } else {
    if (d == 128) return assign_step_td<float, 128>(xhat, chat, L_s, k_s, assign, ws, st);
    if (d == 64) return assign_step_td<float, 64>(xhat, chat, L_s, k_s, assign, ws, st);
  }
  return WAVE_ERR_SHAPE;
}

}  // namespace wave
