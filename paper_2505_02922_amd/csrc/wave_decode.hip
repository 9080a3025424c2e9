// Decode step of the wave index: centroid scoring, top-r cluster selection,
// exact attention over the steady and retrieved tokens, centroid-based
// estimation of every other cluster, and the log-sum-exp merge of the zones
// (paper: decode steps 1-4 of the system overview; "Tripartite Attention
// Approximation"; estimation equations).
//
// All kernels are bandwidth-shaped: a row of d elements is read by LPR lanes as
// 16-byte chunks, so one wave-wide load covers 1 KiB of contiguous rows; dot
// products are reduced over those lanes with DPP.  Logits are kept in base-2
// units (logit * log2 e) so that the exponential is a bare v_exp_f32.
#include <stdlib.h>

#include "wave_common.h"

namespace wave {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no logit seen yet"

// Phase timestamps for tuning (builds with -DWAVE_TRACE only): thread 0 of a selecting
// workgroup writes the 100 MHz wall clock into the head's selection bitmap words, which the
// filtered selection does not otherwise use.
#ifdef WAVE_TRACE
#define WAVE_STAMP(buf, k)                                                                  \
  do {                                                                                      \
    if (threadIdx.x == 0) reinterpret_cast<unsigned long long*>(buf)[k] = wall_clock64();   \
  } while (0)
#else
#define WAVE_STAMP(buf, k) \
  do {                     \
  } while (0)
#endif

// ============================================================================
// 1. Meta-index pass: one workgroup takes DENSE_ROWS clusters of one unit for
//    all G query heads of that KV head and makes a single trip over their
//    centroids and value sums.
//      A  z[b, hq, c] = q[b, hq] . C[b, hkv, c]  (empty clusters -inf), written
//         for the selection step and kept in LDS; it also reports a bound on the
//         largest squared centroid norm of its range (selection's error bound);
//      B  estimation weights of ALL its clusters, w_c = exp(z_c / sqrt(d)) taken
//         relative to the largest score of the range, and sum_c s_c w_c;
//      C  sum_c w_c VS_c.
//    The result is one partial (max, sum, acc[d]) per head and range.  Clusters
//    that a head later selects are taken out again, with the same terms and a
//    minus sign, by the fused selection kernel or by the retrieval kernel (the
//    terms are bounded by the final normaliser, so the cancellation costs about
//    one fp32 ulp of the output).
// ============================================================================
constexpr int DENSE_ROWS = 256;
constexpr int SCORE_TILE = 16;  // clusters per entry of the score pass's table of maxima

// LDS of the meta-index pass for a workgroup of NT threads over NT clusters.
template <typename T, int D, int G, int NT>
struct DenseLds {
  static constexpr int NWV = NT / 64, STR = D + 2;
  static constexpr int PITCH = D * 2 + 16;  // bf16 tile row pitch: 16 lanes of a k-block hit 64 distinct banks
  static constexpr int ZG = (G + 3) / 4 * 4;                       // heads per row of zw, padded to whole float4s
  static constexpr size_t ZW = sizeof(float) * NT * ZG;            // [cluster][head]: z, then w
  static constexpr size_t SMEM = sizeof(float) * NWV * G * STR;    // per-wave partial sums
  static constexpr size_t RED = sizeof(float) * NWV * (2 * G + 1);
  static constexpr size_t ZREF = sizeof(float) * G;
  static constexpr size_t TILE = sizeof(T) == 2 ? (size_t)NWV * 16 * PITCH : 0;
  // zw, red, zref live through all phases; the scoring tiles (phase A) and the
  // per-wave partial sums (end of phase C) never live at the same time and share
  // one region, which lets one more workgroup fit on a CU.
  static constexpr size_t FIXED = (ZW + RED + ZREF + 15) / 16 * 16;
  static constexpr size_t estimate_bytes = FIXED + (SMEM + 15) / 16 * 16;
  static constexpr size_t score_bytes = FIXED + ((TILE > SMEM ? TILE : SMEM) + 15) / 16 * 16;
  float* zw;
  float* smem;
  float (*red)[2 * G + 1];
  float* zref_s;
  char* tile;
  __device__ __forceinline__ explicit DenseLds(char* base) {
    zw = reinterpret_cast<float*>(base);
    red = reinterpret_cast<float (*)[2 * G + 1]>(base + ZW);
    zref_s = reinterpret_cast<float*>(base + ZW + RED);
    smem = reinterpret_cast<float*>(base + FIXED);
    tile = base + FIXED;
  }
};

// A: scores of clusters [c0, c0 + nrows) of one unit for its G heads, written to
// z and left in lds.zw; every wave leaves the largest squared centroid norm it
// saw in lds.red[wave][2 G].  The caller synchronises.
template <typename T, int D, int G, int NT, bool PREFETCH = false>
__device__ __forceinline__ void dense_scores(const T* __restrict__ q, const T* __restrict__ C,
                                             const int32_t* __restrict__ su, float* __restrict__ z,
                                             int unit, int bh0, int m, int mc, int c0, int nrows,
                                             const DenseLds<T, D, G, NT>& lds,
                                             float* __restrict__ tile_max = nullptr) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64, GROUPS = NWV * RPW;
  constexpr int ZG = DenseLds<T, D, G, NT>::ZG;
  constexpr int U = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  float* zw = lds.zw;
  if constexpr (sizeof(T) == 2) {
    // bf16: the G x d by d x 16 products of a 16-cluster tile are MFMA work
    // (v_mfma_f32_16x16x32_bf16, heads padded to 16 columns).  Rows arrive with
    // fully coalesced loads (a wave-wide load is 1 KiB of consecutive rows), pass
    // through a padded per-wave LDS tile to reach the operand layout (lane =
    // cluster row + 16 * k-block), and a second MFMA of the tile with itself
    // yields the squared norms on the diagonal.
    typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
    typedef __attribute__((ext_vector_type(4))) float floatx4_t;
    constexpr int KS = D / 32;            // MFMA k-steps
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int RPL = 64 / CPR;         // rows per wave-wide load
    constexpr int NL = 16 / RPL;          // loads per 16-row tile
    constexpr int PITCH = DenseLds<T, D, G, NT>::PITCH;
    char* tile = lds.tile + (size_t)wave * 16 * PITCH;
    const int hj = lane & 15, kb = lane >> 4;
    bf16x8_t qb[KS];
#pragma unroll
    for (int s2 = 0; s2 < KS; ++s2) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (hj < G) v = load16(q + ((size_t)(bh0 + hj) * D + 32 * s2 + 8 * kb));
      qb[s2] = __builtin_bit_cast(bf16x8_t, v);
    }
    const T* Cu = C + ((size_t)unit * mc + c0) * D;
    const int lrow = lane / CPR, lch = lane % CPR;
    float cn2 = 0.f;
    const int ntile = (nrows + 15) / 16;
    // PREFETCH: the next tile's rows are requested before this tile is worked on
    // (for short-lived workgroups, where few other waves cover the round trip).
    auto load_tile = [&](int t, uint4 (&raw)[NL], int (&sz)[4]) {
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const int rr = min(16 * t + RPL * u + lrow, nrows - 1);
        raw[u] = load16_stream(Cu + (size_t)rr * D + lch * 8);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) sz[v] = su[min(16 * t + 4 * kb + v, nrows - 1)];
    };
    uint4 nraw[NL];
    int nsz[4];
    if (PREFETCH && wave < ntile) load_tile(wave, nraw, nsz);
    for (int t = wave; t < ntile; t += NWV) {
      uint4 raw[NL];
      int sz[4];
      if constexpr (PREFETCH) {
#pragma unroll
        for (int u = 0; u < NL; ++u) raw[u] = nraw[u];
#pragma unroll
        for (int v = 0; v < 4; ++v) sz[v] = nsz[v];
        if (t + NWV < ntile) load_tile(t + NWV, nraw, nsz);
      } else {
        load_tile(t, raw, sz);
      }
#pragma unroll
      for (int u = 0; u < NL; ++u) store16(&tile[(RPL * u + lrow) * PITCH + lch * 16], raw[u]);
      __builtin_amdgcn_wave_barrier();  // the tile is wave-private: LDS executes a wave's accesses in order
      floatx4_t acc = {0.f, 0.f, 0.f, 0.f}, gram = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s2 = 0; s2 < KS; ++s2) {
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, load16(&tile[hj * PITCH + (4 * s2 + kb) * 16]));
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[s2], acc, 0, 0, 0);
        gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, a, gram, 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
      // acc[v] = z[row 4 kb + v][head hj]; gram[v] is on the diagonal when 4 kb + v == hj
      const int dv = hj & 3;
      const float dg = dv == 0 ? gram[0] : (dv == 1 ? gram[1] : (dv == 2 ? gram[2] : gram[3]));
      if ((hj >> 2) == kb) cn2 = fmaxf(cn2, dg);
      float tmx = -INFINITY;
      if (hj < G) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int cc = 16 * t + 4 * kb + v;
          if (cc < nrows) {
            const float val = sz[v] > 0 ? acc[v] : -INFINITY;
            z[(size_t)(bh0 + hj) * m + c0 + cc] = val;
            zw[cc * ZG + hj] = val;
            tmx = fmaxf(tmx, val);
          }
        }
      }
      if (tile_max) {  // the tile's largest score per head (the tile is SCORE_TILE = 16 clusters)
        static_assert(SCORE_TILE == 16, "one MFMA tile per table entry");
        tmx = fmaxf(tmx, __shfl_xor(tmx, 16));
        tmx = fmaxf(tmx, __shfl_xor(tmx, 32));
        if (kb == 0 && hj < G)
          tile_max[(size_t)(bh0 + hj) * ((m + SCORE_TILE - 1) / SCORE_TILE) + c0 / SCORE_TILE + t] = tmx;
      }
    }
    cn2 = wave_max(cn2);
    if (lane == 0) lds.red[wave][2 * G] = cn2;
  } else {
    float qf[G][EPC];
#pragma unroll
    for (int g = 0; g < G; ++g) unpack<T>(load16(q + ((size_t)(bh0 + g) * D + sub * EPC)), qf[g]);
    const T* Cu = C + ((size_t)unit * mc + c0) * D + sub * EPC;
    float cn2 = 0.f;  // per-lane maximum of its chunk's squared sum; summed over lanes below
    for (int c = grp; c < nrows; c += GROUPS * U) {
      uint4 raw[U];
      int sz[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int cc = min(c + u * GROUPS, nrows - 1);
        raw[u] = load16(Cu + (size_t)cc * D);
        sz[u] = su[cc];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int cc = c + u * GROUPS;
        float cf[EPC];
        unpack<T>(raw[u], cf);
        float n2 = 0.f, sc[G];
#pragma unroll
        for (int e = 0; e < EPC; ++e) n2 = fmaf(cf[e], cf[e], n2);
        cn2 = fmaxf(cn2, n2);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float a = 0.f;
#pragma unroll
          for (int e = 0; e < EPC; ++e) a = fmaf(qf[g][e], cf[e], a);
          sc[g] = group_sum<LPR>(a);
        }
        float mine = sc[0];
#pragma unroll
        for (int g = 1; g < G; ++g) mine = (sub == g) ? sc[g] : mine;
        if (cc < nrows && sub < G) {
          const float v = sz[u] > 0 ? mine : -INFINITY;
          z[(size_t)(bh0 + sub) * m + c0 + cc] = v;
          zw[cc * ZG + sub] = v;
        }
      }
    }
    // sum over the LPR lanes of a row of per-lane maxima >= maximum over rows of the row sums
    cn2 = group_sum<LPR>(cn2);
    cn2 = wave_max(cn2);
    if (lane == 0) lds.red[wave][2 * G] = cn2;
  }
}

// Largest squared centroid norm of the range, after dense_scores and a barrier.
template <typename T, int D, int G, int NT>
__device__ __forceinline__ float dense_cn2(const DenseLds<T, D, G, NT>& lds) {
  float v = lds.red[0][2 * G];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) v = fmaxf(v, lds.red[w][2 * G]);
  return v;
}

// B, C: estimation terms of clusters [c0, c0 + nrows) for the unit's G heads from
// the scores in lds.zw (visible to all threads): one partial per head at
// part_head0 + g * head_stride.  All NT threads call this.
template <typename T, int D, int G, int NT>
__device__ __forceinline__ void dense_estimate(const T* __restrict__ vsum,
                                               const int32_t* __restrict__ su, int unit, int m, int mc, int c0,
                                               int nrows, float scale_log2,
                                               const DenseLds<T, D, G, NT>& lds,
                                               float* __restrict__ part_head0, size_t head_stride) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64, GROUPS = NWV * RPW;
  constexpr int ZG = DenseLds<T, D, G, NT>::ZG;
  constexpr int STR = D + 2;
  constexpr int UC = 4;  // rows in flight per group
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  float* zw = lds.zw;
  float* smem = lds.smem;
  const T* Vu = vsum + ((size_t)unit * mc + c0) * D + sub * EPC;
  // ---- B: weights relative to the range maximum -----------------------------------
  float zmax[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mx = -INFINITY;
    for (int i = threadIdx.x; i < nrows; i += NT) mx = fmaxf(mx, zw[i * ZG + g]);
    zmax[g] = wave_max(mx);
  }
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) lds.red[wave][g] = zmax[g];
  }
  __syncthreads();
  float lsum[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mx = lds.red[0][g];
#pragma unroll
    for (int w = 1; w < NWV; ++w) mx = fmaxf(mx, lds.red[w][g]);
    if (threadIdx.x == 0) lds.zref_s[g] = mx;   // -inf: a range of empty clusters only
    zmax[g] = mx > -INFINITY ? mx : 0.f;          // (every weight is 0 then)
    const float ref2 = zmax[g] * scale_log2;
    float ls = 0.f;
    for (int i = threadIdx.x; i < nrows; i += NT) {
      const float w = exp2f(fmaf(zw[i * ZG + g], scale_log2, -ref2));  // exp2(-inf) = 0
      zw[i * ZG + g] = w;
      ls = fmaf((float)su[i], w, ls);
    }
    lsum[g] = wave_sum_f(ls);
  }
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) lds.red[wave][G + g] = lsum[g];
  }
  __syncthreads();

  // ---- C: value sums --------------------------------------------------------------
  float acc[G][EPC];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[g][e] = 0.f;
  for (int c = grp; c < nrows; c += GROUPS * UC) {
    uint4 raw[UC];
#pragma unroll
    for (int u = 0; u < UC; ++u) raw[u] = load16_stream(Vu + (size_t)min(c + u * GROUPS, nrows - 1) * D);
#pragma unroll
    for (int u = 0; u < UC; ++u) {
      const int cc = c + u * GROUPS;
      float vf[EPC], w[G];
      unpack<T>(raw[u], vf);
      if (cc < nrows) {
        float wp[ZG];
#pragma unroll
        for (int g4 = 0; g4 < ZG; g4 += 4) {
          const float4 t = *reinterpret_cast<const float4*>(&zw[cc * ZG + g4]);
          wp[g4] = t.x; wp[g4 + 1] = t.y; wp[g4 + 2] = t.z; wp[g4 + 3] = t.w;
        }
#pragma unroll
        for (int g = 0; g < G; ++g) w[g] = wp[g];
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g) w[g] = 0.f;
      }
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[g][e] = fmaf(w[g], vf[e], acc[g][e]);
    }
  }
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] += __shfl_xor(acc[g][e], off);
    }
  }
  if (lane < LPR) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float* dst = smem + (size_t)(wave * G + g) * STR;
#pragma unroll
      for (int e = 0; e < EPC; ++e) dst[2 + sub * EPC + e] = acc[g][e];
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * STR; idx += NT) {
    const int g = idx / STR, e = idx - g * STR;
    float v = 0.f;
    if (e == 0) {
      v = lds.zref_s[g] > -INFINITY ? lds.zref_s[g] * scale_log2 : kNegBig;  // no cluster: an empty partial
    } else if (e == 1) {
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += lds.red[w][G + g];
    } else {
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += smem[(size_t)(w * G + g) * STR + e];
    }
    part_head0[(size_t)g * head_stride + e] = v;
  }
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256, 4) void dense_kernel(const T* __restrict__ q, const T* __restrict__ C,
                                                    const T* __restrict__ vsum,
                                                    const int32_t* __restrict__ sizes,
                                                    float* __restrict__ z, float* __restrict__ cn2part,
                                                    int Hkv, int m, int mc, int chunks, int slots, int slot0,
                                                    float scale_log2, float* __restrict__ part) {
  using Lds = DenseLds<T, D, G, 256>;
  __shared__ __attribute__((aligned(16))) char lds_raw[Lds::score_bytes];
  const Lds lds(lds_raw);
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int unit = wg / chunks, chunk = wg - unit * chunks;
  const int b = unit / Hkv, h = unit - b * Hkv, Hq = Hkv * G;
  const int bh0 = b * Hq + h * G;
  const int c0 = chunk * DENSE_ROWS, nrows = min(DENSE_ROWS, m - c0);
  const int32_t* su = sizes + (size_t)unit * mc + c0;
  dense_scores<T, D, G, 256, true>(q, C, su, z, unit, bh0, m, mc, c0, nrows, lds);
  __syncthreads();
  if (threadIdx.x == 0) cn2part[(size_t)unit * chunks + chunk] = dense_cn2(lds);
  dense_estimate<T, D, G, 256>(vsum, su, unit, m, mc, c0, nrows, scale_log2, lds,
                               part + ((size_t)bh0 * slots + slot0 + chunk) * (D + 2),
                               (size_t)slots * (D + 2));
}

// The scores alone (the estimation terms are made by other launches, next to
// the selection).
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void score_kernel(const T* __restrict__ q, const T* __restrict__ C,
                                                    const int32_t* __restrict__ sizes,
                                                    float* __restrict__ z, float* __restrict__ cn2part,
                                                    int Hkv, int m, int mc, int chunks,
                                                    float* __restrict__ tile_max) {
  using Lds = DenseLds<T, D, G, 256>;
  __shared__ __attribute__((aligned(16))) char lds_raw[Lds::score_bytes];
  const Lds lds(lds_raw);
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int unit = wg / chunks, chunk = wg - unit * chunks;
  const int b = unit / Hkv, h = unit - b * Hkv, Hq = Hkv * G;
  const int bh0 = b * Hq + h * G;
  const int c0 = chunk * DENSE_ROWS, nrows = min(DENSE_ROWS, m - c0);
  dense_scores<T, D, G, 256, true>(q, C, sizes + (size_t)unit * mc + c0, z, unit, bh0, m, mc, c0, nrows, lds,
                                   sizeof(T) == 2 ? tile_max : nullptr);
  __syncthreads();
  if (threadIdx.x == 0) cn2part[(size_t)unit * chunks + chunk] = dense_cn2(lds);
  if (sizeof(T) != 2 && tile_max) {  // (the bf16 pass writes them tile by tile)
    // largest score of every run of SCORE_TILE clusters, per head (-inf: all empty)
    constexpr int TPC = DENSE_ROWS / SCORE_TILE, ZG = Lds::ZG;
    static_assert(TPC * G <= 256, "one thread per (tile, head)");
    const int t = threadIdx.x % TPC, g = threadIdx.x / TPC;
    if (g < G && SCORE_TILE * t < nrows) {
      float mx = -INFINITY;
      for (int j = SCORE_TILE * t; j < min(SCORE_TILE * (t + 1), nrows); ++j) mx = fmaxf(mx, lds.zw[j * ZG + g]);
      const int ntile = (m + SCORE_TILE - 1) / SCORE_TILE;
      tile_max[(size_t)(bh0 + g) * ntile + chunk * TPC + t] = mx;
    }
  }
}

// ============================================================================
// 2. Top-r selection per query head.
//    The r-th largest score tau is searched on the order-preserving integer
//    image of the fp32 scores.  Scores accumulate in fp32, so clusters within the
//    accumulation error bound of tau are re-scored in fp64 and ranked exactly
//    (ties to the lower id).  Outputs: the selected ids in ascending order and
//    their number; on the fused path also first rows and running token counts.
// ============================================================================
constexpr int CAND_CAP = 1024;
constexpr int SURV_CAP = 256;  // scores left for the single-wave end of the threshold search
constexpr int SEL_BINS = 2048; // buckets of the one-sweep histogram that starts the threshold search
constexpr int SEL_TOP_BINS = 256;  // of which are counted one by one when there are few scores
constexpr int SEL_HIST_MIN = 6144;  // below this many scores plain halving steps are as fast

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Exclusive prefix sum of one int per thread across a workgroup of NT threads;
// returns the thread's prefix and the total.  scratch: NT / 64 ints.
template <int NT>
__device__ __forceinline__ int block_excl_scan(int v, int* scratch, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(inc, off);
    if (lane >= off) inc += t;
  }
  __syncthreads();  // scratch may still be read from a previous call
  if (lane == 63) scratch[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int s = scratch[w];
    if (w < wave) base += s;
    tot += s;
  }
  total = tot;
  return base + inc - v;
}

// Room for `n` entries per lane in a list whose length is the LDS counter *counter: one
// atomic per wave (same-address LDS atomics run one after the other), then a prefix over
// the lanes.  Returns the lane's first position.  All 64 lanes call this.
__device__ __forceinline__ int wave_excl_scan_alloc(int n, int* counter) {
  const int lane = threadIdx.x & 63;
  int inc = n;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(inc, off);
    if (lane >= off) inc += t;
  }
  const int total = __shfl(inc, 63);
  int base = 0;
  if (lane == 0 && total > 0) base = atomicAdd(counter, total);
  base = __shfl(base, 0);
  return base + inc - n;
}

template <int NT>
__device__ __forceinline__ int block_sum_i(int v, int* scratch) {
  int t;
  block_excl_scan<NT>(v, scratch, t);
  return t;
}

// The estimation terms of the clusters a head selected, with a minus sign: the
// meta-index pass added them for every cluster, the selected ones are attended
// exactly instead.  ids[0..nsel) are read from global memory (written by this
// workgroup before a barrier).
template <typename T, int D, int NT>
__device__ __forceinline__ void negative_partial(const T* __restrict__ vsum_u,
                                                 const int32_t* __restrict__ off,
                                                 const float* __restrict__ zz,
                                                 const int32_t* __restrict__ ids, int nsel,
                                                 float zmax, float scale_log2,
                                                 float* __restrict__ slot) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64;
  constexpr int GROUPS = NWV * RPW, STR = D + 2;
  __shared__ float scratch[NWV * STR];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  const float ref2 = zmax * scale_log2;
  float l = 0.f, acc[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
  constexpr int UN = 8;  // clusters in flight per group: the loads of a cluster depend on its id
  for (int t0 = grp; t0 < nsel; t0 += GROUPS * UN) {
    int c[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) c[u] = ids[min(t0 + u * GROUPS, nsel - 1)];
    float zc[UN];
    int o0[UN], o1[UN];
    uint4 raw[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      zc[u] = zz[c[u]];
      o0[u] = off[c[u]];
      o1[u] = off[c[u] + 1];
      raw[u] = load16(vsum_u + (size_t)c[u] * D + sub * EPC);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const float w = t0 + u * GROUPS < nsel ? exp2f(fmaf(zc[u], scale_log2, -ref2)) : 0.f;
      float vf[EPC];
      unpack<T>(raw[u], vf);
      l = fmaf(-(float)(o1[u] - o0[u]), w, l);
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[e] = fmaf(-w, vf[e], acc[e]);
    }
  }
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
    l += __shfl_xor(l, o);
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] += __shfl_xor(acc[e], o);
  }
  if (lane < LPR) {
    float* dst = scratch + (size_t)wave * STR;
#pragma unroll
    for (int e = 0; e < EPC; ++e) dst[2 + sub * EPC + e] = acc[e];
    if (sub == 0) dst[1] = l;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < STR; e += NT) {
    float v;
    if (e == 0) {
      v = nsel > 0 ? ref2 : kNegBig;  // nothing selected: an empty partial
    } else {
      v = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += scratch[(size_t)w * STR + e];
    }
    slot[e] = v;
  }
}

// The fallback for more clusters than the LDS-keyed selections below take: NT
// threads per query head, the scores re-read from memory in every pass (radix
// select, 4 passes of 8 bits, on the integer keys).
template <typename T, int D, int NT>
__device__ __forceinline__ void select_streaming(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot, int bh /* b * Hq + hq */, int write_neg = 1) {
  constexpr int NW = NT / 64;
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* zz = z + (size_t)bh * m;
  const int32_t* off = offsets + (size_t)unit * (mc + 1);
  int32_t* ids = sel_ids + (size_t)bh * rcap;
  int32_t* pref = sel_pref + (size_t)bh * (rcap + 1);
  int32_t* srow = sel_row + (size_t)bh * rcap;
  uint32_t* bits = bitmap + (size_t)bh * mwords;
  int32_t* usel = user_selected ? user_selected + (size_t)bh * usel_stride : nullptr;

  __shared__ int hist[256];
  __shared__ int scan_scratch[NW];
  __shared__ float fred[NW];
  __shared__ int cand_id[CAND_CAP];
  __shared__ double cand_z[CAND_CAP];
  __shared__ int sh_i[4];
  __shared__ float sh_f[2];

  // fn(i, v) runs for every i in [0, round_up(m, NT)), v = -inf past the end;
  // all lanes of a wave make the same calls, so fn may use wave-wide operations.
  auto scan = [&](auto fn) {
    for (int base = 0; base < m; base += NT) {
      const int i = base + tid;
      fn(i, i < m ? zz[i] : -INFINITY);
    }
  };

  // ---- valid count and maximum -------------------------------------------
  int nv = 0;
  float zmax = -INFINITY;
  scan([&](int, float v) {
    nv += (v > -INFINITY) ? 1 : 0;
    zmax = fmaxf(zmax, v);
  });
  zmax = wave_max(zmax);
  if (lane == 0) fred[wave] = zmax;
  const int nvalid = block_sum_i<NT>(nv, scan_scratch);  // its barriers publish fred
  zmax = fred[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) zmax = fmaxf(zmax, fred[w]);
  const int r_eff = min(r, nvalid);

  // mode 0: nothing selected; 1: every valid cluster; 2: threshold + exact band; 3: fp32 rule
  int mode;
  float tau = 0.f, lo = 0.f, hi = 0.f;
  int need_eq = 0;  // mode 3: how many clusters with score == tau are taken (lowest ids)
  int n_cand = 0, need = 0;
  if (r_eff == 0) {
    mode = 0;
  } else if (r_eff == nvalid) {
    mode = 1;
  } else {
    // ---- radix select: key of the r_eff-th largest score --------------------
    uint32_t prefix = 0, pmask = 0;
    int remaining = r_eff;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      scan([&](int, float v) {
        const uint32_t k = order_key(v);
        const bool in = (k & pmask) == prefix;
        const int dgt = (k >> shift) & 255;
        // scores crowd into few leading digits: when the whole wave agrees, one
        // lane adds for all (same-address LDS atomics would serialise)
        const uint64_t act = __ballot(in);
        if (act) {
          const int first = __shfl(dgt, __ffsll((long long)act) - 1);
          const uint64_t same = __ballot(in && dgt == first);
          if (same == act) {
            if (lane == __ffsll((long long)act) - 1) atomicAdd(&hist[first], __popcll(act));
          } else if (in) {
            atomicAdd(&hist[dgt], 1);
          }
        }
      });
      __syncthreads();
      // thread t (< 256) learns how many keys have a digit above t
      if (tid < 256) {
        int above = 0;
        for (int dgt = tid + 1; dgt < 256; ++dgt) above += hist[dgt];
        const int here = hist[tid];
        if (above < remaining && remaining <= above + here) {
          sh_i[0] = tid;
          sh_i[1] = remaining - above;
        }
      }
      __syncthreads();
      prefix |= ((uint32_t)sh_i[0]) << shift;
      pmask |= 255u << shift;
      remaining = sh_i[1];
      __syncthreads();
    }
    tau = key_to_float(prefix);
    need_eq = remaining;

    // ---- error bound of an fp32-accumulated score ---------------------------
    float qn2 = 0.f;
    for (int i = tid; i < D; i += NT) {
      const float v = to_f32(q[(size_t)bh * D + i]);
      qn2 += v * v;
    }
    qn2 = wave_sum_f(qn2);
    __syncthreads();
    if (lane == 0) fred[wave] = qn2;
    __syncthreads();
    if (tid == 0) {
      float s = 0.f;
      for (int w = 0; w < NW; ++w) s += fred[w];
      float c2 = 0.f;
      for (int i = 0; i < cn2_chunks; ++i) c2 = fmaxf(c2, cn2part[(size_t)unit * cn2_chunks + i]);
      // |fp32 score - exact| <= (chunk chain + reduction tree + slack) * 2^-24 * |q| |C|
      const float steps = (float)(Elem<T>::EPC + 6 + 4);
      sh_f[0] = 2.0f * steps * 5.9604645e-8f * sqrtf(s) * sqrtf(c2);
      sh_i[2] = 0;  // candidate counter
    }
    __syncthreads();
    const float guard = sh_f[0];
    lo = tau - guard;
    hi = tau + guard;

    // ---- classify: sure-in above the band, candidates inside it --------------
    int n_hi = 0;
    scan([&](int i, float v) {
      if (v > hi) {
        ++n_hi;
      } else if (v >= lo) {
        const int slot = atomicAdd(&sh_i[2], 1);
        if (slot < CAND_CAP) cand_id[slot] = i;
      }
    });
    n_hi = block_sum_i<NT>(n_hi, scan_scratch);
    n_cand = sh_i[2];
    need = r_eff - n_hi;
    if (n_cand > CAND_CAP) {
      mode = 3;  // too many near-equal scores: keep the fp32 ranking
    } else if (n_cand == need) {
      mode = 2;  // the whole band is taken; no ranking needed
    } else {
      mode = 2;
      // exact fp64 scores of the candidates
      const T* Cu = C + (size_t)unit * mc * D;
      for (int i = tid; i < n_cand; i += NT) {
        const T* row = Cu + (size_t)cand_id[i] * D;
        double acc = 0.0;
        for (int e = 0; e < D; ++e) acc = fma(to_f64(q[(size_t)bh * D + e]), to_f64(row[e]), acc);
        cand_z[i] = acc;
      }
      __syncthreads();
      for (int i = tid; i < n_cand; i += NT) {
        const double zi = cand_z[i];
        const int idi = cand_id[i];
        int rank = 0;
        for (int j = 0; j < n_cand; ++j) {
          const double zj = cand_z[j];
          rank += (zj > zi || (zj == zi && cand_id[j] < idi)) ? 1 : 0;
        }
        if (rank >= need) cand_id[i] = -1 - idi;  // dropped (kept negative so the id survives)
      }
      __syncthreads();
    }
  }

  // ---- bitmap of the selected clusters ---------------------------------------
  if (mode != 3) {
    // 64 consecutive clusters sit in the 64 lanes of a wave: a ballot is two bitmap words
    scan([&](int i, float v) {
      const bool on = mode == 1 ? (v > -INFINITY) : (mode == 2 ? (v > hi) : false);
      const uint64_t mk = __ballot(on);
      const int w = (i - lane) >> 5;
      if (lane == 0 && w < mwords) bits[w] = (uint32_t)mk;
      if (lane == 32 && w + 1 < mwords) bits[w + 1] = (uint32_t)(mk >> 32);
    });
    __syncthreads();
    if (mode == 2) {
      for (int i = tid; i < n_cand; i += NT) {
        const int id = cand_id[i];
        if (id >= 0) atomicOr(&bits[id >> 5], 1u << (id & 31));
      }
      __syncthreads();
    }
  } else {
    // fp32 rule: every score above tau, and of those equal to tau the need_eq
    // lowest ids.  Each thread owns a contiguous range of words so that "lowest
    // ids" is an exclusive count over the threads.
    const int words_per = (mwords + NT - 1) / NT;
    const int w0 = min(mwords, tid * words_per), w1 = min(mwords, w0 + words_per);
    int cnt = 0;
    for (int w = w0; w < w1; ++w)
      for (int j = 0; j < 32; ++j) {
        const int i = w * 32 + j;
        if (i < m && zz[i] == tau) ++cnt;
      }
    int tot;
    int eq_seen = block_excl_scan<NT>(cnt, scan_scratch, tot);
    for (int w = w0; w < w1; ++w) {
      uint32_t word = 0;
      for (int j = 0; j < 32; ++j) {
        const int i = w * 32 + j;
        if (i >= m) break;
        const float v = zz[i];
        bool on = v > tau;
        if (v == tau) {
          on = eq_seen < need_eq;
          ++eq_seen;
        }
        word |= on ? (1u << j) : 0u;
      }
      bits[w] = word;
    }
    __syncthreads();
  }

  // ---- ascending id list and running token counts -----------------------------
  {
    const int words_per = (mwords + NT - 1) / NT;
    const int w0 = min(mwords, tid * words_per), w1 = min(mwords, w0 + words_per);
    int cnt = 0, tok = 0;
    for (int w = w0; w < w1; ++w) {
      uint32_t word = bits[w];
      cnt += __popc(word);
      while (word) {
        const int j = __ffs(word) - 1;
        word &= word - 1;
        const int c = w * 32 + j;
        tok += off[c + 1] - off[c];
      }
    }
    int nsel, ntok;
    int pos = block_excl_scan<NT>(cnt, scan_scratch, nsel);
    int tpos = block_excl_scan<NT>(tok, scan_scratch, ntok);
    for (int w = w0; w < w1; ++w) {
      uint32_t word = bits[w];
      while (word) {
        const int j = __ffs(word) - 1;
        word &= word - 1;
        const int c = w * 32 + j;
        if (pos < rcap) {  // always true for a consistent selection; keeps a slip in bounds
          ids[pos] = c;
          srow[pos] = off[c];
          if (usel) usel[pos] = c;
          pref[pos] = tpos;
        }
        tpos += off[c + 1] - off[c];
        ++pos;
      }
    }
    for (int i = nsel + tid; i < rcap; i += NT) ids[i] = -1;
    if (usel)
      for (int i = nsel + tid; i < usel_stride; i += NT) usel[i] = -1;
    if (tid == 0) {
      pref[min(nsel, rcap)] = ntok;
      nsel_out[bh] = min(nsel, rcap);
    }
    __syncthreads();  // ids[] complete
    if (write_neg)
      negative_partial<T, D, NT>(vsum + (size_t)unit * mc * D, off, zz, ids, min(nsel, rcap),
                                 nvalid > 0 ? zmax : 0.f, scale_log2,
                                 part + ((size_t)bh * slots + neg_slot) * (D + 2));
  }
}

template <typename T, int D, int NT>
__global__ __launch_bounds__(NT) void select_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot) {
  select_streaming<T, D, NT>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc,
                             usel_stride, sel_ids, sel_pref, sel_row, bitmap, nsel_out, user_selected,
                             vsum, scale_log2, part, slots, neg_slot, blockIdx.x);
}

// ----------------------------------------------------------------------------
// Selection with the keys of all ranked positions in LDS (at most NT * VPT).
// Thread tid owns positions k * NT + tid, so the 64 lanes of a wave hold 64
// consecutive positions for every k, and popcounts of ballots give counts and
// ranks in position order without atomics.
//   1. threshold: a one-sweep histogram of the keys' upper bits, then halving of
//      the value interval (one ballot/popcount sweep and one barrier per step)
//      until few scores are left, which one wave finishes;
//   2. guard band around it, fp64 ranking of the few scores inside;
//   3. ids (and, unless told to stop there, first rows and running token counts)
//      in ascending order from a small table of per-(k, wave) counts.
// ----------------------------------------------------------------------------
// skeys: LDS for NT * ceil(m / NT) keys when LDSK.  If stage_cap > 0 the first rows
// and running token counts of the first stage_cap selected clusters are also left
// in the LDS arrays s_row / s_pref (s_pref gets nsel + 1 entries when nsel <=
// stage_cap).  Returns the number of selected clusters; *ntok_out their tokens.
// What a selection ranks: `npos` positions, position i standing for cluster
// id_base + i, or idmap[i] when a map is given (ascending ids, so that "lower
// position" is "lower id").  ids_only: stop after the ascending id list (written to
// ids_ptr, padded with -1 to rcap).
struct SelView {
  int npos, id_base;
  const int32_t* idmap;
  const float* zmap;   // with an id map: the scores by position (-inf at holes), saves the lookup in z
  int ids_only;        // 1: a slice (ids and scores to ids_ptr / z_out); 2: the head's list and count,
                       // nothing after them (the retrieval kernel derives the rest)
  int32_t* ids_ptr;
  float* z_out;        // the scores of the listed ids (ids_only: -inf padded like the ids)
  int32_t* s_ids = nullptr;  // LDS copy of the first stage_cap selected ids (saves reading them back)
  int no_neg = 0;      // 1: the caller's retrieval launch takes the selected clusters' estimation
                       // terms out again; no partial is written for them here
  float guard = -1.f;  // >= 0: the fp32 error bound of a score, already known to the caller
};

template <typename T, int D, int NT, int VPT, bool LDSK>
__device__ __forceinline__ int select_core(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot, int bh, uint32_t* skeys, int* s_pref,
    int* s_row, int stage_cap, int* ntok_out, const SelView view) {
  constexpr int NW = NT / 64;
  constexpr int TBL = VPT * NW;  // (k, wave) pairs in ascending cluster order
  static_assert(TBL <= NT && TBL >= 2 * NW, "one table entry per thread; scratch for extrema");
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* zz = z + (size_t)bh * m;
  const int32_t* off = offsets + (size_t)unit * (mc + 1);
  int32_t* ids = view.ids_ptr ? view.ids_ptr : sel_ids + (size_t)bh * rcap;
  const int npos = view.npos;  // positions ranked here; position i is cluster cid(i)
  auto cid = [&](int i) { return view.idmap ? view.idmap[i] : view.id_base + i; };
  int32_t* pref = sel_pref + (size_t)bh * (rcap + 1);
  int32_t* srow = sel_row + (size_t)bh * rcap;
  int32_t* usel = user_selected ? user_selected + (size_t)bh * usel_stride : nullptr;
  const uint64_t lt_mask = (1ull << lane) - 1ull;

  __shared__ int scan_scratch[NW];
  __shared__ int tbl_cnt[TBL];
  __shared__ int cand_id[CAND_CAP];
  __shared__ double cand_z[CAND_CAP];
  __shared__ int cnt3[3];
  __shared__ int sh_i[4];
  __shared__ float sh_f[2];
  static_assert(SEL_BINS * sizeof(int) <= CAND_CAP * sizeof(double), "the histogram borrows cand_z");
  int* hist = reinterpret_cast<int*>(cand_z);  // free until the candidates are re-scored
  uint32_t* trace = bitmap + (size_t)bh * mwords;
  (void)trace;
  WAVE_STAMP(trace, 10);

  // ---- this thread's scores as order-preserving integer keys -------------------
  // Error bound inputs first, so that their loads overlap with the key loads:
  // |fp32 score - exact| <= (chunk chain + reduction tree + slack) * 2^-24 * |q| |C|
  // (the loads are issued here and reduced after the key loads, so that the
  // last wave does not reach the first barrier a memory round trip late)
  static_assert(D <= 128, "two query elements per lane");
  float gq[2] = {0.f, 0.f}, gc[4] = {0.f, 0.f, 0.f, 0.f};
  if (wave == NW - 1 && view.guard < 0.f) {
#pragma unroll
    for (int j = 0; j < 2; ++j) gq[j] = to_f32(q[(size_t)bh * D + min(lane + 64 * j, D - 1)]);
#pragma unroll
    for (int j = 0; j < 4; ++j) gc[j] = cn2part[(size_t)unit * cn2_chunks + min(lane + 64 * j, cn2_chunks - 1)];
#pragma unroll
    for (int j = 0; j < 2; ++j) gq[j] = lane + 64 * j < D ? gq[j] : 0.f;  // (a repeated maximum is harmless)
  }
  // The keys live in LDS and every sweep is a short rolled loop (this code runs
  // once per workgroup, so unrolled sweeps over registers would cost more in
  // instruction fetch than they save).  LDSK: full 32-bit keys (m <= 16384).
  // Otherwise only the upper 16 bits are kept (m <= 65536): a sweep sees the
  // start of a key's 2^16-wide bucket, except for buckets inside the "hot" range
  // around the threshold, whose exact keys are re-read from memory.  All
  // comparisons below are made against bounds that are either bucket-aligned or
  // lie inside the hot range, so the truncated keys compare correctly.
  constexpr uint32_t kKeyNegInf = LDSK ? 0x007fffffu : 0x007f0000u;  // (bucket of) order_key(-inf)
  uint16_t* skeys16 = reinterpret_cast<uint16_t*>(skeys);
  const int nk = (npos + NT - 1) / NT;  // sweeps; <= VPT
  uint32_t hot_lo = 1, hot_hi = 0;    // hot buckets (16-bit), empty to begin with
  constexpr int KB = 16;  // loads in flight per thread
  for (int k0 = 0; k0 < nk; k0 += KB) {
    // Unconditional loads at clamped positions, masked afterwards: a load under a
    // lane condition is compiled into a branch with its own wait, which would
    // serialise the KB round trips.
    float v[KB];
    if (view.zmap) {  // scores by position; holes of the id map are -inf here
#pragma unroll
      for (int u = 0; u < KB; ++u) v[u] = view.zmap[min((k0 + u) * NT + tid, npos - 1)];
    } else if (!view.idmap) {
#pragma unroll
      for (int u = 0; u < KB; ++u) v[u] = zz[view.id_base + min((k0 + u) * NT + tid, npos - 1)];
    } else {
      int c[KB];
#pragma unroll
      for (int u = 0; u < KB; ++u) c[u] = view.idmap[min((k0 + u) * NT + tid, npos - 1)];
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        v[u] = zz[max(c[u], 0)];
        v[u] = c[u] >= 0 ? v[u] : -INFINITY;
      }
    }
#pragma unroll
    for (int u = 0; u < KB; ++u)
      if (k0 + u < nk) {
        if ((k0 + u) * NT + tid >= npos) v[u] = -INFINITY;
        const uint32_t ky = order_key(v[u] + 0.0f);  // + 0.0f folds -0 into +0
        if constexpr (LDSK) skeys[(k0 + u) * NT + tid] = ky;
        else skeys16[(k0 + u) * NT + tid] = (uint16_t)(ky >> 16);
      }
  }
  float guard_in = view.guard;
  if (wave == NW - 1 && view.guard < 0.f) {
    float qn2 = gq[0] * gq[0] + gq[1] * gq[1];
    float c2 = fmaxf(fmaxf(gc[0], gc[1]), fmaxf(gc[2], gc[3]));
    for (int i = lane + 256; i < cn2_chunks; i += 64) c2 = fmaxf(c2, cn2part[(size_t)unit * cn2_chunks + i]);
    qn2 = wave_sum_f(qn2);
    c2 = wave_max(c2);
    const float steps = 48.f;  // covers the vector chain + tree and the MFMA accumulation alike
    guard_in = 2.0f * steps * 5.9604645e-8f * sqrtf(qn2) * sqrtf(c2);
  }
  // fn(k, key of cluster k * NT + tid) for every sweep; wave-uniform trip count
  auto for_k = [&](auto fn) {
    for (int k = 0; k < nk; ++k) {
      if constexpr (LDSK) {
        fn(k, skeys[k * NT + tid]);
      } else {
        const uint32_t b16 = skeys16[k * NT + tid];
        uint32_t ky = b16 << 16;
        if (b16 >= hot_lo && b16 <= hot_hi) {
          const int i = k * NT + tid;
          ky = i < npos ? order_key(zz[cid(i)] + 0.0f) : ky;
        }
        fn(k, ky);
      }
    }
  };
  // fp64 score of position i as an order-preserving 64-bit integer (for the rare ranking of a
  // band too large for the candidate list); a thread caches its first four band positions
  uint64_t zc64[4] = {0, 0, 0, 0}, t64 = 0;
  int need_eq64 = 0;
  auto key64_of = [&](int i) -> uint64_t {
    const T* rowp = C + ((size_t)unit * mc + cid(i)) * D;
    double acc = 0.0;
    for (int e = 0; e < D; ++e) acc = fma(to_f64(q[(size_t)bh * D + e]), to_f64(rowp[e]), acc);
    const uint64_t u = (uint64_t)__double_as_longlong(acc + 0.0);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
  };
  auto band_key = [&](int j, int i) -> uint64_t {
    if (j < 4) return j == 0 ? zc64[0] : (j == 1 ? zc64[1] : (j == 2 ? zc64[2] : zc64[3]));
    return key64_of(i);
  };
  // ---- valid count, maximum, |q|^2, max |C|^2 ----------------------------------
  int nv = 0;
  uint32_t kmax = kKeyNegInf, kmin = 0xffffffffu;  // over the valid scores
  for_k([&](int, uint32_t ky) {
    nv += __popcll(__ballot(ky > kKeyNegInf));
    kmax = max(kmax, ky);
    kmin = min(kmin, ky > kKeyNegInf ? ky : 0xffffffffu);
  });
  for (int o = 32; o >= 1; o >>= 1) {
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
  }
  if (lane == 0) {
    scan_scratch[wave] = nv;
    tbl_cnt[wave] = (int)kmax;       // tbl_cnt doubles as scratch for the two extrema
    tbl_cnt[NW + wave] = (int)kmin;
  }
  if (tid < 3) cnt3[tid] = 0;
  if (wave == NW - 1) sh_f[0] = guard_in;
  __syncthreads();
  int nvalid = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) nvalid += scan_scratch[w];
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    kmax = max(kmax, (uint32_t)tbl_cnt[w]);
    kmin = min(kmin, (uint32_t)tbl_cnt[NW + w]);
  }
  if constexpr (!LDSK) kmax |= 0xffffu;  // end of the top bucket: an upper bound of every key
  const float zmax = key_to_float(kmax);
  const float guard = sh_f[0];
  const int r_eff = min(r, nvalid);
  WAVE_STAMP(trace, 11);

  // mode 0: nothing selected; 1: every valid cluster; 2: threshold + exact band (fp64 scores
  // kept in LDS); 3: the same band ranked in fp64 without keeping its scores
  int mode;
  uint32_t ktau = 0, klo_band = 0, khi_band = 0;
  float hi = 0.f;
  int n_cand = 0, need = 0;
  if (r_eff == 0) {
    mode = 0;
  } else if (r_eff == nvalid) {
    mode = 1;
  } else {
    // ---- threshold: largest key t with count(key >= t) >= r_eff ----------------
    // Stage 1, whole workgroup: halve the VALUE interval [klo, khi) (midpoint of
    // the two floats) until few scores are left inside; one ballot sweep and one
    // barrier per step.  Stage 2, one wave: the survivors sit in LDS and the
    // search finishes on integer keys without any barrier.
    uint32_t klo = kmin;       // count(>= klo) = nvalid >= r_eff
    uint32_t khi = kmax + 1;   // count(>= khi) = 0 < r_eff
    int cnt_lo = nvalid, cnt_hi = 0;
    int it = 0;
    if (npos > SEL_HIST_MIN || view.idmap) {
      // Stage 0, one sweep: count the valid keys by their upper 16 bits (sign,
      // exponent, 7 mantissa bits) in the SEL_BINS buckets below the maximum's
      // (everything lower shares bin 0); a scan from the top finds the bucket
      // that holds the r-th largest key, which replaces most halving steps.
      const uint32_t top16 = kmax >> 16;
      const uint32_t lo16 = top16 >= (uint32_t)(SEL_BINS - 1) ? top16 - (SEL_BINS - 1) : 0u;
      // LDS atomics run at about a lane per clock, so with few scores only the
      // top SEL_TOP_BINS buckets (two binades below the maximum) are counted one
      // by one; the keys below them are counted by ballot into bin 0.
      const uint32_t first_bin = npos <= 16384 ? (uint32_t)(SEL_BINS - SEL_TOP_BINS) : 1u;
      for (int i = tid; i < SEL_BINS; i += NT) hist[i] = 0;
      __syncthreads();
      int low = 0;
      for_k([&](int, uint32_t ky) {
        const bool valid = ky > kKeyNegInf;
        const uint32_t b16 = ky >> 16;
        const uint32_t rel = b16 > lo16 ? b16 - lo16 : 0u;
        if (valid && rel >= first_bin) atomicAdd(&hist[rel], 1);
        low += __popcll(__ballot(valid && rel < first_bin));
      });
      if (lane == 0 && low > 0) atomicAdd(&hist[0], low);
      __syncthreads();
      constexpr int PER = SEL_BINS / NT;
      static_assert(PER >= 1 && PER * NT == SEL_BINS, "bins per thread");
      int mine[PER], s = 0;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        mine[j] = hist[SEL_BINS - 1 - (tid * PER + j)];  // thread 0 holds the top bins
        s += mine[j];
      }
      int tot;
      int above = block_excl_scan<NT>(s, scan_scratch, tot);  // keys in the bins above mine[0]'s
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        if (above < r_eff && above + mine[j] >= r_eff) {  // exactly one (thread, j): r_eff <= nvalid
          sh_i[0] = SEL_BINS - 1 - (tid * PER + j);
          sh_i[1] = above;
          sh_i[3] = above + mine[j];
        }
        above += mine[j];
      }
      __syncthreads();
      const int bsel = sh_i[0];
      cnt_hi = sh_i[1];
      cnt_lo = sh_i[3];
      if (bsel > 0) klo = (lo16 + (uint32_t)bsel) << 16;                  // count(>= klo) = cnt_lo
      if (bsel < SEL_BINS - 1)                                            // count(>= khi) = cnt_hi
        khi = (lo16 + (bsel > 0 ? (uint32_t)bsel + 1u : first_bin)) << 16;
      __syncthreads();  // sh_i is reused below
    }
    if constexpr (!LDSK) {
      // bucket-aligned steps while the keys are only known to 16 bits
      while (khi - klo > 0x10000u && cnt_lo - cnt_hi > SURV_CAP) {
        uint32_t mid = order_key(0.5f * key_to_float(klo) + 0.5f * key_to_float(khi - 1) + 0.0f) & 0xffff0000u;
        if (mid <= klo) mid = klo + 0x10000u;   // klo is bucket-aligned here
        if (mid >= khi) mid = khi - 0x10000u;   // so is khi
        int c = 0;
        for_k([&](int, uint32_t ky) { c += __popcll(__ballot(ky >= mid)); });
        const int slot = it % 3;
        if (lane == 0) atomicAdd(&cnt3[slot], c);
        if (tid == 0) cnt3[(it + 1) % 3] = 0;
        __syncthreads();
        const int total = cnt3[slot];
        if (total >= r_eff) {
          klo = mid;
          cnt_lo = total;
        } else {
          khi = mid;
          cnt_hi = total;
        }
        ++it;
      }
      hot_lo = klo >> 16;
      hot_hi = (khi - 1) >> 16;  // from here on the keys inside [klo, khi) are exact
    }
    while (khi - klo > 1 && cnt_lo - cnt_hi > SURV_CAP) {
      uint32_t mid = order_key(0.5f * key_to_float(klo) + 0.5f * key_to_float(khi - 1) + 0.0f);
      if (mid <= klo || mid >= khi) mid = klo + ((khi - klo) >> 1);
      int c = 0;
      for_k([&](int, uint32_t ky) { c += __popcll(__ballot(ky >= mid)); });
      const int slot = it % 3;
      if (lane == 0) atomicAdd(&cnt3[slot], c);
      if (tid == 0) cnt3[(it + 1) % 3] = 0;
      __syncthreads();
      const int total = cnt3[slot];
      if (total >= r_eff) {
        klo = mid;
        cnt_lo = total;
      } else {
        khi = mid;
        cnt_hi = total;
      }
      ++it;
    }
      if (khi - klo > 1) {
      // survivors: klo <= key < khi, at most SURV_CAP of them
      __syncthreads();
      if (tid == 0) sh_i[2] = 0;
      __syncthreads();
      for_k([&](int, uint32_t ky) {
        if (ky >= klo && ky < khi) {
          const int slot = atomicAdd(&sh_i[2], 1);
          if (slot < SURV_CAP) cand_id[slot] = (int)ky;  // cnt_lo - cnt_hi <= SURV_CAP entries
        }
      });
      __syncthreads();
      if (wave == 0) {
        constexpr int PER = SURV_CAP / 64;
        const int ns = min(sh_i[2], SURV_CAP);
        uint32_t sk[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) sk[j] = lane + 64 * j < ns ? (uint32_t)cand_id[lane + 64 * j] : 0u;
        uint32_t a = klo, e = khi;  // invariant: cnt_hi + count(sk >= a) >= r_eff > cnt_hi + count(sk >= e)
        int ce = 0;
        while (e - a > 1) {
          const uint32_t mid = a + ((e - a) >> 1);
          int c = 0;
#pragma unroll
          for (int j = 0; j < PER; ++j) c += __popcll(__ballot(sk[j] >= mid));
          if (cnt_hi + c >= r_eff) {
            a = mid;
          } else {
            e = mid;
            ce = c;
          }
        }
        if (lane == 0) {
          sh_i[0] = (int)a;
          sh_i[1] = cnt_hi + ce;
        }
      }
      __syncthreads();
      klo = (uint32_t)sh_i[0];
      cnt_hi = sh_i[1];
    }
      ktau = klo;
    WAVE_STAMP(trace, 12);
    const float tau = key_to_float(ktau);
    hi = tau + guard;
    klo_band = order_key((tau - guard) + 0.0f);
    khi_band = order_key(hi + 0.0f);
    if constexpr (!LDSK) {
      hot_lo = klo_band >> 16;
      hot_hi = khi_band >> 16;
    }
    __syncthreads();
    if (tid == 0) sh_i[2] = 0;
    __syncthreads();

    // ---- classify: sure-in above the band, candidates inside it --------------
    int n_hi = 0;
    for_k([&](int k, uint32_t ky) {
      n_hi += __popcll(__ballot(ky > khi_band));
      if (ky >= klo_band && ky <= khi_band) {
        const int slot = atomicAdd(&sh_i[2], 1);
        if (slot < CAND_CAP) cand_id[slot] = k * NT + tid;
      }
    });
    if (lane == 0) scan_scratch[wave] = n_hi;
    __syncthreads();
    n_hi = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) n_hi += scan_scratch[w];
    n_cand = sh_i[2];
    need = r_eff - n_hi;
    if (n_cand > CAND_CAP) {
      // More scores inside the band than the candidate list holds: their fp64 scores are not
      // kept.  The need-th largest is found bit by bit on the order-preserving 64-bit image
      // of the fp64 score (64 counting steps, each re-scoring what a thread could not cache):
      // slow, exact, and only ever reached with over a thousand nearly equal centroids.
      mode = 3;
      {
        int j = 0;
        for_k([&](int k, uint32_t ky) {
          if (ky >= klo_band && ky <= khi_band) {
            const uint64_t v = key64_of(k * NT + tid);
            if (j == 0) zc64[0] = v;
            if (j == 1) zc64[1] = v;
            if (j == 2) zc64[2] = v;
            if (j == 3) zc64[3] = v;
            ++j;
          }
        });
      }
      auto count_band = [&](uint64_t bound, bool strict) {
        int c = 0, j = 0;
        for_k([&](int k, uint32_t ky) {
          if (ky >= klo_band && ky <= khi_band) {
            const uint64_t v = band_key(j, k * NT + tid);
            c += (strict ? v > bound : v >= bound) ? 1 : 0;
            ++j;
          }
        });
        return block_sum_i<NT>(c, scan_scratch);
      };
      uint64_t t = 0;
      for (int bit = 63; bit >= 0; --bit) {
        const uint64_t trial = t | (1ull << bit);
        if (count_band(trial, false) >= need) t = trial;
      }
      t64 = t;  // the need-th largest: count(>= t) >= need > count(>= t + 1)
      need_eq64 = need - count_band(t, true);
    } else if (n_cand == need) {
      mode = 2;  // the whole band is taken; no ranking needed
    } else {
      mode = 2;
      const T* Cu = C + (size_t)unit * mc * D;
      for (int i = tid; i < n_cand; i += NT) {
        const T* rowp = Cu + (size_t)cid(cand_id[i]) * D;
        double acc = 0.0;
        for (int e = 0; e < D; ++e) acc = fma(to_f64(q[(size_t)bh * D + e]), to_f64(rowp[e]), acc);
        cand_z[i] = acc;
      }
      __syncthreads();
      constexpr int NR = (CAND_CAP + NT - 1) / NT;
      bool drop[NR];
#pragma unroll
      for (int rr = 0; rr < NR; ++rr) {
        const int i = tid + rr * NT;
        drop[rr] = false;
        if (i < n_cand) {
          const double zi = cand_z[i];
          const int idi = cand_id[i];
          int rank = 0;
          for (int j = 0; j < n_cand; ++j) {
            const double zj = cand_z[j];
            rank += (zj > zi || (zj == zi && cand_id[j] < idi)) ? 1 : 0;
          }
          drop[rr] = rank >= need;
        }
      }
      __syncthreads();
#pragma unroll
      for (int rr = 0; rr < NR; ++rr)
        if (drop[rr]) cand_id[tid + rr * NT] = -1 - cand_id[tid + rr * NT];  // dropped
      __syncthreads();
    }
  }

  // ---- which of this thread's clusters are selected ------------------------------
  WAVE_STAMP(trace, 13);
  // bit k of `sel`; mode 3 needs the rank among equal scores in id order.
  uint64_t sel = 0;
  if (mode == 1) {
    for_k([&](int k, uint32_t ky) { sel |= (uint64_t)(ky > kKeyNegInf ? 1 : 0) << k; });
  } else if (mode == 2) {
    for_k([&](int k, uint32_t ky) {
      bool on = ky > khi_band;
      if (!on && ky >= klo_band) {  // in the band: look the decision up
        const int me = k * NT + tid;
        for (int j = 0; j < n_cand; ++j) on |= cand_id[j] == me;
      }
      sel |= (uint64_t)(on ? 1 : 0) << k;
    });
  } else if (mode == 3) {
    // above the band: in; inside it: fp64 score above the need-th largest, or equal to it and
    // among the need_eq64 lowest ids of those (positions are in id order)
    if (tid < TBL) tbl_cnt[tid] = 0;  // sweeps beyond nk stay empty
    __syncthreads();
    {
      int j = 0;
      for_k([&](int k, uint32_t ky) {
        const bool inb = ky >= klo_band && ky <= khi_band;
        uint64_t v = 0;
        if (inb) v = band_key(j++, k * NT + tid);
        const uint64_t eq = __ballot(inb && v == t64);
        if (lane == 0) tbl_cnt[k * NW + wave] = __popcll(eq);
      });
    }
    __syncthreads();
    int tot;
    const int base = block_excl_scan<NT>(tid < TBL ? tbl_cnt[tid] : 0, scan_scratch, tot);
    __syncthreads();
    if (tid < TBL) tbl_cnt[tid] = base;
    __syncthreads();
    {
      int j = 0;
      for_k([&](int k, uint32_t ky) {
        const bool inb = ky >= klo_band && ky <= khi_band;
        uint64_t v = 0;
        if (inb) v = band_key(j++, k * NT + tid);
        const uint64_t eq = __ballot(inb && v == t64);
        const int rank = tbl_cnt[k * NW + wave] + __popcll(eq & lt_mask);
        const bool on = ky > khi_band || (inb && (v > t64 || (v == t64 && rank < need_eq64)));
        sel |= (uint64_t)(on ? 1 : 0) << k;
      });
    }
    __syncthreads();
  }

  // ---- bitmap and ascending id list ------------------------------------------------
  if (tid < TBL) tbl_cnt[tid] = 0;  // sweeps beyond nk stay empty
  __syncthreads();
  for_k([&](int k, uint32_t) {
    const uint64_t mk = __ballot((sel >> k) & 1ull);
    if (lane == 0) tbl_cnt[k * NW + wave] = __popcll(mk);
  });
  __syncthreads();
  int nsel;
  const int cbase = block_excl_scan<NT>(tid < TBL ? tbl_cnt[tid] : 0, scan_scratch, nsel);
  __syncthreads();
  if (tid < TBL) tbl_cnt[tid] = cbase;
  __syncthreads();
  for_k([&](int k, uint32_t ky) {
    const bool on = (sel >> k) & 1ull;
    const uint64_t mk = __ballot(on);
    const int pos = tbl_cnt[k * NW + wave] + __popcll(mk & lt_mask);
    if (on && pos < rcap) {  // pos < rcap always holds for a consistent selection
      const int c = cid(k * NT + tid);
      ids[pos] = c;
      if (usel) usel[pos] = c;
      if (LDSK && view.z_out) view.z_out[pos] = key_to_float(ky);  // the key is the score, bit for bit
      if (view.s_ids && pos < stage_cap) view.s_ids[pos] = c;
    }
  });
  nsel = min(nsel, rcap);
  if (view.ids_only) {
    for (int i = nsel + tid; i < rcap; i += NT) {
      ids[i] = -1;
      if (view.z_out) view.z_out[i] = -INFINITY;
    }
    if (view.ids_only == 2) {
      if (usel)
        for (int i = nsel + tid; i < usel_stride; i += NT) usel[i] = -1;
      if (tid == 0) nsel_out[bh] = nsel;
    }
    *ntok_out = 0;
    return nsel;
  }
  __syncthreads();  // ids[] written by other waves are read below
  WAVE_STAMP(trace, 14);

  // ---- first row and running token count of every selected cluster -------------------
  int carry = 0;
  for (int base = 0; base < nsel; base += NT) {
    const int t = base + tid;
    int r0 = 0, size = 0;
    if (t < nsel) {
      int c;
      if (view.s_ids && nsel <= stage_cap) c = view.s_ids[t];
      else c = ids[t];
      r0 = off[c];
      size = off[c + 1] - r0;
      srow[t] = r0;
      if (t < stage_cap) s_row[t] = r0;
    }
    int tot;
    const int ex = block_excl_scan<NT>(size, scan_scratch, tot);
    if (t < nsel) {
      pref[t] = carry + ex;
      if (t < stage_cap) s_pref[t] = carry + ex;
    }
    carry += tot;
  }
  for (int i = nsel + tid; i < rcap; i += NT) ids[i] = -1;
  if (usel)
    for (int i = nsel + tid; i < usel_stride; i += NT) usel[i] = -1;
  if (tid == 0) {
    pref[nsel] = carry;
    if (nsel < stage_cap) s_pref[nsel] = carry;
    nsel_out[bh] = nsel;
  }
  __syncthreads();
  WAVE_STAMP(trace, 15);
  if (!view.no_neg)
    negative_partial<T, D, NT>(vsum + (size_t)unit * mc * D, off, zz, ids, nsel, nvalid > 0 ? zmax : 0.f,
                               scale_log2, part + ((size_t)bh * slots + neg_slot) * (D + 2));
  WAVE_STAMP(trace, 16);
  *ntok_out = carry;
  return nsel;
}

template <typename T, int D, int NT, int VPT, bool LDSK>
__global__ __launch_bounds__(NT) void select_cached_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot) {
  extern __shared__ uint32_t dyn_keys[];  // NT * ceil(m / NT) keys when LDSK
  int ntok;
  select_core<T, D, NT, VPT, LDSK>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc,
                                   usel_stride, sel_ids, sel_pref, sel_row, bitmap, nsel_out,
                                   user_selected, vsum, scale_log2, part, slots, neg_slot, blockIdx.x,
                                   dyn_keys, nullptr, nullptr, 0, &ntok,
                                   SelView{m, 0, nullptr, nullptr, 2, nullptr, nullptr});
}

// ============================================================================
// Exact attention over a list of rows for NG query heads that share the rows.
// Each group of LPR lanes owns rows grp, grp + GROUPS, ... and keeps its own
// online-softmax state; groups are merged at the end.
// ============================================================================
template <typename T, int D, int NG>
struct AttnState {
  static constexpr int EPC = Elem<T>::EPC;
  float qf[NG][EPC];
  float mx[NG], l[NG], acc[NG][EPC];

  __device__ __forceinline__ void init(const T* qbase, int sub, float scale_log2) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      unpack<T>(load16(qbase + (size_t)g * D + sub * EPC), qf[g]);
      mx[g] = kNegBig;
      l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        qf[g][e] *= scale_log2;
        acc[g][e] = 0.f;
      }
    }
  }

  // For rows_given only: no queries needed.
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      mx[g] = kNegBig;
      l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] = 0.f;
    }
  }

  // U rows whose logits s[g][u] (base-2 units) are known and which count mult[u]
  // times in the normaliser: a cluster standing for its members.
  // NEG: the rows are taken out again (terms added elsewhere for every cluster).
  template <int U, bool NEG = false>
  __device__ __forceinline__ void rows_given(const float (&s)[NG][U], const float (&mult)[U],
                                             const uint4 (&vraw)[U]) {
    float p[NG][U];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float mn = mx[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[g][u]);   // -inf for rows that do not count
      const float alpha = exp2f(mx[g] - mn);
      float ps = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        p[g][u] = NEG ? -exp2f(s[g][u] - mn) : exp2f(s[g][u] - mn);
        ps = fmaf(mult[u], p[g][u], ps);
      }
      l[g] = fmaf(l[g], alpha, ps);
      mx[g] = mn;
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPC];
      unpack<T>(vraw[u], vf);
#pragma unroll
      for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[g][e] = fmaf(p[g][u], vf[e], acc[g][e]);
    }
  }

  // U rows at once: kraw/vraw hold this lane's chunk of each row.
  template <int U, int LPR>
  __device__ __forceinline__ void rows(const uint4 (&kraw)[U], const uint4 (&vraw)[U],
                                       const bool (&valid)[U]) {
    float s[NG][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPC];
      unpack<T>(kraw[u], kf);
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        float a = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) a = fmaf(qf[g][e], kf[e], a);
        s[g][u] = group_sum<LPR>(a);
      }
    }
    float p[NG][U];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float mn = mx[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, valid[u] ? s[g][u] : kNegBig);
      const float alpha = exp2f(mx[g] - mn);
      float ps = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        p[g][u] = valid[u] ? exp2f(s[g][u] - mn) : 0.f;
        ps += p[g][u];
      }
      l[g] = fmaf(l[g], alpha, ps);
      mx[g] = mn;
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPC];
      unpack<T>(vraw[u], vf);
#pragma unroll
      for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[g][e] = fmaf(p[g][u], vf[e], acc[g][e]);
    }
  }
};

// Merge the per-group states of a 256-thread workgroup and write one partial
// result (max, sum, acc[D]) per head.  part_base points at head 0's slot;
// consecutive heads are head_stride floats apart.
template <typename T, int D, int NG, int NWV = 4>
__device__ __forceinline__ void merge_groups_and_store(AttnState<T, D, NG>& st, float* smem,
                                                       float* part_base, size_t head_stride) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane % LPR;
  // within the wave: combine the 64 / LPR groups
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const float mo = __shfl_xor(st.mx[g], off), lo = __shfl_xor(st.l[g], off);
      const float mn = fmaxf(st.mx[g], mo);
      const float a = exp2f(st.mx[g] - mn), bo = exp2f(mo - mn);
      st.l[g] = st.l[g] * a + lo * bo;
#pragma unroll
      for (int e = 0; e < EPC; ++e)
        st.acc[g][e] = st.acc[g][e] * a + __shfl_xor(st.acc[g][e], off) * bo;
      st.mx[g] = mn;
    }
  }
  // across the NWV waves through LDS: smem[wave][g][D + 2]
  constexpr int STR = D + 2;
  if (lane < LPR) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float* dst = smem + (size_t)(wave * NG + g) * STR;
#pragma unroll
      for (int e = 0; e < EPC; ++e) dst[2 + sub * EPC + e] = st.acc[g][e];
      if (sub == 0) {
        dst[0] = st.mx[g];
        dst[1] = st.l[g];
      }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < NG * STR; idx += 64 * NWV) {
    const int g = idx / STR, e = idx - g * STR;
    float m4[NWV], mn = kNegBig;
#pragma unroll
    for (int w = 0; w < NWV; ++w) {
      m4[w] = smem[(size_t)(w * NG + g) * STR];
      mn = fmaxf(mn, m4[w]);
    }
    float v;
    if (e == 0) {
      v = mn;
    } else {
      v = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += smem[(size_t)(w * NG + g) * STR + e] * exp2f(m4[w] - mn);
    }
    part_base[(size_t)g * head_stride + e] = v;
  }
}

// ============================================================================
// 4. Merge: one normalisation over the partial results of the three zones.
// ============================================================================
// All NT threads of the workgroup must call this (it contains barriers).  Thread
// t owns output dimension t % D and every (NT / D)-th partial result, which it
// folds into a running (max, sum, acc) of its own, UB partials per trip to memory
// (three loads each, all unconditional and in flight together); the NT / D
// running results then meet in LDS.
// p: the head's `slots` partial results (max, sum, acc[D]).  A partial without any
// term carries max = kNegBig and is skipped; a partial's sum may be zero or
// negative (the selected clusters' estimation terms are taken out with a minus
// sign, and may cancel a range's exact terms to the last bit), so the sum says
// nothing about whether a partial counts.
// p2, n2: a second run of partials that counts after the first (slots n1 .. n1 + n2 - 1).
template <int D, int NT, int UB = 4>
__device__ __forceinline__ void merge_head(const float* __restrict__ p, int n1,
                                           float* __restrict__ out_head, float* __restrict__ lse_head,
                                           const float* __restrict__ p2 = nullptr, int n2 = 0) {
  constexpr int STR = D + 2, NSG = NT / D;
  const int slots = n1 + n2;
  static_assert(NT % D == 0 && NT >= D, "whole slot groups");
  const int tid = threadIdx.x, e = tid % D, sg = tid / D;
  __shared__ float s_m[NSG], s_z[NSG];
  __shared__ float s_a[NSG * D];
  float M = kNegBig, Z = 0.f, A = 0.f;
  for (int s0 = sg; s0 < slots; s0 += NSG * UB) {
    float mm[UB], ll[UB], aa[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int sl = min(s0 + u * NSG, slots - 1);
      const float* ps = sl < n1 ? p + (size_t)sl * STR : p2 + (size_t)(sl - n1) * STR;
      mm[u] = ps[0];
      ll[u] = ps[1];
      aa[u] = ps[2 + e];
    }
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      if (s0 + u * NSG < slots && mm[u] > 0.5f * kNegBig) {
        const float mn = fmaxf(M, mm[u]);
        const float a = exp2f(M - mn), b = exp2f(mm[u] - mn);  // (M = kNegBig at first: a = 0)
        Z = fmaf(Z, a, ll[u] * b);
        A = fmaf(A, a, aa[u] * b);
        M = mn;
      }
    }
  }
  if (e == 0) {
    s_m[sg] = M;
    s_z[sg] = Z;
  }
  s_a[sg * D + e] = A;
  __syncthreads();
  if (sg == 0) {
    float Mx = s_m[0];
#pragma unroll
    for (int g = 1; g < NSG; ++g) Mx = fmaxf(Mx, s_m[g]);
    float Zt = 0.f, At = 0.f;
#pragma unroll
    for (int g = 0; g < NSG; ++g) {
      const float w = s_m[g] > 0.5f * kNegBig ? exp2f(s_m[g] - Mx) : 0.f;
      Zt = fmaf(s_z[g], w, Zt);
      At = fmaf(s_a[g * D + e], w, At);
    }
    // Zt > 0 for every index whose stored centroids are the means of their stored rows (the
    // estimation bound: a selected cluster's term never exceeds its rows' exact terms).  An
    // index that breaks this can cancel the normaliser away: that is reported as NaN, not
    // as a silent zero.
    const float bad = __uint_as_float(0x7fc00000u);
    out_head[e] = Zt > 0.f ? At / Zt : bad;
    if (e == 0) *lse_head = Zt > 0.f ? (Mx + log2f(Zt)) * kLn2 : bad;
  }
}

// ============================================================================
// 3a. Retrieval zone: one workgroup handles a share of the clusters selected by
//     one query head, reading their tokens in place from the cluster-contiguous
//     K/V.
// ============================================================================
constexpr int GATHER_TILE = 256;  // tokens (and clusters) per pass of a workgroup

// Workgroup `chunk` of a head takes an equal share of the head's selected
// clusters, by their position in the ascending id list: it reads their row
// ranges from the offsets, attends their tokens exactly, and, when own_neg is
// set, takes the same clusters' estimation terms (which the estimation pass
// added for every cluster) out again, in the same online-softmax state.
template <typename T, int D>
__device__ __forceinline__ void gather_role(
    int block, int nblocks, const T* __restrict__ q, const T* __restrict__ k_perm,
    const T* __restrict__ v_perm, const int32_t* __restrict__ sel_ids,
    const int32_t* __restrict__ nsel_arr, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const T* __restrict__ vsum, int Hq, int Hkv,
    int N_idx /* rows per unit in k_perm / v_perm */, int m, int mc, int rcap, int chunks, int slots,
    float scale_log2, int own_neg, float* __restrict__ part) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW, U = 4;
  const int wg = xcd_logical_block(block, nblocks);
  const int bh = wg / chunks, chunk = wg - bh * chunks;
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;

  __shared__ int rowidx[GATHER_TILE];
  __shared__ int cl_pref[GATHER_TILE + 1];
  __shared__ int cl_row[GATHER_TILE];
  __shared__ int cl_id[GATHER_TILE];
  __shared__ float cl_logit[GATHER_TILE];
  __shared__ int scan_scratch[4];
  __shared__ float smem[4 * (D + 2)];

  const int nsel = nsel_arr[bh];
  const int c_lo = (int)((long long)chunk * nsel / chunks), c_hi = (int)((long long)(chunk + 1) * nsel / chunks);
  const int32_t* ids = sel_ids + (size_t)bh * rcap;
  const int32_t* off = offsets + (size_t)unit * (mc + 1);
  const float* zz = z + (size_t)bh * m;

  AttnState<T, D, 1> st;
  st.init(q + (size_t)bh * D, sub, scale_log2);
  const T* Ku = k_perm + (size_t)unit * N_idx * D + sub * EPC;
  const T* Vu = v_perm + (size_t)unit * N_idx * D + sub * EPC;
  const T* VSu = vsum + (size_t)unit * mc * D + sub * EPC;

  for (int cb = c_lo; cb < c_hi; cb += GATHER_TILE) {
    const int nc = min(GATHER_TILE, c_hi - cb);
    // (first row, running token count, id, logit) of the pass's clusters
    int r0 = 0, size = 0, id = 0;
    float zc = -INFINITY;
    if ((int)threadIdx.x < nc) {
      id = ids[cb + threadIdx.x];
      r0 = off[id];
      size = off[id + 1] - r0;
      zc = zz[id];
    }
    int total;
    const int ex = block_excl_scan<256>(size, scan_scratch, total);  // barriers inside: the LDS arrays are free
    if ((int)threadIdx.x < nc) {
      cl_pref[threadIdx.x] = ex;
      cl_row[threadIdx.x] = r0;
      cl_id[threadIdx.x] = id;
      cl_logit[threadIdx.x] = zc * scale_log2;
    }
    if (threadIdx.x == 0) cl_pref[nc] = total;
    for (int base = 0; base < total; base += GATHER_TILE) {
      const int n = min(GATHER_TILE, total - base);
      __syncthreads();
      if ((int)threadIdx.x < n) {
        const int t = base + threadIdx.x;
        int a = 0, e = nc;  // largest a with cl_pref[a] <= t
        while (e - a > 1) {
          const int mid = (a + e) >> 1;
          if (cl_pref[mid] <= t) a = mid; else e = mid;
        }
        rowidx[threadIdx.x] = cl_row[a] + (t - cl_pref[a]);
      }
      __syncthreads();
      for (int i = grp; i < n; i += GROUPS * U) {
        uint4 kraw[U], vraw[U];
        bool valid[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int ii = i + u * GROUPS;
          valid[u] = ii < n;
          const int row = rowidx[valid[u] ? ii : i];
          kraw[u] = load16_stream(Ku + (size_t)row * D);
          vraw[u] = load16_stream(Vu + (size_t)row * D);
        }
        st.template rows<U, LPR>(kraw, vraw, valid);
      }
    }
    __syncthreads();  // cl_* complete even when the pass has no tokens
    if (own_neg) {
      for (int i = grp; i < nc; i += GROUPS * U) {
        uint4 vraw[U];
        float sc[1][U], mult[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int ii = i + u * GROUPS;
          const int j = ii < nc ? ii : i;
          vraw[u] = load16(VSu + (size_t)cl_id[j] * D);
          sc[0][u] = ii < nc ? cl_logit[j] : -INFINITY;
          mult[u] = (float)(cl_pref[j + 1] - cl_pref[j]);
        }
        st.template rows_given<U, true>(sc, mult, vraw);
      }
    }
    __syncthreads();  // before the next pass overwrites cl_*
  }
  merge_groups_and_store<T, D, 1>(st, smem, part + ((size_t)bh * slots + chunk) * (D + 2), 0);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_kernel(
    const T* __restrict__ q, const T* __restrict__ k_perm, const T* __restrict__ v_perm,
    const int32_t* __restrict__ sel_ids, const int32_t* __restrict__ nsel_arr,
    const int32_t* __restrict__ offsets, const float* __restrict__ z, const T* __restrict__ vsum,
    int Hq, int Hkv, int N_idx, int m, int mc, int rcap, int chunks, int slots, float scale_log2, int own_neg,
    float* __restrict__ part) {
  gather_role<T, D>(blockIdx.x, gridDim.x, q, k_perm, v_perm, sel_ids, nsel_arr, offsets, z, vsum, Hq, Hkv,
                    N_idx, m, mc, rcap, chunks, slots, scale_log2, own_neg, part);
}

// Estimation zone with a budget: the clusters of the (ascending) list ids2 that
// are not in the (ascending) list ids1 enter with their centroid's score as the
// logit, their size as the multiplicity and their value sum as the value.
// Workgroup `chunk` of a head takes an equal share of the positions of ids2.
constexpr int EST_STAGE = 4096;  // retrieved ids kept in LDS for the membership test

template <typename T, int D>
__device__ __forceinline__ void est_gather_role(
    int block, const int32_t* __restrict__ ids2_all, const int32_t* __restrict__ nsel2_arr,
    const int32_t* __restrict__ ids1_all, const int32_t* __restrict__ nsel1_arr,
    const int32_t* __restrict__ offsets, const float* __restrict__ z, const T* __restrict__ vsum,
    int Hq, int Hkv, int m, int mc, int rcap2, int rcap1, int chunks, int slots, int slot0, float scale_log2,
    float* __restrict__ part) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW;
  const int bh = block / chunks, chunk = block - bh * chunks;
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  __shared__ int s_ids1[EST_STAGE];
  __shared__ float smem[4 * (D + 2)];
  const int nsel2 = nsel2_arr[bh], nsel1 = nsel1_arr[bh];
  const int32_t* ids2 = ids2_all + (size_t)bh * rcap2;
  const int32_t* ids1g = ids1_all + (size_t)bh * rcap1;
  const bool staged = nsel1 <= EST_STAGE;
  if (staged)
    for (int i = threadIdx.x; i < nsel1; i += 256) s_ids1[i] = ids1g[i];
  __syncthreads();
  const int32_t* ids1 = staged ? s_ids1 : ids1g;
  const int32_t* off = offsets + (size_t)unit * (mc + 1);
  const float* zz = z + (size_t)bh * m;
  const T* VSu = vsum + (size_t)unit * mc * D + sub * EPC;
  const int c_lo = (int)((long long)chunk * nsel2 / chunks), c_hi = (int)((long long)(chunk + 1) * nsel2 / chunks);
  AttnState<T, D, 1> st;
  st.reset();
  // Passes of 256 list positions: one thread per position reads the id, looks it up in the
  // retrieved list, and reads the cluster's score and size (three dependent trips to memory
  // for 256 clusters at once); the value-sum rows then stream, eight per lane group in flight.
  __shared__ int t_id[256];
  __shared__ float t_logit[256], t_mult[256];
  constexpr int UE = 8;
  for (int p0 = c_lo; p0 < c_hi; p0 += 256) {
    const int n = min(256, c_hi - p0);
    __syncthreads();  // the previous pass is done with the tables
    {
      const int id = ids2[min(p0 + (int)threadIdx.x, c_hi - 1)];
      bool retrieved = false;
      if (nsel1 > 0) {  // largest a with ids1[a] <= id
        int a = 0, e = nsel1;
        while (e - a > 1) {
          const int mid = (a + e) >> 1;
          if (ids1[mid] <= id) a = mid; else e = mid;
        }
        retrieved = ids1[a] == id;
      }
      const float zc = zz[id];
      const int o0 = off[id], o1 = off[id + 1];
      t_id[threadIdx.x] = id;
      t_logit[threadIdx.x] = ((int)threadIdx.x < n && !retrieved) ? zc * scale_log2 : -INFINITY;
      t_mult[threadIdx.x] = (float)(o1 - o0);
    }
    __syncthreads();
    for (int i = grp; i < n; i += GROUPS * UE) {
      uint4 vraw[UE];
      float sc[1][UE], mult[UE];
#pragma unroll
      for (int u = 0; u < UE; ++u) {
        const int j = min(i + u * GROUPS, 255);  // entries at or beyond n carry -inf
        vraw[u] = load16(VSu + (size_t)t_id[j] * D);
        sc[0][u] = i + u * GROUPS < n ? t_logit[j] : -INFINITY;
        mult[u] = t_mult[j];
      }
      st.template rows_given<UE>(sc, mult, vraw);
    }
  }
  __syncthreads();
  merge_groups_and_store<T, D, 1>(st, smem, part + ((size_t)bh * slots + slot0 + chunk) * (D + 2), 0);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void est_gather_kernel(
    const int32_t* __restrict__ ids2_all, const int32_t* __restrict__ nsel2_arr,
    const int32_t* __restrict__ ids1_all, const int32_t* __restrict__ nsel1_arr,
    const int32_t* __restrict__ offsets, const float* __restrict__ z, const T* __restrict__ vsum,
    int Hq, int Hkv, int m, int mc, int rcap2, int rcap1, int chunks, int slots, int slot0, float scale_log2,
    float* __restrict__ part) {
  est_gather_role<T, D>(blockIdx.x, ids2_all, nsel2_arr, ids1_all, nsel1_arr, offsets, z, vsum, Hq, Hkv, m, mc,
                        rcap2, rcap1, chunks, slots, slot0, scale_log2, part);
}

// The retrieval zone and the budgeted estimation zone in one launch: both only need the two
// id lists, neither needs the other.  The estimation workgroups come first: they have the
// scattered value-sum rows, the retrieval workgroups the long contiguous ranges.
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_est_kernel(
    const T* __restrict__ q, const T* __restrict__ k_perm, const T* __restrict__ v_perm,
    const int32_t* __restrict__ ids1, const int32_t* __restrict__ nsel1,
    const int32_t* __restrict__ ids2, const int32_t* __restrict__ nsel2,
    const int32_t* __restrict__ offsets, const float* __restrict__ z, const T* __restrict__ vsum,
    int Hq, int Hkv, int N_idx, int m, int mc, int rcap1, int rcap2, int gather_chunks, int est_chunks, int slots,
    int gather_slot0, int est_slot0, int n_est_wgs, float scale_log2, float* __restrict__ part) {
  if ((int)blockIdx.x < n_est_wgs) {
    est_gather_role<T, D>(blockIdx.x, ids2, nsel2, ids1, nsel1, offsets, z, vsum, Hq, Hkv, m, mc, rcap2, rcap1,
                          est_chunks, slots, est_slot0, scale_log2, part);
    return;
  }
  gather_role<T, D>((int)blockIdx.x - n_est_wgs, (int)gridDim.x - n_est_wgs, q, k_perm, v_perm, ids1, nsel1,
                    offsets, z, vsum, Hq, Hkv, N_idx, m, mc, rcap1, gather_chunks, slots, scale_log2, 0,
                    part + (size_t)gather_slot0 * (D + 2));
}

constexpr int MERGE_THREADS = 1024;

template <int D, int NT = MERGE_THREADS>
__global__ __launch_bounds__(NT) void merge_kernel(const float* __restrict__ part, int slots, int slot_stride,
                                                   float* __restrict__ out, float* __restrict__ lse) {
  const int bh = blockIdx.x;  // a head's partials are slot_stride slots apart; the first `slots` count
  merge_head<D, NT, 16>(part + (size_t)bh * slot_stride * (D + 2), slots, out + (size_t)bh * D, lse + bh);
}

// ----------------------------------------------------------------------------
// Selection and retrieval zone of one query head in ONE workgroup: with many
// heads in flight (>= 2 per CU) the latency-bound selection of one workgroup
// overlaps with the streaming of its neighbours, the selected ranges never
// leave LDS, and the head produces a single partial result.
// ----------------------------------------------------------------------------
constexpr int FUSED_STAGE = 2048;  // selected clusters whose ranges stay in LDS

template <typename T, int D, int NT, int VPT, bool LDSK>
__global__ __launch_bounds__(NT) void select_gather_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot, const T* __restrict__ k_perm,
    const T* __restrict__ v_perm, int N_idx, const T* __restrict__ k_steady,
    const T* __restrict__ v_steady, int p, int p_stride, int stagger_period, float* __restrict__ out,
    float* __restrict__ lse) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64;
  constexpr int GROUPS = NWV * RPW, U = 4, TILE = NT;
  extern __shared__ uint32_t dyn_keys[];
  __shared__ int s_pref[FUSED_STAGE + 1];
  __shared__ int s_row[FUSED_STAGE];
  __shared__ int rowidx[TILE];
  __shared__ float smem[NWV * (D + 2)];
  __shared__ int sh_n[2];

  const int bh = xcd_logical_block(blockIdx.x, gridDim.x);
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;

  WAVE_STAMP(bitmap + (size_t)bh * mwords, 20);
  AttnState<T, D, 1> st;
  st.init(q + (size_t)bh * D, sub, scale_log2);

  // The steady rows of the head's KV unit (p > 0 only when this kernel owns the
  // steady zone).  Selection is latency-bound and leaves the memory system idle;
  // workgroups that share a CU are dispatched stagger_period ids apart, so every
  // other period streams its steady rows first and the rest does it last: one
  // neighbour streams while the other selects.
  auto steady_rows = [&]() {
    const T* Ks = k_steady + (size_t)unit * p_stride * D + sub * EPC;
    const T* Vs = v_steady + (size_t)unit * p_stride * D + sub * EPC;
    for (int i = grp; i < p; i += GROUPS * U) {
      uint4 kraw[U], vraw[U];
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ii = i + u * GROUPS;
        valid[u] = ii < p;
        const int row = valid[u] ? ii : i;
        kraw[u] = load16(Ks + (size_t)row * D);
        vraw[u] = load16(Vs + (size_t)row * D);
      }
      st.template rows<U, LPR>(kraw, vraw, valid);
    }
  };
  const bool steady_first = ((blockIdx.x / stagger_period) & 1) == 0;
  if (p > 0 && steady_first) steady_rows();
  int ntok;
  const int nsel = select_core<T, D, NT, VPT, LDSK>(
      q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc, usel_stride, sel_ids,
      sel_pref, sel_row, bitmap, nsel_out, user_selected, vsum, scale_log2, part, slots,
      neg_slot, bh, dyn_keys, s_pref, s_row, FUSED_STAGE, &ntok,
      SelView{m, 0, nullptr, nullptr, 0, nullptr, nullptr});
  if (threadIdx.x == 0) {
    sh_n[0] = nsel;
    sh_n[1] = ntok;
  }
  __syncthreads();  // publishes s_pref / s_row (and the global copies) to every wave
  const int nsel_all = sh_n[0], total = sh_n[1];

  const bool staged = nsel_all <= FUSED_STAGE;
  const T* Ku = k_perm + (size_t)unit * N_idx * D + sub * EPC;
  const T* Vu = v_perm + (size_t)unit * N_idx * D + sub * EPC;
  for (int base = 0; base < total; base += TILE) {
    const int n = min(TILE, total - base);
    __syncthreads();
    if ((int)threadIdx.x < n) {
      const int t = base + threadIdx.x;
      // largest a with pref[a] <= t; two copies so that the staged tables are read
      // with LDS instructions (one pointer for both would make every read a flat load)
      auto row_of = [&](const int32_t* pf, const int32_t* sr) {
        int a = 0, e = nsel_all;
        while (e - a > 1) {
          const int mid = (a + e) >> 1;
          if (pf[mid] <= t) a = mid; else e = mid;
        }
        return sr[a] + (t - pf[a]);
      };
      rowidx[threadIdx.x] = staged ? row_of(s_pref, s_row)
                                   : row_of(sel_pref + (size_t)bh * (rcap + 1), sel_row + (size_t)bh * rcap);
    }
    __syncthreads();
    for (int i = grp; i < n; i += GROUPS * U) {
      uint4 kraw[U], vraw[U];
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ii = i + u * GROUPS;
        valid[u] = ii < n;
        const int row = rowidx[valid[u] ? ii : i];
        kraw[u] = load16_stream(Ku + (size_t)row * D);
        vraw[u] = load16_stream(Vu + (size_t)row * D);
      }
      st.template rows<U, LPR>(kraw, vraw, valid);
    }
  }
  if (p > 0 && !steady_first) steady_rows();
  __syncthreads();
  merge_groups_and_store<T, D, 1, NWV>(st, smem, part + (size_t)bh * slots * (D + 2), 0);
  // Every partial result of this head now exists (the meta-index pass ran before
  // this kernel; the exact and the negative partials were just written by this
  // workgroup): normalise here instead of in a separate launch.
  __syncthreads();
  merge_head<D, NT, 8>(part + (size_t)bh * slots * (D + 2), slots, out + (size_t)bh * D, lse + bh);
  WAVE_STAMP(bitmap + (size_t)bh * mwords, 21);
}

// ============================================================================
// 3b. Steady zone: sink + local rows of one unit, shared by its G query heads.
// ============================================================================
// Rows [r0, r1) of one unit's steady buffers for its G query heads; smem:
// (NT / 64) * G * (D + 2) floats.  All NT threads call this.
template <typename T, int D, int G, int NT>
__device__ __forceinline__ void steady_rows_partial(const T* __restrict__ q,
                                                    const T* __restrict__ k_steady,
                                                    const T* __restrict__ v_steady, int unit, int bh0,
                                                    int p_stride, int r0, int r1, float scale_log2,
                                                    float* smem, float* __restrict__ part_head0,
                                                    size_t head_stride) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64, GROUPS = NWV * RPW;
  constexpr int U = (G <= 4) ? 4 : 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  AttnState<T, D, G> st;
  st.init(q + (size_t)bh0 * D, sub, scale_log2);
  const T* Ku = k_steady + (size_t)unit * p_stride * D + sub * EPC;  // p_stride: rows per unit
  const T* Vu = v_steady + (size_t)unit * p_stride * D + sub * EPC;
  for (int i = r0 + grp; i < r1; i += GROUPS * U) {
    uint4 kraw[U], vraw[U];
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ii = i + u * GROUPS;
      valid[u] = ii < r1;
      const int row = valid[u] ? ii : i;
      kraw[u] = load16_stream(Ku + (size_t)row * D);
      vraw[u] = load16_stream(Vu + (size_t)row * D);
    }
    st.template rows<U, LPR>(kraw, vraw, valid);
  }
  merge_groups_and_store<T, D, G, NWV>(st, smem, part_head0, head_stride);
}

// Two selections of every head in one launch (the r best and the r + e best clusters of the
// budgeted estimation zone): even workgroups take the first, odd ones the second.  Each
// leaves its ascending id list and count.
template <typename T, int D, int NT, int VPT, bool LDSK>
__global__ __launch_bounds__(NT) void select_two_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int mwords, int mc, uint32_t* __restrict__ bitmap, int r1, int rcap1, int32_t* __restrict__ ids1,
    int32_t* __restrict__ nsel1, int32_t* __restrict__ user_selected, int r2, int rcap2,
    int32_t* __restrict__ ids2, int32_t* __restrict__ nsel2, const T* __restrict__ vsum, float scale_log2) {
  extern __shared__ uint32_t dyn_keys[];
  const int bh = blockIdx.x >> 1;
  const bool second = blockIdx.x & 1;
  int ntok;
  select_core<T, D, NT, VPT, LDSK>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, second ? r2 : r1,
                                   second ? rcap2 : rcap1, mwords, mc, second ? r2 : r1, second ? ids2 : ids1,
                                   nullptr, nullptr, bitmap, second ? nsel2 : nsel1,
                                   second ? nullptr : user_selected, vsum, scale_log2, nullptr, 0, 0, bh,
                                   dyn_keys, nullptr, nullptr, 0, &ntok,
                                   SelView{m, 0, nullptr, nullptr, 2, nullptr, nullptr});
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void steady_kernel(const T* __restrict__ q,
                                                     const T* __restrict__ k_steady,
                                                     const T* __restrict__ v_steady, int Hkv, int p,
                                                     int p_stride, int chunks, int rows_per_chunk,
                                                     int slots, int slot0, float scale_log2,
                                                     float* __restrict__ part) {
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int unit = wg / chunks, chunk = wg - unit * chunks;
  const int b = unit / Hkv, h = unit - b * Hkv, Hq = Hkv * G;
  __shared__ float smem[4 * G * (D + 2)];
  const int bh0 = b * Hq + h * G;
  const int r0 = chunk * rows_per_chunk, r1 = min(p, r0 + rows_per_chunk);
  steady_rows_partial<T, D, G, 256>(q, k_steady, v_steady, unit, bh0, p_stride, r0, r1, scale_log2, smem,
                                    part + ((size_t)bh0 * slots + slot0 + chunk) * (D + 2),
                                    (size_t)slots * (D + 2));
}

// The meta-index pass with the steady-zone pieces as extra workgroups (few heads:
// neither fills the chip alone, and a launch less is a few microseconds less).
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void dense_steady_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const T* __restrict__ vsum,
    const int32_t* __restrict__ sizes, float* __restrict__ z, float* __restrict__ cn2part, int Hkv,
    int m, int mc, int chunks, int slots, int slot0, float scale_log2, float* __restrict__ part,
    int n_dense_wgs, const T* __restrict__ k_steady, const T* __restrict__ v_steady, int p,
    int p_stride, int steady_chunks, int steady_rows, int steady_slot0) {
  using Lds = DenseLds<T, D, G, 256>;
  constexpr size_t kSteadyBytes = sizeof(float) * 4 * G * (D + 2);
  __shared__ __attribute__((aligned(16))) char
      lds_raw[Lds::score_bytes > kSteadyBytes ? Lds::score_bytes : kSteadyBytes];
  const int Hq = Hkv * G;
  if ((int)blockIdx.x < n_dense_wgs) {
    const Lds lds(lds_raw);
    const int wg = xcd_logical_block(blockIdx.x, n_dense_wgs);
    const int unit = wg / chunks, chunk = wg - unit * chunks;
    const int b = unit / Hkv, h = unit - b * Hkv;
    const int bh0 = b * Hq + h * G;
    const int c0 = chunk * DENSE_ROWS, nrows = min(DENSE_ROWS, m - c0);
    const int32_t* su = sizes + (size_t)unit * mc + c0;
    dense_scores<T, D, G, 256, true>(q, C, su, z, unit, bh0, m, mc, c0, nrows, lds);
    __syncthreads();
    if (threadIdx.x == 0) cn2part[(size_t)unit * chunks + chunk] = dense_cn2(lds);
    dense_estimate<T, D, G, 256>(vsum, su, unit, m, mc, c0, nrows, scale_log2, lds,
                                 part + ((size_t)bh0 * slots + slot0 + chunk) * (D + 2),
                                 (size_t)slots * (D + 2));
    return;
  }
  const int wg = (int)blockIdx.x - n_dense_wgs;
  const int unit = wg / steady_chunks, chunk = wg - unit * steady_chunks;
  const int b = unit / Hkv, h = unit - b * Hkv;
  const int bh0 = b * Hq + h * G;
  const int r0 = chunk * steady_rows, r1 = min(p, r0 + steady_rows);
  steady_rows_partial<T, D, G, 256>(q, k_steady, v_steady, unit, bh0, p_stride, r0, r1, scale_log2,
                                    reinterpret_cast<float*>(lds_raw),
                                    part + ((size_t)bh0 * slots + steady_slot0 + chunk) * (D + 2),
                                    (size_t)slots * (D + 2));
}

// Work that does not depend on the selection, carried by the launches of the
// sliced selection: estimation ranges [est_first, est_first + n_est_wgs) over
// all units' ranges of NT clusters, then the steady-zone pieces.
struct SideWork {
  const int32_t* sizes;
  int est_rows, est_chunks, est_slot0, est_first, n_est_wgs;
  const void* k_steady;
  const void* v_steady;
  int p, p_stride, steady_chunks, steady_rows, steady_slot0;
};

template <typename T, int D, int G, int NT>
__device__ __forceinline__ void side_role(int wg, const SideWork& sw, const T* __restrict__ q,
                                          const float* __restrict__ z, const T* __restrict__ vsum,
                                          int Hq, int Hkv, int m, int mc, float scale_log2,
                                          float* __restrict__ part, int slots, char* lds_raw) {
  if (wg < sw.n_est_wgs) {
    // Estimation terms of sw.est_rows clusters of one unit for its G heads, as a
    // stream: every group of LPR lanes takes rows of value sums with their
    // scores (read back from z) and sizes and keeps an online-softmax state, the
    // cluster's score as the logit and its size as the multiplicity.
    constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64;
    constexpr int GROUPS = NWV * RPW, U = 4, UH = 4;
    static_assert(G <= LPR, "one lane per head's score");
    wg = xcd_logical_block(wg, sw.n_est_wgs) + sw.est_first;
    const int unit = wg / sw.est_chunks, chunk = wg - unit * sw.est_chunks;
    const int b = unit / Hkv, h = unit - b * Hkv;
    const int bh0 = b * Hq + h * G;
    const int c0 = chunk * sw.est_rows, nrows = min(sw.est_rows, m - c0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
    AttnState<T, D, G> st;
    st.reset();  // the queries are not needed: the scores are given
    const T* Vu = vsum + ((size_t)unit * mc + c0) * D + sub * EPC;
    // The range's scores and sizes are staged in LDS with coalesced loads (a
    // group's own 4-byte reads of them would be one memory request per row and
    // head); the value sums stream with the next pass's rows already in flight.
    float* zs = reinterpret_cast<float*>(lds_raw);              // [G][est_rows]
    float* ms = zs + (size_t)G * sw.est_rows;                   // [est_rows], the size as a float
    auto load_rows = [&](int i, uint4 (&dst)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) dst[u] = load16_stream(Vu + (size_t)min(i + u * GROUPS, nrows - 1) * D);
    };
    uint4 vnext[U];
    load_rows(grp, vnext);  // (grp may lie beyond a short range: the clamped rows get weight 0)
    for (int i = threadIdx.x; i < nrows; i += NT) {
      float zv[G];
#pragma unroll
      for (int g = 0; g < G; ++g) zv[g] = z[(size_t)(bh0 + g) * m + c0 + i];
      const int sz = sw.sizes[(size_t)unit * mc + c0 + i];
#pragma unroll
      for (int g = 0; g < G; ++g) zs[g * sw.est_rows + i] = zv[g] * scale_log2;
      ms[i] = (float)sz;
    }
    __syncthreads();
    for (int i = grp; i < nrows; i += GROUPS * U) {
      uint4 vraw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) vraw[u] = vnext[u];
      if (i + GROUPS * U < nrows) load_rows(i + GROUPS * U, vnext);
#pragma unroll
      for (int h0 = 0; h0 < U; h0 += UH) {  // UH rows per update of the state
        float sc[G][UH], mult[UH];
        uint4 vh[UH];
#pragma unroll
        for (int u = 0; u < UH; ++u) {
          const int ii = i + (h0 + u) * GROUPS;
          const int row = min(ii, nrows - 1);
          vh[u] = vraw[h0 + u];
          mult[u] = ms[row];
#pragma unroll
          for (int g = 0; g < G; ++g) sc[g][u] = ii < nrows ? zs[g * sw.est_rows + row] : -INFINITY;  // beyond: weight 0
        }
        st.template rows_given<UH>(sc, mult, vh);
      }
    }
    __syncthreads();  // the staged scores are read no more: the merge reuses the space
    merge_groups_and_store<T, D, G, NWV>(st, reinterpret_cast<float*>(lds_raw),
                                         part + ((size_t)bh0 * slots + sw.est_slot0 + chunk) * (D + 2),
                                         (size_t)slots * (D + 2));
    return;
  }
  wg -= sw.n_est_wgs;
  const int unit = wg / sw.steady_chunks, chunk = wg - unit * sw.steady_chunks;
  const int b = unit / Hkv, h = unit - b * Hkv;
  const int bh0 = b * Hq + h * G;
  const int r0 = chunk * sw.steady_rows, r1 = min(sw.p, r0 + sw.steady_rows);
  steady_rows_partial<T, D, G, NT>(q, static_cast<const T*>(sw.k_steady),
                                   static_cast<const T*>(sw.v_steady), unit, bh0, sw.p_stride, r0, r1,
                                   scale_log2, reinterpret_cast<float*>(lds_raw),
                                   part + ((size_t)bh0 * slots + sw.steady_slot0 + chunk) * (D + 2),
                                   (size_t)slots * (D + 2));
}

// Estimation terms of one range of sw.est_rows clusters of a unit for its G heads, from
// the scores an earlier launch left in z: the range's scores and sizes are staged in LDS
// with coalesced loads, turned into weights relative to the range's largest score (and
// the sum of size x weight), and the value sums then stream through with the weights read
// from LDS, the next pass's rows already in flight.  One partial per head.
template <typename T, int D, int G, int NT, int U = 4>
__device__ __forceinline__ void estimate_range(int wg, const SideWork& sw, const float* __restrict__ z,
                                               const T* __restrict__ vsum, int Hq, int Hkv, int m, int mc,
                                               float scale_log2, float* __restrict__ part, int slots,
                                               char* lds_raw) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, NWV = NT / 64;
  constexpr int GROUPS = NWV * RPW, ZG = (G + 3) / 4 * 4, STR = D + 2;
  wg = xcd_logical_block(wg, sw.n_est_wgs) + sw.est_first;
  const int unit = wg / sw.est_chunks, chunk = wg - unit * sw.est_chunks;
  const int b = unit / Hkv, h = unit - b * Hkv;
  const int bh0 = b * Hq + h * G;
  const int c0 = chunk * sw.est_rows, nrows = min(sw.est_rows, m - c0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  float* zw = reinterpret_cast<float*>(lds_raw);   // [est_rows][ZG]: scores in base-2 units, then weights
  float* ms = zw + (size_t)sw.est_rows * ZG;        // [est_rows]: the size as a float
  float* smem = zw;                                 // the last step reuses the space
  __shared__ float red[NWV][2 * G];
  const T* Vu = vsum + ((size_t)unit * mc + c0) * D + sub * EPC;
  auto load_rows = [&](int i, uint4 (&dst)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) dst[u] = load16_stream(Vu + (size_t)min(i + u * GROUPS, nrows - 1) * D);
  };
  uint4 vnext[U];
  load_rows(grp, vnext);  // (grp may lie beyond a short range: the clamped rows get weight 0)
  float mx[G];
#pragma unroll
  for (int g = 0; g < G; ++g) mx[g] = -INFINITY;
  for (int i = tid; i < nrows; i += NT) {
    float zv[G];
#pragma unroll
    for (int g = 0; g < G; ++g) zv[g] = z[(size_t)(bh0 + g) * m + c0 + i];
    const int sz = sw.sizes[(size_t)unit * mc + c0 + i];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float v = zv[g] * scale_log2;  // -inf for an empty cluster
      zw[i * ZG + g] = v;
      mx[g] = fmaxf(mx[g], v);
    }
    ms[i] = (float)sz;
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    mx[g] = wave_max(mx[g]);
    if (lane == 0) red[wave][g] = mx[g];
  }
  __syncthreads();
  float ref[G], ls[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = red[0][g];
#pragma unroll
    for (int w = 1; w < NWV; ++w) v = fmaxf(v, red[w][g]);
    mx[g] = v;
    ref[g] = v > -INFINITY ? v : 0.f;  // a range of empty clusters only: every weight is 0
    ls[g] = 0.f;
  }
  for (int i = tid; i < nrows; i += NT) {  // the entries this thread wrote itself
    const float sz = ms[i];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float w = exp2f(zw[i * ZG + g] - ref[g]);  // exp2(-inf) = 0
      zw[i * ZG + g] = w;
      ls[g] = fmaf(sz, w, ls[g]);
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    ls[g] = wave_sum_f(ls[g]);
    if (lane == 0) red[wave][G + g] = ls[g];
  }
  __syncthreads();
  float acc[G][EPC];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[g][e] = 0.f;
  for (int i = grp; i < nrows; i += GROUPS * U) {
    uint4 vraw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) vraw[u] = vnext[u];
    if (i + GROUPS * U < nrows) load_rows(i + GROUPS * U, vnext);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ii = i + u * GROUPS;
      const int row = min(ii, nrows - 1);
      float w[ZG], vf[EPC];
#pragma unroll
      for (int g4 = 0; g4 < ZG; g4 += 4) {
        const float4 t = *reinterpret_cast<const float4*>(&zw[row * ZG + g4]);
        w[g4] = t.x; w[g4 + 1] = t.y; w[g4 + 2] = t.z; w[g4 + 3] = t.w;
      }
      unpack<T>(vraw[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float wg_ = ii < nrows ? w[g] : 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[g][e] = fmaf(wg_, vf[e], acc[g][e]);
      }
    }
  }
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] += __shfl_xor(acc[g][e], off);
    }
  }
  __syncthreads();  // the weights are read no more: their space takes the waves' sums
  if (lane < LPR) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float* dst = smem + (size_t)(wave * G + g) * STR;
#pragma unroll
      for (int e = 0; e < EPC; ++e) dst[2 + sub * EPC + e] = acc[g][e];
    }
  }
  __syncthreads();
  float* part_head0 = part + ((size_t)bh0 * slots + sw.est_slot0 + chunk) * STR;
  for (int idx = tid; idx < G * STR; idx += NT) {
    const int g = idx / STR, e = idx - g * STR;
    float v = 0.f;
    if (e == 0) {
      float mxg = red[0][g];
#pragma unroll
      for (int w = 1; w < NWV; ++w) mxg = fmaxf(mxg, red[w][g]);
      v = mxg > -INFINITY ? mxg : kNegBig;  // no cluster: an empty partial
    } else if (e == 1) {
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += red[w][G + g];
    } else {
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += smem[(size_t)(w * G + g) * STR + e];
    }
    part_head0[(size_t)g * slots * STR + e] = v;
  }
}

// ----------------------------------------------------------------------------
// Few heads over many clusters: ranking a slice (and then the union of the
// slices' lists) is a chain of short dependent steps that leaves the memory
// system idle, so the two launches also carry the work that does not depend on
// the selection: the estimation terms of all clusters (from the scores of the
// first launch) and the steady zone.  The selecting workgroups have the lowest
// ids, so they are dispatched first.
// ----------------------------------------------------------------------------
template <typename T, int D, int G, int NT, int VPT>
__global__ __launch_bounds__(NT, G <= 4 ? 4 : 2) void slices_side_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot, int nslices, int slice_len,
    int32_t* __restrict__ slice_ids, float* __restrict__ slice_z, int n_select_wgs,
    const SideWork sw) {
  extern __shared__ __attribute__((aligned(16))) uint32_t dyn_keys[];  // a slice's keys, or the other roles' LDS
  if ((int)blockIdx.x < n_select_wgs) {
    const int bh = blockIdx.x / nslices, sl = blockIdx.x - bh * nslices;
    const int base = sl * slice_len, len = min(slice_len, m - base);
    int ntok;
    select_core<T, D, NT, VPT, true>(
        q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, r, mwords, mc, usel_stride, sel_ids, sel_pref,
        sel_row, bitmap, nsel_out, nullptr, vsum, scale_log2, part, slots, neg_slot, bh,
        dyn_keys, nullptr, nullptr, 0, &ntok,
        SelView{len, base, nullptr, nullptr, 1, slice_ids + ((size_t)bh * nslices + sl) * r,
                slice_z + ((size_t)bh * nslices + sl) * r});
    return;
  }
  side_role<T, D, G, NT>((int)blockIdx.x - n_select_wgs, sw, q, z, vsum, Hq, Hkv, m, mc, scale_log2, part,
                         slots, reinterpret_cast<char*>(dyn_keys));
}

// ----------------------------------------------------------------------------
// A cheap first stage for the slices.  The score pass left the largest score of
// every run of SCORE_TILE clusters.  Any value T that at least r of those maxima
// reach is a lower bound of the head's r-th largest score (r different clusters
// score at least T), so with the fp32 error bound `guard` below it, every
// cluster that the exact ranking could select scores at least T - guard.  T is
// the lower edge of the bucket (upper 16 key bits) in which the count of maxima,
// taken from the top, reaches r: one histogram sweep and a scan, no search.  A
// slice then only lists its clusters at or above T - guard, ascending, padded
// to r entries like the lists of the exact slice ranking.  Returns false, with
// nothing written, when the slice holds more than r such clusters (or no T
// exists); the caller then ranks the slice exactly.
// The buckets are the SEL_BINS ones below the bucket of |q| max|C|, an upper
// bound of every score.
// ----------------------------------------------------------------------------
template <typename T, int D, int NT, int VPT>
__device__ __forceinline__ bool filter_slice(const T* __restrict__ q, const float* __restrict__ z,
                                             const float* __restrict__ tile_max,
                                             const float* __restrict__ cn2part, int cn2_chunks,
                                             int unit, int bh, int m, int r, int base, int len,
                                             uint32_t* skeys, int32_t* __restrict__ ids_out,
                                             float* __restrict__ z_out) {
  constexpr int NW = NT / 64, TBL = VPT * NW;
  static_assert(TBL <= NT, "one table entry per thread");
  constexpr uint32_t kKeyNegInf = 0x007fffffu;  // order_key(-inf)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const float* zz = z + (size_t)bh * m + base;
  const int ntile = (m + SCORE_TILE - 1) / SCORE_TILE;
  const float* tm = tile_max + (size_t)bh * ntile;
  __shared__ int f_hist[SEL_BINS];
  __shared__ int f_scan[NW];
  __shared__ int f_tbl[TBL];
  __shared__ int f_sh[4];
  __shared__ float f_shf[2];

  // |q|^2 and max |C|^2 (the error bound and the bound of the scores) and the
  // first tile maxima: all loads are issued before any is waited for
  static_assert(D <= 128, "two query elements per lane");
  float gq[2] = {0.f, 0.f}, gc[4] = {0.f, 0.f, 0.f, 0.f};
  if (wave == NW - 1) {
#pragma unroll
    for (int j = 0; j < 2; ++j) gq[j] = to_f32(q[(size_t)bh * D + min(lane + 64 * j, D - 1)]);
#pragma unroll
    for (int j = 0; j < 4; ++j) gc[j] = cn2part[(size_t)unit * cn2_chunks + min(lane + 64 * j, cn2_chunks - 1)];
#pragma unroll
    for (int j = 0; j < 2; ++j) gq[j] = lane + 64 * j < D ? gq[j] : 0.f;  // (a repeated maximum is harmless)
  }
  float tm0[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) tm0[u] = tm[min(u * NT + tid, ntile - 1)];  // clamped: repeats are masked below
  // the slice's keys into LDS
  const int nk = (len + NT - 1) / NT;  // <= VPT
  constexpr int KB = 16;
  for (int k0 = 0; k0 < nk; k0 += KB) {
    float v[KB];
#pragma unroll
    for (int u = 0; u < KB; ++u) v[u] = zz[min((k0 + u) * NT + tid, len - 1)];
#pragma unroll
    for (int u = 0; u < KB; ++u)
      if (k0 + u < nk)
        skeys[(k0 + u) * NT + tid] = order_key(((k0 + u) * NT + tid < len ? v[u] : -INFINITY) + 0.0f);
  }
  if (wave == NW - 1) {
    float qn2 = gq[0] * gq[0] + gq[1] * gq[1];
    float c2 = fmaxf(fmaxf(gc[0], gc[1]), fmaxf(gc[2], gc[3]));
    for (int i = lane + 256; i < cn2_chunks; i += 64) c2 = fmaxf(c2, cn2part[(size_t)unit * cn2_chunks + i]);
    qn2 = wave_sum_f(qn2);
    c2 = wave_max(c2);
    const float qc = sqrtf(qn2) * sqrtf(c2);
    if (lane == 0) {
      f_shf[0] = 2.0f * 48.f * 5.9604645e-8f * qc;  // as in the exact ranking
      f_shf[1] = qc * 1.001f;
    }
  }
  for (int i = tid; i < SEL_BINS; i += NT) f_hist[i] = 0;
  if (tid < TBL) f_tbl[tid] = 0;
  __syncthreads();
  const float guard = f_shf[0];
  const uint32_t top16 = order_key(f_shf[1] + 0.0f) >> 16;
  const uint32_t lo16 = top16 >= (uint32_t)(SEL_BINS - 1) ? top16 - (SEL_BINS - 1) : 0u;
  // histogram of the head's tile maxima
  for (int i0 = 0; i0 < ntile; i0 += NT * 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = i0 == 0 ? tm0[u] : tm[min(i0 + u * NT + tid, ntile - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t ky = order_key((i0 + u * NT + tid < ntile ? v[u] : -INFINITY) + 0.0f);
      if (ky > kKeyNegInf) {
        uint32_t b16 = ky >> 16;
        b16 = b16 > top16 ? top16 : b16;  // cannot happen for finite inputs; keeps the index in range
        atomicAdd(&f_hist[b16 > lo16 ? b16 - lo16 : 0u], 1);
      }
    }
  }
  __syncthreads();
  constexpr int PER = SEL_BINS / NT;
  static_assert(PER >= 1 && PER * NT == SEL_BINS, "bins per thread");
  int mine[PER], sum = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    mine[j] = f_hist[SEL_BINS - 1 - (tid * PER + j)];  // thread 0 holds the top bins
    sum += mine[j];
  }
  if (tid == 0) f_sh[0] = -1;
  int tot;
  int above = block_excl_scan<NT>(sum, f_scan, tot);  // also orders the store to f_sh[0] before the ones below
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (above < r && above + mine[j] >= r) f_sh[0] = SEL_BINS - 1 - (tid * PER + j);  // at most one (thread, j)
    above += mine[j];
  }
  __syncthreads();
  const int bsel = f_sh[0];
  if (bsel <= 0) return false;  // fewer than r maxima, or the bound lies in the catch-all bucket
  const float t_edge = key_to_float((lo16 + (uint32_t)bsel) << 16);
  uint32_t kt = order_key((t_edge - guard) + 0.0f);
  kt = kt > kKeyNegInf + 3u ? kt - 2u : kKeyNegInf + 1u;  // two ulps for the rounding of the subtraction

  // the slice's clusters at or above the bound, in ascending order
  for (int k = 0; k < nk; ++k) {
    const uint64_t mk = __ballot(skeys[k * NT + tid] >= kt);
    if (lane == 0) f_tbl[k * NW + wave] = __popcll(mk);
  }
  __syncthreads();
  int cnt;
  const int cbase = block_excl_scan<NT>(tid < TBL ? f_tbl[tid] : 0, f_scan, cnt);
  if (cnt > r) return false;
  __syncthreads();
  if (tid < TBL) f_tbl[tid] = cbase;
  __syncthreads();
  for (int k = 0; k < nk; ++k) {
    const uint32_t ky = skeys[k * NT + tid];
    const bool on = ky >= kt;
    const uint64_t mk = __ballot(on);
    if (on) {
      const int pos = f_tbl[k * NW + wave] + __popcll(mk & lt_mask);
      ids_out[pos] = base + k * NT + tid;
      z_out[pos] = key_to_float(ky);
    }
  }
  for (int i = cnt + tid; i < r; i += NT) {
    ids_out[i] = -1;
    z_out[i] = -INFINITY;
  }
  return true;
}

template <typename T, int D, int G, int NT, int VPT>
__global__ __launch_bounds__(NT, G <= 4 ? 4 : 2) void filter_side_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot, int nslices, int slice_len,
    int32_t* __restrict__ slice_ids, float* __restrict__ slice_z, int n_select_wgs,
    const SideWork sw, const float* __restrict__ tile_max) {
  extern __shared__ __attribute__((aligned(16))) uint32_t dyn_keys[];  // a slice's keys, or the other roles' LDS
  if ((int)blockIdx.x < n_select_wgs) {
    const int bh = blockIdx.x / nslices, sl = blockIdx.x - bh * nslices;
    const int base = sl * slice_len, len = min(slice_len, m - base);
    const int b = bh / Hq, hq = bh - b * Hq;
    const int unit = b * Hkv + hq / (Hq / Hkv);
    int32_t* ids_out = slice_ids + ((size_t)bh * nslices + sl) * r;
    float* z_out = slice_z + ((size_t)bh * nslices + sl) * r;
    if (filter_slice<T, D, NT, VPT>(q, z, tile_max, cn2part, cn2_chunks, unit, bh, m, r, base, len,
                                    dyn_keys, ids_out, z_out))
      return;
    __syncthreads();
    int ntok;
    select_core<T, D, NT, VPT, true>(
        q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, r, mwords, mc, usel_stride, sel_ids, sel_pref,
        sel_row, bitmap, nsel_out, nullptr, vsum, scale_log2, part, slots, neg_slot, bh,
        dyn_keys, nullptr, nullptr, 0, &ntok, SelView{len, base, nullptr, nullptr, 1, ids_out, z_out});
    return;
  }
  side_role<T, D, G, NT>((int)blockIdx.x - n_select_wgs, sw, q, z, vsum, Hq, Hkv, m, mc, scale_log2, part,
                         slots, reinterpret_cast<char*>(dyn_keys));
}

template <typename T, int D, int G, int NT, int VPT>
__global__ __launch_bounds__(NT, G <= 4 ? 4 : 2) void combine_side_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out,
    int32_t* __restrict__ user_selected, const T* __restrict__ vsum, float scale_log2,
    float* __restrict__ part, int slots, int neg_slot, int nslices,
    const int32_t* __restrict__ slice_ids, const float* __restrict__ slice_z, int n_select_wgs,
    const SideWork sw) {
  extern __shared__ __attribute__((aligned(16))) uint32_t dyn_keys[];
  if ((int)blockIdx.x < n_select_wgs) {
    // A slice's list is ascending and padded with -1 to r entries, and the
    // slices are ascending id ranges: read one after the other, with the padding
    // as holes, the lists are one ascending id map of nslices * r positions.
    const int bh = blockIdx.x;
    int ntok;
    select_core<T, D, NT, VPT, true>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc,
                                     usel_stride, sel_ids, sel_pref, sel_row, bitmap,
                                     nsel_out, user_selected, vsum, scale_log2, part, slots, neg_slot,
                                     bh, dyn_keys, nullptr, nullptr, 0, &ntok,
                                     SelView{nslices * r, 0, slice_ids + (size_t)bh * nslices * r,
                                             slice_z + (size_t)bh * nslices * r, 2, nullptr, nullptr});
    return;
  }
  side_role<T, D, G, NT>((int)blockIdx.x - n_select_wgs, sw, q, z, vsum, Hq, Hkv, m, mc, scale_log2, part,
                         slots, reinterpret_cast<char*>(dyn_keys));
}

// ----------------------------------------------------------------------------
// What a selecting workgroup leaves for the retrieval launch.  A head's selected
// tokens (ntok of them, in the order of its ascending cluster list) are cut into
// nch = ceil(ntok / chunk_tokens) equal token ranges; range c starts at token
// c * ct (ct = ceil(ntok / nch)), which lies in cluster chunk_first[c] of the
// head's list.  The ranges of all heads go onto ONE work list (a head's ranges
// are consecutive entries, claimed with one atomic), so the retrieval launch has
// as many equal pieces as there are tokens, however unevenly the heads share
// them (heavy-tailed cluster sizes: one head can hold ten times the mean).
// The list holds wmain entries plus one spare entry per head: a head that finds
// the list full takes its spare entry and retrieves as ONE range.  Entries not
// claimed stay -1 (an earlier launch of the step fills the list and zeroes the
// counter).  An entry is head * 256 + range.
// ----------------------------------------------------------------------------
constexpr int LIST_MAX_CHUNKS = 255;  // ranges per head
struct ListOut {
  int32_t* chunk_first;  // [heads][LIST_MAX_CHUNKS + 1]
  int4* head_info;       // [heads]: first list entry, ranges, tokens per range, tokens
  int32_t* work;         // [wmain + heads]
  int32_t* work_count;   // entries claimed so far (may run past wmain)
  int wmain, chunk_tokens;
};

// pref: the head's running token counts, nsel + 1 entries (LDS or global).  All
// NT threads call this.
template <int NT>
__device__ __forceinline__ void publish_token_ranges(int bh, int nsel, int ntok, const int* pref,
                                                     const ListOut& lo) {
  __shared__ int s_pub[3];
  if (threadIdx.x == 0) {
    int nch = ntok > 0 ? min((ntok + lo.chunk_tokens - 1) / lo.chunk_tokens, LIST_MAX_CHUNKS) : 0;
    int base = 0;
    if (nch > 0) {
      base = atomicAdd(lo.work_count, nch);
      if (base + nch > lo.wmain) {  // the list is full: the head's spare entry, one range
        base = lo.wmain + bh;
        nch = 1;
      }
    }
    const int ct = nch > 0 ? (ntok + nch - 1) / nch : 0;
    s_pub[0] = base;
    s_pub[1] = nch;
    s_pub[2] = ct;
    lo.head_info[bh] = make_int4(base, nch, ct, ntok);
  }
  __syncthreads();
  const int base = s_pub[0], nch = s_pub[1], ct = s_pub[2];
  int32_t* cf = lo.chunk_first + (size_t)bh * (LIST_MAX_CHUNKS + 1);
  if (nch == 0) return;
  for (int c = threadIdx.x; c <= nch; c += NT) {
    const long long t = (long long)c * ct;
    int a = 0, e = nsel;  // largest a in [0, nsel) with pref[a] <= t
    while (e - a > 1) {
      const int mid = (a + e) >> 1;
      if (pref[mid] <= t) a = mid; else e = mid;
    }
    cf[c] = a;
    if (c < nch) lo.work[base + c] = bh * 256 + c;
  }
}

// ----------------------------------------------------------------------------
// Few heads over many clusters (16384 < m <= FILT_NT * FILT_MAX_SWEEPS) in three
// launches and a merge:
//   1. scores of all clusters (with the largest score of every run of SCORE_TILE
//      clusters) and, as extra workgroups, the steady zone;
//   2. one workgroup per head selects; beside them, workgroups that do not depend
//      on the selection stream the value sums of ALL clusters (estimation terms),
//      so the memory system is busy while the selection's chain of short
//      dependent steps runs;
//   3. the selected clusters' tokens, cut into equal token ranges per workgroup.
// Selection of a head, one workgroup: the table of tile maxima gives a lower
// bound T of the head's r-th largest score (at least r maxima reach T, so r
// different clusters score at least T): one histogram sweep over m / 16 values
// and a scan.  With the fp32 error bound `guard`, every cluster the exact ranking
// could select scores at least T - guard.  Only tiles whose maximum reaches that
// bound can hold such a cluster: they are listed from the table, their scores
// read (16 per tile) and the passing ones marked in an LDS bitmap of all
// clusters, one atomic per tile; a scan of the bitmap gives the passing clusters
// in ascending order (about 1.1 r on clustered data), their scores are read
// again in that order, and the exact ranking (select_core: fp64 re-scoring
// inside the guard band, ties to the lower id) runs on that list.  The workgroup then leaves everything the retrieval launch
// needs: ids, first rows, running token counts, the first cluster of every token
// range, and the selected clusters' estimation terms with a minus sign.  When no
// bound exists (fewer than r tiles) or more than FILT_CAP clusters pass (many
// equal scores), the head is ranked by the streaming selection instead.
// ----------------------------------------------------------------------------
constexpr int FILT_NT = 512;
constexpr int FILT_CAP = 2048;         // clusters that pass the filter, kept in LDS
constexpr int FILT_VPT = FILT_CAP / FILT_NT;
constexpr int FILT_MAX_SWEEPS = 256;   // of FILT_NT scores each
// LDS of the selecting role: ids and scores of the clusters that pass, the bitmap of all
// clusters (whose space the histogram uses before it and the exact ranking's keys after it),
// the selected ids, and FILT_CAP spare words
constexpr size_t FILT_LDS = sizeof(int) * (4 * (size_t)FILT_CAP + (size_t)FILT_MAX_SWEEPS * FILT_NT / 32);
// largest r the filtered selection is used for: about 1.1 r clusters pass on clustered data
inline int filtered_max_r() { return (FILT_CAP - 64) * 4 / 5; }

template <typename T, int D, int NT>
__device__ __forceinline__ void select_filtered(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out, int32_t* __restrict__ user_selected, const T* __restrict__ vsum,
    float scale_log2, float* __restrict__ part, int slots, int neg_slot, int bh,
    const float* __restrict__ tile_max, const ListOut lo, char* dyn) {
  constexpr int NW = NT / 64;
  static_assert(NT == FILT_NT, "LDS layout");
  static_assert(SEL_BINS * sizeof(int) <= FILT_CAP * sizeof(int), "the histogram borrows the key region");
  static_assert(FILT_MAX_SWEEPS * NT / 32 >= FILT_CAP, "the exact ranking's keys use the bitmap's space");
  constexpr uint32_t kKeyNegInf = 0x007fffffu;  // order_key(-inf)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = bh / Hq, hq = bh - b * Hq;
  const int unit = b * Hkv + hq / (Hq / Hkv);
  const float* zz = z + (size_t)bh * m;
  const int ntile = (m + SCORE_TILE - 1) / SCORE_TILE;
  const float* tm = tile_max + (size_t)bh * ntile;
  int* cand_id = reinterpret_cast<int*>(dyn);
  float* cand_z = reinterpret_cast<float*>(dyn) + FILT_CAP;
  uint32_t* skeys = reinterpret_cast<uint32_t*>(dyn) + 2 * FILT_CAP;
  int* f_hist = reinterpret_cast<int*>(skeys);            // free until the exact ranking loads its keys
  uint32_t* fbits = reinterpret_cast<uint32_t*>(dyn) + 2 * FILT_CAP;  // bitmap of the clusters that pass
  int32_t* s_ids = reinterpret_cast<int32_t*>(dyn) + 2 * FILT_CAP + FILT_MAX_SWEEPS * NT / 32;
  __shared__ int f_scan[NW];
  __shared__ int f_sh[4];
  __shared__ float f_shf[2];
  uint32_t* trace = bitmap + (size_t)bh * mwords;
  (void)trace;
  WAVE_STAMP(trace, 0);

  // |q|^2 and max |C|^2 (error bound; bound of every score): loads first, reduced later
  static_assert(D <= 128, "two query elements per lane");
  float gq[2] = {0.f, 0.f}, gc[4] = {0.f, 0.f, 0.f, 0.f};
  if (wave == NW - 1) {
#pragma unroll
    for (int j = 0; j < 2; ++j) gq[j] = to_f32(q[(size_t)bh * D + min(lane + 64 * j, D - 1)]);
#pragma unroll
    for (int j = 0; j < 4; ++j) gc[j] = cn2part[(size_t)unit * cn2_chunks + min(lane + 64 * j, cn2_chunks - 1)];
#pragma unroll
    for (int j = 0; j < 2; ++j) gq[j] = lane + 64 * j < D ? gq[j] : 0.f;
  }
  // the head's tile maxima stay in registers: first for the histogram, then to pick the tiles
  // that can hold a cluster at or above the bound
  constexpr int TMV = FILT_MAX_SWEEPS * NT / SCORE_TILE / NT;  // tile maxima per thread at the largest m
  float tmv[TMV];
#pragma unroll
  for (int u = 0; u < TMV; ++u) tmv[u] = tm[min(u * NT + tid, ntile - 1)];
  if (wave == NW - 1) {
    float qn2 = gq[0] * gq[0] + gq[1] * gq[1];
    float c2 = fmaxf(fmaxf(gc[0], gc[1]), fmaxf(gc[2], gc[3]));
    for (int i = lane + 256; i < cn2_chunks; i += 64) c2 = fmaxf(c2, cn2part[(size_t)unit * cn2_chunks + i]);
    qn2 = wave_sum_f(qn2);
    c2 = wave_max(c2);
    const float qc = sqrtf(qn2) * sqrtf(c2);
    if (lane == 0) {
      f_shf[0] = 2.0f * 48.f * 5.9604645e-8f * qc;  // as in the exact ranking
      f_shf[1] = qc * 1.001f;
    }
  }
  for (int i = tid; i < SEL_BINS; i += NT) f_hist[i] = 0;
  if (tid == 0) f_sh[1] = f_sh[2] = 0;
  __syncthreads();
  const float guard = f_shf[0];
  const uint32_t top16 = order_key(f_shf[1] + 0.0f) >> 16;
  const uint32_t lo16 = top16 >= (uint32_t)(SEL_BINS - 1) ? top16 - (SEL_BINS - 1) : 0u;
  uint32_t tkey[TMV];
#pragma unroll
  for (int u = 0; u < TMV; ++u) {
    tkey[u] = order_key((u * NT + tid < ntile ? tmv[u] : -INFINITY) + 0.0f);
    if (tkey[u] > kKeyNegInf) {
      uint32_t b16 = tkey[u] >> 16;
      b16 = b16 > top16 ? top16 : b16;  // cannot happen for finite inputs; keeps the index in range
      atomicAdd(&f_hist[b16 > lo16 ? b16 - lo16 : 0u], 1);
    }
  }
  __syncthreads();
  constexpr int PER = SEL_BINS / NT;
  static_assert(PER >= 1 && PER * NT == SEL_BINS, "bins per thread");
  int hmine[PER], hsum = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    hmine[j] = f_hist[SEL_BINS - 1 - (tid * PER + j)];  // thread 0 holds the top bins
    hsum += hmine[j];
  }
  if (tid == 0) f_sh[0] = -1;
  int htot;
  int above = block_excl_scan<NT>(hsum, f_scan, htot);  // its barriers order the store to f_sh[0] first
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (above < r && above + hmine[j] >= r) f_sh[0] = SEL_BINS - 1 - (tid * PER + j);  // at most one (thread, j)
    above += hmine[j];
  }
  __syncthreads();
  const int bsel = f_sh[0];
  WAVE_STAMP(trace, 1);
  uint32_t kt = kKeyNegInf + 1u;  // no bound: every non-empty cluster passes
  if (bsel > 0) {
    const float t_edge = key_to_float((lo16 + (uint32_t)bsel) << 16);
    kt = order_key((t_edge - guard) + 0.0f);
    kt = kt > kKeyNegInf + 3u ? kt - 2u : kKeyNegInf + 1u;  // two ulps for the rounding of the subtraction
  }

  // Tiles whose maximum reaches the bound (only they hold clusters at or above it), as an
  // unordered list in LDS; their scores then set bits in a bitmap of all clusters, which
  // yields the passing clusters in ascending order.  More than FILT_CAP tiles pass only if
  // more than FILT_CAP clusters do.
  constexpr int BM_WORDS = FILT_MAX_SWEEPS * NT / 32, BM_PER = BM_WORDS / NT;
  int* tile_list = cand_id;  // free until the passing clusters are listed
  for (int i = tid; i < BM_WORDS; i += NT) fbits[i] = 0u;  // (the histogram, in the same space, is dead)
  {
    // (one LDS atomic per wave: hundreds of atomics on one address would run one after the other)
    int nmine = 0;
#pragma unroll
    for (int u = 0; u < TMV; ++u) nmine += tkey[u] >= kt ? 1 : 0;
    int base = wave_excl_scan_alloc(nmine, &f_sh[1]);
#pragma unroll
    for (int u = 0; u < TMV; ++u)
      if (tkey[u] >= kt) {
        if (base < FILT_CAP) tile_list[base] = u * NT + tid;
        ++base;
      }
  }
  __syncthreads();
  WAVE_STAMP(trace, 6);
  const int ntl = f_sh[1];
  const bool aligned = (m & 3) == 0;  // then every head's scores start at a 16-byte boundary
  if (ntl <= FILT_CAP) {
    constexpr int TB = 2;  // tiles in flight per thread
    for (int e0 = 0; e0 < ntl; e0 += TB * NT) {
      float sc[TB][SCORE_TILE];
      int t16[TB];
#pragma unroll
      for (int u = 0; u < TB; ++u) {
        t16[u] = SCORE_TILE * tile_list[min(e0 + u * NT + tid, ntl - 1)];
        if (aligned) {
#pragma unroll
          for (int j4 = 0; j4 < SCORE_TILE / 4; ++j4) {
            // (the last tile of a head may be short: m is a multiple of 4, so whole float4s)
            const float4 v = *reinterpret_cast<const float4*>(zz + min(t16[u] + 4 * j4, m - 4));
            sc[u][4 * j4] = v.x; sc[u][4 * j4 + 1] = v.y; sc[u][4 * j4 + 2] = v.z; sc[u][4 * j4 + 3] = v.w;
          }
        } else {
#pragma unroll
          for (int j = 0; j < SCORE_TILE; ++j) sc[u][j] = zz[min(t16[u] + j, m - 1)];
        }
      }
      // a tile's 16 pass bits are half a bitmap word: one LDS atomic per tile
      static_assert(SCORE_TILE == 16, "a tile is half a bitmap word");
#pragma unroll
      for (int u = 0; u < TB; ++u) {
        uint32_t pm = 0u;  // bit j: score j of tile u passes
        if (e0 + u * NT + tid < ntl) {
#pragma unroll
          for (int j = 0; j < SCORE_TILE; ++j)
            if (t16[u] + j < m && order_key(sc[u][j] + 0.0f) >= kt) pm |= 1u << j;
        }
        if (pm) atomicOr(&fbits[t16[u] >> 5], pm << (t16[u] & 31));
      }
    }
  }
  __syncthreads();
  WAVE_STAMP(trace, 7);
  uint32_t words[BM_PER];
  int tsum = 0;
#pragma unroll
  for (int j = 0; j < BM_PER; ++j) {
    words[j] = fbits[BM_PER * tid + j];
    tsum += __popc(words[j]);
  }
  int cnt;
  int tbase = block_excl_scan<NT>(tsum, f_scan, cnt);
  if (ntl > FILT_CAP) cnt = FILT_CAP + 1;  // too many tiles pass: ranked by the streaming selection
  WAVE_STAMP(trace, 2);

  int nsel, ntok;
  int* s_pref = reinterpret_cast<int*>(cand_z);  // both lists are dead once the ids are out
  int* s_row = reinterpret_cast<int*>(skeys);
  if (cnt <= FILT_CAP) {
#pragma unroll
    for (int j = 0; j < BM_PER; ++j) {
      uint32_t w = words[j];
      while (w) {
        const int bit = __ffs(w) - 1;
        w &= w - 1;
        cand_id[tbase++] = 32 * (BM_PER * tid + j) + bit;
      }
    }
    __syncthreads();  // (also: every thread has read its bitmap words; the key region is free)
    // the listed clusters' scores, read again in list order (four requests in flight per thread)
    static_assert(FILT_CAP == 4 * NT, "four candidates per thread");
    {
      float zv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) zv[u] = zz[cand_id[min(u * NT + tid, cnt - 1)]];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (u * NT + tid < cnt) cand_z[u * NT + tid] = zv[u] + 0.0f;
    }
    __syncthreads();
    WAVE_STAMP(trace, 3);
    nsel = select_core<T, D, NT, FILT_VPT, true>(
        q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc, usel_stride, sel_ids, sel_pref,
        sel_row, bitmap, nsel_out, user_selected, vsum, scale_log2, part, slots, neg_slot, bh, skeys,
        s_pref, s_row, FILT_CAP - 1, &ntok,
        SelView{cnt, 0, cand_id, cand_z, 0, nullptr, nullptr, s_ids, 1, guard});
    __syncthreads();
    WAVE_STAMP(trace, 4);
  } else {
    select_streaming<T, D, NT>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc,
                               usel_stride, sel_ids, sel_pref, sel_row, bitmap, nsel_out, user_selected,
                               vsum, scale_log2, part, slots, neg_slot, bh, 0);
    __syncthreads();
    const int32_t* pref = sel_pref + (size_t)bh * (rcap + 1);
    nsel = nsel_out[bh];
    for (int i = tid; i <= nsel && i < FILT_CAP; i += NT) s_pref[i] = pref[i];
    ntok = pref[nsel];
    __syncthreads();
  }
  publish_token_ranges<NT>(bh, nsel, ntok, s_pref, lo);
  WAVE_STAMP(trace, 5);
}

// Selection of a head when its clusters' keys fit in LDS (m <= 16384): the exact ranking on
// all of them, then the lists for the retrieval launch.  dyn: keys, then the staged running
// token counts, first rows and ids of up to `stage` selected clusters.
template <typename T, int D, int NT>
__device__ __forceinline__ void select_direct(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out, int32_t* __restrict__ user_selected, const T* __restrict__ vsum,
    float scale_log2, float* __restrict__ part, int slots, int neg_slot, int bh, int stage,
    const ListOut lo, char* dyn) {
  uint32_t* skeys = reinterpret_cast<uint32_t*>(dyn);
  int* s_pref = reinterpret_cast<int*>(skeys + (size_t)NT * ((m + NT - 1) / NT));
  int* s_row = s_pref + stage + 1;
  int32_t* s_ids = s_row + stage;
  int ntok;
  const int nsel = select_core<T, D, NT, 64, true>(
      q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc, usel_stride, sel_ids, sel_pref,
      sel_row, bitmap, nsel_out, user_selected, vsum, scale_log2, part, slots, neg_slot, bh, skeys, s_pref,
      s_row, stage, &ntok, SelView{m, 0, nullptr, nullptr, 0, nullptr, nullptr, s_ids, 1});
  __syncthreads();
  // (more selected clusters than are staged: the running token counts are read from memory)
  const int* pref = nsel < stage ? s_pref : sel_pref + (size_t)bh * (rcap + 1);
  publish_token_ranges<NT>(bh, nsel, ntok, pref, lo);
}

// Threads of a selecting workgroup when the keys fit in LDS (many heads): small workgroups, so
// that more heads' chains of short dependent steps are in flight per CU; a thread holds at most
// 64 keys' marks.
inline int select_direct_threads(int m) { return m <= 64 * 128 ? 128 : 256; }
inline size_t select_direct_lds(int m, int stage) {
  const int nt = select_direct_threads(m);
  return sizeof(uint32_t) * nt * (size_t)((m + nt - 1) / nt) + sizeof(int) * (3 * (size_t)stage + 1);
}

// One workgroup per head selects (FILTERED: through the tile maxima, for more clusters than
// fit in LDS); beside them, workgroups that do not depend on the selection take the
// estimation ranges of all clusters.
template <typename T, int D, int G, int NT, bool FILTERED>
__global__ __launch_bounds__(NT, (G <= 4 || !FILTERED) ? 4 : 2) void select_estimate_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int mc, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap,
    int32_t* __restrict__ nsel_out, int32_t* __restrict__ user_selected, const T* __restrict__ vsum,
    float scale_log2, float* __restrict__ part, int slots, int neg_slot,
    const float* __restrict__ tile_max, const ListOut lo, int stage, int n_select_wgs,
    const SideWork sw) {
  extern __shared__ __attribute__((aligned(16))) uint32_t dyn_keys[];
  // FILTERED (few heads, all workgroups resident at once): the selecting workgroups come
  // first.  Otherwise the two kinds alternate in proportion, so that at any time some
  // workgroups stream value sums while others run their selection's short dependent steps.
  const int total = gridDim.x, b = blockIdx.x;
  const int sel_before = FILTERED ? min(b, n_select_wgs) : (int)((long long)b * n_select_wgs / total);
  const bool is_select = FILTERED ? b < n_select_wgs
                                  : (int)((long long)(b + 1) * n_select_wgs / total) > sel_before;
  if (is_select) {
    if constexpr (FILTERED)
      select_filtered<T, D, NT>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc,
                                usel_stride, sel_ids, sel_pref, sel_row, bitmap, nsel_out, user_selected,
                                vsum, scale_log2, part, slots, neg_slot, sel_before, tile_max, lo,
                                reinterpret_cast<char*>(dyn_keys));
    else
      select_direct<T, D, NT>(q, C, offsets, z, cn2part, cn2_chunks, Hq, Hkv, m, r, rcap, mwords, mc,
                              usel_stride, sel_ids, sel_pref, sel_row, bitmap, nsel_out, user_selected,
                              vsum, scale_log2, part, slots, neg_slot, sel_before, stage, lo,
                              reinterpret_cast<char*>(dyn_keys));
    return;
  }
  if (b - sel_before >= sw.n_est_wgs) {
    // the steady-zone pieces (rows shared by the G heads of a KV head, read once per KV head)
    const int wg = b - sel_before - sw.n_est_wgs;
    const int unit = wg / sw.steady_chunks, chunk = wg - unit * sw.steady_chunks;
    const int bq = unit / Hkv, h = unit - bq * Hkv;
    const int bh0 = bq * Hq + h * G;
    const int r0 = chunk * sw.steady_rows, r1 = min(sw.p, r0 + sw.steady_rows);
    // (more than 4 heads at once would cost the launch its occupancy: the rows are read a
    // second time, from cache, for the heads beyond the fourth)
    constexpr int G1 = G <= 4 ? G : 4;
    float* smem = reinterpret_cast<float*>(dyn_keys);
    steady_rows_partial<T, D, G1, NT>(q, static_cast<const T*>(sw.k_steady), static_cast<const T*>(sw.v_steady),
                                      unit, bh0, sw.p_stride, r0, r1, scale_log2, smem,
                                      part + ((size_t)bh0 * slots + sw.steady_slot0 + chunk) * (D + 2),
                                      (size_t)slots * (D + 2));
    if constexpr (G > 4) {
      __syncthreads();
      steady_rows_partial<T, D, G - 4, NT>(q, static_cast<const T*>(sw.k_steady),
                                           static_cast<const T*>(sw.v_steady), unit, bh0 + 4, sw.p_stride, r0, r1,
                                           scale_log2, smem,
                                           part + ((size_t)(bh0 + 4) * slots + sw.steady_slot0 + chunk) * (D + 2),
                                           (size_t)slots * (D + 2));
    }
    return;
  }
#ifdef WAVE_TRACE
  const int te = b - sel_before;
  uint32_t* tbuf = bitmap + (size_t)(te % n_select_wgs) * mwords;
  WAVE_STAMP(tbuf, 32 + 2 * (te / n_select_wgs));
#endif
  // (small workgroups: twice the rows in flight per lane group)
  estimate_range<T, D, G, NT, (NT <= 256 && G <= 4 ? 8 : 4)>(b - sel_before, sw, z, vsum, Hq, Hkv, m, mc, scale_log2,
                                                             part, slots, reinterpret_cast<char*>(dyn_keys));
#ifdef WAVE_TRACE
  WAVE_STAMP(tbuf, 33 + 2 * (te / n_select_wgs));
#endif
}

// The scores with the steady-zone pieces as extra workgroups.
template <typename T, int D, int G>
__global__ __launch_bounds__(256, 4) void score_steady_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ sizes,
    float* __restrict__ z, float* __restrict__ cn2part, int Hkv, int m, int mc, int chunks,
    float* __restrict__ tile_max, int n_score_wgs, const T* __restrict__ k_steady,
    const T* __restrict__ v_steady, int p, int p_stride, int steady_chunks, int steady_rows, int slots,
    int steady_slot0, float scale_log2, float* __restrict__ part, int32_t* __restrict__ work,
    int32_t* __restrict__ work_count, int wtotal) {
  using Lds = DenseLds<T, D, G, 256>;
  constexpr size_t kSteadyBytes = sizeof(float) * 4 * G * (D + 2);
  __shared__ __attribute__((aligned(16))) char
      lds_raw[Lds::score_bytes > kSteadyBytes ? Lds::score_bytes : kSteadyBytes];
  const int Hq = Hkv * G;
  // the retrieval work list of this step starts empty (the next launch fills it)
  for (int i = blockIdx.x * 256 + threadIdx.x; i < wtotal; i += gridDim.x * 256) work[i] = -1;
  if (blockIdx.x == 0 && threadIdx.x == 0 && work_count) *work_count = 0;
  if ((int)blockIdx.x < n_score_wgs) {
    const Lds lds(lds_raw);
    const int wg = xcd_logical_block(blockIdx.x, n_score_wgs);
    const int unit = wg / chunks, chunk = wg - unit * chunks;
    const int b = unit / Hkv, h = unit - b * Hkv;
    const int bh0 = b * Hq + h * G;
    const int c0 = chunk * DENSE_ROWS, nrows = min(DENSE_ROWS, m - c0);
    dense_scores<T, D, G, 256, true>(q, C, sizes + (size_t)unit * mc + c0, z, unit, bh0, m, mc, c0, nrows, lds,
                                     sizeof(T) == 2 ? tile_max : nullptr);
    __syncthreads();
    if (threadIdx.x == 0) cn2part[(size_t)unit * chunks + chunk] = dense_cn2(lds);
    if (sizeof(T) != 2 && tile_max) {  // (the bf16 pass writes the tile maxima tile by tile)
      constexpr int TPC = DENSE_ROWS / SCORE_TILE, ZG = Lds::ZG;
      static_assert(TPC * G <= 256, "one thread per (tile, head)");
      const int t = threadIdx.x % TPC, g = threadIdx.x / TPC;
      if (g < G && SCORE_TILE * t < nrows) {
        float mx = -INFINITY;
        for (int j = SCORE_TILE * t; j < min(SCORE_TILE * (t + 1), nrows); ++j) mx = fmaxf(mx, lds.zw[j * ZG + g]);
        const int ntile = (m + SCORE_TILE - 1) / SCORE_TILE;
        tile_max[(size_t)(bh0 + g) * ntile + chunk * TPC + t] = mx;
      }
    }
    return;
  }
  const int wg = (int)blockIdx.x - n_score_wgs;
  const int unit = wg / steady_chunks, chunk = wg - unit * steady_chunks;
  const int b = unit / Hkv, h = unit - b * Hkv;
  const int bh0 = b * Hq + h * G;
  const int r0 = chunk * steady_rows, r1 = min(p, r0 + steady_rows);
  // (more than 4 heads at once would take the registers of the scoring role's occupancy:
  // the rows are read a second time, from cache, for the heads beyond the fourth)
  constexpr int G1 = G <= 4 ? G : 4;
  steady_rows_partial<T, D, G1, 256>(q, k_steady, v_steady, unit, bh0, p_stride, r0, r1, scale_log2,
                                     reinterpret_cast<float*>(lds_raw),
                                     part + ((size_t)bh0 * slots + steady_slot0 + chunk) * (D + 2),
                                     (size_t)slots * (D + 2));
  if constexpr (G > 4) {
    __syncthreads();
    steady_rows_partial<T, D, G - 4, 256>(q, k_steady, v_steady, unit, bh0 + 4, p_stride, r0, r1, scale_log2,
                                          reinterpret_cast<float*>(lds_raw),
                                          part + ((size_t)(bh0 + 4) * slots + steady_slot0 + chunk) * (D + 2),
                                          (size_t)slots * (D + 2));
  }
}

// Retrieval zone from the work list the selecting workgroups left: a workgroup takes list
// entry blockIdx.x (and every gridDim.x-th after it): range `c` of head `bh`, tokens
// [c * ct, (c + 1) * ct) of the head's selected tokens, which lie in clusters
// chunk_first[c] .. chunk_first[c + 1] of the head's list.  One partial per entry.
template <typename T, int D>
__global__ __launch_bounds__(256) void gather_list_kernel(
    const T* __restrict__ q, const T* __restrict__ k_perm, const T* __restrict__ v_perm,
    const int32_t* __restrict__ sel_pref, const int32_t* __restrict__ sel_row,
    const int32_t* __restrict__ sel_ids, const ListOut lo, int wtotal, const float* __restrict__ z,
    const T* __restrict__ vsum, int Hq, int Hkv, int N_idx /* rows per unit */, int m, int mc, int rcap,
    float scale_log2, float* __restrict__ part_g) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW, U = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  __shared__ int rowidx[GATHER_TILE];
  __shared__ int cl_pref[GATHER_TILE + 1];
  __shared__ int cl_row[GATHER_TILE];
  __shared__ int cl_id[GATHER_TILE];
  __shared__ float smem[4 * (D + 2)];
  const int claimed = *lo.work_count;
  const int cnt = min(claimed, lo.wmain);
  // entries [0, cnt), then (only if some head found the list full) the heads' spare entries
  const int items = cnt + (claimed > lo.wmain ? wtotal - lo.wmain : 0);
  for (int w = blockIdx.x; w < items; w += gridDim.x) {
    const int idx = w < cnt ? w : lo.wmain + (w - cnt);
    const int item = lo.work[idx];
    if (item < 0) continue;  // (the same for every thread of the workgroup)
    const int bh = item >> 8, chunk = item & 255;
    const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
    const int unit = b * Hkv + hq / G;
    const int4 info = lo.head_info[bh];
    const int32_t* cf = lo.chunk_first + (size_t)bh * (LIST_MAX_CHUNKS + 1);
    const int a0 = cf[chunk], a1 = cf[chunk + 1], ct = info.z, ntok = info.w;
    const long long t0l = (long long)chunk * ct;
    const int t0 = t0l < ntok ? (int)t0l : ntok, t1 = min(t0 + ct, ntok);
    const int32_t* pref = sel_pref + (size_t)bh * (rcap + 1);
    const int32_t* srow = sel_row + (size_t)bh * rcap;
    const int32_t* ids = sel_ids + (size_t)bh * rcap;
    const float* zz = z + (size_t)bh * m;

    AttnState<T, D, 1> st;
    st.init(q + (size_t)bh * D, sub, scale_log2);
    const T* Ku = k_perm + (size_t)unit * N_idx * D + sub * EPC;
    const T* Vu = v_perm + (size_t)unit * N_idx * D + sub * EPC;
    const T* VSu = vsum + (size_t)unit * mc * D + sub * EPC;
    const int nc_all = t0 < t1 ? a1 - a0 + 1 : 0;
    for (int cb = 0; cb < nc_all; cb += GATHER_TILE) {
      const int nc = min(GATHER_TILE, nc_all - cb);
      __syncthreads();  // the previous pass is done with the tables
      {
        const int i = min((int)threadIdx.x, nc);  // entry nc is the end of the pass's last cluster
        const int pv = pref[a0 + cb + i];
        const int rv = srow[a0 + cb + min((int)threadIdx.x, nc - 1)];
        const int iv = ids[a0 + cb + min((int)threadIdx.x, nc - 1)];
        if ((int)threadIdx.x <= nc) cl_pref[i] = pv;
        if ((int)threadIdx.x < nc) {
          cl_row[threadIdx.x] = rv;
          cl_id[threadIdx.x] = iv;
        }
      }
      __syncthreads();
      // The estimation pass added a term for every cluster; the selected ones are attended
      // exactly, so the clusters that START in this token range have theirs taken out again
      // (every selected cluster starts in exactly one range).  The first GROUPS * U clusters'
      // value sums are requested here, before the rows stream, and used after it.
      uint4 nraw[U];
      float nsc[1][U], nmult[U];
      auto neg_load = [&](int i0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int ii = i0 + u * GROUPS;
          const int j = ii < nc ? ii : nc - 1;
          const int id = cl_id[j];
          const int ps = cl_pref[j];
          nraw[u] = load16(VSu + (size_t)id * D);
          nsc[0][u] = zz[id];
          nmult[u] = (float)(cl_pref[j + 1] - ps);
          if (!(ii < nc && ps >= t0 && ps < t1)) nmult[u] = -1.f;  // not this range's: marked, masked below
        }
      };
      auto neg_apply = [&]() {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          nsc[0][u] = nmult[u] >= 0.f ? nsc[0][u] * scale_log2 : -INFINITY;
          nmult[u] = fmaxf(nmult[u], 0.f);
        }
        st.template rows_given<U, true>(nsc, nmult, nraw);
      };
      neg_load(grp);
      const int lo_t = max(t0, cl_pref[0]), hi_t = min(t1, cl_pref[nc]);
      for (int base = lo_t; base < hi_t; base += GATHER_TILE) {
        const int n = min(GATHER_TILE, hi_t - base);
        __syncthreads();
        if ((int)threadIdx.x < n) {
          const int t = base + threadIdx.x;
          int a = 0, e = nc;  // largest a with cl_pref[a] <= t
          while (e - a > 1) {
            const int mid = (a + e) >> 1;
            if (cl_pref[mid] <= t) a = mid; else e = mid;
          }
          rowidx[threadIdx.x] = cl_row[a] + (t - cl_pref[a]);
        }
        __syncthreads();
        for (int i = grp; i < n; i += GROUPS * U) {
          uint4 kraw[U], vraw[U];
          bool valid[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int ii = i + u * GROUPS;
            valid[u] = ii < n;
            const int row = rowidx[valid[u] ? ii : i];
            kraw[u] = load16_stream(Ku + (size_t)row * D);
            vraw[u] = load16_stream(Vu + (size_t)row * D);
          }
          st.template rows<U, LPR>(kraw, vraw, valid);
        }
      }
      neg_apply();
      for (int i = grp + GROUPS * U; i < nc; i += GROUPS * U) {
        neg_load(i);
        neg_apply();
      }
    }
    __syncthreads();
    merge_groups_and_store<T, D, 1>(st, smem, part_g + (size_t)idx * (D + 2), 0);
    __syncthreads();  // smem and the tables are free for the next entry
  }
}

// The merge for heads whose retrieval partials sit on the work list: the head's partials of
// the other zones, then its list entries' partials.
template <int D, int NT>
__global__ __launch_bounds__(NT) void merge_list_kernel(
    const float* __restrict__ part, int slots, int slot_stride, const float* __restrict__ part_g,
    const int4* __restrict__ head_info, float* __restrict__ out, float* __restrict__ lse) {
  const int bh = blockIdx.x;
  const int4 info = head_info[bh];
  merge_head<D, NT, 16>(part + (size_t)bh * slot_stride * (D + 2), slots, out + (size_t)bh * D, lse + bh,
                        part_g + (size_t)info.x * (D + 2), info.y);
}

__global__ void fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ============================================================================
// Host: geometry and launches
// ============================================================================
DecodeGeom decode_geometry(const wave_index& ix, int Hq, int topk) {
  DecodeGeom g{};
  const int m = ix.m, units = ix.B * ix.Hkv, heads = ix.B * Hq, D = ix.d;
  g.score_rows = DENSE_ROWS;   // one meta-index workgroup covers this many clusters
  g.score_chunks = m > 0 ? (m + DENSE_ROWS - 1) / DENSE_ROWS : 0;
  g.est_rows = DENSE_ROWS;
  g.est_chunks = g.score_chunks;
  g.steady_rows = units >= 64 ? 256 : 64;  // few units: smaller pieces to spread over the CUs
  g.steady_chunks = ix.p > 0 ? (ix.p + g.steady_rows - 1) / g.steady_rows : 0;
  const int r = m > 0 ? (topk < m ? topk : m) : 0;
  g.rcap = r > 0 ? r : 1;
  double expect = m > 0 ? (double)r * (double)ix.N_idx / (double)m : 0.0;
  int gc = (int)((expect + GATHER_TILE - 1) / GATHER_TILE);
  if (gc < 1) gc = 1;
  if (gc > 256) gc = 256;
  g.gather_chunks = (m > 0 && r > 0) ? gc : 0;
  // With at least ~1.5 query heads per CU, selection and retrieval of a head run
  // fused in one workgroup and leave one partial result.
  g.fused = (m > 0 && r > 0 && heads >= 384 && m <= 512 * 32) ? 1 : 0;
  if (g.fused) {
    g.gather_chunks = 1;
    g.steady_chunks = 0;  // the fused kernel attends the steady rows per head as well
  }
  // Few heads over many clusters: rank slices of 8192 clusters in parallel, then
  // the union of their lists (at most nslices * r <= 16384 ids).
  g.slice_len = 8192;
  g.nslices = (m + g.slice_len - 1) / g.slice_len;
  g.sliced = (!g.fused && r > 0 && m > 16384 && g.nslices <= 64 &&
              (long long)g.nslices * r <= 16384) ? 1 : 0;
  // Selection in one launch (one workgroup per head, beside the estimation ranges of all
  // clusters), retrieval in the next from ONE work list of equal token ranges over all heads:
  // with many heads whose clusters' keys fit in LDS, or with few heads over many clusters and
  // a moderate r (filtered through the tile maxima, see select_filtered).
  g.list_filtered = (r > 0 && m > 16384 && m <= FILT_NT * FILT_MAX_SWEEPS && r <= filtered_max_r()) ? 1 : 0;
  // (up to about three heads per CU the fused kernel below, one workgroup per head with all
  // of them resident at once, is faster; beyond that, or with uneven heads, its tail is long)
  int listed_min_heads = 768;
#ifdef WAVE_TUNE  // tuning builds only: launch shapes from the environment
  if (const char* e = getenv("WAVE_LISTED_MIN_HEADS")) listed_min_heads = atoi(e);
#endif
  g.listed = (g.list_filtered || (m > 0 && r > 0 && heads > listed_min_heads && m <= 512 * 32)) ? 1 : 0;
  if (g.listed) {
    g.fused = 0;
    g.sliced = 0;
    g.gather_chunks = 0;  // the retrieval partials are the work list's, not per-head slots
    g.steady_chunks = ix.p > 0 ? (ix.p + g.steady_rows - 1) / g.steady_rows : 0;
    const int G = Hq / ix.Hkv;
    if (g.list_filtered) {
      // Estimation ranges sized so that their 512-thread workgroups and the selecting ones are
      // all resident at once (2 per CU up to 4 heads per KV head, else 1, by their registers): a
      // second round of long-lived workgroups would double the launch.  The staged scores and
      // sizes of a range, (ZG + 1) * rows floats, share the selecting role's LDS budget.
      int chunks = (256 * (G <= 4 ? 2 : 1) - heads) / units;
      if (chunks < 1) chunks = 1;
      int rows = (m + chunks - 1) / chunks;
      rows = (rows + 63) / 64 * 64;
      const int rows_max = (int)(FILT_LDS / sizeof(float)) / ((G + 3) / 4 * 4 + 1) / 64 * 64;
      if (rows > rows_max) rows = rows_max;
      if (rows < 512) rows = 512;
      g.est_rows = rows;
    } else {
      g.est_rows = G <= 4 ? 1024 : 512;  // many heads: several rounds of workgroups anyway
    }
#ifdef WAVE_TUNE
    if (const char* e = getenv("WAVE_EST_ROWS")) g.est_rows = atoi(e);
#endif
    g.est_chunks = (m + g.est_rows - 1) / g.est_rows;
    // tokens per range: about one resident round of retrieval workgroups (4 per CU) when
    // there are few tokens, never more than 512 (several rounds of equal pieces then)
    const double tokens = expect * heads;
    int ctok = (int)((tokens + 1023) / 1024);
    g.chunk_tokens = ctok < 256 ? 256 : (ctok > 512 ? 512 : ctok);
#ifdef WAVE_TUNE
    if (const char* e = getenv("WAVE_CHUNK_TOKENS")) g.chunk_tokens = atoi(e);
#endif
    const long long ranges = (long long)(tokens / g.chunk_tokens) + 1;
    // heavy-tailed cluster sizes select large clusters: room for three times the expected
    // ranges (a head that finds the list full still retrieves, as one range)
    g.wmain = (int)(3 * ranges + heads);
    g.wtotal = g.wmain + heads;
    const long long grid = 2 * ranges + heads;
    g.gather_wgs = (int)(grid < g.wtotal ? grid : g.wtotal);
    g.stage = (r < FUSED_STAGE ? r : FUSED_STAGE) + 1;  // (+ 1: the end of the last staged cluster)
  }
  // partial results per head: retrieval, steady, estimation of all clusters per
  // range, and (see below) the selected clusters' estimation terms with a minus sign
  if (g.sliced) {
    // The estimation terms come from 512-thread workgroups in the launch that ranks the
    // union of the slices' lists.  A range is sized so that those workgroups and the
    // ranking ones are all resident at once (2 workgroups per CU up to 4 heads per KV
    // head, else 1): a second round of long-lived workgroups would double the launch.
    const int G = Hq / ix.Hkv;
    const int resident = 256 * (G <= 4 ? 2 : 1);
    int chunks = (resident - heads) / units;
    if (chunks < 1) chunks = 1;
    int rows = (m + chunks - 1) / chunks;
    rows = (rows + 63) / 64 * 64;
    const int rows_max = 10240 / (G + 1) / 64 * 64;  // staged scores and sizes: (G + 1) * rows floats of LDS
    if (rows > rows_max) rows = rows_max;
    if (rows < 512) rows = 512;
    g.est_rows = rows;
    g.est_chunks = (m + g.est_rows - 1) / g.est_rows;
    g.est_with_slices_pct = 0;  // share of the estimation ranges in the slices' launch instead
  }
  // Who takes the selected clusters' estimation terms out again: the retrieval
  // kernel itself (no partial of their own), except after the fused kernel and
  // after the streaming selection, which write them as one more partial.
  g.neg_in_gather = (m > 0 && !g.fused && (g.listed || g.sliced || m <= 1024 * 64)) ? 1 : 0;
  g.neg_slots = (m > 0 && !g.neg_in_gather) ? 1 : 0;
  g.slots = g.gather_chunks + g.steady_chunks + g.est_chunks + g.neg_slots;
  if (g.slots < 1) g.slots = 1;
  g.mwords = (m + 31) / 32;
  size_t o = 0;
  g.off_z = o;       o = align_up(o + sizeof(float) * (size_t)heads * (m > 0 ? m : 1));
  g.off_cn2 = o;     o = align_up(o + sizeof(float) * (size_t)units * (g.score_chunks > 0 ? g.score_chunks : 1));
  g.off_sel = o;     o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap);
  g.off_pref = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * (g.rcap + 1));
  g.off_srow = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap);
  g.off_bitmap = o;  o = align_up(o + sizeof(uint32_t) * (size_t)heads * (g.mwords > 0 ? g.mwords : 1));
  g.off_nsel = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads);
  g.off_part = o;    o = align_up(o + sizeof(float) * (size_t)heads * g.slots * (D + 2));
  if (g.sliced) {
    g.off_slice_ids = o; o = align_up(o + sizeof(int32_t) * (size_t)heads * g.nslices * r);
    g.off_slice_z = o;   o = align_up(o + sizeof(float) * (size_t)heads * g.nslices * r);
    g.off_tile_max = o;  o = align_up(o + sizeof(float) * (size_t)heads * ((m + SCORE_TILE - 1) / SCORE_TILE));
  }
  if (g.listed) {
    if (g.list_filtered) {
      g.off_tile_max = o;  o = align_up(o + sizeof(float) * (size_t)heads * ((m + SCORE_TILE - 1) / SCORE_TILE));
    }
    g.off_chunk_first = o; o = align_up(o + sizeof(int32_t) * (size_t)heads * (LIST_MAX_CHUNKS + 1));
    g.off_head_info = o;   o = align_up(o + sizeof(int4) * (size_t)heads);
    g.off_work = o;        o = align_up(o + sizeof(int32_t) * (size_t)g.wtotal);
    g.off_work_count = o;  o = align_up(o + sizeof(int32_t));
    g.off_part_g = o;      o = align_up(o + sizeof(float) * (size_t)g.wtotal * (D + 2));
  }
  g.total = o;
  return g;
}

template <typename T, int D, int G>
static wave_status decode_tdg(const void* q_, const wave_index& ix, int Hq, int topk, float* out,
                              float* lse, int32_t* selected, void* ws, hipStream_t st) {
  const DecodeGeom g = decode_geometry(ix, Hq, topk);
  char* w = static_cast<char*>(ws);
  float* z = reinterpret_cast<float*>(w + g.off_z);
  float* cn2 = reinterpret_cast<float*>(w + g.off_cn2);
  int32_t* sel = reinterpret_cast<int32_t*>(w + g.off_sel);
  int32_t* pref = reinterpret_cast<int32_t*>(w + g.off_pref);
  int32_t* srow = reinterpret_cast<int32_t*>(w + g.off_srow);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(w + g.off_bitmap);
  int32_t* nsel = reinterpret_cast<int32_t*>(w + g.off_nsel);
  float* part = reinterpret_cast<float*>(w + g.off_part);
  const T* q = static_cast<const T*>(q_);
  const int units = ix.B * ix.Hkv, heads = ix.B * Hq, m = ix.m;
  const int mc = cluster_stride(ix);  // clusters per unit in the meta-index arrays
  const float scale_log2 = kLog2e / sqrtf((float)D);
  const int r = m > 0 ? (topk < m ? topk : m) : 0;

  if (m > 0) {
    const int est_slot0 = g.gather_chunks + g.steady_chunks;
    const int neg_slot = est_slot0 + g.est_chunks;  // exists when g.neg_slots is 1
    ListOut lo{};
    if (g.listed) {
      lo = ListOut{reinterpret_cast<int32_t*>(w + g.off_chunk_first), reinterpret_cast<int4*>(w + g.off_head_info),
                   reinterpret_cast<int32_t*>(w + g.off_work), reinterpret_cast<int32_t*>(w + g.off_work_count),
                   g.wmain, g.chunk_tokens};
      // (the steady zone rides with the selection launch; this kernel's steady role stays idle)
      WAVE_LAUNCH("scores", (score_steady_kernel<T, D, G>), units * g.score_chunks, 256, 0, st, q,
                  static_cast<const T*>(ix.centroids), ix.sizes, z, cn2, ix.Hkv, m, mc, g.score_chunks,
                  g.list_filtered ? reinterpret_cast<float*>(w + g.off_tile_max) : nullptr,
                  units * g.score_chunks, static_cast<const T*>(ix.k_steady),
                  static_cast<const T*>(ix.v_steady), ix.p, steady_stride(ix), 0, g.steady_rows,
                  g.slots, 0, scale_log2, part, lo.work, lo.work_count, g.wtotal);
    } else if (g.sliced)
      WAVE_LAUNCH("scores", (score_kernel<T, D, G>), units * g.score_chunks, 256, 0, st, q,
                  static_cast<const T*>(ix.centroids), ix.sizes, z, cn2, ix.Hkv, m, mc, g.score_chunks,
                  reinterpret_cast<float*>(w + g.off_tile_max));
    else if (!g.fused && g.steady_chunks > 0)
      WAVE_LAUNCH("meta_index+steady", (dense_steady_kernel<T, D, G>),
                  units * (g.score_chunks + g.steady_chunks), 256, 0, st, q,
                  static_cast<const T*>(ix.centroids), static_cast<const T*>(ix.vsum), ix.sizes, z, cn2,
                  ix.Hkv, m, mc, g.score_chunks, g.slots, est_slot0, scale_log2, part,
                  units * g.score_chunks, static_cast<const T*>(ix.k_steady),
                  static_cast<const T*>(ix.v_steady), ix.p, steady_stride(ix), g.steady_chunks, g.steady_rows,
                  g.gather_chunks);
    else
      WAVE_LAUNCH("meta_index", (dense_kernel<T, D, G>), units * g.score_chunks, 256, 0, st, q,
                  static_cast<const T*>(ix.centroids), static_cast<const T*>(ix.vsum), ix.sizes, z, cn2,
                  ix.Hkv, m, mc, g.score_chunks, g.slots, est_slot0, scale_log2, part);
#define WAVE_SELECT_ARGS                                                                           \
  q, static_cast<const T*>(ix.centroids), ix.offsets, z, cn2, g.score_chunks, Hq, ix.Hkv, m, r,    \
      g.rcap, g.mwords, mc, topk, sel, pref, srow, bitmap, nsel, selected,                        \
      static_cast<const T*>(ix.vsum), scale_log2, part, g.slots, neg_slot
    const size_t key_lds = sizeof(uint32_t) * 512 * (size_t)((m + 511) / 512);
    if (g.fused) {
      WAVE_LAUNCH("select_gather_steady", (select_gather_kernel<T, D, 512, 32, true>), heads, 512,
                  key_lds, st, WAVE_SELECT_ARGS, static_cast<const T*>(ix.k_perm),
                  static_cast<const T*>(ix.v_perm), row_stride(ix), static_cast<const T*>(ix.k_steady),
                  static_cast<const T*>(ix.v_steady), ix.p, steady_stride(ix), 2, out, lse);
    } else if (g.listed) {
      const size_t lds_est = sizeof(float) * ((G + 3) / 4 * 4 + 1) * (size_t)g.est_rows;
      int nt = g.list_filtered ? FILT_NT : select_direct_threads(m);
#ifdef WAVE_TUNE
      if (const char* e = getenv("WAVE_SEL_NT")) nt = g.list_filtered ? nt : atoi(e);
#endif
      const size_t lds_merge = sizeof(float) * (nt / 64) * G * (D + 2);  // the estimation role's last step
      size_t lds = g.list_filtered ? FILT_LDS : select_direct_lds(m, g.stage);
      if (lds < lds_est) lds = lds_est;
      if (lds < lds_merge) lds = lds_merge;  // (also covers the steady role's, at most 4 heads at a time)
      SideWork sw{ix.sizes, g.est_rows, g.est_chunks, g.steady_chunks, 0, units * g.est_chunks, ix.k_steady,
                  ix.v_steady, ix.p, steady_stride(ix), g.steady_chunks, g.steady_rows, 0};
      const int n_side = sw.n_est_wgs + units * g.steady_chunks;
      if (g.list_filtered)
        WAVE_LAUNCH("select+estimate+steady", (select_estimate_kernel<T, D, G, FILT_NT, true>),
                    heads + n_side, FILT_NT, lds, st, WAVE_SELECT_ARGS,
                    reinterpret_cast<const float*>(w + g.off_tile_max), lo, g.stage, heads, sw);
      else if (nt == 128)
        WAVE_LAUNCH("select+estimate+steady", (select_estimate_kernel<T, D, G, 128, false>),
                    heads + n_side, 128, lds, st, WAVE_SELECT_ARGS,
                    static_cast<const float*>(nullptr), lo, g.stage, heads, sw);
      else
        WAVE_LAUNCH("select+estimate+steady", (select_estimate_kernel<T, D, G, 256, false>),
                    heads + n_side, 256, lds, st, WAVE_SELECT_ARGS,
                    static_cast<const float*>(nullptr), lo, g.stage, heads, sw);
      WAVE_LAUNCH("gather", (gather_list_kernel<T, D>), g.gather_wgs, 256, 0, st, q,
                  static_cast<const T*>(ix.k_perm), static_cast<const T*>(ix.v_perm), pref, srow, sel, lo,
                  g.wtotal, z, static_cast<const T*>(ix.vsum), Hq, ix.Hkv, row_stride(ix), m, mc, g.rcap,
                  scale_log2, reinterpret_cast<float*>(w + g.off_part_g));
      // (few heads: many threads per head, every partial in one trip; many heads: small workgroups)
      if (heads <= 256)
        WAVE_LAUNCH("merge", (merge_list_kernel<D, MERGE_THREADS>), heads, MERGE_THREADS, 0, st, part,
                    g.steady_chunks + g.est_chunks, g.slots, reinterpret_cast<const float*>(w + g.off_part_g),
                    lo.head_info, out, lse);
      else
        WAVE_LAUNCH("merge", (merge_list_kernel<D, 256>), heads, 256, 0, st, part,
                    g.steady_chunks + g.est_chunks, g.slots, reinterpret_cast<const float*>(w + g.off_part_g),
                    lo.head_info, out, lse);
    } else {
      if (g.sliced) {
        int32_t* slice_ids = reinterpret_cast<int32_t*>(w + g.off_slice_ids);
        float* slice_z = reinterpret_cast<float*>(w + g.off_slice_z);
        // Each head's clusters are cut into slices ranked by workgroups of their own
        // (the r best of a slice contain every cluster of the slice that is among the
        // r best overall); the second launch ranks the union of the slices' lists.
        const int npos_max = g.nslices * r;
        size_t lds_a = sizeof(uint32_t) * 512 * (size_t)((g.slice_len + 511) / 512);
        size_t lds_b = sizeof(uint32_t) * 512 * (size_t)((npos_max + 511) / 512);
        // the side roles' final merge; the staged scores and sizes of an estimation range,
        // (G + 1) * est_rows floats, use the same space before it
        size_t lds_side = sizeof(float) * 8 * G * (D + 2);
        if (lds_side < sizeof(float) * (G + 1) * (size_t)g.est_rows) lds_side = sizeof(float) * (G + 1) * (size_t)g.est_rows;
        if (lds_a < lds_side) lds_a = lds_side;
        if (lds_b < lds_side) lds_b = lds_side;
        const int n_est = units * g.est_chunks;
        const int n_est_a = (int)((long long)n_est * g.est_with_slices_pct / 100);
        SideWork sw{ix.sizes, g.est_rows, g.est_chunks, est_slot0, 0, n_est_a, ix.k_steady,
                    ix.v_steady, ix.p, steady_stride(ix), g.steady_chunks, g.steady_rows, g.gather_chunks};
        WAVE_LAUNCH("select_slices+side", (filter_side_kernel<T, D, G, 512, 32>),
                    heads * g.nslices + n_est_a + units * g.steady_chunks, 512, lds_a, st,
                    WAVE_SELECT_ARGS, g.nslices, g.slice_len, slice_ids, slice_z, heads * g.nslices, sw,
                    reinterpret_cast<const float*>(w + g.off_tile_max));
        sw.est_first = n_est_a;
        sw.n_est_wgs = n_est - n_est_a;
        sw.steady_chunks = 0;  // done by the first launch
        WAVE_LAUNCH("select+side", (combine_side_kernel<T, D, G, 512, 32>), heads + sw.n_est_wgs, 512,
                    lds_b, st, WAVE_SELECT_ARGS, g.nslices, slice_ids, slice_z, heads, sw);
      } else if (m <= 512 * 32)  // keys in LDS (64 KiB at most)
        WAVE_LAUNCH("select", (select_cached_kernel<T, D, 512, 32, true>), heads, 512, key_lds, st,
                    WAVE_SELECT_ARGS);
      else if (m <= 1024 * 64)  // upper halves of the keys in LDS (128 KiB at most)
        WAVE_LAUNCH("select", (select_cached_kernel<T, D, 1024, 64, false>), heads, 1024,
                    sizeof(uint16_t) * 1024 * (size_t)((m + 1023) / 1024), st, WAVE_SELECT_ARGS);
      else
        WAVE_LAUNCH("select", (select_kernel<T, D, 512>), heads, 512, 0, st, WAVE_SELECT_ARGS);
      if (g.gather_chunks > 0)
        WAVE_LAUNCH("gather", (gather_kernel<T, D>), heads * g.gather_chunks, 256, 0, st, q,
                    static_cast<const T*>(ix.k_perm), static_cast<const T*>(ix.v_perm), sel, nsel,
                    ix.offsets, z, static_cast<const T*>(ix.vsum), Hq, ix.Hkv, row_stride(ix), m, mc, g.rcap,
                    g.gather_chunks, g.slots, scale_log2, g.neg_in_gather, part);
    }
#undef WAVE_SELECT_ARGS
  }
  if (m == 0 && selected && topk > 0) {
    const size_t n = (size_t)heads * topk;  // no clusters exist: nothing is selected
    WAVE_LAUNCH("fill", fill_i32_kernel, (unsigned)((n + 255) / 256), 256, 0, st, selected, n, -1);
  }
  if (m == 0 && g.steady_chunks > 0)  // with clusters, the steady pieces ride with an earlier launch
    WAVE_LAUNCH("steady", (steady_kernel<T, D, G>), units * g.steady_chunks, 256, 0, st, q,
                static_cast<const T*>(ix.k_steady), static_cast<const T*>(ix.v_steady), ix.Hkv, ix.p,
                steady_stride(ix),
                g.steady_chunks, g.steady_rows, g.slots, g.gather_chunks, scale_log2, part);
  if (!g.fused && !g.listed)  // (the fused kernel normalises each head itself; the listed path has its own merge)
    WAVE_LAUNCH("merge", (merge_kernel<D>), heads, MERGE_THREADS, 0, st, part,
                g.gather_chunks + g.steady_chunks + g.est_chunks + g.neg_slots, g.slots, out, lse);
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

template <typename T, int D>
static wave_status decode_td(int G, const void* q, const wave_index& ix, int Hq, int topk, float* out,
                             float* lse, int32_t* selected, void* ws, hipStream_t st) {
  switch (G) {
#define WAVE_G(n) \
  case n: return decode_tdg<T, D, n>(q, ix, Hq, topk, out, lse, selected, ws, st);
    WAVE_G(1) WAVE_G(2) WAVE_G(3) WAVE_G(4) WAVE_G(5) WAVE_G(6) WAVE_G(7) WAVE_G(8)
#undef WAVE_G
    default: return WAVE_ERR_SHAPE;
  }
}

// ---------------------------------------------------------------------------
// Decode with an estimation budget.  Not a tuned path: the scores alone, two
// selections (the r best and the r + e best), then the steady zone, the retrieved
// tokens, the estimated clusters and the merge as launches of their own.
// ---------------------------------------------------------------------------
BudgetGeom budget_geometry(const wave_index& ix, int Hq, int topk, int est_clusters) {
  BudgetGeom g{};
  const int m = ix.m, units = ix.B * ix.Hkv, heads = ix.B * Hq, D = ix.d;
  const int r = m > 0 ? (topk < m ? topk : m) : 0;
  if (m == 0 || est_clusters < 0 || (long long)r + est_clusters >= m) {
    g.delegate = 1;
    g.total = decode_geometry(ix, Hq, topk).total;
    return g;
  }
  g.r = r;
  g.k2 = r + est_clusters;
  g.rcap1 = r > 0 ? r : 1;
  g.rcap2 = g.k2 > 0 ? g.k2 : 1;
  g.mwords = (m + 31) / 32;
  g.slice_len = 8192;
  g.nslices = (m + g.slice_len - 1) / g.slice_len;
  auto sliced = [&](int k) {
    return (k > 0 && m > 16384 && g.nslices <= 64 && (long long)g.nslices * k <= 16384) ? 1 : 0;
  };
  g.sliced1 = sliced(r);
  g.sliced2 = sliced(g.k2);
  g.score_chunks = (m + DENSE_ROWS - 1) / DENSE_ROWS;
  g.steady_rows = units >= 64 ? 256 : 64;
  g.steady_chunks = ix.p > 0 ? (ix.p + g.steady_rows - 1) / g.steady_rows : 0;
  double expect = (double)r * (double)ix.N_idx / (double)m;
  int gc = (int)((expect + GATHER_TILE - 1) / GATHER_TILE);
  gc = gc < 1 ? 1 : (gc > 256 ? 256 : gc);
  g.gather_chunks = r > 0 ? gc : 0;
  int ec = (est_clusters + 255) / 256;
  ec = ec < 1 ? 1 : (ec > 256 ? 256 : ec);
  g.est_chunks = est_clusters > 0 ? ec : 0;
  g.slots = g.steady_chunks + g.gather_chunks + g.est_chunks;
  size_t o = 0;
  g.off_z = o;       o = align_up(o + sizeof(float) * (size_t)heads * m);
  g.off_cn2 = o;     o = align_up(o + sizeof(float) * (size_t)units * g.score_chunks);
  g.off_ids1 = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap1);
  g.off_ids2 = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap2);
  g.off_nsel1 = o;   o = align_up(o + sizeof(int32_t) * (size_t)heads);
  g.off_nsel2 = o;   o = align_up(o + sizeof(int32_t) * (size_t)heads);
  g.off_pref = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * (g.rcap2 + 1));
  g.off_srow = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap2);
  g.off_bitmap = o;  o = align_up(o + sizeof(uint32_t) * (size_t)heads * g.mwords);
  if (g.sliced1 || g.sliced2) {
    g.off_slice_ids = o; o = align_up(o + sizeof(int32_t) * (size_t)heads * g.nslices * g.rcap2);
    g.off_slice_z = o;   o = align_up(o + sizeof(float) * (size_t)heads * g.nslices * g.rcap2);
  }
  // one more slot than the merge reads: the streaming selection leaves a partial there
  g.off_part = o;    o = align_up(o + sizeof(float) * (size_t)heads * (g.slots + 1) * (D + 2));
  g.total = o;
  return g;
}

template <typename T, int D, int G>
static wave_status budget_tdg(const void* q_, const wave_index& ix, int Hq, int est_clusters, float* out,
                              float* lse, int32_t* selected, int topk, void* ws, hipStream_t st) {
  const BudgetGeom g = budget_geometry(ix, Hq, topk, est_clusters);
  char* w = static_cast<char*>(ws);
  float* z = reinterpret_cast<float*>(w + g.off_z);
  float* cn2 = reinterpret_cast<float*>(w + g.off_cn2);
  int32_t* ids1 = reinterpret_cast<int32_t*>(w + g.off_ids1);
  int32_t* ids2 = reinterpret_cast<int32_t*>(w + g.off_ids2);
  int32_t* nsel1 = reinterpret_cast<int32_t*>(w + g.off_nsel1);
  int32_t* nsel2 = reinterpret_cast<int32_t*>(w + g.off_nsel2);
  int32_t* pref = reinterpret_cast<int32_t*>(w + g.off_pref);
  int32_t* srow = reinterpret_cast<int32_t*>(w + g.off_srow);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(w + g.off_bitmap);
  int32_t* slice_ids = reinterpret_cast<int32_t*>(w + g.off_slice_ids);
  float* slice_z = reinterpret_cast<float*>(w + g.off_slice_z);
  float* part = reinterpret_cast<float*>(w + g.off_part);
  const T* q = static_cast<const T*>(q_);
  const T* C = static_cast<const T*>(ix.centroids);
  const T* VS = static_cast<const T*>(ix.vsum);
  const int units = ix.B * ix.Hkv, heads = ix.B * Hq, m = ix.m;
  const int mc = cluster_stride(ix);  // clusters per unit in the meta-index arrays
  const float scale_log2 = kLog2e / sqrtf((float)D);
  const int slots = g.slots + 1, spare_slot = g.slots;

  // Keys of a head fit in LDS (whole, or their upper halves with a re-read hot range): four
  // launches.  The scores with the steady zone as extra workgroups; both selections at once (two
  // workgroups per head); retrieval and estimation in one launch (neither needs the other); the merge.
  if (m <= 1024 * 64 && est_clusters > 0) {
    WAVE_LAUNCH("scores+steady", (score_steady_kernel<T, D, G>), units * (g.score_chunks + g.steady_chunks),
                256, 0, st, q, C, ix.sizes, z, cn2, ix.Hkv, m, mc, g.score_chunks, static_cast<float*>(nullptr),
                units * g.score_chunks, static_cast<const T*>(ix.k_steady), static_cast<const T*>(ix.v_steady),
                ix.p, steady_stride(ix), g.steady_chunks, g.steady_rows, slots, 0, scale_log2, part,
                static_cast<int32_t*>(nullptr), static_cast<int32_t*>(nullptr), 0);
#define WAVE_TWO_ARGS                                                                                   \
  q, C, ix.offsets, z, cn2, g.score_chunks, Hq, ix.Hkv, m, g.mwords, mc, bitmap, g.r, g.rcap1, ids1, nsel1, \
      selected, g.k2, g.rcap2, ids2, nsel2, VS, scale_log2
    // (with 16-bit keys four workgroups fit a CU instead of three: 769 .. 1024 selections are then
    // all resident at once instead of running in two rounds; a selection by itself is slower so)
    if (m <= 512 * 32 && (2 * heads <= 768 || 2 * heads > 1024))
      WAVE_LAUNCH("select x2", (select_two_kernel<T, D, 512, 32, true>), 2 * heads, 512,
                  sizeof(uint32_t) * 512 * (size_t)((m + 511) / 512), st, WAVE_TWO_ARGS);
    else if (m <= 512 * 32)
      WAVE_LAUNCH("select x2", (select_two_kernel<T, D, 512, 32, false>), 2 * heads, 512,
                  sizeof(uint16_t) * 512 * (size_t)((m + 511) / 512), st, WAVE_TWO_ARGS);
    else
      WAVE_LAUNCH("select x2", (select_two_kernel<T, D, 1024, 64, false>), 2 * heads, 1024,
                  sizeof(uint16_t) * 1024 * (size_t)((m + 1023) / 1024), st, WAVE_TWO_ARGS);
#undef WAVE_TWO_ARGS
    const int n_est = heads * g.est_chunks;
    WAVE_LAUNCH("gather+estimate", (gather_est_kernel<T, D>), n_est + heads * g.gather_chunks, 256, 0, st, q,
                static_cast<const T*>(ix.k_perm), static_cast<const T*>(ix.v_perm), ids1, nsel1, ids2, nsel2,
                ix.offsets, z, VS, Hq, ix.Hkv, row_stride(ix), m, mc, g.rcap1, g.rcap2, g.gather_chunks,
                g.est_chunks, slots, g.steady_chunks, g.steady_chunks + g.gather_chunks, n_est, scale_log2,
                part);
    if (heads <= 256)
      WAVE_LAUNCH("merge", (merge_kernel<D, MERGE_THREADS>), heads, MERGE_THREADS, 0, st, part, g.slots, slots,
                  out, lse);
    else
      WAVE_LAUNCH("merge", (merge_kernel<D, 256>), heads, 256, 0, st, part, g.slots, slots, out, lse);
    return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
  }
  WAVE_LAUNCH("scores", (score_kernel<T, D, G>), units * g.score_chunks, 256, 0, st, q, C, ix.sizes, z,
              cn2, ix.Hkv, m, mc, g.score_chunks, static_cast<float*>(nullptr));
  // the k best clusters of every head as an ascending id list (ids, nsel)
  auto select_ids = [&](int k, int rcap, int sliced, int32_t* ids, int32_t* nsel, int32_t* usel) {
#define WAVE_SEL(k_)                                                                                \
  q, C, ix.offsets, z, cn2, g.score_chunks, Hq, ix.Hkv, m, k_, rcap, g.mwords, mc, k_, ids, pref, srow,   \
      bitmap, nsel, usel, VS, scale_log2, part, slots, spare_slot
    if (sliced) {
      const int npos_max = g.nslices * k;
      const size_t lds_a = sizeof(uint32_t) * 512 * (size_t)((g.slice_len + 511) / 512);
      const size_t lds_b = sizeof(uint32_t) * 512 * (size_t)((npos_max + 511) / 512);
      SideWork none{ix.sizes, 512, 1, 0, 0, 0, ix.k_steady, ix.v_steady, ix.p, steady_stride(ix), 0, 64, 0};
      WAVE_LAUNCH("select_slices", (slices_side_kernel<T, D, G, 512, 32>), heads * g.nslices, 512, lds_a,
                  st, WAVE_SEL(k), g.nslices, g.slice_len, slice_ids, slice_z, heads * g.nslices, none);
      WAVE_LAUNCH("select", (combine_side_kernel<T, D, G, 512, 32>), heads, 512, lds_b, st, WAVE_SEL(k),
                  g.nslices, slice_ids, slice_z, heads, none);
    } else if (m <= 512 * 32) {
      WAVE_LAUNCH("select", (select_cached_kernel<T, D, 512, 32, true>), heads, 512,
                  sizeof(uint32_t) * 512 * (size_t)((m + 511) / 512), st, WAVE_SEL(k));
    } else if (m <= 1024 * 64) {
      WAVE_LAUNCH("select", (select_cached_kernel<T, D, 1024, 64, false>), heads, 1024,
                  sizeof(uint16_t) * 1024 * (size_t)((m + 1023) / 1024), st, WAVE_SEL(k));
    } else {
      WAVE_LAUNCH("select", (select_kernel<T, D, 512>), heads, 512, 0, st, WAVE_SEL(k));
    }
#undef WAVE_SEL
  };
  select_ids(g.r, g.rcap1, g.sliced1, ids1, nsel1, selected);
  if (est_clusters > 0) select_ids(g.k2, g.rcap2, g.sliced2, ids2, nsel2, nullptr);

  if (g.steady_chunks > 0)
    WAVE_LAUNCH("steady", (steady_kernel<T, D, G>), units * g.steady_chunks, 256, 0, st, q,
                static_cast<const T*>(ix.k_steady), static_cast<const T*>(ix.v_steady), ix.Hkv, ix.p,
                steady_stride(ix),
                g.steady_chunks, g.steady_rows, slots, 0, scale_log2, part);
  if (g.gather_chunks > 0)
    WAVE_LAUNCH("gather", (gather_kernel<T, D>), heads * g.gather_chunks, 256, 0, st, q,
                static_cast<const T*>(ix.k_perm), static_cast<const T*>(ix.v_perm), ids1, nsel1,
                ix.offsets, z, VS, Hq, ix.Hkv, row_stride(ix), m, mc, g.rcap1, g.gather_chunks, slots, scale_log2, 0,
                part + (size_t)g.steady_chunks * (D + 2));
  if (g.est_chunks > 0)
    WAVE_LAUNCH("estimate", (est_gather_kernel<T, D>), heads * g.est_chunks, 256, 0, st, ids2, nsel2, ids1,
                nsel1, ix.offsets, z, VS, Hq, ix.Hkv, m, mc, g.rcap2, g.rcap1, g.est_chunks, slots,
                g.steady_chunks + g.gather_chunks, scale_log2, part);
  WAVE_LAUNCH("merge", (merge_kernel<D>), heads, MERGE_THREADS, 0, st, part, g.slots, slots, out, lse);
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

template <typename T, int D>
static wave_status budget_td(int G, const void* q, const wave_index& ix, int Hq, int est_clusters,
                             float* out, float* lse, int32_t* selected, int topk, void* ws,
                             hipStream_t st) {
  switch (G) {
#define WAVE_G(n) \
  case n: return budget_tdg<T, D, n>(q, ix, Hq, est_clusters, out, lse, selected, topk, ws, st);
    WAVE_G(1) WAVE_G(2) WAVE_G(3) WAVE_G(4) WAVE_G(5) WAVE_G(6) WAVE_G(7) WAVE_G(8)
#undef WAVE_G
    default: return WAVE_ERR_SHAPE;
  }
}

// Full attention = the steady-zone kernel over all N rows of K and V, then the merge.
template <typename T, int D, int G>
static wave_status full_tdg(const void* q, const void* K, const void* V, int B, int Hkv, int N,
                            float* out, float* lse, void* ws, hipStream_t st) {
  const int units = B * Hkv, heads = units * G, chunks = full_attention_chunks(N);
  float* part = static_cast<float*>(ws);
  const float scale_log2 = kLog2e / sqrtf((float)D);
  WAVE_LAUNCH("full_attention", (steady_kernel<T, D, G>), units * chunks, 256, 0, st,
              static_cast<const T*>(q), static_cast<const T*>(K), static_cast<const T*>(V), Hkv, N, N,
              chunks, FULL_ATTN_ROWS, chunks, 0, scale_log2, part);
  WAVE_LAUNCH("merge", (merge_kernel<D>), heads, MERGE_THREADS, 0, st, part, chunks, chunks, out, lse);
  return hipGetLastError() == hipSuccess ? WAVE_OK : WAVE_ERR_HIP;
}

template <typename T, int D>
static wave_status full_td(int G, const void* q, const void* K, const void* V, int B, int Hkv, int N,
                           float* out, float* lse, void* ws, hipStream_t st) {
  switch (G) {
#define WAVE_G(n) \
  case n: return full_tdg<T, D, n>(q, K, V, B, Hkv, N, out, lse, ws, st);
    WAVE_G(1) WAVE_G(2) WAVE_G(3) WAVE_G(4) WAVE_G(5) WAVE_G(6) WAVE_G(7) WAVE_G(8)
#undef WAVE_G
    default: return WAVE_ERR_SHAPE;
  }
}

wave_status launch_full_attention(const void* q, const void* K, const void* V, int dtype, int B, int Hq,
                                  int Hkv, int N, int d, float* out, float* lse, void* ws,
                                  hipStream_t st) {
  const int G = Hq / Hkv;
  if (dtype == WAVE_BF16) {
    if (d == 128) return full_td<bf16_t, 128>(G, q, K, V, B, Hkv, N, out, lse, ws, st);
    if (d == 64) return full_td<bf16_t, 64>(G, q, K, V, B, Hkv, N, out, lse, ws, st);
  } else {
    if (d == 128) return full_td<float, 128>(G, q, K, V, B, Hkv, N, out, lse, ws, st);
    if (d == 64) return full_td<float, 64>(G, q, K, V, B, Hkv, N, out, lse, ws, st);
  }
  return WAVE_ERR_SHAPE;
}

wave_status launch_decode(const void* q, const wave_index& ix, int Hq, int topk, float* out,
                          float* lse, int32_t* selected, void* ws, hipStream_t st) {
  const int G = Hq / ix.Hkv;
  if (ix.dtype == WAVE_BF16) {
    if (ix.d == 128) return decode_td<bf16_t, 128>(G, q, ix, Hq, topk, out, lse, selected, ws, st);
    if (ix.d == 64) return decode_td<bf16_t, 64>(G, q, ix, Hq, topk, out, lse, selected, ws, st);
  } else {
    if (ix.d == 128) return decode_td<float, 128>(G, q, ix, Hq, topk, out, lse, selected, ws, st);
    if (ix.d == 64) return decode_td<float, 64>(G, q, ix, Hq, topk, out, lse, selected, ws, st);
  }
  return WAVE_ERR_SHAPE;
}

wave_status launch_decode_budget(const void* q, const wave_index& ix, int Hq, int topk, int est_clusters,
                                 float* out, float* lse, int32_t* selected, void* ws, hipStream_t st) {
  if (budget_geometry(ix, Hq, topk, est_clusters).delegate)
    return launch_decode(q, ix, Hq, topk, out, lse, selected, ws, st);
  const int G = Hq / ix.Hkv;
  if (ix.dtype == WAVE_BF16) {
    if (ix.d == 128) return budget_td<bf16_t, 128>(G, q, ix, Hq, est_clusters, out, lse, selected, topk, ws, st);
    if (ix.d == 64) return budget_td<bf16_t, 64>(G, q, ix, Hq, est_clusters, out, lse, selected, topk, ws, st);
  } else {
    if (ix.d == 128) return budget_td<float, 128>(G, q, ix, Hq, est_clusters, out, lse, selected, topk, ws, st);
    if (ix.d == 64) return budget_td<float, 64>(G, q, ix, Hq, est_clusters, out, lse, selected, topk, ws, st);
  }
  return WAVE_ERR_SHAPE;
}

}  // namespace wave
