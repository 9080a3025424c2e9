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
#include "wave_common.h"

namespace wave {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no logit seen yet"

// ============================================================================
// 1. Centroid scoring: z[b, hq, c] = q[b, hq] . C[b, hkv, c], empty clusters -inf.
//    One workgroup streams a contiguous range of one unit's centroids for all G
//    query heads of that KV head.  It also reports the largest squared centroid
//    norm of its range (the selection step turns it into an error bound).
// ============================================================================
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void score_kernel(const T* __restrict__ q, const T* __restrict__ C,
                                                    const int32_t* __restrict__ sizes,
                                                    float* __restrict__ z, float* __restrict__ cn2part,
                                                    int Hkv, int m, int chunks, int rows_per_chunk) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW, U = 4;
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int unit = wg / chunks, chunk = wg - unit * chunks;
  const int b = unit / Hkv, h = unit - b * Hkv, Hq = Hkv * G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;

  float qf[G][EPC];
#pragma unroll
  for (int g = 0; g < G; ++g)
    unpack<T>(load16(q + ((size_t)(b * Hq + h * G + g) * D + sub * EPC)), qf[g]);

  const int c0 = chunk * rows_per_chunk;
  const int c1 = min(m, c0 + rows_per_chunk);
  const T* Cu = C + (size_t)unit * m * D + sub * EPC;
  const int32_t* su = sizes + (size_t)unit * m;
  float cn2 = 0.f;

  for (int c = c0 + grp; c < c1; c += GROUPS * U) {
    uint4 raw[U];
    int sz[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cc = min(c + u * GROUPS, c1 - 1);
      raw[u] = load16(Cu + (size_t)cc * D);
      sz[u] = su[cc];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cc = c + u * GROUPS;
      float cf[EPC];
      unpack<T>(raw[u], cf);
      float n2 = 0.f, s[G];
#pragma unroll
      for (int e = 0; e < EPC; ++e) n2 = fmaf(cf[e], cf[e], n2);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) a = fmaf(qf[g][e], cf[e], a);
        s[g] = group_sum<LPR>(a);
      }
      n2 = group_sum<LPR>(n2);
      cn2 = fmaxf(cn2, n2);
      float mine = s[0];
#pragma unroll
      for (int g = 1; g < G; ++g) mine = (sub == g) ? s[g] : mine;
      if (cc < c1 && sub < G)
        z[(size_t)(b * Hq + h * G + sub) * m + cc] = sz[u] > 0 ? mine : -INFINITY;
    }
  }

  __shared__ float red[4];
  cn2 = wave_max(cn2);
  if (lane == 0) red[wave] = cn2;
  __syncthreads();
  if (threadIdx.x == 0)
    cn2part[(size_t)unit * chunks + chunk] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// ============================================================================
// 2. Top-r selection per query head.
//    Radix select (4 passes of 8 bits) on the order-preserving integer image of
//    the fp32 scores gives the r-th largest score tau.  Scores accumulate in
//    fp32, so clusters within the accumulation error bound of tau are re-scored
//    in fp64 and ranked exactly (ties to the lower id).  Outputs: a bitmap of
//    the selected clusters, their ids ascending, the running token count of the
//    selected clusters, and the reference score for the estimation zone.
// ============================================================================
constexpr int SEL_THREADS = 512;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int CAND_CAP = 1024;

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Exclusive prefix sum of one int per thread across the workgroup; returns the
// thread's prefix and the total through `total`.  scratch: SEL_WAVES + 1 ints.
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
  for (int w = 0; w < SEL_WAVES; ++w) {
    const int s = scratch[w];
    if (w < wave) base += s;
    tot += s;
  }
  total = tot;
  return base + inc - v;
}

__device__ __forceinline__ int block_sum_i(int v, int* scratch) {
  int t;
  block_excl_scan(v, scratch, t);
  return t;
}

template <typename T, int D>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    const T* __restrict__ q, const T* __restrict__ C, const int32_t* __restrict__ offsets,
    const float* __restrict__ z, const float* __restrict__ cn2part, int cn2_chunks, int Hq, int Hkv,
    int m, int r, int rcap, int mwords, int usel_stride, int32_t* __restrict__ sel_ids,
    int32_t* __restrict__ sel_pref, int32_t* __restrict__ sel_row, uint32_t* __restrict__ bitmap, float* __restrict__ zref_out,
    int32_t* __restrict__ nsel_out, int32_t* __restrict__ user_selected) {
  const int bh = blockIdx.x;  // b * Hq + hq
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* zz = z + (size_t)bh * m;
  const int32_t* off = offsets + (size_t)unit * (m + 1);
  int32_t* ids = sel_ids + (size_t)bh * rcap;
  int32_t* pref = sel_pref + (size_t)bh * (rcap + 1);
  uint32_t* bits = bitmap + (size_t)bh * mwords;
  int32_t* usel = user_selected ? user_selected + (size_t)bh * usel_stride : nullptr;
  int32_t* srow = sel_row + (size_t)bh * rcap;

  __shared__ int hist[256];
  __shared__ int scan_scratch[SEL_WAVES + 1];
  __shared__ float fred[SEL_WAVES];
  __shared__ int cand_id[CAND_CAP];
  __shared__ double cand_z[CAND_CAP];
  __shared__ int sh_i[4];
  __shared__ float sh_f[2];

  // ---- valid count and maximum -------------------------------------------
  int nv = 0;
  float zmax = -INFINITY;
  for (int i = tid; i < m; i += SEL_THREADS) {
    const float v = zz[i];
    nv += (v > -INFINITY) ? 1 : 0;
    zmax = fmaxf(zmax, v);
  }
  zmax = wave_max(zmax);
  if (lane == 0) fred[wave] = zmax;
  const int nvalid = block_sum_i(nv, scan_scratch);  // contains the barriers that publish fred
  zmax = fred[0];
#pragma unroll
  for (int w = 1; w < SEL_WAVES; ++w) zmax = fmaxf(zmax, fred[w]);
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
      for (int i = tid; i < m; i += SEL_THREADS) {
        const uint32_t k = order_key(zz[i]);
        if ((k & pmask) == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
      }
      __syncthreads();
      // thread t (< 256) learns how many keys have a digit above t
      int above = 0;
      if (tid < 256) {
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
    for (int i = tid; i < D; i += SEL_THREADS) {
      const float v = to_f32(q[(size_t)bh * D + i]);
      qn2 += v * v;
    }
    qn2 = wave_sum_f(qn2);
    __syncthreads();
    if (lane == 0) fred[wave] = qn2;
    __syncthreads();
    if (tid == 0) {
      float s = 0.f;
      for (int w = 0; w < SEL_WAVES; ++w) s += fred[w];
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
    for (int i = tid; i < m; i += SEL_THREADS) {
      const float v = zz[i];
      if (v > hi) {
        ++n_hi;
      } else if (v >= lo) {
        const int slot = atomicAdd(&sh_i[2], 1);
        if (slot < CAND_CAP) cand_id[slot] = i;
      }
    }
    n_hi = block_sum_i(n_hi, scan_scratch);
    n_cand = sh_i[2];
    need = r_eff - n_hi;
    if (n_cand > CAND_CAP) {
      mode = 3;  // too many near-equal scores: keep the fp32 ranking
    } else if (n_cand == need) {
      mode = 2;  // the whole band is taken; no ranking needed
    } else {
      mode = 2;
      // exact fp64 scores of the candidates
      const T* Cu = C + (size_t)unit * m * D;
      for (int i = tid; i < n_cand; i += SEL_THREADS) {
        const T* row = Cu + (size_t)cand_id[i] * D;
        double acc = 0.0;
        for (int e = 0; e < D; ++e) acc = fma(to_f64(q[(size_t)bh * D + e]), to_f64(row[e]), acc);
        cand_z[i] = acc;
      }
      __syncthreads();
      for (int i = tid; i < n_cand; i += SEL_THREADS) {
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
  // Each thread owns whole 32-cluster words, so no atomics are needed except
  // for the few band candidates added afterwards.
  int eq_before = 0;
  if (mode == 3) {
    // exclusive count of score == tau before each thread's word range
    int cnt = 0;
    const int words_per = (mwords + SEL_THREADS - 1) / SEL_THREADS;
    const int w0 = tid * words_per, w1 = min(mwords, w0 + words_per);
    for (int w = w0; w < w1; ++w)
      for (int j = 0; j < 32; ++j) {
        const int i = w * 32 + j;
        if (i < m && zz[i] == tau) ++cnt;
      }
    int tot;
    eq_before = block_excl_scan(cnt, scan_scratch, tot);
  }
  {
    const int words_per = (mwords + SEL_THREADS - 1) / SEL_THREADS;
    const int w0 = tid * words_per, w1 = min(mwords, w0 + words_per);
    int eq_seen = eq_before;
    for (int w = w0; w < w1; ++w) {
      uint32_t word = 0;
      if (mode != 0) {
        for (int j = 0; j < 32; ++j) {
          const int i = w * 32 + j;
          if (i >= m) break;
          const float v = zz[i];
          bool on;
          if (mode == 1) {
            on = v > -INFINITY;
          } else if (mode == 2) {
            on = v > hi;
          } else {
            on = v > tau;
            if (v == tau) {
              on = eq_seen < need_eq;
              ++eq_seen;
            }
          }
          word |= on ? (1u << j) : 0u;
        }
      }
      bits[w] = word;
    }
  }
  __syncthreads();
  if (mode == 2) {
    for (int i = tid; i < n_cand; i += SEL_THREADS) {
      const int id = cand_id[i];
      if (id >= 0) atomicOr(&bits[id >> 5], 1u << (id & 31));
    }
    __syncthreads();
  }

  // ---- ascending id list and running token counts -----------------------------
  {
    const int words_per = (mwords + SEL_THREADS - 1) / SEL_THREADS;
    const int w0 = tid * words_per, w1 = min(mwords, w0 + words_per);
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
    int pos = block_excl_scan(cnt, scan_scratch, nsel);
    int tpos = block_excl_scan(tok, scan_scratch, ntok);
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
    for (int i = nsel + tid; i < rcap; i += SEL_THREADS) ids[i] = -1;
    if (usel)
      for (int i = nsel + tid; i < usel_stride; i += SEL_THREADS) usel[i] = -1;
    if (tid == 0) {
      nsel = min(nsel, rcap);
      pref[nsel] = ntok;
      nsel_out[bh] = nsel;
      // reference score of the estimation zone: every estimated cluster scores <= it
      float ref = 0.f;
      if (nvalid > 0) ref = (mode == 2 || mode == 3) ? fminf(hi, zmax) : zmax;
      zref_out[bh] = ref;
    }
  }
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
template <typename T, int D, int NG>
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
  // across the 4 waves through LDS: smem[wave][g][D + 2]
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
  for (int idx = threadIdx.x; idx < NG * STR; idx += 256) {
    const int g = idx / STR, e = idx - g * STR;
    float m4[4], mn = kNegBig;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      m4[w] = smem[(size_t)(w * NG + g) * STR];
      mn = fmaxf(mn, m4[w]);
    }
    float v;
    if (e == 0) {
      v = mn;
    } else {
      v = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) v += smem[(size_t)(w * NG + g) * STR + e] * exp2f(m4[w] - mn);
    }
    part_base[(size_t)g * head_stride + e] = v;
  }
}

// ============================================================================
// 3a. Retrieval zone: one workgroup handles one slice of the tokens of the
//     clusters selected by one query head, reading them in place from the
//     cluster-contiguous K/V.
// ============================================================================
constexpr int GATHER_TILE = 256;
constexpr int GATHER_STAGE = 2048;  // selected clusters whose ranges are staged in LDS

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_kernel(
    const T* __restrict__ q, const T* __restrict__ k_perm, const T* __restrict__ v_perm,
    const int32_t* __restrict__ sel_pref, const int32_t* __restrict__ sel_row,
    const int32_t* __restrict__ nsel_arr, int Hq, int Hkv, int N_idx, int rcap, int chunks,
    int slots, float scale_log2, float* __restrict__ part) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW, U = 4;
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int bh = wg / chunks, chunk = wg - bh * chunks;
  const int b = bh / Hq, hq = bh - b * Hq, G = Hq / Hkv;
  const int unit = b * Hkv + hq / G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;

  __shared__ int rowidx[GATHER_TILE];
  __shared__ int s_pref[GATHER_STAGE + 1];
  __shared__ int s_row[GATHER_STAGE];
  __shared__ float smem[4 * (D + 2)];

  const int nsel = nsel_arr[bh];
  const int32_t* gpref = sel_pref + (size_t)bh * (rcap + 1);
  const int32_t* grow = sel_row + (size_t)bh * rcap;
  const int total = gpref[nsel];
  const int per = (total + chunks - 1) / chunks;
  const int t0 = min(total, chunk * per), t1 = min(total, t0 + per);

  // The token range [t0, t1) of the concatenated selected clusters maps to rows
  // through (running token count, first row) per selected cluster.
  const bool staged = nsel <= GATHER_STAGE;
  if (staged && t0 < t1) {
    for (int i = threadIdx.x; i <= nsel; i += 256) s_pref[i] = gpref[i];
    for (int i = threadIdx.x; i < nsel; i += 256) s_row[i] = grow[i];
  }
  const int32_t* pref = staged ? s_pref : gpref;
  const int32_t* srow = staged ? s_row : grow;

  AttnState<T, D, 1> st;
  st.init(q + (size_t)bh * D, sub, scale_log2);
  const T* Ku = k_perm + (size_t)unit * N_idx * D + sub * EPC;
  const T* Vu = v_perm + (size_t)unit * N_idx * D + sub * EPC;

  for (int base = t0; base < t1; base += GATHER_TILE) {
    const int n = min(GATHER_TILE, t1 - base);
    __syncthreads();
    if ((int)threadIdx.x < n) {
      const int t = base + threadIdx.x;
      int a = 0, e = nsel;  // largest a with pref[a] <= t
      while (e - a > 1) {
        const int mid = (a + e) >> 1;
        if (pref[mid] <= t) a = mid; else e = mid;
      }
      rowidx[threadIdx.x] = srow[a] + (t - pref[a]);
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
        kraw[u] = load16(Ku + (size_t)row * D);
        vraw[u] = load16(Vu + (size_t)row * D);
      }
      st.template rows<U, LPR>(kraw, vraw, valid);
    }
  }
  __syncthreads();
  merge_groups_and_store<T, D, 1>(st, smem, part + ((size_t)bh * slots + chunk) * (D + 2), 0);
}

// ============================================================================
// 3b. Steady zone: sink + local rows of one unit, shared by its G query heads.
// ============================================================================
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void steady_kernel(const T* __restrict__ q,
                                                     const T* __restrict__ k_steady,
                                                     const T* __restrict__ v_steady, int Hkv, int p,
                                                     int chunks, int rows_per_chunk, int slots,
                                                     int slot0, float scale_log2,
                                                     float* __restrict__ part) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW;
  constexpr int U = (G <= 4) ? 4 : 2;
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int unit = wg / chunks, chunk = wg - unit * chunks;
  const int b = unit / Hkv, h = unit - b * Hkv, Hq = Hkv * G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  __shared__ float smem[4 * G * (D + 2)];

  const int bh0 = b * Hq + h * G;
  AttnState<T, D, G> st;
  st.init(q + (size_t)bh0 * D, sub, scale_log2);
  const T* Ku = k_steady + (size_t)unit * p * D + sub * EPC;
  const T* Vu = v_steady + (size_t)unit * p * D + sub * EPC;
  const int r0 = chunk * rows_per_chunk, r1 = min(p, r0 + rows_per_chunk);
  for (int i = r0 + grp; i < r1; i += GROUPS * U) {
    uint4 kraw[U], vraw[U];
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ii = i + u * GROUPS;
      valid[u] = ii < r1;
      const int row = valid[u] ? ii : i;
      kraw[u] = load16(Ku + (size_t)row * D);
      vraw[u] = load16(Vu + (size_t)row * D);
    }
    st.template rows<U, LPR>(kraw, vraw, valid);
  }
  merge_groups_and_store<T, D, G>(st, smem, part + ((size_t)bh0 * slots + slot0 + chunk) * (D + 2),
                                  (size_t)slots * (D + 2));
}

// ============================================================================
// 3c. Estimation zone: every non-empty cluster that the head did not select
//     adds s_c * w_c to the normaliser and w_c * VS_c to the numerator, with
//     w_c = exp(q.C_c / sqrt(d)) taken relative to a fixed reference so that
//     partial sums of different workgroups add up directly.
// ============================================================================
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void est_kernel(const T* __restrict__ vsum,
                                                  const int32_t* __restrict__ sizes,
                                                  const float* __restrict__ z,
                                                  const uint32_t* __restrict__ bitmap,
                                                  const float* __restrict__ zref, int Hkv, int m,
                                                  int mwords, int chunks, int rows_per_chunk,
                                                  int slots, int slot0, float scale_log2,
                                                  float* __restrict__ part) {
  constexpr int EPC = Elem<T>::EPC, LPR = D / EPC, RPW = 64 / LPR, GROUPS = 4 * RPW, U = 4;
  const int wg = xcd_logical_block(blockIdx.x, gridDim.x);
  const int unit = wg / chunks, chunk = wg - unit * chunks;
  const int b = unit / Hkv, h = unit - b * Hkv, Hq = Hkv * G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, grp = wave * RPW + lane / LPR;
  __shared__ float smem[4 * G * (D + 2)];

  const int bh0 = b * Hq + h * G;
  float ref2[G], l[G], acc[G][EPC];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    ref2[g] = zref[bh0 + g] * scale_log2;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[g][e] = 0.f;
  }
  const T* Vu = vsum + (size_t)unit * m * D + sub * EPC;
  const int32_t* su = sizes + (size_t)unit * m;
  const int c0 = chunk * rows_per_chunk, c1 = min(m, c0 + rows_per_chunk);

  for (int c = c0 + grp; c < c1; c += GROUPS * U) {
    uint4 raw[U];
    int sz[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cc = min(c + u * GROUPS, c1 - 1);
      raw[u] = load16(Vu + (size_t)cc * D);
      sz[u] = (c + u * GROUPS < c1) ? su[cc] : 0;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cc = min(c + u * GROUPS, c1 - 1);
      float vf[EPC];
      unpack<T>(raw[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const size_t bh = bh0 + g;
        const uint32_t word = bitmap[bh * mwords + (cc >> 5)];
        const bool use = sz[u] > 0 && !((word >> (cc & 31)) & 1u);
        const float zc = z[bh * m + cc];
        const float w = use ? exp2f(fmaf(zc, scale_log2, -ref2[g])) : 0.f;
        l[g] = fmaf((float)sz[u], w, l[g]);
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[g][e] = fmaf(w, vf[e], acc[g][e]);
      }
    }
  }
  // all groups share the reference: plain sums
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      l[g] += __shfl_xor(l[g], off);
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] += __shfl_xor(acc[g][e], off);
    }
  }
  constexpr int STR = D + 2;
  if (lane < LPR) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float* dst = smem + (size_t)(wave * G + g) * STR;
#pragma unroll
      for (int e = 0; e < EPC; ++e) dst[2 + sub * EPC + e] = acc[g][e];
      if (sub == 0) dst[1] = l[g];
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * STR; idx += 256) {
    const int g = idx / STR, e = idx - g * STR;
    float v;
    if (e == 0) {
      v = zref[bh0 + g] * scale_log2;
    } else {
      v = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) v += smem[(size_t)(w * G + g) * STR + e];
    }
    part[((size_t)(bh0 + g) * slots + slot0 + chunk) * STR + e] = v;
  }
}

// ============================================================================
// 4. Merge: one normalisation over the partial results of the three zones.
// ============================================================================
template <int D>
__global__ __launch_bounds__(D) void merge_kernel(const float* __restrict__ part, int slots,
                                                  float* __restrict__ out, float* __restrict__ lse) {
  constexpr int STR = D + 2;
  const int bh = blockIdx.x, e = threadIdx.x;
  const float* p = part + (size_t)bh * slots * STR;
  float M = kNegBig;
  for (int s = 0; s < slots; ++s)
    if (p[(size_t)s * STR + 1] > 0.f) M = fmaxf(M, p[(size_t)s * STR]);
  float Z = 0.f, A = 0.f;
  for (int s = 0; s < slots; ++s) {
    const float ls = p[(size_t)s * STR + 1];
    if (ls > 0.f) {
      const float w = exp2f(p[(size_t)s * STR] - M);
      Z = fmaf(ls, w, Z);
      A = fmaf(p[(size_t)s * STR + 2 + e], w, A);
    }
  }
  out[(size_t)bh * D + e] = Z > 0.f ? A / Z : 0.f;
  if (e == 0) lse[bh] = Z > 0.f ? (M + log2f(Z)) * kLn2 : -INFINITY;
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
  g.score_rows = 512;
  g.score_chunks = m > 0 ? (m + g.score_rows - 1) / g.score_rows : 0;
  g.est_rows = 512;
  g.est_chunks = g.score_chunks;
  g.steady_rows = 256;
  g.steady_chunks = ix.p > 0 ? (ix.p + g.steady_rows - 1) / g.steady_rows : 0;
  const int r = m > 0 ? (topk < m ? topk : m) : 0;
  g.rcap = r > 0 ? r : 1;
  double expect = m > 0 ? (double)r * (double)ix.N_idx / (double)m : 0.0;
  int gc = (int)((expect + GATHER_TILE - 1) / GATHER_TILE);
  if (gc < 1) gc = 1;
  if (gc > 256) gc = 256;
  g.gather_chunks = (m > 0 && r > 0) ? gc : 0;
  g.slots = g.gather_chunks + g.steady_chunks + g.est_chunks;
  if (g.slots < 1) g.slots = 1;
  g.mwords = (m + 31) / 32;
  size_t o = 0;
  g.off_z = o;       o = align_up(o + sizeof(float) * (size_t)heads * (m > 0 ? m : 1));
  g.off_cn2 = o;     o = align_up(o + sizeof(float) * (size_t)units * (g.score_chunks > 0 ? g.score_chunks : 1));
  g.off_sel = o;     o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap);
  g.off_pref = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * (g.rcap + 1));
  g.off_srow = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads * g.rcap);
  g.off_bitmap = o;  o = align_up(o + sizeof(uint32_t) * (size_t)heads * (g.mwords > 0 ? g.mwords : 1));
  g.off_zref = o;    o = align_up(o + sizeof(float) * (size_t)heads);
  g.off_nsel = o;    o = align_up(o + sizeof(int32_t) * (size_t)heads);
  g.off_part = o;    o = align_up(o + sizeof(float) * (size_t)heads * g.slots * (D + 2));
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
  float* zref = reinterpret_cast<float*>(w + g.off_zref);
  int32_t* nsel = reinterpret_cast<int32_t*>(w + g.off_nsel);
  float* part = reinterpret_cast<float*>(w + g.off_part);
  const T* q = static_cast<const T*>(q_);
  const int units = ix.B * ix.Hkv, heads = ix.B * Hq, m = ix.m;
  const float scale_log2 = kLog2e / sqrtf((float)D);
  const int r = m > 0 ? (topk < m ? topk : m) : 0;

  if (m > 0) {
    WAVE_LAUNCH("score", (score_kernel<T, D, G>), units * g.score_chunks, 256, 0, st, q,
                static_cast<const T*>(ix.centroids), ix.sizes, z, cn2, ix.Hkv, m, g.score_chunks,
                g.score_rows);
    WAVE_LAUNCH("select", (select_kernel<T, D>), heads, SEL_THREADS, 0, st, q,
                static_cast<const T*>(ix.centroids), ix.offsets, z, cn2, g.score_chunks, Hq, ix.Hkv,
                m, r, g.rcap, g.mwords, topk, sel, pref, srow, bitmap, zref, nsel, selected);
    if (g.gather_chunks > 0)
      WAVE_LAUNCH("gather", (gather_kernel<T, D>), heads * g.gather_chunks, 256, 0, st, q,
                  static_cast<const T*>(ix.k_perm), static_cast<const T*>(ix.v_perm), pref, srow,
                  nsel, Hq, ix.Hkv, ix.N_idx, g.rcap, g.gather_chunks, g.slots, scale_log2, part);
    WAVE_LAUNCH("estimate", (est_kernel<T, D, G>), units * g.est_chunks, 256, 0, st,
                static_cast<const T*>(ix.vsum), ix.sizes, z, bitmap, zref, ix.Hkv, m, g.mwords,
                g.est_chunks, g.est_rows, g.slots, g.gather_chunks + g.steady_chunks, scale_log2,
                part);
  }
  if (m == 0 && selected && topk > 0) {
    const size_t n = (size_t)heads * topk;  // no clusters exist: nothing is selected
    WAVE_LAUNCH("fill", fill_i32_kernel, (unsigned)((n + 255) / 256), 256, 0, st, selected, n, -1);
  }
  if (g.steady_chunks > 0)
    WAVE_LAUNCH("steady", (steady_kernel<T, D, G>), units * g.steady_chunks, 256, 0, st, q,
                static_cast<const T*>(ix.k_steady), static_cast<const T*>(ix.v_steady), ix.Hkv, ix.p,
                g.steady_chunks, g.steady_rows, g.slots, g.gather_chunks, scale_log2, part);
  WAVE_LAUNCH("merge", (merge_kernel<D>), heads, D, 0, st, part,
              g.gather_chunks + g.steady_chunks + g.est_chunks, out, lse);
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

}  // namespace wave
