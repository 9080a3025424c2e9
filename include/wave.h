/*
 * wave.h -- C ABI of the wave-index library for AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of the wave index of
 * "RetroInfer: A Vector Storage Engine for Scalable Long-Context LLM
 * Inference": the segmented spherical k-means that builds the cluster index
 * over a key/value cache (section "Wave Index", paragraphs "Index
 * Organization" and "Lightweight Index Construction and Updates") and the
 * decode step that replaces full attention by tripartite attention (paragraph
 * "Tripartite Attention Approximation", the estimation equations, and the
 * decode steps 1-4 of the system overview).
 *
 * Conventions
 *  - Every pointer marked DEVICE is caller-owned GPU memory; HOST pointers are
 *    ordinary host memory.  The library allocates no device memory and keeps
 *    no state between calls (the optional profiler below excepted).
 *  - Every call returns a wave_status; nothing aborts or throws.  Argument
 *    errors are found on the host before any kernel is launched.
 *  - wave_index_build and wave_attention_decode only ENQUEUE work on the given
 *    HIP stream (a hipStream_t passed as void*; NULL is the default stream).
 *    Results are valid once the caller has synchronised that stream.  Two
 *    calls that share a workspace must be ordered on one stream.
 *  - Tensors are dense, row-major, last index fastest.  dtype is the storage
 *    type of q, K, V and of the index's floating arrays.  Accumulation is
 *    fp32 in decode and fp64/fp32-MFMA in the build (see each call).
 *  - Notation follows the paper: d head dimension, N context tokens, p steady
 *    tokens (n_sink + n_local), m clusters per (sequence, KV head), r retrieved
 *    clusters, C centroids, s sizes, VS value sums, L segment length, k
 *    clusters per segment, T k-means iterations, G = Hq / Hkv.
 *  - Supported shapes: d in {64, 128}; 1 <= G <= 8; dtype f32 or bf16;
 *    clusters_per_segment <= WAVE_MAX_CLUSTERS_PER_SEGMENT (8192: one segment
 *    over a 128K-token sequence at 16 tokens per cluster, the "global k-means"
 *    of the segment-size study); N < 2^31.
 */
#ifndef WAVE_H
#define WAVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  WAVE_OK = 0,
  WAVE_ERR_ARG = 1,             /* null pointer, negative count, iters < 1, ...        */
  WAVE_ERR_SHAPE = 2,           /* unsupported d, G, k, or inconsistent dimensions     */
  WAVE_ERR_DTYPE = 3,           /* dtype not WAVE_F32 / WAVE_BF16                      */
  WAVE_ERR_WORKSPACE = 4,       /* workspace null, misaligned (256 B) or too small     */
  WAVE_ERR_STEADY_MISMATCH = 5, /* decode's n_sink/n_local differ from the index's     */
  WAVE_ERR_HIP = 6              /* a HIP runtime call or kernel launch failed          */
} wave_status;

typedef enum { WAVE_F32 = 0, WAVE_BF16 = 1 } wave_dtype;

enum { WAVE_MAX_CLUSTERS_PER_SEGMENT = 8192 };

/* Index of B x Hkv independent (sequence, KV head) units: the meta index
 * (centroid, value sum, size per cluster: "Index Organization" and the value-sum
 * equation) and the cluster-contiguous key/value rows.  Plain data; the caller
 * fills the dimension fields, calls wave_index_plan for S, m, N_idx and the
 * buffer sizes, allocates the nine buffers on the DEVICE and stores the
 * pointers.  Copying the arrays copies the index. */
typedef struct {
  int32_t dtype;                /* wave_dtype                                          */
  int32_t B, Hkv, d, N;
  int32_t n_sink, n_local;      /* steady zone: first n_sink and last n_local tokens,  */
                                /* attended by position and excluded from clustering   */
  int32_t segment_len;          /* L                                                   */
  int32_t clusters_per_segment; /* k; a ragged last segment of L_s tokens has          */
                                /* min(k, L_s) clusters                                */
  int32_t S, m, N_idx;          /* derived: segments, clusters and indexed tokens per  */
                                /* unit; N_idx = N - (steady tokens)                   */
  int32_t p;                    /* derived: steady tokens = min(N, n_sink) + local part */
  int32_t steady_capacity;      /* rows allocated per unit in k_steady and v_steady: 0  */
                                /* means p (dense); see row_capacity                    */
  void *centroids;              /* DEVICE [B,Hkv,m,d] dtype: mean of raw member keys   */
  void *vsum;                   /* DEVICE [B,Hkv,m,d] dtype: sum of member values      */
  int32_t *sizes;               /* DEVICE [B,Hkv,m]     0 = empty cluster              */
  int32_t *offsets;             /* DEVICE [B,Hkv,m+1]   rows of cluster c in k_perm /  */
                                /*        v_perm are [offsets[c], offsets[c+1])        */
                                /*        (with cluster_capacity > 0 these four have   */
                                /*        cluster_capacity (+ 1) entries per unit)     */
  int32_t *perm;                /* DEVICE [B,Hkv,N_idx] original position of each row  */
  void *k_perm, *v_perm;        /* DEVICE [B,Hkv,N_idx,d] dtype, rows ordered by       */
                                /*        (segment, cluster, original position); with  */
                                /*        row_capacity > 0 the three have row_capacity */
                                /*        rows per unit, the first N_idx in use        */
  void *k_steady, *v_steady;    /* DEVICE [B,Hkv,p,d] dtype: sink rows then local rows */
                                /*        (steady_capacity rows per unit if that is set) */
  int32_t appended_segments;    /* update segments appended by wave_index_append (0 for */
                                /* a freshly built index); they follow the S - this     */
                                /* many segments of the build                           */
  int32_t update_segment_len;   /* their length U and ...                               */
  int32_t update_clusters;      /* ... clusters per update segment (min(k_u, U) each)   */
  int32_t row_capacity;         /* rows allocated per unit in perm, k_perm and v_perm:   */
                                /* 0 means N_idx (dense); a larger value, set by the    */
                                /* caller before wave_index_plan, leaves room for       */
                                /* wave_index_append to add rows in place               */
  int32_t cluster_capacity;     /* clusters allocated per unit in centroids, vsum, sizes */
                                /* (and + 1 entries in offsets): 0 means m (dense); a    */
                                /* larger value, set by the caller before                */
                                /* wave_index_plan, leaves room for wave_index_append to */
                                /* add clusters in place; the first m (m + 1) entries of */
                                /* a unit are in use                                     */
} wave_index;

enum { WAVE_INDEX_BUFFERS = 9 };

/* Host only.  Reads the dimension fields of *ix, writes S, m, N_idx, p into it
 * and the byte size of each of the nine buffers into bytes[] in the order
 * centroids, vsum, sizes, offsets, perm, k_perm, v_perm, k_steady, v_steady.
 * build_workspace_bytes (may be NULL) receives the scratch wave_index_build
 * needs; decode_workspace_bytes (may be NULL) the scratch wave_attention_decode
 * needs for Hq query heads and topk_clusters retrieved clusters.  Sizes of
 * zero-length buffers are reported as 0; their pointers may be NULL. */
wave_status wave_index_plan(wave_index *ix, size_t bytes[WAVE_INDEX_BUFFERS],
                            size_t *build_workspace_bytes, int Hq, int topk_clusters,
                            size_t *decode_workspace_bytes);

/* Index update during decoding ("Lightweight Index Construction", last
 * paragraph): n_new new tokens per unit join the local window of the steady
 * zone; whenever the window holds a whole update segment of U tokens beyond
 * its n_local_min most recent ones, its U oldest tokens are clustered on their
 * own (as a segment of the build: same seeding rule with the segment's number,
 * same arithmetic) into min(k_u, U) clusters, which are appended to the index.
 * Nothing indexed before changes.  The result is written as a NEW index with
 * arrays of its own (this library's arrays are dense per unit, so an index with
 * more clusters has other strides); when no segment is flushed only the steady
 * rows differ from the old index.
 *
 * wave_index_append_plan (host only): fills *new_ix (dimensions, derived
 * fields; N = old N + n_new, n_local = what stays in the window), the byte
 * sizes of its nine buffers and the workspace wave_index_append needs.  An
 * index that already holds update segments takes the same U and k_u again.
 *
 * wave_index_append: old_ix read only; K_new, V_new DEVICE [B,Hkv,n_new,d]
 * dtype (may be NULL when n_new = 0); new_ix as planned, with its nine DEVICE
 * buffers (written; must not overlap old_ix's, with two exceptions: an update
 * which flushes no segment -- the plan's appended_segments equals the old one
 * -- may name old_ix's own seven arrays of the clustered part, which are then
 * left as they are; and perm, k_perm, v_perm may be old_ix's when both indexes
 * have the same row_capacity >= the new N_idx: the new rows are then written
 * behind the old ones in place and old_ix stays valid; centroids, vsum, sizes
 * and offsets may be old_ix's when both indexes have the same cluster_capacity
 * >= the new m: the new clusters are then written behind the old ones in place
 * (an update of 1K tokens then writes its 64 clusters and 1K rows per unit and
 * copies nothing that was indexed before); likewise k_steady and
 * v_steady may be old_ix's when no segment is flushed and both indexes have
 * the same steady_capacity >= the new p: only the new tokens' rows are then
 * written, behind the old window); workspace DEVICE, 256-byte aligned.  The
 * plan keeps old_ix's row_capacity, cluster_capacity and steady_capacity while
 * the grown index fits in them and reports 0 (dense) otherwise.  An array that
 * both indexes name must have the same stride per unit in both
 * (WAVE_ERR_ARG otherwise).  Errors: as wave_index_build; WAVE_ERR_SHAPE if new_ix is not the
 * plan of (old_ix, n_new, n_local_min, U, k_u) or old N < n_sink. */
wave_status wave_index_append_plan(const wave_index *old_ix, int n_new, int n_local_min,
                                   int update_segment_len, int update_clusters, wave_index *new_ix,
                                   size_t bytes[WAVE_INDEX_BUFFERS], size_t *workspace_bytes);
wave_status wave_index_append(const wave_index *old_ix, const void *K_new, const void *V_new,
                              int n_new, int n_local_min, int update_segment_len,
                              int update_clusters, int iters, uint64_t seed, wave_index *new_ix,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Index construction ("Index Organization", "Lightweight Index Construction"):
 * per unit and per segment of L tokens, spherical k-means on the centred,
 * unit-normalised keys (seeded distinct-point initialisation, `iters` rounds of
 * assign + update, ties to the lowest cluster id, empty clusters keep their
 * centroid; the partition is the one of the last assign); then per cluster its
 * size, the mean of its raw keys, the sum of its values, and the key/value rows
 * permuted so that clusters are contiguous.  Similarities are bf16 MFMA
 * products accumulated in fp32 (fp32 FMA for f32 data); any point whose two
 * best similarities are closer than the accumulation error bound is re-decided
 * in fp64; centring, normalisation, centroid updates, means and value sums
 * accumulate in fp64 and are rounded once (to nearest even) to dtype.
 *   K, V       DEVICE [B,Hkv,N,d] dtype, read only, may be released after the
 *              stream work completes
 *   ix         dimensions + planned fields + the nine DEVICE buffers (written)
 *   workspace  DEVICE, 256-byte aligned, >= build_workspace_bytes
 * From the second round on, only clusters that a point entered or left are
 * summed again (the others keep their centroid bit for bit).  bf16 segments of
 * at most 2048 tokens and 128 clusters are clustered by one workgroup each that
 * runs all rounds; WAVE_NO_SMALL_KMEANS=1 in the environment keeps them on the
 * kernels of the long segments (same result, one launch per step). */
wave_status wave_index_build(const void *K, const void *V, wave_index *ix, int iters,
                             uint64_t seed, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/* One decode step of tripartite attention for B x Hq query heads (query head
 * hq uses the index of KV head hq / G and ranks clusters on its own):
 * score every non-empty centroid against q, take the topk_clusters best
 * (ties to the lower id), attend exactly over the steady tokens and over every
 * token of the selected clusters, let each other cluster contribute
 * s_i * exp(q.C_i / sqrt(d)) to the normaliser and exp(q.C_i / sqrt(d)) * VS_i
 * to the numerator (estimation equations), and merge the zones under one
 * softmax normalisation by log-sum-exp.
 *   q          DEVICE [B,Hq,d] dtype
 *   out        DEVICE [B,Hq,d] fp32; lse DEVICE [B,Hq] fp32 = log sum of
 *              exp(scaled logits) over the three zones (natural log)
 *   selected   DEVICE [B,Hq,topk_clusters] int32 or NULL: selected cluster ids
 *              ascending, padded with -1
 *   n_sink, n_local  must equal the index's, else WAVE_ERR_STEADY_MISMATCH
 *   topk_clusters >= number of non-empty clusters retrieves everything (the
 *   result is then exact attention); 0 leaves steady + estimation only.
 * Scores accumulate in fp32; a cluster whose fp32 score lies within the
 * accumulation error bound of the selection threshold is re-scored in fp64, so
 * the selected set is the fp64 ranking's (also when thousands of scores lie
 * inside that bound: they are then ranked in fp64 without being kept, slowly).
 * One exception: a head ranked by the streaming selection (more than 131072
 * clusters per KV head, or more than 2048 clusters passing the first-stage
 * filter of the many-cluster path) AND with more than 1024 scores inside the
 * bound keeps the fp32 ranking, ties to the lower id.
 *
 * Precondition on the index (it holds for every index this library builds or
 * grows; a caller that fills the arrays itself must keep it): each stored
 * centroid is the mean of the cluster's stored key rows and each stored value
 * sum the sum of its value rows, up to one rounding to dtype.  The estimation
 * terms are computed for ALL clusters in one pass over the meta index and the
 * selected clusters' terms are taken out again; by the estimation bound
 * (s_i exp(q.C_i / sqrt(d)) <= sum over the cluster's rows of exp(q.K_j /
 * sqrt(d)) when C_i is the mean) a term that is taken out never exceeds what
 * the cluster's exact rows put in, so the cancellation costs about one fp32
 * ulp of the result.  A centroid whose logit lies delta above that bound costs
 * about exp(delta) ulps (storage rounding of a bf16 centroid: delta <=
 * 2^-8 |q| |C_i| / sqrt(d), harmless); an index that breaks the bound grossly
 * loses the retrieved part of the result to cancellation.  If the normaliser
 * itself cancels to zero or below, out and lse of that head are NaN: never a
 * silent zero. */
wave_status wave_attention_decode(const void *q, const wave_index *ix, int Hq, int topk_clusters,
                                  int n_sink, int n_local, float *out, float *lse,
                                  int32_t *selected, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/* wave_attention_decode for callers that cannot allocate device memory or hand a
 * workspace over: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and kernels as
 * wave_attention_decode, without the workspace: the step's scratch (scores,
 * selected ids, partial results) lives in a static device array of
 * WAVE_STATIC_SCRATCH_BYTES inside the library, which every GPU the library
 * runs on holds from the first call on it until the process ends.  The call
 * allocates and frees nothing.  A step whose scratch would not fit (the size is
 * what wave_index_plan reports as decode_workspace_bytes) is refused with
 * WAVE_ERR_WORKSPACE before anything is launched; the five benchmark workloads
 * fit (the largest, 64 sequences x 28 query heads x 4096 clusters, needs 47 MB).
 * All calls on one GPU share the one array: calls that overlap in time on the
 * same GPU (two streams, two threads) race; order them on one stream or by
 * events.  Nothing in the array has to be zero when a step starts, so nothing is
 * cleared between calls.  wave_attention_decode_static_capacity returns
 * WAVE_STATIC_SCRATCH_BYTES. */
#define WAVE_STATIC_SCRATCH_BYTES (64u << 20)
size_t wave_attention_decode_static_capacity(void);
wave_status wave_attention_decode_static(const void *q, const wave_index *ix, int Hq,
                                         int topk_clusters, int n_sink, int n_local, float *out,
                                         float *lse, int32_t *selected, void *hip_stream);

/* The decode step with a budget for the estimation zone, as in the paper's
 * evaluation (parameter paragraph: an estimation zone of 23.2 % of the clusters
 * so that the three zones cover about a quarter of the context) and its
 * ablation without estimation: of the clusters that are not retrieved, only the
 * est_clusters best-scoring ones (same ranking and tie rule as the retrieval)
 * enter through their centroid, size and value sum; the others are ignored.
 * est_clusters < 0, or a budget that reaches every cluster, is
 * wave_attention_decode itself; est_clusters = 0 leaves the exact zones only.
 * Same arguments otherwise; the workspace size comes from
 * wave_attention_decode_budget_workspace (0 if the arguments are invalid).
 * Up to 65536 clusters per KV head it runs in four launches (scores with the
 * steady zone, both selections at once, retrieval with estimation, merge);
 * beyond that its steps are launches of their own.  Every head reads its own
 * estimated clusters' value sums, so a budget moves about as many bytes as
 * estimating every cluster once per KV head and is not faster than
 * wave_attention_decode. */
size_t wave_attention_decode_budget_workspace(const wave_index *ix, int Hq, int topk_clusters,
                                              int est_clusters);
wave_status wave_attention_decode_budget(const void *q, const wave_index *ix, int Hq,
                                         int topk_clusters, int est_clusters, int n_sink,
                                         int n_local, float *out, float *lse, int32_t *selected,
                                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Full decode attention, the operation the wave index approximates (the
 * attention equation of the background section): for every query head,
 * o = softmax(q K^T / sqrt(d)) V over all N tokens of its KV head, by streaming
 * K and V once per KV head with an online softmax (fp32 accumulation) and one
 * log-sum-exp merge.  It is the same-hardware baseline for the decode step and
 * the limit wave_attention_decode reaches when every cluster is retrieved.
 *   q          DEVICE [B,Hq,d] dtype;  K, V  DEVICE [B,Hkv,N,d] dtype
 *   out        DEVICE [B,Hq,d] fp32;   lse   DEVICE [B,Hq] fp32 (natural log)
 *   workspace  DEVICE, 256-byte aligned, >= wave_full_attention_workspace(...)
 * wave_full_attention_workspace returns 0 for unsupported shapes. */
size_t wave_full_attention_workspace(int B, int Hq, int N, int d);
wave_status wave_full_attention_decode(const void *q, const void *K, const void *V, int dtype, int B,
                                       int Hq, int Hkv, int N, int d, float *out, float *lse,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Test hook, host only: the k_s distinct seed-token indices (relative to the
 * segment start) with which segment s of unit (b, h) starts k-means: the first
 * k_s entries of a Fisher-Yates shuffle of 0..L_s-1 driven by splitmix64 keyed
 * on (seed, b, h, s).  out: HOST [k_s]. */
wave_status wave_init_indices(uint64_t seed, int b, int h, int s, int L_s, int k_s, int32_t *out);

/* Test hook: one assign step of the build on one segment, with the build's
 * own kernels.  xhat DEVICE [L_s,d] dtype (normalised keys), chat DEVICE
 * [k_s,d] dtype (centroids), assign DEVICE [L_s] int32 (written).
 * workspace DEVICE >= 4*L_s + 1024 bytes, 256-byte aligned. */
wave_status wave_kmeans_assign_step(const void *xhat, const void *chat, int dtype, int L_s, int k_s,
                                    int d, int32_t *assign, void *workspace,
                                    size_t workspace_bytes, void *hip_stream);

/* Calibration: plain streaming kernels over a buffer of known size, for the
 * callers that measure (the benchmark and profiler runs): a profiler counter read
 * for them gives the factor between its unit and bytes, and their rate is the
 * bandwidth a simple kernel reaches on the machine.  src, dst DEVICE, 16-byte
 * aligned, `bytes` a multiple of 16; `workgroups` of 256 threads stride over the
 * buffer.  copy reads src and writes dst; read only reads src (sink: DEVICE, at
 * least 4 bytes, practically never written). */
wave_status wave_calibration_copy(void *dst, const void *src, size_t bytes, int workgroups,
                                  void *hip_stream);
wave_status wave_calibration_read(const void *src, size_t bytes, void *sink, int workgroups,
                                  void *hip_stream);

/* Profiler (the library's only global state).  While enabled, every kernel the
 * library launches is bracketed by HIP events on its stream.
 * wave_profile_read synchronises, adds up the elapsed time per kernel name
 * since the last read and writes up to `cap` entries: names[i] points to a
 * static string, total_ms[i] and launches[i] to the sums.  Returns the number
 * of distinct kernels, or -1 on a HIP error. */
wave_status wave_profile_enable(int on);
int wave_profile_read(const char **names, float *total_ms, int *launches, int cap);

const char *wave_status_string(wave_status st);

#ifdef __cplusplus
}
#endif
#endif /* WAVE_H */
