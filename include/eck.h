/*
 * eck.h -- C ABI of libeck: batched energy-cost-model evaluation for
 * search-based kernel compilation (arXiv 2411.18873), native to MI355X (gfx950).
 *
 * The paper's search round (Alg. 1) is: reproduce a generation of candidate
 * kernels, keep the low-latency ones, pick among them those of least predicted
 * energy with a learned cost model, measure the picked ones, refit the model,
 * and adapt how many to measure next.  This library runs the data-parallel
 * part of that round on one GPU for millions of candidates at once:
 *
 *   candidate_enumerate -> features_compute -> costmodel_score (energy model,
 *   latency model) -> topk_select            [+ costmodel_update when measured
 *   energies arrive]
 *
 * Conventions
 *   - Plain C, every function returns int32_t: ECK_OK or a negative ECK_E*.
 *   - All arguments are validated on the host before anything is launched; an
 *     error return means nothing was enqueued and no output was touched.
 *   - "device" pointers are HIP device memory owned by the caller (the library
 *     never frees or keeps them); "host" pointers are ordinary memory.
 *   - Kernels are enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronises unless its comment says so.
 *   - Results that depend on device data (count, snr, loss) are written to
 *     device memory, never returned through the host.
 *   - Matrices over candidates are structure-of-arrays: row r of a [R][ld]
 *     array is at base + r*ld elements, candidate i at column i, ld >= n.
 *   - There is no CPU fallback: without a usable GPU the compute calls return
 *     ECK_EDEVICE.
 *   - Handles (eck_space, eck_model, eck_trees) belong to the device that was
 *     current when they were created and are not synchronised internally: a
 *     space uploads its tables on first use, models change under update calls.
 *     Calls on one handle from several host threads must be serialised by the
 *     caller; different handles are independent.
 */
#ifndef ECK_H
#define ECK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ECK_OK 0
#define ECK_EINVAL (-1)       /* null pointer, zero size, value out of range */
#define ECK_ESHAPE (-2)       /* sizes inconsistent with each other (ld < n, k > segment, widths) */
#define ECK_EUNSUPPORTED (-3) /* valid request this build has no kernel for */
#define ECK_EALIGN (-4)       /* pointer or leading dimension not aligned as required */
#define ECK_EWORKSPACE (-5)   /* workspace missing or too small */
#define ECK_EDEVICE (-6)      /* HIP runtime error (no device, allocation or launch failure) */

/* operator kinds */
#define ECK_OP_GEMM 0   /* dim = {1, M, N, K} */
#define ECK_OP_BGEMM 1  /* dim = {B, M, N, K} */
#define ECK_OP_CONV2D 2 /* dim = {N, C, K, H, W, R, S, stride | pad << 16} (NCHW, square stride/pad) */

/* schedule-space kinds */
#define ECK_SPACE_KNOB 0  /* genes: tile_M, tile_N in {16..256}, tile_K in {8..64}, threads in {64..512},
                             unroll in {1,2,4,8}, vec in {1,2,4,8}; GEMM/BGEMM only */
#define ECK_SPACE_SPLIT 1 /* one gene per split axis (index into the table of ordered 4-way factorisations of
                             the axis extent, lexicographic), then unroll in {1,2,4,8,16}, vec in {1,2,4,8}.
                             Axis order: GEMM (M,N,K); BGEMM (B,M,N,K); CONV2D (N,K,H_out,W_out,C).
                             The reduction axis is staged through shared memory: f0 = stage loop,
                             f1*f2*f3 = elements per stage */
#define ECK_SPACE_SPLIT_XRED 2 /* the same genes and tables as SPLIT, read as a schedule that splits the
                             reduction across threads (the shape reduction-dominated operators need, such as
                             the matrix-vector products of Sec. 7.2): reduction axis f0 = stage loop,
                             f1 = threads sharing one output's reduction, f2*f3 = serial per thread; no
                             staging, every thread loads its own slice; the f1 partial sums of an output are
                             folded by a halving tree in shared memory (fp32).  Same 64 feature slots */

/* enumeration modes */
#define ECK_MODE_EXHAUSTIVE 0
#define ECK_MODE_SAMPLE 1
#define ECK_MODE_MUTATE 2
#define ECK_MODE_CROSSOVER 3

/* element types of feature matrices and models */
#define ECK_F32 0
#define ECK_BF16 1

/* selection modes */
#define ECK_SELECT_THRESHOLD 0
#define ECK_SELECT_RANK 1

#define ECK_MAX_GENES 16
#define ECK_MAX_K 4096 /* largest k topk_select accepts */
#define ECK_MAX_BATCH 128 /* most spaces one *_batch call takes */

/* The tensor operator being compiled plus the parameters of the GPU the
 * candidate kernels are meant for (they enter the occupancy features; the
 * paper's case study, Sec. 8, reasons with the number of multiprocessors). */
typedef struct {
    int32_t op;
    int32_t dim[8];
    int32_t elem_bytes; /* 2 or 4 */
    int32_t hw_num_cu, hw_wave, hw_lds_bytes, hw_max_threads_cu, hw_max_blocks_cu;
} eck_problem;

typedef struct eck_space eck_space; /* schedule space of one problem (host tables + device copy) */
typedef struct eck_model eck_model; /* cost model: fp32 master weights, Adam moments, packed bf16 weights */

/* ------------------------------------------------------------------ spaces */

/* Build the schedule space of `problem` (Sec. 2.2: the hierarchical search
 * space of an auto-scheduler; Sec. 5.3: kernels represented through loops).
 * Host-only work; the device copy of the tables is made lazily by the first
 * call that launches a kernel.  Every axis extent must be in [1, 65535], every
 * factorisation table at most 65535 entries, and 2*outputs*reduction < 2^48.
 * Errors: ECK_EINVAL (null, bad op/kind/elem_bytes/hw fields, zero extents),
 * ECK_EUNSUPPORTED (KNOB space on a convolution, limits above exceeded). */
int32_t eck_space_create(const eck_problem *problem, int32_t kind, eck_space **out);

/* Makes the device copy of the space's parameters and tables now, on the
 * current device, instead of inside the first call that launches a kernel: one
 * hipMalloc and one synchronous host-to-device copy (at most a few hundred KB).
 * For callers that must not allocate or synchronise later on -- code under HIP
 * graph capture, timed loops.  Does nothing when the copy exists already.
 * Errors: ECK_EINVAL (null), ECK_EDEVICE. */
int32_t eck_space_upload(eck_space *space);

/* Frees host tables and the device copy (synchronises the device first). NULL is ignored. */
void eck_space_destroy(eck_space *space);

/* n_genes, the radix of every gene (radix[ECK_MAX_GENES], unused entries 0)
 * and the size of the space (0 when it does not fit 64 bits).  Host only. */
int32_t eck_space_info(const eck_space *space, int32_t *n_genes, uint32_t *radix, uint64_t *size);

/* Copies the factorisation table of split gene `gene` to `out` (host,
 * [capacity][4] uint32); returns the number of entries, or a negative error.
 * out == NULL just returns the count.  Host only. */
int32_t eck_space_table(const eck_space *space, int32_t gene, uint32_t *out, uint32_t capacity);

/* -------------------------------------------------------------- candidates */

/* Generate the genes of candidates first_index .. first_index+n-1
 * (Sec. 6.4: the search starts from many randomly generated kernels; Alg. 1:
 * the reproduction step of the genetic search).
 *   EXHAUSTIVE: candidate index -> genes by mixed radix, first gene most
 *               significant; first_index+n must not exceed the space size.
 *   SAMPLE:     gene g of candidate c = (low32(u) * radix_g) >> 32 with
 *               u = output number 16*c+g+1 of a SplitMix64 generator whose
 *               state starts at mix(seed + gamma*(round+1)).
 *   MUTATE:     child c copies parent (c mod n_parents); gene g is redrawn as
 *               in SAMPLE when high32(u) < p_mut_q32 (probability p*2^32).
 *   CROSSOVER:  two parents: (c mod n_parents) and one drawn uniformly with
 *               word 14 of the child ((low32(u14) * n_parents) >> 32); gene g
 *               comes from the second parent when bit g of word 15 is set;
 *               then every gene mutates as in MUTATE.  (Alg. 1 names the
 *               reproduction step without fixing its operators.)
 * genes_out: device, uint16 [n_genes][ld].  parents: device, uint16
 * [n_genes][n_parents] (MUTATE and CROSSOVER, else NULL).
 * Errors: EINVAL (nulls, n == 0, bad mode, index range), ESHAPE (ld < n),
 * EALIGN (genes_out not 4-byte aligned or ld odd). */
int32_t candidate_enumerate(const eck_space *space, int32_t mode, uint64_t seed, uint32_t round,
                            uint64_t first_index, uint64_t n, const uint16_t *parents, uint32_t n_parents,
                            uint32_t p_mut_q32, uint16_t *genes_out, uint64_t ld, void *stream);

/* candidate_enumerate for several spaces in one launch (many operator
 * shapes searched side by side; Sec. 7.1 lists the shapes the paper evaluates).  Space s
 * draws from stream (seeds[s], round) and writes its n_per_space candidates to
 * columns [s*n_per_space, (s+1)*n_per_space) of genes_out; in MUTATE its
 * parents are columns [s*n_parents_per_space, ...) of parents, uint16
 * [n_genes][n_spaces*n_parents_per_space].  Every space must have the same
 * kind, operator class and number of genes (ESHAPE otherwise).
 * spaces, seeds: host arrays of n_spaces entries, 1 <= n_spaces <=
 * ECK_MAX_BATCH (EUNSUPPORTED above).  ld >= n_spaces*n_per_space.
 * Other arguments and errors as candidate_enumerate. */
int32_t candidate_enumerate_batch(const eck_space *const *spaces, uint32_t n_spaces, int32_t mode,
                                  const uint64_t *seeds, uint32_t round, uint64_t first_index, uint64_t n_per_space,
                                  const uint16_t *parents, uint32_t n_parents_per_space, uint32_t p_mut_q32,
                                  uint16_t *genes_out, uint64_t ld, void *stream);

/* Collect the genes of selected candidates, e.g. the survivors topk_select
 * returned, as the parents of the next generation (Alg. 1: the kernels picked
 * at the end of a round reproduce the next one):
 *   out[g][j] = genes[g][idx[j]]  for j < k.
 * An index of 0xFFFFFFFF (padding of a short selection) copies candidate
 * idx[0] instead, so the output is always a valid parent set; if idx[0] is
 * padding too the column is zero.  genes: device uint16 [n_genes][ld]; idx:
 * device uint32 [k], every valid entry below n; out: device uint16 [n_genes][ld_out].
 * Errors: EINVAL (nulls, k == 0, n_genes outside 1..ECK_MAX_GENES), ESHAPE (ld_out < k). */
int32_t eck_candidates_gather(const uint16_t *genes, uint64_t ld, uint64_t n, int32_t n_genes, const uint32_t *idx,
                              uint32_t k, uint16_t *out, uint64_t ld_out, void *stream);

/* Duplicate removal before scoring (a generation bred from few parents
 * repeats itself; Alg. 1's reproduction step): candidate i is a first
 * occurrence when no candidate of lower index has the same genes.
 *   overwrite != 0: flags[i] = first occurrence ? 1 : 0
 *   overwrite == 0: flags[i] = flags[i] && first occurrence   (e.g. the legal
 *                   flags of features_compute, so that duplicates drop out of
 *                   topk_select)
 * genes: device uint16 [n_genes][ld]; flags: device uint8 [n]; ws: device, at
 * least eck_candidates_dedup_workspace_bytes(n) bytes (a hash table of candidate
 * indices, 4-byte aligned).  The result does not depend on execution order.
 * Errors: EINVAL, ESHAPE (ld < n), EUNSUPPORTED (n > 2^30), EWORKSPACE, EALIGN. */
uint64_t eck_candidates_dedup_workspace_bytes(uint64_t n);
int32_t eck_candidates_dedup(const uint16_t *genes, uint64_t ld, uint64_t n, int32_t n_genes, uint8_t *flags,
                             int32_t overwrite, void *ws, uint64_t ws_bytes, void *stream);

/* ---------------------------------------------------------------- features */

/* High-level kernel features of each candidate, computed analytically from
 * its loop structure (Sec. 5.3; Sec. 5.4: numbers of floating-point and
 * integer operations, vectorisation-, loop- and cache-access features; the
 * grid / block / global-load / shared-store counts are those of Table 5).
 * Feature f of candidate i is the 64-bit integer raw[f][i]; the model input is
 * its fixed-point log2: with v = raw+1 (saturating), e = floor(log2 v) and m =
 * the 10 bits below v's leading one, feat = e + m/1024 (exact in fp32; rounded
 * to nearest-even for bf16).  n_feat = 32 gives features 0..31, 64 all.
 *   genes:     device, uint16 [n_genes][ld] (values >= radix are clamped to radix-1)
 *   feat_out:  device, [n_feat][ld] of out_dtype (ECK_F32 or ECK_BF16); may be NULL
 *   raw_out:   device, uint64 [n_feat][ld] or NULL
 *   legal_out: device, uint8 [n] or NULL; 1 when the schedule can be launched
 *              (32 <= threads <= 1024, staged bytes -- in a SPLIT_XRED space the
 *              partial sums -- fit the LDS, vector width <= 16 bytes and
 *              divides the contiguous per-thread extent)
 * Errors: EINVAL, ESHAPE (ld < n), EUNSUPPORTED (n_feat not 32/64), EALIGN
 * (ld not a multiple of 2). */
int32_t features_compute(const eck_space *space, const uint16_t *genes, uint64_t ld, uint64_t n,
                         int32_t n_feat, int32_t out_dtype, void *feat_out, uint64_t *raw_out,
                         uint8_t *legal_out, void *stream);

/* features_compute for several spaces in one launch: columns
 * [s*n_per_space, (s+1)*n_per_space) of genes, feat_out, raw_out and legal_out
 * belong to spaces[s].  Same restrictions on the batch as
 * candidate_enumerate_batch; ld >= n_spaces*n_per_space. */
int32_t features_compute_batch(const eck_space *const *spaces, uint32_t n_spaces, const uint16_t *genes,
                               uint64_t ld, uint64_t n_per_space, int32_t n_feat, int32_t out_dtype,
                               void *feat_out, uint64_t *raw_out, uint8_t *legal_out, void *stream);

/* ------------------------------------------------------------------ models */

/* A multilayer perceptron widths[0] -> ... -> widths[n_layers] with ReLU
 * between layers and a linear scalar output: the cost model of Sec. 5.4 in the
 * form the workloads prescribe (the paper's own model is a tree ensemble).
 * dtype ECK_F32: fp32 weights and arithmetic.  ECK_BF16: bf16 weights and
 * bf16 first-hidden activations on the matrix cores, fp32 accumulation.
 * Supported: n_layers == 3, widths[3] == 1, widths[0] in {32, 64}, hidden widths
 * at most 512; a BF16 model must be one of the shapes the matrix-core kernels
 * are built for: 64-512-512-1, 64-256-256-1, 64-128-128-1, 32-64-64-1
 * (ECK_EUNSUPPORTED otherwise, here rather than at the first score call).
 * Allocates device memory (parameters, Adam moments, packed weights). */
int32_t eck_model_create(int32_t n_layers, const int32_t *widths, int32_t dtype, eck_model **out);
void eck_model_destroy(eck_model *model);

/* Number of parameters P: sum over layers of fan_in*fan_out + fan_out. Host only. */
int32_t eck_model_param_count(int32_t n_layers, const int32_t *widths, uint64_t *out);

/* State blob (device, fp32): [theta(P) | m(P) | v(P) | t] with theta = per
 * layer W[fan_in][fan_out] row-major then b[fan_out]; m, v Adam moments, t the
 * step count.  set_state accepts n_floats == P (moments and t reset to zero)
 * or 3P+1; get_state needs 3P+1.  The blob is the checkpoint format. */
int32_t eck_model_set_state(eck_model *model, const float *blob, uint64_t n_floats, void *stream);
int32_t eck_model_get_state(const eck_model *model, float *blob, uint64_t n_floats, void *stream);

/* ------------------------------------------------------------------- score */

/* Predicted score of every candidate (Alg. 1: LatencyEvaAndPick /
 * EnergyModelEvaAndPick evaluate the generation with a model; Sec. 5.4: the
 * model outputs a normalised energy score, lower is better).
 *   feat: device [widths[0]][ld] of feat_dtype; score_out: device float [n].
 * A BF16 model takes BF16 or F32 features (F32 is rounded to bf16 on load); an
 * F32 model takes F32 features.  ws/ws_bytes are reserved (pass NULL, 0).
 * A BF16 model reads two (or four) neighbouring candidates per load: ld must
 * be even and feat aligned to two elements (4 bytes for BF16, 8 for F32
 * features), whatever n is; the four-candidate loads are used only when ld is
 * a multiple of 4 and feat 8-byte aligned.  No load crosses the end of a row.
 * Errors: EINVAL, ESHAPE (ld < n), EUNSUPPORTED (dtype combination), EALIGN. */
int32_t costmodel_score(const eck_model *model, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                        float *score_out, void *ws, uint64_t ws_bytes, void *stream);

/* costmodel_score that also reduces the scores it writes: min_key_out[s] =
 * the least score among the legal candidates of segment s (n_segments equal
 * consecutive segments, as in topk_select), as an order-preserving key
 *     key(x) = bits(x) ^ (x < 0 ? 0xFFFFFFFF : 0x80000000)
 * (unsigned comparison of keys = comparison of the floats, -0 < +0), or
 * 0xFFFFFFFF when the segment has no legal candidate with a score that is a
 * number.  Run on the latency model it yields the L_min of every segment
 * (Alg. 1 LatencyEvaAndPick; the latency gate of Sec. 4.3) in the pass that
 * produces the latencies, so that topk_select_known_min need not read them a
 * second time.  legal: device uint8 [n] or NULL (all legal); min_key_out:
 * device uint32 [n_segments], overwritten.  BF16 models fold the reduction
 * into the scoring kernel (integer atomics: the result does not depend on the
 * order of execution).
 * Errors as costmodel_score; also EINVAL (min_key_out NULL, n_segments 0),
 * ESHAPE (n % n_segments, more than 65535 segments), EALIGN (legal odd). */
int32_t costmodel_score_min(const eck_model *model, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                            float *score_out, const uint8_t *legal, uint32_t n_segments, uint32_t *min_key_out,
                            void *stream);

/* ------------------------------------------------------------------ select */

/* Bytes of workspace topk_select needs for these sizes in THRESHOLD mode or
 * without latencies, and in RANK mode with m_latency (which adds the lists of
 * the latency stage).  0 on invalid sizes. */
uint64_t topk_select_workspace_bytes(uint64_t n, uint32_t n_segments, uint32_t k);
uint64_t topk_select_rank_workspace_bytes(uint64_t n, uint32_t n_segments, uint32_t k, uint32_t m_latency);

/* Selection under the paper's objective -- low latency first, then least
 * energy (Sec. 4.3, 4.4; Alg. 1).  The n candidates form n_segments equal
 * consecutive segments (one per operator); each is handled independently.
 *   THRESHOLD: L_min = least latency among legal candidates; tau = L_min +
 *              (alpha-1)*|L_min| (fp32, product and sum rounded separately;
 *              +inf when alpha is +inf); feasible = legal and latency <= tau.
 *   RANK:      feasible = the m_latency legal candidates of least latency
 *              (Alg. 1's "fastest M"), ties to the lower index.  m_latency is
 *              at most ECK_MAX_K unless it covers the whole segment.
 *   latency == NULL: feasible = legal.  legal == NULL: all legal.
 * Output per segment: the k feasible candidates of least energy in ascending
 * order (IEEE total order, ties to the lower index): idx_out uint32 [S][k]
 * (index within the segment, 0xFFFFFFFF padding), energy_out float [S][k]
 * (+inf padding), count_out uint32 [S] = min(k, #feasible).  NaN energies or
 * latencies are never feasible.  All pointers device; ws device, 16-byte aligned.
 * The score arrays are read once (THRESHOLD with a finite alpha reads the
 * latencies once more, for L_min; RANK reads once per stage); the result does
 * not depend on the order of execution.
 * Errors: EINVAL (nulls, n == 0, k == 0, bad mode, alpha < 1 or NaN), ESHAPE
 * (n % n_segments, k > n/n_segments, segment longer than 2^32-2), EUNSUPPORTED
 * (k or a partial m_latency > ECK_MAX_K), EWORKSPACE, EALIGN (ws). */
int32_t topk_select(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                    uint32_t n_segments, uint32_t k, int32_t mode, float alpha, uint32_t m_latency,
                    uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *ws, uint64_t ws_bytes,
                    void *stream);

/* topk_select in THRESHOLD mode when the least latency of every segment is
 * already known: latency_min_key = what costmodel_score_min wrote for the
 * latency model with the same legal flags and segments (device uint32
 * [n_segments]).  The score arrays are then read exactly once.  Same result as
 * topk_select(..., ECK_SELECT_THRESHOLD, alpha, ...), same workspace
 * (topk_select_workspace_bytes), same errors; EINVAL also for a NULL latency
 * or latency_min_key. */
int32_t topk_select_known_min(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                              uint32_t n_segments, uint32_t k, float alpha, const uint32_t *latency_min_key,
                              uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *ws, uint64_t ws_bytes,
                              void *stream);

/* topk_select for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same result, no ws: the
 * intermediate lists live in an array of ECK_TOPK_STATIC_BYTES that is part of
 * the library's device image (one copy per GPU, held until the process ends).
 * The call allocates and frees nothing; its kernels are those of topk_select.
 * Sizes whose workspace (topk_select_workspace_bytes /
 * topk_select_rank_workspace_bytes) exceeds ECK_TOPK_STATIC_BYTES are refused
 * with ECK_EWORKSPACE before anything is launched.  All calls on one GPU share
 * the one array: calls that overlap in time on the same GPU (different streams
 * or host threads) race and must be serialised by the caller; calls on
 * different GPUs are independent.  Nothing in the array has to be cleared
 * between calls.  Other errors as topk_select; ECK_EUNSUPPORTED also for a
 * device ordinal of 64 or more. */
#define ECK_TOPK_STATIC_BYTES (8u << 20)
int32_t topk_select_static(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                           uint32_t n_segments, uint32_t k, int32_t mode, float alpha, uint32_t m_latency,
                           uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *stream);

/* ------------------------------------------------------------------ update */

uint64_t costmodel_update_workspace_bytes(const eck_model *model, uint64_t n_pairs, int32_t minibatch);

/* ModelUpdate and SNR of Alg. 1 on a buffer of measured kernels.
 *   labels y = energy_measured / max(energy_measured)   ("normalised", Sec. 5.4)
 *   snr  = sum y^2 / sum (pred - y)^2 with the model as it is on entry
 *   then n_steps of Adam (bias-corrected, no weight decay) on the mean of
 *   Eq. (1), (pred - y)^2 / y, over minibatch s = rows [(s mod nb)*minibatch,
 *   +minibatch), nb = n_pairs / minibatch;  loss = the last step's value.
 * BF16 models run forward/backward on bf16 copies of the fp32 master weights.
 *   feat: device [widths[0]][ld]; energy_measured: device float [n_pairs];
 *   snr_out, loss_out: device float (one each).
 * A non-positive or non-finite measured energy is a data error found on the
 * device: snr = loss = NaN and the model is left unchanged.
 * Errors: EINVAL, ESHAPE (n_pairs % minibatch, ld < n_pairs), EUNSUPPORTED,
 * EWORKSPACE, EALIGN (ws not 256-byte aligned; feat / ld as costmodel_score). */
int32_t costmodel_update(eck_model *model, const void *feat, int32_t feat_dtype, uint64_t ld,
                         const float *energy_measured, uint64_t n_pairs, int32_t n_steps, int32_t minibatch,
                         float lr, float beta1, float beta2, float eps, float *snr_out, float *loss_out,
                         void *ws, uint64_t ws_bytes, void *stream);

/* Library version as major*10000 + minor*100 + patch. */
int32_t eck_version(void);

/* The k controller of Alg. 1 (Sec. 6.4): after a round in which round(k*M)
 * kernels were measured and the model updated, a signal-to-noise ratio of the
 * pre-update predictions below mu raises k by 0.2 (more measurements next
 * round), otherwise k falls by 0.2; k stays in [0, 1].  A round that measured
 * nothing (round(k*M) == 0) has no SNR and leaves k unchanged.  Host only;
 * *k_out receives the next k.  EINVAL: nulls, M < 0, k outside [0, 1], NaN. */
int32_t eck_k_step(double k, double snr, double mu, int64_t M, double *k_out);

/* How many of the M fastest kernels a round measures (Alg. 1: "k*M"): round(k*M),
 * halves up.  0 means the round measures nothing.  Host only.  EINVAL: null,
 * M < 0, k outside [0, 1] or NaN. */
int32_t eck_k_count(double k, int64_t M, int64_t *count_out);

/* ------------------------------------------------- boosted-tree cost model */

/* The cost model in the paper's own form (Sec. 5.4 "Approach"): an ensemble of
 * regression trees built one after another by gradient boosting; the
 * prediction is the base score plus the sum of the trees' outputs.  Trees are
 * complete binary trees of one fixed depth d, stored level by level: node j
 * tests x[feature_j] < threshold_j; true -> node 2j+1, false (also NaN) ->
 * node 2j+2; after d tests the walk stands on node (2^d - 1) + leaf.  A node
 * that does not split has threshold +inf.  Arrays (device, per tree):
 *   node_feat uint8 [2^d - 1], node_thr float [2^d - 1], leaf float [2^d].
 * n_feat in 1..256, depth in 1..ECK_MAX_TREE_DEPTH, capacity = most trees the
 * model can hold (<= 65536).  Allocates device memory for `capacity` trees.
 * Errors: EINVAL, EUNSUPPORTED (limits), EDEVICE. */
typedef struct eck_trees eck_trees;
#define ECK_MAX_TREE_DEPTH 8
int32_t eck_trees_create(int32_t n_feat, int32_t depth, int32_t capacity, float base_score, eck_trees **out);
void eck_trees_destroy(eck_trees *trees);

/* Number of trees the model holds now.  Host only. */
int32_t eck_trees_count(const eck_trees *trees, int32_t *n_trees);

/* Replace / read the ensemble (checkpointing).  The arrays are device memory,
 * [n_trees][...] as above; the copies are enqueued on stream.  A feature index
 * >= n_feat is read as n_feat - 1 when scoring.  ESHAPE: n_trees > capacity. */
int32_t eck_trees_set(eck_trees *trees, int32_t n_trees, const uint8_t *node_feat, const float *node_thr,
                      const float *leaf, void *stream);
int32_t eck_trees_get(const eck_trees *trees, uint8_t *node_feat, float *node_thr, float *leaf, void *stream);

/* score_out[i] = base + sum over trees of the leaf candidate i reaches, added in
 * fp32 in tree order.  feat: device, [n_feat][ld] of feat_dtype (ECK_F32 or
 * ECK_BF16; values are compared exactly, never rounded); score_out: device,
 * float [n].  Errors: EINVAL, ESHAPE (ld < n), EUNSUPPORTED (feature tile does
 * not fit the LDS: n_feat * 1 KB fp32 / 512 B bf16 above ~140 KB). */
int32_t treemodel_score(const eck_trees *trees, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                        float *score_out, void *stream);

/* Gradient boosting on the loss of Eq. (1) (Sec. 5.4; Alg. 1 ModelUpdate):
 * appends n_rounds trees fitted to the measured pairs.
 *   labels      y = energy_measured / max(energy_measured) in fp32
 *   prediction  p in fp32: base, then the trees in order
 *   per round   g = 2 (p - y) / y, h = 2 / y (derivatives of Eq. (1) in p),
 *               computed in fp64 and rounded to integers of resolution 2^-20
 *               (|g|, h clamped to 2^20); all sums are exact integer sums
 *   growth      level by level; features are binned into 256 bins of width 1/4
 *               on [0, 64) (the range of the transformed features); a split
 *               "feature f, bins <= b go left" has threshold (b + 1) / 4 and
 *               gain GL^2/(HL+lam) + GR^2/(HR+lam) - G^2/(H+lam), fp64, lam =
 *               lambda * 2^20; both sides non-empty; largest gain > 0 wins, ties
 *               to the lower feature then the lower bin; else no split
 *   leaves      w = -eta * G / (H + lam), fp64 -> fp32; empty leaf 0
 * The result is identical to a sequential evaluation of these steps: nothing
 * depends on the order of execution.
 * snr_out (device float): sum y^2 / sum (p - y)^2 of the ensemble on entry;
 * loss_out (device float): mean Eq. (1) loss after the last round.
 * Any energy <= 0 or not finite: snr = loss = NaN and the appended trees are
 * empty (no split, all leaves 0), so predictions do not change.
 * n_pairs <= 2^20 (EUNSUPPORTED above); ESHAPE: ld < n_pairs or capacity
 * exceeded; EWORKSPACE / EALIGN (256 B) for ws. */
uint64_t treemodel_update_workspace_bytes(const eck_trees *trees, uint64_t n_pairs);
int32_t treemodel_update(eck_trees *trees, const void *feat, int32_t feat_dtype, uint64_t ld,
                         const float *energy_measured, uint64_t n_pairs, int32_t n_rounds, float eta, float lambda,
                         float *snr_out, float *loss_out, void *ws, uint64_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ECK_H */
