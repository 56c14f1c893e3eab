// The cost model in the form the paper itself uses (Sec. 5.4 "Approach"): an ensemble of regression trees
// built one after another by gradient boosting on the weighted squared error of Eq. (1); the prediction is
// the sum of the trees' outputs.  HIP, gfx950.
//
// Trees are complete binary trees of a fixed depth d stored level by level: node j tests
// "x[feature_j] < threshold_j"; true -> node 2j+1, false (also NaN) -> node 2j+2; after d tests the walk stands
// on node (2^d - 1) + leaf.  A node that does not split has threshold +inf.
//
// Scoring: one candidate per lane.  A block stages the features of 256 candidates and a chunk of trees in LDS
// and walks eight trees at a time per lane (eight independent chains of dependent LDS reads); leaf values are
// added in fp32 in tree order, so the result does not depend on how trees are chunked or interleaved.
//
// Boosting: gradient statistics are rounded to integers of resolution 2^-20 and summed with integer atomics,
// so every histogram, and with it every split decision, is independent of the order of execution; gains are
// evaluated in fp64 from those integers.
#include "eck_internal.h"

#include <new>
#include <type_traits>

using namespace eck;

struct eck_trees {
    int32_t n_feat, depth, capacity, n_trees;
    float base;
    uint8_t *d_feat = nullptr; // [capacity][2^d - 1]
    float *d_thr = nullptr;    // [capacity][2^d - 1]
    float *d_leaf = nullptr;   // [capacity][2^d]
    int device = -1;
};

namespace {

constexpr int BLOCK = 256;
constexpr int BINS = 256;
constexpr int WALKS = 8; // trees walked at the same time by one lane
constexpr double FIX = 1048576.0; // 2^20

__device__ __forceinline__ float feature_value(const void *feat, int is_bf16, uint64_t at)
{
    if (is_bf16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(feat)[at] << 16);
    return reinterpret_cast<const float *>(feat)[at];
}

// ------------------------------------------------------------------------------------------------ scoring

// LDS per tree of a chunk: nodes as (threshold bits, feature) pairs, then the leaves
__host__ __device__ inline uint32_t tree_lds_bytes(int depth) { return ((1u << depth) - 1u) * 8u + (1u << depth) * 4u; }

// SCORE_BLOCK: candidates, and threads, per block
template <bool FEAT_BF16, int SCORE_BLOCK>
__global__ __launch_bounds__(SCORE_BLOCK) void tree_score_kernel(const uint8_t *__restrict__ node_feat,
                                                          const float *__restrict__ node_thr,
                                                          const float *__restrict__ leaf, int n_feat, int depth,
                                                          int n_trees, int chunk_trees, float base,
                                                          const void *__restrict__ feat, uint64_t ld, uint64_t n,
                                                          float *__restrict__ out, uint32_t n_tiles)
{
    using Elem = typename std::conditional<FEAT_BF16, uint16_t, float>::type;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const uint32_t nodes = (1u << depth) - 1u, leaves = 1u << depth;
    Elem *x_lds = reinterpret_cast<Elem *>(lds); // [n_feat][SCORE_BLOCK]
    uint2 *node_lds = reinterpret_cast<uint2 *>(lds + (size_t)n_feat * SCORE_BLOCK * sizeof(Elem)); // [chunk][nodes]
    float *leaf_lds = reinterpret_cast<float *>(node_lds + (size_t)chunk_trees * nodes);      // [chunk][leaves]
    const int tid = threadIdx.x;
    // where the dynamic LDS starts within the workgroup's allocation (the hand-written loads below take raw LDS
    // addresses)
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    const Elem *feat_e = reinterpret_cast<const Elem *>(feat);

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t cand = (uint64_t)tile * SCORE_BLOCK + tid;
        __syncthreads(); // the previous tile's walks are over
        // Sixteen rows at a time, every load and store unconditional (a lane beyond n re-reads the last candidate,
        // a row beyond n_feat the last row, and stores that same value where it already is): with a condition on
        // either side the compiler waits for each load right before its store, one round trip per feature.
        {
            const uint64_t col = cand < n ? cand : n - 1;
            for (int f0 = 0; f0 < n_feat; f0 += 16) {
                Elem v[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) v[k] = feat_e[(uint64_t)min(f0 + k, n_feat - 1) * ld + col];
#pragma unroll
                for (int k = 0; k < 16; ++k) x_lds[min(f0 + k, n_feat - 1) * SCORE_BLOCK + tid] = v[k];
            }
        }
        float acc = base;
        for (int t0 = 0; t0 < n_trees; t0 += chunk_trees) {
            const int in_chunk = min(chunk_trees, n_trees - t0);
            __syncthreads(); // features staged / previous chunk consumed
            for (uint32_t e = tid; e < (uint32_t)in_chunk * nodes; e += SCORE_BLOCK) {
                const uint32_t f = min((uint32_t)node_feat[(uint64_t)t0 * nodes + e], (uint32_t)n_feat - 1u);
                node_lds[e] = make_uint2(__float_as_uint(node_thr[(uint64_t)t0 * nodes + e]), f * (uint32_t)(SCORE_BLOCK * sizeof(Elem)));
            }
            for (uint32_t e = tid; e < (uint32_t)in_chunk * leaves; e += SCORE_BLOCK) leaf_lds[e] = leaf[(uint64_t)t0 * leaves + e];
            __syncthreads();
            // feature value from the byte offset of its row (a node's second word)
            auto x_of = [&](uint32_t row_bytes) {
                const Elem v = *reinterpret_cast<const Elem *>(lds + row_bytes + tid * sizeof(Elem));
                if (FEAT_BF16) return __uint_as_float((uint32_t)v << 16);
                else return (float)v;
            };
            // Nodes are numbered from 1 here (children of i: 2i and 2i + 1), so that one step is
            // i <- i + i + (x < t ? 0 : 1): a compare into a scalar mask and an add with that mask as carry-in,
            // two vector instructions, written out because the compiler makes three of it.  Four walks per
            // statement keep the compares four instructions ahead of the adds that read their masks.
            int t = 0;
            for (; t + WALKS <= in_chunk; t += WALKS) {
                uint32_t i[WALKS], upper[WALKS];
#pragma unroll
                for (int w = 0; w < WALKS; ++w) {
                    i[w] = 1;
                    upper[w] = 0;
                }
                const uint2 *first = node_lds + (size_t)t * nodes - 1; // node i of tree w at first[w * nodes + i]
                for (int l = 0; l < depth; ++l) {
                    uint2 nd[WALKS];
#pragma unroll
                    for (int w = 0; w < WALKS; ++w) nd[w] = first[(size_t)w * nodes + i[w]];
                    float x[WALKS];
                    if constexpr (FEAT_BF16 && WALKS == 8) {
                        // A bfloat16 is the upper half of the float of the same value.  The load below writes
                        // only the upper half of its destination, whose lower half is zero from the start and
                        // stays so: the float arrives ready, without a shift.  The compiler has no such load, so
                        // it is issued here, followed by its wait; nothing but these two statements touches the
                        // eight registers in between.
                        uint32_t at[WALKS];
#pragma unroll
                        for (int w = 0; w < WALKS; ++w) at[w] = lds_base + nd[w].y + tid * 2;
                        asm volatile("ds_read_u16_d16_hi %0, %8\n\t"
                                     "ds_read_u16_d16_hi %1, %9\n\t"
                                     "ds_read_u16_d16_hi %2, %10\n\t"
                                     "ds_read_u16_d16_hi %3, %11\n\t"
                                     "ds_read_u16_d16_hi %4, %12\n\t"
                                     "ds_read_u16_d16_hi %5, %13\n\t"
                                     "ds_read_u16_d16_hi %6, %14\n\t"
                                     "ds_read_u16_d16_hi %7, %15"
                                     : "+v"(upper[0]), "+v"(upper[1]), "+v"(upper[2]), "+v"(upper[3]), "+v"(upper[4]),
                                       "+v"(upper[5]), "+v"(upper[6]), "+v"(upper[7])
                                     : "v"(at[0]), "v"(at[1]), "v"(at[2]), "v"(at[3]), "v"(at[4]), "v"(at[5]), "v"(at[6]),
                                       "v"(at[7]));
                        asm volatile("s_waitcnt lgkmcnt(0)"
                                     : "+v"(upper[0]), "+v"(upper[1]), "+v"(upper[2]), "+v"(upper[3]), "+v"(upper[4]),
                                       "+v"(upper[5]), "+v"(upper[6]), "+v"(upper[7]));
#pragma unroll
                        for (int w = 0; w < WALKS; ++w) x[w] = __uint_as_float(upper[w]);
                    } else {
#pragma unroll
                        for (int w = 0; w < WALKS; ++w) x[w] = x_of(nd[w].y);
                    }
#pragma unroll
                    for (int w = 0; w < WALKS; w += 4) {
                        unsigned long long m0, m1, m2, m3;
                        asm("v_cmp_nlt_f32_e64 %4, %8, %12\n\t"
                            "v_cmp_nlt_f32_e64 %5, %9, %13\n\t"
                            "v_cmp_nlt_f32_e64 %6, %10, %14\n\t"
                            "v_cmp_nlt_f32_e64 %7, %11, %15\n\t"
                            "v_addc_co_u32_e64 %0, %4, %0, %0, %4\n\t"
                            "v_addc_co_u32_e64 %1, %5, %1, %1, %5\n\t"
                            "v_addc_co_u32_e64 %2, %6, %2, %2, %6\n\t"
                            "v_addc_co_u32_e64 %3, %7, %3, %3, %7"
                            : "+v"(i[w]), "+v"(i[w + 1]), "+v"(i[w + 2]), "+v"(i[w + 3]), "=&s"(m0), "=&s"(m1), "=&s"(m2),
                              "=&s"(m3)
                            : "v"(x[w]), "v"(x[w + 1]), "v"(x[w + 2]), "v"(x[w + 3]), "v"(__uint_as_float(nd[w].x)),
                              "v"(__uint_as_float(nd[w + 1].x)), "v"(__uint_as_float(nd[w + 2].x)),
                              "v"(__uint_as_float(nd[w + 3].x)));
                    }
                }
                const float *lf = leaf_lds + (size_t)t * leaves;
                float v[WALKS];
#pragma unroll
                for (int w = 0; w < WALKS; ++w) v[w] = lf[(size_t)w * leaves + i[w] - leaves]; // i in [2^d, 2^(d+1))
#pragma unroll
                for (int w = 0; w < WALKS; ++w) acc = acc + v[w]; // tree order
            }
            for (; t < in_chunk; ++t) {
                uint32_t j = 0;
                const uint2 *nd = node_lds + (size_t)t * nodes;
                for (int l = 0; l < depth; ++l) {
                    const uint2 a = nd[j];
                    j = 2 * j + (x_of(a.y) < __uint_as_float(a.x) ? 1u : 2u);
                }
                acc = acc + leaf_lds[(size_t)t * leaves + j - nodes];
            }
        }
        if (cand < n) out[cand] = acc;
    }
}

int32_t launch_score(const eck_trees *m, int n_trees, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                     float *out, hipStream_t st)
{
    const size_t elem = feat_dtype == ECK_BF16 ? 2 : 4;
    const size_t per_tree = tree_lds_bytes(m->depth);
    const size_t lds_cu = 156 * 1024;
    // 512 candidates per block when two such blocks fit a compute unit (a staged chunk of trees then serves
    // twice as many candidates; measured 2.49 against 2.70 ms for 256, and 2.71 ms for one block of 1024), else 256
    const size_t floor512 = (size_t)m->n_feat * 512 * elem + WALKS * per_tree;
    const int block = 2 * floor512 <= lds_cu ? 512 : 256;
    const uint64_t tiles64 = (n + block - 1) / block;
    if (tiles64 > 0xFFFFFFFFull) return ECK_EUNSUPPORTED;
    const size_t x_bytes = (size_t)m->n_feat * block * elem;
    // Trees per chunk.  The walks are chains of dependent LDS reads, so what counts is how many wavefronts a
    // compute unit holds: the smallest chunk (one group of simultaneous walks) beside the feature tile lets
    // the most blocks share the 160 KB; blocks per unit = what fits, chunk = what is left of a block's share.
    const size_t floor_bytes = x_bytes + WALKS * per_tree;
    if (floor_bytes > lds_cu) return ECK_EUNSUPPORTED;
    size_t blocks_cu = lds_cu / floor_bytes;
    if (blocks_cu > (size_t)(2048 / block)) blocks_cu = 2048 / block; // 2048 threads per unit
    const size_t share = lds_cu / blocks_cu;
    int chunk = (int)((share - x_bytes) / per_tree);
    chunk -= chunk % WALKS;
    const int rounded = (n_trees + WALKS - 1) / WALKS * WALKS;
    if (n_trees > 0 && chunk > rounded) chunk = rounded;
    if (chunk < WALKS) chunk = WALKS;
    const size_t lds = x_bytes + (size_t)chunk * per_tree;
    int cus = 256;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device);
    const uint32_t n_tiles = (uint32_t)tiles64;
    const uint32_t want = (uint32_t)cus * (uint32_t)blocks_cu;
    const uint32_t grid = n_tiles < want ? n_tiles : want;
    auto kern = feat_dtype == ECK_BF16 ? (block == 512 ? tree_score_kernel<true, 512> : tree_score_kernel<true, 256>)
                                       : (block == 512 ? tree_score_kernel<false, 512> : tree_score_kernel<false, 256>);
    ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(block), lds, st, m->d_feat, m->d_thr, m->d_leaf, m->n_feat, m->depth,
                       n_trees, chunk, m->base, feat, ld, n, out, n_tiles);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

// ----------------------------------------------------------------------------------------------- boosting

struct BoostScalars {
    float emax;
    uint32_t bad;
    float snr, loss;
};

// feature value -> histogram bin: 256 bins of width 1/4 on [0, 64); "bin(x) <= b" is "x < (b + 1) / 4"
__device__ __forceinline__ uint32_t bin_of(float x)
{
    if (!(x >= 0.0f)) return x != x ? 255u : 0u;
    const float s = x * 4.0f;
    return s >= 255.0f ? 255u : (uint32_t)(int)s;
}

__device__ __forceinline__ long long quantise(double v)
{
    if (v > FIX) v = FIX; // |g| and h are clamped to 2^20: 2^20 samples cannot overflow 63 bits
    if (v < -FIX) v = -FIX;
    return __double2ll_rn(v * FIX);
}

__device__ double block_sum_f64(double v, double *scratch)
{
    scratch[threadIdx.x] = v;
    __syncthreads();
    for (int off = blockDim.x / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) scratch[threadIdx.x] += scratch[threadIdx.x + off];
        __syncthreads();
    }
    const double r = scratch[0];
    __syncthreads();
    return r;
}

// one block: validate the measured energies and normalise them by their maximum (fp32 division)
__global__ __launch_bounds__(1024) void tree_labels_kernel(const float *__restrict__ e, uint64_t n, float *__restrict__ y,
                                                           BoostScalars *sc)
{
    __shared__ float smax[1024];
    __shared__ uint32_t sbad[1024];
    float mx = 0.0f;
    uint32_t bad = 0;
    for (uint64_t i = threadIdx.x; i < n; i += 1024) {
        const float v = e[i];
        if (!(v > 0.0f) || v == __builtin_inff()) bad = 1;
        mx = fmaxf(mx, v);
    }
    smax[threadIdx.x] = mx;
    sbad[threadIdx.x] = bad;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
            smax[threadIdx.x] = fmaxf(smax[threadIdx.x], smax[threadIdx.x + off]);
            sbad[threadIdx.x] |= sbad[threadIdx.x + off];
        }
        __syncthreads();
    }
    const float emax = smax[0];
    for (uint64_t i = threadIdx.x; i < n; i += 1024) y[i] = e[i] / emax;
    if (threadIdx.x == 0) {
        sc->emax = emax;
        sc->bad = sbad[0];
        sc->snr = sc->loss = __builtin_nanf("");
    }
}

// bins of every (feature, pair), computed once per call
__global__ void tree_bins_kernel(const void *__restrict__ feat, int is_bf16, uint64_t ld, uint64_t n_pairs, int n_feat,
                                 uint8_t *__restrict__ bins)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int f = blockIdx.y;
    if (i >= n_pairs || f >= n_feat) return;
    bins[(uint64_t)f * n_pairs + i] = (uint8_t)bin_of(feature_value(feat, is_bf16, (uint64_t)f * ld + i));
}

// SNR = sum y^2 / sum (p - y)^2 (which == 0: the ensemble on entry) or the mean Eq.-(1) loss (which == 1)
__global__ __launch_bounds__(1024) void tree_quality_kernel(const float *__restrict__ p, const float *__restrict__ y,
                                                            uint64_t n, int which, BoostScalars *sc)
{
    __shared__ double scratch[1024];
    double a = 0.0, b = 0.0;
    for (uint64_t i = threadIdx.x; i < n; i += 1024) {
        const double yi = y[i], d = (double)p[i] - yi;
        if (which == 0) {
            a += yi * yi;
            b += d * d;
        } else {
            a += d * d / yi;
        }
    }
    a = block_sum_f64(a, scratch);
    b = block_sum_f64(b, scratch);
    if (threadIdx.x == 0 && !sc->bad) {
        if (which == 0) sc->snr = (float)(a / b);
        else sc->loss = (float)(a / (double)n);
    }
}

// first and second derivative of Eq. (1) in the prediction, as integers of resolution 2^-20
// (also: every node of the tree about to be built starts as "does not split"; the grid is at least 256 threads,
// a tree at most 255 nodes)
__global__ void tree_grad_kernel(const float *__restrict__ p, const float *__restrict__ y, uint64_t n,
                                 long long *__restrict__ gq, long long *__restrict__ hq, uint32_t *__restrict__ at,
                                 uint8_t *__restrict__ nf, float *__restrict__ nt, uint32_t nodes)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nodes) {
        nf[i] = 0;
        nt[i] = __builtin_inff();
    }
    if (i >= n) return;
    const double yi = (double)y[i], d = (double)p[i] - yi;
    gq[i] = quantise(2.0 * d / yi);
    hq[i] = quantise(2.0 / yi);
    at[i] = 0;
}

__global__ void tree_zero_kernel(unsigned long long *ptr, uint64_t words)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) ptr[i] = 0;
}

// Histograms of one level: hist[node in level][feature][bin] = (sum g, sum h, count) over the pairs that
// stand on that node.  Every pair of a level hits the few cells of one feature, and device-wide atomics on
// them serialise, so a block takes one feature, a group of 8 nodes and a slice of the pairs, accumulates in
// LDS (integer atomics) and merges its non-empty cells once.
constexpr uint32_t LDS_HIST_NODES = 8;
__global__ __launch_bounds__(BLOCK) void tree_hist_lds_kernel(const uint8_t *__restrict__ bins,
                                                             const long long *__restrict__ gq,
                                                             const long long *__restrict__ hq,
                                                             const uint32_t *__restrict__ at, uint64_t n_pairs,
                                                             int n_feat, uint32_t first_node, uint32_t level_nodes,
                                                             unsigned long long *__restrict__ hist)
{
    __shared__ unsigned long long cells[LDS_HIST_NODES * BINS * 3];
    const uint32_t group0 = blockIdx.z * LDS_HIST_NODES; // first node (within the level) of this block's group
    const uint32_t in_group = min(LDS_HIST_NODES, level_nodes - group0);
    const uint32_t n_cells = in_group * BINS * 3;
    for (uint32_t c = threadIdx.x; c < n_cells; c += BLOCK) cells[c] = 0;
    __syncthreads();
    const int f = blockIdx.y;
    for (uint64_t i = (uint64_t)blockIdx.x * BLOCK + threadIdx.x; i < n_pairs; i += (uint64_t)gridDim.x * BLOCK) {
        const uint32_t r = at[i] - first_node - group0; // wraps for nodes below the group
        if (r >= in_group) continue;
        const uint32_t b = bins[(uint64_t)f * n_pairs + i];
        unsigned long long *cell = cells + ((uint64_t)r * BINS + b) * 3;
        atomicAdd(cell, (unsigned long long)gq[i]);
        atomicAdd(cell + 1, (unsigned long long)hq[i]);
        atomicAdd(cell + 2, 1ull);
    }
    __syncthreads();
    for (uint32_t c = threadIdx.x; c < n_cells; c += BLOCK) {
        const unsigned long long v = cells[c];
        if (!v) continue;
        const uint32_t r = group0 + c / (BINS * 3), rest = c % (BINS * 3);
        atomicAdd(hist + ((uint64_t)r * n_feat + f) * BINS * 3 + rest, v);
    }
}

// The split of largest gain, in two parts.  tree_split_kernel: one block per (node of the level, group of four
// features), a wavefront per feature, a lane per four consecutive bins; prefix sums over the bins by shuffles.
// gain(f, b) = GL^2/(HL+lam) + GR^2/(HR+lam) - G^2/(H+lam) in fp64; the largest gain > 0 wins, ties to the
// lower feature, then the lower bin (the candidate's rank f * 256 + b breaks ties in every comparison).  The
// block leaves its best (gain, rank) in `partial`; the kernel that moves the pairs to their children compares
// the groups' results.  The fp64 divisions of a node are thus spread over up to 64 compute units instead of
// one.  Every cell read is set back to zero, so that the histogram buffer is clear again for the next level
// without a pass of its own.
struct SplitPartial {
    double gain;
    uint32_t rank, pad;
};
constexpr int SPLIT_FEATS = 4; // features, and wavefronts, per block

__device__ __forceinline__ bool better_split(double og, uint32_t orank, double g, uint32_t rank)
{
    return og > g || (og == g && orank < rank);
}

__global__ __launch_bounds__(SPLIT_FEATS * 64) void tree_split_kernel(unsigned long long *__restrict__ hist, int n_feat,
                                                                      double lam, SplitPartial *__restrict__ partial)
{
    const uint32_t r = blockIdx.x; // node within the level
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int f = blockIdx.y * SPLIT_FEATS + wave;
    double best = 0.0;
    uint32_t best_rank = 0xFFFFFFFFu;
    if (f < n_feat) { // wave-uniform
        unsigned long long *cells = hist + (((uint64_t)r * n_feat + f) * BINS + 4 * lane) * 3;
        long long g[4], hh[4], c[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            g[q] = (long long)cells[3 * q];
            hh[q] = (long long)cells[3 * q + 1];
            c[q] = (long long)cells[3 * q + 2];
        }
#pragma unroll
        for (int q = 0; q < 12; ++q) cells[q] = 0;
#pragma unroll
        for (int q = 1; q < 4; ++q) {
            g[q] += g[q - 1];
            hh[q] += hh[q - 1];
            c[q] += c[q - 1];
        }
        // inclusive prefix of the lanes' totals; its last lane holds the node's totals (every pair of the node is
        // in exactly one bin of every feature, so each feature's histogram sums to the same G, H, N)
        long long pg = g[3], ph = hh[3], pc = c[3];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long ug = __shfl_up(pg, off), uh = __shfl_up(ph, off), uc = __shfl_up(pc, off);
            if (lane >= off) {
                pg += ug;
                ph += uh;
                pc += uc;
            }
        }
        const long long G = __shfl(pg, 63), H = __shfl(ph, 63), N = __shfl(pc, 63);
        if (N > 1) {
            const double parent = (double)G * (double)G / ((double)H + lam);
            pg -= g[3];
            ph -= hh[3];
            pc -= c[3];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int b = 4 * lane + q;
                const long long GL = pg + g[q], HL = ph + hh[q], NL = pc + c[q];
                if (b >= 255 || NL == 0 || NL == N) continue;
                const long long GR = G - GL, HR = H - HL;
                const double gain = (double)GL * (double)GL / ((double)HL + lam) +
                                    (double)GR * (double)GR / ((double)HR + lam) - parent;
                const uint32_t rank = (uint32_t)f * BINS + (uint32_t)b;
                if (gain > best || (gain == best && gain > 0.0 && rank < best_rank)) {
                    best = gain;
                    best_rank = rank;
                }
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double og = __shfl_xor(best, off);
        const uint32_t orank = __shfl_xor(best_rank, off);
        if (better_split(og, orank, best, best_rank)) {
            best = og;
            best_rank = orank;
        }
    }
    __shared__ double s_gain[SPLIT_FEATS];
    __shared__ uint32_t s_rank[SPLIT_FEATS];
    if (lane == 0) {
        s_gain[wave] = best;
        s_rank[wave] = best_rank;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < SPLIT_FEATS; ++w)
            if (better_split(s_gain[w], s_rank[w], best, best_rank)) {
                best = s_gain[w];
                best_rank = s_rank[w];
            }
        SplitPartial out;
        out.gain = best;
        out.rank = best_rank;
        out.pad = 0;
        partial[(uint64_t)r * gridDim.y + blockIdx.y] = out;
    }
}

// Move every pair to the child its node's test sends it to.  The node's test is settled here, from the feature
// groups' partial results: every pair standing on a node arrives at the same (feature, threshold) and writes it
// (equal values, so the order does not matter); nodes no pair stands on keep "does not split".
__global__ void tree_partition_kernel(const void *__restrict__ feat, int is_bf16, uint64_t ld, uint64_t n_pairs,
                                      const SplitPartial *__restrict__ partial, uint32_t groups, uint32_t first_node,
                                      const BoostScalars *sc, uint8_t *__restrict__ nf, float *__restrict__ nt,
                                      uint32_t *__restrict__ at)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs) return;
    const uint32_t j = at[i];
    const SplitPartial *mine = partial + (uint64_t)(j - first_node) * groups;
    double best = 0.0;
    uint32_t best_rank = 0xFFFFFFFFu;
    for (uint32_t g = 0; g < groups; ++g) {
        const SplitPartial o = mine[g];
        if (better_split(o.gain, o.rank, best, best_rank)) {
            best = o.gain;
            best_rank = o.rank;
        }
    }
    uint32_t f = 0;
    float thr = __builtin_inff();
    if (!sc->bad && best_rank != 0xFFFFFFFFu && best > 0.0) {
        f = best_rank / BINS;
        thr = (float)((best_rank % BINS) + 1) * 0.25f;
    }
    nf[j] = (uint8_t)f;
    nt[j] = thr;
    const float x = feature_value(feat, is_bf16, (uint64_t)f * ld + i);
    at[i] = 2 * j + (x < thr ? 1u : 2u);
}

// one block: statistics of every leaf by integer atomics in LDS, then w = -eta G / (H + lam) (fp64 -> fp32)
__global__ __launch_bounds__(1024) void tree_leaf_kernel(const long long *__restrict__ gq, const long long *__restrict__ hq,
                                                         const uint32_t *__restrict__ at, uint64_t n_pairs,
                                                         uint32_t nodes, uint32_t leaves, double eta, double lam,
                                                         float *__restrict__ leaf_out, const BoostScalars *sc)
{
    __shared__ unsigned long long sg[256], sh[256], sn[256];
    for (uint32_t l = threadIdx.x; l < leaves; l += 1024) sg[l] = sh[l] = sn[l] = 0;
    __syncthreads();
    for (uint64_t i = threadIdx.x; i < n_pairs; i += 1024) {
        const uint32_t l = at[i] - nodes;
        atomicAdd(&sg[l], (unsigned long long)gq[i]);
        atomicAdd(&sh[l], (unsigned long long)hq[i]);
        atomicAdd(&sn[l], 1ull);
    }
    __syncthreads();
    for (uint32_t l = threadIdx.x; l < leaves; l += 1024) {
        const long long G = (long long)sg[l], H = (long long)sh[l];
        float w = 0.0f;
        if (sn[l] && !sc->bad) w = (float)(-eta * (double)G / ((double)H + lam));
        leaf_out[l] = w;
    }
}

__global__ void tree_advance_kernel(float *__restrict__ p, const uint32_t *__restrict__ at, const float *__restrict__ lw,
                                    uint32_t nodes, uint64_t n_pairs)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_pairs) p[i] = p[i] + lw[at[i] - nodes];
}

__global__ void tree_finish_kernel(const BoostScalars *sc, float *snr_out, float *loss_out)
{
    if (threadIdx.x || blockIdx.x) return;
    *snr_out = sc->snr;
    *loss_out = sc->loss;
}

struct BoostWs {
    uint64_t scalars, y, p, gq, hq, at, bins, hist, partial, total;
};

BoostWs boost_layout(const eck_trees *m, uint64_t n_pairs)
{
    auto up = [](uint64_t v) { return (v + 255) & ~255ull; };
    BoostWs w;
    uint64_t o = 0;
    w.scalars = o; o = up(o + sizeof(BoostScalars));
    w.y = o; o = up(o + n_pairs * 4);
    w.p = o; o = up(o + n_pairs * 4);
    w.gq = o; o = up(o + n_pairs * 8);
    w.hq = o; o = up(o + n_pairs * 8);
    w.at = o; o = up(o + n_pairs * 4);
    w.bins = o; o = up(o + n_pairs * (uint64_t)m->n_feat);
    w.hist = o; o = up(o + ((uint64_t)1 << (m->depth - 1)) * m->n_feat * BINS * 3 * 8);
    w.partial = o; o = up(o + ((uint64_t)1 << (m->depth - 1)) * ((m->n_feat + SPLIT_FEATS - 1) / SPLIT_FEATS) * sizeof(SplitPartial));
    w.total = o;
    return w;
}

} // namespace

extern "C" int32_t eck_trees_create(int32_t n_feat, int32_t depth, int32_t capacity, float base_score, eck_trees **out)
{
    if (!out) return ECK_EINVAL;
    *out = nullptr;
    if (n_feat < 1 || depth < 1 || capacity < 1 || !(base_score == base_score)) return ECK_EINVAL;
    if (n_feat > 256 || depth > ECK_MAX_TREE_DEPTH || capacity > 65536) return ECK_EUNSUPPORTED;
    eck_trees *m = new (std::nothrow) eck_trees();
    if (!m) return ECK_EDEVICE;
    m->n_feat = n_feat;
    m->depth = depth;
    m->capacity = capacity;
    m->n_trees = 0;
    m->base = base_score;
    const size_t nodes = ((size_t)1 << depth) - 1, leaves = (size_t)1 << depth;
    if (hipGetDevice(&m->device) != hipSuccess || hipMalloc((void **)&m->d_feat, capacity * nodes) != hipSuccess ||
        hipMalloc((void **)&m->d_thr, capacity * nodes * 4) != hipSuccess ||
        hipMalloc((void **)&m->d_leaf, capacity * leaves * 4) != hipSuccess) {
        (void)hipGetLastError();
        if (m->d_feat) (void)hipFree(m->d_feat);
        if (m->d_thr) (void)hipFree(m->d_thr);
        if (m->d_leaf) (void)hipFree(m->d_leaf);
        delete m;
        return ECK_EDEVICE;
    }
    *out = m;
    return ECK_OK;
}

extern "C" void eck_trees_destroy(eck_trees *m)
{
    if (!m) return;
    (void)hipDeviceSynchronize();
    (void)hipFree(m->d_feat);
    (void)hipFree(m->d_thr);
    (void)hipFree(m->d_leaf);
    delete m;
}

extern "C" int32_t eck_trees_count(const eck_trees *m, int32_t *n_trees)
{
    if (!m || !n_trees) return ECK_EINVAL;
    *n_trees = m->n_trees;
    return ECK_OK;
}

extern "C" int32_t eck_trees_set(eck_trees *m, int32_t n_trees, const uint8_t *node_feat, const float *node_thr,
                                 const float *leaf, void *stream)
{
    if (!m || n_trees < 0) return ECK_EINVAL;
    if (n_trees > m->capacity) return ECK_ESHAPE;
    if (n_trees && (!node_feat || !node_thr || !leaf)) return ECK_EINVAL;
    const size_t nodes = ((size_t)1 << m->depth) - 1, leaves = (size_t)1 << m->depth;
    hipStream_t st = as_stream(stream);
    if (n_trees) {
        ECK_HIP_TRY(hipMemcpyAsync(m->d_feat, node_feat, n_trees * nodes, hipMemcpyDeviceToDevice, st));
        ECK_HIP_TRY(hipMemcpyAsync(m->d_thr, node_thr, n_trees * nodes * 4, hipMemcpyDeviceToDevice, st));
        ECK_HIP_TRY(hipMemcpyAsync(m->d_leaf, leaf, n_trees * leaves * 4, hipMemcpyDeviceToDevice, st));
    }
    m->n_trees = n_trees;
    return ECK_OK;
}

extern "C" int32_t eck_trees_get(const eck_trees *m, uint8_t *node_feat, float *node_thr, float *leaf, void *stream)
{
    if (!m) return ECK_EINVAL;
    if (m->n_trees == 0) return ECK_OK;
    if (!node_feat || !node_thr || !leaf) return ECK_EINVAL;
    const size_t nodes = ((size_t)1 << m->depth) - 1, leaves = (size_t)1 << m->depth;
    hipStream_t st = as_stream(stream);
    ECK_HIP_TRY(hipMemcpyAsync(node_feat, m->d_feat, m->n_trees * nodes, hipMemcpyDeviceToDevice, st));
    ECK_HIP_TRY(hipMemcpyAsync(node_thr, m->d_thr, m->n_trees * nodes * 4, hipMemcpyDeviceToDevice, st));
    ECK_HIP_TRY(hipMemcpyAsync(leaf, m->d_leaf, m->n_trees * leaves * 4, hipMemcpyDeviceToDevice, st));
    return ECK_OK;
}

extern "C" int32_t treemodel_score(const eck_trees *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                                   float *score_out, void *stream)
{
    if (!m || !feat || !score_out || n == 0) return ECK_EINVAL;
    if (feat_dtype != ECK_F32 && feat_dtype != ECK_BF16) return ECK_EINVAL;
    if (ld < n) return ECK_ESHAPE;
    if (n > (1ull << 40)) return ECK_EINVAL;
    return launch_score(m, m->n_trees, feat, feat_dtype, ld, n, score_out, as_stream(stream));
}

extern "C" uint64_t treemodel_update_workspace_bytes(const eck_trees *m, uint64_t n_pairs)
{
    if (!m || n_pairs == 0 || n_pairs > (1ull << 20)) return 0;
    return boost_layout(m, n_pairs).total;
}

extern "C" int32_t treemodel_update(eck_trees *m, const void *feat, int32_t feat_dtype, uint64_t ld,
                                    const float *energy_measured, uint64_t n_pairs, int32_t n_rounds, float eta,
                                    float lambda, float *snr_out, float *loss_out, void *ws, uint64_t ws_bytes,
                                    void *stream)
{
    if (!m || !feat || !energy_measured || !snr_out || !loss_out) return ECK_EINVAL;
    if (n_pairs == 0 || n_rounds < 0 || !(eta > 0.0f) || !(lambda >= 0.0f)) return ECK_EINVAL;
    if (feat_dtype != ECK_F32 && feat_dtype != ECK_BF16) return ECK_EINVAL;
    if (n_pairs > (1ull << 20)) return ECK_EUNSUPPORTED;
    if (ld < n_pairs || m->n_trees + n_rounds > m->capacity) return ECK_ESHAPE;
    const BoostWs w = boost_layout(m, n_pairs);
    if (!ws || ws_bytes < w.total) return ECK_EWORKSPACE;
    if ((uintptr_t)ws & 255) return ECK_EALIGN;

    hipStream_t st = as_stream(stream);
    char *base = static_cast<char *>(ws);
    BoostScalars *sc = reinterpret_cast<BoostScalars *>(base + w.scalars);
    float *y = reinterpret_cast<float *>(base + w.y), *p = reinterpret_cast<float *>(base + w.p);
    long long *gq = reinterpret_cast<long long *>(base + w.gq), *hq = reinterpret_cast<long long *>(base + w.hq);
    uint32_t *at = reinterpret_cast<uint32_t *>(base + w.at);
    uint8_t *bins = reinterpret_cast<uint8_t *>(base + w.bins);
    unsigned long long *hist = reinterpret_cast<unsigned long long *>(base + w.hist);
    SplitPartial *partial = reinterpret_cast<SplitPartial *>(base + w.partial);
    const unsigned split_groups = (unsigned)((m->n_feat + SPLIT_FEATS - 1) / SPLIT_FEATS);
    const int is_bf16 = feat_dtype == ECK_BF16;
    const uint32_t nodes = (1u << m->depth) - 1u, leaves = 1u << m->depth;
    const unsigned pair_blocks = (unsigned)((n_pairs + 255) / 256);
    const double lam = (double)lambda * FIX;

    hipLaunchKernelGGL(tree_labels_kernel, dim3(1), dim3(1024), 0, st, energy_measured, n_pairs, y, sc);
    // predictions of the ensemble as it stands: the scoring kernel (fp32, base first, trees in order)
    int32_t rc = launch_score(m, m->n_trees, feat, feat_dtype, ld, n_pairs, p, st);
    if (rc != ECK_OK) return rc;
    hipLaunchKernelGGL(tree_quality_kernel, dim3(1), dim3(1024), 0, st, p, y, n_pairs, 0, sc);
    hipLaunchKernelGGL(tree_bins_kernel, dim3(pair_blocks, m->n_feat), dim3(256), 0, st, feat, is_bf16, ld, n_pairs,
                       m->n_feat, bins);
    {
        // the histogram buffer starts clear; from then on the split kernel clears what it reads
        const uint64_t words = ((uint64_t)1 << (m->depth - 1)) * m->n_feat * BINS * 3;
        hipLaunchKernelGGL(tree_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, hist, words);
    }
    for (int32_t r = 0; r < n_rounds; ++r) {
        const size_t t = (size_t)m->n_trees + r;
        uint8_t *nf = m->d_feat + t * nodes;
        float *nt = m->d_thr + t * nodes;
        float *lw = m->d_leaf + t * leaves;
        hipLaunchKernelGGL(tree_grad_kernel, dim3(pair_blocks), dim3(256), 0, st, p, y, n_pairs, gq, hq, at, nf, nt, nodes);
        for (int l = 0; l < m->depth; ++l) {
            const uint32_t level_nodes = 1u << l, first = level_nodes - 1u;
            {
                unsigned slices = (unsigned)(n_pairs / 2048);
                slices = slices < 1 ? 1 : (slices > 64 ? 64 : slices);
                const unsigned groups = (level_nodes + LDS_HIST_NODES - 1) / LDS_HIST_NODES;
                hipLaunchKernelGGL(tree_hist_lds_kernel, dim3(slices, m->n_feat, groups), dim3(BLOCK), 0, st, bins, gq, hq,
                                   at, n_pairs, m->n_feat, first, level_nodes, hist);
            }
            hipLaunchKernelGGL(tree_split_kernel, dim3(level_nodes, split_groups), dim3(SPLIT_FEATS * 64), 0, st, hist,
                               m->n_feat, lam, partial);
            hipLaunchKernelGGL(tree_partition_kernel, dim3(pair_blocks), dim3(256), 0, st, feat, is_bf16, ld, n_pairs,
                               partial, split_groups, first, sc, nf, nt, at);
        }
        hipLaunchKernelGGL(tree_leaf_kernel, dim3(1), dim3(1024), 0, st, gq, hq, at, n_pairs, nodes, leaves, (double)eta,
                           lam, lw, sc);
        hipLaunchKernelGGL(tree_advance_kernel, dim3(pair_blocks), dim3(256), 0, st, p, at, lw, nodes, n_pairs);
    }
    hipLaunchKernelGGL(tree_quality_kernel, dim3(1), dim3(1024), 0, st, p, y, n_pairs, 1, sc);
    hipLaunchKernelGGL(tree_finish_kernel, dim3(1), dim3(64), 0, st, sc, snr_out, loss_out);
    ECK_HIP_TRY(hipGetLastError());
    m->n_trees += n_rounds;
    return ECK_OK;
}
