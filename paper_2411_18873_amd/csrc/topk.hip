// Selection under the "low latency first, then least energy" objective
// (Sec. 4.3, 4.4; Alg. 1 LatencyEvaAndPick / EnergyModelEvaAndPick).  HIP, gfx950.
//
// Method: a tournament of exact block-local selections.  Every candidate is the composite key
// (order-preserving score bits, index within its segment); composites of one segment are distinct, so
// "the k smallest" is a unique set and ties fall to the lower index.  Level 0 reads the score arrays
// ONCE: a block takes a chunk of one segment, keeps the composites of its feasible candidates in
// registers, finds its own k smallest with a radix select on LDS histograms (nothing leaves the
// block) and writes just those.  Every further level does the same on the lists of the level before
// it, until one block per segment holds the segment's k smallest, sorts them in LDS and writes the
// result.  The k smallest of a segment are among the k smallest of each chunk, so the result is exact;
// no global atomics, no flags between blocks: blocks only meet at kernel boundaries, and the output does
// not depend on execution order.  Inside a block: a cheap upper bound on its k-th smallest key first (from
// the least key of every thread), then the few candidates under the bound are ranked against each other,
// which selects and orders them at once; a radix select on LDS histograms takes over when many remain.
#include <mutex>

#include "eck_internal.h"

using namespace eck;

namespace {

constexpr int DIGIT_BITS = 11;
constexpr int BINS = 1 << DIGIT_BITS;
#ifndef ECK_TOPK_ITEMS
#define ECK_TOPK_ITEMS 16
#endif
constexpr int ITEMS = ECK_TOPK_ITEMS;                // composites a thread holds
constexpr uint64_t NONE = ~0ull;         // no candidate (a NaN score never makes a composite, so no composite is all ones)
constexpr uint32_t LATMIN_PARTS = 256;   // most per-block latency minima per segment

enum Pred { PRED_PLAIN = 0, PRED_THRESHOLD = 1, PRED_RANK_STAGE_A = 2, PRED_RANK_STAGE_B = 3 };
enum Source { SRC_SCORES_VEC = 0, SRC_SCORES = 1, SRC_LIST = 2 };

__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_to_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

struct SelectArgs {
    const float *energy;
    const float *latency;
    const uint8_t *legal;
    uint64_t seg_len;
    uint32_t idx_bits;          // composite = key << idx_bits | idx
    float slack_factor;         // alpha - 1 (THRESHOLD)
    int alpha_inf;
    const uint32_t *lat_parts;  // THRESHOLD: [S][lat_parts_n] least latency order keys, one per block of latmin_kernel
    uint32_t lat_parts_n;
    const uint64_t *lat_thr;    // RANK stage B: [S] feasible = latency composite <= lat_thr[s]
    const uint64_t *list_in;    // SRC_LIST: [S][list_len] composites of the level before, NONE where empty
    uint64_t list_len;
    uint64_t *list_out;         // not the last level: [S][gridDim.x][k]
    uint32_t k;
    uint32_t *idx_out;          // last level: the result ...
    float *energy_out;
    uint32_t *count_out;
    uint64_t *thr_out;          // ... or (RANK stage A) only the composite the k-th smallest does not exceed
};

// ---------------------------------------------------------------- latency minimum (THRESHOLD)

// least order key of a legal, non-NaN latency in this block's slice of the segment; no atomics, so nothing
// has to be initialised: every block writes its slot
template <bool VEC>
__global__ __launch_bounds__(256) void latmin_kernel(const float *__restrict__ latency, const uint8_t *__restrict__ legal,
                                                     uint64_t seg_len, uint64_t slice, uint32_t *__restrict__ parts)
{
    const uint32_t s = blockIdx.y;
    const uint64_t seg_base = (uint64_t)s * seg_len;
    const uint64_t lo = (uint64_t)blockIdx.x * slice, hi = lo + slice < seg_len ? lo + slice : seg_len;
    uint32_t best = 0xFFFFFFFFu;
    if (VEC) {
        for (uint64_t i = lo + 4ull * threadIdx.x; i < hi; i += 4ull * 256) {
            const uint64_t g = seg_base + i;
            uint32_t flags = 0x01010101u;
            if (legal) flags = *reinterpret_cast<const uint32_t *>(legal + g);
            if (!flags) continue;
            const float4 l = *reinterpret_cast<const float4 *>(latency + g);
            const float lv[4] = {l.x, l.y, l.z, l.w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (((flags >> (8 * t)) & 0xFFu) && lv[t] == lv[t]) best = min(best, order_key(lv[t]));
        }
    } else {
        for (uint64_t i = lo + threadIdx.x; i < hi; i += 256) {
            const uint64_t g = seg_base + i;
            if (legal && !legal[g]) continue;
            const float l = latency[g];
            if (l == l) best = min(best, order_key(l));
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) best = min(best, (uint32_t)__shfl_xor((int)best, off));
    __shared__ uint32_t wave_best[4];
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) best = min(best, wave_best[w]);
        parts[(uint64_t)s * gridDim.x + blockIdx.x] = best;
    }
}

// ---------------------------------------------------------------- one level of the tournament

constexpr uint32_t NO_KEY = 0xFFFFFFFFu; // the order key of no number (only a NaN pattern maps to it): "not a candidate"
constexpr uint32_t SMALL = 512;          // a selection among at most this many composites is ranked directly

// order key of a legal candidate's value under predicate PRED, or NO_KEY if infeasible
template <int PRED>
__device__ __forceinline__ uint32_t feasible_key(const SelectArgs &a, uint32_t i, float e, float l, float tau,
                                                 uint64_t lat_thr)
{
    float value;
    if (PRED == PRED_RANK_STAGE_A) {
        value = l;
    } else {
        value = e;
        if (PRED == PRED_THRESHOLD) {
            if (!(l <= tau)) return NO_KEY;
        } else if (PRED == PRED_RANK_STAGE_B) {
            if (l != l) return NO_KEY;
            if ((((uint64_t)order_key(l) << a.idx_bits) | i) > lat_thr) return NO_KEY;
        }
    }
    if (value != value) return NO_KEY;
    return order_key(value);
}

// LDS of a block: the digit histogram of the radix select, or the arrays of the direct ranking (never both at
// once), a handful of words, and (last level) the sort buffer behind them
template <int T>
struct Shared {
    union {
        uint32_t hist[BINS];
        struct {
            uint64_t pool[SMALL];   // the composites left after the bound ...
            uint64_t ranked[SMALL]; // ... the selection in ascending order ...
            uint32_t rank[SMALL];   // ... and the number of smaller composites of each pool entry
        } small;
    };
    uint32_t wave_sum[T / 64];
    uint64_t wave_bound[T / 64];
    uint32_t found_digit, found_below, found_count, cursor;
    uint32_t lat_min;
    uint64_t any_composite; // radix select: one of the block's composites, to find the leading bits all of them share
};

// one compare-exchange step of a bitonic network over the 64 lanes of a wavefront
template <class V>
__device__ __forceinline__ V lane_exchange(V v, uint32_t stride);
template <>
__device__ __forceinline__ uint32_t lane_exchange<uint32_t>(uint32_t v, uint32_t stride)
{
    return (uint32_t)__shfl_xor((int)v, (int)stride);
}
template <>
__device__ __forceinline__ uint64_t lane_exchange<uint64_t>(uint64_t v, uint32_t stride)
{
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, (int)stride);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), (int)stride);
    return ((uint64_t)hi << 32) | lo;
}

// the 64 values of a wavefront in ascending order over the lanes (bitonic sorting network)
template <class V>
__device__ __forceinline__ V wave_sort(V v)
{
    const uint32_t lane = threadIdx.x & 63;
#pragma unroll
    for (uint32_t size = 2; size <= 64; size <<= 1)
#pragma unroll
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            const V other = lane_exchange<V>(v, stride);
            const bool keep_min = ((lane & stride) == 0) == ((lane & size) == 0);
            const V lo = v < other ? v : other, hi = v < other ? other : v;
            v = keep_min ? lo : hi;
        }
    return v;
}

template <int T>
__device__ __forceinline__ uint32_t block_sum(uint32_t v, Shared<T> &sh)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += (uint32_t)__shfl_xor((int)v, off);
    __syncthreads(); // wave_sum may still be read from an earlier use
    if ((threadIdx.x & 63) == 0) sh.wave_sum[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t total = 0;
#pragma unroll
    for (int w = 0; w < T / 64; ++w) total += sh.wave_sum[w];
    return total;
}

// A bound on the block's k-th smallest value, from the least value of every thread (V = order key or composite,
// `none` = the largest value of V, which stands for "nothing").  Each of the W wavefronts contributes
// need = ceil(k / W) values that are at most its part of the bound, k or more in all, so the k-th smallest of the
// block does not exceed the largest part.  A wavefront's part: the need-th smallest of its 64 sorted values (for
// need <= 2 the larger of the minima of `need` halves of the wavefront does: six exchange steps instead of 21).  `none` when some wavefront has too few values (then nothing may be dropped) or k is too
// large for this.
template <int T, class V>
__device__ __forceinline__ V block_bound(V least, uint32_t k, V none, Shared<T> &sh)
{
    constexpr uint32_t W = T / 64;
    const uint32_t need = (k + W - 1) / W;
    if (need > 64) return none;
    V part;
    if (need <= 2) {
        const uint32_t groups = need, lanes = 64 / groups;
        part = least;
#pragma unroll
        for (uint32_t stride = 1; stride < 64; stride <<= 1) {
            const V other = lane_exchange<V>(part, stride);
            const V lo = part < other ? part : other, hi = part < other ? other : part;
            part = stride < lanes ? lo : hi;
        }
    } else {
        const V sorted = wave_sort<V>(least);
        uint64_t picked = (uint32_t)__shfl((int)(uint32_t)sorted, (int)(need - 1));
        if (sizeof(V) == 8)
            picked |= (uint64_t)(uint32_t)__shfl((int)(uint32_t)((uint64_t)sorted >> 32), (int)(need - 1)) << 32;
        part = (V)picked;
    }
    if ((threadIdx.x & 63) == 0) sh.wave_bound[threadIdx.x >> 6] = part;
    __syncthreads();
    uint64_t bound = 0;
#pragma unroll
    for (uint32_t w = 0; w < W; ++w) bound = sh.wave_bound[w] > bound ? sh.wave_bound[w] : bound;
    return (V)bound; // one wavefront without enough values makes `none` the bound
}

// Ranks the `kept` (<= SMALL) composites of sh.small.pool: the rank of a composite is the number of smaller ones,
// which is selection and order at once (composites are distinct, so the ranks are a permutation).  With fewer
// entries than threads the counting of one entry is shared by as many threads as the block can spare.  On return
// sh.small.ranked[0 .. min(kept, k)) is the selection in ascending order.  sh.small.rank must be zero on entry.
template <int T>
__device__ __forceinline__ void rank_pool(uint32_t kept, uint32_t k, Shared<T> &sh)
{
    if (kept > T) {
        for (uint32_t entry = threadIdx.x; entry < kept; entry += T) {
            const uint64_t mine = sh.small.pool[entry];
            uint32_t smaller = 0;
            for (uint32_t j = 0; j < kept; ++j) smaller += sh.small.pool[j] < mine;
            sh.small.rank[entry] = smaller;
        }
    } else if (kept) {
        const uint32_t sharers = T / kept;                      // threads per entry, >= 1
        const uint32_t span = (kept + sharers - 1) / sharers;   // pool entries each of them compares with
        const uint32_t entry = threadIdx.x % kept, part = threadIdx.x / kept;
        if (part < sharers) {
            const uint64_t mine = sh.small.pool[entry];
            const uint32_t lo = part * span, hi = lo + span < kept ? lo + span : kept;
            uint32_t smaller = 0;
            for (uint32_t j = lo; j < hi; ++j) smaller += sh.small.pool[j] < mine;
            if (smaller) atomicAdd(&sh.small.rank[entry], smaller);
        }
    }
    __syncthreads();
    for (uint32_t entry = threadIdx.x; entry < kept; entry += T) {
        const uint32_t r = sh.small.rank[entry];
        if (r < k) sh.small.ranked[r] = sh.small.pool[entry];
    }
    __syncthreads();
}

// Radix select from the top digit down over the composites a thread holds (NONE entries do not count): the
// composite that exactly k of them do not exceed (there are at least k).  Histogram of the digit over the
// composites that match the digits fixed so far, prefix sums over the bins, the bin holding the wanted rank
// fixes the next digit; ends as soon as a whole bin is wanted.
template <int T>
__device__ uint64_t radix_threshold(const uint64_t (&c)[ITEMS], uint32_t k, uint32_t total_bits, Shared<T> &sh)
{
    constexpr int PER = BINS / T; // consecutive bins per thread in the scan
    // The leading bits that all composites of the block share select nothing: scores of one segment lie in a narrow
    // range, so without this the first digit (sign, exponent, two mantissa bits) sends every composite to a
    // handful of bins, whose LDS atomics serialise, and a pass is spent on it.
    uint64_t mine = NONE;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) mine = c[j] != NONE ? c[j] : mine;
    __syncthreads(); // the words used below may still be read from what came before
    if (mine != NONE) sh.any_composite = mine; // whichever thread's store lands last
    __syncthreads();
    const uint64_t ref = sh.any_composite;
    uint64_t differ = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) differ |= c[j] != NONE ? c[j] ^ ref : 0;
#pragma unroll
    for (uint32_t stride = 32; stride > 0; stride >>= 1) differ |= lane_exchange<uint64_t>(differ, stride);
    if ((threadIdx.x & 63) == 0) sh.wave_bound[threadIdx.x >> 6] = differ;
    __syncthreads();
    differ = 0;
#pragma unroll
    for (int w = 0; w < T / 64; ++w) differ |= sh.wave_bound[w];
    if (differ == 0) return ref; // a single composite
    uint32_t top = 64 - (uint32_t)__clzll((long long)differ);
    top = top < total_bits ? top : total_bits;
    uint64_t prefix = top < 64 ? (ref >> top) << top : 0;
    uint32_t remaining = k;
    for (;;) {
        const uint32_t bits = top < (uint32_t)DIGIT_BITS ? top : (uint32_t)DIGIT_BITS;
        const uint32_t shift = top - bits, mask = (1u << bits) - 1;
        __syncthreads(); // the histogram's space and found_* may still be read from the pass (or the use) before
#pragma unroll
        for (int j = 0; j < PER; ++j) sh.hist[threadIdx.x * PER + j] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint64_t v = c[j];
            // (a shift by 64 is undefined: the first pass of a 64-bit composite has no digits above it)
            const bool in_prefix = top >= 64 || (v >> top) == (prefix >> top);
            if (v != NONE && in_prefix) atomicAdd(&sh.hist[(uint32_t)(v >> shift) & mask], 1u);
        }
        __syncthreads();
        uint32_t local[PER], sum = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            local[j] = sh.hist[threadIdx.x * PER + j];
            sum += local[j];
        }
        uint32_t incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = (uint32_t)__shfl_up((int)incl, off);
            if ((threadIdx.x & 63) >= (uint32_t)off) incl += up;
        }
        if ((threadIdx.x & 63) == 63) sh.wave_sum[threadIdx.x >> 6] = incl;
        __syncthreads();
        uint32_t below = incl - sum;
#pragma unroll
        for (int w = 0; w < T / 64; ++w)
            if (w < (int)(threadIdx.x >> 6)) below += sh.wave_sum[w];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (below < remaining && remaining <= below + local[j]) {
                sh.found_digit = threadIdx.x * PER + j;
                sh.found_below = below;
                sh.found_count = local[j];
            }
            below += local[j];
        }
        __syncthreads();
        const uint64_t digit = sh.found_digit;
        const uint32_t under = sh.found_below, count = sh.found_count;
        prefix |= digit << shift;
        remaining -= under;
        if (shift == 0 || remaining == count) return prefix | ((shift ? (1ull << shift) : 1ull) - 1);
        top = shift;
    }
}

// The block's min(k, #candidates) smallest composites, c[j] = NONE standing for "no candidate" (entries above the
// bound are set to NONE on the way).  Returns their number n.  Either *ranked is set and sh.small.ranked[0 .. n)
// holds them in ascending order, or it is clear and they are the composites c[j] <= *thr.
// `kept`: how many entries of c are candidates within the bound; when at most SMALL, they are already in
// sh.small.pool (the caller compacted them while it built c) and get ranked directly; more go through the radix
// select.  `bounded`: a bound was applied, which only happens when at least k candidates lie within it.
template <int T>
__device__ uint32_t select_kept(const uint64_t (&c)[ITEMS], uint32_t kept, bool bounded, uint32_t k, uint32_t total_bits,
                                Shared<T> &sh, bool *ranked, uint64_t *thr)
{
    const uint32_t n = kept < k ? kept : k;
    *thr = NONE - 1; // every composite is below NONE
    *ranked = false;
    if (kept <= SMALL) {
        rank_pool<T>(kept, k, sh);
        *ranked = true;
        return n;
    }
    if (!bounded && kept <= k) return n; // all of them, in no order
    *thr = radix_threshold<T>(c, k, total_bits, sh);
    return n;
}

// Number of the block's candidates c[j] != NONE when no bound is applied (k > SMALL: at least k candidates survive
// any bound, so the direct ranking only applies when the block has few candidates to begin with): per-thread
// counts, added within the wavefront, one LDS atomic per wavefront.  With SMALL or fewer the candidates are
// compacted into the pool for the direct ranking after all.  sh.cursor must have been set to zero.
template <int T>
__device__ __forceinline__ uint32_t count_candidates(const uint64_t (&c)[ITEMS], Shared<T> &sh)
{
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) mine += c[j] != NONE;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine += (uint32_t)__shfl_xor((int)mine, off);
    __syncthreads(); // the cursor's zero is in place
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&sh.cursor, mine);
    __syncthreads();
    const uint32_t kept = sh.cursor;
    if (kept > SMALL) return kept;
    __syncthreads();
    if (threadIdx.x == 0) sh.cursor = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if (c[j] != NONE) sh.small.pool[atomicAdd(&sh.cursor, 1u)] = c[j];
    __syncthreads();
    return kept;
}

// The block's share of a list of composites (the selections of the level before): held in c, bounded, the
// survivors compacted into the pool.
template <int T>
__device__ __forceinline__ void gather_list(const uint64_t *in, uint64_t list_len, uint64_t start, uint32_t k,
                                            Shared<T> &sh, uint64_t (&c)[ITEMS], uint32_t *kept, bool *bounded)
{
    // a thread takes consecutive entries, the block's share spread evenly over its threads: the lists of blocks
    // that ranked their selection are ascending, so the least entries of the threads are spread over the lists'
    // quantiles and the bound comes out tight
    const uint64_t share = list_len - start < (uint64_t)(T * ITEMS) ? list_len - start : (uint64_t)(T * ITEMS);
    if (k > SMALL) {
        // no bound can leave few enough for the direct ranking: plain coalesced loads, everything kept
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint64_t i = (uint64_t)j * T + threadIdx.x;
            c[j] = i < share ? in[start + i] : NONE;
        }
        *bounded = false;
        *kept = count_candidates<T>(c, sh);
        return;
    }
    const uint32_t per_thread = (uint32_t)((share + T - 1) / T); // <= ITEMS
    uint64_t least = NONE;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const uint64_t i = (uint64_t)threadIdx.x * per_thread + j;
        uint64_t v = NONE;
        if ((uint32_t)j < per_thread && i < share) v = in[start + i];
        c[j] = v;
        least = v < least ? v : least;
    }
    const uint64_t bound = block_bound<T, uint64_t>(least, k, NONE, sh);
    *bounded = bound != NONE;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        if (c[j] > bound) c[j] = NONE; // bound == NONE keeps everything
        if (c[j] != NONE) {
            const uint32_t slot = atomicAdd(&sh.cursor, 1u);
            if (slot < SMALL) sh.small.pool[slot] = c[j];
        }
    }
    __syncthreads();
    *kept = sh.cursor;
}

// The block's chunk of T * ITEMS candidates of segment s (four consecutive candidates per load where VEC allows
// it): order keys of the feasible ones, bounded, the survivors turned into composites (held in c and compacted into
// the pool).
template <int T, int SRC, int PRED>
__device__ __forceinline__ void gather_scores(const SelectArgs &a, uint32_t s, Shared<T> &sh, uint64_t (&c)[ITEMS],
                                              uint32_t *kept, bool *bounded)
{
    constexpr bool NEED_E = PRED != PRED_RANK_STAGE_A, NEED_L = PRED != PRED_PLAIN;
    const uint64_t seg_base = (uint64_t)s * a.seg_len;
    const uint64_t start = (uint64_t)blockIdx.x * (T * ITEMS);
    // VEC: every load of the thread is issued here, before anything waits; none depends on another (the flags
    // decide afterwards).  Groups past the end of the segment re-read its first group and are discarded.
    // Exception: under a finite latency gate few candidates are feasible as a rule, so the energies are fetched
    // afterwards and only for groups of four that hold a feasible candidate -- a second round trip for those, but
    // close to half the bytes of the pass stay unread.
    constexpr bool ENERGY_LATER = PRED == PRED_THRESHOLD && SRC == SRC_SCORES_VEC;
    const bool energy_later = ENERGY_LATER && !a.alpha_inf;
    uint32_t flags[ITEMS / 4];
    float4 e[ITEMS / 4], l[ITEMS / 4];
    if (SRC == SRC_SCORES_VEC) {
#pragma unroll
        for (int j = 0; j < ITEMS / 4; ++j) {
            const uint64_t i = start + ((uint64_t)j * T + threadIdx.x) * 4;
            const uint64_t g = seg_base + (i < a.seg_len ? i : 0); // seg_len is a multiple of 4 on this path
            flags[j] = a.legal ? *reinterpret_cast<const uint32_t *>(a.legal + g) : 0x01010101u;
            if (NEED_L) l[j] = *reinterpret_cast<const float4 *>(a.latency + g);
            if (NEED_E && !energy_later) e[j] = *reinterpret_cast<const float4 *>(a.energy + g);
        }
    }
    // the gate, while the loads are under way
    float tau = 0.0f;
    uint64_t lat_thr = 0;
    if (PRED == PRED_THRESHOLD) {
        // tau = L_min + (alpha - 1) |L_min|, product and sum rounded separately; L_min from the per-block minima
        if (a.alpha_inf) {
            tau = __builtin_inff();
        } else {
            uint32_t best = 0xFFFFFFFFu;
            for (uint32_t p = threadIdx.x; p < a.lat_parts_n; p += T) best = min(best, a.lat_parts[(uint64_t)s * a.lat_parts_n + p]);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) best = min(best, (uint32_t)__shfl_xor((int)best, off));
            if (threadIdx.x == 0) sh.lat_min = 0xFFFFFFFFu;
            __syncthreads();
            if ((threadIdx.x & 63) == 0) atomicMin(&sh.lat_min, best);
            __syncthreads();
            best = sh.lat_min;
            if (best == 0xFFFFFFFFu) {
                tau = __builtin_inff(); // nothing legal: nothing will be feasible either
            } else {
                const float lmin = key_to_float(best);
                tau = __fadd_rn(lmin, __fmul_rn(a.slack_factor, fabsf(lmin)));
            }
        }
    } else if (PRED == PRED_RANK_STAGE_B) {
        lat_thr = a.lat_thr[s];
    }
    // order keys of the feasible candidates (32 bits each: the index is implied by the position), their least
    // per thread, the bound from those
    uint32_t key[ITEMS], least = NO_KEY;
    auto index_of = [&](int j) -> uint32_t {
        if (SRC == SRC_SCORES_VEC) return (uint32_t)(start + ((uint64_t)(j / 4) * T + threadIdx.x) * 4 + (j % 4));
        return (uint32_t)(start + (uint64_t)j * T + threadIdx.x);
    };
    if (SRC == SRC_SCORES_VEC) {
        if (ENERGY_LATER && energy_later) {
            // keep the flags of the feasible candidates only, then fetch the energies of the groups that have any
#pragma unroll
            for (int j = 0; j < ITEMS / 4; ++j) {
                const float lv[4] = {l[j].x, l[j].y, l[j].z, l[j].w};
                uint32_t f = flags[j];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (!(lv[t] <= tau)) f &= ~(0xFFu << (8 * t));
                flags[j] = f;
            }
#pragma unroll
            for (int j = 0; j < ITEMS / 4; ++j) {
                const uint64_t i = start + ((uint64_t)j * T + threadIdx.x) * 4;
                e[j] = float4{0.0f, 0.0f, 0.0f, 0.0f};
                if (flags[j] && i < a.seg_len) e[j] = *reinterpret_cast<const float4 *>(a.energy + seg_base + i);
            }
        }
#pragma unroll
        for (int j = 0; j < ITEMS / 4; ++j) {
            const uint64_t i = start + ((uint64_t)j * T + threadIdx.x) * 4;
            const uint32_t f = i < a.seg_len ? flags[j] : 0u;
            const float ev[4] = {NEED_E ? e[j].x : 0.0f, NEED_E ? e[j].y : 0.0f, NEED_E ? e[j].z : 0.0f, NEED_E ? e[j].w : 0.0f};
            const float lv[4] = {NEED_L ? l[j].x : 0.0f, NEED_L ? l[j].y : 0.0f, NEED_L ? l[j].z : 0.0f, NEED_L ? l[j].w : 0.0f};
#pragma unroll
            for (int t = 0; t < 4; ++t)
                key[4 * j + t] = ((f >> (8 * t)) & 0xFFu) ? feasible_key<PRED>(a, (uint32_t)i + t, ev[t], lv[t], tau, lat_thr)
                                                          : NO_KEY;
        }
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const uint64_t i = start + (uint64_t)j * T + threadIdx.x;
            uint32_t v = NO_KEY;
            if (i < a.seg_len) {
                const uint64_t g = seg_base + i;
                if (!a.legal || a.legal[g])
                    v = feasible_key<PRED>(a, (uint32_t)i, NEED_E ? a.energy[g] : 0.0f, NEED_L ? a.latency[g] : 0.0f, tau,
                                           lat_thr);
            }
            key[j] = v;
        }
    }
    if (a.k > SMALL) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) c[j] = key[j] != NO_KEY ? ((uint64_t)key[j] << a.idx_bits) | index_of(j) : NONE;
        *bounded = false;
        *kept = count_candidates<T>(c, sh);
        return;
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) least = min(least, key[j]);
    const uint32_t bound = block_bound<T, uint32_t>(least, a.k, NO_KEY, sh);
    *bounded = bound != NO_KEY;
    __syncthreads();
    // the candidates within the bound (all of one key, ties included) become composites
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        c[j] = NONE;
        if (key[j] != NO_KEY && key[j] <= bound) {
            c[j] = ((uint64_t)key[j] << a.idx_bits) | index_of(j);
            const uint32_t slot = atomicAdd(&sh.cursor, 1u);
            if (slot < SMALL) sh.small.pool[slot] = c[j];
        }
    }
    __syncthreads();
    *kept = sh.cursor;
}

// Selection among the gathered composites, then either the block's k slots of list_out (unused slots NONE) or,
// last level, the result.
template <int T>
__device__ __forceinline__ void select_and_emit(const SelectArgs &a, uint32_t s, const uint64_t (&c)[ITEMS], uint32_t kept,
                                                bool bounded, bool last_level, Shared<T> &sh, uint64_t *sort_buf)
{
    bool ranked;
    uint64_t thr;
    const uint32_t n_selected = select_kept<T>(c, kept, bounded, a.k, 32 + a.idx_bits, sh, &ranked, &thr);
    if (last_level && a.thr_out) {
        // RANK stage A: feasible = latency composite <= the k-th smallest (everything legal when fewer than k exist)
        if (threadIdx.x == 0) {
            uint64_t gate = NONE;
            if (n_selected == a.k) gate = ranked ? sh.small.ranked[a.k - 1] : thr;
            a.thr_out[s] = gate;
        }
        return;
    }
    if (!last_level) {
        uint64_t *out = a.list_out + ((uint64_t)s * gridDim.x + blockIdx.x) * a.k;
        if (ranked) {
            for (uint32_t i = threadIdx.x; i < n_selected; i += T) out[i] = sh.small.ranked[i];
        } else {
            __syncthreads(); // the histogram's space is done with
            if (threadIdx.x == 0) sh.cursor = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                if (c[j] <= thr) out[atomicAdd(&sh.cursor, 1u)] = c[j]; // NONE > thr; exactly n_selected qualify
        }
        for (uint32_t i = n_selected + threadIdx.x; i < a.k; i += T) out[i] = NONE;
        return;
    }
    // last level: the selection in ascending order, then unpack
    const uint64_t idx_mask = (1ull << a.idx_bits) - 1;
    auto emit = [&](uint32_t i, uint64_t v) {
        const bool valid = i < n_selected;
        a.idx_out[(uint64_t)s * a.k + i] = valid ? (uint32_t)(v & idx_mask) : 0xFFFFFFFFu;
        a.energy_out[(uint64_t)s * a.k + i] = valid ? key_to_float((uint32_t)(v >> a.idx_bits)) : __builtin_inff();
    };
    if (threadIdx.x == 0) a.count_out[s] = n_selected;
    if (ranked) {
        for (uint32_t i = threadIdx.x; i < a.k; i += T) emit(i, i < n_selected ? sh.small.ranked[i] : 0);
        return;
    }
    // bitonic sort of the selection (padded to a power of two with NONE)
    uint32_t pow2 = 2;
    while (pow2 < a.k) pow2 <<= 1;
    for (uint32_t i = threadIdx.x; i < pow2; i += T) sort_buf[i] = NONE;
    if (threadIdx.x == 0) sh.cursor = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if (c[j] <= thr) sort_buf[atomicAdd(&sh.cursor, 1u)] = c[j];
    __syncthreads();
    if (pow2 <= (uint32_t)T) {
        // one element per thread: steps whose partner sits in the same wavefront exchange registers, only the
        // wider ones go through LDS (10 of the 55 steps for 1024 elements)
        const uint32_t i = threadIdx.x;
        uint64_t v = i < pow2 ? sort_buf[i] : NONE;
        for (uint32_t size = 2; size <= pow2; size <<= 1) {
            const bool ascending = (i & size) == 0;
            for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
                uint64_t other;
                if (stride < 64) {
                    other = lane_exchange<uint64_t>(v, stride);
                } else {
                    __syncthreads(); // the reads of the step before are done
                    if (i < pow2) sort_buf[i] = v;
                    __syncthreads();
                    other = i < pow2 ? sort_buf[i ^ stride] : NONE;
                }
                const bool lower = (i & stride) == 0; // this thread keeps the smaller one of an ascending pair
                const uint64_t lo = v < other ? v : other, hi = v < other ? other : v;
                v = (lower == ascending) ? lo : hi;
            }
        }
        if (i < a.k) emit(i, v);
        return;
    }
    for (uint32_t size = 2; size <= pow2; size <<= 1)
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t t = threadIdx.x; t < pow2 / 2; t += T) {
                const uint32_t lo = 2 * t - (t & (stride - 1)); // index with the `stride` bit clear
                const uint32_t hi = lo + stride;
                const bool ascending = (lo & size) == 0;
                const uint64_t x = sort_buf[lo], y = sort_buf[hi];
                if ((x > y) == ascending) {
                    sort_buf[lo] = y;
                    sort_buf[hi] = x;
                }
            }
            __syncthreads();
        }
    for (uint32_t i = threadIdx.x; i < a.k; i += T) emit(i, i < n_selected ? sort_buf[i] : 0);
}

// One block = T threads x ITEMS candidates of segment blockIdx.y: a chunk of the score arrays, or the same number
// of composites of the list the level before wrote.  With one block per segment (gridDim.x == 1) this is the
// last level and writes the result; otherwise the block's selection goes to its k slots of list_out and a further
// launch works on the lists.  (Letting the block that finishes a segment last merge the lists inside the same
// launch was tried: on this chip blocks of one launch sit on eight dies with separate L2 caches, so lists and
// tickets have to be written through to memory -- device-scope stores and atomics, or a release fence, which
// writes the whole L2 back -- and that costs far more than the second launch: 73 us and 400 us against 32.)
template <int T, int SRC, int PRED>
__global__ __launch_bounds__(T) void select_kernel(SelectArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    Shared<T> &sh = *reinterpret_cast<Shared<T> *>(lds_raw);
    uint64_t *sort_buf = reinterpret_cast<uint64_t *>(lds_raw + ((sizeof(Shared<T>) + 15) & ~(size_t)15));
    const uint32_t s = blockIdx.y;
    uint64_t c[ITEMS];
    uint32_t kept;
    bool bounded;
    // the direct ranking's counters start at zero, the pool's cursor too (ordered before their use by the barriers
    // of the gather step)
    for (uint32_t i = threadIdx.x; i < SMALL; i += T) sh.small.rank[i] = 0;
    if (threadIdx.x == 0) sh.cursor = 0;
    if (SRC == SRC_LIST) gather_list<T>(a.list_in + (uint64_t)s * a.list_len, a.list_len, (uint64_t)blockIdx.x * (T * ITEMS), a.k, sh, c, &kept, &bounded);
    else gather_scores<T, SRC, PRED>(a, s, sh, c, &kept, &bounded);
    select_and_emit<T>(a, s, c, kept, bounded, gridDim.x == 1, sh, sort_buf);
}

// ---------------------------------------------------------------- host side

// Threads per block for a selection of k per block: 1024 (chunks of 16384) when k is large, so that a level
// still shrinks its input at least fourfold, or when the whole job is too small to fill the chip anyway and
// fewer levels matter more; 256 (chunks of 4096) otherwise.
int threads_for(uint64_t seg_len, uint32_t n_seg, uint32_t k)
{
    if (k > 256) return 1024;
    const uint64_t blocks = (uint64_t)n_seg * ((seg_len + 4095) / 4096);
    return blocks < 512 ? 1024 : 256;
}

struct Plan {
    int threads;
    uint64_t blocks0;     // level-0 blocks per segment
    uint64_t list_a, list_b; // composites per segment in the two list buffers (level 0 writes A)
};

Plan plan_for(uint64_t seg_len, uint32_t n_seg, uint32_t k)
{
    Plan p;
    p.threads = threads_for(seg_len, n_seg, k);
    const uint64_t chunk = (uint64_t)p.threads * ITEMS;
    p.blocks0 = (seg_len + chunk - 1) / chunk;
    p.list_a = p.blocks0 > 1 ? p.blocks0 * k : 0;
    const uint64_t blocks1 = (p.list_a + chunk - 1) / chunk;
    p.list_b = blocks1 > 1 ? blocks1 * k : 0;
    return p;
}

struct WsLayout {
    uint64_t lat_parts, lat_thr, list_a, list_b, total;
};

// m_latency: the latency gate of a RANK-mode call when it needs a stage of its own, else 0
WsLayout ws_layout(uint64_t seg_len, uint32_t n_seg, uint32_t k, uint32_t m_latency)
{
    Plan p = plan_for(seg_len, n_seg, k);
    if (m_latency && m_latency < seg_len) {
        const Plan q = plan_for(seg_len, n_seg, m_latency);
        p.list_a = p.list_a > q.list_a ? p.list_a : q.list_a;
        p.list_b = p.list_b > q.list_b ? p.list_b : q.list_b;
    }
    WsLayout w;
    w.lat_parts = 0;
    w.lat_thr = w.lat_parts + (uint64_t)n_seg * LATMIN_PARTS * sizeof(uint32_t);
    w.list_a = w.lat_thr + (((uint64_t)n_seg * sizeof(uint64_t) + 15) & ~15ull);
    w.list_b = w.list_a + (uint64_t)n_seg * p.list_a * sizeof(uint64_t);
    w.total = w.list_b + (uint64_t)n_seg * p.list_b * sizeof(uint64_t);
    return w;
}

bool sizes_ok(uint64_t n, uint32_t n_seg, uint32_t k)
{
    return n && n_seg && k && n % n_seg == 0 && k <= n / n_seg && n / n_seg <= 0xFFFFFFFEull && k <= ECK_MAX_K &&
           n_seg <= 65535;
}

template <int T, int SRC, int PRED>
void launch_select(const SelectArgs &a, uint32_t blocks, uint32_t n_seg, hipStream_t st)
{
    size_t lds = (sizeof(Shared<T>) + 15) & ~(size_t)15;
    if (blocks == 1 && !a.thr_out) {
        uint32_t pow2 = 2;
        while (pow2 < a.k) pow2 <<= 1;
        lds += (size_t)pow2 * sizeof(uint64_t);
    }
    hipLaunchKernelGGL((select_kernel<T, SRC, PRED>), dim3(blocks, n_seg), dim3(T), lds, st, a);
}

template <int T, int PRED>
void launch_level0(const SelectArgs &a, uint32_t blocks, uint32_t n_seg, bool vec, hipStream_t st)
{
    if (vec) launch_select<T, SRC_SCORES_VEC, PRED>(a, blocks, n_seg, st);
    else launch_select<T, SRC_SCORES, PRED>(a, blocks, n_seg, st);
}

// All levels of one selection of a.k per segment: level 0 on the score arrays, further levels on the lists.
// The last level writes idx/energy/count (or thr_out when that is set).
template <int PRED>
int32_t run_tournament(SelectArgs a, uint32_t n_seg, bool vec, uint64_t *list_a, uint64_t *list_b, hipStream_t st)
{
    const Plan p = plan_for(a.seg_len, n_seg, a.k);
    const uint64_t chunk = (uint64_t)p.threads * ITEMS;
    uint64_t blocks = p.blocks0;
    if (blocks > 0x7FFFFFFFull) return ECK_EUNSUPPORTED;
    a.list_out = list_a;
    if (p.threads == 256) launch_level0<256, PRED>(a, (uint32_t)blocks, n_seg, vec, st);
    else launch_level0<1024, PRED>(a, (uint32_t)blocks, n_seg, vec, st);
    uint64_t *in = list_a, *out = list_b;
    while (blocks > 1) {
        a.list_in = in;
        a.list_len = blocks * a.k;
        a.list_out = out;
        blocks = (a.list_len + chunk - 1) / chunk;
        if (p.threads == 256) launch_select<256, SRC_LIST, PRED_PLAIN>(a, (uint32_t)blocks, n_seg, st);
        else launch_select<1024, SRC_LIST, PRED_PLAIN>(a, (uint32_t)blocks, n_seg, st);
        uint64_t *t = in;
        in = out;
        out = t;
    }
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

} // namespace

extern "C" uint64_t topk_select_workspace_bytes(uint64_t n, uint32_t n_segments, uint32_t k)
{
    if (!sizes_ok(n, n_segments, k)) return 0;
    return ws_layout(n / n_segments, n_segments, k, 0).total;
}

extern "C" uint64_t topk_select_rank_workspace_bytes(uint64_t n, uint32_t n_segments, uint32_t k, uint32_t m_latency)
{
    if (!sizes_ok(n, n_segments, k) || m_latency == 0) return 0;
    const uint64_t seg_len = n / n_segments;
    if (m_latency < seg_len && m_latency > ECK_MAX_K) return 0;
    return ws_layout(seg_len, n_segments, k, m_latency < seg_len ? m_latency : 0).total;
}

namespace {

// argument checks shared by the entry points; *need = bytes of workspace the call takes
int32_t check_arguments(const float *energy, const float *latency, uint64_t n, uint32_t n_segments, uint32_t k, int32_t mode,
                        float alpha, uint32_t m_latency, const uint32_t *idx_out, const float *energy_out,
                        const uint32_t *count_out, bool *stage_a, WsLayout *layout)
{
    if (!energy || !idx_out || !energy_out || !count_out || n == 0 || k == 0 || n_segments == 0) return ECK_EINVAL;
    if (mode != ECK_SELECT_THRESHOLD && mode != ECK_SELECT_RANK) return ECK_EINVAL;
    if (latency && mode == ECK_SELECT_THRESHOLD && !(alpha >= 1.0f)) return ECK_EINVAL;
    if (latency && mode == ECK_SELECT_RANK && m_latency == 0) return ECK_EINVAL;
    if (n % n_segments || k > n / n_segments || n / n_segments > 0xFFFFFFFEull || n_segments > 65535) return ECK_ESHAPE;
    if (k > ECK_MAX_K) return ECK_EUNSUPPORTED;
    const uint64_t seg_len = n / n_segments;
    // a latency gate that admits the whole segment needs no first stage
    *stage_a = latency && mode == ECK_SELECT_RANK && m_latency < seg_len;
    if (*stage_a && m_latency > ECK_MAX_K) return ECK_EUNSUPPORTED;
    *layout = ws_layout(seg_len, n_segments, k, *stage_a ? m_latency : 0);
    return ECK_OK;
}

} // namespace

int32_t eck::topk_select_impl(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                              uint32_t n_segments, uint32_t k, int32_t mode, float alpha, uint32_t m_latency,
                              uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *ws, uint64_t ws_bytes,
                              void *stream, const uint32_t *known_min)
{
    bool stage_a;
    WsLayout w;
    const int32_t bad = check_arguments(energy, latency, n, n_segments, k, mode, alpha, m_latency, idx_out, energy_out,
                                        count_out, &stage_a, &w);
    if (bad != ECK_OK) return bad;
    if (!ws || ws_bytes < w.total) return ECK_EWORKSPACE;
    if ((uintptr_t)ws & 15) return ECK_EALIGN;
    const uint64_t seg_len = n / n_segments;

    SelectArgs a = {};
    a.energy = energy;
    a.latency = latency;
    a.legal = legal;
    a.seg_len = seg_len;
    a.idx_bits = 1;
    while (a.idx_bits < 32 && (1ull << a.idx_bits) < a.seg_len) ++a.idx_bits;
    a.slack_factor = alpha - 1.0f;
    a.alpha_inf = __builtin_isinf(alpha) ? 1 : 0;
    a.k = k;
    a.idx_out = idx_out;
    a.energy_out = energy_out;
    a.count_out = count_out;
    uint32_t *lat_parts = reinterpret_cast<uint32_t *>((char *)ws + w.lat_parts);
    uint64_t *lat_thr = reinterpret_cast<uint64_t *>((char *)ws + w.lat_thr);
    uint64_t *list_a = reinterpret_cast<uint64_t *>((char *)ws + w.list_a);
    uint64_t *list_b = reinterpret_cast<uint64_t *>((char *)ws + w.list_b);

    hipStream_t st = as_stream(stream);
    // four candidates per load when every group of four is aligned in all three arrays
    const bool vec = seg_len % 4 == 0 && ((uintptr_t)energy & 15) == 0 && (!latency || ((uintptr_t)latency & 15) == 0) &&
                     (!legal || ((uintptr_t)legal & 3) == 0);
    if (!latency) return run_tournament<PRED_PLAIN>(a, n_segments, vec, list_a, list_b, st);
    if (mode == ECK_SELECT_THRESHOLD) {
        if (!a.alpha_inf && known_min) {
            // L_min came with the call (one order key per segment)
            a.lat_parts = known_min;
            a.lat_parts_n = 1;
        } else if (!a.alpha_inf) {
            // L_min first: one pass over the latencies, a slice of the segment per block
            uint64_t parts = (seg_len + 4095) / 4096;
            if (parts > LATMIN_PARTS) parts = LATMIN_PARTS;
            uint64_t slice = (seg_len + parts - 1) / parts;
            slice = (slice + 1023) & ~1023ull; // whole groups of four per thread
            parts = (seg_len + slice - 1) / slice;
            if (vec) hipLaunchKernelGGL(latmin_kernel<true>, dim3((uint32_t)parts, n_segments), dim3(256), 0, st, latency, legal,
                                        seg_len, slice, lat_parts);
            else hipLaunchKernelGGL(latmin_kernel<false>, dim3((uint32_t)parts, n_segments), dim3(256), 0, st, latency, legal,
                                    seg_len, slice, lat_parts);
            a.lat_parts = lat_parts;
            a.lat_parts_n = (uint32_t)parts;
        }
        return run_tournament<PRED_THRESHOLD>(a, n_segments, vec, list_a, list_b, st);
    }
    if (!stage_a) {
        // every legal candidate with a latency that is a number passes the gate
        SelectArgs b = a;
        b.alpha_inf = 1;
        return run_tournament<PRED_THRESHOLD>(b, n_segments, vec, list_a, list_b, st);
    }
    SelectArgs first = a;
    first.k = m_latency;
    first.thr_out = lat_thr;
    const int32_t rc = run_tournament<PRED_RANK_STAGE_A>(first, n_segments, vec, list_a, list_b, st);
    if (rc != ECK_OK) return rc;
    a.lat_thr = lat_thr;
    return run_tournament<PRED_RANK_STAGE_B>(a, n_segments, vec, list_a, list_b, st);
}

extern "C" int32_t topk_select(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                               uint32_t n_segments, uint32_t k, int32_t mode, float alpha, uint32_t m_latency,
                               uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *ws, uint64_t ws_bytes,
                               void *stream)
{
    return topk_select_impl(energy, latency, legal, n, n_segments, k, mode, alpha, m_latency, idx_out, energy_out,
                            count_out, ws, ws_bytes, stream, nullptr);
}

extern "C" int32_t topk_select_known_min(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                                         uint32_t n_segments, uint32_t k, float alpha, const uint32_t *latency_min_key,
                                         uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *ws,
                                         uint64_t ws_bytes, void *stream)
{
    if (!latency || !latency_min_key) return ECK_EINVAL;
    return topk_select_impl(energy, latency, legal, n, n_segments, k, ECK_SELECT_THRESHOLD, alpha, 0, idx_out, energy_out,
                            count_out, ws, ws_bytes, stream, latency_min_key);
}

// ---------------------------------------------------------------- the entry point that allocates nothing

namespace {
constexpr int MAX_DEVICES = 64;
// the workspace of topk_select_static: one copy per GPU the library runs on, held until the process ends
__device__ __align__(256) unsigned char scratch[ECK_TOPK_STATIC_BYTES];
void *scratch_address[MAX_DEVICES]; // per device: where that device's copy of `scratch` lives
std::mutex scratch_mutex;
} // namespace

extern "C" int32_t topk_select_static(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                                      uint32_t n_segments, uint32_t k, int32_t mode, float alpha, uint32_t m_latency,
                                      uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *stream)
{
    bool stage_a;
    WsLayout w;
    const int32_t bad = check_arguments(energy, latency, n, n_segments, k, mode, alpha, m_latency, idx_out, energy_out,
                                        count_out, &stage_a, &w);
    if (bad != ECK_OK) return bad;
    if (w.total > ECK_TOPK_STATIC_BYTES) return ECK_EWORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return ECK_EDEVICE;
    }
    if (dev < 0 || dev >= MAX_DEVICES) return ECK_EUNSUPPORTED;
    void *ws;
    {
        // the array's name is a host-side stand-in; its address on the current device is looked up once per device
        std::lock_guard<std::mutex> guard(scratch_mutex);
        if (!scratch_address[dev]) {
            void *found = nullptr;
            if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) {
                (void)hipGetLastError();
                return ECK_EDEVICE;
            }
            scratch_address[dev] = found;
        }
        ws = scratch_address[dev];
    }
    // nothing in the workspace has to start at zero: every word a kernel reads was written by an earlier kernel of
    // the same call
    return topk_select_impl(energy, latency, legal, n, n_segments, k, mode, alpha, m_latency, idx_out, energy_out,
                            count_out, ws, ECK_TOPK_STATIC_BYTES, stream, nullptr);
}
