// Selection under the "low latency first, then least energy" objective
// (Sec. 4.3, 4.4; Alg. 1 LatencyEvaAndPick / EnergyModelEvaAndPick).  HIP, gfx950.
//
// Method: radix select on the composite key (order-preserving energy bits,
// index within segment), 12 bits per pass from the top, with per-block LDS
// histograms merged by integer atomics; every feasible candidate whose
// composite is at most the k-th one is then gathered and the (at most k)
// gathered entries are sorted in LDS.  Composites are distinct, so exactly
// min(k, #feasible) entries qualify and ties fall to the lower index.  Only
// integer atomics are used and the gathered set is sorted afterwards, so the
// result does not depend on execution order.
#include "eck_internal.h"

using namespace eck;

namespace {

constexpr int DIGIT_BITS = 12;
constexpr int BINS = 1 << DIGIT_BITS;
constexpr int MAX_ITEMS = 64; // most candidates per thread in the streaming kernels (a multiple of 4)
constexpr int BLOCK = 256;

enum Pred { PRED_PLAIN = 0, PRED_THRESHOLD = 1, PRED_RANK_STAGE_A = 2, PRED_RANK_STAGE_B = 3 };

struct SegState {
    uint32_t lat_min_key; // least order-key of a legal latency (THRESHOLD)
    uint32_t remaining;   // rank still to be found inside the current prefix (1-based count)
    uint32_t done;        // threshold final
    uint32_t gathered;    // entries appended by the gather kernel
    uint64_t prefix;      // composite bits fixed so far (in place, low bits zero)
    uint64_t threshold;   // final: take composites <= threshold
    uint64_t lat_threshold; // RANK: composite threshold of stage A
    uint32_t arrived;       // blocks of the running histogram pass that have merged their bins
    uint32_t pad;
};

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
    uint32_t idx_bits;   // composite = key << idx_bits | idx
    float slack_factor;  // alpha - 1 (THRESHOLD)
    int alpha_inf;
    SegState *state;
    uint32_t *hist;      // [S][BINS]
    uint64_t *gather;    // [S][k]
    uint32_t k;
    uint32_t items;      // candidates per thread in the streaming kernels (multiple of 4)
};

__device__ __forceinline__ float threshold_tau(const SelectArgs &a, const SegState &st)
{
    if (a.alpha_inf || st.lat_min_key == 0xFFFFFFFFu) return __builtin_inff();
    const float lmin = key_to_float(st.lat_min_key);
    return __fadd_rn(lmin, __fmul_rn(a.slack_factor, fabsf(lmin)));
}

__global__ void init_kernel(SegState *state, uint32_t n_seg, uint32_t *hist, uint32_t k)
{
    const uint32_t s = blockIdx.x;
    for (uint32_t b = threadIdx.x; b < BINS; b += blockDim.x) hist[(uint64_t)s * BINS + b] = 0;
    if (threadIdx.x == 0) {
        SegState st;
        st.lat_min_key = 0xFFFFFFFFu;
        st.remaining = k;
        st.done = 0;
        st.gathered = 0;
        st.prefix = 0;
        st.threshold = 0;
        st.lat_threshold = ~0ull;
        st.arrived = 0;
        st.pad = 0;
        state[s] = st;
    }
    (void)n_seg;
}

// restart the radix rounds (between RANK stage A and B)
__global__ void restart_kernel(SegState *state, uint32_t k)
{
    SegState &st = state[blockIdx.x];
    if (threadIdx.x == 0) {
        st.lat_threshold = st.threshold;
        st.remaining = k;
        st.done = 0;
        st.prefix = 0;
        st.threshold = 0;
    }
}

// Streaming order of the three full passes: a thread takes items / 4 groups of four consecutive candidates,
// consecutive lanes consecutive groups (16-byte loads of the float arrays, 4-byte loads of the flags).  The
// host launches the VEC form when segment length and pointers allow it, the scalar form otherwise.
template <bool VEC, class Visit>
__device__ __forceinline__ void stream_segment(const SelectArgs &a, uint64_t seg_base, bool want_energy,
                                               bool want_latency, Visit visit)
{
    const uint64_t start = (uint64_t)blockIdx.x * ((uint64_t)BLOCK * a.items);
    if (VEC) {
#pragma unroll 4
        for (uint32_t j = 0; j < a.items / 4; ++j) {
            const uint64_t i = start + ((uint64_t)j * BLOCK + threadIdx.x) * 4;
            if (i >= a.seg_len) break;
            const uint64_t g = seg_base + i;
            uint32_t flags = 0x01010101u;
            if (a.legal) flags = *reinterpret_cast<const uint32_t *>(a.legal + g);
            float4 e = {0, 0, 0, 0}, l = {0, 0, 0, 0};
            if (flags) {
                if (want_energy) e = *reinterpret_cast<const float4 *>(a.energy + g);
                if (want_latency) l = *reinterpret_cast<const float4 *>(a.latency + g);
            }
            const float ev[4] = {e.x, e.y, e.z, e.w}, lv[4] = {l.x, l.y, l.z, l.w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if ((flags >> (8 * t)) & 0xFFu) visit((uint32_t)i + t, ev[t], lv[t]);
        }
    } else {
#pragma unroll 4
        for (uint32_t j = 0; j < a.items; ++j) {
            const uint64_t i = start + (uint64_t)j * BLOCK + threadIdx.x;
            if (i >= a.seg_len) break;
            const uint64_t g = seg_base + i;
            if (a.legal && !a.legal[g]) continue;
            visit((uint32_t)i, want_energy ? a.energy[g] : 0.0f, want_latency ? a.latency[g] : 0.0f);
        }
    }
}

// composite of a legal candidate with scores (e, l) under predicate PRED, or false if infeasible
template <int PRED>
__device__ __forceinline__ bool composite_from(const SelectArgs &a, uint32_t i, float e, float l, float tau,
                                               uint64_t lat_thr, uint64_t *comp)
{
    float value;
    if (PRED == PRED_RANK_STAGE_A) {
        value = l;
    } else {
        value = e;
        if (PRED == PRED_THRESHOLD) {
            if (!(l <= tau)) return false;
        } else if (PRED == PRED_RANK_STAGE_B) {
            if (l != l) return false;
            if ((((uint64_t)order_key(l) << a.idx_bits) | i) > lat_thr) return false;
        }
    }
    if (value != value) return false;
    *comp = ((uint64_t)order_key(value) << a.idx_bits) | i;
    return true;
}

template <bool VEC>
__global__ __launch_bounds__(BLOCK) void latmin_kernel(SelectArgs a)
{
    const uint32_t s = blockIdx.y;
    uint32_t best = 0xFFFFFFFFu;
    stream_segment<VEC>(a, (uint64_t)s * a.seg_len, false, true, [&](uint32_t, float, float l) {
        if (l == l) best = min(best, order_key(l));
    });
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) best = min(best, (uint32_t)__shfl_xor((int)best, off));
    __shared__ uint32_t wave_best[BLOCK / 64];
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < BLOCK / 64; ++w) best = min(best, wave_best[w]);
        if (best != 0xFFFFFFFFu) atomicMin(&a.state[s].lat_min_key, best);
    }
}

__device__ void scan_segment(const SelectArgs &a, uint32_t s, uint32_t shift, uint32_t bits, int first_pass);

// histogram of the digit at `shift` (width `bits`) over feasible composites that match the prefix above
// it.  The block that finishes a segment last (a ticket from an integer atomic, after a device-wide
// fence) also locates the bin of the wanted rank and prepares the next pass.
template <int PRED, bool VEC>
__global__ __launch_bounds__(BLOCK) void hist_kernel(SelectArgs a, uint32_t shift, uint32_t bits, int first_pass)
{
    const uint32_t s = blockIdx.y;
    const SegState st = a.state[s];
    if (st.done) return;
    __shared__ uint32_t bins[BINS];
    for (uint32_t b = threadIdx.x; b < BINS; b += BLOCK) bins[b] = 0;
    __syncthreads();
    const float tau = PRED == PRED_THRESHOLD ? threshold_tau(a, st) : 0.0f;
    const uint32_t top = shift + bits; // bits at and above `top` must equal the prefix
    const uint32_t mask = (1u << bits) - 1;
    constexpr bool NEED_E = PRED != PRED_RANK_STAGE_A, NEED_L = PRED != PRED_PLAIN;
    stream_segment<VEC>(a, (uint64_t)s * a.seg_len, NEED_E, NEED_L, [&](uint32_t i, float e, float l) {
        uint64_t comp;
        if (!composite_from<PRED>(a, i, e, l, tau, st.lat_threshold, &comp)) return;
        if (top < 64 && (comp >> top) != (st.prefix >> top)) return;
        atomicAdd(&bins[(uint32_t)(comp >> shift) & mask], 1u);
    });
    __syncthreads();
    uint32_t *out = a.hist + (uint64_t)s * BINS;
    for (uint32_t b = threadIdx.x; b < BINS; b += BLOCK)
        if (bins[b]) atomicAdd(&out[b], bins[b]);
    // Last block of the segment?  Every merge above is a device-scope atomic, complete (performed where
    // all compute units see it) once this wavefront's memory counter has drained, which the barrier's
    // release makes every wavefront do; the ticket is drawn after that, and the block that draws the last
    // one reads the bins with device-scope atomic loads.  No cache write-back is involved, so no
    // device-wide fence (which costs a full L2 write-back per block) is needed.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    __shared__ uint32_t ticket;
    if (threadIdx.x == 0) ticket = atomicAdd(&a.state[s].arrived, 1u);
    __syncthreads();
    if (ticket != gridDim.x - 1) return;
    scan_segment(a, s, shift, bits, first_pass);
}

// Run by one block per segment once the segment's histogram is complete: locate the bin that holds the
// remaining-th smallest, fix its digit, clear the histogram and the arrival count for the next pass.
__device__ void scan_segment(const SelectArgs &a, uint32_t s, uint32_t shift, uint32_t bits, int first_pass)
{
    SegState &st = a.state[s];
    // read before any thread may update the state (updates happen after the barriers below)
    const uint32_t remaining = st.remaining;
    const uint64_t prefix_in = st.prefix;
    uint32_t *h = a.hist + (uint64_t)s * BINS;
    const uint32_t nbins = 1u << bits;
    constexpr int PER = BINS / BLOCK; // consecutive bins per thread
    uint32_t local[PER], sum = 0;
    (void)nbins; // bins at and above nbins were never incremented
    // The other blocks' contributions were made by device-scope atomics and are complete; read them past
    // every cache level that is not shared by the whole device, then leave zero behind for
    // the next pass (a later kernel).
    static_assert(PER == 16, "four 16-byte loads per thread");
    {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        u32x4 q0, q1, q2, q3;
        const uint32_t *mine = h + threadIdx.x * PER;
        // the compiler would wait for each cache-bypassing load separately; here all four are in flight
        asm volatile("global_load_dwordx4 %0, %4, off sc0 sc1\n\t"
                     "global_load_dwordx4 %1, %4, off offset:16 sc0 sc1\n\t"
                     "global_load_dwordx4 %2, %4, off offset:32 sc0 sc1\n\t"
                     "global_load_dwordx4 %3, %4, off offset:48 sc0 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3)
                     : "v"(mine)
                     : "memory");
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            local[e] = q0[e];
            local[4 + e] = q1[e];
            local[8 + e] = q2[e];
            local[12 + e] = q3[e];
        }
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        h[threadIdx.x * PER + j] = 0;
        sum += local[j];
    }
    // exclusive prefix of the per-thread sums: shuffles inside a wavefront, then the four wavefront totals
    uint32_t incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, off);
        if ((threadIdx.x & 63) >= (uint32_t)off) incl += up;
    }
    __shared__ uint32_t wave_total[BLOCK / 64];
    if ((threadIdx.x & 63) == 63) wave_total[threadIdx.x >> 6] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < BLOCK / 64; ++w) {
        if (w < (int)(threadIdx.x >> 6)) before += wave_total[w];
        total += wave_total[w];
    }
    const uint32_t first_below = before + incl - sum; // candidates in the bins of lower threads
    if (threadIdx.x == 0) st.arrived = 0;
    if (first_pass && total < remaining) {
        // fewer feasible candidates than k: take them all
        if (threadIdx.x == 0) {
            st.threshold = ~0ull;
            st.done = 1;
        }
        return;
    }
    uint32_t below = first_below;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const uint32_t c = local[j];
        if (below < remaining && remaining <= below + c) {
            // this bin holds the target
            const uint64_t digit = threadIdx.x * PER + j;
            const uint64_t prefix = prefix_in | (digit << shift);
            st.prefix = prefix;
            st.remaining = remaining - below;
            if (shift == 0 || remaining == below + c) {
                // last digit fixed, or the whole bin is wanted: everything up to the bin's top qualifies
                st.threshold = prefix | ((shift ? (1ull << shift) : 1ull) - 1);
                st.done = 1;
            }
        }
        below += c;
    }
}

template <int PRED, bool VEC>
__global__ __launch_bounds__(BLOCK) void gather_kernel(SelectArgs a)
{
    const uint32_t s = blockIdx.y;
    const SegState st = a.state[s];
    const float tau = PRED == PRED_THRESHOLD ? threshold_tau(a, st) : 0.0f;
    constexpr bool NEED_E = PRED != PRED_RANK_STAGE_A, NEED_L = PRED != PRED_PLAIN;
    stream_segment<VEC>(a, (uint64_t)s * a.seg_len, NEED_E, NEED_L, [&](uint32_t i, float e, float l) {
        uint64_t comp;
        if (!composite_from<PRED>(a, i, e, l, tau, st.lat_threshold, &comp)) return;
        if (comp > st.threshold) return;
        const uint32_t slot = atomicAdd(&a.state[s].gathered, 1u);
        if (slot < a.k) a.gather[(uint64_t)s * a.k + slot] = comp; // never more than k qualify
    });
}

// one block per segment: bitonic sort of the gathered composites, then unpack
__global__ __launch_bounds__(BLOCK) void sort_kernel(SelectArgs a, uint32_t pow2, uint32_t *idx_out, float *energy_out,
                                                     uint32_t *count_out)
{
    extern __shared__ uint64_t keys[];
    const uint32_t s = blockIdx.x;
    const uint32_t count = min(a.state[s].gathered, a.k);
    for (uint32_t i = threadIdx.x; i < pow2; i += BLOCK) keys[i] = i < count ? a.gather[(uint64_t)s * a.k + i] : ~0ull;
    __syncthreads();
    for (uint32_t size = 2; size <= pow2; size <<= 1)
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t t = threadIdx.x; t < pow2 / 2; t += BLOCK) {
                const uint32_t lo = 2 * t - (t & (stride - 1)); // index with the `stride` bit clear
                const uint32_t hi = lo + stride;
                const bool ascending = (lo & size) == 0;
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x > y) == ascending) {
                    keys[lo] = y;
                    keys[hi] = x;
                }
            }
            __syncthreads();
        }
    const uint64_t idx_mask = (1ull << a.idx_bits) - 1;
    for (uint32_t i = threadIdx.x; i < a.k; i += BLOCK) {
        const uint64_t c = keys[i];
        const bool valid = i < count;
        idx_out[(uint64_t)s * a.k + i] = valid ? (uint32_t)(c & idx_mask) : 0xFFFFFFFFu;
        energy_out[(uint64_t)s * a.k + i] = valid ? key_to_float((uint32_t)(c >> a.idx_bits)) : __builtin_inff();
    }
    if (threadIdx.x == 0) count_out[s] = count;
}

uint32_t next_pow2(uint32_t v)
{
    uint32_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

struct WsLayout {
    uint64_t state, hist, gather, total;
};

WsLayout ws_layout(uint32_t n_seg, uint32_t k)
{
    WsLayout w;
    w.state = 0;
    w.hist = w.state + (uint64_t)n_seg * sizeof(SegState);
    w.gather = w.hist + (uint64_t)n_seg * BINS * sizeof(uint32_t);
    w.total = w.gather + (uint64_t)n_seg * k * sizeof(uint64_t);
    return w;
}

bool sizes_ok(uint64_t n, uint32_t n_seg, uint32_t k)
{
    return n && n_seg && k && n % n_seg == 0 && k <= n / n_seg && n / n_seg <= 0xFFFFFFFEull && k <= ECK_MAX_K &&
           n_seg <= 65535;
}

template <int PRED>
int32_t radix_rounds(const SelectArgs &a, uint32_t n_seg, bool vec, hipStream_t st)
{
    const uint32_t total_bits = 32 + a.idx_bits;
    const uint32_t blocks = (uint32_t)((a.seg_len + (uint64_t)BLOCK * a.items - 1) / ((uint64_t)BLOCK * a.items));
    int first = 1;
    for (uint32_t consumed = 0; consumed < total_bits; consumed += DIGIT_BITS) {
        const uint32_t bits = total_bits - consumed < DIGIT_BITS ? total_bits - consumed : DIGIT_BITS;
        const uint32_t shift = total_bits - consumed - bits;
        if (vec)
            hipLaunchKernelGGL((hist_kernel<PRED, true>), dim3(blocks, n_seg), dim3(BLOCK), 0, st, a, shift, bits, first);
        else
            hipLaunchKernelGGL((hist_kernel<PRED, false>), dim3(blocks, n_seg), dim3(BLOCK), 0, st, a, shift, bits, first);
        first = 0;
    }
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

template <int PRED>
void launch_gather(const SelectArgs &a, dim3 grid, bool vec, hipStream_t st)
{
    if (vec) hipLaunchKernelGGL((gather_kernel<PRED, true>), grid, dim3(BLOCK), 0, st, a);
    else hipLaunchKernelGGL((gather_kernel<PRED, false>), grid, dim3(BLOCK), 0, st, a);
}

} // namespace

extern "C" uint64_t topk_select_workspace_bytes(uint64_t n, uint32_t n_segments, uint32_t k)
{
    if (!sizes_ok(n, n_segments, k)) return 0;
    return ws_layout(n_segments, k).total;
}

extern "C" int32_t topk_select(const float *energy, const float *latency, const uint8_t *legal, uint64_t n,
                               uint32_t n_segments, uint32_t k, int32_t mode, float alpha, uint32_t m_latency,
                               uint32_t *idx_out, float *energy_out, uint32_t *count_out, void *ws, uint64_t ws_bytes,
                               void *stream)
{
    if (!energy || !idx_out || !energy_out || !count_out || n == 0 || k == 0 || n_segments == 0) return ECK_EINVAL;
    if (mode != ECK_SELECT_THRESHOLD && mode != ECK_SELECT_RANK) return ECK_EINVAL;
    if (latency && mode == ECK_SELECT_THRESHOLD && !(alpha >= 1.0f)) return ECK_EINVAL;
    if (latency && mode == ECK_SELECT_RANK && m_latency == 0) return ECK_EINVAL;
    if (n % n_segments || k > n / n_segments || n / n_segments > 0xFFFFFFFEull || n_segments > 65535) return ECK_ESHAPE;
    if (k > ECK_MAX_K) return ECK_EUNSUPPORTED;
    const WsLayout w = ws_layout(n_segments, k);
    if (!ws || ws_bytes < w.total) return ECK_EWORKSPACE;
    if ((uintptr_t)ws & 15) return ECK_EALIGN;

    SelectArgs a;
    a.energy = energy;
    a.latency = latency;
    a.legal = legal;
    a.seg_len = n / n_segments;
    a.idx_bits = 1;
    while (a.idx_bits < 32 && (1ull << a.idx_bits) < a.seg_len) ++a.idx_bits;
    a.slack_factor = alpha - 1.0f;
    a.alpha_inf = __builtin_isinf(alpha) ? 1 : 0;
    a.state = reinterpret_cast<SegState *>((char *)ws + w.state);
    a.hist = reinterpret_cast<uint32_t *>((char *)ws + w.hist);
    a.gather = reinterpret_cast<uint64_t *>((char *)ws + w.gather);
    a.k = k;
    // Work per block: every block pays for clearing and merging a 4096-bin histogram and for one ticket,
    // so blocks are made as large as keeps about eight of them per compute unit.
    {
        int cus = 256;
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const uint64_t per_thread = n / ((uint64_t)BLOCK * 8 * (uint64_t)cus);
        a.items = 4;
        while (a.items < MAX_ITEMS && a.items < per_thread) a.items *= 2;
    }

    hipStream_t st = as_stream(stream);
    const uint32_t blocks = (uint32_t)((a.seg_len + (uint64_t)BLOCK * a.items - 1) / ((uint64_t)BLOCK * a.items));
    const dim3 stream_grid(blocks, n_segments);
    hipLaunchKernelGGL(init_kernel, dim3(n_segments), dim3(BLOCK), 0, st, a.state, n_segments, a.hist, k);
    // four candidates per load when every group of four is aligned in all three arrays
    const bool vec = a.seg_len % 4 == 0 && ((uintptr_t)energy & 15) == 0 && (!latency || ((uintptr_t)latency & 15) == 0) &&
                     (!legal || ((uintptr_t)legal & 3) == 0);
    int32_t rc = ECK_OK;
    if (!latency) {
        rc = radix_rounds<PRED_PLAIN>(a, n_segments, vec, st);
        if (rc == ECK_OK) launch_gather<PRED_PLAIN>(a, stream_grid, vec, st);
    } else if (mode == ECK_SELECT_THRESHOLD) {
        if (vec) hipLaunchKernelGGL(latmin_kernel<true>, stream_grid, dim3(BLOCK), 0, st, a);
        else hipLaunchKernelGGL(latmin_kernel<false>, stream_grid, dim3(BLOCK), 0, st, a);
        rc = radix_rounds<PRED_THRESHOLD>(a, n_segments, vec, st);
        if (rc == ECK_OK) launch_gather<PRED_THRESHOLD>(a, stream_grid, vec, st);
    } else {
        SelectArgs stage_a = a;
        stage_a.k = m_latency;
        hipLaunchKernelGGL(restart_kernel, dim3(n_segments), dim3(64), 0, st, a.state, m_latency);
        rc = radix_rounds<PRED_RANK_STAGE_A>(stage_a, n_segments, vec, st);
        if (rc == ECK_OK) {
            hipLaunchKernelGGL(restart_kernel, dim3(n_segments), dim3(64), 0, st, a.state, k);
            rc = radix_rounds<PRED_RANK_STAGE_B>(a, n_segments, vec, st);
        }
        if (rc == ECK_OK) launch_gather<PRED_RANK_STAGE_B>(a, stream_grid, vec, st);
    }
    if (rc != ECK_OK) return rc;
    const uint32_t pow2 = next_pow2(k < 2 ? 2 : k);
    hipLaunchKernelGGL(sort_kernel, dim3(n_segments), dim3(BLOCK), pow2 * sizeof(uint64_t), st, a, pow2, idx_out,
                       energy_out, count_out);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}
