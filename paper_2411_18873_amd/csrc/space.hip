// Schedule spaces, candidate generation and analytic features (HIP, gfx950).
//
// candidate_enumerate: Sec. 6.4 (random initial population) and Alg. 1
// GeneticReproduction (mutation).  features_compute: Sec. 5.3 / 5.4 feature
// categories; Table 5 fixes grid, block, global-load, global-store and
// shared-store counts.
#include <algorithm>
#include <cstring>
#include <new>

#include "eck_internal.h"

using namespace eck;

// ------------------------------------------------------------------ host side

namespace {

// ordered factorisations n = f0*f1*f2*f3, lexicographic, appended as 4 x uint16
uint32_t append_factorisations(uint32_t n, std::vector<uint16_t> *out)
{
    std::vector<uint32_t> divs;
    for (uint32_t d = 1; d * d <= n; ++d)
        if (n % d == 0) {
            divs.push_back(d);
            if (d != n / d) divs.push_back(n / d);
        }
    std::sort(divs.begin(), divs.end());
    uint32_t count = 0;
    for (uint32_t a : divs)
        for (uint32_t b : divs) {
            if ((n / a) % b) continue;
            const uint32_t rest = n / a / b;
            for (uint32_t c : divs) {
                if (c > rest) break;
                if (rest % c) continue;
                if (out) {
                    out->push_back((uint16_t)a);
                    out->push_back((uint16_t)b);
                    out->push_back((uint16_t)c);
                    out->push_back((uint16_t)(rest / c));
                }
                ++count;
            }
        }
    return count;
}

bool pow2_leq(uint64_t v, int bits) { return v < (1ull << bits); }

// floor(log2) fixed point with 10 mantissa bits, as 1024*e + m  (v >= 1)
__host__ __device__ inline uint32_t log2_q10(uint64_t v)
{
    int e = 0;
#if defined(__HIP_DEVICE_COMPILE__)
    e = 63 - __clzll((long long)v);
#else
    while ((v >> e) > 1) ++e;
#endif
    const uint64_t frac = v ^ (1ull << e);
    const uint32_t m = e >= 10 ? (uint32_t)(frac >> (e - 10)) : (uint32_t)(frac << (10 - e));
    return ((uint32_t)e << 10) + m;
}


// Upload the space once: its parameters, then its factorisation tables.
int32_t ensure_device_copy(eck_space *sp)
{
    if (sp->d_blob) return ECK_OK;
    int dev = 0;
    ECK_HIP_TRY(hipGetDevice(&dev));
    const size_t table_bytes = sp->tables.size() * sizeof(uint16_t);
    std::vector<unsigned char> host(kDevHeader + ((table_bytes + 15) & ~(size_t)15), 0); // tables are read 16 bytes at a time
    memcpy(host.data(), &sp->prm, sizeof(SpaceParams));
    if (table_bytes) memcpy(host.data() + kDevHeader, sp->tables.data(), table_bytes);
    ECK_HIP_TRY(hipMalloc((void **)&sp->d_blob, host.size()));
    if (hipMemcpy(sp->d_blob, host.data(), host.size(), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(sp->d_blob);
        sp->d_blob = nullptr;
        return ECK_EDEVICE;
    }
    sp->device = dev;
    return ECK_OK;
}

} // namespace

extern "C" int32_t eck_version(void) { return 100; }

extern "C" int32_t eck_space_create(const eck_problem *pb, int32_t kind, eck_space **out)
{
    if (!pb || !out) return ECK_EINVAL;
    *out = nullptr;
    if (kind != ECK_SPACE_KNOB && kind != ECK_SPACE_SPLIT && kind != ECK_SPACE_SPLIT_XRED) return ECK_EINVAL;
    if (pb->elem_bytes != 2 && pb->elem_bytes != 4) return ECK_EINVAL;
    if (pb->hw_num_cu < 1 || pb->hw_wave < 1 || pb->hw_lds_bytes < 1 || pb->hw_max_threads_cu < 1 ||
        pb->hw_max_blocks_cu < 1)
        return ECK_EINVAL;

    SpaceParams p;
    std::memset(&p, 0, sizeof(p));
    p.kind = kind;
    p.op = pb->op;
    p.R = p.S = p.stride = 1;
    p.elem_bytes = (uint32_t)pb->elem_bytes;
    p.hw_num_cu = (uint32_t)pb->hw_num_cu;
    p.hw_wave = (uint32_t)pb->hw_wave;
    p.hw_lds_bytes = (uint32_t)pb->hw_lds_bytes;
    p.hw_max_threads_cu = (uint32_t)pb->hw_max_threads_cu;
    p.hw_max_blocks_cu = (uint32_t)pb->hw_max_blocks_cu;
    bool present[NAX] = {false, false, false, false, false};
    uint64_t in_elems = 0, w_elems = 0, opA_bound = 0, opB_bound = 0, halo_growth = 1;

    for (int i = 0; i < 8; ++i)
        if (pb->dim[i] < 0) return ECK_EINVAL;
    if (pb->op == ECK_OP_GEMM || pb->op == ECK_OP_BGEMM) {
        const uint64_t B = pb->dim[0], M = pb->dim[1], N = pb->dim[2], K = pb->dim[3];
        if (pb->op == ECK_OP_GEMM && B != 1) return ECK_EINVAL;
        p.ext[0] = (uint32_t)B; p.ext[1] = (uint32_t)M; p.ext[2] = (uint32_t)N; p.ext[3] = 1; p.ext[4] = (uint32_t)K;
        present[0] = pb->op == ECK_OP_BGEMM;
        present[1] = present[2] = present[4] = true;
        p.vec_axis = 2;
        in_elems = B * M * K;
        w_elems = B * K * N;
    } else if (pb->op == ECK_OP_CONV2D) {
        if (kind == ECK_SPACE_KNOB) return ECK_EUNSUPPORTED;
        const uint64_t N = pb->dim[0], C = pb->dim[1], K = pb->dim[2], H = pb->dim[3], W = pb->dim[4];
        const uint64_t R = pb->dim[5], S = pb->dim[6];
        const uint64_t stride = (uint32_t)pb->dim[7] & 0xFFFFu, pad = ((uint32_t)pb->dim[7] >> 16) & 0xFFFFu;
        if (!R || !S || !stride || H + 2 * pad < R || W + 2 * pad < S) return ECK_EINVAL;
        if (R > 255 || S > 255 || stride > 255) return ECK_EUNSUPPORTED;
        p.R = (uint32_t)R; p.S = (uint32_t)S; p.stride = (uint32_t)stride;
        p.ext[0] = (uint32_t)N; p.ext[1] = (uint32_t)K;
        p.ext[2] = (uint32_t)((H + 2 * pad - R) / stride + 1);
        p.ext[3] = (uint32_t)((W + 2 * pad - S) / stride + 1);
        p.ext[4] = (uint32_t)C;
        for (bool &b : present) b = true;
        p.vec_axis = 3;
        in_elems = N * C * H * W;
        w_elems = K * C * R * S;
        halo_growth = (stride + R) * (stride + S);
    } else {
        return ECK_EINVAL;
    }
    for (int a = 0; a < NAX; ++a)
        if (p.ext[a] == 0) return ECK_EINVAL;
    // original dims must fit 16 bits too (ext[] was narrowed from them)
    for (int i = 0; i < (pb->op == ECK_OP_CONV2D ? 5 : 4); ++i)
        if (pb->dim[i] < 1 || pb->dim[i] > 65535) return pb->dim[i] < 1 ? ECK_EINVAL : ECK_EUNSUPPORTED;

    // range limits that keep the kernels' 32/64-bit arithmetic exact.  Knob tiles pad M and N to
    // below ext + 256 (M twice that when the thread rows overhang the tile) and K to below ext + 64.
    const uint64_t pad_sp = kind == ECK_SPACE_KNOB ? 255 : 0, pad_red = kind == ECK_SPACE_KNOB ? 63 : 0;
    uint64_t out_pad = 1;
    for (int a = 0; a < RED_AXIS; ++a) {
        uint64_t e = p.ext[a] + ((a == 1 || a == 2) ? pad_sp : 0);
        if (a == 1 && kind == ECK_SPACE_KNOB) e *= 2;
        if (out_pad > (1ull << 40)) return ECK_EUNSUPPORTED;
        out_pad *= e;
    }
    const uint64_t red_pad = (uint64_t)(p.ext[RED_AXIS] + pad_red) * p.R * p.S;
    if (!pow2_leq(out_pad + 1, 32) || !pow2_leq(red_pad, 24) || !pow2_leq(out_pad * red_pad, 47))
        return ECK_EUNSUPPORTED;
    if (pb->op == ECK_OP_CONV2D) {
        opA_bound = (uint64_t)p.ext[0] * p.ext[4] * ((uint64_t)(p.ext[2] - 1) * p.stride + p.R) *
                    ((uint64_t)(p.ext[3] - 1) * p.stride + p.S);
        opB_bound = (uint64_t)p.ext[1] * p.ext[4] * p.R * p.S;
        if (!pow2_leq(out_pad * p.ext[4] * halo_growth, 46)) return ECK_EUNSUPPORTED;
    } else {
        opA_bound = (uint64_t)p.ext[0] * 2 * (p.ext[1] + pad_sp) * (p.ext[4] + pad_red);
        opB_bound = (uint64_t)p.ext[0] * (p.ext[2] + pad_sp) * (p.ext[4] + pad_red);
    }
    if (!pow2_leq(opA_bound, 31) || !pow2_leq(opB_bound, 31)) return ECK_EUNSUPPORTED;

    p.true_out = (uint64_t)p.ext[0] * p.ext[1] * p.ext[2] * p.ext[3];
    p.true_red = (uint64_t)p.ext[4] * p.R * p.S;
    p.flop_useful = 2 * p.true_out * p.true_red;
    p.compulsory_in_bytes = (in_elems + w_elems) * p.elem_bytes;
    p.compulsory_bytes = (in_elems + w_elems + p.true_out) * p.elem_bytes;
    {
        const uint64_t constants[6] = {p.flop_useful, p.compulsory_bytes, p.elem_bytes, (uint64_t)p.op, p.true_out,
                                       p.true_red};
        for (int c = 0; c < 6; ++c) p.const_q10[c] = log2_q10(constants[c] + 1);
    }

    eck_space *sp = new (std::nothrow) eck_space();
    if (!sp) return ECK_EDEVICE;
    sp->pb = *pb;
    std::memset(sp->table_n, 0, sizeof(sp->table_n));
    if (kind == ECK_SPACE_KNOB) {
        static const uint32_t radices[6] = {5, 5, 4, 4, 4, 4};
        p.n_genes = 6;
        for (int g = 0; g < 6; ++g) p.radix[g] = radices[g];
    } else {
        int s = 0;
        for (int a = 0; a < NAX; ++a) {
            if (!present[a]) continue;
            p.table_off[s] = (uint32_t)(sp->tables.size() / 4);
            const uint32_t cnt = append_factorisations(p.ext[a], &sp->tables);
            if (cnt > 65535) {
                delete sp;
                return ECK_EUNSUPPORTED;
            }
            sp->table_n[s] = cnt;
            p.split_axis[s] = a;
            p.radix[s] = cnt;
            ++s;
        }
        p.n_split = s;
        p.radix[s] = 5;
        p.radix[s + 1] = 4;
        p.n_genes = s + 2;
        p.table_total = (uint32_t)(sp->tables.size() / 4);
    }
    uint64_t size = 1;
    for (int g = 0; g < p.n_genes; ++g) {
        if (size && size > UINT64_MAX / p.radix[g]) size = 0;
        size *= p.radix[g];
    }
    sp->size = size;
    sp->prm = p;
    *out = sp;
    return ECK_OK;
}

extern "C" int32_t eck_space_upload(eck_space *sp)
{
    if (!sp) return ECK_EINVAL;
    return ensure_device_copy(sp);
}

extern "C" void eck_space_destroy(eck_space *sp)
{
    if (!sp) return;
    if (sp->d_blob) {
        (void)hipDeviceSynchronize();
        (void)hipFree(sp->d_blob);
    }
    delete sp;
}

extern "C" int32_t eck_space_info(const eck_space *sp, int32_t *n_genes, uint32_t *radix, uint64_t *size)
{
    if (!sp || !n_genes || !radix || !size) return ECK_EINVAL;
    *n_genes = sp->prm.n_genes;
    for (int g = 0; g < ECK_MAX_GENES; ++g) radix[g] = g < sp->prm.n_genes ? sp->prm.radix[g] : 0;
    *size = sp->size;
    return ECK_OK;
}

extern "C" int32_t eck_space_table(const eck_space *sp, int32_t gene, uint32_t *out, uint32_t capacity)
{
    if (!sp || sp->prm.kind == ECK_SPACE_KNOB || gene < 0 || gene >= sp->prm.n_split) return ECK_EINVAL;
    const uint32_t n = sp->table_n[gene];
    if (out) {
        const uint16_t *src = sp->tables.data() + 4ull * sp->prm.table_off[gene];
        for (uint32_t i = 0; i < n && i < capacity; ++i)
            for (int l = 0; l < 4; ++l) out[4 * i + l] = src[4 * i + l];
    }
    return (int32_t)n;
}

// --------------------------------------------------------------- enumeration

namespace {

__device__ __forceinline__ uint64_t splitmix_finalise(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

// Kernel arguments of a batch: where each space's device copy lives, and the
// SplitMix64 state its stream starts from.  Block row y works on space y, whose
// candidates occupy columns [y*n, (y+1)*n) of the gene / feature matrices.
struct SpaceBatch {
    const unsigned char *dev[ECK_MAX_BATCH];
};
struct StreamBatch {
    uint64_t state[ECK_MAX_BATCH];
};

template <int MODE>
__global__ __launch_bounds__(256) void enumerate_kernel(SpaceBatch spaces, StreamBatch streams, uint64_t first,
                                                        uint64_t n, const uint16_t *__restrict__ parents,
                                                        uint32_t n_parents, uint64_t ld_parents, uint32_t p_mut,
                                                        uint16_t *__restrict__ genes, uint64_t ld)
{
    const uint32_t s = blockIdx.y;
    const SpaceParams &p = *reinterpret_cast<const SpaceParams *>(spaces.dev[s]);
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t c = first + i;
    const uint64_t col = (uint64_t)s * n + i;
    if (MODE == ECK_MODE_EXHAUSTIVE) {
        uint64_t rest = c;
        for (int g = p.n_genes - 1; g >= 0; --g) {
            const uint64_t q = rest / p.radix[g];
            genes[(uint64_t)g * ld + col] = (uint16_t)(rest - q * p.radix[g]);
            rest = q;
        }
    } else {
        // generator state before the first gene's word: stream state + gamma * 16c
        uint64_t state = streams.state[s] + kGamma * (c << 4);
        constexpr bool INHERITS = MODE == ECK_MODE_MUTATE || MODE == ECK_MODE_CROSSOVER;
        const uint64_t parent = INHERITS ? (uint64_t)s * n_parents + (uint32_t)(c % n_parents) : 0;
        // crossover: the second parent comes from word 14 of the child, the per-gene source bits from word 15
        uint64_t second = parent, from_second = 0;
        if (MODE == ECK_MODE_CROSSOVER) {
            second = (uint64_t)s * n_parents + __umulhi((uint32_t)splitmix_finalise(state + kGamma * 15), n_parents);
            from_second = splitmix_finalise(state + kGamma * 16);
        }
        for (int g = 0; g < p.n_genes; ++g) {
            state += kGamma;
            const uint64_t u = splitmix_finalise(state);
            uint32_t value = __umulhi((uint32_t)u, p.radix[g]);
            if (INHERITS) {
                const uint64_t source = ((from_second >> g) & 1) ? second : parent;
                const uint32_t inherited = parents[(uint64_t)g * ld_parents + source];
                value = ((uint32_t)(u >> 32) < p_mut) ? value : inherited;
            }
            genes[(uint64_t)g * ld + col] = (uint16_t)value;
        }
    }
}

// SplitMix64 state of stream (seed, round)
uint64_t stream_state(uint64_t seed, uint32_t round)
{
    uint64_t z = seed + kGamma * ((uint64_t)round + 1);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// The spaces of one launch must agree in what the kernels' template and loop bounds depend on.
int32_t check_batch(const eck_space *const *spaces, uint32_t n_spaces)
{
    if (!spaces || n_spaces == 0) return ECK_EINVAL;
    if (n_spaces > ECK_MAX_BATCH) return ECK_EUNSUPPORTED;
    for (uint32_t s = 0; s < n_spaces; ++s) {
        if (!spaces[s]) return ECK_EINVAL;
        const SpaceParams &a = spaces[s]->prm, &b = spaces[0]->prm;
        if (a.kind != b.kind || a.op != b.op || a.n_genes != b.n_genes) return ECK_ESHAPE;
    }
    return ECK_OK;
}

// Makes sure every space is resident on the device and fills the kernels' batch argument.
int32_t upload_batch(const eck_space *const *spaces, uint32_t n_spaces, SpaceBatch *batch)
{
    for (uint32_t s = 0; s < n_spaces; ++s) {
        eck_space *sp = const_cast<eck_space *>(spaces[s]);
        const int32_t rc = ensure_device_copy(sp);
        if (rc != ECK_OK) return rc;
        batch->dev[s] = sp->d_blob;
    }
    return ECK_OK;
}

int32_t enumerate_launch(const eck_space *const *spaces, uint32_t n_spaces, int32_t mode, const uint64_t *seeds,
                         uint32_t round, uint64_t first_index, uint64_t n, const uint16_t *parents,
                         uint32_t n_parents, uint32_t p_mut_q32, uint16_t *genes_out, uint64_t ld, void *stream)
{
    if (!seeds || !genes_out || n == 0) return ECK_EINVAL;
    int32_t rc = check_batch(spaces, n_spaces);
    if (rc != ECK_OK) return rc;
    if (mode != ECK_MODE_EXHAUSTIVE && mode != ECK_MODE_SAMPLE && mode != ECK_MODE_MUTATE &&
        mode != ECK_MODE_CROSSOVER)
        return ECK_EINVAL;
    if (n > (1ull << 40) || first_index > UINT64_MAX - n) return ECK_EINVAL;
    if (ld / n_spaces < n) return ECK_ESHAPE;
    if ((ld & 1) || ((uintptr_t)genes_out & 3)) return ECK_EALIGN;
    if ((mode == ECK_MODE_MUTATE || mode == ECK_MODE_CROSSOVER) && (!parents || n_parents == 0)) return ECK_EINVAL;
    SpaceBatch batch;
    StreamBatch streams;
    for (uint32_t s = 0; s < n_spaces; ++s) {
        if (mode == ECK_MODE_EXHAUSTIVE) {
            if (spaces[s]->size == 0) return ECK_EUNSUPPORTED;
            if (first_index + n > spaces[s]->size) return ECK_EINVAL;
        }
        streams.state[s] = stream_state(seeds[s], round);
    }
    rc = upload_batch(spaces, n_spaces, &batch);
    if (rc != ECK_OK) return rc;

    const dim3 block(256), grid((unsigned)((n + 255) / 256), n_spaces);
    hipStream_t st = as_stream(stream);
    const uint64_t ld_parents = (uint64_t)n_parents * n_spaces;
    if (mode == ECK_MODE_EXHAUSTIVE)
        hipLaunchKernelGGL(enumerate_kernel<ECK_MODE_EXHAUSTIVE>, grid, block, 0, st, batch, streams, first_index, n,
                           parents, n_parents, ld_parents, p_mut_q32, genes_out, ld);
    else if (mode == ECK_MODE_SAMPLE)
        hipLaunchKernelGGL(enumerate_kernel<ECK_MODE_SAMPLE>, grid, block, 0, st, batch, streams, first_index, n,
                           parents, n_parents, ld_parents, p_mut_q32, genes_out, ld);
    else if (mode == ECK_MODE_MUTATE)
        hipLaunchKernelGGL(enumerate_kernel<ECK_MODE_MUTATE>, grid, block, 0, st, batch, streams, first_index, n,
                           parents, n_parents, ld_parents, p_mut_q32, genes_out, ld);
    else
        hipLaunchKernelGGL(enumerate_kernel<ECK_MODE_CROSSOVER>, grid, block, 0, st, batch, streams, first_index, n,
                           parents, n_parents, ld_parents, p_mut_q32, genes_out, ld);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

} // namespace

extern "C" int32_t candidate_enumerate(const eck_space *space, int32_t mode, uint64_t seed, uint32_t round,
                                       uint64_t first_index, uint64_t n, const uint16_t *parents,
                                       uint32_t n_parents, uint32_t p_mut_q32, uint16_t *genes_out, uint64_t ld,
                                       void *stream)
{
    if (!space) return ECK_EINVAL;
    return enumerate_launch(&space, 1, mode, &seed, round, first_index, n, parents, n_parents, p_mut_q32, genes_out,
                            ld, stream);
}

extern "C" int32_t candidate_enumerate_batch(const eck_space *const *spaces, uint32_t n_spaces, int32_t mode,
                                             const uint64_t *seeds, uint32_t round, uint64_t first_index,
                                             uint64_t n_per_space, const uint16_t *parents,
                                             uint32_t n_parents_per_space, uint32_t p_mut_q32, uint16_t *genes_out,
                                             uint64_t ld, void *stream)
{
    return enumerate_launch(spaces, n_spaces, mode, seeds, round, first_index, n_per_space, parents,
                            n_parents_per_space, p_mut_q32, genes_out, ld, stream);
}

namespace {
__global__ void gather_genes_kernel(const uint16_t *__restrict__ genes, uint64_t ld, uint64_t n, int n_genes,
                                    const uint32_t *__restrict__ idx, uint32_t k, uint16_t *__restrict__ out,
                                    uint64_t ld_out)
{
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= k) return;
    uint32_t src = idx[j];
    if (src == 0xFFFFFFFFu) src = idx[0];
    const bool valid = src != 0xFFFFFFFFu && src < n;
    for (int g = 0; g < n_genes; ++g) out[(uint64_t)g * ld_out + j] = valid ? genes[(uint64_t)g * ld + src] : (uint16_t)0;
}
} // namespace

extern "C" int32_t eck_candidates_gather(const uint16_t *genes, uint64_t ld, uint64_t n, int32_t n_genes,
                                         const uint32_t *idx, uint32_t k, uint16_t *out, uint64_t ld_out, void *stream)
{
    if (!genes || !idx || !out || k == 0 || n == 0 || n_genes < 1 || n_genes > ECK_MAX_GENES) return ECK_EINVAL;
    if (ld_out < k || ld < n) return ECK_ESHAPE;
    hipLaunchKernelGGL(gather_genes_kernel, dim3((k + 255) / 256), dim3(256), 0, as_stream(stream), genes, ld, n,
                       (int)n_genes, idx, k, out, ld_out);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

// ------------------------------------------------------------ de-duplication

namespace {
constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;

__device__ __forceinline__ uint64_t genes_hash(const uint16_t *__restrict__ genes, uint64_t ld, int n_genes, uint32_t i)
{
    uint64_t h = 0;
    for (int g = 0; g < n_genes; ++g) h = splitmix_finalise(h + kGamma + genes[(uint64_t)g * ld + i]);
    return h;
}

__device__ __forceinline__ bool same_genes(const uint16_t *__restrict__ genes, uint64_t ld, int n_genes, uint32_t a,
                                           uint32_t b)
{
    for (int g = 0; g < n_genes; ++g)
        if (genes[(uint64_t)g * ld + a] != genes[(uint64_t)g * ld + b]) return false;
    return true;
}

__global__ void dedup_clear_kernel(uint32_t *table, uint64_t slots)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < slots) table[i] = kEmptySlot;
}

// Open-addressing table of candidate indices, one slot per distinct gene tuple; a slot ends up holding the
// lowest index with its tuple (integer atomics only, so the outcome does not depend on execution order).
// The table has at least 2n slots, so a probe sequence always meets a free slot or its own tuple.
__global__ void dedup_insert_kernel(const uint16_t *__restrict__ genes, uint64_t ld, uint32_t n, int n_genes,
                                    uint32_t *table, uint32_t mask)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t slot = (uint32_t)genes_hash(genes, ld, n_genes, i) & mask;
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const uint32_t seen = atomicCAS(&table[slot], kEmptySlot, i);
        if (seen == kEmptySlot) return; // this candidate now stands for its tuple
        if (seen == i || same_genes(genes, ld, n_genes, seen, i)) {
            atomicMin(&table[slot], i);
            return;
        }
        slot = (slot + 1) & mask;
    }
}

__global__ void dedup_mark_kernel(const uint16_t *__restrict__ genes, uint64_t ld, uint32_t n, int n_genes,
                                  const uint32_t *__restrict__ table, uint32_t mask, uint8_t *__restrict__ flags,
                                  int overwrite)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t slot = (uint32_t)genes_hash(genes, ld, n_genes, i) & mask;
    bool first = false;
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const uint32_t seen = table[slot];
        if (seen == kEmptySlot) break; // cannot happen after the insert pass
        if (seen == i || same_genes(genes, ld, n_genes, seen, i)) {
            first = seen == i;
            break;
        }
        slot = (slot + 1) & mask;
    }
    flags[i] = overwrite ? (first ? 1 : 0) : (flags[i] && first ? 1 : 0);
}

uint64_t dedup_slots(uint64_t n)
{
    uint64_t slots = 2;
    while (slots < 2 * n) slots <<= 1;
    return slots;
}
} // namespace

extern "C" uint64_t eck_candidates_dedup_workspace_bytes(uint64_t n)
{
    if (n == 0 || n > (1ull << 30)) return 0;
    return dedup_slots(n) * sizeof(uint32_t);
}

extern "C" int32_t eck_candidates_dedup(const uint16_t *genes, uint64_t ld, uint64_t n, int32_t n_genes, uint8_t *flags,
                                        int32_t overwrite, void *ws, uint64_t ws_bytes, void *stream)
{
    if (!genes || !flags || n == 0 || n_genes < 1 || n_genes > ECK_MAX_GENES) return ECK_EINVAL;
    if (ld < n) return ECK_ESHAPE;
    if (n > (1ull << 30)) return ECK_EUNSUPPORTED;
    const uint64_t slots = dedup_slots(n);
    if (!ws || ws_bytes < slots * sizeof(uint32_t)) return ECK_EWORKSPACE;
    if ((uintptr_t)ws & 3) return ECK_EALIGN;
    uint32_t *table = static_cast<uint32_t *>(ws);
    hipStream_t st = as_stream(stream);
    const uint32_t mask = (uint32_t)(slots - 1);
    hipLaunchKernelGGL(dedup_clear_kernel, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, st, table, slots);
    hipLaunchKernelGGL(dedup_insert_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, genes, ld, (uint32_t)n,
                       (int)n_genes, table, mask);
    hipLaunchKernelGGL(dedup_mark_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, genes, ld, (uint32_t)n,
                       (int)n_genes, table, mask, flags, (int)overwrite);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

// ------------------------------------------------------------------ features

namespace {

// loop-nest levels of one candidate; every factor is below 2^16
struct Levels {
    uint32_t f[NAX][4];
    uint32_t log2_unroll, log2_vec;
    bool shape_ok;
};

__device__ __forceinline__ uint32_t ceil_div_u32(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

// the knob tables are powers of two, so they are kept as exponents
__device__ __forceinline__ void levels_from_knobs(const SpaceParams &p, const uint32_t *g, Levels *lv)
{
    const uint32_t tm = 16u << g[0], tn = 16u << g[1], tk = 8u << g[2], threads = 64u << g[3];
    const uint32_t along_n = threads < tn ? threads : tn;
    const uint32_t along_m = threads / along_n;
    lv->shape_ok = along_m <= tm;
    lv->f[0][0] = p.ext[0];
    lv->f[1][0] = ceil_div_u32(p.ext[1], tm);
    lv->f[1][1] = along_m;
    lv->f[1][2] = along_m <= tm ? tm / along_m : 1;
    lv->f[2][0] = ceil_div_u32(p.ext[2], tn);
    lv->f[2][1] = along_n;
    lv->f[2][3] = tn / along_n;
    lv->f[4][0] = ceil_div_u32(p.ext[4], tk);
    lv->f[4][3] = tk;
    lv->log2_unroll = g[4];
    lv->log2_vec = g[5];
}

// Device form of the fixed-point log2: x = e + m / 1024 with e = floor(log2 v) and m the ten bits below v's
// leading one.  A double holds an integer v in [1, 2^53] exactly, and its upper word then reads
// [0 | 1023 + e | the twenty bits below the leading one], so w = (upper word >> 10) = 1024 * (1023 + e) + m: no
// count of leading zeros, no shifts by a variable amount.  One funnel shift drops the low ten bits and sets the
// exponent field of 2^23 above what is left ((300 << 22) = 0x4B000000, w < 2^21), which read as a float is
// 2^23 + w exactly: no conversion either.  Then x = (2^23 + w) / 1024 - (8192 + 1023), one fused multiply-add,
// exact (x has at most 16 significant bits).  `bias` is -9215 held in a register by the caller (as a literal it
// costs a move per use).
__device__ __forceinline__ float log2_fixed(double v, float bias)
{
    uint32_t upper = (uint32_t)__double2hiint(v);
    asm("" : "+v"(upper)); // opaque, or the shift below is rewritten as a 64-bit one
    const float biased = __uint_as_float(__builtin_amdgcn_alignbit(300u, upper, 10u));
    return __builtin_fmaf(biased, 1.0f / 1024.0f, bias);
}

// floor(a / b) for a < 2^53, 0 < b < 2^53 through one IEEE double division: both conversions are exact
// and the correctly rounded quotient can exceed the true one only by rounding up across an integer, so
// one downward correction suffices.  (A 64-bit integer division costs several times more instructions.)
__device__ __forceinline__ uint64_t floor_div_f64(uint64_t a, uint64_t b)
{
    uint64_t q = (uint64_t)((double)a / (double)b);
    if (q * b > a) --q;
    return q;
}

// Threads, and candidates, per block of the feature kernel.  1024 measured 9 % faster than 256 on the
// benchmark workload (the tables are staged once per 1024 candidates and a block writes 2 KB of every row).
constexpr uint32_t kFeatBlock = 1024;

// WANT_X: the transformed features are wanted (feat_out is not NULL; without them OUT_DTYPE means nothing).
template <int OUT_DTYPE, bool TABLES_IN_LDS, int N_FEAT, bool WANT_RAW, bool XRED, bool WANT_X>
__global__ __launch_bounds__(kFeatBlock) void features_kernel(SpaceBatch spaces, const uint16_t *__restrict__ genes,
                                                       uint64_t ld, uint64_t n, void *__restrict__ feat_out,
                                                       uint64_t *__restrict__ raw_out,
                                                       uint8_t *__restrict__ legal_out, int n_genes)
{
    extern __shared__ uint2 lds_tables[];
    const unsigned char *blob = spaces.dev[blockIdx.y];
    const SpaceParams p = *reinterpret_cast<const SpaceParams *>(blob);
    const uint2 *tab = reinterpret_cast<const uint2 *>(blob + kDevHeader);
    const uint64_t in_space = (uint64_t)blockIdx.x * kFeatBlock + threadIdx.x;
    const uint64_t block_col = (uint64_t)blockIdx.y * n + (uint64_t)blockIdx.x * kFeatBlock; // wave-uniform
    const uint64_t i = block_col + threadIdx.x;                                       // column in the matrices

    // The gene loads are issued together, before the tables are staged, so that one round trip covers them
    // all (rows beyond the space's gene count and columns beyond n re-read a valid element).
    uint32_t g[8];
    {
        const uint64_t col = in_space < n ? i : block_col;
#pragma unroll
        // (the number of genes comes with the kernel arguments, the same for every space of a batch, so these
        // loads do not wait for the space's parameters)
        for (int j = 0; j < 8; ++j) g[j] = genes[(uint64_t)(j < n_genes ? j : 0) * ld + col];
    }
    if (TABLES_IN_LDS) {
        // two entries per 16-byte load (the device copy is padded to a multiple of 16 bytes), four per thread
        // and trip.  (The compiler lets each load wait for itself; forcing the four into flight together
        // measured 4 % slower.)
        const uint4 *src = reinterpret_cast<const uint4 *>(tab);
        uint4 *dst = reinterpret_cast<uint4 *>(lds_tables);
        const uint32_t quads = (p.table_total + 1) >> 1;
        for (uint32_t base = 0; base < quads; base += 4 * kFeatBlock) {
            uint4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t t = base + k * kFeatBlock + threadIdx.x;
                v[k] = src[t < quads ? t : quads - 1];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t t = base + k * kFeatBlock + threadIdx.x;
                if (t < quads) dst[t] = v[k];
            }
        }
        __syncthreads();
        tab = lds_tables;
    }
    if (in_space >= n) return;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t top = j < p.n_genes ? p.radix[j] - 1 : 0;
        g[j] = g[j] < top ? g[j] : top;
    }

    Levels lv;
#pragma unroll
    for (int a = 0; a < NAX; ++a)
#pragma unroll
        for (int l = 0; l < 4; ++l) lv.f[a][l] = 1;
    lv.shape_ok = true;
    if (p.kind == ECK_SPACE_KNOB) {
        levels_from_knobs(p, g, &lv);
    } else {
        // all table reads first (split genes beyond the space's count re-read entry 0), then the sorting
        // into axis slots, which is wave-uniform control flow over registers
        uint2 e[NAX];
#pragma unroll
        for (int s = 0; s < NAX; ++s) e[s] = tab[s < p.n_split ? p.table_off[s] + g[s] : 0];
#pragma unroll
        for (int s = 0; s < NAX; ++s) {
            if (s < p.n_split) {
                const int a = p.split_axis[s];
                // static indexing keeps lv in registers
#pragma unroll
                for (int aa = 0; aa < NAX; ++aa)
                    if (aa == a) {
                        lv.f[aa][0] = e[s].x & 0xFFFFu;
                        lv.f[aa][1] = e[s].x >> 16;
                        lv.f[aa][2] = e[s].y & 0xFFFFu;
                        lv.f[aa][3] = e[s].y >> 16;
                    }
            }
        }
        uint32_t gu = 0, gv = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j == p.n_split) gu = g[j];
            if (j == p.n_split + 1) gv = g[j];
        }
        lv.log2_unroll = gu;
        lv.log2_vec = gv;
    }

    // ---- transform and store.  Three flavours: per-space constants (transformed on the host), 32-bit values
    // and 64-bit values (all below 2^53 by the limits checked at space creation, so the conversion to double
    // and the + 1 are exact).
    // Row f of an output starts at a wave-uniform address (row base + first column of the block), so the
    // per-lane part of every store address is the same small offset.
    float bias = -9215.0f;
    asm("" : "+v"(bias)); // one register for the whole kernel
    // bfloat16 output: features come in order, an even one waits for its odd neighbour, one instruction converts
    // both (round to nearest even) and the two halves go to their rows
    float held = 0.0f;
    // Features are emitted below in increasing order, each exactly once, so the address of a row is the address of
    // the row before plus the row stride: two scalar additions per row.  (Computed as f * ld + column for every
    // store, the 64-bit products and sums were most of the kernel's 562 scalar instructions, and scalar and vector
    // instructions of one wavefront do not issue together.)  The empty asm keeps the compiler from folding the
    // chain of additions back into products.
    typedef __attribute__((address_space(1))) unsigned char global_byte;
    const uint64_t feat_stride = ld * (OUT_DTYPE == ECK_F32 ? 4 : 2);
    uint64_t feat_row = reinterpret_cast<uint64_t>(feat_out) + block_col * (OUT_DTYPE == ECK_F32 ? 4 : 2);
    uint64_t raw_row = reinterpret_cast<uint64_t>(raw_out) + block_col * 8;
    // Features 32-63 (level factors, tiles, footprints: a few instructions each) are emitted first, with a row
    // chain of their own, so that a block's stores begin early and drain under the arithmetic of features 0-31
    // instead of all coming in its last third.
    uint64_t feat_row_upper = feat_row + 32 * feat_stride;
    uint64_t raw_row_upper = raw_row + 32 * (ld * 8);
    const uint32_t lane_x = threadIdx.x * (OUT_DTYPE == ECK_F32 ? 4 : 2), lane_raw = threadIdx.x * 8;
    auto next_row = [&](uint64_t &row, uint64_t stride) {
        row += stride;
        asm volatile("" : "+s"(row));
    };
    // (a scalar base plus a 32-bit lane offset: the store's address costs no vector instruction; the stores are
    // marked non-temporal: the matrix is far larger than the caches and is read by a later kernel, and streaming
    // writes that need no place in the L2 take the kernel from 0.49 to 0.39 ms per 2^24 candidates)
    auto at = [&](uint64_t row, uint32_t lane_bytes) { return reinterpret_cast<global_byte *>(row) + lane_bytes; };
    auto store_x = [&](int f, float x) {
        if (!WANT_X) return;
        uint64_t &row = f < 32 ? feat_row : feat_row_upper;
        if (OUT_DTYPE == ECK_F32) {
            __builtin_nontemporal_store(x, reinterpret_cast<__attribute__((address_space(1))) float *>(at(row, lane_x)));
            next_row(row, feat_stride);
        } else if (!(f & 1)) {
            held = x;
        } else {
            typedef float float2_t __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
            const float2_t both = {held, x};
            const uint32_t packed = __builtin_bit_cast(uint32_t, __builtin_convertvector(both, bf16x2_t));
            __builtin_nontemporal_store((uint16_t)packed, reinterpret_cast<__attribute__((address_space(1))) uint16_t *>(at(row, lane_x)));
            next_row(row, feat_stride);
            __builtin_nontemporal_store((uint16_t)(packed >> 16), reinterpret_cast<__attribute__((address_space(1))) uint16_t *>(at(row, lane_x)));
            next_row(row, feat_stride);
        }
    };
    auto store_raw = [&](int f, uint64_t raw) {
        if (WANT_RAW) {
            uint64_t &row = f < 32 ? raw_row : raw_row_upper;
            __builtin_nontemporal_store(raw, reinterpret_cast<__attribute__((address_space(1))) uint64_t *>(at(row, lane_raw)));
            next_row(row, ld * 8);
        }
    };
    auto emit_const = [&](int f, int slot, uint64_t raw) {
        if (f >= N_FEAT) return;
        store_raw(f, raw);
        store_x(f, (float)p.const_q10[slot] * (1.0f / 1024.0f)); // exact: below 2^16
    };
    auto emit32 = [&](int f, uint32_t raw) {
        if (f >= N_FEAT) return;
        store_raw(f, raw);
        store_x(f, log2_fixed((double)(raw + 1), bias)); // raw <= 2^32 - 2 by the limits checked at space creation
    };
    auto emit64 = [&](int f, uint64_t raw) {
        if (f >= N_FEAT) return;
        store_raw(f, raw);
        store_x(f, log2_fixed(__builtin_fma((double)(uint32_t)(raw >> 32), 4294967296.0, (double)(uint32_t)raw + 1.0), bias));
    };

    // ---- derived quantities
    uint32_t tile[NAX], per_thread[NAX];
#pragma unroll
    for (int a = 0; a < NAX; ++a) {
        per_thread[a] = lv.f[a][2] * lv.f[a][3];
        tile[a] = lv.f[a][1] * per_thread[a];
    }
    const uint32_t grid = lv.f[0][0] * lv.f[1][0] * lv.f[2][0] * lv.f[3][0];
    const uint32_t threads = lv.f[0][1] * lv.f[1][1] * lv.f[2][1] * lv.f[3][1];
    const uint32_t outs_thread = per_thread[0] * per_thread[1] * per_thread[2] * per_thread[3];
    const uint32_t grid_threads = grid * threads; // <= padded outputs < 2^32
    const uint32_t stages = lv.f[RED_AXIS][0];
    const uint32_t rs = p.R * p.S;
    const uint32_t stage_red = tile[RED_AXIS] * rs;
    const uint32_t inner_trip = lv.f[RED_AXIS][3];
    const uint32_t lu = lv.log2_unroll, lvv = lv.log2_vec;
    const uint32_t unroll = 1u << lu, vec = 1u << lvv;
    const bool conv = p.op == ECK_OP_CONV2D;

    uint32_t fp_a, fp_b, thr_a, thr_b;
    uint64_t halo_q8;
    if (conv) {
        const uint32_t in_h = (tile[2] - 1) * p.stride + p.R, in_w = (tile[3] - 1) * p.stride + p.S;
        const uint32_t patch = in_h * in_w;
        fp_a = tile[0] * tile[4] * patch;
        fp_b = tile[1] * tile[4] * rs;
        thr_a = per_thread[0] * per_thread[2] * per_thread[3];
        thr_b = per_thread[1];
        halo_q8 = floor_div_f64((uint64_t)patch << 8, tile[2] * tile[3]); // numerator < 2^40
    } else {
        fp_a = tile[0] * tile[1] * tile[4];
        fp_b = tile[0] * tile[2] * tile[4];
        thr_a = per_thread[0] * per_thread[1];
        thr_b = per_thread[0] * per_thread[2];
        halo_q8 = 256;
    }
    const uint32_t fp = fp_a + fp_b;

    // ---- features 32-63 first (see the row chains above)
    if (N_FEAT > 32) {
#pragma unroll
        for (int a = 0; a < NAX; ++a)
#pragma unroll
            for (int l = 0; l < 4; ++l) emit32(32 + 4 * a + l, lv.f[a][l]);
#pragma unroll
        for (int a = 0; a < NAX; ++a) emit32(52 + a, tile[a]);
        emit32(57, fp_a);
        emit32(58, fp_b);
        emit64(59, halo_q8);
        emit_const(60, 2, p.elem_bytes);
        emit_const(61, 3, (uint64_t)p.op);
        emit_const(62, 4, p.true_out);
        emit_const(63, 5, p.true_red);
    }

    const uint64_t padded_out = (uint64_t)grid_threads * outs_thread;
    const uint64_t st_sectors = (padded_out * p.elem_bytes + 31) >> 5;

    // ---- what depends on where the reduction runs
    uint64_t block_threads, smem_bytes, ld_bytes, flop_exec, fma_thread, int_ops, ld_instr, shared_st_tx, shared_ld;
    uint64_t waves_block;
    uint32_t blocks_cu;
    if (XRED) {
        // the reduction axis's second level is spread over threads; nothing is staged, every thread loads its
        // own slice; the partial sums of an output meet in a halving tree in shared memory
        const uint32_t kt = lv.f[RED_AXIS][1], kser = per_thread[RED_AXIS];
        const uint32_t red_thread = stages * kser * rs;
        uint32_t elems_a, elems_b; // operand elements of one thread in one stage (each below 2^31)
        if (conv) {
            const uint32_t th = (per_thread[2] - 1) * p.stride + p.R, tw = (per_thread[3] - 1) * p.stride + p.S;
            elems_a = per_thread[0] * kser * th * tw;
            elems_b = per_thread[1] * kser * rs;
        } else {
            elems_a = thr_a * kser;
            elems_b = thr_b * kser;
        }
        const uint64_t elems = (uint64_t)elems_a + elems_b;
        const uint64_t loads_thread_stage = (elems + vec - 1) >> lvv;
        const uint64_t all_threads = (uint64_t)grid_threads * kt; // grid * block
        const uint32_t tree_steps = kt > 1 ? 32u - (uint32_t)__clz((int)(kt - 1)) : 0u;
        block_threads = (uint64_t)threads * kt;
        smem_bytes = kt > 1 ? block_threads * outs_thread * 4 : 0; // fp32 partial sums
        ld_bytes = all_threads * stages * elems * p.elem_bytes;
        flop_exec = 2 * all_threads * outs_thread * red_thread + padded_out * (kt - 1);
        fma_thread = (uint64_t)outs_thread * red_thread;
        int_ops = all_threads * ((uint64_t)stages * (4 * loads_thread_stage + 2) +
                                 2ull * ((red_thread + unroll - 1) >> lu) + 2ull * tree_steps);
        ld_instr = all_threads * stages * loads_thread_stage;
        shared_st_tx = kt > 1 ? (padded_out * (2ull * kt - 1) * 4 + 127) >> 7 : 0;
        shared_ld = padded_out * 2 * (kt - 1);
        waves_block = floor_div_f64(block_threads + p.hw_wave - 1, p.hw_wave); // block_threads < 2^48
        blocks_cu = block_threads > p.hw_max_threads_cu ? 0u : p.hw_max_threads_cu / (uint32_t)block_threads;
    } else {
        // the reduction is staged through shared memory, stage by stage, by the whole block
        const uint32_t red = stages * stage_red;
        // vector loads per thread per stage: ceil(fp / (threads * vec)) == ceil(ceil(fp / threads) / vec)
        const uint32_t loads_thread_stage = (ceil_div_u32(fp, threads) + vec - 1) >> lvv;
        block_threads = threads;
        smem_bytes = (uint64_t)fp * p.elem_bytes;
        ld_bytes = (uint64_t)grid * stages * fp * p.elem_bytes;
        flop_exec = 2 * padded_out * red;
        fma_thread = (uint64_t)outs_thread * red;
        int_ops = (uint64_t)grid_threads *
                  ((uint64_t)stages * (4ull * loads_thread_stage + 2) + 2ull * ((red + unroll - 1) >> lu));
        ld_instr = (uint64_t)grid_threads * stages * loads_thread_stage;
        shared_st_tx = (ld_bytes + 127) >> 7;
        shared_ld = (uint64_t)grid_threads * ((uint64_t)thr_a + thr_b) * red;
        waves_block = ceil_div_u32(threads, p.hw_wave);
        blocks_cu = p.hw_max_threads_cu / threads;
    }
    const uint64_t ld_sectors = (ld_bytes + 31) >> 5;

    if (smem_bytes > p.hw_lds_bytes) blocks_cu = 0;
    else if (smem_bytes > 0) blocks_cu = min(blocks_cu, p.hw_lds_bytes / (uint32_t)smem_bytes);
    blocks_cu = min(blocks_cu, p.hw_max_blocks_cu);
    const uint32_t slots = p.hw_num_cu * (blocks_cu ? blocks_cu : 1);
    const uint32_t waves = grid / slots;
    const uint32_t tail = grid - waves * slots;
    const uint32_t active = min(grid, p.hw_num_cu);

    // loop levels above one trip: every factor is at least 1, so min(f, 2) - 1 is the indicator (a min and an
    // add per level; comparisons cost a mask, a select and wait states each)
    uint32_t depth = (p.R > 1) + (p.S > 1);
#pragma unroll
    for (int a = 0; a < NAX; ++a)
#pragma unroll
        for (int l = 0; l < 4; ++l) depth += min(lv.f[a][l], 2u);
    depth -= NAX * 4;

    const uint32_t contiguous = p.vec_axis == 3 ? lv.f[3][3] : lv.f[2][3];
    // gcd with a power of two: the power of two dividing both
    const uint32_t low_bit = contiguous & (0u - contiguous);
    const uint32_t vec_contig = low_bit < vec ? low_bit : vec;

    const bool legal = block_threads >= 32 && block_threads <= 1024 && lv.shape_ok && smem_bytes <= p.hw_lds_bytes &&
                       vec * p.elem_bytes <= 16 && (contiguous & (vec - 1)) == 0;
    if (legal_out) legal_out[i] = legal ? 1 : 0;

    emit_const(0, 0, p.flop_useful);
    emit64(1, flop_exec);
    emit64(2, fma_thread);
    emit64(3, int_ops);
    emit32(4, outs_thread);
    emit64(5, (uint64_t)outs_thread + thr_a + thr_b);
    emit32(6, grid);
    if (XRED) emit64(7, block_threads);
    else emit32(7, threads);
    if (XRED) emit64(8, waves_block);
    else emit32(8, (uint32_t)waves_block);
    emit32(9, blocks_cu);
    emit32(10, active);
    emit32(11, p.hw_num_cu - active);
    emit32(12, waves + (tail != 0));
    emit32(13, tail);
    emit64(14, ld_instr);
    emit64(15, ld_sectors);
    emit64(16, st_sectors);
    emit64(17, (uint64_t)grid_threads * ((outs_thread + vec - 1) >> lvv));
    emit64(18, smem_bytes);
    emit64(19, shared_st_tx);
    emit64(20, shared_ld);
    emit64(21, floor_div_f64(flop_exec << 3, ld_sectors + st_sectors)); // numerator < 2^52
    emit_const(22, 1, p.compulsory_bytes);
    {
        // (ld_bytes * 256) / c with ld_bytes < 2^50 and c < 2^34, as two exact steps
        const uint64_t c = p.compulsory_in_bytes;
        const uint64_t q1 = floor_div_f64(ld_bytes, c);
        const uint64_t r1 = ld_bytes - q1 * c;
        emit64(23, (q1 << 8) + floor_div_f64(r1 << 8, c));
    }
    emit32(24, stages);
    emit32(25, stage_red);
    emit32(26, inner_trip);
    emit32(27, unroll);
    emit64(28, (uint64_t)(unroll < inner_trip ? unroll : inner_trip) * outs_thread);
    emit32(29, depth);
    emit32(30, vec);
    emit32(31, vec_contig);
}

} // namespace

namespace {
int32_t features_launch(const eck_space *const *spaces, uint32_t n_spaces, const uint16_t *genes, uint64_t ld,
                        uint64_t n, int32_t n_feat, int32_t out_dtype, void *feat_out, uint64_t *raw_out,
                        uint8_t *legal_out, void *stream)
{
    if (!genes || n == 0) return ECK_EINVAL;
    if (!feat_out && !raw_out && !legal_out) return ECK_EINVAL;
    int32_t rc = check_batch(spaces, n_spaces);
    if (rc != ECK_OK) return rc;
    if (out_dtype != ECK_F32 && out_dtype != ECK_BF16) return ECK_EINVAL;
    if (n_feat != 32 && n_feat != 64) return ECK_EUNSUPPORTED;
    if (n > (1ull << 40)) return ECK_EINVAL;
    if (ld / n_spaces < n) return ECK_ESHAPE;
    if (ld & 1) return ECK_EALIGN;
    SpaceBatch batch;
    rc = upload_batch(spaces, n_spaces, &batch);
    if (rc != ECK_OK) return rc;

    // the tables go to the LDS when those of every space in the batch fit
    uint32_t largest = 0;
    for (uint32_t s = 0; s < n_spaces; ++s) largest = std::max(largest, spaces[s]->prm.table_total);
    const bool xred = spaces[0]->prm.kind == ECK_SPACE_SPLIT_XRED;
    const bool in_lds = spaces[0]->prm.kind != ECK_SPACE_KNOB && largest <= 6144;
    const size_t lds = in_lds ? (size_t)((largest + 1) / 2) * 16 : 0; // staged two entries at a time
    const dim3 block(kFeatBlock), grid((unsigned)((n + kFeatBlock - 1) / kFeatBlock), n_spaces);
    hipStream_t st = as_stream(stream);
    const bool raw = raw_out != nullptr;
#define ECK_LAUNCH_FEATURES(DT, INLDS, NF, RAW, XR)                                                                 \
    do {                                                                                                           \
        if (feat_out)                                                                                              \
            hipLaunchKernelGGL((features_kernel<DT, INLDS, NF, RAW, XR, true>), grid, block, lds, st, batch, genes, ld, \
                               n, feat_out, raw_out, legal_out, spaces[0]->prm.n_genes);                           \
        else                                                                                                       \
            hipLaunchKernelGGL((features_kernel<ECK_F32, INLDS, NF, RAW, XR, false>), grid, block, lds, st, batch,   \
                               genes, ld, n, feat_out, raw_out, legal_out, spaces[0]->prm.n_genes);                \
    } while (0)
#define ECK_PICK_RAW(DT, INLDS, NF)                    \
    do {                                               \
        if (raw && xred) ECK_LAUNCH_FEATURES(DT, INLDS, NF, true, true);        \
        else if (raw) ECK_LAUNCH_FEATURES(DT, INLDS, NF, true, false);          \
        else if (xred) ECK_LAUNCH_FEATURES(DT, INLDS, NF, false, true);         \
        else ECK_LAUNCH_FEATURES(DT, INLDS, NF, false, false);                  \
    } while (0)
#define ECK_PICK_NF(DT, INLDS)                          \
    do {                                                \
        if (n_feat == 32) ECK_PICK_RAW(DT, INLDS, 32);  \
        else ECK_PICK_RAW(DT, INLDS, 64);               \
    } while (0)
    if (out_dtype == ECK_F32) {
        if (in_lds) ECK_PICK_NF(ECK_F32, true);
        else ECK_PICK_NF(ECK_F32, false);
    } else {
        if (in_lds) ECK_PICK_NF(ECK_BF16, true);
        else ECK_PICK_NF(ECK_BF16, false);
    }
#undef ECK_PICK_NF
#undef ECK_PICK_RAW
#undef ECK_LAUNCH_FEATURES
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}
} // namespace

extern "C" int32_t features_compute(const eck_space *space, const uint16_t *genes, uint64_t ld, uint64_t n,
                                    int32_t n_feat, int32_t out_dtype, void *feat_out, uint64_t *raw_out,
                                    uint8_t *legal_out, void *stream)
{
    if (!space) return ECK_EINVAL;
    return features_launch(&space, 1, genes, ld, n, n_feat, out_dtype, feat_out, raw_out, legal_out, stream);
}

extern "C" int32_t features_compute_batch(const eck_space *const *spaces, uint32_t n_spaces, const uint16_t *genes,
                                          uint64_t ld, uint64_t n_per_space, int32_t n_feat, int32_t out_dtype,
                                          void *feat_out, uint64_t *raw_out, uint8_t *legal_out, void *stream)
{
    return features_launch(spaces, n_spaces, genes, ld, n_per_space, n_feat, out_dtype, feat_out, raw_out, legal_out,
                           stream);
}
