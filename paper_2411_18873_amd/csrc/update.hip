// Dynamic cost-model update: SNR of the current predictions, then minibatch
// Adam on the weighted squared error of Eq. (1)  (Alg. 1: ModelUpdate, SNR;
// Sec. 6.4).  HIP, gfx950.
//
// One optimisation step is a short chain of launches of one strided tile GEMM
// (forward, the three weight-gradient products with the bias gradient folded
// in as an extra all-ones row, the two back-propagated deltas), a one-block
// loss/delta kernel and an element-wise Adam kernel.  For BF16 models the five
// large products run on the matrix cores with bf16 operands (weights,
// activations and back-propagated deltas rounded as they are staged) and fp32
// accumulation; the width-1 products of the output layer stay in fp32.  All
// reductions have a fixed order, so a run is reproducible bit for bit.
#include <algorithm>
#include <cmath>

#include "eck_internal.h"

using namespace eck;

namespace {

__device__ __forceinline__ float through_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) == 0x7F800000u) return x;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xFFFF0000u);
}

struct GemmArgs {
    // C[m][n] = epilogue( sum_k A(m,k) * B(k,n) )
    const void *A;
    int a_is_bf16;      // A holds bf16 bits (feature matrix) instead of fp32
    int64_t sa_m, sa_k; // element strides
    int a_ones_row;     // A(m == a_ones_row, k) reads as 1 (bias-gradient row); -1 = none
    const float *B;
    int64_t sb_k, sb_n;
    float *C;
    int64_t ldc;
    int M, N, K;
    const float *bias; // added per column n, or NULL
    int relu;
    const float *mask; // same layout as C: result kept where mask > 0, else 0; or NULL
    int round_a, round_b, round_c; // pass operands / result through bf16
};

constexpr int TM = 64, TN = 64, TK = 16;

__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs first, GemmArgs second)
{
    const GemmArgs g = blockIdx.z ? second : first;
    if ((int)blockIdx.x * TN >= g.N || (int)blockIdx.y * TM >= g.M) return;
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[TK][TN + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4; // 16 x 16 threads, 4 x 4 outputs each
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.K; k0 += TK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q;
            {
                const int m = e & (TM - 1), k = e >> 6;
                const int gm = m0 + m, gk = k0 + k;
                float v = 0.0f;
                if (gm < g.M && gk < g.K) {
                    if (gm == g.a_ones_row) v = 1.0f;
                    else {
                        const int64_t at = (int64_t)gm * g.sa_m + (int64_t)gk * g.sa_k;
                        v = g.a_is_bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(g.A)[at] << 16)
                                        : reinterpret_cast<const float *>(g.A)[at];
                        if (g.round_a) v = through_bf16(v);
                    }
                }
                As[k][m] = v;
            }
            {
                const int n = e & (TN - 1), k = e >> 6;
                const int gn = n0 + n, gk = k0 + k;
                float v = 0.0f;
                if (gn < g.N && gk < g.K) {
                    v = g.B[(int64_t)gk * g.sb_k + (int64_t)gn * g.sb_n];
                    if (g.round_b) v = through_bf16(v);
                }
                Bs[k][n] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < TK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m >= g.M || n >= g.N) continue;
            float v = acc[i][j];
            if (g.bias) v += g.round_b ? through_bf16(g.bias[n]) : g.bias[n];
            if (g.relu) v = fmaxf(v, 0.0f);
            const int64_t at = (int64_t)m * g.ldc + n;
            if (g.mask && !(g.mask[at] > 0.0f)) v = 0.0f;
            if (g.round_c) v = through_bf16(v);
            g.C[at] = v;
        }
}

// The same product on the matrix cores for BF16 models: both operands are rounded to bf16 while they
// are staged into LDS, accumulation is fp32 (v_mfma_f32_32x32x16_bf16).  64 x 64 output tile per block,
// one 32 x 32 quadrant per wavefront, 64-deep stages; the next stage's operands are already in
// flight (in registers) while the current one is multiplied.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int MK = 64;      // stage depth
constexpr int MLD = MK + 8; // LDS row stride in bf16: 144 bytes keeps the 16-byte fragment reads conflict-free

__device__ __forceinline__ uint16_t to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// The reduction dimension is also split inside the block: KG groups of four wavefronts take every KG-th
// stage each (these products are latency-bound -- 64 blocks, 8 dependent stages), and their partial tiles
// are added through LDS in group order, so the result does not depend on scheduling.
constexpr int KG = 2;
constexpr size_t GEMM_MFMA_LDS = (size_t)KG * (TM + TN) * MLD * sizeof(uint16_t);
static_assert((KG - 1) * TM * TN * sizeof(float) <= GEMM_MFMA_LDS, "partial tiles reuse the operand buffers");

__global__ __launch_bounds__(256 * KG) void gemm_mfma_kernel(GemmArgs first, GemmArgs second)
{
    // blockIdx.z picks the problem; blocks outside that problem's tile grid leave before any barrier
    const GemmArgs g = blockIdx.z ? second : first;
    if ((int)blockIdx.x * TN >= g.N || (int)blockIdx.y * TM >= g.M) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_lds[];
    const int group = threadIdx.x >> 8, tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    uint16_t *As = reinterpret_cast<uint16_t *>(gemm_lds) + (size_t)group * (TM + TN) * MLD; // [m][k]
    uint16_t *Bs = As + TM * MLD;                                                            // [n][k]
    const int h = lane >> 5, c = lane & 31;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32; // quadrant of this wavefront
    const bool a_k_fast = g.sa_k == 1, b_k_fast = g.sb_k == 1;
    constexpr int PER = TM * MK / 256; // elements per thread per operand per stage

    // fetch() only loads: every address is clamped into the operand, nothing is decided on what arrives, so the
    // 2 * PER loads of a stage are in flight together (a value that is tested, or loaded under a condition, is
    // waited for on the spot).  stage() then zeroes what lies outside M, N, K, sets the row of ones, converts
    // and stores to the LDS.
    uint32_t ra[PER], rb[PER]; // raw bits as loaded
    int fetched_k0 = 0;
    const int last_a_row = g.a_ones_row == g.M - 1 ? g.M - 2 : g.M - 1; // last row of A that is in memory
    auto fetch = [&](int k0) {
        fetched_k0 = k0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = tid + 256 * q;
            {
                const int m = a_k_fast ? e / MK : e % TM, k = a_k_fast ? e % MK : e / TM;
                const int gm = max(min(m0 + m, last_a_row), 0), gk = min(k0 + k, g.K - 1);
                const int64_t at = (int64_t)gm * g.sa_m + (int64_t)gk * g.sa_k;
                ra[q] = g.a_is_bf16 ? (uint32_t)reinterpret_cast<const uint16_t *>(g.A)[at]
                                    : reinterpret_cast<const uint32_t *>(g.A)[at];
            }
            {
                const int n = b_k_fast ? e / MK : e % TN, k = b_k_fast ? e % MK : e / TN;
                const int gn = min(n0 + n, g.N - 1), gk = min(k0 + k, g.K - 1);
                rb[q] = reinterpret_cast<const uint32_t *>(g.B)[(int64_t)gk * g.sb_k + (int64_t)gn * g.sb_n];
            }
        }
    };
    auto stage = [&]() {
        const int k0 = fetched_k0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = tid + 256 * q;
            const int m = a_k_fast ? e / MK : e % TM, ka = a_k_fast ? e % MK : e / TM;
            const int gm = m0 + m;
            float va = __uint_as_float(g.a_is_bf16 ? ra[q] << 16 : ra[q]);
            if (gm == g.a_ones_row) va = 1.0f;
            if (gm >= g.M || k0 + ka >= g.K) va = 0.0f;
            As[m * MLD + ka] = to_bf16_bits(va);
            const int n = b_k_fast ? e / MK : e % TN, kb = b_k_fast ? e % MK : e / TN;
            float vb = __uint_as_float(rb[q]);
            if (n0 + n >= g.N || k0 + kb >= g.K) vb = 0.0f;
            Bs[n * MLD + kb] = to_bf16_bits(vb);
        }
    };

    f32x16 acc;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
    // every group runs the same number of rounds (stages past K read as zero), so the barriers match
    const int n_stages = (g.K + MK - 1) / MK, rounds = (n_stages + KG - 1) / KG;
    fetch(group * MK);
    for (int r = 0; r < rounds; ++r) {
        stage();
        __syncthreads();
        if (r + 1 < rounds) fetch(((r + 1) * KG + group) * MK);
#pragma unroll
        for (int ks = 0; ks < MK / 16; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&As[(wm + c) * MLD + 16 * ks + 8 * h]);
            const bf16x8 b = *reinterpret_cast<const bf16x8 *>(&Bs[(wn + c) * MLD + 16 * ks + 8 * h]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    // partial tiles of groups 1 .. KG-1 through LDS, added by group 0 in group order
    float *partial = reinterpret_cast<float *>(gemm_lds); // [KG-1][4 wavefronts][16][64 lanes]
    if (group > 0) {
#pragma unroll
        for (int q = 0; q < 16; ++q) partial[(((group - 1) * 4 + wave) * 16 + q) * 64 + lane] = acc[q];
    }
    __syncthreads();
    if (group > 0) return;
#pragma unroll
    for (int other = 0; other < KG - 1; ++other)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[q] += partial[((other * 4 + wave) * 16 + q) * 64 + lane];
    // accumulator register q of lane (h, c): row 8*(q/4) + 4h + q%4, column c of the quadrant
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int m = m0 + wm + 8 * (q >> 2) + 4 * h + (q & 3), n = n0 + wn + c;
        if (m >= g.M || n >= g.N) continue;
        float v = acc[q];
        if (g.bias) v += g.round_b ? through_bf16(g.bias[n]) : g.bias[n];
        if (g.relu) v = fmaxf(v, 0.0f);
        const int64_t at = (int64_t)m * g.ldc + n;
        if (g.mask && !(g.mask[at] > 0.0f)) v = 0.0f;
        if (g.round_c) v = through_bf16(v);
        g.C[at] = v;
    }
}

struct Scalars {
    float emax;
    uint32_t bad;
    float snr, loss;
};

// one block: validate the measured energies, normalise them by their maximum
__global__ __launch_bounds__(1024) void labels_kernel(const float *__restrict__ e, uint64_t n, float *__restrict__ y,
                                                      Scalars *sc)
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

// fixed-order block reduction in double
__device__ double block_sum(double v, double *scratch)
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

// SNR = sum y^2 / sum (pred - y)^2 over the whole buffer (one block)
__global__ __launch_bounds__(1024) void snr_kernel(const float *__restrict__ pred, const float *__restrict__ y,
                                                   uint64_t n, Scalars *sc)
{
    __shared__ double scratch[1024];
    double sig = 0.0, noise = 0.0;
    for (uint64_t i = threadIdx.x; i < n; i += 1024) {
        const double yi = y[i], d = (double)pred[i] - yi;
        sig += yi * yi;
        noise += d * d;
    }
    sig = block_sum(sig, scratch);
    noise = block_sum(noise, scratch);
    if (threadIdx.x == 0 && !sc->bad) sc->snr = (float)(sig / noise);
}

__global__ void adam_kernel(float *__restrict__ state, const float *__restrict__ grad, uint64_t P, int step_in_call,
                            float lr, float beta1, float beta2, float eps, const Scalars *sc)
{
    if (sc->bad) return;
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    const double t = (double)state[3 * P] + step_in_call + 1; // t itself is advanced once, after the last step
    const float c1 = (float)(1.0 - pow((double)beta1, t)), c2 = (float)(1.0 - pow((double)beta2, t));
    const float g = grad[i];
    const float m = beta1 * state[P + i] + (1.0f - beta1) * g;
    const float v = beta2 * state[2 * P + i] + (1.0f - beta2) * g * g;
    state[P + i] = m;
    state[2 * P + i] = v;
    state[i] -= lr * (m / c1) / (sqrtf(v / c2) + eps);
}

__global__ void finish_kernel(float *state, uint64_t P, int n_steps, const Scalars *sc, float *snr_out, float *loss_out)
{
    if (threadIdx.x || blockIdx.x) return;
    if (!sc->bad) state[3 * P] += (float)n_steps;
    *snr_out = sc->snr;
    *loss_out = sc->loss;
}

// Output layer, forward and backward, fused and row-local: one wavefront per minibatch row computes
//   pred = h2 . w3 + b3,  the row's Eq.-(1) loss term,  dy = 2 (pred - y) / (y * rows),
//   d2[row][j] = dy * w3[j] where h2[row][j] > 0.
// The dot product is a fixed-order tree (per-lane strided partial sums, then a butterfly).
__global__ __launch_bounds__(256) void output_layer_kernel(const float *__restrict__ h2, const float *__restrict__ theta_w3,
                                                           const float *__restrict__ theta_b3, int H2, int rows,
                                                           const float *__restrict__ y, int round_w,
                                                           float *__restrict__ pred, float *__restrict__ dy,
                                                           float *__restrict__ loss_terms, float *__restrict__ d2)
{
    const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const float *row = h2 + (int64_t)r * H2;
    float part = 0.0f;
    for (int j = lane; j < H2; j += 64) {
        const float w = round_w ? through_bf16(theta_w3[j]) : theta_w3[j];
        part = fmaf(row[j], w, part);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    const float b3 = round_w ? through_bf16(theta_b3[0]) : theta_b3[0];
    const float p = part + b3, t = y[r], d = p - t;
    const float g = 2.0f * d / (t * (float)rows);
    if (lane == 0) {
        pred[r] = p;
        dy[r] = g;
        loss_terms[r] = d * d / t;
    }
    for (int j = lane; j < H2; j += 64) {
        const float w = round_w ? through_bf16(theta_w3[j]) : theta_w3[j];
        d2[(int64_t)r * H2 + j] = row[j] > 0.0f ? g * w : 0.0f;
    }
}

// [gW3 ; gb3] = [h2 ; 1]^T dy.  A block owns 64 columns; its 16 wavefronts each sum a contiguous
// range of rows (rows in order, loads batched eight at a time) and the 16 partial sums are added in
// wavefront order, so the result does not depend on scheduling.  Block 0 also reduces the loss terms
// (fixed order, double) when this is the step whose loss is reported.
__global__ __launch_bounds__(1024) void output_grad_kernel(const float *__restrict__ h2, const float *__restrict__ dy,
                                                           int H2, int rows, float *__restrict__ grad_w3b3,
                                                           const float *__restrict__ loss_terms, Scalars *sc, int is_last)
{
    __shared__ float partial[16][64];
    const int cg = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + cg;
    const int per = (rows + 15) / 16, r0 = rg * per, r1 = min(rows, r0 + per);
    float acc = 0.0f;
    if (j < H2) {
        int r = r0;
        for (; r + 8 <= r1; r += 8) {
            float v[8], d[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v[u] = h2[(int64_t)(r + u) * H2 + j];
                d[u] = dy[r + u];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = fmaf(v[u], d[u], acc);
        }
        for (; r < r1; ++r) acc = fmaf(h2[(int64_t)r * H2 + j], dy[r], acc);
    } else if (j == H2) {
        for (int r = r0; r < r1; ++r) acc += dy[r];
    }
    partial[rg][cg] = acc;
    __syncthreads();
    if (rg == 0 && j <= H2) {
        float total = partial[0][cg];
#pragma unroll
        for (int g = 1; g < 16; ++g) total += partial[g][cg];
        grad_w3b3[j] = total;
    }
    if (blockIdx.x == 0 && is_last) {
        __shared__ double scratch[1024];
        double sum = 0.0;
        for (int r = threadIdx.x; r < rows; r += 1024) sum += (double)loss_terms[r];
        sum = block_sum(sum, scratch);
        if (threadIdx.x == 0 && !sc->bad) sc->loss = (float)(sum / rows);
    }
}

struct UpdWs {
    uint64_t scalars, y, pred, h1, h2, dy, lterm, d2, d1, grad, refit, total;
};

UpdWs upd_layout(const eck_model *m, uint64_t n_pairs, int mb)
{
    auto align = [](uint64_t v) { return (v + 255) & ~255ull; };
    UpdWs w;
    uint64_t o = 0;
    w.scalars = o; o = align(o + sizeof(Scalars));
    w.y = o;       o = align(o + n_pairs * 4);
    w.pred = o;    o = align(o + n_pairs * 4);
    w.h1 = o;      o = align(o + (uint64_t)mb * m->widths[1] * 4);
    w.h2 = o;      o = align(o + (uint64_t)mb * m->widths[2] * 4);
    w.dy = o;      o = align(o + (uint64_t)mb * 4);
    w.lterm = o;   o = align(o + (uint64_t)mb * 4);
    w.d2 = o;      o = align(o + (uint64_t)mb * m->widths[2] * 4);
    w.d1 = o;      o = align(o + (uint64_t)mb * m->widths[1] * 4);
    w.grad = o;    o = align(o + m->n_params * 4);
    w.refit = o;   // the two-launch step of BF16 models keeps its own buffers behind the others
    if (m->dtype == ECK_BF16 && mb % 64 == 0) o += refit_workspace_bytes(m, mb);
    w.total = o;
    return w;
}

// One launch for one product, or for two products that do not depend on each other (grid.z = 2).
void launch_gemm(const GemmArgs &g, hipStream_t st, bool matrix_cores = false, const GemmArgs *also = nullptr)
{
    const GemmArgs &h = also ? *also : g;
    const dim3 grid((std::max(g.N, h.N) + TN - 1) / TN, (std::max(g.M, h.M) + TM - 1) / TM, also ? 2 : 1);
    if (matrix_cores) {
        // set per call: the attribute belongs to the current device
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_mfma_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMM_MFMA_LDS);
        hipLaunchKernelGGL(gemm_mfma_kernel, grid, dim3(256 * KG), GEMM_MFMA_LDS, st, g, h);
    }
    else hipLaunchKernelGGL(gemm_kernel, grid, dim3(256), 0, st, g, h);
}

} // namespace

extern "C" uint64_t costmodel_update_workspace_bytes(const eck_model *m, uint64_t n_pairs, int32_t minibatch)
{
    if (!m || n_pairs == 0 || minibatch <= 0) return 0;
    return upd_layout(m, n_pairs, minibatch).total;
}

extern "C" int32_t costmodel_update(eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld,
                                    const float *energy_measured, uint64_t n_pairs, int32_t n_steps, int32_t minibatch,
                                    float lr, float beta1, float beta2, float eps, float *snr_out, float *loss_out,
                                    void *ws, uint64_t ws_bytes, void *stream)
{
    if (!m || !feat || !energy_measured || !snr_out || !loss_out) return ECK_EINVAL;
    if (n_pairs == 0 || minibatch <= 0 || n_steps < 0 || n_pairs > (1u << 30)) return ECK_EINVAL;
    if (feat_dtype != ECK_F32 && feat_dtype != ECK_BF16) return ECK_EINVAL;
    if (!(lr > 0.0f) || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps >= 0.0f))
        return ECK_EINVAL;
    if (n_pairs % (uint64_t)minibatch || ld < n_pairs) return ECK_ESHAPE;
    if (m->dtype == ECK_F32 && feat_dtype != ECK_F32) return ECK_EUNSUPPORTED;
    const UpdWs w = upd_layout(m, n_pairs, minibatch);
    if (!ws || ws_bytes < w.total) return ECK_EWORKSPACE;
    if ((uintptr_t)ws & 255) return ECK_EALIGN;

    hipStream_t st = as_stream(stream);
    char *base = static_cast<char *>(ws);
    Scalars *sc = reinterpret_cast<Scalars *>(base + w.scalars);
    float *y = reinterpret_cast<float *>(base + w.y), *pred = reinterpret_cast<float *>(base + w.pred);
    float *h1 = reinterpret_cast<float *>(base + w.h1), *h2 = reinterpret_cast<float *>(base + w.h2);
    float *dy = reinterpret_cast<float *>(base + w.dy), *d2 = reinterpret_cast<float *>(base + w.d2);
    float *lterm = reinterpret_cast<float *>(base + w.lterm);
    float *d1 = reinterpret_cast<float *>(base + w.d1), *grad = reinterpret_cast<float *>(base + w.grad);
    const int F = m->widths[0], H1 = m->widths[1], H2 = m->widths[2], B = minibatch;
    const uint64_t P = m->n_params;
    const int bf = m->dtype == ECK_BF16;
    float *theta = m->d_state;
    const int elem = feat_dtype == ECK_BF16 ? 2 : 4;

    hipLaunchKernelGGL(labels_kernel, dim3(1), dim3(1024), 0, st, energy_measured, n_pairs, y, sc);
    // predictions of the model as it stands: the same forward pass that scores candidates
    int32_t rc = costmodel_score(m, feat, feat_dtype, ld, n_pairs, pred, nullptr, 0, stream);
    if (rc != ECK_OK) return rc;
    hipLaunchKernelGGL(snr_kernel, dim3(1), dim3(1024), 0, st, pred, y, n_pairs, sc);

    if (refit_applies(m, feat, feat_dtype, ld, minibatch)) {
        // BF16 model: two launches per step
        rc = refit_steps(m, feat, feat_dtype, ld, y, n_pairs, n_steps, minibatch, lr, beta1, beta2, eps, &sc->bad, &sc->loss,
                         base + w.refit, st);
        if (rc != ECK_OK) return rc;
        hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(64), 0, st, theta, P, n_steps, sc, snr_out, loss_out);
        ECK_HIP_TRY(hipGetLastError());
        return model_repack(m, st);
    }
    const uint64_t nb = n_pairs / (uint64_t)B;
    for (int s = 0; s < n_steps; ++s) {
        const uint64_t row0 = ((uint64_t)s % nb) * (uint64_t)B;
        const void *x = static_cast<const char *>(feat) + row0 * elem; // X(r, f) = feat[f*ld + row0 + r]
        GemmArgs g;
        // h1 = relu(X W1 + b1)
        g = GemmArgs{x, elem == 2, 1, (int64_t)ld, -1, theta + m->off_w[0], H1, 1, h1, H1, B, H1, F,
                     theta + m->off_b[0], 1, nullptr, bf, bf, bf};
        launch_gemm(g, st, bf);
        // h2 = relu(h1 W2 + b2)
        g = GemmArgs{h1, 0, H1, 1, -1, theta + m->off_w[1], H2, 1, h2, H2, B, H2, H1,
                     theta + m->off_b[1], 1, nullptr, 0, bf, 0};
        launch_gemm(g, st, bf);
        // output layer forward + loss + backward into d2, then its weight gradient
        hipLaunchKernelGGL(output_layer_kernel, dim3((B + 3) / 4), dim3(256), 0, st, h2, theta + m->off_w[2],
                           theta + m->off_b[2], H2, B, y + row0, bf, pred, dy, lterm, d2);
        hipLaunchKernelGGL(output_grad_kernel, dim3((H2 + 1 + 63) / 64), dim3(1024), 0, st, h2, dy, H2, B,
                           grad + m->off_w[2], lterm, sc, s == n_steps - 1);
        // [gW2 ; gb2] = [h1 ; 1]^T d2
        g = GemmArgs{h1, 0, 1, H1, H1, d2, H2, 1, grad + m->off_w[1], H2, H1 + 1, H2, B, nullptr, 0, nullptr, 0, 0, 0};
        // d1 = (d2 W2^T) where h1 > 0: needs d2 only, like the product above, so both go in one launch
        const GemmArgs back{d2, 0, H2, 1, -1, theta + m->off_w[1], 1, H2, d1, H1, B, H1, H2, nullptr, 0, h1, 0, bf, 0};
        launch_gemm(g, st, bf, &back);
        // [gW1 ; gb1] = [X ; 1]^T d1
        g = GemmArgs{x, elem == 2, (int64_t)ld, 1, F, d1, H1, 1, grad + m->off_w[0], H1, F + 1, H1, B, nullptr, 0, nullptr,
                     bf, 0, 0};
        launch_gemm(g, st, bf);
        hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, theta, grad, P, s, lr, beta1,
                           beta2, eps, sc);
    }
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(64), 0, st, theta, P, n_steps, sc, snr_out, loss_out);
    ECK_HIP_TRY(hipGetLastError());
    return model_repack(m, st);
}

extern "C" int32_t eck_k_count(double k, int64_t M, int64_t *count_out)
{
    if (!count_out || M < 0 || !(k >= 0.0 && k <= 1.0)) return ECK_EINVAL;
    *count_out = (int64_t)__builtin_floor(k * (double)M + 0.5);
    return ECK_OK;
}

extern "C" int32_t eck_k_step(double k, double snr, double mu, int64_t M, double *k_out)
{
    if (!k_out || M < 0 || !(k >= 0.0 && k <= 1.0) || mu != mu) return ECK_EINVAL;
    const int64_t measured = (int64_t)__builtin_floor(k * (double)M + 0.5);
    if (measured == 0) {
        *k_out = k;
        return ECK_OK;
    }
    // a NaN ratio (rejected energies) counts as a poor model: measure more
    const bool poor = !(snr >= mu);
    const double next = poor ? k + 0.2 : k - 0.2;
    *k_out = next > 1.0 ? 1.0 : (next < 0.0 ? 0.0 : next);
    return ECK_OK;
}
