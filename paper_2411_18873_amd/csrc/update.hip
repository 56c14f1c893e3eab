// Dynamic cost-model update: SNR of the current predictions, then minibatch
// Adam on the weighted squared error of Eq. (1)  (Alg. 1: ModelUpdate, SNR;
// Sec. 6.4).  HIP, gfx950.
//
// One optimisation step is a short chain of launches of one strided tile GEMM
// (forward, the three weight-gradient products with the bias gradient folded
// in as an extra all-ones row, the two back-propagated deltas), a one-block
// loss/delta kernel and an element-wise Adam kernel.  All reductions have a
// fixed order, so a run is reproducible bit for bit.
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

__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g)
{
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

// per-sample Eq. (1) loss, its mean, and dL/dpred = 2 (p - y) / (y * rows)   (one block)
__global__ __launch_bounds__(1024) void loss_kernel(const float *__restrict__ pred, const float *__restrict__ y,
                                                    int rows, float *__restrict__ dy, Scalars *sc, int is_last)
{
    __shared__ double scratch[1024];
    double sum = 0.0;
    for (int r = threadIdx.x; r < rows; r += 1024) {
        const float p = pred[r], t = y[r];
        const float d = p - t;
        sum += (double)d * d / t;
        dy[r] = 2.0f * d / (t * (float)rows);
    }
    sum = block_sum(sum, scratch);
    if (threadIdx.x == 0 && is_last && !sc->bad) sc->loss = (float)(sum / rows);
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

struct UpdWs {
    uint64_t scalars, y, pred, h1, h2, dy, d2, d1, grad, total;
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
    w.d2 = o;      o = align(o + (uint64_t)mb * m->widths[2] * 4);
    w.d1 = o;      o = align(o + (uint64_t)mb * m->widths[1] * 4);
    w.grad = o;    o = align(o + m->n_params * 4);
    w.total = o;
    return w;
}

void launch_gemm(const GemmArgs &g, hipStream_t st)
{
    hipLaunchKernelGGL(gemm_kernel, dim3((g.N + TN - 1) / TN, (g.M + TM - 1) / TM), dim3(256), 0, st, g);
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

    const uint64_t nb = n_pairs / (uint64_t)B;
    for (int s = 0; s < n_steps; ++s) {
        const uint64_t row0 = ((uint64_t)s % nb) * (uint64_t)B;
        const void *x = static_cast<const char *>(feat) + row0 * elem; // X(r, f) = feat[f*ld + row0 + r]
        GemmArgs g;
        // h1 = relu(X W1 + b1)
        g = GemmArgs{x, elem == 2, 1, (int64_t)ld, -1, theta + m->off_w[0], H1, 1, h1, H1, B, H1, F,
                     theta + m->off_b[0], 1, nullptr, bf, bf, bf};
        launch_gemm(g, st);
        // h2 = relu(h1 W2 + b2)
        g = GemmArgs{h1, 0, H1, 1, -1, theta + m->off_w[1], H2, 1, h2, H2, B, H2, H1,
                     theta + m->off_b[1], 1, nullptr, 0, bf, 0};
        launch_gemm(g, st);
        // pred = h2 w3 + b3
        g = GemmArgs{h2, 0, H2, 1, -1, theta + m->off_w[2], 1, 1, pred, 1, B, 1, H2,
                     theta + m->off_b[2], 0, nullptr, 0, bf, 0};
        launch_gemm(g, st);
        hipLaunchKernelGGL(loss_kernel, dim3(1), dim3(1024), 0, st, pred, y + row0, B, dy, sc, s == n_steps - 1);
        // [gW3 ; gb3] = [h2 ; 1]^T dy
        g = GemmArgs{h2, 0, 1, H2, H2, dy, 1, 1, grad + m->off_w[2], 1, H2 + 1, 1, B, nullptr, 0, nullptr, 0, 0, 0};
        launch_gemm(g, st);
        // d2 = (dy w3^T) where h2 > 0
        g = GemmArgs{dy, 0, 1, 1, -1, theta + m->off_w[2], 1, 1, d2, H2, B, H2, 1, nullptr, 0, h2, 0, bf, 0};
        launch_gemm(g, st);
        // [gW2 ; gb2] = [h1 ; 1]^T d2
        g = GemmArgs{h1, 0, 1, H1, H1, d2, H2, 1, grad + m->off_w[1], H2, H1 + 1, H2, B, nullptr, 0, nullptr, 0, 0, 0};
        launch_gemm(g, st);
        // d1 = (d2 W2^T) where h1 > 0
        g = GemmArgs{d2, 0, H2, 1, -1, theta + m->off_w[1], 1, H2, d1, H1, B, H1, H2, nullptr, 0, h1, 0, bf, 0};
        launch_gemm(g, st);
        // [gW1 ; gb1] = [X ; 1]^T d1
        g = GemmArgs{x, elem == 2, (int64_t)ld, 1, F, d1, H1, 1, grad + m->off_w[0], H1, F + 1, H1, B, nullptr, 0, nullptr,
                     bf, 0, 0};
        launch_gemm(g, st);
        hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, theta, grad, P, s, lr, beta1,
                           beta2, eps, sc);
    }
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(64), 0, st, theta, P, n_steps, sc, snr_out, loss_out);
    ECK_HIP_TRY(hipGetLastError());
    return model_repack(m, st);
}
