// Cost model: state handling, weight packing and the forward pass (HIP, gfx950).
//
// costmodel_score evaluates the energy / latency model over a generation of
// candidates (Alg. 1: LatencyEvaAndPick, EnergyModelEvaAndPick; Sec. 5.4).
#include <cstring>
#include <new>

#include "eck_internal.h"

using namespace eck;

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// -------------------------------------------------------------------- layout
//
// Matrix-core tiling (v_mfma_f32_32x32x16_bf16, D = A*B + C, one wavefront):
//   A (32 rows x 16 k):  lane (h = lane/32, r = lane%32) holds A[r][8h .. 8h+7]
//   B (16 k x 32 cols):  lane (h, c) holds B[8h .. 8h+7][c]
//   D (32 x 32):         lane (h, c) register q holds D[8*(q/4) + 4h + q%4][c]
// The network is evaluated transposed, rows = hidden units, columns =
// candidates, with the weights as A and the activations as B.  A lane then
// owns one candidate column throughout, and the 16 outputs it holds after a
// layer-1 tile are exactly two B fragments of layer 2 (k slots 8h..8h+7 of two
// consecutive k-steps) once layer 2's k index is permuted to match:
//   hidden unit of (k-step s, half h, slot t) = 32*(s/2) + 8*((8*(s%2) + t)/4) + 4h + t%4.
// So activations never leave registers between layers.
//
// Packed buffer of a BF16 model (byte offsets 16-aligned):
//   W1 fragments [H1/32][F/16][64 lanes][8 bf16]
//   W2 fragments [H2/32][H1/16][64 lanes][8 bf16]   (k permuted as above)
//   b1 [H1/32][2][16] fp32, b2 [H2/32][2][16], w3 [H2/32][2][16]  (D-register order), b3 (1 float, padded to 4)

__host__ __device__ inline uint32_t unit_of_dreg(uint32_t chunk, uint32_t h, uint32_t q)
{
    return 32 * chunk + 8 * (q >> 2) + 4 * h + (q & 3);
}

struct PackedLayout {
    uint64_t w1, w2, b1, b2, w3, b3, total; // byte offsets
};

PackedLayout packed_layout(int F, int H1, int H2)
{
    PackedLayout L;
    L.w1 = 0;
    L.w2 = L.w1 + (uint64_t)F * H1 * 2;
    L.b1 = L.w2 + (uint64_t)H1 * H2 * 2;
    L.b2 = L.b1 + (uint64_t)H1 * 4;
    L.w3 = L.b2 + (uint64_t)H2 * 4;
    L.b3 = L.w3 + (uint64_t)H2 * 4;
    L.total = L.b3 + 16;
    return L;
}

__device__ __forceinline__ float round_through_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xFFFF0000u);
}

__device__ __forceinline__ uint16_t bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// theta (fp32 master) -> packed buffer.  One thread per packed element.
__global__ void pack_kernel(const float *__restrict__ theta, int F, int H1, int H2, uint64_t off_w1, uint64_t off_b1,
                            uint64_t off_w2, uint64_t off_b2, uint64_t off_w3, uint64_t off_b3,
                            unsigned char *__restrict__ packed, PackedLayout L)
{
    const uint32_t n_w1 = F * H1, n_w2 = H1 * H2;
    const uint32_t total = n_w1 + n_w2 + H1 + 2 * H2 + 1;
    for (uint32_t e = blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gridDim.x * blockDim.x) {
        if (e < n_w1) {
            // [oc][ks][lane][t]
            const uint32_t t = e & 7, lane = (e >> 3) & 63, frag = e >> 9;
            const uint32_t ksteps = F / 16, ks = frag % ksteps, oc = frag / ksteps;
            const uint32_t h = lane >> 5, r = lane & 31;
            const uint32_t k = 16 * ks + 8 * h + t, unit = 32 * oc + r;
            reinterpret_cast<uint16_t *>(packed + L.w1)[e] = bf16_bits(theta[off_w1 + (uint64_t)k * H1 + unit]);
        } else if (e < n_w1 + n_w2) {
            const uint32_t x = e - n_w1;
            const uint32_t t = x & 7, lane = (x >> 3) & 63, frag = x >> 9;
            const uint32_t ksteps = H1 / 16, ks = frag % ksteps, oc = frag / ksteps;
            const uint32_t h = lane >> 5, r = lane & 31;
            const uint32_t k = unit_of_dreg(ks >> 1, h, 8 * (ks & 1) + t), unit = 32 * oc + r;
            reinterpret_cast<uint16_t *>(packed + L.w2)[x] = bf16_bits(theta[off_w2 + (uint64_t)k * H2 + unit]);
        } else {
            uint32_t x = e - n_w1 - n_w2;
            if (x < (uint32_t)H1) {
                const uint32_t q = x & 15, h = (x >> 4) & 1, chunk = x >> 5;
                reinterpret_cast<float *>(packed + L.b1)[x] = round_through_bf16(theta[off_b1 + unit_of_dreg(chunk, h, q)]);
            } else if ((x -= H1) < (uint32_t)H2) {
                const uint32_t q = x & 15, h = (x >> 4) & 1, chunk = x >> 5;
                reinterpret_cast<float *>(packed + L.b2)[x] = round_through_bf16(theta[off_b2 + unit_of_dreg(chunk, h, q)]);
            } else if ((x -= H2) < (uint32_t)H2) {
                const uint32_t q = x & 15, h = (x >> 4) & 1, chunk = x >> 5;
                reinterpret_cast<float *>(packed + L.w3)[x] = round_through_bf16(theta[off_w3 + unit_of_dreg(chunk, h, q)]);
            } else {
                reinterpret_cast<float *>(packed + L.b3)[0] = round_through_bf16(theta[off_b3]);
            }
        }
    }
}

__global__ void fill_zero_kernel(float *p, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = 0.0f;
}

} // namespace

int32_t eck::model_repack(eck_model *m, hipStream_t stream)
{
    if (m->dtype != ECK_BF16) return ECK_OK;
    const int F = m->widths[0], H1 = m->widths[1], H2 = m->widths[2];
    const PackedLayout L = packed_layout(F, H1, H2);
    const uint32_t total = F * H1 + H1 * H2 + H1 + 2 * H2 + 1;
    hipLaunchKernelGGL(pack_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, m->d_state, F, H1, H2,
                       m->off_w[0], m->off_b[0], m->off_w[1], m->off_b[1], m->off_w[2], m->off_b[2],
                       (unsigned char *)m->d_packed, L);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

static int32_t check_widths(int32_t n_layers, const int32_t *widths, int32_t dtype)
{
    if (!widths || n_layers < 1) return ECK_EINVAL;
    for (int l = 0; l <= n_layers && l < 8; ++l)
        if (widths[l] < 1) return ECK_EINVAL;
    if (dtype != ECK_F32 && dtype != ECK_BF16) return ECK_EINVAL;
    if (n_layers != 3) return ECK_EUNSUPPORTED;
    if (widths[3] != 1) return ECK_ESHAPE;
    if (widths[0] != 32 && widths[0] != 64) return ECK_EUNSUPPORTED;
    if (widths[1] > 512 || widths[2] > 512) return ECK_EUNSUPPORTED;
    if (dtype == ECK_BF16 && ((widths[1] % 32) || (widths[2] % 32))) return ECK_EUNSUPPORTED;
    return ECK_OK;
}

extern "C" int32_t eck_model_param_count(int32_t n_layers, const int32_t *widths, uint64_t *out)
{
    if (!widths || !out || n_layers < 1 || n_layers > 8) return ECK_EINVAL;
    uint64_t p = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (widths[l] < 1 || widths[l + 1] < 1) return ECK_EINVAL;
        p += (uint64_t)widths[l] * widths[l + 1] + widths[l + 1];
    }
    *out = p;
    return ECK_OK;
}

extern "C" int32_t eck_model_create(int32_t n_layers, const int32_t *widths, int32_t dtype, eck_model **out)
{
    if (!out) return ECK_EINVAL;
    *out = nullptr;
    const int32_t rc = check_widths(n_layers, widths, dtype);
    if (rc != ECK_OK) return rc;
    eck_model *m = new (std::nothrow) eck_model();
    if (!m) return ECK_EDEVICE;
    m->n_layers = n_layers;
    m->dtype = dtype;
    uint64_t off = 0;
    for (int l = 0; l <= n_layers; ++l) m->widths[l] = widths[l];
    for (int l = 0; l < n_layers; ++l) {
        m->off_w[l] = off;
        off += (uint64_t)widths[l] * widths[l + 1];
        m->off_b[l] = off;
        off += widths[l + 1];
    }
    m->n_params = off;
    if (hipGetDevice(&m->device) != hipSuccess ||
        hipMalloc((void **)&m->d_state, (3 * off + 1) * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        delete m;
        return ECK_EDEVICE;
    }
    if (dtype == ECK_BF16) {
        m->packed_bytes = packed_layout(widths[0], widths[1], widths[2]).total;
        if (hipMalloc(&m->d_packed, m->packed_bytes) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(m->d_state);
            delete m;
            return ECK_EDEVICE;
        }
    }
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, 0, m->d_state, 3 * off + 1);
    if (hipGetLastError() != hipSuccess || model_repack(m, 0) != ECK_OK) {
        eck_model_destroy(m);
        return ECK_EDEVICE;
    }
    *out = m;
    return ECK_OK;
}

extern "C" void eck_model_destroy(eck_model *m)
{
    if (!m) return;
    (void)hipDeviceSynchronize();
    if (m->d_state) (void)hipFree(m->d_state);
    if (m->d_packed) (void)hipFree(m->d_packed);
    delete m;
}

extern "C" int32_t eck_model_set_state(eck_model *m, const float *blob, uint64_t n_floats, void *stream)
{
    if (!m || !blob) return ECK_EINVAL;
    const uint64_t P = m->n_params;
    if (n_floats != P && n_floats != 3 * P + 1) return ECK_ESHAPE;
    hipStream_t st = as_stream(stream);
    ECK_HIP_TRY(hipMemcpyAsync(m->d_state, blob, n_floats * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (n_floats == P) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, st, m->d_state + P, 2 * P + 1);
        ECK_HIP_TRY(hipGetLastError());
    }
    return model_repack(m, st);
}

extern "C" int32_t eck_model_get_state(const eck_model *m, float *blob, uint64_t n_floats, void *stream)
{
    if (!m || !blob) return ECK_EINVAL;
    if (n_floats != 3 * m->n_params + 1) return ECK_ESHAPE;
    ECK_HIP_TRY(hipMemcpyAsync(blob, m->d_state, n_floats * sizeof(float), hipMemcpyDeviceToDevice, as_stream(stream)));
    return ECK_OK;
}

// ------------------------------------------------------------ fp32 forward

namespace {

constexpr int F32_TILE = 32; // candidates per block

// 256 threads = 32 candidates x 8 unit groups.  Activations of the three
// layers sit in LDS as [unit][candidate]; weights come straight from theta
// (each load is shared by the 32 candidate lanes).  Accumulation is a plain
// in-order fp32 FMA chain per output.
__global__ __launch_bounds__(256) void score_f32_kernel(const float *__restrict__ theta, int F, int H1, int H2,
                                                        uint64_t off_w1, uint64_t off_b1, uint64_t off_w2,
                                                        uint64_t off_b2, uint64_t off_w3, uint64_t off_b3,
                                                        const float *__restrict__ feat, uint64_t ld, uint64_t n,
                                                        float *__restrict__ out)
{
    extern __shared__ float act[];
    float *a0 = act, *a1 = a0 + F * F32_TILE, *a2 = a1 + H1 * F32_TILE;
    const int c = threadIdx.x & 31, ug = threadIdx.x >> 5;
    const uint64_t cand = (uint64_t)blockIdx.x * F32_TILE + c;
    for (int i = ug; i < F; i += 8) a0[i * F32_TILE + c] = cand < n ? feat[(uint64_t)i * ld + cand] : 0.0f;
    __syncthreads();
    for (int j = ug; j < H1; j += 8) {
        float acc = theta[off_b1 + j];
        const float *w = theta + off_w1 + j;
        for (int i = 0; i < F; ++i) acc = fmaf(a0[i * F32_TILE + c], w[(uint64_t)i * H1], acc);
        a1[j * F32_TILE + c] = fmaxf(acc, 0.0f);
    }
    __syncthreads();
    for (int j = ug; j < H2; j += 8) {
        float acc = theta[off_b2 + j];
        const float *w = theta + off_w2 + j;
        for (int i = 0; i < H1; ++i) acc = fmaf(a1[i * F32_TILE + c], w[(uint64_t)i * H2], acc);
        a2[j * F32_TILE + c] = fmaxf(acc, 0.0f);
    }
    __syncthreads();
    if (ug == 0 && cand < n) {
        float acc = theta[off_b3];
        for (int i = 0; i < H2; ++i) acc = fmaf(a2[i * F32_TILE + c], theta[off_w3 + i], acc);
        out[cand] = acc;
    }
}

// ------------------------------------------------------------ bf16 forward

// One block = 4 wavefronts; a wavefront carries NC tiles of 32 candidates
// through all three layers in registers.  W1 and the small vectors stay in LDS
// for the block's lifetime; W2 is streamed through LDS one 32-unit output
// chunk at a time and shared by the four wavefronts.
template <int F, int H1, int H2, int NC, bool FEAT_BF16>
__global__ __launch_bounds__(256) void score_bf16_kernel(const unsigned char *__restrict__ packed, PackedLayout L,
                                                         const void *__restrict__ feat, uint64_t ld, uint64_t n,
                                                         float *__restrict__ out, uint32_t n_tiles)
{
    constexpr int KS1 = F / 16, OC1 = H1 / 32, KS2 = H1 / 16, OC2 = H2 / 32;
    constexpr int TILE = 4 * NC * 32;
    constexpr uint32_t W1_BYTES = F * H1 * 2, CHUNK_BYTES = 64 * H1; // one W2 output chunk: KS2 fragments of 1 KB
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    bf16x8 *lds_w1 = reinterpret_cast<bf16x8 *>(lds);
    bf16x8 *lds_w2 = reinterpret_cast<bf16x8 *>(lds + W1_BYTES);
    float *lds_b1 = reinterpret_cast<float *>(lds + W1_BYTES + CHUNK_BYTES);
    float *lds_b2 = lds_b1 + H1;
    float *lds_w3 = lds_b2 + H2;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, col = lane & 31;

    // resident part: W1 fragments and the three vectors
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(packed + L.w1);
        uint4 *dst = reinterpret_cast<uint4 *>(lds);
        for (uint32_t i = tid; i < W1_BYTES / 16; i += 256) dst[i] = src[i];
        const float *vb = reinterpret_cast<const float *>(packed + L.b1);
        for (uint32_t i = tid; i < (uint32_t)(H1 + 2 * H2); i += 256) lds_b1[i] = vb[i]; // b1, b2, w3 are contiguous
    }
    const float b3 = *reinterpret_cast<const float *>(packed + L.b3);
    const uint4 *w2_src = reinterpret_cast<const uint4 *>(packed + L.w2);

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t base = (uint64_t)tile * TILE + (uint64_t)wave * (NC * 32);

        // ---- layer-1 B fragments: 8 consecutive features of one candidate per lane
        bf16x8 x[NC][KS1];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const uint64_t cand = base + 32 * c + col;
            const bool ok = cand < n;
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const uint64_t at = (uint64_t)(16 * ks + 8 * h + t) * ld + cand;
                    if (FEAT_BF16) {
                        const uint16_t bits = ok ? reinterpret_cast<const uint16_t *>(feat)[at] : (uint16_t)0;
                        x[c][ks][t] = __builtin_bit_cast(__bf16, bits);
                    } else {
                        x[c][ks][t] = (__bf16)(ok ? reinterpret_cast<const float *>(feat)[at] : 0.0f);
                    }
                }
        }
        __syncthreads(); // resident LDS data visible (first trip); harmless afterwards

        // ---- layer 1: h1 = relu(W1^T x + b1), kept as layer-2 B fragments
        bf16x8 h1[NC][KS2];
#pragma unroll
        for (int oc = 0; oc < OC1; ++oc) {
            f32x16 acc[NC];
            const f32x4 *bias = reinterpret_cast<const f32x4 *>(lds_b1 + (oc * 2 + h) * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const f32x4 b = bias[v];
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    acc[c][4 * v + 0] = b[0];
                    acc[c][4 * v + 1] = b[1];
                    acc[c][4 * v + 2] = b[2];
                    acc[c][4 * v + 3] = b[3];
                }
            }
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) {
                const bf16x8 a = lds_w1[(oc * KS1 + ks) * 64 + lane];
#pragma unroll
                for (int c = 0; c < NC; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, x[c][ks], acc[c], 0, 0, 0);
            }
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int t = 0; t < 8; ++t) h1[c][2 * oc + half][t] = (__bf16)fmaxf(acc[c][8 * half + t], 0.0f);
        }

        // ---- layer 2 + output layer, one 32-unit chunk of W2 at a time
        float y[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) y[c] = 0.0f;
        for (int oc = 0; oc < OC2; ++oc) {
            __syncthreads(); // everyone is done with the previous chunk
            {
                const uint4 *src = w2_src + (uint64_t)oc * (CHUNK_BYTES / 16);
                uint4 *dst = reinterpret_cast<uint4 *>(lds_w2);
#pragma unroll
                for (uint32_t i = 0; i < CHUNK_BYTES / 16 / 256; ++i) dst[tid + 256 * i] = src[tid + 256 * i];
            }
            __syncthreads();
            f32x16 acc[NC];
            const f32x4 *bias = reinterpret_cast<const f32x4 *>(lds_b2 + (oc * 2 + h) * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const f32x4 b = bias[v];
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    acc[c][4 * v + 0] = b[0];
                    acc[c][4 * v + 1] = b[1];
                    acc[c][4 * v + 2] = b[2];
                    acc[c][4 * v + 3] = b[3];
                }
            }
#pragma unroll
            for (int ks = 0; ks < KS2; ++ks) {
                const bf16x8 a = lds_w2[ks * 64 + lane];
#pragma unroll
                for (int c = 0; c < NC; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, h1[c][ks], acc[c], 0, 0, 0);
            }
            const f32x4 *wout = reinterpret_cast<const f32x4 *>(lds_w3 + (oc * 2 + h) * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const f32x4 w = wout[v];
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[c] = fmaf(fmaxf(acc[c][4 * v + e], 0.0f), w[e], y[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const float total = y[c] + __shfl_xor(y[c], 32);
            const uint64_t cand = base + 32 * c + col;
            if (h == 0 && cand < n) out[cand] = total + b3;
        }
    }
}

template <int F, int H1, int H2, int NC>
int32_t launch_bf16(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n, float *out,
                    hipStream_t st)
{
    const PackedLayout L = packed_layout(F, H1, H2);
    constexpr int TILE = 4 * NC * 32;
    const uint64_t tiles64 = (n + TILE - 1) / TILE;
    if (tiles64 > 0xFFFFFFFFull) return ECK_EUNSUPPORTED;
    const uint32_t n_tiles = (uint32_t)tiles64;
    int cus = 256;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device);
    const uint32_t grid = n_tiles < (uint32_t)cus ? n_tiles : (uint32_t)cus;
    const size_t lds = (size_t)F * H1 * 2 + 64 * H1 + (H1 + 2 * H2) * 4;
    auto kern_b = score_bf16_kernel<F, H1, H2, NC, true>;
    auto kern_f = score_bf16_kernel<F, H1, H2, NC, false>;
    auto kern = feat_dtype == ECK_BF16 ? kern_b : kern_f;
    ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, (const unsigned char *)m->d_packed, L, feat, ld, n, out,
                       n_tiles);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

} // namespace

extern "C" int32_t costmodel_score(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                                   float *score_out, void *ws, uint64_t ws_bytes, void *stream)
{
    (void)ws;
    (void)ws_bytes;
    if (!m || !feat || !score_out || n == 0) return ECK_EINVAL;
    if (feat_dtype != ECK_F32 && feat_dtype != ECK_BF16) return ECK_EINVAL;
    if (ld < n) return ECK_ESHAPE;
    if (n > (1ull << 40)) return ECK_EINVAL;
    hipStream_t st = as_stream(stream);
    const int F = m->widths[0], H1 = m->widths[1], H2 = m->widths[2];
    if (m->dtype == ECK_F32) {
        if (feat_dtype != ECK_F32) return ECK_EUNSUPPORTED;
        const size_t lds = (size_t)(F + H1 + H2) * F32_TILE * sizeof(float);
        ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(score_f32_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        const uint64_t blocks = (n + F32_TILE - 1) / F32_TILE;
        if (blocks > 0x7FFFFFFFull) return ECK_EUNSUPPORTED;
        hipLaunchKernelGGL(score_f32_kernel, dim3((unsigned)blocks), dim3(256), lds, st, m->d_state, F, H1, H2,
                           m->off_w[0], m->off_b[0], m->off_w[1], m->off_b[1], m->off_w[2], m->off_b[2], (const float *)feat,
                           ld, n, score_out);
        ECK_HIP_TRY(hipGetLastError());
        return ECK_OK;
    }
    if (feat_dtype == ECK_BF16 && (ld & 1)) return ECK_EALIGN;
    if (F == 64 && H1 == 512 && H2 == 512) return launch_bf16<64, 512, 512, 2>(m, feat, feat_dtype, ld, n, score_out, st);
    if (F == 64 && H1 == 256 && H2 == 256) return launch_bf16<64, 256, 256, 2>(m, feat, feat_dtype, ld, n, score_out, st);
    if (F == 64 && H1 == 128 && H2 == 128) return launch_bf16<64, 128, 128, 2>(m, feat, feat_dtype, ld, n, score_out, st);
    if (F == 32 && H1 == 64 && H2 == 64) return launch_bf16<32, 64, 64, 2>(m, feat, feat_dtype, ld, n, score_out, st);
    return ECK_EUNSUPPORTED;
}
