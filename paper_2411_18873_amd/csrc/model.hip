// Cost model: state handling, weight packing and the forward pass (HIP, gfx950).
//
// costmodel_score evaluates the energy / latency model over a generation of
// candidates (Alg. 1: LatencyEvaAndPick, EnergyModelEvaAndPick; Sec. 5.4).
#include <cstring>
#include <new>
#include <type_traits>

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
//   W1 fragments   [H1/32][F/16][64 lanes][8 bf16]
//   b1             [H1/32][2][16] fp32 in D-register order: a chunk's first matrix instruction takes its 16
//                  values as the C operand, so the bias costs neither a vector instruction nor a k-step
//   W2 fragments   [H2/32][H1/16][64 lanes][8 bf16]   (k permuted as above)
//   b2 [H2/32][2][16] fp32, w3 [H2/32][2][16] fp32   (D-register order), b3 (1 float, padded to 4)

__host__ __device__ inline uint32_t unit_of_dreg(uint32_t chunk, uint32_t h, uint32_t q)
{
    return 32 * chunk + 8 * (q >> 2) + 4 * h + (q & 3);
}

struct PackedLayout {
    uint64_t w1, w1b, w2, b2, w3, b3, total; // byte offsets
};

PackedLayout packed_layout(int F, int H1, int H2)
{
    PackedLayout L;
    L.w1 = 0;
    L.w1b = L.w1 + (uint64_t)F * H1 * 2;
    L.w2 = L.w1b + (uint64_t)H1 * 4;
    L.b2 = L.w2 + (uint64_t)H1 * H2 * 2;
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
    const uint32_t n_w1 = F * H1, n_w1b = H1, n_w2 = H1 * H2;
    const uint32_t total = n_w1 + n_w1b + n_w2 + 2 * H2 + 1;
    for (uint32_t e = blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gridDim.x * blockDim.x) {
        if (e < n_w1) {
            // [oc][ks][lane][t]
            const uint32_t t = e & 7, lane = (e >> 3) & 63, frag = e >> 9;
            const uint32_t ksteps = F / 16, ks = frag % ksteps, oc = frag / ksteps;
            const uint32_t h = lane >> 5, r = lane & 31;
            const uint32_t k = 16 * ks + 8 * h + t, unit = 32 * oc + r;
            reinterpret_cast<uint16_t *>(packed + L.w1)[e] = bf16_bits(theta[off_w1 + (uint64_t)k * H1 + unit]);
        } else if (e < n_w1 + n_w1b) {
            const uint32_t x = e - n_w1;
            const uint32_t q = x & 15, h = (x >> 4) & 1, chunk = x >> 5;
            reinterpret_cast<float *>(packed + L.w1b)[x] = round_through_bf16(theta[off_b1 + unit_of_dreg(chunk, h, q)]);
        } else if (e < n_w1 + n_w1b + n_w2) {
            const uint32_t x = e - n_w1 - n_w1b;
            const uint32_t t = x & 7, lane = (x >> 3) & 63, frag = x >> 9;
            const uint32_t ksteps = H1 / 16, ks = frag % ksteps, oc = frag / ksteps;
            const uint32_t h = lane >> 5, r = lane & 31;
            const uint32_t k = unit_of_dreg(ks >> 1, h, 8 * (ks & 1) + t), unit = 32 * oc + r;
            reinterpret_cast<uint16_t *>(packed + L.w2)[x] = bf16_bits(theta[off_w2 + (uint64_t)k * H2 + unit]);
        } else {
            uint32_t x = e - n_w1 - n_w1b - n_w2;
            if (x < (uint32_t)H2) {
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
    const uint32_t total = F * H1 + (H1 / 32) * 512 + H1 * H2 + 2 * H2 + 1;
    hipLaunchKernelGGL(pack_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, m->d_state, F, H1, H2,
                       m->off_w[0], m->off_b[0], m->off_w[1], m->off_b[1], m->off_w[2], m->off_b[2],
                       (unsigned char *)m->d_packed, L);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

// the shapes the matrix-core forward pass is instantiated for
static bool bf16_shape_supported(int F, int H1, int H2)
{
    return (F == 64 && H1 == 512 && H2 == 512) || (F == 64 && H1 == 256 && H2 == 256) ||
           (F == 64 && H1 == 128 && H2 == 128) || (F == 32 && H1 == 64 && H2 == 64);
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
    if (dtype == ECK_BF16 && !bf16_shape_supported(widths[0], widths[1], widths[2])) return ECK_EUNSUPPORTED;
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

// The same network with four consecutive units per thread and pass (hidden widths that are multiples of four): one
// activation read and one 16-byte weight load feed four multiply-adds, a quarter of the loads per multiply-add.  Every
// output is still the same in-order chain, so the scores are the bits the kernel above gives.
__global__ __launch_bounds__(256) void score_f32x4_kernel(const float *__restrict__ theta, int F, int H1, int H2,
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
    auto layer = [&](const float *in, float *res, int K, int H, uint64_t off_w, uint64_t off_b) {
        for (int j = 4 * ug; j < H; j += 32) {
            float4 acc = *reinterpret_cast<const float4 *>(theta + off_b + j);
            const float *w = theta + off_w + j;
#pragma unroll 8
            for (int i = 0; i < K; ++i) {
                const float a = in[i * F32_TILE + c];
                const float4 wv = *reinterpret_cast<const float4 *>(w + (uint64_t)i * H);
                acc.x = fmaf(a, wv.x, acc.x);
                acc.y = fmaf(a, wv.y, acc.y);
                acc.z = fmaf(a, wv.z, acc.z);
                acc.w = fmaf(a, wv.w, acc.w);
            }
            res[(j + 0) * F32_TILE + c] = fmaxf(acc.x, 0.0f);
            res[(j + 1) * F32_TILE + c] = fmaxf(acc.y, 0.0f);
            res[(j + 2) * F32_TILE + c] = fmaxf(acc.z, 0.0f);
            res[(j + 3) * F32_TILE + c] = fmaxf(acc.w, 0.0f);
        }
    };
    layer(a0, a1, F, H1, off_w1, off_b1);
    __syncthreads();
    layer(a1, a2, H1, H2, off_w2, off_b2);
    __syncthreads();
    if (ug == 0 && cand < n) {
        float acc = theta[off_b3];
#pragma unroll 8
        for (int i = 0; i < H2; ++i) acc = fmaf(a2[i * F32_TILE + c], theta[off_w3 + i], acc);
        out[cand] = acc;
    }
}

// ------------------------------------------------------------ bf16 forward

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// max(x, 0) as one integer instruction on the float's bits: every negative float (and -0) is a negative
// integer.  (fmaxf costs a second, canonicalising max.)
__device__ __forceinline__ float relu(float x)
{
    const int bits = __float_as_int(x);
    return __int_as_float(bits > 0 ? bits : 0);
}

// Move a fragment into accumulation registers.  The 256 activation registers of a wavefront do not fit
// the 256 architectural vector registers next to everything else; matrix instructions read their A/B
// operands from accumulation registers just as well, so the fragments are parked there once and used
// in place (a value defined by an "a"-constrained output stays in that register file).
__device__ __forceinline__ bf16x8 park_in_acc(bf16x8 v)
{
    const u32x4 in = __builtin_bit_cast(u32x4, v);
    u32x4 out;
    uint32_t o0, o1, o2, o3;
    asm("v_accvgpr_write_b32 %0, %1" : "=a"(o0) : "v"(in[0]));
    asm("v_accvgpr_write_b32 %0, %1" : "=a"(o1) : "v"(in[1]));
    asm("v_accvgpr_write_b32 %0, %1" : "=a"(o2) : "v"(in[2]));
    asm("v_accvgpr_write_b32 %0, %1" : "=a"(o3) : "v"(in[3]));
    out[0] = o0;
    out[1] = o1;
    out[2] = o2;
    out[3] = o3;
    return __builtin_bit_cast(bf16x8, out);
}

// One block = 4 wavefronts; a wavefront carries NC tiles of 32 candidates
// through all three layers in registers: lane (h, col) owns candidates
// base + NC*col + c, c < NC (consecutive in memory, so one 4- or 8-byte load per
// feature row serves all of a lane's columns).  W1 (with b1) and
// the b2 / w3 vectors stay in LDS for the block's lifetime.  W2 streams through
// a ring of four LDS slots in pieces of half an output chunk (32 units x H1/2
// inputs), shared by the four wavefronts and written into LDS directly by the
// load unit (no register staging), three pieces ahead of their use.
//
// Ring protocol, piece g (numbered along the block's whole run): at its top a
// wavefront waits until its own share of piece g+1 has landed, then the block
// barrier -- after which (i) all of piece g+1 is visible to everyone, so the
// weight fragments can be read ahead across the piece boundary without exposing
// LDS latency, and (ii) everyone has finished piece g-1, whose slot the fetch of
// piece g+3 may now overwrite.
//
// With one wavefront per SIMD nothing else hides latency, so the code is
// software-pipelined by hand: the ReLU / bf16 conversion of layer-1 chunk i-1
// and the bias / ReLU / w3 product of layer-2 chunk i-1 are issued in between the
// matrix instructions of chunk i, and the next tile's features are requested
// while the current tile is still in layer 2.
template <int NC, bool FEAT_BF16>
struct RawFeat {
    static constexpr int WORDS = FEAT_BF16 ? NC / 2 : NC;
    uint32_t w[WORDS];
};

template <int NC, bool FEAT_BF16>
__device__ __forceinline__ RawFeat<NC, FEAT_BF16> load_raw(const void *ptr)
{
    RawFeat<NC, FEAT_BF16> r;
    if (FEAT_BF16) {
        if (NC == 2) r.w[0] = *reinterpret_cast<const uint32_t *>(ptr);
        else {
            const uint2 v = *reinterpret_cast<const uint2 *>(ptr);
            r.w[0] = v.x;
            r.w[NC / 2 - 1] = v.y;
        }
    } else {
        if (NC == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(ptr);
            r.w[0] = v.x;
            r.w[1] = v.y;
        } else {
            const uint4 v = *reinterpret_cast<const uint4 *>(ptr);
            r.w[0] = v.x;
            r.w[1] = v.y;
            r.w[NC - 2] = v.z;
            r.w[NC - 1] = v.w;
        }
    }
    return r;
}

template <int NC, bool FEAT_BF16>
__device__ __forceinline__ __bf16 raw_element(const RawFeat<NC, FEAT_BF16> &r, int c)
{
    if (FEAT_BF16) return __builtin_bit_cast(__bf16, (uint16_t)(r.w[c >> 1] >> (16 * (c & 1))));
    return (__bf16)__uint_as_float(r.w[c]);
}

// Ties an accumulator tile to the architectural register file.  The matrix instruction accepts its
// accumulator in either file, ordinary vector instructions only read the architectural one: an
// accumulator the compiler puts in the accumulation file costs one extra copy per register before the
// ReLU / output-layer arithmetic can touch it.
__device__ __forceinline__ void keep_in_vgprs(f32x16 &tile) { asm volatile("" : "+v"(tile)); }

// N direct-to-LDS loads of 1 KB per wavefront each: in load i every lane moves 16 bytes from
// (wave-uniform base) + lane_offset + 1024 i, and the load unit writes them to LDS at lds_byte_address
// (wave-uniform, handed over in M0) + 1024 i + 16 * lane -- the instruction's immediate offset applies to
// the global and to the LDS address alike.  The scalar-base form keeps all addressing of the weight
// stream in one register per lane.  Written as assembly on purpose: issued through the compiler's own
// intrinsic, a load of this kind in flight makes the compiler drain *all* LDS reads at every dependency
// (it may no longer wait for just the oldest), which stalls the matrix pipeline at every weight fragment.
// Completion is tracked by hand instead: the s_waitcnt vmcnt(...) + barrier protocol of the caller.
template <int N>
__device__ __forceinline__ void lds_dma_kb(const unsigned char *uniform_base, uint32_t lane_offset,
                                           uint32_t lds_byte_address)
{
    static_assert(N >= 1 && N <= 4, "immediate offsets of a global load end at 4095");
    const uint64_t b = (uint64_t)uniform_base;
    const uint64_t base = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                          (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_byte_address);
    if (N == 1)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(m0), "v"(lane_offset), "s"(base)
                     : "memory", "m0");
    else if (N == 2)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:1024"
                     :
                     : "s"(m0), "v"(lane_offset), "s"(base)
                     : "memory", "m0");
    else if (N == 3)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:1024\n\tglobal_load_lds_dwordx4 %1, %2 offset:2048"
                     :
                     : "s"(m0), "v"(lane_offset), "s"(base)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:1024\n\tglobal_load_lds_dwordx4 %1, %2 offset:2048\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:3072"
                     :
                     : "s"(m0), "v"(lane_offset), "s"(base)
                     : "memory", "m0");
}

// wait until only the operations issued after the fetch in question may still be outstanding:
// one later piece fetch (N_DMA loads) and / or NX feature loads of the next tile
template <int N_DMA, int NX>
__device__ __forceinline__ void wait_vm(bool dma_after)
{
    if (dma_after) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_DMA + NX) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NX) : "memory");
}

// WITH_MIN: the kernel also reduces its scores to the least one per segment of seg_len candidates, over the legal
// candidates (a number, not NaN), as order keys -- what the selection's latency gate needs, without a pass of
// its own over the scores.  Every lane keeps a running minimum for the segment its wavefront is in; the lanes are
// combined and handed to memory with one integer atomic when the wavefront moves on to another segment or ends; a
// wavefront whose 32 NC candidates straddle two segments sends them one by one.  The legality flags of a tile travel with its features.
struct MinArgs {
    const uint8_t *legal; // or NULL: all legal
    uint64_t seg_len;
    uint32_t *min_key;    // [n / seg_len], preset to 0xFFFFFFFF
    uint32_t tiles_per_seg; // seg_len / (candidates per tile) when that is whole (set by the launcher), else 0
};

__device__ __forceinline__ uint32_t score_order_key(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int F, int H1, int H2, int NC, bool FEAT_BF16, bool WIDE_ROWS, bool WITH_MIN>
__global__ __launch_bounds__(256) void score_bf16_kernel(const unsigned char *__restrict__ packed, PackedLayout L,
                                                         const void *__restrict__ feat, uint64_t ld, uint64_t n,
                                                         float *__restrict__ out, uint32_t n_tiles, MinArgs mn)
{
    constexpr int KS1 = F / 16, OC1 = H1 / 32, KS2 = H1 / 16, OC2 = H2 / 32;
    constexpr int TILE = 4 * NC * 32;
    constexpr int NXLOADS = KS1 * 8;                 // feature loads per lane per tile
    constexpr int NX = NXLOADS + (WITH_MIN ? 1 : 0); // ... and the load of the legality flags that goes with them
    constexpr int KSP = KS2 / 2;                     // k-steps (= 1 KB fragments) per piece
    constexpr int PIECES = 2 * OC2;                  // pieces per tile
    constexpr int RING = KSP < 4 ? KSP : 4;          // weight fragments held in registers
    constexpr int PF = RING - 1;                     // LDS read-ahead in k-steps
    constexpr int N_DMA = KSP / 4 > 0 ? KSP / 4 : 1; // 1 KB fetches per wavefront per piece
    constexpr uint32_t W1_BYTES = F * H1 * 2, W1B_BYTES = H1 * 4, PIECE_BYTES = KSP * 1024;
    // The feature loads of the next tile.  Issued in one burst they fill the load path, and the wavefront -- and with
    // it the matrix pipe -- stands still until the first of them are through (2 300 cycles of a 47 000-cycle tile at
    // 512 units, 3 500 of 30 000 at 256 units with four candidate tiles per wavefront); one at a time, a few k-steps
    // apart, they cost next to nothing.  So they are spread over pieces 1 .. XSPAN, load i in piece
    // 1 + i * XSPAN / NXLOADS.  The waits on the load counter depend on how many loads the two pieces before
    // issued, so those pieces have their index known at compile time: the head of the tile and the first PEEL
    // iterations of the loop over output chunks, written out (two with two candidate tiles per wavefront; one with
    // four, where a second one makes the compiler spill: the 256 architectural registers hold 128 of accumulators
    // and 64 of loaded features there).
    constexpr int LOOP_ITERS = (OC2 - 2) / 2;
    constexpr int PEEL_WANT = NC == 2 ? 2 : 1;
    constexpr int PEEL = LOOP_ITERS < PEEL_WANT ? LOOP_ITERS : PEEL_WANT;
    constexpr int XSPAN_FREE = PEEL == LOOP_ITERS ? PIECES - 4 : 4 * PEEL - 1;
    constexpr int XSPAN = XSPAN_FREE < 1 ? 1 : (XSPAN_FREE > NXLOADS ? NXLOADS : XSPAN_FREE);
    static_assert(XSPAN + 2 < PIECES || (XSPAN == 1 && PIECES == 4), "the last two pieces of a tile issue no feature loads");
    // WITH_MIN: the piece that requests the legality flags of the tile.  Piece 2 where the loads are spread: requested
    // in piece 1, next to the set-up of the feature loads, the one load made the compiler permute 104 parked
    // registers in every tile (+ 27 registers, + 1 % cycles).
    constexpr int LEGAL_PIECE = XSPAN > 1 ? 2 : 1;
    static_assert(KS2 % 2 == 0 && KSP % RING == 0 && OC2 % 2 == 0 && PIECES % 4 == 0, "unsupported shape");
    static_assert(NC == 2 || NC == 4, "unsupported tile width");
    static_assert(N_DMA + NX < 63, "outstanding loads must fit the load counter");
    using Raw = RawFeat<NC, FEAT_BF16>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const bf16x8 *lds_w1 = reinterpret_cast<const bf16x8 *>(lds);
    const float *lds_b1 = reinterpret_cast<const float *>(lds + W1_BYTES); // [OC1][2][16], D-register order
    unsigned char *lds_ring = lds + W1_BYTES + W1B_BYTES; // four slots of PIECE_BYTES; piece p uses slot p & 3
    float *lds_b2 = reinterpret_cast<float *>(lds_ring + 4 * PIECE_BYTES);
    float *lds_w3 = lds_b2 + H2;
    uint32_t *lds_run = reinterpret_cast<uint32_t *>(lds_w3 + H2); // WITH_MIN: [256] least key of the lane's segment

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, col = lane & 31;
    const unsigned char *w2_src = packed + L.w2;
    const uint32_t ring_lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds_ring;

    // asynchronous fetch of piece p (0 <= p < PIECES, the same for every tile) into slot p & 3: every lane
    // moves 16 bytes per call, the load unit writes them to LDS at (wave-uniform base) + 16 * lane
    const uint32_t dma_lane_offset = (uint32_t)wave * (N_DMA * 1024u) + (uint32_t)lane * 16u;
    auto fetch_piece = [&](int p) {
        const unsigned char *src = w2_src + (uint64_t)p * PIECE_BYTES;                            // uniform
        const uint32_t dst = ring_lds_addr + (p & 3) * PIECE_BYTES + (uint32_t)wave * (N_DMA * 1024u); // per wave
        if (KSP >= 4) lds_dma_kb<N_DMA>(src, dma_lane_offset, dst);
        else if (wave < KSP) lds_dma_kb<1>(src, dma_lane_offset, dst); // fewer fragments than wavefronts
    };
    // the NC candidates of this lane in tile `tile` start at:
    auto first_candidate = [&](uint32_t tile) { return (uint64_t)tile * TILE + (uint64_t)wave * (NC * 32) + NC * col; };
    // request the features of one tile: rows 16*ks + 8*h + t, NC consecutive candidates each, as loads
    // i = 8*ks + t = 0 .. NXLOADS-1 in that order (x_begin fixes the tile, x_one requests the next load).  Lanes
    // past the end read the tile's first candidate group instead (their columns are computed but never stored).
    // Row addresses are wave-uniform (scalar base, one scalar add per row); the per-lane part -- half-wave
    // row block plus position inside the tile -- is one 32-bit offset that only changes in a ragged last
    // tile.  Matrices too large for that offset to fit (WIDE_ROWS) take per-lane 64-bit pointers.
    const unsigned char *x_row = nullptr;
    uint32_t x_lane_off = 0;
    auto x_begin = [&](uint32_t tile) {
        constexpr uint64_t ELEM = FEAT_BF16 ? 2 : 4;
        const uint64_t row_bytes = ld * ELEM;
        // cand and ld are multiples of NC, so a group that starts below n lies inside its row
        const uint32_t in_tile = first_candidate(tile) < n ? (uint32_t)((wave * (NC * 32) + NC * col) * ELEM) : 0u;
        x_row = reinterpret_cast<const unsigned char *>(feat) + (uint64_t)tile * (TILE * ELEM);
        if (WIDE_ROWS) x_row += (uint64_t)h * (8 * row_bytes) + in_tile;
        else x_lane_off = (uint32_t)h * (uint32_t)(8 * row_bytes) + in_tile;
    };
    auto x_one = [&](int i, Raw(&raw)[NXLOADS]) {
        const uint64_t row_bytes = ld * (FEAT_BF16 ? 2 : 4);
        raw[i] = load_raw<NC, FEAT_BF16>(WIDE_ROWS ? x_row : x_row + x_lane_off);
        x_row += (i % 8 == 7) ? 9 * row_bytes : row_bytes;
    };
    auto load_tile = [&](uint32_t tile, Raw(&raw)[NXLOADS]) {
        x_begin(tile);
#pragma unroll
        for (int i = 0; i < NXLOADS; ++i) x_one(i, raw);
    };

    // legality flags of this lane's NC candidates (one byte each): requested early in the tile whose epilogue reads
    // them, among the feature loads of the next tile (the waits on the load counter see one more load in that piece)
    uint32_t legal_bits = 0x01010101u;
    auto load_legal = [&](uint32_t tile) {
        const uint64_t cand = first_candidate(tile);
        // without flags the load still happens (the waits on the load counter count it): any readable address does.
        // The host checks that the flags are aligned to the NC-byte word, so a word whose first byte is a flag lies
        // in that flag's page even when its last bytes are past the array (those are ignored below).
        const unsigned char *p = mn.legal ? mn.legal + (cand < n ? cand : (uint64_t)tile * TILE)
                                          : reinterpret_cast<const unsigned char *>(feat);
        legal_bits = NC == 2 ? (uint32_t)*reinterpret_cast<const uint16_t *>(p) : *reinterpret_cast<const uint32_t *>(p);
    };
    Raw raw[NXLOADS];
    if (blockIdx.x < n_tiles) {
        fetch_piece(0);
        fetch_piece(1);
        fetch_piece(2);
        load_tile(blockIdx.x, raw);
    }
    // resident part: W1 fragments, b1 and the two vectors of the output side
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(packed + L.w1); // w1 and b1 are contiguous
        uint4 *dst = reinterpret_cast<uint4 *>(lds);
        for (uint32_t i = tid; i < (W1_BYTES + W1B_BYTES) / 16; i += 256) dst[i] = src[i];
        const float *vb = reinterpret_cast<const float *>(packed + L.b2);
        for (uint32_t i = tid; i < (uint32_t)(2 * H2); i += 256) lds_b2[i] = vb[i]; // b2 and w3 are contiguous
    }
    const float b3 = *reinterpret_cast<const float *>(packed + L.b3);
    __syncthreads();

    // WITH_MIN: the segment of this wavefront's candidates in the tile before and, per lane, the least key it has
    // seen there; the lanes are only combined when the segment changes and at the end
    uint64_t seg = 0, seg_begin = 0;
    uint32_t seg_tile0 = 0; // first tile of that segment, when segments are whole tiles
    if (WITH_MIN) lds_run[tid] = 0xFFFFFFFFu; // only this lane ever touches its word
    auto flush_running_min = [&]() {
        uint32_t best = lds_run[tid];
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) best = min(best, (uint32_t)__shfl_xor((int)best, off));
        if (lane == 0 && best != 0xFFFFFFFFu) // both halves of the wavefront hold the same scores
            (void)__hip_atomic_fetch_min(mn.min_key + seg, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lds_run[tid] = 0xFFFFFFFFu;
    };
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const bool more_tiles = tile + gridDim.x < n_tiles;

        // ---- layer-1 B fragments from the words requested earlier
        bf16x8 x[NC][KS1];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
                for (int t = 0; t < 8; ++t) x[c][ks][t] = raw_element<NC, FEAT_BF16>(raw[ks * 8 + t], c);

        // ---- layer 1: h1 = relu(W1^T x + b1), kept as layer-2 B fragments; the conversion of chunk oc-1
        // is issued behind the matrix instructions of chunk oc
        bf16x8 h1[NC][KS2];
        // Two candidate tiles at a time (a "group"; NG groups per chunk): the accumulators of the group before are
        // converted while the matrix instructions of this one run, so two groups' accumulators are live, 64
        // registers, whatever NC is.
        constexpr int NG = NC / 2;
        constexpr int UNPARKED = (NC == 2 && KS2 == 32) ? 10 : 0; // measured at 512 units: 8, 10, 12 -> -1.2, -1.5, -1.4 % cycles
        f32x16 acc1[2][2];
        auto convert_group = [&](int oc, int g, const f32x16(&acc)[2]) {
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    // two floats -> one register of two bf16, then ReLU on the packed bits: a negative bf16 is
                    // a negative 16-bit integer, so one packed integer max clamps both halves
                    u32x4 words;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const f32x2 pair = {acc[cc][8 * half + 2 * d], acc[cc][8 * half + 2 * d + 1]};
                        const bf16x2 cv = __builtin_convertvector(pair, bf16x2);
                        const s16x2 clamped = __builtin_elementwise_max(__builtin_bit_cast(s16x2, cv), (s16x2)(0));
                        words[d] = __builtin_bit_cast(uint32_t, clamped);
                    }
                    // the first UNPARKED k-steps' fragments stay where the conversion left them: the compiler keeps
                    // about that many in architectural registers anyway, and parked ones it copies straight back
                    if (2 * oc + half < UNPARKED) h1[2 * g + cc][2 * oc + half] = __builtin_bit_cast(bf16x8, words);
                    else h1[2 * g + cc][2 * oc + half] = park_in_acc(__builtin_bit_cast(bf16x8, words));
                }
        };
        bf16x8 a1[2][KS1]; // weight fragments of two chunks: one in use, one on its way from LDS
        f32x16 b1c[2];     // and their bias in accumulator order
        auto load_chunk = [&](int oc) {
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) a1[oc & 1][ks] = lds_w1[(oc * KS1 + ks) * 64 + lane];
            b1c[oc & 1] = *reinterpret_cast<const f32x16 *>(lds_b1 + (oc * 2 + h) * 16);
        };
        load_chunk(0);
#pragma unroll
        for (int oc = 0; oc < OC1; ++oc) {
            const bf16x8(&a)[KS1] = a1[oc & 1];
            const f32x16 bias = b1c[oc & 1];
            if (oc + 1 < OC1) load_chunk(oc + 1);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int s = oc * NG + g; // groups in the order they are computed
                f32x16(&acc)[2] = acc1[s & 1];
#pragma unroll
                for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
                    for (int cc = 0; cc < 2; ++cc)
                        acc[cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], x[2 * g + cc][ks], ks == 0 ? bias : acc[cc], 0, 0, 0);
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) keep_in_vgprs(acc[cc]);
                if (s > 0) convert_group((s - 1) / NG, (s - 1) % NG, acc1[(s - 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        convert_group(OC1 - 1, NG - 1, acc1[(OC1 * NG - 1) & 1]);

        // ---- layer 2 + output layer
        float y[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) y[c] = 0.0f;
        f32x16 acc2[2][NC];
        bf16x8 a[RING]; // weight fragments in flight; fragment j of the tile's piece stream sits in a[j % RING]
        // b2 of the chunk about to start, in accumulator-register order: the chunk's first matrix instruction
        // takes it as its C operand, so the bias never costs a vector instruction.  With two candidate tiles it waits
        // in 16 registers of its own; with four there are none to spare and it is read straight into the chunk's NC
        // accumulators (free once the output terms of the chunk before the last are through).
        constexpr bool BIAS_IN_ACC = NC == 4;
        static_assert(!BIAS_IN_ACC || KSP >= 2, "the output terms of a one-k-step piece come after its loop");
        auto bias_fragment = [&](int oc) { return *reinterpret_cast<const f32x16 *>(lds_b2 + (oc * 2 + h) * 16); };
        f32x16 bias_c;
        if (BIAS_IN_ACC) {
#pragma unroll
            for (int c = 0; c < NC; ++c) acc2[0][c] = bias_fragment(0);
        } else {
            bias_c = bias_fragment(0);
        }

        // first feature load of piece q (loads x_first(q) .. x_first(q + 1) - 1 go out in piece q, 1 <= q <= XSPAN), and
        // the entries the load counter sees for piece q (piece LEGAL_PIECE also requests the legality flags)
        constexpr auto x_first = [](int q) constexpr {
            return q < 1 ? 0 : (q > XSPAN ? NXLOADS : ((q - 1) * NXLOADS + XSPAN - 1) / XSPAN);
        };
        constexpr auto x_loads_in = [x_first](int q) constexpr {
            return q < 1 || q > XSPAN ? 0 : x_first(q + 1) - x_first(q) + ((WITH_MIN && q == LEGAL_PIECE) ? 1 : 0);
        };
        // piece p = 2 * oc + HALF of this tile: matrix work into acc2[PAR] (PAR = oc & 1); in between, the
        // output-layer terms of chunk oc - 1 (held in acc2[PAR ^ 1]) for 8 of its 16 accumulator registers
        auto run_piece = [&](auto par_tag, auto half_tag, auto has_prev_tag, auto pidx_tag, int oc) {
            constexpr int PIDX = decltype(pidx_tag)::value; // the piece's index where known at compile time, else -1
            constexpr int PAR = decltype(par_tag)::value, HALF = decltype(half_tag)::value;
            constexpr bool HAS_PREV = decltype(has_prev_tag)::value;
            constexpr int SLOT = 2 * PAR + HALF; // (2 * oc + HALF) & 3
            const int p = 2 * oc + HALF;
            // piece p+1 must have landed.  Operations issued after its fetch: the feature loads of pieces p-2 and
            // p-1 and, between them, the fetch of piece p+2 (if there is one).  Where iterations are written out, the
            // pieces whose index is not known come after the loads and the two pieces behind them.
            if (PIDX >= 0 || PEEL > 0)
                wait_vm<N_DMA, (PIDX < 0 ? 0 : x_loads_in(PIDX - 2) + x_loads_in(PIDX - 1))>(p + 2 < PIECES || more_tiles);
            else if (p == 2 || p == 3) // nothing written out: all loads went out in piece 1
                wait_vm<N_DMA, x_loads_in(1)>(p + 2 < PIECES || more_tiles);
            else wait_vm<N_DMA, 0>(p + 2 < PIECES || more_tiles);
            __syncthreads();
            if (p + 3 < PIECES) fetch_piece(p + 3);
            else if (more_tiles) fetch_piece(p + 3 - PIECES);
            if (WITH_MIN && LEGAL_PIECE != 1 && PIDX == LEGAL_PIECE) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
                load_legal(tile);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
            if (PIDX == 1) {
                // the feature loads must be issued after the piece fetch: the counter waits rely on that order
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
                if (WITH_MIN && LEGAL_PIECE == 1) load_legal(tile);
                if (XSPAN == 1) load_tile(more_tiles ? tile + gridDim.x : tile, raw);
                else x_begin(more_tiles ? tile + gridDim.x : tile);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
            const bf16x8 *mine = reinterpret_cast<const bf16x8 *>(lds_ring + SLOT * PIECE_BYTES);
            const bf16x8 *next = reinterpret_cast<const bf16x8 *>(lds_ring + ((SLOT + 1) & 3) * PIECE_BYTES);
            if (p == 0) {
#pragma unroll
                for (int i = 0; i < PF; ++i) a[i] = mine[i * 64 + lane];
            }
            f32x16(&acc)[NC] = acc2[PAR];
            const f32x16(&prev)[NC] = acc2[PAR ^ 1];
            f32x4 wprev[2];
            if (HAS_PREV) {
                const f32x4 *wsrc = reinterpret_cast<const f32x4 *>(lds_w3 + ((oc - 1) * 2 + h) * 16 + 8 * HALF);
                wprev[0] = wsrc[0];
                wprev[1] = wsrc[1];
            }
            // the eight output-layer steps of a piece sit in consecutive k-steps, started late enough for the
            // bias / weight vectors requested above to have arrived from LDS
            constexpr int EPI_FIRST = KSP >= 16 ? (KSP - 8) / 2 : 0;
#pragma unroll
            for (int ks = 0; ks < KSP; ++ks) {
                // read ahead, across the piece boundary if need be
                if (PF > 0) {
                    if (ks + PF < KSP) a[(ks + PF) % RING] = mine[(ks + PF) * 64 + lane];
                    else a[(ks + PF) % RING] = next[(ks + PF - KSP) * 64 + lane];
                } else {
                    a[0] = mine[ks * 64 + lane];
                }
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks % RING], h1[c][HALF * KSP + ks],
                                                                     (!BIAS_IN_ACC && HALF == 0 && ks == 0) ? bias_c : acc[c], 0, 0, 0);
                if (XSPAN > 1 && PIDX >= 1 && PIDX <= XSPAN) {
                    // this piece's feature loads, evenly over its k-steps
                    constexpr int LO = x_first(PIDX), CNT = x_first(PIDX + 1) - LO, DIV = CNT > 0 ? CNT : 1;
#pragma unroll
                    for (int m = 0; m < CNT; ++m)
                        if (ks == (m * KSP) / DIV + (KSP >= 2 * CNT ? 1 : 0)) x_one(LO + m, raw);
                }
                if (HAS_PREV) {
                    // Pieces of 16 k-steps: one output-layer step in each of eight k-steps in the middle.  Shorter
                    // pieces: the eight steps spread over the k-steps after the first, which leaves the first for
                    // the weight vector requested above to arrive (a step in k-step 0 stalled the wavefront, and
                    // with it the matrix pipe, for an LDS round trip per piece).
                    constexpr int SPREAD = KSP > 1 ? KSP - 1 : 1;
                    const int first_step = KSP >= 16 ? ks - EPI_FIRST : (ks >= 1 ? 8 * (ks - 1) / SPREAD : 0);
                    const int end_step = KSP >= 16 ? ks - EPI_FIRST + 1 : (ks >= 1 ? 8 * ks / SPREAD : 0);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (j < first_step || j >= end_step) continue;
                        const int q = 8 * HALF + j;
#pragma unroll
                        for (int c = 0; c < NC; ++c) {
                            y[c] = fmaf(relu(prev[c][q]), wprev[j >> 2][j & 3], y[c]);
                            // an empty statement that "uses" the sum: without it the compiler gathers the output
                            // terms of several chunks into one stretch of vector work that no matrix
                            // instruction overlaps
                            asm volatile("" : "+v"(y[c]));
                        }
                    }
                }
                // the next chunk's bias, once the output-layer steps are through (its registers are free
                // again after that chunk's first matrix instructions)
                if (HALF == 1 && ks == (EPI_FIRST + 8 < KSP ? EPI_FIRST + 8 : KSP - 1)) {
                    if (!BIAS_IN_ACC) {
                        bias_c = bias_fragment(oc + 1 < OC2 ? oc + 1 : oc);
                    } else if (oc + 1 < OC2) {
#pragma unroll
                        for (int c = 0; c < NC; ++c) acc2[PAR ^ 1][c] = bias_fragment(oc + 1);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (HAS_PREV && KSP == 1) {
                // (a piece of one k-step has no k-step after the first)
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int c = 0; c < NC; ++c)
                        y[c] = fmaf(relu(prev[c][8 * HALF + j]), wprev[j >> 2][j & 3], y[c]);
            }
        };

        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using NoIdx = std::integral_constant<int, -1>;
        run_piece(I0{}, I0{}, std::false_type{}, std::integral_constant<int, 0>{}, 0);
        run_piece(I0{}, I1{}, std::false_type{}, std::integral_constant<int, 1>{}, 0);
        // chunks oc and oc + 1, the index P0 of their first piece known (>= 0) or not
        auto run_pair = [&](auto p0_tag, int oc) {
            constexpr int P0 = decltype(p0_tag)::value;
            run_piece(I1{}, I0{}, std::true_type{}, std::integral_constant<int, P0 < 0 ? -1 : P0>{}, oc);
            run_piece(I1{}, I1{}, std::true_type{}, std::integral_constant<int, P0 < 0 ? -1 : P0 + 1>{}, oc);
            run_piece(I0{}, I0{}, std::true_type{}, std::integral_constant<int, P0 < 0 ? -1 : P0 + 2>{}, oc + 1);
            run_piece(I0{}, I1{}, std::true_type{}, std::integral_constant<int, P0 < 0 ? -1 : P0 + 3>{}, oc + 1);
        };
        static_assert(PEEL <= 2, "more iterations to write out than there are below");
        if (PEEL >= 1) run_pair(std::integral_constant<int, 2>{}, 1);
        if (PEEL >= 2) run_pair(std::integral_constant<int, 6>{}, 3);
        for (int oc = 1 + 2 * PEEL; oc + 1 < OC2; oc += 2) run_pair(NoIdx{}, oc);
        run_piece(I1{}, I0{}, std::true_type{}, std::integral_constant<int, PIECES - 2>{}, OC2 - 1);
        run_piece(I1{}, I1{}, std::true_type{}, std::integral_constant<int, PIECES - 1>{}, OC2 - 1);
        {
            const f32x16(&last)[NC] = acc2[(OC2 - 1) & 1];
            const f32x4 *wsrc = reinterpret_cast<const f32x4 *>(lds_w3 + ((OC2 - 1) * 2 + h) * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const f32x4 w = wsrc[v];
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[c] = fmaf(relu(last[c][4 * v + e]), w[e], y[c]);
            }
        }
        const uint64_t cand = first_candidate(tile);
        uint32_t key[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const float total = y[c] + __shfl_xor(y[c], 32);
            const float score = total + b3;
            if (h == 0 && cand + c < n) out[cand + c] = score;
            if (WITH_MIN) {
                // (no short-circuit: the three tests are one compare each, a branch per test costs more)
                const bool legal = !mn.legal | (((legal_bits >> (8 * c)) & 0xFFu) != 0);
                const bool counts = legal & (cand + c < n) & (score == score);
                key[c] = counts ? score_order_key(score) : 0xFFFFFFFFu;
            }
        }
        if (WITH_MIN && mn.tiles_per_seg) {
            // segments are whole tiles: 32-bit scalar bookkeeping per tile, no wavefront straddles two segments
            if (tile - seg_tile0 >= mn.tiles_per_seg) {
                flush_running_min();
                seg = tile / mn.tiles_per_seg;
                seg_tile0 = (uint32_t)seg * mn.tiles_per_seg;
            }
            uint32_t best = key[0];
#pragma unroll
            for (int c = 1; c < NC; ++c) best = min(best, key[c]);
            (void)atomicMin(&lds_run[tid], best); // in LDS: no register is held across tiles
        } else if (WITH_MIN) {
            // this wavefront's candidates; everything about the segment is the same in every lane and is kept in
            // scalar registers (the wavefront's number, derived from the thread's, is uniform but not known to be)
            const uint64_t first = (uint64_t)tile * TILE + (uint64_t)__builtin_amdgcn_readfirstlane(wave) * (NC * 32);
            if (first < n) {
                const uint64_t last = first + NC * 32 - 1 < n ? first + NC * 32 - 1 : n - 1;
                // the segment of `first`: tiles come in increasing order, so it is usually the one of the tile before
                // or the next one (a 64-bit division costs as much as a twentieth of a tile's matrix work)
                if (first - seg_begin >= mn.seg_len) {
                    flush_running_min();
                    if (first - seg_begin < 2 * mn.seg_len) {
                        seg += 1;
                        seg_begin += mn.seg_len;
                    } else {
                        seg = first / mn.seg_len;
                        seg_begin = seg * mn.seg_len;
                    }
                }
                if (last - seg_begin < mn.seg_len) {
                    uint32_t best = key[0];
#pragma unroll
                    for (int c = 1; c < NC; ++c) best = min(best, key[c]);
                    (void)atomicMin(&lds_run[tid], best); // in LDS: no register is held across tiles
                } else if (h == 0) {
#pragma unroll
                    for (int c = 0; c < NC; ++c)
                        if (key[c] != 0xFFFFFFFFu)
                            (void)__hip_atomic_fetch_min(mn.min_key + (cand + c) / mn.seg_len, key[c], __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
    if (WITH_MIN) flush_running_min();
}

template <int F, int H1, int H2, int NC, bool WITH_MIN>
int32_t launch_bf16(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n, float *out,
                    const MinArgs &mn, hipStream_t st)
{
    const PackedLayout L = packed_layout(F, H1, H2);
    constexpr int TILE = 4 * NC * 32;
    const uint64_t tiles64 = (n + TILE - 1) / TILE;
    if (tiles64 > 0xFFFFFFFFull) return ECK_EUNSUPPORTED;
    const uint32_t n_tiles = (uint32_t)tiles64;
    int cus = 256;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device);
    const uint32_t grid = n_tiles < (uint32_t)cus ? n_tiles : (uint32_t)cus;
    // W1 and b1, four ring slots of half a W2 chunk, b2 and w3, a running minimum per lane
    const size_t lds = (size_t)F * H1 * 2 + (size_t)H1 * 4 + 4 * (size_t)(H1 / 32) * 1024 + 2 * H2 * 4 + (WITH_MIN ? 1024 : 0);
    // the per-lane part of a feature address is a 32-bit offset unless eight rows exceed it
    const uint64_t elem = feat_dtype == ECK_BF16 ? 2 : 4;
    const bool wide = 8 * ld * elem > 0xFFFFFFFFull - TILE * elem;
    auto kern = feat_dtype == ECK_BF16 ? (wide ? score_bf16_kernel<F, H1, H2, NC, true, true, WITH_MIN>
                                                : score_bf16_kernel<F, H1, H2, NC, true, false, WITH_MIN>)
                                       : (wide ? score_bf16_kernel<F, H1, H2, NC, false, true, WITH_MIN>
                                               : score_bf16_kernel<F, H1, H2, NC, false, false, WITH_MIN>);
    ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    MinArgs mn_tiles = mn;
    mn_tiles.tiles_per_seg = (mn.seg_len % TILE == 0 && mn.seg_len / TILE <= 0xFFFFFFFFull) ? (uint32_t)(mn.seg_len / TILE) : 0;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, (const unsigned char *)m->d_packed, L, feat, ld, n, out,
                       n_tiles, mn_tiles);
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

// least order key per segment of fp32 scores (the small fp32 models, whose forward kernel has no matrix-core epilogue)
__global__ __launch_bounds__(256) void min_key_kernel(const float *__restrict__ score, const uint8_t *__restrict__ legal,
                                                      uint64_t n, uint64_t seg_len, uint32_t *__restrict__ min_key)
{
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float v = score[i];
    if ((legal && !legal[i]) || v != v) return;
    (void)__hip_atomic_fetch_min(min_key + i / seg_len, score_order_key(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void fill_keys_kernel(uint32_t *p, uint32_t n)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0xFFFFFFFFu;
}

template <bool WITH_MIN>
int32_t score_any(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n, float *score_out,
                  const MinArgs &mn, uint32_t n_segments, void *stream)
{
    if (!m || !feat || !score_out || n == 0) return ECK_EINVAL;
    if (feat_dtype != ECK_F32 && feat_dtype != ECK_BF16) return ECK_EINVAL;
    if (ld < n) return ECK_ESHAPE;
    if (n > (1ull << 40)) return ECK_EINVAL;
    hipStream_t st = as_stream(stream);
    const int F = m->widths[0], H1 = m->widths[1], H2 = m->widths[2];
    if (m->dtype == ECK_F32 && feat_dtype != ECK_F32) return ECK_EUNSUPPORTED;
    if (m->dtype == ECK_BF16) {
        // A lane fetches the NC consecutive candidates it owns with one load per feature row.  Groups start at
        // multiples of NC, so with ld a multiple of NC a group that starts below n ends inside its row; otherwise
        // the last group of a row would run into the next row and, in the last row, past the matrix.  The pointer
        // must be aligned to the load as well.
        const uint64_t elem = feat_dtype == ECK_BF16 ? 2 : 4;
        if ((ld & 1) || ((uintptr_t)feat & (2 * elem - 1))) return ECK_EALIGN;
    }
    if (WITH_MIN) {
        hipLaunchKernelGGL(fill_keys_kernel, dim3((n_segments + 255) / 256), dim3(256), 0, st, mn.min_key, n_segments);
    }
    if (m->dtype == ECK_F32) {
        const size_t lds = (size_t)(F + H1 + H2) * F32_TILE * sizeof(float);
        ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(score_f32_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        const uint64_t blocks = (n + F32_TILE - 1) / F32_TILE;
        if (blocks > 0x7FFFFFFFull) return ECK_EUNSUPPORTED;
        // (parameter offsets are then multiples of four floats as well, and the state is 256-byte aligned)
        const bool by_four = H1 % 4 == 0 && H2 % 4 == 0;
        if (by_four) {
            ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(score_f32x4_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(score_f32x4_kernel, dim3((unsigned)blocks), dim3(256), lds, st, m->d_state, F, H1, H2,
                               m->off_w[0], m->off_b[0], m->off_w[1], m->off_b[1], m->off_w[2], m->off_b[2],
                               (const float *)feat, ld, n, score_out);
        } else {
            hipLaunchKernelGGL(score_f32_kernel, dim3((unsigned)blocks), dim3(256), lds, st, m->d_state, F, H1, H2,
                               m->off_w[0], m->off_b[0], m->off_w[1], m->off_b[1], m->off_w[2], m->off_b[2],
                               (const float *)feat, ld, n, score_out);
        }
        if (WITH_MIN)
            hipLaunchKernelGGL(min_key_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, score_out, mn.legal, n,
                               mn.seg_len, mn.min_key);
        ECK_HIP_TRY(hipGetLastError());
        return ECK_OK;
    }
    // four candidate tiles per wavefront (half the weight traffic per candidate) where 256 or fewer hidden units
    // leave the registers for it, the features arrive as bf16 and groups of four stay inside a row (the flags of
    // four candidates are then one 4-byte load)
    const bool four = feat_dtype == ECK_BF16 && ld % 4 == 0 && ((uintptr_t)feat & 7) == 0 &&
                      (!WITH_MIN || !mn.legal || ((uintptr_t)mn.legal & 3) == 0);
    if (F == 64 && H1 == 512 && H2 == 512) return launch_bf16<64, 512, 512, 2, WITH_MIN>(m, feat, feat_dtype, ld, n, score_out, mn, st);
    if (F == 64 && H1 == 256 && H2 == 256 && four)
        return launch_bf16<64, 256, 256, 4, WITH_MIN>(m, feat, feat_dtype, ld, n, score_out, mn, st);
    if (F == 64 && H1 == 256 && H2 == 256) return launch_bf16<64, 256, 256, 2, WITH_MIN>(m, feat, feat_dtype, ld, n, score_out, mn, st);
    if (F == 64 && H1 == 128 && H2 == 128 && four)
        return launch_bf16<64, 128, 128, 4, WITH_MIN>(m, feat, feat_dtype, ld, n, score_out, mn, st);
    if (F == 64 && H1 == 128 && H2 == 128) return launch_bf16<64, 128, 128, 2, WITH_MIN>(m, feat, feat_dtype, ld, n, score_out, mn, st);
    if (F == 32 && H1 == 64 && H2 == 64) return launch_bf16<32, 64, 64, 2, WITH_MIN>(m, feat, feat_dtype, ld, n, score_out, mn, st);
    return ECK_EUNSUPPORTED;
}

} // namespace

extern "C" int32_t costmodel_score(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                                   float *score_out, void *ws, uint64_t ws_bytes, void *stream)
{
    (void)ws;
    (void)ws_bytes;
    return score_any<false>(m, feat, feat_dtype, ld, n, score_out, MinArgs{nullptr, 1, nullptr, 0}, 0, stream);
}

extern "C" int32_t costmodel_score_min(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, uint64_t n,
                                       float *score_out, const uint8_t *legal, uint32_t n_segments, uint32_t *min_key_out,
                                       void *stream)
{
    if (!min_key_out || n_segments == 0) return ECK_EINVAL;
    if (n == 0 || n % n_segments) return n == 0 ? ECK_EINVAL : ECK_ESHAPE;
    if (n / n_segments > 0xFFFFFFFEull || n_segments > 65535) return ECK_ESHAPE;
    if (legal && ((uintptr_t)legal & 1)) return ECK_EALIGN; // two flags per load
    return score_any<true>(m, feat, feat_dtype, ld, n, score_out, MinArgs{legal, n / n_segments, min_key_out, 0}, n_segments,
                           stream);
}
