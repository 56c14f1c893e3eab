// Minibatch Adam steps on the weighted squared error of Eq. (1) for BF16 models, two launches per step
// (Alg. 1: ModelUpdate; Sec. 6.4).  HIP, gfx950.
//
// A step of the refit is a chain of small dependent products; launched one by one it is bound by launch latency.
// Here it is cut where the data dependencies allow no less:
//   rows kernel:     everything that is local to a minibatch row, for 32 rows per block -- both hidden layers, the
//                    output layer, the Eq.-(1) loss term and its derivative, and the deltas of both hidden layers
//                    (the back-propagation through W2 included).  Activations pass from layer to layer through LDS.
//   weights kernel:  everything that sums over the rows of the minibatch -- the three weight gradients and the
//                    bias gradients -- one 32 x 32 tile of a weight matrix per block, the reduction over the rows
//                    split over the block's four wavefronts and added in wavefront order; the Adam update of the
//                    tile's parameters follows at once in the same block (each parameter's gradient is complete
//                    there), together with the bf16 copies the next step's rows kernel multiplies with.
// All large products run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) with the same operand
// roundings as the launch-per-product path: features, weights, first hidden activations and both deltas in bf16,
// biases and the output weights rounded through bf16, the second hidden layer and the output layer in fp32.
// Every reduction has a fixed order, so a run is reproducible bit for bit.
#include "eck_internal.h"

using namespace eck;

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float through_bf16(float x) { return __uint_as_float((uint32_t)bf16_bits(x) << 16); }

// Matrix-core tile (v_mfma_f32_32x32x16_bf16, D = A * B + C, one wavefront, lane = 32 h + c):
//   A (32 rows x 16 k): lane (h, r = c) holds A[r][8h .. 8h+7]      -> 16 contiguous bytes of a k-major row
//   B (16 k x 32 cols): lane (h, c) holds B[8h .. 8h+7][c]           -> 16 contiguous bytes of a k-major column
//   D (32 x 32):        lane (h, c) register q holds D[8 (q / 4) + 4h + q % 4][c]
__device__ __forceinline__ int d_row(int q, int h) { return 8 * (q >> 2) + 4 * h + (q & 3); }

// Operands of the matrix instructions live in memory in fragment order, so that the 64 lanes of a load read one
// contiguous kilobyte: element (n, k) of a matrix whose k index is the reduction index and whose n index picks the
// row (A) or column (B) of the tile sits at
//   ((n / 32 * (K / 16) + k / 16) * 64 + 32 * (k % 16 / 8) + n % 32) * 8 + k % 8        (K = length of the reduction)
__device__ __forceinline__ int64_t frag_at(int n, int k, int K)
{
    return ((int64_t)((n >> 5) * (K >> 4) + (k >> 4)) * 64 + 32 * ((k >> 3) & 1) + (n & 31)) * 8 + (k & 7);
}

// Block barrier that orders LDS traffic only.  __syncthreads() also waits for every global load and store the
// wavefront has in flight (its fence covers global memory); these kernels keep weight fragments for a later phase on
// their way across barriers on purpose, and what they exchange between wavefronts goes through LDS alone.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct StepArgs {
    const void *feat;   // [F][ld] bf16 or fp32, minibatch row r = column row0 + r
    uint64_t ld, row0;
    int rows;           // minibatch size B (a multiple of 64)
    float *theta;       // fp32 master [theta | m | v | t], n_params = P
    uint64_t P;
    uint64_t off_w1, off_b1, off_w2, off_b2, off_w3, off_b3;
    // bf16 copies of the weights, in fragment order:
    uint16_t *w1t;      // n = unit of layer 1, k = feature       (x W1)
    uint16_t *w2t;      // n = unit of layer 2, k = unit of layer 1   (h1 W2)
    uint16_t *w2;       // n = unit of layer 1, k = unit of layer 2   (d2 W2^T)
    const float *y;     // labels of the whole buffer
    // what the weight gradients sum over the minibatch, bf16 in fragment order with n = unit, k = minibatch row:
    uint16_t *h1t;      // first hidden layer
    uint16_t *d2t;      // delta of the second hidden layer
    uint16_t *d1t;      // delta of the first hidden layer
    float *h2;          // fp32 [B][H2]
    float *dy;          // fp32 [B]
    float *lterm;       // fp32 [B]  Eq.-(1) terms of the rows
    const uint32_t *bad; // data error found in the labels: leave the model alone
    float *loss_out;    // mean of the Eq.-(1) terms, written in the step with report_loss set
    float *corr;        // [2] Adam's bias corrections 1 - beta^t of the step (rows kernel -> weights kernel)
    int step_in_call, report_loss;
    float lr, beta1, beta2, eps;
};

// ------------------------------------------------------------------------------------------------ rows kernel

// Weight fragments of one 32-column tile (k-major columns starting at b_col) are fetched up to 16 k-steps at a time,
// so that one round trip to the L2 covers that much of the reduction; the first batch is requested long before
// its product starts (EARLY k-steps), the rest -- reductions deeper than 256 -- inside the product.
template <int K>
struct Fragments {
    static constexpr int EARLY = K / 16 < 16 ? K / 16 : 16;
    bf16x8 b[EARLY];
};

template <int K>
__device__ __forceinline__ void fetch_fragments(const uint16_t *tile, int lane, Fragments<K> &f)
{
    // `tile`: the K / 16 fragments of one 32-column tile, 512 elements each
    const uint16_t *bp = tile + lane * 8;
#pragma unroll
    for (int ks = 0; ks < Fragments<K>::EARLY; ++ks) f.b[ks] = *reinterpret_cast<const bf16x8 *>(bp + 512 * ks);
}

// A (32 x K, bf16, in LDS with row stride LDA) * B (K x 32, fragments starting at `tile`, first batch in f)
template <int K, int LDA>
__device__ __forceinline__ f32x16 row_tile_product(const uint16_t *a_lds, const uint16_t *tile, const Fragments<K> &f, int lane)
{
    constexpr int EARLY = Fragments<K>::EARLY;
    const uint16_t *ap = a_lds + (lane & 31) * LDA + 8 * (lane >> 5);
    const uint16_t *bp = tile + lane * 8;
    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.0f;
    bf16x8 later[K / 16 > EARLY ? EARLY : 1];
    if (K / 16 > EARLY) {
#pragma unroll
        for (int ks = 0; ks < EARLY; ++ks) later[ks] = *reinterpret_cast<const bf16x8 *>(bp + 512 * (EARLY + ks));
    }
#pragma unroll
    for (int ks = 0; ks < EARLY; ++ks)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(ap + 16 * ks), f.b[ks], acc, 0, 0, 0);
    if (K / 16 > EARLY) {
        static_assert(K / 16 <= 2 * EARLY, "reductions of at most 512");
#pragma unroll
        for (int ks = 0; ks < K / 16 - EARLY; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(ap + 16 * (EARLY + ks)), later[ks], acc,
                                                          0, 0, 0);
    }
    return acc;
}

// Registers 4g .. 4g+3 of a D tile -- rows 8g + 4h .. +3 of column c -- as bf16 into a fragment-ordered matrix with
// n = column (unit), k = minibatch row: four consecutive k of one lane's fragment, one 8-byte store.
__device__ __forceinline__ void store_rows4(uint16_t *t, int unit, int rows_total, int row, const uint16_t (&v)[4])
{
    u16x4 packed = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<u16x4 *>(t + frag_at(unit, row, rows_total)) = packed;
}

// One block = 32 minibatch rows; one wavefront per 32-column tile of the widest layer (H / 32 wavefronts), so every
// layer is one tile product per wavefront.  A wavefront fetches the weight fragments of its next product before it
// waits for anything else: those of the first two layers at the very start, those of the back-propagation while the
// output layer is being reduced.  Spare thread: the last thread of block 0 computes Adam's bias corrections of this
// step for the weights kernel (two double-precision powers that would otherwise sit on that kernel's critical path).
template <int F, int H1, int H2, bool FEAT_BF16>
__global__ __launch_bounds__((H1 > H2 ? H1 : H2) * 2) void step_rows_kernel(StepArgs a)
{
    constexpr int NW = (H1 > H2 ? H1 : H2) / 32, NT = NW * 64;
    constexpr int LDX = F + 8, LD1 = H1 + 8, LD2 = H2 + 8; // LDS row strides in bf16: 16-byte fragment reads without conflicts
    static_assert(H1 % 32 == 0 && H2 % 32 == 0 && F % 16 == 0 && NW <= 16, "tile shapes");
    extern __shared__ __attribute__((aligned(16))) unsigned char rows_lds[];
    uint16_t *x_l = reinterpret_cast<uint16_t *>(rows_lds);      // [32][LDX]
    uint16_t *h1_l = x_l + 32 * LDX;                             // [32][LD1]
    uint16_t *d2_l = h1_l + 32 * LD1;                            // [32][LD2]
    float *part_l = reinterpret_cast<float *>(d2_l + 32 * LD2);  // [NW][32] per-wavefront partial dot products
    float *dy_l = part_l + NW * 32;                              // [32]
    float *tile_l = dy_l + 32;                                   // [NW][32][33] output-layer terms
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
    const int r0 = blockIdx.x * 32; // first minibatch row of this block
    const bool has1 = wave < H1 / 32, has2 = wave < H2 / 32; // this wavefront owns a tile of the first / second layer
    const int col = 32 * wave + c;

    Fragments<F> w1f;
    Fragments<H1> w2f;
    float bias1 = 0.0f, bias2 = 0.0f, w3 = 0.0f;
    if (has1) {
        fetch_fragments<F>(a.w1t + (int64_t)wave * 32 * F, lane, w1f); // tile `wave`: 32 * F elements
        bias1 = through_bf16(a.theta[a.off_b1 + col]);
    }
    if (has2) {
        fetch_fragments<H1>(a.w2t + (int64_t)wave * 32 * H1, lane, w2f);
        bias2 = through_bf16(a.theta[a.off_b2 + col]);
        w3 = through_bf16(a.theta[a.off_w3 + col]);
    }
    // the block's 32 feature rows, as bf16, k-major
    for (int e = tid; e < 32 * F; e += NT) {
        const int r = e & 31, f = e >> 5;
        const uint64_t at = (uint64_t)f * a.ld + a.row0 + r0 + r;
        x_l[r * LDX + f] = FEAT_BF16 ? reinterpret_cast<const uint16_t *>(a.feat)[at]
                                     : bf16_bits(reinterpret_cast<const float *>(a.feat)[at]);
    }
    // what the output layer will want from memory, requested now
    float target = 1.0f, bias3 = 0.0f;
    if (tid < 32) {
        target = a.y[a.row0 + r0 + tid];
        bias3 = through_bf16(a.theta[a.off_b3]);
    }
    const float step_count = (blockIdx.x == 0 && tid == NT - 1) ? a.theta[3 * a.P] : 0.0f;
    lds_barrier();

    // ---- h1 = relu(x W1 + b1), bf16
    if (has1) {
        const f32x16 acc = row_tile_product<F, LDX>(x_l, a.w1t + (int64_t)wave * 32 * F, w1f, lane);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint16_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = bf16_bits(fmaxf(acc[4 * g + e] + bias1, 0.0f));
                h1_l[d_row(4 * g + e, h) * LD1 + col] = v[e];
            }
            store_rows4(a.h1t, col, a.rows, r0 + d_row(4 * g, h), v);
        }
    }
    lds_barrier();

    // ---- h2 = relu(h1 W2 + b2), fp32; the partial output-layer products of this wavefront's columns
    float h2v[16], dot[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) h2v[q] = dot[q] = 0.0f;
    if (has2) {
        const f32x16 acc = row_tile_product<H1, LD1>(h1_l, a.w2t + (int64_t)wave * 32 * H1, w2f, lane);
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            h2v[q] = fmaxf(acc[q] + bias2, 0.0f);
            a.h2[(int64_t)(r0 + d_row(q, h)) * H2 + col] = h2v[q];
            dot[q] = h2v[q] * w3;
        }
    }
    // the fragments of W2 for the way back are under way while the output layer is summed
    Fragments<H2> wbf;
    if (has1) fetch_fragments<H2>(a.w2 + (int64_t)wave * 32 * H2, lane, wbf);
    // Output layer: every lane holds 16 row-terms of one column.  The wavefront's 32 x 32 terms go through LDS so
    // that a lane can add up 16 columns of one row (fixed order); the two halves of the row meet in one exchange.
    {
        float *terms = tile_l + wave * (32 * 33); // [32 rows][33]: rows a bank apart
#pragma unroll
        for (int q = 0; q < 16; ++q) terms[d_row(q, h) * 33 + c] = dot[q];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the wavefront reads back what its own lanes wrote
        float sum = 0.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j) sum += terms[c * 33 + 16 * h + j];
        sum += __shfl_xor(sum, 32);
        if (h == 0) part_l[wave * 32 + c] = sum;
    }
    lds_barrier();
    if (tid < 32) {
        float pred = part_l[tid];
#pragma unroll
        for (int w = 1; w < H2 / 32; ++w) pred += part_l[w * 32 + tid];
        pred += bias3;
        const float d = pred - target;
        const float g = 2.0f * d / (target * (float)a.rows);
        a.dy[r0 + tid] = g;
        a.lterm[r0 + tid] = d * d / target;
        dy_l[tid] = g;
    }
    lds_barrier();
    // ---- d2 = dy w3 where h2 > 0, bf16
    if (has2) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint16_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = d_row(4 * g + e, h);
                v[e] = bf16_bits(h2v[4 * g + e] > 0.0f ? dy_l[row] * w3 : 0.0f);
                d2_l[row * LD2 + col] = v[e];
            }
            store_rows4(a.d2t, col, a.rows, r0 + d_row(4 * g, h), v);
        }
    }
    lds_barrier();
    // ---- d1 = (d2 W2^T) where h1 > 0, bf16
    if (has1) {
        const f32x16 acc = row_tile_product<H2, LD2>(d2_l, a.w2 + (int64_t)wave * 32 * H2, wbf, lane);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint16_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = d_row(4 * g + e, h);
                const bool active = h1_l[row * LD1 + col] != 0; // a ReLU output: positive unless its bits are zero
                v[e] = active ? bf16_bits(acc[4 * g + e]) : (uint16_t)0;
            }
            store_rows4(a.d1t, col, a.rows, r0 + d_row(4 * g, h), v);
        }
    }
    if (blockIdx.x == 0 && tid == NT - 1) {
        const double t = (double)step_count + a.step_in_call + 1; // t itself is advanced once, after the last step
        a.corr[0] = (float)(1.0 - pow((double)a.beta1, t));
        a.corr[1] = (float)(1.0 - pow((double)a.beta2, t));
    }
}

// --------------------------------------------------------------------------------------------- weights kernel

// Adam on one parameter (bias-corrected, no weight decay) from its state as fetched earlier; returns the new value
__device__ __forceinline__ float adam_one(float *theta, uint64_t P, uint64_t i, float w, float m, float v, float g,
                                          float beta1, float beta2, float lr, float eps, float c1, float c2)
{
    m = beta1 * m + (1.0f - beta1) * g;
    v = beta2 * v + (1.0f - beta2) * g * g;
    theta[P + i] = m;
    theta[2 * P + i] = v;
    const float next = w - lr * (m / c1) / (sqrtf(v / c2) + eps);
    theta[i] = next;
    return next;
}

// Blocks, in order: the 32 x 32 tiles of W2 (H1/32 x H2/32), the tiles of W1 (F/32 x H1/32), then blocks of 16
// columns of the output layer.  A tile block: C[m][n] = sum_r A[m][r] B[r][n] with both operands stored row-index
// fastest (A = h1^T or x^T, B = d2^T or d1^T); wavefront w sums rows [w B/4, (w+1) B/4) -- its fragments fetched
// eight k-steps at a time, and the Adam state of the four parameters each thread will update fetched before that --
// the four partial tiles are added in wavefront order through LDS, then 256 threads update four parameters each.
// The blocks of the first tile row also sum the columns of B: the bias gradient.
template <int F, int H1, int H2, bool FEAT_BF16>
__global__ __launch_bounds__(256) void step_weights_kernel(StepArgs a)
{
    __shared__ float part[4][16][64];   // partial tiles of the four wavefronts
    __shared__ float colsum[4][32];     // partial bias gradients
    __shared__ double lsum[256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
    constexpr int TILES_W2 = (H1 / 32) * (H2 / 32), TILES_W1 = (F / 32) * (H1 / 32);
    const int B = a.rows;
    const bool bad = *a.bad != 0;
    const float c1 = a.corr[0], c2 = a.corr[1]; // Adam's bias corrections of this step, from the rows kernel
    int block = blockIdx.x;
    if (block < TILES_W2 + TILES_W1) {
        const bool second = block < TILES_W2; // a tile of W2, else of W1
        if (!second) block -= TILES_W2;
        const int nt = second ? H2 / 32 : H1 / 32;
        const int mt = block / nt, ntile = block % nt;
        // the parameters this thread updates: tile elements (q = 4 wave + e, lane) -> row d_row(q, h), column c
        uint64_t at[4];
        float w_old[4], m_old[4], v_old[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = 32 * mt + d_row(4 * wave + e, h), n = 32 * ntile + c;
            at[e] = second ? a.off_w2 + (uint64_t)m * H2 + n : a.off_w1 + (uint64_t)m * H1 + n;
            w_old[e] = a.theta[at[e]];
            m_old[e] = a.theta[a.P + at[e]];
            v_old[e] = a.theta[2 * a.P + at[e]];
        }
        // A rows: hidden unit (W2) or feature (W1) 32 mt + m; B columns: unit 32 ntile + n
        const uint16_t *bsrc = (second ? a.d2t : a.d1t) + (int64_t)ntile * 32 * B + lane * 8; // fragments of tile ntile
        const uint16_t *asrc = a.h1t + (int64_t)mt * 32 * B + lane * 8;
        const uint64_t feat_row = (uint64_t)(32 * mt + c) * a.ld + a.row0 + 8 * h;
        const int k0 = wave * (B / 64), k1 = k0 + B / 64; // k-steps of 16 rows; B / 64 is a multiple of... at least 1
        f32x16 acc;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[q] = 0.0f;
        float bsum = 0.0f;
        for (int kb = k0; kb < k1; kb += 8) {
            bf16x8 av[8], bv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int ks = kb + u < k1 ? kb + u : k1 - 1; // clamped: every load stays inside the operands
                bv[u] = *reinterpret_cast<const bf16x8 *>(bsrc + 512 * ks);
                if (second) {
                    av[u] = *reinterpret_cast<const bf16x8 *>(asrc + 512 * ks);
                } else if (FEAT_BF16) {
                    av[u] = *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const uint16_t *>(a.feat) + feat_row + 16 * ks);
                } else {
                    const float4 lo = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(a.feat) + feat_row + 16 * ks);
                    const float4 hi = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(a.feat) + feat_row + 16 * ks + 4);
                    const float f8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) av[u][e] = __builtin_bit_cast(__bf16, bf16_bits(f8[e]));
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (kb + u < k1) {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], bv[u], acc, 0, 0, 0);
                    if (mt == 0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) bsum += (float)bv[u][e];
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) part[wave][q][lane] = acc[q];
        if (mt == 0) {
            bsum += __shfl_xor(bsum, 32); // the two halves of a wavefront hold different rows of the same column
            if (h == 0) colsum[wave][c] = bsum;
        }
        lds_barrier();
        if (bad) return;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int q = 4 * wave + e;
            const float g = ((part[0][q][lane] + part[1][q][lane]) + part[2][q][lane]) + part[3][q][lane];
            const int m = 32 * mt + d_row(q, h), n = 32 * ntile + c;
            const float w = adam_one(a.theta, a.P, at[e], w_old[e], m_old[e], v_old[e], g, a.beta1, a.beta2, a.lr, a.eps, c1, c2);
            const uint16_t wb = bf16_bits(w);
            if (second) {
                a.w2[frag_at(m, n, H2)] = wb;
                a.w2t[frag_at(n, m, H1)] = wb;
            } else {
                a.w1t[frag_at(n, m, F)] = wb;
            }
        }
        if (mt == 0 && tid < 32) {
            const float g = ((colsum[0][tid] + colsum[1][tid]) + colsum[2][tid]) + colsum[3][tid];
            const uint64_t i = (second ? a.off_b2 : a.off_b1) + 32 * ntile + tid;
            (void)adam_one(a.theta, a.P, i, a.theta[i], a.theta[a.P + i], a.theta[2 * a.P + i], g, a.beta1, a.beta2, a.lr, a.eps,
                           c1, c2);
        }
        return;
    }
    // ---- output layer: [gW3 ; gb3] = [h2 ; 1]^T dy, 16 columns per block, 16 row groups summed in order (short
    // chains of loads: every batch of them is a round trip to memory the rows kernel wrote on other dies)
    block -= TILES_W2 + TILES_W1;
    float *psum = &part[0][0][0]; // [16 row groups][16 columns]
    const int cg = tid & 15, rg = tid >> 4;
    const int col = block * 16 + cg;
    float acc = 0.0f;
    {
        const int per = B / 16, rlo = rg * per, rhi = rlo + per; // B is a multiple of 64: per is a multiple of 4
        if (col < H2) {
            for (int r = rlo; r < rhi; r += 4) {
                float v[4], d[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    v[u] = a.h2[(int64_t)(r + u) * H2 + col];
                    d[u] = a.dy[r + u];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc = fmaf(v[u], d[u], acc);
            }
        } else if (col == H2) {
            for (int r = rlo; r < rhi; ++r) acc += a.dy[r];
        }
    }
    psum[rg * 16 + cg] = acc;
    if (block == 0 && a.report_loss) {
        double s = 0.0;
        for (int r = tid; r < B; r += 256) s += (double)a.lterm[r];
        lsum[tid] = s;
    }
    __syncthreads();
    if (block == 0 && a.report_loss) {
        for (int off = 128; off > 0; off >>= 1) {
            if (tid < off) lsum[tid] += lsum[tid + off];
            __syncthreads();
        }
        if (tid == 0 && !bad) *a.loss_out = (float)(lsum[0] / B);
    }
    if (bad) return;
    if (tid < 16 && col <= H2) {
        float g = psum[cg];
#pragma unroll
        for (int r = 1; r < 16; ++r) g += psum[r * 16 + cg];
        const uint64_t i = col < H2 ? a.off_w3 + col : a.off_b3;
        (void)adam_one(a.theta, a.P, i, a.theta[i], a.theta[a.P + i], a.theta[2 * a.P + i], g, a.beta1, a.beta2, a.lr, a.eps,
                       c1, c2);
    }
}

// bf16 copies of W1 and W2 in the fragment order the rows kernel multiplies with
__global__ void step_prepare_kernel(const float *theta, uint64_t off_w1, uint64_t off_w2, int F, int H1, int H2,
                                    uint16_t *w1t, uint16_t *w2t, uint16_t *w2)
{
    const int n1 = F * H1, n2 = H1 * H2;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < n1 + n2; e += gridDim.x * blockDim.x) {
        if (e < n1) {
            const int f = e / H1, i = e % H1;
            w1t[frag_at(i, f, F)] = bf16_bits(theta[off_w1 + e]);
        } else {
            const int x = e - n1, i = x / H2, j = x % H2;
            const uint16_t b = bf16_bits(theta[off_w2 + x]);
            w2[frag_at(i, j, H2)] = b;
            w2t[frag_at(j, i, H1)] = b;
        }
    }
}

template <int F, int H1, int H2>
int32_t launch_steps(const eck_model *m, StepArgs a, int32_t feat_dtype, int32_t n_steps, uint64_t n_pairs, float *loss_scalar,
                     hipStream_t st)
{
    constexpr int NW = (H1 > H2 ? H1 : H2) / 32;
    const size_t lds = (size_t)32 * ((F + 8) + (H1 + 8) + (H2 + 8)) * sizeof(uint16_t) + (NW * 32 + 32 + NW * 32 * 33) * sizeof(float);
    auto rows_kernel = feat_dtype == ECK_BF16 ? step_rows_kernel<F, H1, H2, true> : step_rows_kernel<F, H1, H2, false>;
    auto weights_kernel = feat_dtype == ECK_BF16 ? step_weights_kernel<F, H1, H2, true> : step_weights_kernel<F, H1, H2, false>;
    ECK_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(rows_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    hipLaunchKernelGGL(step_prepare_kernel, dim3(128), dim3(256), 0, st, a.theta, a.off_w1, a.off_w2, F, H1, H2, a.w1t, a.w2t,
                       a.w2);
    const int B = a.rows;
    const uint64_t nb = n_pairs / (uint64_t)B;
    const unsigned weight_blocks = (H1 / 32) * (H2 / 32) + (F / 32) * (H1 / 32) + (H2 + 1 + 15) / 16;
    for (int s = 0; s < n_steps; ++s) {
        a.row0 = ((uint64_t)s % nb) * (uint64_t)B;
        a.step_in_call = s;
        a.report_loss = s == n_steps - 1;
        a.loss_out = loss_scalar;
        hipLaunchKernelGGL(rows_kernel, dim3(B / 32), dim3(NW * 64), lds, st, a);
        hipLaunchKernelGGL(weights_kernel, dim3(weight_blocks), dim3(256), 0, st, a);
    }
    (void)m;
    ECK_HIP_TRY(hipGetLastError());
    return ECK_OK;
}

} // namespace

uint64_t eck::refit_workspace_bytes(const eck_model *m, int minibatch)
{
    auto align = [](uint64_t v) { return (v + 255) & ~255ull; };
    const uint64_t F = m->widths[0], H1 = m->widths[1], H2 = m->widths[2], B = (uint64_t)minibatch;
    return align(F * H1 * 2) + align(H1 * H2 * 2) * 2 + align(H1 * B * 2) * 2 + align(H2 * B * 2) + align(B * H2 * 4) +
           align(B * 4) * 2 + 256;
}

bool eck::refit_applies(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, int minibatch)
{
    if (m->dtype != ECK_BF16 || minibatch % 64) return false;
    // the weights kernel reads eight consecutive rows of a feature with 16-byte loads
    const uint64_t elem = feat_dtype == ECK_BF16 ? 2 : 4;
    if ((ld * elem) % 16 || ((uintptr_t)feat & 15)) return false;
    return m->widths[0] % 32 == 0; // tiles of W1 are 32 features tall
}

int32_t eck::refit_steps(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, const float *y, uint64_t n_pairs,
                         int32_t n_steps, int32_t minibatch, float lr, float beta1, float beta2, float eps,
                         const uint32_t *bad_flag, float *loss_scalar, void *ws, hipStream_t st)
{
    auto align = [](uint64_t v) { return (v + 255) & ~255ull; };
    const uint64_t F = m->widths[0], H1 = m->widths[1], H2 = m->widths[2], B = (uint64_t)minibatch;
    char *p = static_cast<char *>(ws);
    auto take = [&](uint64_t bytes) {
        char *at = p;
        p += align(bytes);
        return at;
    };
    StepArgs a = {};
    a.feat = feat;
    a.ld = ld;
    a.rows = minibatch;
    a.theta = m->d_state;
    a.P = m->n_params;
    a.off_w1 = m->off_w[0];
    a.off_b1 = m->off_b[0];
    a.off_w2 = m->off_w[1];
    a.off_b2 = m->off_b[1];
    a.off_w3 = m->off_w[2];
    a.off_b3 = m->off_b[2];
    a.w1t = reinterpret_cast<uint16_t *>(take(F * H1 * 2));
    a.w2t = reinterpret_cast<uint16_t *>(take(H1 * H2 * 2));
    a.w2 = reinterpret_cast<uint16_t *>(take(H1 * H2 * 2));
    a.h1t = reinterpret_cast<uint16_t *>(take(H1 * B * 2));
    a.d1t = reinterpret_cast<uint16_t *>(take(H1 * B * 2));
    a.d2t = reinterpret_cast<uint16_t *>(take(H2 * B * 2));
    a.h2 = reinterpret_cast<float *>(take(B * H2 * 4));
    a.dy = reinterpret_cast<float *>(take(B * 4));
    a.lterm = reinterpret_cast<float *>(take(B * 4));
    a.corr = reinterpret_cast<float *>(take(2 * sizeof(float)));
    a.y = y;
    a.bad = bad_flag;
    a.lr = lr;
    a.beta1 = beta1;
    a.beta2 = beta2;
    a.eps = eps;
    if (F == 64 && H1 == 512 && H2 == 512) return launch_steps<64, 512, 512>(m, a, feat_dtype, n_steps, n_pairs, loss_scalar, st);
    if (F == 64 && H1 == 256 && H2 == 256) return launch_steps<64, 256, 256>(m, a, feat_dtype, n_steps, n_pairs, loss_scalar, st);
    if (F == 64 && H1 == 128 && H2 == 128) return launch_steps<64, 128, 128>(m, a, feat_dtype, n_steps, n_pairs, loss_scalar, st);
    if (F == 32 && H1 == 64 && H2 == 64) return launch_steps<32, 64, 64>(m, a, feat_dtype, n_steps, n_pairs, loss_scalar, st);
    return ECK_EUNSUPPORTED;
}
