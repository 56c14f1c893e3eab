// Internal declarations shared by the translation units of libeck (HIP, gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "eck.h"

#define ECK_HIP_TRY(expr)                       \
    do {                                        \
        if ((expr) != hipSuccess) {             \
            (void)hipGetLastError();            \
            return ECK_EDEVICE;                 \
        }                                       \
    } while (0)

namespace eck {

constexpr int NAX = 5;      // axis slots: four spatial, one reduction
constexpr int RED_AXIS = 4; // GEMM/BGEMM: (B, M, N, -, K); CONV2D: (N, K_out, H_out, W_out, C)

// Everything the enumerate / feature kernels need about one space; passed by value.
struct SpaceParams {
    int32_t kind, op, n_genes, n_split;
    uint32_t radix[8];
    int32_t split_axis[NAX];   // axis slot of split gene s
    uint32_t table_off[NAX];   // first entry of split gene s in the concatenated table
    uint32_t table_total;      // entries in the concatenated table
    uint32_t ext[NAX];         // true extents per axis slot
    uint32_t R, S, stride;
    uint32_t elem_bytes;
    uint32_t hw_num_cu, hw_wave, hw_lds_bytes, hw_max_threads_cu, hw_max_blocks_cu;
    int32_t vec_axis;          // spatial axis whose innermost level is contiguous in memory
    uint64_t true_out, true_red, flop_useful, compulsory_bytes, compulsory_in_bytes;
    uint32_t const_q10[6];     // transformed per-space constants: features 0, 22, 60, 61, 62, 63
};

// bytes before the tables in a space's device copy
constexpr size_t kDevHeader = (sizeof(SpaceParams) + 15) & ~(size_t)15;

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

} // namespace eck

struct eck_space {
    eck_problem pb;
    eck::SpaceParams prm;
    std::vector<uint16_t> tables; // [table_total][4]
    uint32_t table_n[eck::NAX];
    uint64_t size;                // 0 when it overflows
    unsigned char *d_blob = nullptr; // device copy [SpaceParams, padded to kDevHeader | tables], made on first use
    int device = -1;
};

struct eck_model {
    int32_t n_layers;
    int32_t widths[4];
    int32_t dtype;
    uint64_t n_params;
    uint64_t off_w[3], off_b[3]; // offsets of W_l and b_l in theta
    float *d_state = nullptr;    // [theta | m | v | t]  (3P+1 floats)
    void *d_packed = nullptr;    // BF16: weights in matrix-core fragment order + fp32 bias/output vectors
    uint64_t packed_bytes = 0;
    int device = -1;
};

namespace eck {
// re-derive the packed weights from theta (BF16 models); enqueued on stream
int32_t model_repack(eck_model *m, hipStream_t stream);
// Adam steps of a BF16 model in two launches per step (refit.hip): whether that path takes this call, the bytes it
// needs behind the other buffers of costmodel_update's workspace, and the steps themselves (labels y and the
// data-error flag come from the caller's kernels; the last step's mean loss goes to *loss_scalar, device memory)
bool refit_applies(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, int minibatch);
uint64_t refit_workspace_bytes(const eck_model *m, int minibatch);
int32_t refit_steps(const eck_model *m, const void *feat, int32_t feat_dtype, uint64_t ld, const float *y, uint64_t n_pairs,
                    int32_t n_steps, int32_t minibatch, float lr, float beta1, float beta2, float eps,
                    const uint32_t *bad_flag, float *loss_scalar, void *ws, hipStream_t st);
// topk_select on a workspace of the caller's or of the library's; known_min: THRESHOLD mode with the least latency
// of every segment already known (device, one order key per segment), else NULL
int32_t topk_select_impl(const float *energy, const float *latency, const uint8_t *legal, uint64_t n, uint32_t n_segments,
                         uint32_t k, int32_t mode, float alpha, uint32_t m_latency, uint32_t *idx_out, float *energy_out,
                         uint32_t *count_out, void *ws, uint64_t ws_bytes, void *stream, const uint32_t *known_min);
} // namespace eck
