// Internal interface between the C-ABI host code (tp_api.cpp) and the gfx950 kernels
// (tp_kernels.hip).  Not installed; the public interface is include/tp_linear.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "tp_linear.h"

namespace tpl {

// Memory form of a product C[m,n] = sum_k A(m,k) B(k,n).  "kc" = the operand is stored with the
// contraction index contiguous (A as [m][k], B as [n][k]); otherwise the other index is contiguous
// (A as [k][m], B as [k][n]) and the tile is transposed on its way into LDS.
enum GemmForm {
    FORM_NN = 0,   // forward : A = X  [m][k] (kc),  B = W  [k][n]
    FORM_NT = 1,   // dX      : A = dA [m][k] (kc),  B = W  [n][k] (kc)
    FORM_TN = 2    // dW      : A = X  [k][m],       B = dA [k][n]
};

struct GemmArgs {
    const void* a[TP_MAX_STEPS];
    const void* b[TP_MAX_STEPS];
    int32_t lda[TP_MAX_STEPS];   // elements
    int32_t ldb[TP_MAX_STEPS];
    int32_t M, N, K;             // output extents and the contraction length of ONE step
    int32_t n_steps;
    int32_t tiles_m, tiles_n;
    int32_t split_k;             // >= 1; > 1 writes fp32 partials to ws
    int32_t group_m;             // tile-order group height (tile rows)
    // epilogue (used when split_k == 1)
    void* out;   int64_t ldo;   int32_t out_f32;
    void* pre;   int64_t ldp;           // optional bf16 copy of the pre-activation
    const void* bias;                   // bf16 [N] or null
    int32_t gelu;                       // apply erf-GeLU after the bias
    const void* dg; int64_t lddg;       // optional bf16 [M][N]: multiply by GeLU'(dg)
    float* ws;                          // [split_k][M][N] fp32 partials
    int32_t rotate;                     // rotate the K-tile order inside a step per C tile
    int32_t max_workgroups;             // persistent grid size cap (workgroups resident at once)
    // Grouped launch (n_groups > 1): n_groups independent single-step products of the same extents
    // in one grid, product g = a[g] x b[g] -> outs[g] (no epilogue).  The groups are laid side by
    // side along N (group_along_n) or along M in the tile grid: tiles_m / tiles_n then count the
    // tiles of all groups together and group_tiles is one group's tile count along that axis.
    // With split_k > 1 the partial planes are ws[(z * n_groups + g)][M][N].
    int32_t n_groups, group_along_n, group_tiles;
    void* outs[TP_MAX_STEPS];
    int64_t ldos[TP_MAX_STEPS];
};

struct ReduceArgs {
    const float* ws; int64_t plane;      // first partial plane and the distance between planes, in floats
    int32_t split_k; int32_t M, N;
    void* out;   int64_t ldo;   int32_t out_f32;
    void* pre;   int64_t ldp;
    const void* bias; int32_t gelu;
    const void* dg; int64_t lddg;
};

// tile ids: macro-tile shapes the GEMM kernel is instantiated for
enum TileId { TILE_256x256 = 1, TILE_128x256 = 2, TILE_256x128 = 3, TILE_128x128 = 4,
              TILE_256x256_W4 = 5 };   // 256 x 256 by the four-wave stream kernel (tp_gemm4.hip)
void tile_shape(int tile_id, int* bm, int* bn);

hipError_t launch_gemm(int form, int tile_id, const GemmArgs& args, hipStream_t stream);
hipError_t launch_gemm4(int form, const GemmArgs& args, hipStream_t stream);   // TILE_256x256_W4 (args already normalised)
hipError_t launch_reduce(const ReduceArgs& args, hipStream_t stream);
hipError_t launch_dgelu(const void* dy, int64_t ld_dy, const void* pre, int64_t ld_pre,
                        void* da, int64_t ld_da, int64_t rows, int64_t cols, hipStream_t stream);
hipError_t launch_colsum(const void* da, int64_t ld, int64_t rows, int64_t cols, float* out, float* ws, hipStream_t stream);
size_t colsum_ws_bytes(int64_t rows, int64_t cols);     // 0: the column sum needs no workspace
// y = [GeLU](c + bias) over an fp32 [rows][cols] block, optional bf16 copy of c + bias
hipError_t launch_bias_act(const float* c, int64_t ldc, const void* bias, int gelu, void* y, int64_t ldy, int y_f32,
                           void* pre, int64_t ldp, int64_t rows, int64_t cols, hipStream_t stream);

}  // namespace tpl
