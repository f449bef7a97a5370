// Internal interface between the expert-MLP entry points and their two kernel families.
#pragma once

#include "xmoe_internal.h"
#include "xmoe_sizes.h"

namespace xmoe {

struct FfnArgs {
    int B, E, d, f, dt;
    const int32_t* off;          // expert_offsets [E+1], device
    const void *xd, *wg, *wu, *wd;
    const int32_t* row_index;    // NULL, or: xd is the token matrix and row i of the expert input is xd[row_index[i]]
    // forward: outputs g, u, y; backward: inputs g, u, dy and outputs dxd, dwg, dwu, dwd
    void *g, *u, *y;
    const void* dy;
    // backward: NULL, or dy is the [T,d] gradient of the layer's output and row i of dY is dy_scale[i] * dy[dy_index[i]]
    const int32_t* dy_index;
    const float* dy_scale;       // NULL = 1
    void *dxd, *dwg, *dwu, *dwd;
    // workspace carve-up
    int32_t* map;                // tile map
    int32_t* sched;              // experts by descending row count [E], then kSchedCounters counters
    void *act, *dg, *du;         // A = silu(G)*U, dG, dU   [B,f]
    // backward, optional: row_grad [B] (caller's) receives <unscaled row of dY, Y[row]> for every row; row_part is
    // the workspace for its partial sums, row_grad_parts(f) x B floats laid out [part][row]
    float* row_grad;
    float* row_part;
};

// the two-matrix expert (xmoe_expert_mlp2_fwd / _bwd)
struct Mlp2Args {
    int B, E, d, f, dt, act;
    const int32_t* off;          // expert_offsets [E+1], device
    const void *xd, *w1, *w2;
    const int32_t* row_index;    // as in FfnArgs
    void *h, *y;                 // forward: outputs; backward: h is an input
    const void* dy;
    const int32_t* dy_index;     // as in FfnArgs
    const float* dy_scale;
    void *dxd, *dw1, *dw2;
    int32_t* map;
    int32_t* sched;
    void *a_buf, *dh;            // A = act(H), dH   [B,f]
    float* row_grad;             // as in FfnArgs
    float* row_part;
};

int launch_tile_map(const int32_t* off, int E, int tile_rows, int max_tiles, int32_t* map, int32_t* sched,
                    hipStream_t s);

// row_grad[i] = sum over p < parts of row_part[p * B + i], p ascending (fixed order: the result is reproducible)
int launch_row_grad_reduce(const float* row_part, int parts, int B, float* row_grad, hipStream_t s);

int ffn_fwd_simt(const FfnArgs& a, hipStream_t s);
int ffn_bwd_simt(const FfnArgs& a, hipStream_t s);

// bf16 MFMA family (needs d % 64 == 0, f % 64 == 0 and 16-byte aligned operands): 256x256 tiles, operands streamed
// global -> LDS directly, transposing LDS reads
bool ffn_dma_supported(const FfnArgs& a);
int ffn_fwd_dma(const FfnArgs& a, hipStream_t s);
int ffn_bwd_dma(const FfnArgs& a, hipStream_t s);

int mlp2_fwd_simt(const Mlp2Args& a, hipStream_t s);
int mlp2_bwd_simt(const Mlp2Args& a, hipStream_t s);
bool mlp2_dma_supported(const Mlp2Args& a);
int mlp2_fwd_dma(const Mlp2Args& a, hipStream_t s);
int mlp2_bwd_dma(const Mlp2Args& a, hipStream_t s);

}  // namespace xmoe
