// Host-side workspace layouts of libxmoe (shared by xmoe_workspace_bytes and the entry points).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "xmoe_internal.h"

namespace xmoe {

// ----- ERI construction: one histogram row of E counters per chunk of kEriChunk flat entries -----
constexpr int kEriChunk = 1024;
static inline int eri_num_chunks(long long B) { return (int)((B + kEriChunk - 1) / kEriChunk); }
static inline size_t eri_ws_bytes(int T, int E, int k) {
    long long B = (long long)T * k;
    return align_up((size_t)(eri_num_chunks(B) > 0 ? eri_num_chunks(B) : 1) * (size_t)E * sizeof(int32_t), 256);
}

// token-dropping construction: the above, then the dropless table it selects from (offsets, counts, flat entry and
// weight of every row)
static inline size_t eri_capped_ws_bytes(int T, int E, int k) {
    long long B = (long long)T * k;
    return eri_ws_bytes(T, E, k) + align_up((size_t)(E + 1) * sizeof(int32_t), 256) +
           align_up((size_t)E * sizeof(int32_t), 256) + 2 * align_up((size_t)(B > 0 ? B : 1) * sizeof(int32_t), 256);
}

// ----- ragged grouped GEMM: the tile map lists, for every row tile, its expert and first row -----
// Sized for the smallest row tile any kernel uses (kMinRowTile rows): at most ceil(B/tile) + E tiles.
constexpr int kMinRowTile = 64;
static inline int ffn_max_tiles(int B, int E, int tile_rows) { return (B + tile_rows - 1) / tile_rows + E; }
// After the pairs comes the schedule block of the weight-gradient kernels: the experts in order of descending row
// count (E ints), then kSchedCounters work counters zeroed by the tile-map kernel: 8 (one per XCD) for each of the two
// weight-gradient launches of a call, then 8 for each of its two row-GEMM launches.
constexpr int kSchedCounters = 32;
static inline size_t ffn_sched_offset(int B, int E) { return 4 + 2 * (size_t)ffn_max_tiles(B, E, kMinRowTile); }
static inline size_t ffn_tilemap_bytes(int B, int E) {
    // header of 4 ints (total tiles, ...) followed by (expert, row0) pairs, then the schedule block
    return align_up((ffn_sched_offset(B, E) + (size_t)E + kSchedCounters) * sizeof(int32_t), 256);
}
static inline size_t ffn_act_bytes(int B, int f, int dt) { return align_up((size_t)B * (size_t)f * dtype_size(dt), 256); }

// partial sums of the per-row inner products <dY row, Y row> that the dAct kernels produce: one per row and per
// 64 output columns of the matrix-core kernels' 256-column tiles (the float32-ALU kernels, 64-column tiles, use fewer)
static inline int row_grad_parts(int f) { return (f + 255) / 256 * 4; }
static inline size_t row_part_bytes(int B, int f) {
    return align_up((size_t)row_grad_parts(f) * (size_t)(B > 0 ? B : 1) * sizeof(float), 256);
}

static inline size_t ffn_fwd_ws_bytes(int B, int E, int d, int f, int dt) {
    (void)d;
    return ffn_tilemap_bytes(B, E) + ffn_act_bytes(B, f, dt);                 // tile map | A = silu(G)*U
}
static inline size_t ffn_bwd_ws_bytes(int B, int E, int d, int f, int dt) {
    (void)d;
    return ffn_tilemap_bytes(B, E) + 3 * ffn_act_bytes(B, f, dt) + row_part_bytes(B, f);   // tile map | dG | dU | A | partials
}

// two-matrix expert: tile map | A = act(H)   and   tile map | dH | A
static inline size_t mlp2_fwd_ws_bytes(int B, int E, int d, int f, int dt) {
    (void)d;
    return ffn_tilemap_bytes(B, E) + ffn_act_bytes(B, f, dt);
}
static inline size_t mlp2_bwd_ws_bytes(int B, int E, int d, int f, int dt) {
    (void)d;
    return ffn_tilemap_bytes(B, E) + 2 * ffn_act_bytes(B, f, dt) + row_part_bytes(B, f);
}

// ----- stage 0 of the redundancy-bypassing dispatch: pilot flags, pilot row of every row, pilot prefix, chunk counts
static inline int rbd_num_chunks(long long B) { return (int)((B + 1023) / 1024); }
static inline size_t rbd_ws_bytes(int T, int k) {
    const long long B = (long long)T * k;
    return 2 * align_up((size_t)(B > 0 ? B : 1) * sizeof(int32_t), 256) + align_up((size_t)(B + 1) * sizeof(int32_t), 256) +
           align_up((size_t)(rbd_num_chunks(B) + 1) * sizeof(int32_t), 256);
}

// ----- gate projection backward: split-K partial sums of dWr -----
static inline int gate_bwd_splits(int T) {
    int s = (T + 255) / 256;
    return s < 1 ? 1 : (s > 32 ? 32 : s);
}
static inline size_t gate_bwd_ws_bytes(int T, int d, int E) {
    return align_up((size_t)gate_bwd_splits(T) * (size_t)d * (size_t)E * sizeof(float), 256);
}

}  // namespace xmoe
