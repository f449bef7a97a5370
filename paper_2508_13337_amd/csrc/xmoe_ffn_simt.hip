// Expert MLP over ragged segments (paper: Listing 1 mlp(); Appendix B.4 "Sequential GeMM"), float32-ALU version:
// serves float32 workloads and any shape the MFMA kernels do not take.  One launch covers every expert: a tile
// map built on the device says which expert and which rows each row tile belongs to, so there is no host
// round trip on tokens_per_expert and no per-expert launch.
#include "xmoe_ffn.h"
#include "xmoe_simt_gemm.h"

namespace xmoe {

// ---------------------------------------------------------------------------------------------------------
// tile map: header {total tiles, 0, 0, 0} then (expert, first row) per row tile; unused entries have expert -1.
// sched: the experts sorted by descending row count (ties: lower index first), then kSchedCounters zeroed counters
// (the weight-gradient kernels hand out their tiles longest first from these).
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void tile_map_kernel(const int32_t* __restrict__ off, int E, int tile_rows,
                                                       int max_tiles, int32_t* __restrict__ map,
                                                       int32_t* __restrict__ sched) {
    __shared__ int start[XMOE_MAX_EXPERTS + 1];
    __shared__ int count[XMOE_MAX_EXPERTS];
    const int e = threadIdx.x;
    int nt = 0, lo = 0, m = 0;
    if (e < E) {
        lo = off[e];
        m = off[e + 1] - lo;
        nt = m > 0 ? (m + tile_rows - 1) / tile_rows : 0;
        start[e] = nt;
        count[e] = m;
    }
    __syncthreads();
    if (e < E) {
        int rank = 0;
        for (int i = 0; i < E; ++i) {
            const int c = count[i];
            rank += (c > m || (c == m && i < e)) ? 1 : 0;
        }
        sched[rank] = e;
    }
    if (threadIdx.x < kSchedCounters) sched[E + threadIdx.x] = 0;
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < E; ++i) {
            int v = start[i];
            start[i] = run;
            run += v;
        }
        start[E] = run < max_tiles ? run : max_tiles;
        map[0] = start[E];
        map[1] = map[2] = map[3] = 0;
    }
    __syncthreads();
    if (e < E) {
        for (int i = 0; i < nt; ++i) {
            int ti = start[e] + i;
            if (ti < max_tiles) {
                map[4 + 2 * ti] = e;
                map[4 + 2 * ti + 1] = lo + i * tile_rows;
            }
        }
    }
    for (int ti = start[E] + threadIdx.x; ti < max_tiles; ti += 512) {
        map[4 + 2 * ti] = -1;
        map[4 + 2 * ti + 1] = 0;
    }
}

int launch_tile_map(const int32_t* off, int E, int tile_rows, int max_tiles, int32_t* map, int32_t* sched,
                    hipStream_t s) {
    XMOE_LAUNCH(K_TILE_MAP, s, hipLaunchKernelGGL(tile_map_kernel, dim3(1), dim3(512), 0, s, off, E, tile_rows,
                                                  max_tiles, map, sched));
    return XMOE_OK;
}

// row_grad[i] = sum_p row_part[p * B + i], p ascending
__global__ __launch_bounds__(256) void row_grad_reduce_kernel(const float* __restrict__ row_part, int parts, int B,
                                                              float* __restrict__ row_grad) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= B) return;
    float s = 0.f;
    for (int p = 0; p < parts; ++p) s += row_part[(size_t)p * B + i];
    row_grad[i] = s;
}

int launch_row_grad_reduce(const float* row_part, int parts, int B, float* row_grad, hipStream_t s) {
    if (B <= 0) return XMOE_OK;
    XMOE_LAUNCH(K_ROW_GRAD_REDUCE, s,
                hipLaunchKernelGGL(row_grad_reduce_kernel, dim3((B + 255) / 256), dim3(256), 0, s, row_part, parts, B,
                                   row_grad));
    return XMOE_OK;
}

// sum of v over the 16 threads that share a row patch (tx = 0..15: consecutive lanes), in a fixed order
__device__ __forceinline__ float sum_over_tx(float v) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---------------------------------------------------------------------------------------------------------
// forward 1: G = Xd Wg, U = Xd Wu, A = silu(G) * U          rows: ragged, K = d, N = f
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ffn_gateup_simt_kernel(const T* __restrict__ xd,
                                                              const int32_t* __restrict__ row_index,   // or NULL
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ map, int d, int f,
                                                              const T* __restrict__ wg, const T* __restrict__ wu,
                                                              T* __restrict__ G, T* __restrict__ U,
                                                              T* __restrict__ A) {
    __shared__ SimtSmem sm;
    const int e = map[4 + 2 * blockIdx.x];
    if (e < 0) return;
    const int row0 = map[4 + 2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int n0 = blockIdx.y * kSimtTile;
    const T* wge = wg + (size_t)e * d * f;
    const T* wue = wu + (size_t)e * d * f;
    auto loadA = [&](int mm, int kk) {
        int r = row0 + mm;
        if (r >= row_end) return 0.f;
        if (row_index) r = row_index[r];   // gather fused: row r of the expert input is row row_index[r] of xd
        return to_float(xd[(size_t)r * d + kk]);
    };
    float accg[4][4] = {}, accu[4][4] = {};
    simt_mainloop<true, true>(accg, d, sm, loadA,
                              [&](int kk, int nn) { int n = n0 + nn; return n < f ? to_float(wge[(size_t)kk * f + n]) : 0.f; });
    simt_mainloop<true, true>(accu, d, sm, loadA,
                              [&](int kk, int nn) { int n = n0 + nn; return n < f ? to_float(wue[(size_t)kk * f + n]) : 0.f; });
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int r = row0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (r < row_end && n < f) {
                float g = accg[i][j], u = accu[i][j];
                G[(size_t)r * f + n] = from_float<T>(g);
                U[(size_t)r * f + n] = from_float<T>(u);
                A[(size_t)r * f + n] = from_float<T>(siluf_(g) * u);
            }
        }
}

// ---------------------------------------------------------------------------------------------------------
// forward 2: Y = A Wd                                       rows: ragged, K = f, N = d
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ffn_down_simt_kernel(const T* __restrict__ A, const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ map, int d, int f,
                                                            const T* __restrict__ wd, T* __restrict__ Y) {
    __shared__ SimtSmem sm;
    const int e = map[4 + 2 * blockIdx.x];
    if (e < 0) return;
    const int row0 = map[4 + 2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int n0 = blockIdx.y * kSimtTile;
    const T* wde = wd + (size_t)e * f * d;
    float acc[4][4] = {};
    simt_mainloop<true, true>(
        acc, f, sm, [&](int mm, int kk) { int r = row0 + mm; return r < row_end ? to_float(A[(size_t)r * f + kk]) : 0.f; },
        [&](int kk, int nn) { int n = n0 + nn; return n < d ? to_float(wde[(size_t)kk * d + n]) : 0.f; });
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int r = row0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (r < row_end && n < d) Y[(size_t)r * d + n] = from_float<T>(acc[i][j]);
        }
}

// ---------------------------------------------------------------------------------------------------------
// backward 1: dA = dY Wd^T, then dG = dA * U * silu'(G), dU = dA * silu(G), A = silu(G) * U
//                                                            rows: ragged, K = d, N = f
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ffn_dact_simt_kernel(const T* __restrict__ dY,
                                                            const int32_t* __restrict__ dy_index,   // or NULL
                                                            const float* __restrict__ dy_scale,     // or NULL
                                                            const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ map, int d, int f,
                                                            const T* __restrict__ wd, const T* __restrict__ G,
                                                            const T* __restrict__ U, T* __restrict__ dG,
                                                            T* __restrict__ dU, T* __restrict__ A,
                                                            float* __restrict__ row_part, int B) {
    __shared__ SimtSmem sm;
    const int e = map[4 + 2 * blockIdx.x];
    if (e < 0) return;
    const int row0 = map[4 + 2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int n0 = blockIdx.y * kSimtTile;
    const T* wde = wd + (size_t)e * f * d;
    float acc[4][4] = {};
    simt_mainloop<true, false>(
        acc, d, sm,
        [&](int mm, int kk) {
            int r = row0 + mm;
            if (r >= row_end) return 0.f;
            if (dy_index) r = dy_index[r];   // row r of dY is dy_scale[r] * dY[dy_index[r]]; the scale follows below
            return to_float(dY[(size_t)r * d + kk]);
        },
        [&](int kk, int nn) { int n = n0 + nn; return n < f ? to_float(wde[(size_t)n * d + kk]) : 0.f; });
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float part = 0.f;   // <unscaled dY row, Y row> over this thread's columns (the gradient of the row's scale)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int r = row0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (r < row_end && n < f) {
                size_t ix = (size_t)r * f + n;
                const float sc = (dy_index && dy_scale) ? dy_scale[r] : 1.0f;
                float g = to_float(G[ix]), u = to_float(U[ix]), da = acc[i][j] * sc;
                float sg = sigmoidf_(g);
                float sl = g * sg;
                dG[ix] = from_float<T>(da * u * (sg * (1.0f + g * (1.0f - sg))));
                dU[ix] = from_float<T>(da * sl);
                A[ix] = from_float<T>(sl * u * sc);   // scaled: the weight gradient multiplies it with unscaled rows
                part = fmaf(acc[i][j], sl * u, part);
            }
        }
        if (row_part) {   // block-uniform
            part = sum_over_tx(part);
            const int r = row0 + ty * 4 + i;
            if (tx == 0 && r < row_end) row_part[(size_t)blockIdx.y * B + r] = part;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// backward 2: dXd = dG Wg^T + dU Wu^T                        rows: ragged, K = f (twice), N = d
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ffn_dx_simt_kernel(const T* __restrict__ dG, const T* __restrict__ dU,
                                                          const int32_t* __restrict__ off,
                                                          const int32_t* __restrict__ map, int d, int f,
                                                          const T* __restrict__ wg, const T* __restrict__ wu,
                                                          T* __restrict__ dXd) {
    __shared__ SimtSmem sm;
    const int e = map[4 + 2 * blockIdx.x];
    if (e < 0) return;
    const int row0 = map[4 + 2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int n0 = blockIdx.y * kSimtTile;
    const T* wge = wg + (size_t)e * d * f;
    const T* wue = wu + (size_t)e * d * f;
    float acc[4][4] = {};
    simt_mainloop<true, false>(
        acc, f, sm, [&](int mm, int kk) { int r = row0 + mm; return r < row_end ? to_float(dG[(size_t)r * f + kk]) : 0.f; },
        [&](int kk, int nn) { int n = n0 + nn; return n < d ? to_float(wge[(size_t)n * f + kk]) : 0.f; });
    if (dU)   // the two-matrix expert has a single pair (dH, W1)
        simt_mainloop<true, false>(
            acc, f, sm, [&](int mm, int kk) { int r = row0 + mm; return r < row_end ? to_float(dU[(size_t)r * f + kk]) : 0.f; },
            [&](int kk, int nn) { int n = n0 + nn; return n < d ? to_float(wue[(size_t)n * f + kk]) : 0.f; });
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int r = row0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (r < row_end && n < d) dXd[(size_t)r * d + n] = from_float<T>(acc[i][j]);
        }
}

// ---------------------------------------------------------------------------------------------------------
// weight gradients: dW_e[m,n] = sum over the expert's rows r of P[r,m] * Q[r,n]   (K = ragged)
//   dWd = A^T dY (M=f, N=d);  dWg = Xd^T dG, dWu = Xd^T dU (M=d, N=f).  Empty experts get zeros.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ffn_wgrad_simt_kernel(const T* __restrict__ P,
                                                             const int32_t* __restrict__ row_index,   // of P, or NULL
                                                             const T* __restrict__ Q,
                                                             const int32_t* __restrict__ q_index,     // of Q, or NULL
                                                             const int32_t* __restrict__ off, int M, int N,
                                                             T* __restrict__ dW) {
    __shared__ SimtSmem sm;
    const int e = blockIdx.z;
    const int lo = off[e], hi = off[e + 1];
    const int m0 = blockIdx.x * kSimtTile, n0 = blockIdx.y * kSimtTile;
    float acc[4][4] = {};
    simt_mainloop<false, true>(
        acc, hi - lo, sm,
        [&](int mm, int kk) {
            int m = m0 + mm;
            if (m >= M) return 0.f;
            const int r = row_index ? row_index[lo + kk] : lo + kk;
            return to_float(P[(size_t)r * M + m]);
        },
        [&](int kk, int nn) {
            int n = n0 + nn;
            if (n >= N) return 0.f;
            const int r = q_index ? q_index[lo + kk] : lo + kk;
            return to_float(Q[(size_t)r * N + n]);
        });
    T* out = dW + (size_t)e * M * N;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) out[(size_t)m * N + n] = from_float<T>(acc[i][j]);
        }
}

// ---------------------------------------------------------------------------------------------------------
// two-matrix expert, forward 1: H = Xd W1, A = act(H)         rows: ragged, K = d, N = f
// ---------------------------------------------------------------------------------------------------------
template <typename T, int ACT>
__global__ __launch_bounds__(256) void mlp2_up_simt_kernel(const T* __restrict__ xd,
                                                           const int32_t* __restrict__ row_index,   // or NULL
                                                           const int32_t* __restrict__ off,
                                                           const int32_t* __restrict__ map, int d, int f,
                                                           const T* __restrict__ w1, T* __restrict__ H,
                                                           T* __restrict__ A) {
    __shared__ SimtSmem sm;
    const int e = map[4 + 2 * blockIdx.x];
    if (e < 0) return;
    const int row0 = map[4 + 2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int n0 = blockIdx.y * kSimtTile;
    const T* w1e = w1 + (size_t)e * d * f;
    float acc[4][4] = {};
    simt_mainloop<true, true>(
        acc, d, sm,
        [&](int mm, int kk) {
            int r = row0 + mm;
            if (r >= row_end) return 0.f;
            if (row_index) r = row_index[r];
            return to_float(xd[(size_t)r * d + kk]);
        },
        [&](int kk, int nn) { int n = n0 + nn; return n < f ? to_float(w1e[(size_t)kk * f + n]) : 0.f; });
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int r = row0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (r < row_end && n < f) {
                H[(size_t)r * f + n] = from_float<T>(acc[i][j]);
                A[(size_t)r * f + n] = from_float<T>(act_fwd<ACT>(acc[i][j]));
            }
        }
}

// ---------------------------------------------------------------------------------------------------------
// two-matrix expert, backward 1: dA = dY W2^T, then dH = dA * act'(H), A = act(H)     K = d, N = f
// ---------------------------------------------------------------------------------------------------------
template <typename T, int ACT>
__global__ __launch_bounds__(256) void mlp2_dact_simt_kernel(const T* __restrict__ dY,
                                                             const int32_t* __restrict__ dy_index,   // or NULL
                                                             const float* __restrict__ dy_scale,     // or NULL
                                                             const int32_t* __restrict__ off,
                                                             const int32_t* __restrict__ map, int d, int f,
                                                             const T* __restrict__ w2, const T* __restrict__ H,
                                                             T* __restrict__ dH, T* __restrict__ A,
                                                             float* __restrict__ row_part, int B) {
    __shared__ SimtSmem sm;
    const int e = map[4 + 2 * blockIdx.x];
    if (e < 0) return;
    const int row0 = map[4 + 2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int n0 = blockIdx.y * kSimtTile;
    const T* w2e = w2 + (size_t)e * f * d;
    float acc[4][4] = {};
    simt_mainloop<true, false>(
        acc, d, sm,
        [&](int mm, int kk) {
            int r = row0 + mm;
            if (r >= row_end) return 0.f;
            if (dy_index) r = dy_index[r];
            return to_float(dY[(size_t)r * d + kk]);
        },
        [&](int kk, int nn) { int n = n0 + nn; return n < f ? to_float(w2e[(size_t)n * d + kk]) : 0.f; });
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float part = 0.f;   // as in ffn_dact_simt_kernel
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int r = row0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (r < row_end && n < f) {
                const size_t ix = (size_t)r * f + n;
                float a, g;
                act_fwd_grad<ACT>(to_float(H[ix]), a, g);
                const float sc = (dy_index && dy_scale) ? dy_scale[r] : 1.0f;
                dH[ix] = from_float<T>(acc[i][j] * sc * g);
                A[ix] = from_float<T>(a * sc);
                part = fmaf(acc[i][j], a, part);
            }
        }
        if (row_part) {
            part = sum_over_tx(part);
            const int r = row0 + ty * 4 + i;
            if (tx == 0 && r < row_end) row_part[(size_t)blockIdx.y * B + r] = part;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// host-side drivers
// ---------------------------------------------------------------------------------------------------------
template <typename T>
static int fwd_simt(const FfnArgs& a, hipStream_t s) {
    const int max_tiles = ffn_max_tiles(a.B, a.E, kSimtTile);
    int st = launch_tile_map(a.off, a.E, kSimtTile, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    dim3 g1(max_tiles, (a.f + kSimtTile - 1) / kSimtTile), g2(max_tiles, (a.d + kSimtTile - 1) / kSimtTile);
    XMOE_LAUNCH(K_FFN_GATEUP_SIMT, s,
                hipLaunchKernelGGL(ffn_gateup_simt_kernel<T>, g1, dim3(256), 0, s, (const T*)a.xd, a.row_index, a.off,
                                   a.map, a.d,
                                   a.f, (const T*)a.wg, (const T*)a.wu, (T*)a.g, (T*)a.u, (T*)a.act));
    XMOE_LAUNCH(K_FFN_DOWN_SIMT, s,
                hipLaunchKernelGGL(ffn_down_simt_kernel<T>, g2, dim3(256), 0, s, (const T*)a.act, a.off, a.map, a.d,
                                   a.f, (const T*)a.wd, (T*)a.y));
    return XMOE_OK;
}

template <typename T>
static int bwd_simt(const FfnArgs& a, hipStream_t s) {
    const int max_tiles = ffn_max_tiles(a.B, a.E, kSimtTile);
    int st = launch_tile_map(a.off, a.E, kSimtTile, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const int tf = (a.f + kSimtTile - 1) / kSimtTile, td = (a.d + kSimtTile - 1) / kSimtTile;
    XMOE_LAUNCH(K_FFN_DACT_SIMT, s,
                hipLaunchKernelGGL(ffn_dact_simt_kernel<T>, dim3(max_tiles, tf), dim3(256), 0, s, (const T*)a.dy,
                                   a.dy_index, a.dy_scale, a.off, a.map, a.d, a.f, (const T*)a.wd, (const T*)a.g, (const T*)a.u, (T*)a.dg, (T*)a.du,
                                   (T*)a.act, a.row_part, a.B));
    if (a.row_grad) {
        st = launch_row_grad_reduce(a.row_part, tf, a.B, a.row_grad, s);
        if (st != XMOE_OK) return st;
    }
    XMOE_LAUNCH(K_FFN_DX_SIMT, s,
                hipLaunchKernelGGL(ffn_dx_simt_kernel<T>, dim3(max_tiles, td), dim3(256), 0, s, (const T*)a.dg,
                                   (const T*)a.du, a.off, a.map, a.d, a.f, (const T*)a.wg, (const T*)a.wu, (T*)a.dxd));
    XMOE_LAUNCH(K_FFN_WGRAD_SIMT, s,
                hipLaunchKernelGGL(ffn_wgrad_simt_kernel<T>, dim3(tf, td, a.E), dim3(256), 0, s, (const T*)a.act,
                                   nullptr, (const T*)a.dy, a.dy_index, a.off, a.f, a.d, (T*)a.dwd));
    XMOE_LAUNCH(K_FFN_WGRAD_SIMT, s,
                hipLaunchKernelGGL(ffn_wgrad_simt_kernel<T>, dim3(td, tf, a.E), dim3(256), 0, s, (const T*)a.xd,
                                   a.row_index, (const T*)a.dg, nullptr, a.off, a.d, a.f, (T*)a.dwg));
    XMOE_LAUNCH(K_FFN_WGRAD_SIMT, s,
                hipLaunchKernelGGL(ffn_wgrad_simt_kernel<T>, dim3(td, tf, a.E), dim3(256), 0, s, (const T*)a.xd,
                                   a.row_index, (const T*)a.du, nullptr, a.off, a.d, a.f, (T*)a.dwu));
    return XMOE_OK;
}

template <typename T>
static int mlp2_fwd_simt_t(const Mlp2Args& a, hipStream_t s) {
    const int max_tiles = ffn_max_tiles(a.B, a.E, kSimtTile);
    int st = launch_tile_map(a.off, a.E, kSimtTile, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    dim3 g1(max_tiles, (a.f + kSimtTile - 1) / kSimtTile), g2(max_tiles, (a.d + kSimtTile - 1) / kSimtTile);
#define XMOE_CALL(ACT)                                                                                              \
    XMOE_LAUNCH(K_MLP2_UP_SIMT, s,                                                                                  \
                hipLaunchKernelGGL((mlp2_up_simt_kernel<T, ACT>), g1, dim3(256), 0, s, (const T*)a.xd, a.row_index, \
                                   a.off, a.map, a.d, a.f, (const T*)a.w1, (T*)a.h, (T*)a.a_buf))
    XMOE_DISPATCH_ACT(a.act, XMOE_CALL);
#undef XMOE_CALL
    XMOE_LAUNCH(K_FFN_DOWN_SIMT, s,
                hipLaunchKernelGGL(ffn_down_simt_kernel<T>, g2, dim3(256), 0, s, (const T*)a.a_buf, a.off, a.map, a.d,
                                   a.f, (const T*)a.w2, (T*)a.y));
    return XMOE_OK;
}

template <typename T>
static int mlp2_bwd_simt_t(const Mlp2Args& a, hipStream_t s) {
    const int max_tiles = ffn_max_tiles(a.B, a.E, kSimtTile);
    int st = launch_tile_map(a.off, a.E, kSimtTile, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const int tf = (a.f + kSimtTile - 1) / kSimtTile, td = (a.d + kSimtTile - 1) / kSimtTile;
#define XMOE_CALL(ACT)                                                                                          \
    XMOE_LAUNCH(K_MLP2_DACT_SIMT, s,                                                                            \
                hipLaunchKernelGGL((mlp2_dact_simt_kernel<T, ACT>), dim3(max_tiles, tf), dim3(256), 0, s,       \
                                   (const T*)a.dy, a.dy_index, a.dy_scale, a.off, a.map, a.d, a.f,              \
                                   (const T*)a.w2, (const T*)a.h, (T*)a.dh, (T*)a.a_buf, a.row_part, a.B))
    XMOE_DISPATCH_ACT(a.act, XMOE_CALL);
#undef XMOE_CALL
    if (a.row_grad) {
        st = launch_row_grad_reduce(a.row_part, tf, a.B, a.row_grad, s);
        if (st != XMOE_OK) return st;
    }
    XMOE_LAUNCH(K_FFN_DX_SIMT, s,
                hipLaunchKernelGGL(ffn_dx_simt_kernel<T>, dim3(max_tiles, td), dim3(256), 0, s, (const T*)a.dh,
                                   (const T*)nullptr, a.off, a.map, a.d, a.f, (const T*)a.w1, (const T*)nullptr,
                                   (T*)a.dxd));
    XMOE_LAUNCH(K_FFN_WGRAD_SIMT, s,
                hipLaunchKernelGGL(ffn_wgrad_simt_kernel<T>, dim3(tf, td, a.E), dim3(256), 0, s, (const T*)a.a_buf,
                                   nullptr, (const T*)a.dy, a.dy_index, a.off, a.f, a.d, (T*)a.dw2));
    XMOE_LAUNCH(K_FFN_WGRAD_SIMT, s,
                hipLaunchKernelGGL(ffn_wgrad_simt_kernel<T>, dim3(td, tf, a.E), dim3(256), 0, s, (const T*)a.xd,
                                   a.row_index, (const T*)a.dh, nullptr, a.off, a.d, a.f, (T*)a.dw1));
    return XMOE_OK;
}

int mlp2_fwd_simt(const Mlp2Args& a, hipStream_t s) {
    return a.dt == XMOE_F32 ? mlp2_fwd_simt_t<float>(a, s) : mlp2_fwd_simt_t<bf16_t>(a, s);
}
int mlp2_bwd_simt(const Mlp2Args& a, hipStream_t s) {
    return a.dt == XMOE_F32 ? mlp2_bwd_simt_t<float>(a, s) : mlp2_bwd_simt_t<bf16_t>(a, s);
}

int ffn_fwd_simt(const FfnArgs& a, hipStream_t s) {
    return a.dt == XMOE_F32 ? fwd_simt<float>(a, s) : fwd_simt<bf16_t>(a, s);
}
int ffn_bwd_simt(const FfnArgs& a, hipStream_t s) {
    return a.dt == XMOE_F32 ? bwd_simt<float>(a, s) : bwd_simt<bf16_t>(a, s);
}

}  // namespace xmoe
