// Expert MLP over ragged segments (paper: Listing 1 mlp(); Appendix B.4 "Sequential GeMM") on the gfx950 matrix
// cores: one ragged grouped GEMM per stage instead of a host loop of per-expert GEMMs.
//
//   block = 256 threads = 4 waves (2 x 2), block tile 128 x 128, K stepped by 64 through double-buffered LDS,
//   wave tile 64 x 64 = 2 x 2 tiles of v_mfma_f32_32x32x16_bf16 (float32 accumulators).
//
// Operand tiles live in LDS as [128 rows][64 k] bf16 (128 bytes per row, 16-byte chunks XOR-swizzled by row so
// that fragment reads, row stores and transposing stores all spread over the banks).  An operand whose K index
// is contiguous in memory is copied row by row; an operand whose K index is the strided one (weights stored
// "in x out", and both operands of the weight-gradient GEMMs) is read with 16-byte loads along its contiguous
// index and transposed in registers (4 k x 8 n per thread) on its way into LDS.
//
// Row tiles never cross an expert boundary: a device-built tile map gives each 128-row tile its expert and first
// row, tail rows are zero-filled in LDS and masked on store, so no padded row ever exists in HBM.
// Workgroups are renumbered so that each XCD (they receive workgroups round-robin) works on a contiguous run of
// tiles and re-uses operand panels from its own L2.
#include "xmoe_ffn.h"

namespace xmoe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kTileBytes = 128 * BK * 2;   // one operand tile: 16 KiB
constexpr int kNumXcd = 8;

// byte offset of 16-byte chunk c (0..7) of row r inside a tile
__device__ __forceinline__ int lds_off(int r, int c) { return r * 128 + (((c ^ r ^ (r >> 3)) & 7) << 4); }

// A 128-row operand tile as two 64-row halves (so that two matrices can feed one tile).
//   row mode (K contiguous):  element (row, k)  at p + row * ld + k;   n_* = valid rows of the half
//   col mode (K strided):     element (k, col)  at p + k * ld + col;   n_* = valid columns of the half (multiple of 8)
struct Src {
    const bf16_t* p_lo;
    const bf16_t* p_hi;
    long ld;
    int n_lo, n_hi;
    int k_valid;   // col mode only: k >= k_valid reads as zero
};

template <bool COL>
__device__ __forceinline__ void tile_load(const Src& s, int k0, uint4 (&r)[4]) {
    const int tid = threadIdx.x;
    if (!COL) {
        const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = r0 + 32 * i;               // i < 2: low half, i >= 2: high half
            const bf16_t* p = (i < 2) ? s.p_lo : s.p_hi;
            const int rr = row & 63;
            const int nv = (i < 2) ? s.n_lo : s.n_hi;
            r[i] = make_uint4(0, 0, 0, 0);
            if (rr < nv) r[i] = *reinterpret_cast<const uint4*>(p + (long)rr * s.ld + k0 + c * 8);
        }
    } else {
        const int g = tid & 15, kq = tid >> 4;
        const int half = g >> 3, col = (g & 7) * 8;
        const bf16_t* p = half ? s.p_hi : s.p_lo;
        const int nv = half ? s.n_hi : s.n_lo;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + 4 * kq + i;
            r[i] = make_uint4(0, 0, 0, 0);
            if (col < nv && kk < s.k_valid) r[i] = *reinterpret_cast<const uint4*>(p + (long)kk * s.ld + col);
        }
    }
}

template <bool COL>
__device__ __forceinline__ void tile_store(char* lds, const uint4 (&r)[4]) {
    const int tid = threadIdx.x;
    if (!COL) {
        const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(lds + lds_off(r0 + 32 * i, c)) = r[i];
    } else {
        // r[i] holds k = 4*kq + i for 8 consecutive columns; column j becomes LDS row n with 4 consecutive k
        const int g = tid & 15, kq = tid >> 4;
        const int n0 = g * 8;
        const uint32_t w[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w}, {r[1].x, r[1].y, r[1].z, r[1].w},
                                  {r[2].x, r[2].y, r[2].z, r[2].w}, {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int q = j >> 1;
            uint32_t lo, hi;
            if ((j & 1) == 0) {
                lo = (w[0][q] & 0xffffu) | (w[1][q] << 16);
                hi = (w[2][q] & 0xffffu) | (w[3][q] << 16);
            } else {
                lo = (w[0][q] >> 16) | (w[1][q] & 0xffff0000u);
                hi = (w[2][q] >> 16) | (w[3][q] & 0xffff0000u);
            }
            *reinterpret_cast<uint2*>(lds + lds_off(n0 + j, kq >> 1) + (kq & 1) * 8) = make_uint2(lo, hi);
        }
    }
}

// B fragment rows: plain tiles put wave column wn at rows wn*64 + ni*32; the gate/up tile keeps the gate
// columns in rows 0..63 and the up columns in rows 64..127, and a wave takes the same 32 columns of both.
template <bool GU>
__device__ __forceinline__ int b_row(int wn, int ni) { return GU ? ni * 64 + wn * 32 : wn * 64 + ni * 32; }

template <bool GU>
__device__ __forceinline__ void tile_mma(f32x16_t (&acc)[2][2], const char* la, const char* lb) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8_t a[2], b[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
            a[mi] = *reinterpret_cast<const bf16x8_t*>(la + lds_off(wm * 64 + mi * 32 + lr, 2 * ks + lk));
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
            b[ni] = *reinterpret_cast<const bf16x8_t*>(lb + lds_off(b_row<GU>(wn, ni) + lr, 2 * ks + lk));
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
}

// acc += A_tile x B_tile over K (K > 0; a multiple of 64 unless the operands are in col mode with k_valid = K)
template <bool A_COL, bool B_COL, bool GU>
__device__ __forceinline__ void mainloop(f32x16_t (&acc)[2][2], const Src& a, const Src& b, int K, char* smem) {
    const int nk = (K + BK - 1) / BK;
    if (nk <= 0) return;
    uint4 ra[4], rb[4];
    tile_load<A_COL>(a, 0, ra);
    tile_load<B_COL>(b, 0, rb);
    tile_store<A_COL>(smem, ra);
    tile_store<B_COL>(smem + kTileBytes, rb);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        char* cur = smem + (kt & 1) * 2 * kTileBytes;
        char* nxt = smem + ((kt + 1) & 1) * 2 * kTileBytes;
        const bool more = kt + 1 < nk;
        if (more) {
            tile_load<A_COL>(a, (kt + 1) * BK, ra);
            tile_load<B_COL>(b, (kt + 1) * BK, rb);
        }
        tile_mma<GU>(acc, cur, cur + kTileBytes);
        if (more) {
            tile_store<A_COL>(nxt, ra);
            tile_store<B_COL>(nxt + kTileBytes, rb);
        }
        __syncthreads();
    }
}

__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[2][2]) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
}

// row (inside the 128-row tile) of accumulator element v of m-tile mi
__device__ __forceinline__ int acc_row(int mi, int v) {
    const int lane = threadIdx.x & 63, wm = threadIdx.x >> 7;
    return wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

// Each XCD gets a contiguous run of the `total` logical tiles.  Returns -1 for a workgroup with nothing to do.
__device__ __forceinline__ int xcd_tile(int total) {
    const int b = blockIdx.x;
    const int chunk = (total + kNumXcd - 1) / kNumXcd;
    const int within = b / kNumXcd;
    const int t = (b % kNumXcd) * chunk + within;
    return (within < chunk && t < total) ? t : -1;
}

struct RowTile {
    int e, row0, rows;   // expert, first row, valid rows (1..128)
};
__device__ __forceinline__ RowTile get_row_tile(const int32_t* __restrict__ map, const int32_t* __restrict__ off,
                                                int mt) {
    RowTile t;
    t.e = map[4 + 2 * mt];
    t.row0 = map[4 + 2 * mt + 1];
    int r = off[t.e + 1] - t.row0;
    t.rows = r < BM ? r : BM;
    return t;
}

__device__ __forceinline__ Src row_src(const bf16_t* p, long ld, int rows) {
    Src s;
    s.p_lo = p;
    s.p_hi = p + 64 * ld;
    s.ld = ld;
    s.n_lo = rows < 64 ? rows : 64;
    s.n_hi = rows > 64 ? rows - 64 : 0;
    s.k_valid = 0;
    return s;
}
__device__ __forceinline__ Src col_src(const bf16_t* p, long ld, int cols, int k_valid) {
    Src s;
    s.p_lo = p;
    s.p_hi = p + 64;
    s.ld = ld;
    s.n_lo = cols < 64 ? cols : 64;
    s.n_hi = cols > 64 ? cols - 64 : 0;
    s.k_valid = k_valid;
    return s;
}

__device__ __forceinline__ void store_bf16(bf16_t* p, float v) { p->bits = float_to_bf16_bits(v); }

}  // namespace

// =========================================================================================================
// forward 1: G = Xd Wg, U = Xd Wu, A = silu(G) * U.   Block tile: 128 rows x (64 gate + 64 up columns).
// =========================================================================================================
__global__ __launch_bounds__(256) void ffn_gateup_mfma_kernel(const bf16_t* __restrict__ xd,
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ map, int d, int f,
                                                              const bf16_t* __restrict__ wg,
                                                              const bf16_t* __restrict__ wu, bf16_t* __restrict__ G,
                                                              bf16_t* __restrict__ U, bf16_t* __restrict__ A) {
    __shared__ __align__(16) char smem[4 * kTileBytes];
    const int nt = f / 64;
    const int t = xcd_tile(map[0] * nt);
    if (t < 0) return;
    const RowTile rt = get_row_tile(map, off, t / nt);
    const int n0 = (t % nt) * 64;
    Src a = row_src(xd + (long)rt.row0 * d, d, rt.rows);
    Src b;
    b.p_lo = wg + (long)rt.e * d * f + n0;
    b.p_hi = wu + (long)rt.e * d * f + n0;
    b.ld = f;
    b.n_lo = b.n_hi = 64;
    b.k_valid = d;
    f32x16_t acc[2][2];
    zero_acc(acc);
    mainloop<false, true, true>(acc, a, b, d, smem);
    const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) & 1;
    const int col = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = acc_row(mi, v);
            if (r < rt.rows) {
                const long ix = (long)(rt.row0 + r) * f + col;
                const float g = acc[mi][0][v], u = acc[mi][1][v];
                store_bf16(G + ix, g);
                store_bf16(U + ix, u);
                store_bf16(A + ix, siluf_(g) * u);
            }
        }
}

// =========================================================================================================
// forward 2: Y = A Wd          (K = f, N = d, weights "in x out" -> transposing loads)
// backward 1: dA = dY Wd^T     (K = d, N = f, weights K-contiguous) + dG, dU, A in the epilogue
// =========================================================================================================
template <bool DACT>
__global__ __launch_bounds__(256) void ffn_rowgemm_mfma_kernel(const bf16_t* __restrict__ X,
                                                               const int32_t* __restrict__ off,
                                                               const int32_t* __restrict__ map, int K, int N,
                                                               const bf16_t* __restrict__ W, bf16_t* __restrict__ Y,
                                                               const bf16_t* __restrict__ G,
                                                               const bf16_t* __restrict__ U, bf16_t* __restrict__ dG,
                                                               bf16_t* __restrict__ dU, bf16_t* __restrict__ A) {
    __shared__ __align__(16) char smem[4 * kTileBytes];
    const int nt = (N + BN - 1) / BN;
    const int t = xcd_tile(map[0] * nt);
    if (t < 0) return;
    const RowTile rt = get_row_tile(map, off, t / nt);
    const int n0 = (t % nt) * BN;
    const int ncols = N - n0 < BN ? N - n0 : BN;
    Src a = row_src(X + (long)rt.row0 * K, K, rt.rows);
    const bf16_t* We = W + (long)rt.e * K * N;
    f32x16_t acc[2][2];
    zero_acc(acc);
    if (DACT) {
        // W is [N=f, K=d] per expert here (Wd stored [f, d]): rows of W are the output columns, K contiguous
        Src b = row_src(We + (long)n0 * K, K, ncols);
        mainloop<false, false, false>(acc, a, b, K, smem);
    } else {
        // W is [K=f, N=d] per expert: output columns contiguous
        Src b = col_src(We + n0, N, ncols, K);
        mainloop<false, true, false>(acc, a, b, K, smem);
    }
    const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) & 1;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int c = wn * 64 + ni * 32 + (lane & 31);
            if (c >= ncols) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row(mi, v);
                if (r < rt.rows) {
                    const long ix = (long)(rt.row0 + r) * N + n0 + c;
                    if (DACT) {
                        const float g = to_float(G[ix]), u = to_float(U[ix]), da = acc[mi][ni][v];
                        const float sg = sigmoidf_(g);
                        const float sl = g * sg;
                        store_bf16(dG + ix, da * u * (sg * (1.0f + g * (1.0f - sg))));
                        store_bf16(dU + ix, da * sl);
                        store_bf16(A + ix, sl * u);
                    } else {
                        store_bf16(Y + ix, acc[mi][ni][v]);
                    }
                }
            }
        }
}

// =========================================================================================================
// backward 2: dXd = dG Wg^T + dU Wu^T     (K = f twice, N = d; Wg, Wu [d, f]: rows are output columns)
// =========================================================================================================
__global__ __launch_bounds__(256) void ffn_dx_mfma_kernel(const bf16_t* __restrict__ dG, const bf16_t* __restrict__ dU,
                                                          const int32_t* __restrict__ off,
                                                          const int32_t* __restrict__ map, int d, int f,
                                                          const bf16_t* __restrict__ wg,
                                                          const bf16_t* __restrict__ wu, bf16_t* __restrict__ dXd) {
    __shared__ __align__(16) char smem[4 * kTileBytes];
    const int nt = (d + BN - 1) / BN;
    const int t = xcd_tile(map[0] * nt);
    if (t < 0) return;
    const RowTile rt = get_row_tile(map, off, t / nt);
    const int n0 = (t % nt) * BN;
    const int ncols = d - n0 < BN ? d - n0 : BN;
    f32x16_t acc[2][2];
    zero_acc(acc);
    {
        Src a = row_src(dG + (long)rt.row0 * f, f, rt.rows);
        Src b = row_src(wg + (long)rt.e * d * f + (long)n0 * f, f, ncols);
        mainloop<false, false, false>(acc, a, b, f, smem);
    }
    {
        Src a = row_src(dU + (long)rt.row0 * f, f, rt.rows);
        Src b = row_src(wu + (long)rt.e * d * f + (long)n0 * f, f, ncols);
        mainloop<false, false, false>(acc, a, b, f, smem);
    }
    const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) & 1;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int c = wn * 64 + ni * 32 + (lane & 31);
            if (c >= ncols) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row(mi, v);
                if (r < rt.rows) store_bf16(dXd + (long)(rt.row0 + r) * d + n0 + c, acc[mi][ni][v]);
            }
        }
}

// =========================================================================================================
// weight gradients: dW_e[m, n] = sum over the expert's rows r of P[r, m] * Q[r, n]   (K = ragged row count;
// both operands are strided in K -> both transposed on load).  An expert with no rows gets zeros.
// =========================================================================================================
__global__ __launch_bounds__(256) void ffn_wgrad_mfma_kernel(const bf16_t* __restrict__ P, const bf16_t* __restrict__ Q,
                                                             const int32_t* __restrict__ off, int E, int M, int N,
                                                             bf16_t* __restrict__ dW) {
    __shared__ __align__(16) char smem[4 * kTileBytes];
    const int mt = (M + BM - 1) / BM, nt = (N + BN - 1) / BN;
    const int t = xcd_tile(E * mt * nt);
    if (t < 0) return;
    const int e = t / (mt * nt);
    const int m0 = ((t / nt) % mt) * BM, n0 = (t % nt) * BN;
    const int lo = off[e], hi = off[e + 1];
    const int K = hi - lo;
    const int mrows = M - m0 < BM ? M - m0 : BM, ncols = N - n0 < BN ? N - n0 : BN;
    f32x16_t acc[2][2];
    zero_acc(acc);
    if (K > 0) {
        Src a = col_src(P + (long)lo * M + m0, M, mrows, K);
        Src b = col_src(Q + (long)lo * N + n0, N, ncols, K);
        mainloop<true, true, false>(acc, a, b, K, smem);
    }
    bf16_t* out = dW + (long)e * M * N;
    const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) & 1;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int c = wn * 64 + ni * 32 + (lane & 31);
            if (c >= ncols) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row(mi, v);
                if (r < mrows) store_bf16(out + (long)(m0 + r) * N + n0 + c, acc[mi][ni][v]);
            }
        }
}

// =========================================================================================================
// host side
// =========================================================================================================
bool ffn_mfma_supported(const FfnArgs& a) {
    if (a.dt != XMOE_BF16) return false;
    if (a.d % 64 != 0 || a.f % 64 != 0) return false;
    const void* ptrs[] = {a.xd, a.wg, a.wu, a.wd, a.g, a.u, a.y, a.dy, a.dxd, a.dwg, a.dwu, a.dwd, a.act, a.dg, a.du};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return false;
    return true;
}

static inline unsigned round_up8(long v) { return (unsigned)((v + 7) / 8 * 8); }

int ffn_fwd_mfma(const FfnArgs& a, hipStream_t s) {
    const int max_tiles = ffn_max_tiles(a.B, a.E, BM);
    int st = launch_tile_map(a.off, a.E, BM, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const bf16_t *xd = (const bf16_t*)a.xd, *wg = (const bf16_t*)a.wg, *wu = (const bf16_t*)a.wu,
                 *wd = (const bf16_t*)a.wd;
    XMOE_LAUNCH(K_FFN_GATEUP_MFMA, s,
                hipLaunchKernelGGL(ffn_gateup_mfma_kernel, dim3(round_up8((long)max_tiles * (a.f / 64))), dim3(256), 0,
                                   s, xd, a.off, a.map, a.d, a.f, wg, wu, (bf16_t*)a.g, (bf16_t*)a.u, (bf16_t*)a.act));
    const int ntd = (a.d + BN - 1) / BN;
    XMOE_LAUNCH(K_FFN_DOWN_MFMA, s,
                hipLaunchKernelGGL(ffn_rowgemm_mfma_kernel<false>, dim3(round_up8((long)max_tiles * ntd)), dim3(256), 0,
                                   s, (const bf16_t*)a.act, a.off, a.map, a.f, a.d, wd, (bf16_t*)a.y, nullptr, nullptr,
                                   nullptr, nullptr, nullptr));
    return XMOE_OK;
}

int ffn_bwd_mfma(const FfnArgs& a, hipStream_t s) {
    const int max_tiles = ffn_max_tiles(a.B, a.E, BM);
    int st = launch_tile_map(a.off, a.E, BM, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const bf16_t *xd = (const bf16_t*)a.xd, *wg = (const bf16_t*)a.wg, *wu = (const bf16_t*)a.wu,
                 *wd = (const bf16_t*)a.wd, *dy = (const bf16_t*)a.dy;
    bf16_t *dg = (bf16_t*)a.dg, *du = (bf16_t*)a.du, *act = (bf16_t*)a.act;
    const int ntf = (a.f + BN - 1) / BN, ntd = (a.d + BN - 1) / BN;
    XMOE_LAUNCH(K_FFN_DACT_MFMA, s,
                hipLaunchKernelGGL(ffn_rowgemm_mfma_kernel<true>, dim3(round_up8((long)max_tiles * ntf)), dim3(256), 0,
                                   s, dy, a.off, a.map, a.d, a.f, wd, nullptr, (const bf16_t*)a.g, (const bf16_t*)a.u,
                                   dg, du, act));
    XMOE_LAUNCH(K_FFN_DX_MFMA, s,
                hipLaunchKernelGGL(ffn_dx_mfma_kernel, dim3(round_up8((long)max_tiles * ntd)), dim3(256), 0, s, dg, du,
                                   a.off, a.map, a.d, a.f, wg, wu, (bf16_t*)a.dxd));
    const int mtf = (a.f + BM - 1) / BM, mtd = (a.d + BM - 1) / BM;
    XMOE_LAUNCH(K_FFN_WGRAD_MFMA, s,
                hipLaunchKernelGGL(ffn_wgrad_mfma_kernel, dim3(round_up8((long)a.E * mtf * ntd)), dim3(256), 0, s, act,
                                   dy, a.off, a.E, a.f, a.d, (bf16_t*)a.dwd));
    XMOE_LAUNCH(K_FFN_WGRAD_MFMA, s,
                hipLaunchKernelGGL(ffn_wgrad_mfma_kernel, dim3(round_up8((long)a.E * mtd * ntf)), dim3(256), 0, s, xd,
                                   dg, a.off, a.E, a.d, a.f, (bf16_t*)a.dwg));
    XMOE_LAUNCH(K_FFN_WGRAD_MFMA, s,
                hipLaunchKernelGGL(ffn_wgrad_mfma_kernel, dim3(round_up8((long)a.E * mtd * ntf)), dim3(256), 0, s, xd,
                                   du, a.off, a.E, a.d, a.f, (bf16_t*)a.dwu));
    return XMOE_OK;
}

}  // namespace xmoe
