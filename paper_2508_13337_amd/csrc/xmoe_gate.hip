// Gating of the padding-free MoE layer (paper: Listing 1 gating(); Appendix B.3 "Padding-free Gating"):
// gate projection in a fixed float32 order, softmax + top-k routing, and their backward.
#include "xmoe_internal.h"
#include "xmoe_sizes.h"

namespace xmoe {

// =========================================================================================================
// gate projection, fixed summation order
// =========================================================================================================
// One wave owns GT tokens x GE experts.  Lane l is partial sum l of the contract: it walks i = l, l+64, ...
// and keeps GT*GE accumulators.  The 64 partials of every (token, expert) pair are then folded by halving
// (lane l with lane l^32, then l^16, ...), which is the order the contract prescribes; the fold is done as a
// transposing reduction so that lane v ends up with the finished sum of pair v.
constexpr int kGT = 8;
constexpr int kGE = 8;

template <typename T>
__device__ __forceinline__ void load_w8(const T* __restrict__ wrow, int e0, int E, bool vec, float (&wv)[kGE]);

template <>
__device__ __forceinline__ void load_w8<float>(const float* __restrict__ wrow, int e0, int E, bool vec,
                                               float (&wv)[kGE]) {
    if (vec) {
        const float4* p = reinterpret_cast<const float4*>(wrow + e0);
        float4 a = p[0], b = p[1];
        wv[0] = a.x; wv[1] = a.y; wv[2] = a.z; wv[3] = a.w;
        wv[4] = b.x; wv[5] = b.y; wv[6] = b.z; wv[7] = b.w;
    } else {
#pragma unroll
        for (int j = 0; j < kGE; ++j) wv[j] = (e0 + j < E) ? wrow[e0 + j] : 0.f;
    }
}

template <>
__device__ __forceinline__ void load_w8<bf16_t>(const bf16_t* __restrict__ wrow, int e0, int E, bool vec,
                                                float (&wv)[kGE]) {
    if (vec) {
        uint4 q = *reinterpret_cast<const uint4*>(wrow + e0);
        uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wv[2 * j] = __uint_as_float(u[j] << 16);
            wv[2 * j + 1] = __uint_as_float(u[j] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int j = 0; j < kGE; ++j) wv[j] = (e0 + j < E) ? to_float(wrow[e0 + j]) : 0.f;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gate_logits_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                          const float* __restrict__ bias,
                                                          float* __restrict__ logits, int Tn, int d, int E,
                                                          int vec_w) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * kGT;
    const int e0 = (blockIdx.y * 4 + wave) * kGE;
    if (e0 >= E) return;

    float acc[kGT * kGE];
#pragma unroll
    for (int v = 0; v < kGT * kGE; ++v) acc[v] = 0.0f;

    const T* xrow[kGT];
#pragma unroll
    for (int tt = 0; tt < kGT; ++tt) {
        int t = t0 + tt;
        t = t < Tn ? t : Tn - 1;
        xrow[tt] = x + (size_t)t * d;
    }

    for (int i = lane; i < d; i += 64) {
        float wv[kGE];
        load_w8<T>(w + (size_t)i * E, e0, E, vec_w != 0, wv);
        float xv[kGT];
#pragma unroll
        for (int tt = 0; tt < kGT; ++tt) xv[tt] = to_float(xrow[tt][i]);
#pragma unroll
        for (int tt = 0; tt < kGT; ++tt)
#pragma unroll
            for (int ee = 0; ee < kGE; ++ee) acc[tt * kGE + ee] = fmaf(xv[tt], wv[ee], acc[tt * kGE + ee]);
    }

    // fold the 64 lane partials of each of the 64 (token, expert) pairs: offsets 32, 16, 8, 4, 2, 1
#pragma unroll
    for (int width = 32; width >= 1; width >>= 1) {
        const bool upper = (lane & width) != 0;
#pragma unroll
        for (int v = 0; v < width; ++v) {
            float send = upper ? acc[v] : acc[v + width];
            float keep = upper ? acc[v + width] : acc[v];
            float recv = __shfl_xor(send, width, 64);
            acc[v] = keep + recv;
        }
    }
    // lane v now holds pair v = tt*kGE + ee
    const int t = t0 + (lane / kGE);
    const int e = e0 + (lane % kGE);
    if (t < Tn && e < E) {
        float v = acc[0];
        if (bias) v = v + bias[e];
        logits[(size_t)t * E + e] = v;
    }
}

// The same sums for bf16 operands whose rows are 16-byte aligned and d % 64 == 0, with the operands staged through
// LDS.  In the kernel above a wave's load of w touches 64 different 128-byte lines for 1 KiB of data (lane l reads
// 16 bytes of row l), four waves of a block do that side by side, and every wave fetches the same x values again: the
// L1, not the float32 pipe, sets the pace.  Here the block fetches each 64-row chunk of w (its 32 experts: 64 bytes
// per row) and of x (its 8 tokens) once, coalesced, a chunk ahead through registers, and a lane reads its row of w
// and its 8 token values with two 16-byte LDS reads.  Work split, accumulation order and the fold are those of the
// kernel above, so the results are the same bits.
constexpr int kGWStride = 80;   // bytes per staged row of w: 4 x 16 bytes + 16 bytes of padding

__global__ __launch_bounds__(256) void gate_logits_lds_kernel(const bf16_t* __restrict__ x,
                                                              const bf16_t* __restrict__ w,
                                                              const float* __restrict__ bias,
                                                              float* __restrict__ logits, int Tn, int d, int E) {
    __shared__ __align__(16) char sw[2][64 * kGWStride];   // [i][32 experts]
    __shared__ __align__(16) char sx[2][64 * 16];          // [i][8 tokens]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * kGT;
    const int eb = blockIdx.y * 4 * kGE;
    // staging roles: w row tid/4, 16-byte piece tid%4;  x token tid/32, elements 2*(tid%32) and the next
    const int wr = tid >> 2, wpiece = tid & 3;
    const bool w_ok = eb + kGE * wpiece < E;
    const int xt = tid >> 5, xi = 2 * (tid & 31);
    int tok = t0 + xt;
    tok = tok < Tn ? tok : Tn - 1;
    const bf16_t* xp = x + (size_t)tok * d + xi;
    const bf16_t* wp = w + (size_t)wr * E + eb + kGE * wpiece;
    uint4 wq = make_uint4(0, 0, 0, 0);
    uint32_t xq;
    auto fetch = [&](int i0) {
        if (w_ok) wq = *reinterpret_cast<const uint4*>(wp + (size_t)i0 * E);
        xq = *reinterpret_cast<const uint32_t*>(xp + i0);
    };
    auto stage = [&](int buf) {
        *reinterpret_cast<uint4*>(sw[buf] + wr * kGWStride + wpiece * 16) = wq;
        *reinterpret_cast<uint16_t*>(sx[buf] + xi * 16 + xt * 2) = (uint16_t)(xq & 0xffffu);
        *reinterpret_cast<uint16_t*>(sx[buf] + (xi + 1) * 16 + xt * 2) = (uint16_t)(xq >> 16);
    };

    float acc[kGT * kGE];
#pragma unroll
    for (int v = 0; v < kGT * kGE; ++v) acc[v] = 0.0f;

    const int chunks = d / 64;
    fetch(0);
    stage(0);
    __syncthreads();
    for (int c = 0; c < chunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < chunks) fetch((c + 1) * 64);
        const uint4 wv4 = *reinterpret_cast<const uint4*>(sw[buf] + lane * kGWStride + wave * 16);
        const uint4 xv4 = *reinterpret_cast<const uint4*>(sx[buf] + lane * 16);
        const uint32_t wu[4] = {wv4.x, wv4.y, wv4.z, wv4.w}, xu[4] = {xv4.x, xv4.y, xv4.z, xv4.w};
        float wv[kGE], xv[kGT];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wv[2 * j] = __uint_as_float(wu[j] << 16);
            wv[2 * j + 1] = __uint_as_float(wu[j] & 0xffff0000u);
            xv[2 * j] = __uint_as_float(xu[j] << 16);
            xv[2 * j + 1] = __uint_as_float(xu[j] & 0xffff0000u);
        }
#pragma unroll
        for (int tt = 0; tt < kGT; ++tt)
#pragma unroll
            for (int ee = 0; ee < kGE; ++ee) acc[tt * kGE + ee] = fmaf(xv[tt], wv[ee], acc[tt * kGE + ee]);
        if (c + 1 < chunks) stage(buf ^ 1);
        // the chunk staged above is read after this barrier, and the buffer it went to was last read before the
        // barrier of the previous round
        __syncthreads();
    }

#pragma unroll
    for (int width = 32; width >= 1; width >>= 1) {
        const bool upper = (lane & width) != 0;
#pragma unroll
        for (int v = 0; v < width; ++v) {
            float send = upper ? acc[v] : acc[v + width];
            float keep = upper ? acc[v + width] : acc[v];
            float recv = __shfl_xor(send, width, 64);
            acc[v] = keep + recv;
        }
    }
    const int t = t0 + (lane / kGE);
    const int e = eb + wave * kGE + (lane % kGE);
    if (t < Tn && e < E) {
        float v = acc[0];
        if (bias) v = v + bias[e];
        logits[(size_t)t * E + e] = v;
    }
}

// =========================================================================================================
// softmax + top-k: one wave per token
// =========================================================================================================
constexpr int kMaxPerLane = XMOE_MAX_EXPERTS / 64;   // 8

// order-preserving bit pattern of a float; -0.0 and +0.0 compare equal as numbers, so both map to +0.0's key and
// the lower expert index decides between them like any other tie
__device__ __forceinline__ uint32_t order_key(float v) {
    uint32_t u = __float_as_uint(v);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned long long o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

template <int PER_LANE>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int Tn, int E, int k,
                                                    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const float* row = logits + (size_t)t * E;
    float l[PER_LANE];
    // key = (order-preserving bits of the logit, inverted expert index): the maximum is the largest logit,
    // and among equal logits the smallest index
    unsigned long long key[PER_LANE];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        int e = lane + 64 * j;
        bool ok = e < E;
        l[j] = ok ? row[e] : -INFINITY;
        key[j] = ok ? (((unsigned long long)order_key(l[j]) << 32) | (uint32_t)(0xffffffffu - (uint32_t)e)) : 0ull;
        m = fmaxf(m, l[j]);
    }
    m = wave_max(m);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) s += (lane + 64 * j < E) ? expf(l[j] - m) : 0.f;
    s = wave_sum(s);
    const float inv = 1.0f / s;

    int my_idx = 0;
    float my_w = 0.f;
    for (int slot = 0; slot < k; ++slot) {
        unsigned long long best = 0ull;
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) best = key[j] > best ? key[j] : best;
        best = wave_max_u64(best);
        const int e = (int)(0xffffffffu - (uint32_t)(best & 0xffffffffull));
        // the owner retires the winner
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j)
            if (lane + 64 * j == e) key[j] = 0ull;
        // every lane can rebuild the winning logit from the key
        uint32_t ob = (uint32_t)(best >> 32);
        uint32_t fb = (ob & 0x80000000u) ? (ob & 0x7fffffffu) : ~ob;
        float lw = __uint_as_float(fb);
        if (lane == slot) {
            my_idx = e;
            my_w = expf(lw - m) * inv;
        }
    }
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = my_idx;
        topk_w[(size_t)t * k + lane] = my_w;
    }
}

// backward of softmax + top-k (indices constant): one wave per token
template <int PER_LANE>
__global__ __launch_bounds__(256) void route_bwd_kernel(const float* __restrict__ logits,
                                                        const int32_t* __restrict__ topk_idx,
                                                        const float* __restrict__ dw, int Tn, int E, int k,
                                                        float* __restrict__ dlogits) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const float* row = logits + (size_t)t * E;
    float p[PER_LANE], dp[PER_LANE];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        int e = lane + 64 * j;
        p[j] = e < E ? row[e] : -INFINITY;
        dp[j] = 0.f;
        m = fmaxf(m, p[j]);
    }
    m = wave_max(m);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        p[j] = (lane + 64 * j < E) ? expf(p[j] - m) : 0.f;
        s += p[j];
    }
    s = wave_sum(s);
    const float inv = 1.0f / s;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) p[j] *= inv;
    for (int slot = 0; slot < k; ++slot) {
        int e = topk_idx[(size_t)t * k + slot];
        float g = dw[(size_t)t * k + slot];
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j)
            if (lane + 64 * j == e) dp[j] += g;
    }
    float inner = 0.f;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) inner += p[j] * dp[j];
    inner = wave_sum(inner);
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) {
        int e = lane + 64 * j;
        if (e < E) dlogits[(size_t)t * E + e] = p[j] * (dp[j] - inner);
    }
}

// =========================================================================================================
// backward of the gate projection
// =========================================================================================================
// Both GEMMs of the gate projection's backward run on the float32 matrix instruction v_mfma_f32_32x32x2_f32 (the
// operands are dlogits, float32, and x / w_router widened exactly to float32, so nothing is rounded before the
// float32 accumulation).  A lane supplies one element of each operand per instruction: lane l holds
// A[row l%32][k = l/32] and B[k = l/32][column l%32], and ends up with 16 results
// D[row 8*(v/4) + 4*(l/32) + v%4][column l%32], v = 0..15.
typedef __attribute__((ext_vector_type(16))) float gate_f32x16_t;

// two consecutive elements of a row as float32; vec: one 4-byte (bf16) / 8-byte (float) load
__device__ __forceinline__ void load_pair(const bf16_t* p, bool ok0, bool ok1, bool vec, float& a, float& b) {
    if (vec) {
        const uint32_t u = ok0 ? *reinterpret_cast<const uint32_t*>(p) : 0u;
        a = __uint_as_float(u << 16);
        b = __uint_as_float(u & 0xffff0000u);
    } else {
        a = ok0 ? to_float(p[0]) : 0.f;
        b = ok1 ? to_float(p[1]) : 0.f;
    }
}
__device__ __forceinline__ void load_pair(const float* p, bool ok0, bool ok1, bool vec, float& a, float& b) {
    if (vec) {
        const float2 v = ok0 ? *reinterpret_cast<const float2*>(p) : make_float2(0.f, 0.f);
        a = v.x;
        b = v.y;
    } else {
        a = ok0 ? p[0] : 0.f;
        b = ok1 ? p[1] : 0.f;
    }
}

// partial[s][i][e] = sum over the s-th slice of tokens of x[t,i] * dlogits[t,e]
// The summation index is the token, and both operands are stored token-major, so a half-wave reads consecutive
// elements of one token's row: no transposition.  A block owns 64 rows i x 64 columns e of one slice.  The rows and
// columns of an instruction's 32 x 32 block are interleaved with those of its neighbour (row r of block a is
// i0 + 2r + a, column c of block b is e0 + 2c + b), so that one 4-byte load of x and one 8-byte load of dlogits
// per lane feed four instructions.  The block's four waves take interleaved runs of 16 tokens each (enough waves in
// flight to hide the loads' latency), and their partial tiles are added through LDS in wave order.
// grid = (ceil(d/64), ceil(E/64), splits).  vec_x / vec_e: the pairs may be fetched with one load.
template <typename T>
__global__ __launch_bounds__(256) void gate_bwd_dw_kernel(const T* __restrict__ x, const float* __restrict__ dl,
                                                          float* __restrict__ partial, int Tn, int d, int E,
                                                          int t_per_split, int vec_x, int vec_e) {
    __shared__ float red[4][32][64];   // [wave][accumulator register][lane], used once per row block a
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i0 = blockIdx.x * 64, e0 = blockIdx.y * 64;
    const int tb = blockIdx.z * t_per_split;
    int te = tb + t_per_split;
    te = te < Tn ? te : Tn;
    const int h = lane >> 5, c = lane & 31;
    const int ia = i0 + 2 * c, ea = e0 + 2 * c;
    const bool ok_i0 = ia < d, ok_i1 = ia + 1 < d, ok_e0 = ea < E, ok_e1 = ea + 1 < E;
    const T* xa = x + (ok_i0 ? ia : 0);
    const float* ba = dl + (ok_e0 ? ea : 0);
    gate_f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    constexpr int U = 8;   // instructions' worth of operands fetched before the first is used
    for (int t0 = tb + wave * 2 * U; t0 < te; t0 += 4 * 2 * U) {
        float av[U][2], bv[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + 2 * u + h;
            const bool ok_t = t < te;
            load_pair(xa + (size_t)(ok_t ? t : tb) * d, ok_t && ok_i0, ok_t && ok_i1, vec_x && ok_i1, av[u][0], av[u][1]);
            load_pair(ba + (size_t)(ok_t ? t : tb) * E, ok_t && ok_e0, ok_t && ok_e1, vec_e && ok_e1, bv[u][0], bv[u][1]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][a], bv[u][b], acc[a][b], 0, 0, 0);
    }
    float* out = partial + (size_t)blockIdx.z * d * E;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            red[wave][v][lane] = acc[a][0][v];
            red[wave][16 + v][lane] = acc[a][1][v];
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int n = threadIdx.x + 256 * r;   // (accumulator register, lane) pair
            const int reg = n >> 6, l = n & 63;
            const float sum = ((red[0][reg][l] + red[1][reg][l]) + red[2][reg][l]) + red[3][reg][l];
            const int v = reg & 15;
            const int i = i0 + 2 * (8 * (v >> 2) + 4 * (l >> 5) + (v & 3)) + a;
            const int e = e0 + 2 * (l & 31) + (reg >> 4);
            if (i < d && e < E) out[(size_t)i * E + e] = sum;
        }
        __syncthreads();
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gate_bwd_dw_reduce_kernel(const float* __restrict__ partial, int splits,
                                                                 size_t n, T* __restrict__ dwr) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += partial[(size_t)sp * n + i];
    dwr[i] = from_float<T>(s);
}

// dx_gate[t,i] = sum_e dlogits[t,e] * w[i,e]
// The summation index e is contiguous in both operands.  The instruction sums over its two k-slots and the loop
// over its steps, so any assignment of experts to (step, slot) gives the same sum: slot h of step q takes expert
// 32*h + q of a chunk of 64, and a lane then reads 32 consecutive experts of its row with 16-byte loads.
// One wave: 32 tokens x kDxCols columns i; the token rows of dlogits stay in registers across the columns.
constexpr int kDxCols = 256;

template <typename T>
__device__ __forceinline__ void load_row32(const T* __restrict__ p, int n_valid, bool vec, float (&v)[32]);
template <>
__device__ __forceinline__ void load_row32<float>(const float* __restrict__ p, int n_valid, bool vec, float (&v)[32]) {
    if (vec) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float4 f = reinterpret_cast<const float4*>(p)[q];
            v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
        }
    } else {
#pragma unroll
        for (int q = 0; q < 32; ++q) v[q] = q < n_valid ? p[q] : 0.f;
    }
}
template <>
__device__ __forceinline__ void load_row32<bf16_t>(const bf16_t* __restrict__ p, int n_valid, bool vec,
                                                   float (&v)[32]) {
    if (vec) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 u4 = reinterpret_cast<const uint4*>(p)[q];
            const uint32_t u[4] = {u4.x, u4.y, u4.z, u4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[8 * q + 2 * j] = __uint_as_float(u[j] << 16);
                v[8 * q + 2 * j + 1] = __uint_as_float(u[j] & 0xffff0000u);
            }
        }
    } else {
#pragma unroll
        for (int q = 0; q < 32; ++q) v[q] = q < n_valid ? to_float(p[q]) : 0.f;
    }
}

// vec: E % 64 == 0 and both operands 16-byte aligned
template <typename T>
__global__ __launch_bounds__(256) void gate_bwd_dx_kernel(const float* __restrict__ dl, const T* __restrict__ w,
                                                          T* __restrict__ dxg, int Tn, int d, int E, int vec) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * 4 + wave) * 32;
    if (t0 >= Tn) return;
    const int h = lane >> 5, c = lane & 31;
    const int ibeg = blockIdx.y * kDxCols;
    const int iend = ibeg + kDxCols < d ? ibeg + kDxCols : d;
    const bool ok_t = t0 + c < Tn;
    const float* arow = dl + (size_t)(ok_t ? t0 + c : 0) * E + 32 * h;
    const bool one_chunk = E <= 64;
    float av[32];
    if (one_chunk) load_row32<float>(arow, ok_t ? E - 32 * h : 0, vec && ok_t, av);
    if (one_chunk && !ok_t) {
#pragma unroll
        for (int q = 0; q < 32; ++q) av[q] = 0.f;
    }
    for (int i0 = ibeg; i0 < iend; i0 += 32) {
        const bool ok_i = i0 + c < d;
        const T* brow = w + (size_t)(ok_i ? i0 + c : 0) * E + 32 * h;
        gate_f32x16_t acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        for (int e0 = 0; e0 < E; e0 += 64) {
            float bv[32];
            const int n_valid = E - e0 - 32 * h;   // experts left in this lane's run of 32
            if (!one_chunk) {
                load_row32<float>(arow + e0, ok_t ? n_valid : 0, vec && ok_t, av);
                if (!ok_t) {
#pragma unroll
                    for (int q = 0; q < 32; ++q) av[q] = 0.f;
                }
            }
            load_row32<T>(brow + e0, ok_i ? n_valid : 0, vec && ok_i, bv);
            if (!ok_i) {
#pragma unroll
                for (int q = 0; q < 32; ++q) bv[q] = 0.f;
            }
#pragma unroll
            for (int q = 0; q < 32; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q], bv[q], acc, 0, 0, 0);
        }
        if (ok_i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = t0 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (t < Tn) dxg[(size_t)t * d + i0 + c] = from_float<T>(acc[v]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// The same two products for bf16 operands on the bf16 matrix instruction (16 summands per instruction and operand
// row instead of 2).  x and w are bf16 as stored; dlogits is float32 and goes in as the sum of two bf16 terms,
// hi = bf16(v) and lo = bf16(v - hi), i.e. with 16 significant bits: every product is exact in float32, the sums are
// float32, and what is dropped (2^-17 of a term) is far below the bf16 rounding of the results.
// Used when d % 64 == 0, E % 64 == 0 and the operands are 16-byte aligned; otherwise the kernels above.
// ---------------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 gate_bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short gate_s16x4_t;
typedef __attribute__((ext_vector_type(8))) short gate_s16x8_t;

// v[0..7] -> hi and lo as packed bf16 pairs
__device__ __forceinline__ void split_bf16x8(const float (&v)[8], uint4& hi, uint4& lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        h[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
        const float r0 = v[2 * q] - __uint_as_float(h[q] << 16);
        const float r1 = v[2 * q + 1] - __uint_as_float(h[q] & 0xffff0000u);
        l[q] = pack_bf16x2(r0, r1);
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
}

// partial[s][i][e] = sum over the s-th slice of tokens of x[t,i] * dlogits[t,e].  Both operands are stored
// token-major while the instruction wants 8 consecutive tokens per lane, so a block stages 64 tokens x (64 columns i
// of x, 64 experts of dlogits as hi and lo) in LDS as they lie in memory and takes its operands with the
// transposing LDS read.  Four waves: one 32 x 32 block of the 64 x 64 output each.  grid = (d/64, E/64, splits).
constexpr int kDwTok = 64;
constexpr int kDwStride = 144;   // bytes per staged token row: 64 bf16 + 16 bytes of padding

// operand for v_mfma_f32_32x32x16_bf16 from a token-major tile: column col_base + lane%32, tokens
// 16*ks + 8*(lane/32) .. +7.  In a group of 16 lanes, lane s addresses 4 consecutive columns (s%4) of token row
// (s/4); the transposing read hands every lane one column with 4 consecutive tokens.
__device__ __forceinline__ gate_bf16x8_t dw_frag(const char* tile, int col_base, int ks) {
    const int lane = threadIdx.x & 63;
    const int G = lane >> 4, s = lane & 15;
    const int col = col_base + 16 * (G & 1) + 4 * (s & 3);
    const int k0 = 16 * ks + 8 * (G >> 1) + (s >> 2);
    gate_s16x4_t h[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const char* a = tile + (k0 + 4 * q) * kDwStride + col * 2;
        h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) gate_s16x4_t*)(
            (__attribute__((address_space(3))) void*)a));
    }
    const gate_s16x8_t v = {h[0][0], h[0][1], h[0][2], h[0][3], h[1][0], h[1][1], h[1][2], h[1][3]};
    return __builtin_bit_cast(gate_bf16x8_t, v);
}

__global__ __launch_bounds__(256) void gate_bwd_dw_mfma_kernel(const bf16_t* __restrict__ x,
                                                               const float* __restrict__ dl,
                                                               float* __restrict__ partial, int Tn, int d, int E,
                                                               int t_per_split) {
    __shared__ __align__(16) char xs[kDwTok * kDwStride];
    __shared__ __align__(16) char dhi[kDwTok * kDwStride];
    __shared__ __align__(16) char dlo[kDwTok * kDwStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = blockIdx.x * 64, e0 = blockIdx.y * 64;
    const int tb = blockIdx.z * t_per_split;
    int te = tb + t_per_split;
    te = te < Tn ? te : Tn;
    const int mi = wave >> 1, ni = wave & 1;
    // staging: token rows tid/8 and tid/8 + 32 of a chunk; 8 columns of x (16 bytes) and 8 experts of dlogits each
    const int sr = tid >> 3, sp = tid & 7;
    uint4 xr[2];
    float4 dr[2][2];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int t = t0 + sr + 32 * j;
            xr[j] = make_uint4(0, 0, 0, 0);
            dr[j][0] = dr[j][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (t < te) {
                xr[j] = *reinterpret_cast<const uint4*>(x + (size_t)t * d + i0 + sp * 8);
                const float4* p = reinterpret_cast<const float4*>(dl + (size_t)t * E + e0 + sp * 8);
                dr[j][0] = p[0];
                dr[j][1] = p[1];
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int o = (sr + 32 * j) * kDwStride + sp * 16;
            const float v[8] = {dr[j][0].x, dr[j][0].y, dr[j][0].z, dr[j][0].w,
                                dr[j][1].x, dr[j][1].y, dr[j][1].z, dr[j][1].w};
            uint4 hi, lo;
            split_bf16x8(v, hi, lo);
            *reinterpret_cast<uint4*>(xs + o) = xr[j];
            *reinterpret_cast<uint4*>(dhi + o) = hi;
            *reinterpret_cast<uint4*>(dlo + o) = lo;
        }
    };
    gate_f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    if (tb < te) fetch(tb);
    for (int t0 = tb; t0 < te; t0 += kDwTok) {
        stage();
        __syncthreads();
        if (t0 + kDwTok < te) fetch(t0 + kDwTok);   // in flight while this chunk is multiplied
#pragma unroll
        for (int ks = 0; ks < kDwTok / 16; ++ks) {
            const gate_bf16x8_t a = dw_frag(xs, 32 * mi, ks);
            const gate_bf16x8_t bh = dw_frag(dhi, 32 * ni, ks);
            const gate_bf16x8_t bl = dw_frag(dlo, 32 * ni, ks);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bh, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bl, acc, 0, 0, 0);
        }
        __syncthreads();   // everybody is done reading before the next chunk is staged
    }
    float* out = partial + (size_t)blockIdx.z * d * E;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + 32 * mi + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int e = e0 + 32 * ni + (lane & 31);
        out[(size_t)i * E + e] = acc[v];
    }
}

// dx_gate[t,i] = sum_e dlogits[t,e] * w[i,e]: e is contiguous in both operands, so a lane takes its 8 consecutive
// experts straight from memory (dlogits: 8 floats -> hi, lo; w: 16 bytes).  One wave: 32 tokens x kDxCols columns.
// The wave's rows of dlogits are fetched and split once per 64 experts: for E == 64 they stay in registers across the
// column blocks; for larger E the chunks of 64 experts are the outer loop and the kDxCols / 32 column blocks keep
// an accumulator each.  (Fewer columns per wave, i.e. more and shorter waves, is slower: 64 columns 32 us against 26
// at config 2 - fetching and splitting the rows of dlogits costs more than short waves hide.)
// w is the instruction's first operand: the result block is [column i][token], so that a lane ends up with runs of 4
// consecutive columns of one token row and stores 8 bytes at a time.
constexpr int kDxColsManyExperts = 128;   // E > 64: four accumulators per wave (eight leave one wave per SIMD)
template <bool ONE_CHUNK>
__global__ __launch_bounds__(256) void gate_bwd_dx_mfma_kernel(const float* __restrict__ dl,
                                                               const bf16_t* __restrict__ w,
                                                               bf16_t* __restrict__ dxg, int Tn, int d, int E) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * 4 + wave) * 32;
    if (!ONE_CHUNK && t0 >= Tn) return;   // (E == 64: every wave takes part in the staging and its barrier)
    const int h = lane >> 5, c = lane & 31;
    // columns per wave; d % 64 == 0, so every 32-column block below is complete
    constexpr int COLS = ONE_CHUNK ? kDxCols : kDxColsManyExperts;
    const int ibeg = blockIdx.y * COLS;
    const int iend = ibeg + COLS < d ? ibeg + COLS : d;
    const bool ok_t = t0 + c < Tn;
    const float* arow = dl + (size_t)(ok_t ? t0 + c : 0) * E + 8 * h;
    uint4 ah[4], al[4];
    auto load_a = [&](int e0) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (ok_t) {
                const float4* p = reinterpret_cast<const float4*>(arow + e0 + 16 * ks);
                const float4 f0 = p[0], f1 = p[1];
                v[0] = f0.x; v[1] = f0.y; v[2] = f0.z; v[3] = f0.w;
                v[4] = f1.x; v[5] = f1.y; v[6] = f1.z; v[7] = f1.w;
            }
            split_bf16x8(v, ah[ks], al[ks]);
        }
    };
    auto multiply = [&](int i0, int e0, gate_f32x16_t& acc) {
        const bf16_t* brow = w + (size_t)(i0 + c) * E + 8 * h + e0;
        uint4 b[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) b[ks] = *reinterpret_cast<const uint4*>(brow + 16 * ks);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const gate_bf16x8_t bb = __builtin_bit_cast(gate_bf16x8_t, b[ks]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, __builtin_bit_cast(gate_bf16x8_t, ah[ks]), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, __builtin_bit_cast(gate_bf16x8_t, al[ks]), acc, 0, 0, 0);
        }
    };
    // lane (h, c): token t0 + c, columns i0 + 8j + 4h .. +3 in acc[4j .. 4j+3]
    auto store = [&](int i0, const gate_f32x16_t& acc) {
        if (!ok_t) return;
        bf16_t* orow = dxg + (size_t)(t0 + c) * d + i0 + 4 * h;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            *reinterpret_cast<uint2*>(orow + 8 * j) =
                make_uint2(pack_bf16x2(acc[4 * j], acc[4 * j + 1]), pack_bf16x2(acc[4 * j + 2], acc[4 * j + 3]));
    };
    if (ONE_CHUNK) {
        // E == 64.  The four waves of a block work on the same columns, so the block stages its kDxCols rows of w in
        // LDS once (rows of 128 bytes padded to kDwStride) and the column blocks take their operands from there:
        // with loads from memory between the stores, every wait for an operand would also wait for the stores
        // issued before it (the counter is in issue order).
        __shared__ __align__(16) char wsm[kDxCols * kDwStride];
        {
            const int r = threadIdx.x >> 3, piece = threadIdx.x & 7;   // 32 rows x 8 pieces of 16 bytes per pass
#pragma unroll
            for (int pass = 0; pass < kDxCols / 32; ++pass) {
                const int row = pass * 32 + r;
                uint4 q = make_uint4(0, 0, 0, 0);
                if (ibeg + row < iend) q = *reinterpret_cast<const uint4*>(w + (size_t)(ibeg + row) * E + piece * 8);
                *reinterpret_cast<uint4*>(wsm + row * kDwStride + piece * 16) = q;
            }
        }
        load_a(0);
        __syncthreads();
        for (int i0 = ibeg; i0 < iend; i0 += 32) {
            gate_f32x16_t acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const char* brow = wsm + (i0 - ibeg + c) * kDwStride + 16 * h;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const gate_bf16x8_t bb = *reinterpret_cast<const gate_bf16x8_t*>(brow + 32 * ks);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, __builtin_bit_cast(gate_bf16x8_t, ah[ks]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, __builtin_bit_cast(gate_bf16x8_t, al[ks]), acc, 0, 0, 0);
            }
            store(i0, acc);
        }
    } else {
        constexpr int NB = COLS / 32;
        gate_f32x16_t acc[NB];
#pragma unroll
        for (int n = 0; n < NB; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
        for (int e0 = 0; e0 < E; e0 += 64) {
            load_a(e0);
#pragma unroll
            for (int n = 0; n < NB; ++n)
                if (ibeg + 32 * n < iend) multiply(ibeg + 32 * n, e0, acc[n]);
        }
#pragma unroll
        for (int n = 0; n < NB; ++n)
            if (ibeg + 32 * n < iend) store(ibeg + 32 * n, acc[n]);
    }
}

template <typename T>
static int launch_gate_logits(const void* x, const void* w, const float* bias, float* logits, int Tn, int d,
                              int E, hipStream_t s) {
    int vec = (E % kGE == 0) && aligned16(w) && ((E * sizeof(T)) % 16 == 0);
    dim3 grid((Tn + kGT - 1) / kGT, (E + 4 * kGE - 1) / (4 * kGE));
    if (sizeof(T) == 2 && vec && d % 64 == 0 && (reinterpret_cast<uintptr_t>(x) & 3u) == 0) {
        XMOE_LAUNCH(K_GATE_LOGITS, s,
                    hipLaunchKernelGGL(gate_logits_lds_kernel, grid, dim3(256), 0, s, (const bf16_t*)x,
                                       (const bf16_t*)w, bias, logits, Tn, d, E));
        return XMOE_OK;
    }
    XMOE_LAUNCH(K_GATE_LOGITS, s,
                hipLaunchKernelGGL(gate_logits_kernel<T>, grid, dim3(256), 0, s, (const T*)x, (const T*)w, bias,
                                   logits, Tn, d, E, vec));
    return XMOE_OK;
}

template <typename T>
static int launch_gate_bwd(const void* x, const void* w, const float* dl, int Tn, int d, int E, void* dwr,
                           void* dxg, float* partial, hipStream_t s) {
    const int splits = gate_bwd_splits(Tn);
    const int tps = (Tn + splits - 1) / splits;
    dim3 g1((d + 63) / 64, (E + 63) / 64, splits);
    if (sizeof(T) == 2 && d % 64 == 0 && E % 64 == 0 && aligned16(x) && aligned16(w) && aligned16(dl) &&
        aligned16(dxg)) {
        XMOE_LAUNCH(K_GATE_BWD_DW, s,
                    hipLaunchKernelGGL(gate_bwd_dw_mfma_kernel, g1, dim3(256), 0, s, (const bf16_t*)x, dl, partial, Tn,
                                       d, E, tps));
        const size_t n_ = (size_t)d * E;
        XMOE_LAUNCH(K_GATE_BWD_DW_REDUCE, s,
                    hipLaunchKernelGGL(gate_bwd_dw_reduce_kernel<T>, dim3((unsigned)((n_ + 255) / 256)), dim3(256), 0,
                                       s, partial, splits, n_, (T*)dwr));
        if (E == 64) {
            dim3 g2m((Tn + 127) / 128, (d + kDxCols - 1) / kDxCols);
            XMOE_LAUNCH(K_GATE_BWD_DX, s,
                        hipLaunchKernelGGL(gate_bwd_dx_mfma_kernel<true>, g2m, dim3(256), 0, s, dl, (const bf16_t*)w,
                                           (bf16_t*)dxg, Tn, d, E));
        } else {
            dim3 g2m((Tn + 127) / 128, (d + kDxColsManyExperts - 1) / kDxColsManyExperts);
            XMOE_LAUNCH(K_GATE_BWD_DX, s,
                        hipLaunchKernelGGL(gate_bwd_dx_mfma_kernel<false>, g2m, dim3(256), 0, s, dl, (const bf16_t*)w,
                                           (bf16_t*)dxg, Tn, d, E));
        }
        return XMOE_OK;
    }
    const int vec_x = (d % 2 == 0) && ((reinterpret_cast<uintptr_t>(x) & (2 * sizeof(T) - 1)) == 0);
    const int vec_e = (E % 2 == 0) && ((reinterpret_cast<uintptr_t>(dl) & 7u) == 0);
    XMOE_LAUNCH(K_GATE_BWD_DW, s,
                hipLaunchKernelGGL(gate_bwd_dw_kernel<T>, g1, dim3(256), 0, s, (const T*)x, dl, partial, Tn, d, E,
                                   tps, vec_x, vec_e));
    size_t n = (size_t)d * E;
    XMOE_LAUNCH(K_GATE_BWD_DW_REDUCE, s,
                hipLaunchKernelGGL(gate_bwd_dw_reduce_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                                   s, partial, splits, n, (T*)dwr));
    dim3 g2((Tn + 127) / 128, (d + kDxCols - 1) / kDxCols);
    const int vec = (E % 64 == 0) && aligned16(dl) && aligned16(w);
    XMOE_LAUNCH(K_GATE_BWD_DX, s,
                hipLaunchKernelGGL(gate_bwd_dx_kernel<T>, g2, dim3(256), 0, s, dl, (const T*)w, (T*)dxg, Tn, d, E,
                                   vec));
    return XMOE_OK;
}

template <int PL>
static int launch_route(const float* logits, int Tn, int E, int k, int32_t* idx, float* w, hipStream_t s) {
    XMOE_LAUNCH(K_ROUTE, s,
                hipLaunchKernelGGL(route_kernel<PL>, dim3((Tn + 3) / 4), dim3(256), 0, s, logits, Tn, E, k, idx, w));
    return XMOE_OK;
}
template <int PL>
static int launch_route_bwd(const float* logits, const int32_t* idx, const float* dw, int Tn, int E, int k,
                            float* dl, hipStream_t s) {
    XMOE_LAUNCH(K_ROUTE_BWD, s,
                hipLaunchKernelGGL(route_bwd_kernel<PL>, dim3((Tn + 3) / 4), dim3(256), 0, s, logits, idx, dw, Tn,
                                   E, k, dl));
    return XMOE_OK;
}

}  // namespace xmoe

using namespace xmoe;

extern "C" {

int xmoe_gate_logits(const void* x, const void* w_router, const float* bias, float* logits, int T, int d, int E,
                     int dt, void* stream) {
    if (!dtype_ok(dt)) return XMOE_ERR_UNSUPPORTED;
    if (T < 0 || d < 1 || E < 1) return XMOE_ERR_INVALID_ARG;
    if ((long long)T * E >= (1ll << 31) || (long long)T * d >= (1ll << 40)) return XMOE_ERR_INVALID_ARG;
    if (T == 0) return XMOE_OK;
    if (!x || !w_router || !logits) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    return dt == XMOE_F32 ? launch_gate_logits<float>(x, w_router, bias, logits, T, d, E, s)
                          : launch_gate_logits<bf16_t>(x, w_router, bias, logits, T, d, E, s);
}

int xmoe_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w, void* stream) {
    if (T < 0 || E < 1 || k < 1 || k > E) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS || k > 64) return XMOE_ERR_UNSUPPORTED;
    if ((long long)T * k >= (1ll << 31) || (long long)T * E >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (T == 0) return XMOE_OK;
    if (!logits || !topk_idx || !topk_w) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (E <= 64) return launch_route<1>(logits, T, E, k, topk_idx, topk_w, s);
    if (E <= 128) return launch_route<2>(logits, T, E, k, topk_idx, topk_w, s);
    if (E <= 256) return launch_route<4>(logits, T, E, k, topk_idx, topk_w, s);
    return launch_route<8>(logits, T, E, k, topk_idx, topk_w, s);
}

int xmoe_route_bwd(const float* logits, const int32_t* topk_idx, const float* dw, int T, int E, int k,
                   float* dlogits, void* stream) {
    if (T < 0 || E < 1 || k < 1 || k > E) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS || k > 64) return XMOE_ERR_UNSUPPORTED;
    if ((long long)T * k >= (1ll << 31) || (long long)T * E >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (T == 0) return XMOE_OK;
    if (!logits || !topk_idx || !dw || !dlogits) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (E <= 64) return launch_route_bwd<1>(logits, topk_idx, dw, T, E, k, dlogits, s);
    if (E <= 128) return launch_route_bwd<2>(logits, topk_idx, dw, T, E, k, dlogits, s);
    if (E <= 256) return launch_route_bwd<4>(logits, topk_idx, dw, T, E, k, dlogits, s);
    return launch_route_bwd<8>(logits, topk_idx, dw, T, E, k, dlogits, s);
}

int xmoe_gate_logits_bwd(const void* x, const void* w_router, const float* dlogits, int T, int d, int E, int dt,
                         void* dw_router, void* dx_gate, void* ws, size_t ws_bytes, void* stream) {
    if (!dtype_ok(dt)) return XMOE_ERR_UNSUPPORTED;
    if (T < 0 || d < 1 || E < 1) return XMOE_ERR_INVALID_ARG;
    if ((long long)T * E >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (!dw_router) return XMOE_ERR_INVALID_ARG;
    if (T == 0) {   // a sum over no tokens: dw_router = 0, dx_gate has no rows
        const size_t n = (size_t)d * E;
        const dim3 grid((unsigned)((n + 255) / 256));
        if (dt == XMOE_F32)
            XMOE_LAUNCH(K_GATE_BWD_DW_REDUCE, (hipStream_t)stream,
                        hipLaunchKernelGGL(gate_bwd_dw_reduce_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream,
                                           (const float*)nullptr, 0, n, (float*)dw_router));
        else
            XMOE_LAUNCH(K_GATE_BWD_DW_REDUCE, (hipStream_t)stream,
                        hipLaunchKernelGGL(gate_bwd_dw_reduce_kernel<bf16_t>, grid, dim3(256), 0, (hipStream_t)stream,
                                           (const float*)nullptr, 0, n, (bf16_t*)dw_router));
        return XMOE_OK;
    }
    if (!x || !w_router || !dlogits || !dx_gate) return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < gate_bwd_ws_bytes(T, d, E))
        return XMOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    return dt == XMOE_F32
               ? launch_gate_bwd<float>(x, w_router, dlogits, T, d, E, dw_router, dx_gate, (float*)ws, s)
               : launch_gate_bwd<bf16_t>(x, w_router, dlogits, T, d, E, dw_router, dx_gate, (float*)ws, s);
}

}  // extern "C"
