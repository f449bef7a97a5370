// Row movers of the padding-free MoE layer (paper: Section 4.1.2 and Appendix B.4, gather and scatter kernels):
// dispatch (gather), combine (weighted gather-reduce instead of a scatter with atomics), and their backward.
// All of them are HBM-bound: one wave moves one row (or one token's k rows) with 16-byte accesses per lane
// along the hidden dimension, so every request is fully coalesced whatever the row permutation.
#include "xmoe_internal.h"

namespace xmoe {

// ---- 8 (bf16) or 4 (float) elements per 16-byte vector --------------------------------------------------
template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
    static constexpr int N = 4;
    __device__ static void unpack(const uint4& q, float (&v)[4]) {
        v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y);
        v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
    }
    __device__ static uint4 pack(const float (&v)[4]) {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    }
};
template <>
struct Vec16<bf16_t> {
    static constexpr int N = 8;
    __device__ static void unpack(const uint4& q, float (&v)[8]) {
        const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[2 * j] = __uint_as_float(u[j] << 16);
            v[2 * j + 1] = __uint_as_float(u[j] & 0xffff0000u);
        }
    }
    __device__ static uint4 pack(const float (&v)[8]) {
        uint32_t u[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            u[j] = pack_bf16x2(v[2 * j], v[2 * j + 1]);
        return make_uint4(u[0], u[1], u[2], u[3]);
    }
};

// =========================================================================================================
// dispatch: xd[i,:] = x[token_ids[i],:]     one wave per row
// =========================================================================================================
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void dispatch_kernel(const T* __restrict__ x, const int32_t* __restrict__ token_ids,
                                                       int Tn, int B, int d, T* __restrict__ xd) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= B) return;
    int t = token_ids[row];
    if ((unsigned)t >= (unsigned)Tn) return;   // never true for index arrays built by this library
    const T* src = x + (size_t)t * d;
    T* dst = xd + (size_t)row * d;
    if (VEC) {
        const int nv = d / Vec16<T>::N;
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4* d4 = reinterpret_cast<uint4*>(dst);
        int c = lane;
        for (; c + 192 < nv; c += 256) {   // four independent 16-byte loads in flight per lane
            const uint4 q0 = s4[c], q1 = s4[c + 64], q2 = s4[c + 128], q3 = s4[c + 192];
            d4[c] = q0;
            d4[c + 64] = q1;
            d4[c + 128] = q2;
            d4[c + 192] = q3;
        }
        for (; c < nv; c += 64) d4[c] = s4[c];
    } else {
        for (int c = lane; c < d; c += 64) dst[c] = src[c];
    }
}

// =========================================================================================================
// combine: out[t,:] = sum_j w[t,j] * y[row_of_slot[t*k+j],:] (+ shared rows) (+ addend)
// One block per token, consecutive threads on consecutive 16-byte pieces of the hidden dimension.  Slots are
// taken KU at a time: the KU row pieces of a column chunk are fetched by independent loads before the first is
// used.  The sum keeps the slot order j = 0 .. k-1, then the shared rows, then the addend.  An entry with
// row_of_slot outside [0, B) (a dropped token) contributes nothing.
// =========================================================================================================
template <typename T, bool VEC, int KU>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ y, const int32_t* __restrict__ row_of_slot,
                                                      const float* __restrict__ topk_w, const T* __restrict__ shared,
                                                      int n_shared, const int32_t* __restrict__ shared_row0,
                                                      const T* __restrict__ add, int Tn, int k, int d,
                                                      int B, T* __restrict__ out) {
    const int t = blockIdx.x;
    constexpr int N = Vec16<T>::N;
    // the shared rows start at a row that only the device knows (behind the retained rows of a capacity-limited PFT)
    if (shared_row0 && n_shared > 0) shared += (size_t)shared_row0[0] * d;
    if (VEC) {
        const int nv = d / N;
        for (int c = threadIdx.x; c < nv; c += 256) {
            float acc[N];
#pragma unroll
            for (int i = 0; i < N; ++i) acc[i] = 0.f;
            for (int j0 = 0; j0 < k; j0 += KU) {
                uint4 q[KU];
                float w[KU];
#pragma unroll
                for (int jj = 0; jj < KU; ++jj) {
                    const int j = j0 + jj < k ? j0 + jj : k - 1;   // a slot past k re-reads the last one, weight 0
                    const int r = row_of_slot[(size_t)t * k + j];
                    const bool ok = j0 + jj < k && (unsigned)r < (unsigned)B;
                    w[jj] = ok ? (topk_w ? topk_w[(size_t)t * k + j] : 1.0f) : 0.f;
                    q[jj] = reinterpret_cast<const uint4*>(y + (size_t)(ok ? r : 0) * d)[c];
                    if (!ok) q[jj] = make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int jj = 0; jj < KU; ++jj) {
                    float v[N];
                    Vec16<T>::unpack(q[jj], v);
#pragma unroll
                    for (int i = 0; i < N; ++i) acc[i] = fmaf(w[jj], v[i], acc[i]);
                }
            }
            for (int s = 0; s < n_shared; ++s) {
                float v[N];
                Vec16<T>::unpack(reinterpret_cast<const uint4*>(shared + ((size_t)s * Tn + t) * d)[c], v);
#pragma unroll
                for (int i = 0; i < N; ++i) acc[i] += v[i];
            }
            if (add) {
                float v[N];
                Vec16<T>::unpack(reinterpret_cast<const uint4*>(add + (size_t)t * d)[c], v);
#pragma unroll
                for (int i = 0; i < N; ++i) acc[i] += v[i];
            }
            reinterpret_cast<uint4*>(out + (size_t)t * d)[c] = Vec16<T>::pack(acc);
        }
    } else {
        for (int c = threadIdx.x; c < d; c += 256) {
            float acc = 0.f;
            for (int j = 0; j < k; ++j) {
                const int r = row_of_slot[(size_t)t * k + j];
                if ((unsigned)r >= (unsigned)B) continue;
                const float w = topk_w ? topk_w[(size_t)t * k + j] : 1.0f;
                acc = fmaf(w, to_float(y[(size_t)r * d + c]), acc);
            }
            for (int s = 0; s < n_shared; ++s) acc += to_float(shared[((size_t)s * Tn + t) * d + c]);
            if (add) acc += to_float(add[(size_t)t * d + c]);
            out[(size_t)t * d + c] = from_float<T>(acc);
        }
    }
}

// =========================================================================================================
// combine backward: dy[r,:] = w[t,j] * dout[t,:],  dw[t,j] = <dout[t,:], y[r,:]>,  r = row_of_slot[t*k+j]
// One block per token.  Slots in groups of KU: every chunk of dout[t,:] is read once per group and the group's
// rows of y by independent loads.  A thread accumulates its chunks in ascending order; the 64 lanes of a wave are
// folded by halving, and the four waves' sums are added in wave order.
// =========================================================================================================
template <typename T, bool VEC, int KU>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const T* __restrict__ dout, const T* __restrict__ y,
                                                          const int32_t* __restrict__ row_of_slot,
                                                          const float* __restrict__ topk_w, int Tn, int k, int d,
                                                          int B, T* __restrict__ dy, float* __restrict__ dw) {
    __shared__ float red[4][KU];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x;
    constexpr int N = Vec16<T>::N;
    for (int j0 = 0; j0 < k; j0 += KU) {
        int r8[KU];
        float w8[KU], dot[KU];
#pragma unroll
        for (int jj = 0; jj < KU; ++jj) {
            const int j = j0 + jj < k ? j0 + jj : k - 1;
            const int r = row_of_slot[(size_t)t * k + j];
            const bool ok = j0 + jj < k && (unsigned)r < (unsigned)B;
            r8[jj] = ok ? r : -1;
            w8[jj] = dy ? topk_w[(size_t)t * k + j] : 0.f;
            dot[jj] = 0.f;   // stays 0 for a dropped entry: the output does not depend on its weight
        }
        if (VEC) {
            const int nv = d / N;
            for (int c = threadIdx.x; c < nv; c += 256) {
                float g[N];
                Vec16<T>::unpack(reinterpret_cast<const uint4*>(dout + (size_t)t * d)[c], g);
                uint4 q[KU];
#pragma unroll
                for (int jj = 0; jj < KU; ++jj)
                    q[jj] = reinterpret_cast<const uint4*>(y + (size_t)(r8[jj] >= 0 ? r8[jj] : 0) * d)[c];
#pragma unroll
                for (int jj = 0; jj < KU; ++jj) {
                    if (r8[jj] < 0) continue;   // block-uniform
                    float v[N], o[N];
                    Vec16<T>::unpack(q[jj], v);
#pragma unroll
                    for (int i = 0; i < N; ++i) {
                        dot[jj] = fmaf(g[i], v[i], dot[jj]);
                        o[i] = w8[jj] * g[i];
                    }
                    if (dy) reinterpret_cast<uint4*>(dy + (size_t)r8[jj] * d)[c] = Vec16<T>::pack(o);
                }
            }
        } else {
            for (int c = threadIdx.x; c < d; c += 256) {
                const float g = to_float(dout[(size_t)t * d + c]);
#pragma unroll
                for (int jj = 0; jj < KU; ++jj) {
                    if (r8[jj] < 0) continue;
                    dot[jj] = fmaf(g, to_float(y[(size_t)r8[jj] * d + c]), dot[jj]);
                    if (dy) dy[(size_t)r8[jj] * d + c] = from_float<T>(w8[jj] * g);
                }
            }
        }
#pragma unroll
        for (int jj = 0; jj < KU; ++jj) {
            float v = dot[jj];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0) red[wave][jj] = v;
        }
        __syncthreads();
        if (threadIdx.x < KU && j0 + threadIdx.x < k)
            dw[(size_t)t * k + j0 + threadIdx.x] =
                ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
        __syncthreads();
    }
}

template <typename T>
static bool can_vec(int d, std::initializer_list<const void*> ptrs) {
    if (d % Vec16<T>::N != 0) return false;
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return false;
    return true;
}

template <typename T>
static int launch_dispatch(const void* x, const int32_t* token_ids, int Tn, int B, int d, void* xd, hipStream_t s) {
    dim3 grid((B + 3) / 4), block(256);
    if (can_vec<T>(d, {x, xd}))
        XMOE_LAUNCH(K_DISPATCH, s, hipLaunchKernelGGL((dispatch_kernel<T, true>), grid, block, 0, s, (const T*)x,
                                                      token_ids, Tn, B, d, (T*)xd));
    else
        XMOE_LAUNCH(K_DISPATCH, s, hipLaunchKernelGGL((dispatch_kernel<T, false>), grid, block, 0, s, (const T*)x,
                                                      token_ids, Tn, B, d, (T*)xd));
    return XMOE_OK;
}

// slots unrolled per group: the smallest of 2, 4, 6, 8 that covers k (8 for larger k)
#define XMOE_DISPATCH_KU(k, CALL)  \
    do {                           \
        if ((k) <= 2) { CALL(2); } \
        else if ((k) <= 4) { CALL(4); } \
        else if ((k) <= 6) { CALL(6); } \
        else { CALL(8); }          \
    } while (0)

template <typename T>
static int launch_combine(const void* y, const int32_t* ros, const float* w, const void* sh, int nsh,
                          const int32_t* sh_row0, const void* add, int Tn, int k, int d, void* out, hipStream_t s) {
    dim3 grid(Tn), block(256);
    const int B = Tn * k;
    if (can_vec<T>(d, {y, sh, add, out})) {
#define XMOE_CALL(KU)                                                                                                \
    XMOE_LAUNCH(K_COMBINE, s, hipLaunchKernelGGL((combine_kernel<T, true, KU>), grid, block, 0, s, (const T*)y, ros, \
                                                 w, (const T*)sh, nsh, sh_row0, (const T*)add, Tn, k, d, B, (T*)out))
        XMOE_DISPATCH_KU(k, XMOE_CALL);
#undef XMOE_CALL
    } else {
        XMOE_LAUNCH(K_COMBINE, s, hipLaunchKernelGGL((combine_kernel<T, false, 8>), grid, block, 0, s, (const T*)y,
                                                     ros, w, (const T*)sh, nsh, sh_row0, (const T*)add, Tn, k, d, B,
                                                     (T*)out));
    }
    return XMOE_OK;
}

template <typename T>
static int launch_combine_bwd(const void* dout, const void* y, const int32_t* ros, const float* w, int Tn, int k,
                              int d, void* dy, float* dw, hipStream_t s) {
    dim3 grid(Tn), block(256);
    const int B = Tn * k;
    if (can_vec<T>(d, {dout, y, dy})) {
#define XMOE_CALL(KU)                                                                                      \
    XMOE_LAUNCH(K_COMBINE_BWD, s, hipLaunchKernelGGL((combine_bwd_kernel<T, true, KU>), grid, block, 0, s, \
                                                     (const T*)dout, (const T*)y, ros, w, Tn, k, d, B, (T*)dy, dw))
        XMOE_DISPATCH_KU(k, XMOE_CALL);
#undef XMOE_CALL
    } else {
#define XMOE_CALL(KU)                                                                                       \
    XMOE_LAUNCH(K_COMBINE_BWD, s, hipLaunchKernelGGL((combine_bwd_kernel<T, false, KU>), grid, block, 0, s, \
                                                     (const T*)dout, (const T*)y, ros, w, Tn, k, d, B, (T*)dy, dw))
        XMOE_DISPATCH_KU(k, XMOE_CALL);
#undef XMOE_CALL
    }
    return XMOE_OK;
}

// dw[n] = row_grad[row_of_slot[n]], 0 for a dropped entry
__global__ __launch_bounds__(256) void combine_bwd_weights_kernel(const float* __restrict__ row_grad,
                                                                  const int32_t* __restrict__ ros, int n,
                                                                  float* __restrict__ dw) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int r = ros[i];
    dw[i] = r >= 0 ? row_grad[r] : 0.f;
}

static int check_rows_args(int T, int k, int d, int dt) {
    if (!dtype_ok(dt)) return XMOE_ERR_UNSUPPORTED;
    if (T < 0 || k < 1 || d < 1) return XMOE_ERR_INVALID_ARG;
    if ((long long)T * k >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    return XMOE_OK;
}

}  // namespace xmoe

using namespace xmoe;

extern "C" {

int xmoe_dispatch(const void* x, const int32_t* token_ids, int T, int B, int d, int dt, void* xd, void* stream) {
    if (!dtype_ok(dt)) return XMOE_ERR_UNSUPPORTED;
    if (T < 0 || B < 0 || d < 1) return XMOE_ERR_INVALID_ARG;
    if (B == 0) return XMOE_OK;
    if (T == 0 || !x || !token_ids || !xd) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    return dt == XMOE_F32 ? launch_dispatch<float>(x, token_ids, T, B, d, xd, s)
                          : launch_dispatch<bf16_t>(x, token_ids, T, B, d, xd, s);
}

int xmoe_combine(const void* y, const int32_t* row_of_slot, const float* topk_w, const void* shared_rows,
                 int n_shared, const int32_t* shared_row0, const void* addend, int T, int k, int d, int dt, void* out,
                 void* stream) {
    int st = check_rows_args(T, k, d, dt);
    if (st != XMOE_OK) return st;
    if (n_shared < 0 || (n_shared > 0 && !shared_rows)) return XMOE_ERR_INVALID_ARG;
    if (T == 0) return XMOE_OK;
    if (!y || !row_of_slot || !out) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    return dt == XMOE_F32
               ? launch_combine<float>(y, row_of_slot, topk_w, shared_rows, n_shared, shared_row0, addend, T, k, d, out,
                                       s)
               : launch_combine<bf16_t>(y, row_of_slot, topk_w, shared_rows, n_shared, shared_row0, addend, T, k, d,
                                        out, s);
}

int xmoe_dispatch_bwd(const void* dxd, const int32_t* row_of_slot, const void* shared_rows, int n_shared,
                      const int32_t* shared_row0, const void* addend, int T, int k, int d, int dt, void* dx,
                      void* stream) {
    return xmoe_combine(dxd, row_of_slot, nullptr, shared_rows, n_shared, shared_row0, addend, T, k, d, dt, dx, stream);
}

int xmoe_combine_bwd(const void* dout, const void* y, const int32_t* row_of_slot, const float* topk_w, int T, int k,
                     int d, int dt, void* dy, float* dw, void* stream) {
    int st = check_rows_args(T, k, d, dt);
    if (st != XMOE_OK) return st;
    if (T == 0) return XMOE_OK;
    if (!dout || !y || !row_of_slot || !dw || (dy && !topk_w)) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    return dt == XMOE_F32 ? launch_combine_bwd<float>(dout, y, row_of_slot, topk_w, T, k, d, dy, dw, s)
                          : launch_combine_bwd<bf16_t>(dout, y, row_of_slot, topk_w, T, k, d, dy, dw, s);
}

int xmoe_combine_bwd_weights(const float* row_grad, const int32_t* row_of_slot, int T, int k, float* dw,
                             void* stream) {
    if (T < 0 || k < 1 || (long long)T * k >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (T == 0) return XMOE_OK;
    if (!row_grad || !row_of_slot || !dw) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int n = T * k;
    XMOE_LAUNCH(K_COMBINE_BWD_W, s,
                hipLaunchKernelGGL(combine_bwd_weights_kernel, dim3((n + 255) / 256), dim3(256), 0, s, row_grad,
                                   row_of_slot, n, dw));
    return XMOE_OK;
}

}  // extern "C"
