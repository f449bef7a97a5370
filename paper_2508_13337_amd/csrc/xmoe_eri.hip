// PFT construction (paper: Listing 1 PFT_construction() step 1 + histogram; Section 4.1.1 ERI-arrays):
// a stable counting sort of the T*k flat entries by expert id, in three small kernels.
//   1. per-chunk histograms of expert ids            (chunk = 1024 consecutive flat entries)
//   2. column scan over chunks + scan over experts   -> tokens_per_expert, expert_offsets, chunk bases
//   3. per-chunk stable ranking and scatter          -> token_ids, expert_ids, combine_weights, row_of_slot
// Within an expert, rows keep ascending flat order, so the result is unique and reproducible.
#include "xmoe_internal.h"
#include "xmoe_sizes.h"

namespace xmoe {

constexpr int kSubPerChunk = kEriChunk / 64;   // 16 wave-sized sub-chunks

__global__ __launch_bounds__(256) void eri_hist_kernel(const int32_t* __restrict__ topk_idx, int B, int E,
                                                       int32_t* __restrict__ chunk_counts) {
    __shared__ int hist[XMOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += 256) hist[e] = 0;
    __syncthreads();
    const int base = blockIdx.x * kEriChunk;
#pragma unroll
    for (int r = 0; r < kEriChunk / 256; ++r) {
        int n = base + r * 256 + threadIdx.x;
        if (n < B) {
            int e = topk_idx[n];
            if ((unsigned)e < (unsigned)E) atomicAdd(&hist[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) chunk_counts[(size_t)blockIdx.x * E + e] = hist[e];
}

// one block: turns chunk_counts[c][e] into the exclusive prefix over chunks, writes tokens_per_expert and
// expert_offsets
__global__ __launch_bounds__(512) void eri_scan_kernel(int32_t* __restrict__ chunk_counts, int nchunks, int E,
                                                       int32_t* __restrict__ tokens_per_expert,
                                                       int32_t* __restrict__ expert_offsets) {
    __shared__ int tot[XMOE_MAX_EXPERTS];
    const int e = threadIdx.x;
    if (e < E) {
        // 16 chunks at a time: the loads of a batch are independent, so the walk costs nchunks/16 round trips to
        // memory instead of nchunks
        constexpr int kBatch = 16;
        int run = 0;
        for (int c0 = 0; c0 < nchunks; c0 += kBatch) {
            int v[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) v[j] = c0 + j < nchunks ? chunk_counts[(size_t)(c0 + j) * E + e] : 0;
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (c0 + j < nchunks) chunk_counts[(size_t)(c0 + j) * E + e] = run;
                run += v[j];
            }
        }
        tot[e] = run;
        tokens_per_expert[e] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < E; ++i) {
            expert_offsets[i] = run;
            run += tot[i];
        }
        expert_offsets[E] = run;
    }
}

// FLAT: the intermediate table of the token-dropping construction: token_ids receives the flat entry n itself,
// expert_ids and row_of_slot are not written.
template <bool FLAT>
__global__ __launch_bounds__(256) void eri_scatter_kernel(const int32_t* __restrict__ topk_idx,
                                                          const float* __restrict__ topk_w, int B, int E, int k,
                                                          int ebits, const int32_t* __restrict__ chunk_prefix,
                                                          const int32_t* __restrict__ expert_offsets,
                                                          int32_t* __restrict__ token_ids,
                                                          int32_t* __restrict__ expert_ids,
                                                          float* __restrict__ combine_weights,
                                                          int32_t* __restrict__ row_of_slot) {
    // sub_count[s][e]: entries of expert e in sub-chunk s; turned into an exclusive prefix over s
    extern __shared__ int sub_count[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kSubPerChunk * E; i += 256) sub_count[i] = 0;
    __syncthreads();

    const int base = blockIdx.x * kEriChunk;
    int my_e[kSubPerChunk / 4], my_rank[kSubPerChunk / 4];
#pragma unroll
    for (int r = 0; r < kSubPerChunk / 4; ++r) {
        const int sub = r * 4 + wave;
        const int n = base + sub * 64 + lane;
        const int e = n < B ? topk_idx[n] : -1;
        const bool ok = (unsigned)e < (unsigned)E;   // out-of-range ids (never produced by xmoe_route) are skipped
        // lanes of this wave holding the same expert: intersect ballots bit by bit
        unsigned long long same = __ballot(ok);
        for (int b = 0; b < ebits; ++b) {
            unsigned long long bal = __ballot(ok && ((e >> b) & 1));
            same &= ((e >> b) & 1) ? bal : ~bal;
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        my_e[r] = e;
        my_rank[r] = __popcll(same & below);
        if (ok && (same & below) == 0ull) sub_count[sub * E + e] = __popcll(same);   // first lane of its group
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) {
        int run = chunk_prefix[(size_t)blockIdx.x * E + e] + expert_offsets[e];
#pragma unroll
        for (int s2 = 0; s2 < kSubPerChunk; ++s2) {
            int v = sub_count[s2 * E + e];
            sub_count[s2 * E + e] = run;
            run += v;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSubPerChunk / 4; ++r) {
        const int sub = r * 4 + wave;
        const int n = base + sub * 64 + lane;
        const int e = my_e[r];
        if (n < B && (unsigned)e < (unsigned)E) {
            const int row = sub_count[sub * E + e] + my_rank[r];
            combine_weights[row] = topk_w[n];
            if (FLAT) {
                token_ids[row] = n;
            } else {
                token_ids[row] = n / k;
                expert_ids[row] = e;
                row_of_slot[n] = row;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Token dropping (paper: Listing 1 PFT_construction() step 2; Appendix B.2): every expert keeps at most C rows, the
// ones with the largest combine weights, equal weights keeping the lower flat entry first.  Input is the dropless
// table (rows sorted by expert, ascending flat entry inside an expert): so "lower flat entry" is "earlier row", and
// the survivors, taken in row order, are already in their final order.
// Block e < E handles expert e: a three-pass radix select over the order-preserving bit pattern of the weights
// finds the C-th largest weight, then the segment is compacted in row order.  Blocks >= E write the sentinels of
// the rows behind the last retained one.  No floating-point arithmetic takes part in the decision.
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t weight_key(float w) {
    uint32_t u = __float_as_uint(w);
    if (u == 0x80000000u) u = 0u;                          // -0.0 ties with +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // ascending in w
}

// exclusive prefix of `flag` over the block's 256 threads in thread order; total in *total
__device__ __forceinline__ int block_excl_count(bool flag, int* wave_tot, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long bal = __ballot(flag);
    const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
    __syncthreads();   // wave_tot may still be read from the previous call
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    *total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    return before + in_wave;
}

// exclusive prefix of `v` over the block's 256 threads in thread order; total in *total
__device__ __forceinline__ int block_excl_sum(int v, int* wave_tot, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(inc, o, 64);
        if (lane >= o) inc += up;
    }
    __syncthreads();   // wave_tot may still be read from the previous call
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    *total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    return before + inc - v;
}

__global__ __launch_bounds__(256) void eri_cap_kernel(const int32_t* __restrict__ off0,      // dropless offsets [E+1]
                                                      const int32_t* __restrict__ flat0,     // flat entry of row [B]
                                                      const float* __restrict__ w0,          // weight of row [B]
                                                      int B, int E, int k, int C,
                                                      int32_t* __restrict__ tokens_per_expert,
                                                      int32_t* __restrict__ expert_offsets,
                                                      int32_t* __restrict__ token_ids,
                                                      int32_t* __restrict__ expert_ids,
                                                      float* __restrict__ combine_weights,
                                                      int32_t* __restrict__ row_of_slot) {
    __shared__ int hist[2048];
    __shared__ int wave_tot[4];
    __shared__ uint32_t s_prefix, s_mask;
    __shared__ int s_remaining, s_new_lo, s_kept_total;
    const int tid = threadIdx.x;
    // retained rows before this block's expert, and in total: every block recomputes the short prefix it needs
    {
        int before_me = 0, all = 0;
        for (int i = tid; i < E; i += 256) {
            const int n = off0[i + 1] - off0[i];
            const int c = n < C ? n : C;
            all += c;
            if (i < (int)blockIdx.x) before_me += c;
        }
        int tot_before, tot_all;
        block_excl_sum(before_me, wave_tot, &tot_before);
        block_excl_sum(all, wave_tot, &tot_all);
        if (tid == 0) {
            s_new_lo = tot_before;
            s_kept_total = tot_all;
        }
    }
    __syncthreads();
    const int kept_total = s_kept_total;
    if ((int)blockIdx.x >= E) {
        // rows behind the last retained one
        const int base = ((int)blockIdx.x - E) * kEriChunk;
        for (int r = base + tid; r < base + kEriChunk && r < B; r += 256) {
            if (r >= kept_total) {
                token_ids[r] = -1;
                expert_ids[r] = E;
                combine_weights[r] = 0.0f;
            }
        }
        return;
    }
    const int e = blockIdx.x;
    const int lo = off0[e], n = off0[e + 1] - lo;
    const int new_lo = s_new_lo;
    const int keep_n = n < C ? n : C;
    if (tid == 0) {
        tokens_per_expert[e] = keep_n;
        expert_offsets[e] = new_lo;
        if (e == E - 1) expert_offsets[E] = kept_total;
    }
    // the C-th largest key of the segment (only needed when something is dropped)
    uint32_t vstar = 0;
    int need_eq = 0;   // how many rows with key == vstar are kept
    if (n > C && C > 0) {
        if (tid == 0) {
            s_prefix = 0;
            s_mask = 0;
            s_remaining = C;
        }
        const int shifts[3] = {21, 10, 0}, widths[3] = {11, 11, 10};
        for (int p = 0; p < 3; ++p) {
            const int shift = shifts[p], nb = 1 << widths[p];
            for (int i = tid; i < nb; i += 256) hist[i] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix, mask = s_mask;
            for (int i = tid; i < n; i += 256) {
                const uint32_t key = weight_key(w0[lo + i]);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (nb - 1)], 1);
            }
            __syncthreads();
            // which bin holds the `remaining`-th largest key: thread t owns the bins nb-1 - t*bpt .. (downwards);
            // an exclusive prefix of the threads' sums, then the one thread whose range the target falls into
            // walks its few bins
            {
                const int bpt = nb / 256;
                const int hi = nb - 1 - tid * bpt;
                int mine = 0;
                for (int j = 0; j < bpt; ++j) mine += hist[hi - j];
                int tot_unused;
                const int before = block_excl_sum(mine, wave_tot, &tot_unused);
                const int remaining = s_remaining;
                __syncthreads();   // everyone has read s_remaining before the owner overwrites it
                if (before < remaining && remaining <= before + mine) {
                    int rem = remaining - before, b = hi;
                    while (hist[b] < rem) {
                        rem -= hist[b];
                        --b;
                    }
                    s_remaining = rem;
                    s_prefix = prefix | ((uint32_t)b << shift);
                    s_mask = mask | ((uint32_t)(nb - 1) << shift);
                }
            }
            __syncthreads();
        }
        vstar = s_prefix;
        need_eq = s_remaining;
    }
    // compaction in row order
    int eq_seen = 0, kept_seen = 0;
    for (int base = 0; base < n; base += 256) {
        const int i = base + tid;
        const bool in = i < n;
        uint32_t key = 0;
        int flat = 0;
        float w = 0.f;
        if (in) {
            w = w0[lo + i];
            flat = flat0[lo + i];
            key = weight_key(w);
        }
        bool keep;
        if (n <= C) {
            keep = in;
        } else if (C <= 0) {
            keep = false;
        } else {
            const bool eq = in && key == vstar;
            int eq_total;
            const int eq_rank = eq_seen + block_excl_count(eq, wave_tot, &eq_total);
            eq_seen += eq_total;
            keep = in && (key > vstar || (eq && eq_rank < need_eq));
        }
        int kept_total_chunk;
        const int pos = kept_seen + block_excl_count(keep, wave_tot, &kept_total_chunk);
        kept_seen += kept_total_chunk;
        if (in) {
            if (keep) {
                const int row = new_lo + pos;
                token_ids[row] = flat / k;
                expert_ids[row] = e;
                combine_weights[row] = w;
                row_of_slot[flat] = row;
            } else {
                row_of_slot[flat] = -1;
            }
        }
    }
}

}  // namespace xmoe

using namespace xmoe;

// the three launches of the dropless construction; counts: eri_num_chunks(B) * E ints of scratch (every one of them is
// written by the histogram kernel before it is read, so the memory needs no clearing)
static int build_eri_launch(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                            int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                            int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot, int32_t* counts,
                            hipStream_t s) {
    const int B = T * k;
    const int nchunks = eri_num_chunks(B);
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    if (nchunks > 0)
        XMOE_LAUNCH(K_ERI_HIST, s,
                    hipLaunchKernelGGL(eri_hist_kernel, dim3(nchunks), dim3(256), 0, s, topk_idx, B, E, counts));
    XMOE_LAUNCH(K_ERI_SCAN, s,
                hipLaunchKernelGGL(eri_scan_kernel, dim3(1), dim3(512), 0, s, counts, nchunks, E, tokens_per_expert,
                                   expert_offsets));
    if (nchunks > 0)
        XMOE_LAUNCH(K_ERI_SCATTER, s,
                    hipLaunchKernelGGL(eri_scatter_kernel<false>, dim3(nchunks), dim3(256),
                                       (size_t)kSubPerChunk * E * sizeof(int), s, topk_idx, topk_w, B, E, k, ebits,
                                       counts, expert_offsets, token_ids, expert_ids, combine_weights, row_of_slot));
    return XMOE_OK;
}

static int build_eri_check(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                           int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                           int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot) {
    if (T < 0 || E < 1 || k < 1 || k > E) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS) return XMOE_ERR_UNSUPPORTED;
    if ((long long)T * k >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (!tokens_per_expert || !expert_offsets) return XMOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !topk_w || !token_ids || !expert_ids || !combine_weights || !row_of_slot))
        return XMOE_ERR_INVALID_ARG;
    return XMOE_OK;
}

extern "C" int xmoe_build_eri(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                              int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                              int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot, void* ws,
                              size_t ws_bytes, void* stream) {
    const int st = build_eri_check(topk_idx, topk_w, T, E, k, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                                   combine_weights, row_of_slot);
    if (st != XMOE_OK) return st;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < eri_ws_bytes(T, E, k)) return XMOE_ERR_WORKSPACE;
    return build_eri_launch(topk_idx, topk_w, T, E, k, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                            combine_weights, row_of_slot, (int32_t*)ws, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------------------
// xmoe_build_eri for callers that cannot allocate: the chunk histograms live in a static device array instead of a
// caller-provided workspace.  Every device holds its own copy of the array at its own address, looked up once per
// device (hipGetSymbolAddress with that device current); host code only ever uses that address.
// ---------------------------------------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[XMOE_STATIC_ERI_SCRATCH_BYTES / sizeof(int32_t)];

namespace {
constexpr int kMaxScratchDevices = 64;
int32_t* g_scratch_ptr[kMaxScratchDevices];   // device address of `scratch` on device i, or NULL before the first call there

int scratch_for_current_device(int32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return XMOE_ERR_HIP;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return XMOE_ERR_HIP;
        g_scratch_ptr[dev] = static_cast<int32_t*>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return XMOE_OK;
}
}  // namespace

extern "C" int xmoe_build_eri_static(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                                     int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                                     int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot,
                                     void* stream) {
    const int st = build_eri_check(topk_idx, topk_w, T, E, k, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                                   combine_weights, row_of_slot);
    if (st != XMOE_OK) return st;
    if (eri_ws_bytes(T, E, k) > (size_t)XMOE_STATIC_ERI_SCRATCH_BYTES) return XMOE_ERR_WORKSPACE;
    int32_t* counts = nullptr;
    const int sp = scratch_for_current_device(&counts);
    if (sp != XMOE_OK) return sp;
    return build_eri_launch(topk_idx, topk_w, T, E, k, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                            combine_weights, row_of_slot, counts, (hipStream_t)stream);
}

// Segments of n all-token experts directly behind the PFT's last row, which only the device knows after token
// dropping: offsets[E + 1 + s] = offsets[E] + (s+1)*T, and for the rows of those segments token id t and weight 1.
__global__ __launch_bounds__(256) void shared_segments_kernel(int32_t* __restrict__ offsets,
                                                              int32_t* __restrict__ token_ids,
                                                              float* __restrict__ combine_weights, int T, int E,
                                                              int n) {
    const int base = offsets[E];
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i < (long)n * T) {
        token_ids[base + i] = (int)(i % T);
        combine_weights[base + i] = 1.0f;
    }
    if (i < n) offsets[E + 1 + i] = base + ((int)i + 1) * T;
}

extern "C" int xmoe_append_shared_segments(int32_t* expert_offsets, int32_t* token_ids, float* combine_weights, int T,
                                           int E, int n_shared, void* stream) {
    if (T < 0 || E < 1 || n_shared < 0) return XMOE_ERR_INVALID_ARG;
    if ((long long)T * n_shared >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (n_shared == 0) return XMOE_OK;
    if (!expert_offsets || (T > 0 && (!token_ids || !combine_weights))) return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const long n = (long)n_shared * T > n_shared ? (long)n_shared * T : n_shared;
    XMOE_LAUNCH(K_SHARED_SEGMENTS, s,
                hipLaunchKernelGGL(shared_segments_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                                   expert_offsets, token_ids, combine_weights, T, E, n_shared));
    return XMOE_OK;
}

extern "C" int xmoe_build_eri_capped(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                                     int max_token_count, int32_t* tokens_per_expert, int32_t* expert_offsets,
                                     int32_t* token_ids, int32_t* expert_ids, float* combine_weights,
                                     int32_t* row_of_slot, void* ws, size_t ws_bytes, void* stream) {
    if (T < 0 || E < 1 || k < 1 || k > E || max_token_count < 0) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS) return XMOE_ERR_UNSUPPORTED;
    if ((long long)T * k >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (!tokens_per_expert || !expert_offsets) return XMOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !topk_w || !token_ids || !expert_ids || !combine_weights || !row_of_slot))
        return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < eri_capped_ws_bytes(T, E, k))
        return XMOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int B = T * k;
    const int nchunks = eri_num_chunks(B);
    // workspace: chunk histograms | dropless offsets [E+1] | dropless counts [E] | flat entry of row [B] | weight of row [B]
    char* p = (char*)ws;
    int32_t* counts = (int32_t*)p;
    p += eri_ws_bytes(T, E, k);
    int32_t* off0 = (int32_t*)p;
    p += align_up((size_t)(E + 1) * sizeof(int32_t), 256);
    int32_t* tpe0 = (int32_t*)p;
    p += align_up((size_t)E * sizeof(int32_t), 256);
    int32_t* flat0 = (int32_t*)p;
    p += align_up((size_t)(B > 0 ? B : 1) * sizeof(int32_t), 256);
    float* w0 = (float*)p;
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    if (nchunks > 0)
        XMOE_LAUNCH(K_ERI_HIST, s,
                    hipLaunchKernelGGL(eri_hist_kernel, dim3(nchunks), dim3(256), 0, s, topk_idx, B, E, counts));
    XMOE_LAUNCH(K_ERI_SCAN, s,
                hipLaunchKernelGGL(eri_scan_kernel, dim3(1), dim3(512), 0, s, counts, nchunks, E, tpe0, off0));
    if (nchunks > 0)
        XMOE_LAUNCH(K_ERI_SCATTER, s,
                    hipLaunchKernelGGL(eri_scatter_kernel<true>, dim3(nchunks), dim3(256),
                                       (size_t)kSubPerChunk * E * sizeof(int), s, topk_idx, topk_w, B, E, k, ebits,
                                       counts, off0, flat0, nullptr, w0, nullptr));
    XMOE_LAUNCH(K_ERI_CAP, s,
                hipLaunchKernelGGL(eri_cap_kernel, dim3(E + nchunks), dim3(256), 0, s, off0, flat0, w0, B, E, k,
                                   max_token_count, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                                   combine_weights, row_of_slot));
    return XMOE_OK;
}
