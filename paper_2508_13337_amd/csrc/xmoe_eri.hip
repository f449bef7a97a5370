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
        int run = 0;
        for (int c = 0; c < nchunks; ++c) {
            int v = chunk_counts[(size_t)c * E + e];
            chunk_counts[(size_t)c * E + e] = run;
            run += v;
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
            token_ids[row] = n / k;
            expert_ids[row] = e;
            combine_weights[row] = topk_w[n];
            row_of_slot[n] = row;
        }
    }
}

}  // namespace xmoe

using namespace xmoe;

extern "C" int xmoe_build_eri(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                              int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                              int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot, void* ws,
                              size_t ws_bytes, void* stream) {
    if (T < 0 || E < 1 || k < 1 || k > E) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS) return XMOE_ERR_UNSUPPORTED;
    if ((long long)T * k >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (!tokens_per_expert || !expert_offsets) return XMOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !topk_w || !token_ids || !expert_ids || !combine_weights || !row_of_slot))
        return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < eri_ws_bytes(T, E, k)) return XMOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int B = T * k;
    const int nchunks = eri_num_chunks(B);
    int32_t* counts = (int32_t*)ws;
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
                    hipLaunchKernelGGL(eri_scatter_kernel, dim3(nchunks), dim3(256),
                                       (size_t)kSubPerChunk * E * sizeof(int), s, topk_idx, topk_w, B, E, k, ebits,
                                       counts, expert_offsets, token_ids, expert_ids, combine_weights, row_of_slot));
    return XMOE_OK;
}
