// Stage 0 of the Redundancy-Bypassing Dispatch (paper: Section 4.2, "Pilot Selection and Instantiation"): the rows
// of a PFT are split into pilot tokens - one per token and destination node - and local replicas, each group gets
// its own ERI-arrays, and every replica records where its pilot sits (s1_mapping_indices).  Integer work only.
//   1. mark:    per flat entry n = t*k + j, look at the token's k experts; the entry is its group's pilot if no other
//               entry of the group (same token, same destination node) has a smaller (rand_key, n)
//   2. count:   pilots per chunk of 1024 PFT rows
//   3. scan:    exclusive prefix over the chunks
//   4. scatter: pilot_prefix[i] = pilots before row i; rows go to the pilot or the replica arrays at their rank,
//               which keeps the PFT's order (sorted by expert, ascending token inside an expert)
//   5. map:     per-expert offsets of both groups, the replicas' relative pilot indices, the merge order, sentinels
#include "xmoe_internal.h"
#include "xmoe_sizes.h"

namespace xmoe {

constexpr int kRbdChunk = 1024;

// flag[row] = 1 if the row is a pilot; pilot_row[row] = PFT row of the pilot of the row's group
__global__ __launch_bounds__(256) void rbd_mark_kernel(const int32_t* __restrict__ topk_idx,
                                                       const uint32_t* __restrict__ rand_key,
                                                       const int32_t* __restrict__ row_of_slot, int B, int k,
                                                       int experts_per_node, int32_t* __restrict__ flag,
                                                       int32_t* __restrict__ pilot_row) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= B) return;
    const int t0 = (n / k) * k;
    const int node = topk_idx[n] / experts_per_node;
    uint32_t best_key = rand_key[n];
    int best = n;
    for (int j = 0; j < k; ++j) {
        const int m = t0 + j;
        if (topk_idx[m] / experts_per_node != node) continue;
        const uint32_t key = rand_key[m];
        if (key < best_key || (key == best_key && m < best)) {
            best_key = key;
            best = m;
        }
    }
    const int row = row_of_slot[n];
    flag[row] = best == n ? 1 : 0;
    pilot_row[row] = row_of_slot[best];
}

__global__ __launch_bounds__(256) void rbd_count_kernel(const int32_t* __restrict__ flag, int B,
                                                        int32_t* __restrict__ chunk_count) {
    __shared__ int part[4];
    const int base = blockIdx.x * kRbdChunk;
    int c = 0;
#pragma unroll
    for (int r = 0; r < kRbdChunk / 256; ++r) {
        const int i = base + r * 256 + threadIdx.x;
        c += (i < B) ? flag[i] : 0;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) chunk_count[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// one block: chunk_count -> exclusive prefix; chunk_count[nchunks] = total number of pilots
__global__ __launch_bounds__(1024) void rbd_scan_kernel(int32_t* __restrict__ chunk_count, int nchunks) {
    __shared__ int wave_tot[16];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int c0 = 0; c0 < nchunks; c0 += 1024) {
        const int c = c0 + threadIdx.x;
        const int v = c < nchunks ? chunk_count[c] : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = carry;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        if (c < nchunks) chunk_count[c] = before + incl - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) chunk_count[nchunks] = carry;
}

// pilot_prefix[i] = number of pilots among rows [0, i); pilot_prefix[B] = their total.  A row's rank inside its
// group is pilot_prefix[i] (pilot) or i - pilot_prefix[i] (replica).
__global__ __launch_bounds__(256) void rbd_scatter_kernel(const int32_t* __restrict__ flag,
                                                          const int32_t* __restrict__ chunk_base,
                                                          const int32_t* __restrict__ token_ids,
                                                          const int32_t* __restrict__ expert_ids, int B, int nchunks,
                                                          int32_t* __restrict__ pilot_prefix,
                                                          int32_t* __restrict__ pilot_token_ids,
                                                          int32_t* __restrict__ pilot_expert_ids,
                                                          int32_t* __restrict__ replica_token_ids,
                                                          int32_t* __restrict__ replica_expert_ids) {
    __shared__ int wave_cnt[kRbdChunk / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = blockIdx.x * kRbdChunk;
    int f[kRbdChunk / 256], before_in_wave[kRbdChunk / 256];
#pragma unroll
    for (int r = 0; r < kRbdChunk / 256; ++r) {
        const int i = base + (r * 4 + wave) * 64 + lane;   // sub-chunk r*4 + wave holds 64 consecutive rows
        f[r] = (i < B) ? flag[i] : 0;
        const unsigned long long m = __ballot(f[r] != 0);
        before_in_wave[r] = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[r * 4 + wave] = __popcll(m);
    }
    __syncthreads();
    const int cb = chunk_base[blockIdx.x];
#pragma unroll
    for (int r = 0; r < kRbdChunk / 256; ++r) {
        const int sub = r * 4 + wave;
        const int i = base + sub * 64 + lane;
        if (i >= B) continue;
        int before = cb + before_in_wave[r];
        for (int s = 0; s < sub; ++s) before += wave_cnt[s];
        pilot_prefix[i] = before;
        if (f[r]) {
            pilot_token_ids[before] = token_ids[i];
            pilot_expert_ids[before] = expert_ids[i];
        } else {
            replica_token_ids[i - before] = token_ids[i];
            replica_expert_ids[i - before] = expert_ids[i];
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) pilot_prefix[B] = chunk_base[nchunks];
}

__global__ __launch_bounds__(256) void rbd_map_kernel(const int32_t* __restrict__ flag,
                                                      const int32_t* __restrict__ pilot_row,
                                                      const int32_t* __restrict__ pilot_prefix,
                                                      const int32_t* __restrict__ expert_ids,
                                                      const int32_t* __restrict__ expert_offsets, int B, int E,
                                                      int32_t* __restrict__ pilot_tpe, int32_t* __restrict__ pilot_off,
                                                      int32_t* __restrict__ replica_tpe,
                                                      int32_t* __restrict__ replica_off,
                                                      int32_t* __restrict__ pilot_token_ids,
                                                      int32_t* __restrict__ pilot_expert_ids,
                                                      int32_t* __restrict__ replica_token_ids,
                                                      int32_t* __restrict__ replica_expert_ids,
                                                      int32_t* __restrict__ s1_indices,
                                                      int32_t* __restrict__ s1_experts,
                                                      int32_t* __restrict__ merge_src) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int n_pilot = pilot_prefix[B];
    if (i <= E) {
        const int lo = expert_offsets[i];
        const int p_lo = pilot_prefix[lo];
        pilot_off[i] = p_lo;
        replica_off[i] = lo - p_lo;
        if (i < E) {
            const int hi = expert_offsets[i + 1];
            const int p_hi = pilot_prefix[hi];
            pilot_tpe[i] = p_hi - p_lo;
            replica_tpe[i] = (hi - lo) - (p_hi - p_lo);
        }
    }
    if (i >= B) return;
    // entries behind the last pilot / the last replica: sentinels, as behind the retained rows of a capped PFT
    if (i >= n_pilot) {
        pilot_token_ids[i] = -1;
        pilot_expert_ids[i] = E;
    }
    if (i >= B - n_pilot) {
        replica_token_ids[i] = -1;
        replica_expert_ids[i] = E;
        s1_indices[i] = -1;
        s1_experts[i] = E;
    }
    const int before = pilot_prefix[i];
    if (flag[i]) {
        merge_src[i] = before;
    } else {
        const int r = i - before;
        const int ip = pilot_row[i];
        const int pe = expert_ids[ip];
        s1_indices[r] = pilot_prefix[ip] - pilot_prefix[expert_offsets[pe]];
        s1_experts[r] = pe;
        merge_src[i] = n_pilot + r;
    }
}

// absolute[r] = offsets[experts[r]] + relative[r]; entries whose expert is the sentinel E give -1
__global__ __launch_bounds__(256) void rbd_absolute_kernel(const int32_t* __restrict__ relative,
                                                           const int32_t* __restrict__ experts,
                                                           const int32_t* __restrict__ offsets, int n, int E,
                                                           int32_t* __restrict__ absolute) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    const int e = experts[r];
    absolute[r] = ((unsigned)e < (unsigned)E) ? offsets[e] + relative[r] : -1;
}

}  // namespace xmoe

using namespace xmoe;

extern "C" {

int xmoe_rbd_stage0(const int32_t* topk_idx, const uint32_t* rand_key, const int32_t* token_ids,
                    const int32_t* expert_ids, const int32_t* expert_offsets, const int32_t* row_of_slot, int T, int E,
                    int k, int experts_per_node, int32_t* pilot_token_ids, int32_t* pilot_expert_ids,
                    int32_t* pilot_tokens_per_expert, int32_t* pilot_offsets, int32_t* replica_token_ids,
                    int32_t* replica_expert_ids, int32_t* replica_tokens_per_expert, int32_t* replica_offsets,
                    int32_t* s1_mapping_indices, int32_t* s1_mapping_experts, int32_t* merge_src, void* ws,
                    size_t ws_bytes, void* stream) {
    if (T < 0 || E < 1 || k < 1 || k > E || experts_per_node < 1) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS) return XMOE_ERR_UNSUPPORTED;
    if ((long long)T * k >= (1ll << 31)) return XMOE_ERR_INVALID_ARG;
    if (!expert_offsets || !pilot_tokens_per_expert || !pilot_offsets || !replica_tokens_per_expert ||
        !replica_offsets)
        return XMOE_ERR_INVALID_ARG;
    const int B = T * k;
    if (B > 0 && (!topk_idx || !rand_key || !token_ids || !expert_ids || !row_of_slot || !pilot_token_ids ||
                  !pilot_expert_ids || !replica_token_ids || !replica_expert_ids || !s1_mapping_indices ||
                  !s1_mapping_experts || !merge_src))
        return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < rbd_ws_bytes(T, k)) return XMOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int nchunks = rbd_num_chunks(B);
    char* p = (char*)ws;
    int32_t* flag = (int32_t*)p;
    p += align_up((size_t)(B > 0 ? B : 1) * sizeof(int32_t), 256);
    int32_t* pilot_row = (int32_t*)p;
    p += align_up((size_t)(B > 0 ? B : 1) * sizeof(int32_t), 256);
    int32_t* pilot_prefix = (int32_t*)p;
    p += align_up((size_t)(B + 1) * sizeof(int32_t), 256);
    int32_t* chunk_count = (int32_t*)p;
    const unsigned gB = (unsigned)((B + 255) / 256);
    if (B > 0) {
        XMOE_LAUNCH(K_RBD_MARK, s, hipLaunchKernelGGL(rbd_mark_kernel, dim3(gB), dim3(256), 0, s, topk_idx, rand_key,
                                                      row_of_slot, B, k, experts_per_node, flag, pilot_row));
        XMOE_LAUNCH(K_RBD_COUNT, s, hipLaunchKernelGGL(rbd_count_kernel, dim3(nchunks), dim3(256), 0, s, flag, B,
                                                       chunk_count));
    }
    XMOE_LAUNCH(K_RBD_SCAN, s, hipLaunchKernelGGL(rbd_scan_kernel, dim3(1), dim3(1024), 0, s, chunk_count, nchunks));
    if (B > 0)
        XMOE_LAUNCH(K_RBD_SCATTER, s,
                    hipLaunchKernelGGL(rbd_scatter_kernel, dim3(nchunks), dim3(256), 0, s, flag, chunk_count, token_ids,
                                       expert_ids, B, nchunks, pilot_prefix, pilot_token_ids, pilot_expert_ids,
                                       replica_token_ids, replica_expert_ids));
    else
        XMOE_LAUNCH(K_RBD_SCATTER, s,
                    hipLaunchKernelGGL(rbd_scatter_kernel, dim3(1), dim3(256), 0, s, flag, chunk_count, token_ids,
                                       expert_ids, 0, 0, pilot_prefix, pilot_token_ids, pilot_expert_ids,
                                       replica_token_ids, replica_expert_ids));
    const int nmap = B > E + 1 ? B : E + 1;
    XMOE_LAUNCH(K_RBD_MAP, s,
                hipLaunchKernelGGL(rbd_map_kernel, dim3((unsigned)((nmap + 255) / 256)), dim3(256), 0, s, flag,
                                   pilot_row, pilot_prefix, expert_ids, expert_offsets, B, E, pilot_tokens_per_expert,
                                   pilot_offsets, replica_tokens_per_expert, replica_offsets, pilot_token_ids,
                                   pilot_expert_ids, replica_token_ids, replica_expert_ids, s1_mapping_indices,
                                   s1_mapping_experts, merge_src));
    return XMOE_OK;
}

int xmoe_rbd_absolute_index(const int32_t* s1_mapping_indices, const int32_t* s1_mapping_experts,
                            const int32_t* pilot_offsets_at_destination, int n, int E, int32_t* absolute,
                            void* stream) {
    if (n < 0 || E < 1) return XMOE_ERR_INVALID_ARG;
    if (n == 0) return XMOE_OK;
    if (!s1_mapping_indices || !s1_mapping_experts || !pilot_offsets_at_destination || !absolute)
        return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    XMOE_LAUNCH(K_RBD_ABS, s,
                hipLaunchKernelGGL(rbd_absolute_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                                   s1_mapping_indices, s1_mapping_experts, pilot_offsets_at_destination, n, E,
                                   absolute));
    return XMOE_OK;
}

}  // extern "C"
