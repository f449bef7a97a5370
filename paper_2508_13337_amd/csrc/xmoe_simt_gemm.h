// A plain float32-ALU GEMM tile: 64x64 outputs per 256-thread block, K stepped by 16 through LDS.
// Serves the float32 workloads, shapes the MFMA kernels do not cover, and the small gate-projection GEMMs.
#pragma once

#include "xmoe_internal.h"

namespace xmoe {

constexpr int kSimtTile = 64;   // rows and columns per block
constexpr int kSimtBK = 16;

struct SimtSmem {
    float a[kSimtBK][kSimtTile + 4];
    float b[kSimtBK][kSimtTile + 4];
};

// Accumulates acc[i][j] += sum_k A(m,k) * B(k,n) for the thread's 4x4 patch (rows ty*4+i, cols tx*4+j, with
// tx = tid % 16, ty = tid / 16), k ascending.  loadA(m_local, k) and loadB(k, n_local) return 0 outside the
// operand.  A_K_FAST / B_N_FAST choose which index runs along consecutive threads while staging (pick the one
// that is contiguous in memory).
template <bool A_K_FAST, bool B_N_FAST, class LoadA, class LoadB>
__device__ __forceinline__ void simt_mainloop(float (&acc)[4][4], int K, SimtSmem& sm, LoadA loadA, LoadB loadB) {
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    for (int k0 = 0; k0 < K; k0 += kSimtBK) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int idx = tid + 256 * r;
            int kk, mm;
            if (A_K_FAST) { kk = idx & 15; mm = idx >> 4; } else { mm = idx & 63; kk = idx >> 6; }
            sm.a[kk][mm] = (k0 + kk < K) ? loadA(mm, k0 + kk) : 0.f;
            int kb, nn;
            if (B_N_FAST) { nn = idx & 63; kb = idx >> 6; } else { kb = idx & 15; nn = idx >> 4; }
            sm.b[kb][nn] = (k0 + kb < K) ? loadB(k0 + kb, nn) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kSimtBK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = sm.a[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = sm.b[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
}

}  // namespace xmoe
