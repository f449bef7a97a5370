// Expert MLP over ragged segments (paper: Listing 1 mlp(); Appendix B.4 "Sequential GeMM") on the gfx950 matrix
// cores, with operand tiles streamed straight from global memory into LDS (global_load_lds_dwordx4) through a
// 4-stage ring, so that no tile ever passes through registers and three K-steps of loads are always in flight.
//
//   block = 512 threads = 8 waves (2 x 4); block tile 256 x 256, K stepped by 32; wave tile 128 x 64 =
//   4 x 2 tiles of v_mfma_f32_32x32x16_bf16 with float32 accumulators; one block per CU (128 KiB of LDS for the
//   ring, 8 KiB for the index buffers of gathered operands).
//
// Two LDS tile layouts, chosen by which index of the operand is contiguous in memory:
//   K-contiguous operand ("row" tile): [256 rows][32 k], 64-byte rows; fragments are read with ds_read_b128.
//   K-strided operand    ("col" tile): [32 k][256 n], 512-byte rows, kept as it lies in memory; fragments are read
//                                       with the transposing LDS read ds_read_b64_tr_b16, so neither the weights
//                                       stored "in x out" nor the operands of the weight-gradient GEMMs are ever
//                                       transposed by ALU code.
// A direct-to-LDS load writes lane l's 16 bytes at (wave-uniform base) + 16*l, so the bank-conflict-avoiding XOR
// swizzle is applied on the global-address side (which 16-byte chunk a lane fetches) and undone by the fragment
// reads.  Rows / columns / k-indices outside the operand fetch a 16-byte block of zeros instead, so a ragged tail
// costs no branch and no padded row ever exists in HBM.
//
// The MFMA is issued with the operands swapped (B fragment first), so a lane ends up with 4 consecutive output
// columns of one row; results are rounded to bf16, staged through LDS and written with row-contiguous stores.
#include <stdlib.h>

#include "xmoe_ffn.h"

namespace xmoe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int TM = 256, TN = 256, TK = 32;
#ifndef XMOE_DMA_STAGES
#define XMOE_DMA_STAGES 4
#endif
constexpr int kStages = XMOE_DMA_STAGES;
#ifndef XMOE_RC_RING
#define XMOE_RC_RING 1
#endif
#ifndef XMOE_DEEP_PROLOGUE
#define XMOE_DEEP_PROLOGUE 1
#endif
constexpr int kOpBytes = 256 * TK * 2;          // one operand tile of one stage: 16 KiB
constexpr int kStageBytes = 2 * kOpBytes;       // A + B
// Behind the ring: the index buffers of the gathered K-strided operands (see Loader), per operand and wave two chunks
// of kIdxChunk k-tiles x 4 k-rows x 4 bytes.
constexpr int kIdxChunk = 16;
constexpr int kIdxChunkBytes = kIdxChunk * 4 * 4;             // 256 bytes: one direct-to-LDS dword load of a wave
constexpr int kIdxWaveBytes = 2 * kIdxChunkBytes;
constexpr int kIdxBytes = 2 * 8 * kIdxWaveBytes;              // two operands x eight waves: 8 KiB
constexpr int kIdxScalarTiles = kStages;                      // k-tiles 0 .. kStages-1 of a tile take their rows by scalar loads
// The GEMMs whose two operands are both K-contiguous run a ring of five 32 KiB units instead (mainloop_rr): all of a
// CU's 160 KiB.
constexpr int kUnitBytes = 256 * 64 * 2;                      // one operand, 256 rows x 64 k
constexpr int kUnits = 5;
constexpr int kLdsBytes = kUnits * kUnitBytes;                // 160 KiB
static_assert(kStages * kStageBytes + kIdxBytes <= kLdsBytes && kLdsBytes <= 160 * 1024, "LDS of one CU");
constexpr int kLoadsPerTile = 4;                // per thread: 2 for A, 2 for B
constexpr int kNumXcd = 8;

__device__ __align__(16) const unsigned int kZero16[4] = {0u, 0u, 0u, 0u};
__device__ const float kOneF = 1.0f;

// Shader clock under load: workgroup 0 of every launch of this family notes the shader-clock counter and the
// constant 100 MHz counter when it starts and when it leaves (it is persistent, so that spans the launch); the
// ratio is the clock the kernel really ran at (xmoe_prof_shader_clock).  One slot per kernel of the family.
enum ClockSlot { CS_GATEUP = 0, CS_DOWN, CS_DACT, CS_DX, CS_WGRAD, CS_WGRAD_DUAL, CS_MLP2_UP, CS_MLP2_DACT, CS_BWD_REST,
                 CS_COUNT };
__device__ unsigned long long g_clock_probe[CS_COUNT][4];
// clk: the kernel's slot of g_clock_probe while the launch profiler is enabled, else NULL (nothing is written then,
// so launches on different streams share no device memory outside their arguments)
__device__ __forceinline__ void clock_note(unsigned long long* clk, int at_end) {
    if (clk && blockIdx.x == 0 && threadIdx.x == 0) {
        clk[2 * at_end] = clock64();
        clk[2 * at_end + 1] = wall_clock64();
    }
}

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt in bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// ---------------------------------------------------------------------------------------------------------
// operand descriptions
// ---------------------------------------------------------------------------------------------------------
// row tile: element (row, k) at p + row*ld + k; rows >= rows_valid read as zero.
// col tile: element (k, col) at p_lo + k*ld + col for col < 128 and p_hi + k*ld + (col-128) for col >= 128;
//           columns >= n_lo (resp. n_hi) of a half and k >= k_valid read as zero.
struct Operand {
    const bf16_t* p_lo;
    const bf16_t* p_hi;
    long ld;
    int n_lo, n_hi;    // row tile: n_lo = valid rows (0..256); col tile: valid columns per 128-wide half
    int k_valid;       // col tile only
    // gathered operand (loaders with GATHER): the tile's row r (row tile) or k-row r (col tile) is row gather[r] of
    // the matrix at p_lo - the dispatched copy of the tokens is never made
    const int32_t* gather;
    const int32_t* gather_dma;   // K-strided gathered operand: the same array again (see Loader::gidx_dma)
};

// per-thread state of the two direct-to-LDS loads an operand needs per stage.  TWO: the K range is the
// concatenation of two GEMMs (k-tiles [0, nk1) come from operand set 1, [nk1, nk) from set 2).
// GATHER: rows come through an index array (Operand::gather).  A per-lane vector load of the indices would join the
// ordered queue of direct-to-LDS loads, and waiting for it would drain the ring.  A K-contiguous operand needs its 256
// row indices once per tile and reads them with wave-uniform addresses, i.e. through the scalar unit.
// A K-strided operand needs four new indices per wave and k-tile.  With the chain index -> row -> 64-bit address at
// the head of a k-step, in front of the step's loads and of everything the wave issues after them, such an operand
// costs 10 to 12 % of the loop (measured with an identity index on a contiguous copy: it is this chain, not the
// scattered rows).  So the addresses of a step's loads are formed at the END of the previous step, behind its last
// matrix instruction (prepare_next), from indices that were read in the middle of that step.  For that the indices
// travel like the operands: one direct-to-LDS dword load per wave fetches the wave's rows of 16 k-tiles into a
// wave-private buffer behind the ring (two buffers; chunk c+1 is requested while chunk c is half used, and the k-tile
// loop's own waits cover it long before it is read), and per k-tile a lane reads its two indices from LDS.  (Scalar
// loads do not work here: the per-lane choice between two of them in the same step is folded into the load address,
// which makes them vector loads.)  Only the first kIdxScalarTiles k-tiles of a tile, which are needed before the
// first chunk can have landed, take the scalar path, one call ahead.
template <bool COL, bool TWO, bool GATHER = false>
struct Loader {
    const bf16_t* g[TWO ? 2 : 1][2];   // global address of this lane's 16 bytes for k-tile 0 (or kZero16)
    const int32_t* gidx;  // GATHER: index array
    // GATHER && COL: the same address for the direct-to-LDS index loads, reached through a second kernel parameter.  A
    // direct-to-LDS load counts as a possible write through both of its pointers, so one that visibly reads the index
    // array would turn every ordinary load from that array (the scalar loads of the first k-tiles and of the
    // K-contiguous operand's rows) into a vector load, and waiting for a vector load drains the ring.
    const int32_t* gidx_dma;   // (the kernels take the index array as two __restrict__ parameters for this)
    int gld;              // GATHER && COL: leading dimension of the gathered matrix
    // GATHER && COL: this lane's two source rows (k-rows wave*4 + lane/32 and wave*4 + 2 + lane/32) of the k-tile after
    // the one issued last (issue() is called for k-tiles 0, 1, 2, ... in order)
    mutable int gk2[2];
    mutable const bf16_t* pnext[2];   // the addresses the next main-loop issue() loads from (prepare_next)
    mutable int gk[4];    // the same k-tile's four k-rows of this wave, where they were fetched by scalar loads
    char* ibuf;           // GATHER && COL: this wave's two index chunks in LDS
    // requests chunk c (k-tiles [16c, 16c+16)): lane l fetches the index of k-row (wave*4 + l%4) of k-tile 16c + l/4
    __device__ __forceinline__ void idx_issue(int c, char* __restrict__ dst) const {
        const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int kk = (c * kIdxChunk + (lane >> 2)) * TK + wave * 4 + (lane & 3);
        __builtin_amdgcn_global_load_lds(GLB_PTR(gidx_dma + (kk < k_valid ? kk : k_valid - 1)), LDS_PTR(dst), 4, 0, 0);
    }
    // this lane's two source rows of k-tile kt: k-rows wave*4 + lane/32 and wave*4 + 2 + lane/32
    __device__ __forceinline__ void idx_read(int kt, const char* __restrict__ src) const {
        const int lane = threadIdx.x & 63;
        const int* p = reinterpret_cast<const int*>(src + (kt & (kIdxChunk - 1)) * 16 + (lane >> 5) * 4);
        gk2[0] = p[0];
        gk2[1] = p[2];
    }
    __device__ __forceinline__ char* idx_buf(int chunk) const { return ibuf + (chunk & 1) * kIdxChunkBytes; }
    // before k-tile kt is issued: half way through a chunk, request the next one (if the tile has it).  It lands in the
    // buffer that is not read before k-tile 16*(chunk+1) - 1 is issued, seven k-tiles (and barriers) later.
    __device__ __forceinline__ void request_ahead(int kt) const {
        if (GATHER && COL) {
            const int c = (kt >> 4) + 1;
            if ((kt & (kIdxChunk - 1)) == kIdxChunk / 2 && c * kIdxChunk * TK < k_valid) idx_issue(c, idx_buf(c));
        }
    }
    __device__ __forceinline__ void fetch_rows(int kt) const {   // the scalar path (first k-tiles of a tile)
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int kk = kt * TK + wave * 4 + r;
            gk[r] = gidx[kk < k_valid ? kk : k_valid - 1];   // wave-uniform address
        }
    }
    // the scalar path's rows as this lane's two
    __device__ __forceinline__ void rows_from_scalar() const {
        const bool up = (threadIdx.x & 32) != 0;
        gk2[0] = up ? gk[1] : gk[0];
        gk2[1] = up ? gk[3] : gk[2];
    }
    long step;            // elements to advance per k-tile (wave-uniform; not used by a gathered K-strided operand)
    // this lane's k index inside the tile (col tile; 0 for a row tile), or 2^30 for a lane that fetches zeros for good
    // (a row or column outside the operand): k-tile kt reads zeros where kt*TK + krow >= k_lim
    int krow[2];
    int k_lim;            // col tile: k_valid; row tile: nk * TK
    int lds_off[2];       // wave-uniform byte offset of the instruction's 1 KiB destination inside the tile
    int k_valid;
    int nk1, nk;          // k-tiles of set 1, total k-tiles; tiles past the end fetch zeros

    // ibuf_: this operand's index buffers (kIdxWaveBytes per wave); only touched by a gathered K-strided operand
    __device__ __forceinline__ void init(const Operand& o, const Operand& o2, int num_k1, int num_k, char* ibuf_) {
        const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        ibuf = ibuf_ + wave * kIdxWaveBytes;
        k_valid = o.k_valid;
        nk1 = num_k1;
        nk = num_k;
        gidx = o.gather;
        gidx_dma = o.gather_dma;
        gld = (int)o.ld;
        int grow[2] = {0, 0};   // GATHER && !COL: source rows of this lane's two tile rows
        if (GATHER && !COL) {
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int r = wave * 32 + j;
                const int v = gidx[r < o.n_lo ? r : o.n_lo - 1];   // wave-uniform address
                if ((lane >> 2) == (j & 15)) grow[j >> 4] = v;
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (!COL) {
                const int row = wave * 32 + i * 16 + (lane >> 2);
                const int c = (lane & 3) ^ ((row >> 2) & 3);
                const bool ok = row < o.n_lo;
                const bf16_t* z = reinterpret_cast<const bf16_t*>(kZero16);
                g[0][i] = ok ? o.p_lo + (long)(GATHER ? grow[i] : row) * o.ld + c * 8 : z;
                if (TWO) g[TWO ? 1 : 0][i] = ok ? o2.p_lo + (long)row * o2.ld + c * 8 : z;
                step = TK;
                krow[i] = ok ? 0 : (1 << 30);
                lds_off[i] = (wave * 32 + i * 16) * 64;
            } else {
                const int kr = wave * 4 + i * 2 + (lane >> 5);
                const int c = (lane & 31) ^ ((kr & 3) << 2);
                const int col = (c & 15) * 8;
                const bool hi = c >= 16;
                const bool ok = col < (hi ? o.n_hi : o.n_lo);
                // GATHER: the address of the column inside row 0; the row is looked up per k-tile in issue()
                g[0][i] = ok ? (hi ? o.p_hi : o.p_lo) + (GATHER ? 0 : (long)kr * o.ld) + col
                             : reinterpret_cast<const bf16_t*>(kZero16);
                step = (long)TK * o.ld;
                krow[i] = ok ? kr : (1 << 30);
                lds_off[i] = (wave * 4 + i * 2) * 512;
            }
        }
        k_lim = COL ? k_valid : nk * TK;
        if (!(GATHER && COL)) {   // k-tile 0
#pragma unroll
            for (int i = 0; i < 2; ++i) pnext[i] = krow[i] >= k_lim ? reinterpret_cast<const bf16_t*>(kZero16) : g[0][i];
        }
        if (GATHER && COL) {
            // chunk 0 is older than every operand load of the tile, so the wait that ends the prologue covers it
            idx_issue(0, idx_buf(0));
            fetch_rows(0);
            rows_from_scalar();
        }
    }

    // issues the two loads of k-tile kt into `tile` (LDS address of this operand's tile in the target stage).
    // PROLOGUE: one of the first kStages-1 k-tiles of a tile (gathered K-strided operand: rows by scalar loads, one
    // call ahead); otherwise a main-loop step, whose addresses prepare_next() has formed.
    // Forms the addresses of k-tile kt's two loads.  Called at the END of a main-loop step for the next one, while the
    // step's last matrix instructions still run: formed at the head of the step, the address arithmetic (for a
    // gathered K-strided operand the chain index -> row -> 64-bit address) sits in front of the step's loads and of
    // all that follows them.  Measured against forming them at the head: dX -7 %, down -2 %, gate/up -1 %, the
    // gathered weight gradients -4 to -5 %.
    // Gathered K-strided operand: from the rows in gk2.
    // The other operands do the same with their running addresses: k-tile kt's address is the previous one advanced
    // by `step`, or the block of zeros from the k-tile on where this lane's k index passes the end (it then stays
    // there: the advanced value is never used again), or the start of the second operand set at k-tile nk1 (TWO).
    __device__ __forceinline__ void prepare_next(int kt) const {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bf16_t* p;
            if (GATHER && COL)
                p = g[0][i] + (long)gk2[i] * gld;
            else if (TWO)
                p = kt == nk1 ? g[TWO ? 1 : 0][i] : pnext[i] + step;
            else
                p = pnext[i] + step;
            if (kt * TK + krow[i] >= k_lim) p = reinterpret_cast<const bf16_t*>(kZero16);
            pnext[i] = p;
        }
        // an anchor in front of the barrier that ends the step (volatile asm statements keep their order): the
        // scheduler would otherwise sink this arithmetic behind the barrier, to the head of the next step
        asm volatile("" ::"v"(pnext[0]), "v"(pnext[1]));
    }
    // main loop: the rows of k-tile kt from the index chunk; called in the middle of the step that issued k-tile kt-1,
    // among its fragment reads (right behind the loads, in front of the first matrix instruction, the wait for the
    // step's first fragments would also wait for this read)
    __device__ __forceinline__ void read_rows(int kt, const char* __restrict__ idx_rd) const {
        if (GATHER && COL) idx_read(kt, idx_rd);
    }
    template <bool PROLOGUE>
    __device__ __forceinline__ void issue(char* tile, int kt) const {
        int src_row[2] = {0, 0};
        if (GATHER && COL) {
            src_row[0] = gk2[0];
            src_row[1] = gk2[1];
            // the prologue issues k-tiles 0 .. kStages-2 and prepares k-tiles 1 .. kStages-1 = kIdxScalarTiles-1
            if (PROLOGUE) {
                fetch_rows(kt + 1);
                rows_from_scalar();
                if (kt == kStages - 2) prepare_next(kt + 1);
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bf16_t* p;
            if (GATHER && COL && PROLOGUE) {
                // lanes outside the operand hold the block of zeros in g and a krow beyond every k_lim
                p = g[0][i] + (long)src_row[i] * gld;
                if (kt * TK + krow[i] >= k_lim) p = reinterpret_cast<const bf16_t*>(kZero16);
            } else {
                p = pnext[i];
            }
            __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(tile + lds_off[i]), 16, 0, 0);
        }
    }
};

// ---------------------------------------------------------------------------------------------------------
// fragment reads: 8 bf16 (k = 16*ks + 8*(lane/32) + 0..7) of row / column (base + lane%32)
// ---------------------------------------------------------------------------------------------------------
template <bool COL>
__device__ __forceinline__ bf16x8_t read_frag(const char* tile, int base, int ks) {
    const int lane = threadIdx.x & 63;
    if (!COL) {
        const int r = base + (lane & 31);
        const int chunk = 2 * ks + (lane >> 5);
        return *reinterpret_cast<const bf16x8_t*>(tile + r * 64 + ((chunk ^ ((r >> 2) & 3)) << 4));
    } else {
        // 16-lane groups: group G covers columns base + 16*(G%2) .. +15 and k = 16*ks + 8*(G/2) .. +7; inside a
        // group, lane s addresses 4 consecutive columns (s%4) of k-row (s/4); the transposing read hands every
        // lane one column with 4 consecutive k.
        const int G = lane >> 4, s = lane & 15;
        const int col = base + 16 * (G & 1) + 4 * (s & 3);
        const int k0 = 16 * ks + 8 * (G >> 1) + (s >> 2);
        s16x4_t h[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int kr = k0 + 4 * q;
            const char* a = tile + kr * 512 + ((((col >> 3) ^ ((kr & 3) << 2))) << 4) + (col & 7) * 2;
            h[q] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)LDS_PTR(a));
        }
        s16x8_t v = {h[0][0], h[0][1], h[0][2], h[0][3], h[1][0], h[1][1], h[1][2], h[1][3]};
        return __builtin_bit_cast(bf16x8_t, v);
    }
}

// column base (inside the 256-wide B tile) of the wave's ni-th 32-column block.  Plain tiles: 64 contiguous
// columns per wave.  Dual tiles (two matrices side by side, 128 columns each): the same 32 columns of both.
template <bool DUAL>
__device__ __forceinline__ int b_col(int wn, int ni) { return DUAL ? ni * 128 + wn * 32 : wn * 64 + ni * 32; }

// the 6 fragments (4 of A, 2 of B) a wave needs for one 16-wide k-step
struct Frags {
    bf16x8_t a[4], b[2];
};
__device__ __forceinline__ void zero_frags(Frags& f) {
    const s16x8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) f.a[i] = __builtin_bit_cast(bf16x8_t, z);
#pragma unroll
    for (int i = 0; i < 2; ++i) f.b[i] = __builtin_bit_cast(bf16x8_t, z);
}

template <bool A_COL, bool B_COL, bool DUAL>
__device__ __forceinline__ void read_frags(Frags& f, const char* ta, const char* tb, int ks) {
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) f.b[ni] = read_frag<B_COL>(tb, b_col<DUAL>(wn, ni), ks);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) f.a[mi] = read_frag<A_COL>(ta, wm * 128 + mi * 32, ks);
}

// acc[mi][ni][v] holds C(row = wm*128 + mi*32 + lane%32, col = b_col(wn, ni) + 8*(v/4) + 4*(lane/32) + v%4)
__device__ __forceinline__ void mma_step(f32x16_t (&acc)[4][2], const Frags& f) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ni], f.a[mi], acc[mi][ni], 0, 0, 0);
}

// waits until at most N of this wave's vector-memory operations are outstanding and all of its LDS reads have
// returned (fragments carried across the barrier must be out of the stage that is refilled after it), then joins
// the workgroup barrier.
// Written as one asm block: __syncthreads() would make the compiler wait for ALL outstanding direct-to-LDS loads
// (they are memory writes the fence has to cover) and so serialise the load ring.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
// workgroup barrier that waits only for the wave's LDS traffic (result stores stay in flight)
__device__ __forceinline__ void lds_done_and_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The index chunk a k-tile's loads read (gathered K-strided operands only) is handed to kstep / feed_step as a
// __restrict__ parameter, for the same reason as the ring stages: an LDS read that may observe a direct-to-LDS load
// in flight makes the compiler drain every outstanding load first.  (The chunk requested between two k-tiles goes to
// the other buffer of the pair.)

// a k-tile of a wave that has nothing to multiply: it only feeds the ring
template <bool ISSUE = true, class LA, class LB>
__device__ __forceinline__ void feed_step(const LA& la, const LB& lb, char* __restrict__ st_next, int nt,
                                          const char* __restrict__ ia_rd, const char* __restrict__ ib_rd) {
    if (ISSUE) {
        la.template issue<false>(st_next, nt);
        lb.template issue<false>(st_next + kOpBytes, nt);
    }
    la.read_rows(nt + 1, ia_rd);
    lb.read_rows(nt + 1, ib_rd);
    la.prepare_next(nt + 1);
    lb.prepare_next(nt + 1);
}

// One k-tile of the main loop.  On entry k-tile kt has landed in `st`, every wave has finished reading the stage
// `st_next` (k-tile kt-1), and f1 still holds the second 16-wide k-step of k-tile kt-1.  The body refills st_next
// with k-tile nt = kt+3, fetches the first k-step of k-tile kt while the MFMAs of the carried f1 run, then fetches
// the second k-step while the MFMAs of the first run; the second k-step's MFMAs are carried into the next call.
// Carrying work, rather than fragments of the NEXT tile, across the barrier keeps three k-tiles of loads in
// flight instead of two, which is what the loop is bound by (memory latency / tiles in flight).
// The two stages are distinct, and saying so with __restrict__ matters: without it the compiler assumes an LDS
// read may observe a direct-to-LDS load still in flight and drains every outstanding load (s_waitcnt vmcnt(0))
// before each transposing read, which serialises the ring.
// ISSUE = false: the step of k-tile 0 where the prologue has already requested k-tile nt (see mainloop2).
template <bool A_COL, bool B_COL, bool DUAL, bool TWO, bool A_GATHER, bool B_GATHER, bool ISSUE = true>
__device__ __forceinline__ void kstep(f32x16_t (&acc)[4][2], Frags& f0, Frags& f1,
                                      const Loader<A_COL, TWO, A_GATHER>& la,
                                      const Loader<B_COL, TWO, B_GATHER>& lb, char* __restrict__ st_next,
                                      const char* __restrict__ st, int nt, const char* __restrict__ ia_rd,
                                      const char* __restrict__ ib_rd) {
    // In the kernels whose two operands are both K-strided (the weight gradients) the wave issues its k-tile's loads
    // at raised priority, ahead of the other wave's matrix instructions on the same SIMD: measured -2 to -4 % there,
    // +4 to +10 % in the kernels with a K-contiguous operand, where it is therefore left alone.  (Raising the
    // priority during the matrix instructions instead costs 5 to 10 % everywhere.)
    if (ISSUE) {
        if (A_COL && B_COL) __builtin_amdgcn_s_setprio(1);
        la.template issue<false>(st_next, nt);
        lb.template issue<false>(st_next + kOpBytes, nt);
        if (A_COL && B_COL) __builtin_amdgcn_s_setprio(0);
    }
    read_frags<A_COL, B_COL, DUAL>(f0, st, st + kOpBytes, 0);
    mma_step(acc, f1);
    la.read_rows(nt + 1, ia_rd);
    lb.read_rows(nt + 1, ib_rd);
    read_frags<A_COL, B_COL, DUAL>(f1, st, st + kOpBytes, 1);
    mma_step(acc, f0);
    if (A_COL || B_COL) {
        // instruction order: every MFMA is followed by a share of the k-tile's direct-to-LDS loads and LDS
        // fragment reads (0x008 = MFMA, 0x010 = vector memory, 0x100 = LDS read)
        constexpr int kReadsPerStep = (A_COL ? 8 : 4) + (B_COL ? 4 : 2);   // LDS reads of one k-step
        constexpr int kRd = (kReadsPerStep + 5) / 6;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, kRd, 0);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, kRd, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, kRd, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
    // the next step's load addresses, behind the last matrix instruction (0x002 = VALU)
    la.prepare_next(nt + 1);
    lb.prepare_next(nt + 1);
    if ((A_GATHER && A_COL) || (B_GATHER && B_COL)) __builtin_amdgcn_sched_group_barrier(0x002, 24, 0);
}

// =========================================================================================================
// Both operands K-contiguous (dAct: dOut rows x Wd rows; dX: dG | dU rows x Wg | Wu rows).
// A 32-wide k-tile of such an operand is 64 bytes of each row, half a cache line, and the vector-memory front end of
// a CU takes whole-line requests at twice the rate of half-line ones (measured with this load instruction on
// L2-resident data: 58 against 29 B/clk per CU) - and the time a k-step's requests spend in that front end shows up
// in the loop one to one: k-tiles of the row x row kernels took 0.95 to 1.08 us where the row x column kernels take
// 0.8.  So these GEMMs load 64 k at a time: a unit is one operand's [256 rows][64 k], 128-byte rows, 32 KiB, one
// instruction of a wave fetching eight whole lines.  The CU's 160 KiB hold a ring of five units that alternate
// A(0) B(0) A(1) B(1) ...; the four 16-wide k-steps on A(p), B(p) are one pass of the loop, which refills the two
// units the pass before it released (B(p+1) at its first k-step, A(p+2) at its third), so two to three units are in
// flight at any time and a barrier waits for all but the newest.
// Rows outside the operand are clamped to its last row instead of fetching zeros: the output rows and columns they
// feed are never stored (K itself is a multiple of 64, there is no tail along K), which keeps a lane's address a
// fixed 32-bit offset from a wave-uniform base for the whole tile.
// =========================================================================================================
template <bool GATHER>
struct RowLoader {
    // offset of this lane's 16 bytes in instruction i from (row 0, first k of the unit): source row * ld * 2 +
    // chunk * 16 bytes.  Rows of the tile itself: in bytes.  GATHER: the source row is any row of the gathered
    // matrix, so the offset is kept in units of 16 bytes (ld is a multiple of 64 elements) and reaches 64 GiB.
    uint32_t off[4];
    __device__ __forceinline__ void init(const Operand& o) {
        const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        int grow[4] = {0, 0, 0, 0};
        if (GATHER) {
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int r = wave * 32 + j;
                const int v = o.gather[r < o.n_lo ? r : o.n_lo - 1];   // wave-uniform address: a scalar load
                if ((lane >> 3) == (j & 7)) grow[j >> 3] = v;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = wave * 32 + i * 8 + (lane >> 3);
            const int src = GATHER ? grow[i] : (row < o.n_lo ? row : o.n_lo - 1);
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            off[i] = GATHER ? (uint32_t)src * (uint32_t)(o.ld / 8) + (uint32_t)c
                            : (uint32_t)src * (uint32_t)(o.ld * 2) + (uint32_t)(c * 16);
        }
    }
    // kbase: wave-uniform address of (row 0, first k of the unit); zero: the unit lies past the end of K and every
    // lane fetches the block of zeros (the loads are issued all the same, which keeps the wait counts uniform)
    __device__ __forceinline__ void issue(char* __restrict__ unit, const char* kbase, bool zero) const {
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t o = zero ? 0u : off[i];
            const char* p = GATHER ? kbase + ((unsigned long long)o << 4) : kbase + o;
            __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(unit + (wave * 32 + i * 8) * 128), 16, 0, 0);
        }
    }
};

// 8 bf16 (k = 16*ks4 + 8*(lane/32) + 0..7 of the unit, ks4 = 0..3) of row base + lane%32; the 16-byte chunks of a row
// are XOR-swizzled with (row / 2) % 8, so the 16 rows that one pass of a 16-byte LDS read covers hit 16 distinct
// groups of four banks
__device__ __forceinline__ bf16x8_t read_frag_unit(const char* unit, int base, int ks4) {
    const int lane = threadIdx.x & 63;
    const int r = base + (lane & 31);
    const int chunk = 2 * ks4 + (lane >> 5);
    return *reinterpret_cast<const bf16x8_t*>(unit + r * 128 + ((chunk ^ ((r >> 1) & 7)) << 4));
}
__device__ __forceinline__ void read_frags_unit(Frags& f, const char* ua, const char* ub, int ks4) {
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) f.b[ni] = read_frag_unit(ub, b_col<false>(wn, ni), ks4);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) f.a[mi] = read_frag_unit(ua, wm * 128 + mi * 32, ks4);
}

// where unit u = 2*pair + (0: A, 1: B) comes from
struct UnitSource {
    const char *a1, *b1, *a2, *b2;   // operand sets 1 and 2 (set 2 = set 1 when there is one set)
    int np1, np;                     // pairs (64-wide k ranges) of set 1, total
    __device__ __forceinline__ const char* base(int u, bool& zero) const {
        const int p = u >> 1;
        zero = p >= np;
        if (zero) return reinterpret_cast<const char*>(kZero16);
        const bool second = p >= np1;
        const char* b = (u & 1) ? (second ? b2 : b1) : (second ? a2 : a1);
        return b + (long)(second ? p - np1 : p) * 128;
    }
};

// One pass: the four 16-wide k-steps on A(p) = ua, B(p) = ub.  On entry both have landed for every thread, every wave
// is done with the units of pass p-1 (fill1, fill2: their slots), and f1 holds the last k-step of pass p-1, whose
// matrix instructions run first.  The five slots are distinct, and saying so with __restrict__ matters: see kstep.
template <bool A_GATHER>
__device__ __forceinline__ void rr_pass(f32x16_t (&acc)[4][2], Frags& f0, Frags& f1, const RowLoader<A_GATHER>& la,
                                        const RowLoader<false>& lb, const UnitSource& src, int p,
                                        char* __restrict__ fill1, char* __restrict__ fill2,
                                        const char* __restrict__ ua, const char* __restrict__ ub) {
    // The requests are pinned where they stand (a scheduling barrier behind each group): left to itself the compiler
    // sinks all eight to the end of the pass, where the wait that ends the pass would then sit out B(p+1)'s whole
    // latency.  (Tried: both groups at the head of the pass, +6 %: bursts of requests cost more than they gain in lead;
    // two requests per 16-wide k-step, +1.5 %; raised wave priority while requesting, no change.)
    bool z;
    const char* kb = src.base(2 * p + 3, z);
    lb.issue(fill1, kb, z);                       // B(p+1)
    __builtin_amdgcn_sched_barrier(0);
    read_frags_unit(f0, ua, ub, 0);
    mma_step(acc, f1);
    read_frags_unit(f1, ua, ub, 1);
    mma_step(acc, f0);
    kb = src.base(2 * p + 4, z);
    __builtin_amdgcn_sched_barrier(0);
    la.issue(fill2, kb, z);                       // A(p+2)
    __builtin_amdgcn_sched_barrier(0);
    read_frags_unit(f0, ua, ub, 2);
    mma_step(acc, f1);
    read_frags_unit(f1, ua, ub, 3);
    mma_step(acc, f0);
}
template <bool A_GATHER>
__device__ __forceinline__ void rr_feed(const RowLoader<A_GATHER>& la, const RowLoader<false>& lb,
                                        const UnitSource& src, int p, char* __restrict__ fill1,
                                        char* __restrict__ fill2) {
    bool z;
    const char* kb = src.base(2 * p + 3, z);
    lb.issue(fill1, kb, z);
    kb = src.base(2 * p + 4, z);
    la.issue(fill2, kb, z);
}

// acc += A x B over K (+ A2 x B2 over K2 when TWO); K and K2 are multiples of 64.  mi_count as in mainloop2.
template <bool TWO, bool A_GATHER>
__device__ __forceinline__ void mainloop_rr(f32x16_t (&acc)[4][2], const Operand& oa, const Operand& ob, int K,
                                            const Operand& oa2, const Operand& ob2, int K2, int mi_count,
                                            char* smem) {
    UnitSource src;
    src.np1 = K / 64;
    src.np = src.np1 + (TWO ? K2 / 64 : 0);
    if (src.np <= 0) return;
    src.a1 = reinterpret_cast<const char*>(oa.p_lo);
    src.b1 = reinterpret_cast<const char*>(ob.p_lo);
    src.a2 = reinterpret_cast<const char*>(TWO ? oa2.p_lo : oa.p_lo);
    src.b2 = reinterpret_cast<const char*>(TWO ? ob2.p_lo : ob.p_lo);
    mi_count = __builtin_amdgcn_readfirstlane(mi_count);
    RowLoader<A_GATHER> la;
    RowLoader<false> lb;
    la.init(oa);
    lb.init(ob);
    {   // prologue: A(0), B(0), A(1) into slots 0, 1, 2
        bool z;
        const char* kb = src.base(0, z);
        la.issue(smem, kb, z);
        kb = src.base(1, z);
        lb.issue(smem + kUnitBytes, kb, z);
        kb = src.base(2, z);
        la.issue(smem + 2 * kUnitBytes, kb, z);
    }
    // Invariant at the top of pass p: units <= 2p+1 have landed for every thread, unit 2p+2 (four loads per thread) may
    // still be in flight, and the slots of units 2p-2 and 2p-1 are free for units 2p+3 and 2p+4.
    wait_loads_and_barrier<4>();
    int sa = 0;   // slot of A(p) = (2p) % 5
    if (mi_count > 0) {
        Frags f0, f1;
        zero_frags(f1);
        for (int p = 0; p < src.np; ++p) {
            const int sb = sa + 1 < kUnits ? sa + 1 : sa + 1 - kUnits;
            const int s3 = sa + 3 < kUnits ? sa + 3 : sa + 3 - kUnits;
            const int s4 = sa + 4 < kUnits ? sa + 4 : sa + 4 - kUnits;
            rr_pass<A_GATHER>(acc, f0, f1, la, lb, src, p, smem + s3 * kUnitBytes, smem + s4 * kUnitBytes,
                              smem + sa * kUnitBytes, smem + sb * kUnitBytes);
            wait_loads_and_barrier<4>();
            sa = sa + 2 < kUnits ? sa + 2 : sa + 2 - kUnits;
        }
        mma_step(acc, f1);
    } else {
        for (int p = 0; p < src.np; ++p) {
            const int s3 = sa + 3 < kUnits ? sa + 3 : sa + 3 - kUnits;
            const int s4 = sa + 4 < kUnits ? sa + 4 : sa + 4 - kUnits;
            rr_feed<A_GATHER>(la, lb, src, p, smem + s3 * kUnitBytes, smem + s4 * kUnitBytes);
            wait_loads_and_barrier<4>();
            sa = sa + 2 < kUnits ? sa + 2 : sa + 2 - kUnits;
        }
    }
    // all loads of this tile (and the dummy ones past its end) have landed before the ring is reused as staging
    wait_loads_and_barrier<0>();
}

// =========================================================================================================
// A K-contiguous, B K-strided (gate/up and down: activation rows x weights "in x out").  The same observation as for
// the row x row kernels, applied to the one operand it concerns: A is loaded 64 k at a time as units of
// [256 rows][64 k] (whole 128-byte lines), B stays in 32-wide k-tiles of [32 k][256 n] (512-byte rows, whole lines
// already).  LDS: three A units (96 KiB) and behind them four B tiles (64 KiB).  One pass = the two k-tiles of A(p):
// the first requests A(p+2) and B(2p+3), the second B(2p+4); at every barrier the wave may have eight requests
// outstanding (the two newest B tiles and the newest A unit), so A runs two units and B three tiles ahead, as in the
// rings above.  The hand-over slot of the tile walk lies in the last bytes of the fourth B tile, which a tile first
// refills behind its main loop's first barrier.  The compiler's own order of requests, fragment reads and matrix
// instructions is kept (prescribing kstep's interleaving here measured the same).  Measured against the four-stage
// ring of 32-wide k-tiles for both operands (XMOE_RC_RING=0): down -2 to -3 %, the two-matrix expert's up
// projection -3 %, gate/up -1 to -2 %.
// =========================================================================================================
constexpr int kRcAUnits = 3;
constexpr int kRcBStages = 4;
constexpr int kRcBBase = kRcAUnits * kUnitBytes;
static_assert(kRcBBase + kRcBStages * kOpBytes <= kLdsBytes, "three A units and four B tiles");

// one k-tile: HALF2 = false: the first k-tile of A's unit (requests the unit two passes ahead), true: the second
template <bool DUAL, bool A_GATHER, bool HALF2>
__device__ __forceinline__ void rc_step(f32x16_t (&acc)[4][2], Frags& f0, Frags& f1, const RowLoader<A_GATHER>& la,
                                        const Loader<true, false, false>& lb, char* __restrict__ fill_a,
                                        const char* a_kb, bool a_zero, char* __restrict__ fill_b,
                                        const char* __restrict__ ua, const char* __restrict__ tb, int nt) {
    if (!HALF2) la.issue(fill_a, a_kb, a_zero);
    lb.template issue<false>(fill_b, nt);
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) f0.b[ni] = read_frag<true>(tb, b_col<DUAL>(wn, ni), 0);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) f0.a[mi] = read_frag_unit(ua, wm * 128 + mi * 32, HALF2 ? 2 : 0);
    mma_step(acc, f1);
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) f1.b[ni] = read_frag<true>(tb, b_col<DUAL>(wn, ni), 1);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) f1.a[mi] = read_frag_unit(ua, wm * 128 + mi * 32, HALF2 ? 3 : 1);
    mma_step(acc, f0);
    lb.prepare_next(nt + 1);
}
template <bool A_GATHER, bool HALF2>
__device__ __forceinline__ void rc_feed(const RowLoader<A_GATHER>& la, const Loader<true, false, false>& lb,
                                        char* __restrict__ fill_a, const char* a_kb, bool a_zero,
                                        char* __restrict__ fill_b, int nt) {
    if (!HALF2) la.issue(fill_a, a_kb, a_zero);
    lb.template issue<false>(fill_b, nt);
    lb.prepare_next(nt + 1);
}

// acc += A x B over K, a multiple of 64.  mi_count as in mainloop2.
template <bool DUAL, bool A_GATHER>
__device__ __forceinline__ void mainloop_rc(f32x16_t (&acc)[4][2], const Operand& oa, const Operand& ob, int K,
                                            int mi_count, char* smem) {
    const int np = K / 64, nk = 2 * np;
    if (np <= 0) return;
    mi_count = __builtin_amdgcn_readfirstlane(mi_count);
    RowLoader<A_GATHER> la;
    Loader<true, false, false> lb;
    la.init(oa);
    lb.init(ob, ob, nk, nk, smem);   // (no index buffers: B is not gathered)
    const char* a0 = reinterpret_cast<const char*>(oa.p_lo);
    const char* zero16 = reinterpret_cast<const char*>(kZero16);
    char* bt = smem + kRcBBase;
    // prologue: A(0), B(0), then A(1), B(1), B(2): the first wait leaves exactly those last three outstanding
    la.issue(smem, a0, false);
    lb.template issue<true>(bt, 0);
    lb.prepare_next(1);
    la.issue(smem + kUnitBytes, np > 1 ? a0 + 128 : zero16, np <= 1);
    lb.template issue<true>(bt + kOpBytes, 1);
    lb.prepare_next(2);
    lb.template issue<true>(bt + 2 * kOpBytes, 2);
    lb.prepare_next(3);
    wait_loads_and_barrier<8>();
    int sa = 0;   // slot of A(p) = p % 3
    int sb = 0;   // stage of B(2p) = 2p % 4: 0 or 2
#define XMOE_RC_LOOP(STEP_A, STEP_B)                                                                                  \
    for (int p = 0; p < np; ++p) {                                                                                    \
        const int s2 = sa + 2 < kRcAUnits ? sa + 2 : sa + 2 - kRcAUnits;                                              \
        const bool z = p + 2 >= np;                                                                                   \
        const char* kb = z ? zero16 : a0 + (long)(p + 2) * 128;                                                       \
        STEP_A(smem + s2 * kUnitBytes, kb, z, bt + ((sb + 3) & 3) * kOpBytes, smem + sa * kUnitBytes,                 \
               bt + sb * kOpBytes, 2 * p + 3);                                                                        \
        wait_loads_and_barrier<8>();                                                                                  \
        STEP_B(smem + s2 * kUnitBytes, kb, z, bt + sb * kOpBytes, smem + sa * kUnitBytes, bt + (sb + 1) * kOpBytes,   \
               2 * p + 4);                                                                                            \
        wait_loads_and_barrier<8>();                                                                                  \
        sa = sa + 1 < kRcAUnits ? sa + 1 : 0;                                                                         \
        sb ^= 2;                                                                                                      \
    }
    if (mi_count > 0) {
        Frags f0, f1;
        zero_frags(f1);
#define XMOE_RC_A(fa, kb, z, fb, ua, tb, nt) rc_step<DUAL, A_GATHER, false>(acc, f0, f1, la, lb, fa, kb, z, fb, ua, tb, nt)
#define XMOE_RC_B(fa, kb, z, fb, ua, tb, nt) rc_step<DUAL, A_GATHER, true>(acc, f0, f1, la, lb, fa, kb, z, fb, ua, tb, nt)
        XMOE_RC_LOOP(XMOE_RC_A, XMOE_RC_B)
#undef XMOE_RC_A
#undef XMOE_RC_B
        mma_step(acc, f1);
    } else {
#define XMOE_RC_A(fa, kb, z, fb, ua, tb, nt) rc_feed<A_GATHER, false>(la, lb, fa, kb, z, fb, nt)
#define XMOE_RC_B(fa, kb, z, fb, ua, tb, nt) rc_feed<A_GATHER, true>(la, lb, fa, kb, z, fb, nt)
        XMOE_RC_LOOP(XMOE_RC_A, XMOE_RC_B)
#undef XMOE_RC_A
#undef XMOE_RC_B
    }
#undef XMOE_RC_LOOP
    wait_loads_and_barrier<0>();
}

// acc += A x B over K (+ A2 x B2 over K2 when TWO).  mi_count = number of 32-row blocks of this wave that hold
// valid rows; 0 skips the MFMAs but the wave still takes part in the loads and barriers.  (Skipping single
// 32-row blocks inside the loop is not worth it: guarded accumulator updates make the compiler copy all 128
// accumulator registers around every iteration.)
template <bool A_COL, bool B_COL, bool DUAL, bool TWO, bool A_GATHER = false, bool B_GATHER = false>
__device__ __forceinline__ void mainloop2(f32x16_t (&acc)[4][2], const Operand& oa, const Operand& ob, int K,
                                          const Operand& oa2, const Operand& ob2, int K2, int mi_count,
                                          char* smem) {
#ifndef XMOE_NO_UNIT_RING
    if constexpr (!A_COL && !B_COL && !B_GATHER) {
        mainloop_rr<TWO, A_GATHER>(acc, oa, ob, K, oa2, ob2, K2, mi_count, smem);
        return;
    }
#endif
#if XMOE_RC_RING
    if constexpr (!A_COL && B_COL && !B_GATHER && !TWO) {
        mainloop_rc<DUAL, A_GATHER>(acc, oa, ob, K, mi_count, smem);
        return;
    }
#endif
    const int nk1 = (K + TK - 1) / TK;
    const int nk = nk1 + (TWO ? (K2 + TK - 1) / TK : 0);
    if (nk <= 0) return;
    mi_count = __builtin_amdgcn_readfirstlane(mi_count);
    static_assert(!((A_GATHER || B_GATHER) && TWO), "a gathered operand cannot be one of two concatenated ones");
    static_assert(!(TWO && (A_COL || B_COL)), "concatenated operand sets are K-contiguous");
    Loader<A_COL, TWO, A_GATHER> la;
    Loader<B_COL, TWO, B_GATHER> lb;
    char* idx_area = smem + kStages * kStageBytes;
    la.init(oa, oa2, nk1, nk, idx_area);
    lb.init(ob, ob2, nk1, nk, idx_area + 8 * kIdxWaveBytes);
    // prologue: k-tiles 0 .. kStages-2 (tiles past the end fetch zeros into stages nobody reads, which keeps the
    // number of outstanding loads uniform)
#pragma unroll
    for (int s = 0; s < kStages - 1; ++s) {
        la.template issue<true>(smem + s * kStageBytes, s);
        lb.template issue<true>(smem + s * kStageBytes + kOpBytes, s);
        if (!(A_GATHER && A_COL)) la.prepare_next(s + 1);   // (a gathered K-strided operand does it inside issue())
        if (!(B_GATHER && B_COL)) lb.prepare_next(s + 1);
    }
    // Invariant at the top of iteration kt (established by the barrier before it): k-tiles <= kt have landed for
    // every thread, and every wave is done reading k-tile kt-1, so that stage can be refilled with k-tile kt+3:
    // k-tiles kt+1 .. kt+3 are in flight while k-tile kt is multiplied.
    constexpr int kInFlight = (kStages - 2) * kLoadsPerTile;   // loads that may still be outstanding at the barrier
    // Both operands K-strided (the weight gradients, whose K is an expert's row count: often a handful of k-tiles):
    // nobody reads a stage before the first barrier, so the prologue requests k-tile kStages-1 as well - into the
    // stage that iteration 0 would fill - and iteration 0 requests nothing.  A tile of up to kStages k-tiles then
    // waits for memory once instead of twice.
    constexpr bool kDeep = XMOE_DEEP_PROLOGUE && A_COL && B_COL;
    if (kDeep) {
        la.request_ahead(kStages - 1);
        lb.request_ahead(kStages - 1);
        la.template issue<false>(smem + (kStages - 1) * kStageBytes, kStages - 1);
        lb.template issue<false>(smem + (kStages - 1) * kStageBytes + kOpBytes, kStages - 1);
        wait_loads_and_barrier<kInFlight + kLoadsPerTile>();
    } else {
        wait_loads_and_barrier<kInFlight>();
    }
    if (mi_count > 0) {
        Frags f0, f1;
        zero_frags(f1);   // the first call multiplies the carried fragments: zeros
        int kt = 0;
        if (kDeep) {
            constexpr int nt = kStages - 1;
            kstep<A_COL, B_COL, DUAL, TWO, A_GATHER, B_GATHER, false>(acc, f0, f1, la, lb, smem + nt * kStageBytes, smem,
                                                                      nt, la.idx_buf((nt + 1) >> 4),
                                                                      lb.idx_buf((nt + 1) >> 4));
            wait_loads_and_barrier<kInFlight>();
            kt = 1;
        }
        for (; kt < nk; ++kt) {
            const int nt = kt + kStages - 1;
            la.request_ahead(nt);
            lb.request_ahead(nt);
            kstep<A_COL, B_COL, DUAL, TWO, A_GATHER, B_GATHER>(acc, f0, f1, la, lb, smem + (nt % kStages) * kStageBytes,
                                                               smem + (kt % kStages) * kStageBytes, nt,
                                                               la.idx_buf((nt + 1) >> 4), lb.idx_buf((nt + 1) >> 4));
            wait_loads_and_barrier<kInFlight>();
        }
        mma_step(acc, f1);   // second k-step of the last k-tile
    } else {
        // a wave whose rows (or columns) all lie past the ragged tail: it only feeds the ring and keeps the barriers
        int kt = 0;
        if (kDeep) {
            constexpr int nt = kStages - 1;
            feed_step<false>(la, lb, smem + nt * kStageBytes, nt, la.idx_buf((nt + 1) >> 4), lb.idx_buf((nt + 1) >> 4));
            wait_loads_and_barrier<kInFlight>();
            kt = 1;
        }
        for (; kt < nk; ++kt) {
            const int nt = kt + kStages - 1;
            la.request_ahead(nt);
            lb.request_ahead(nt);
            feed_step(la, lb, smem + (nt % kStages) * kStageBytes, nt, la.idx_buf((nt + 1) >> 4),
                      lb.idx_buf((nt + 1) >> 4));
            wait_loads_and_barrier<kInFlight>();
        }
    }
    // all loads of this tile (and the dummy ones past its end) have landed before the ring is reused as staging
    wait_loads_and_barrier<0>();
}

template <bool A_COL, bool B_COL, bool DUAL, bool A_GATHER = false, bool B_GATHER = false>
__device__ __forceinline__ void mainloop(f32x16_t (&acc)[4][2], const Operand& oa, const Operand& ob, int K,
                                         int mi_count, char* smem) {
    mainloop2<A_COL, B_COL, DUAL, false, A_GATHER, B_GATHER>(acc, oa, ob, K, oa, ob, 0, mi_count, smem);
}

// sigmoid with the hardware exp2 and reciprocal (each good to about 1 ulp): the results are rounded to bf16, and
// the library-grade expf and IEEE division cost as much as a quarter of a tile's main loop in the fused epilogues.
__device__ __forceinline__ float fast_sigmoid(float g) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * g));
}

__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[4][2]) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
}

// ---------------------------------------------------------------------------------------------------------
// epilogue helpers: a wave stages 32 rows x NC columns of bf16 in its private LDS strip, then writes rows out
// ---------------------------------------------------------------------------------------------------------
constexpr int kStripStride = 392;                 // bytes per staged row (192 columns + 8 bytes: conflict-free)
constexpr int kStripBytes = 32 * kStripStride;    // per wave
constexpr int kInBytes = 2 * 32 * 64;             // per wave: 32 x 32 bf16 of G and of U (dAct epilogue)

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
    return make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}

// A strip belongs to one wave, and a wave's LDS operations execute in order, so a strip needs no workgroup
// barrier: waiting for the wave's own LDS traffic (and keeping the compiler from moving accesses across) is enough.
__device__ __forceinline__ void strip_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// writes this lane's 16 values of one 32 x 32 accumulator tile at columns col0 .. col0+31 of the strip
__device__ __forceinline__ void strip_put(char* strip, int col0, const float (&x)[16]) {
    const int lane = threadIdx.x & 63;
    char* row = strip + (lane & 31) * kStripStride;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int n = col0 + 8 * q + 4 * (lane >> 5);
        *reinterpret_cast<uint2*>(row + n * 2) = pack4(x[4 * q], x[4 * q + 1], x[4 * q + 2], x[4 * q + 3]);
    }
}

// the q-th quarter of strip_put: this lane's values 4q .. 4q+3 of a 32 x 32 accumulator tile (written as soon as they
// exist, so that an epilogue that derives several tiles from one accumulator never holds them all as floats)
__device__ __forceinline__ void strip_put4(char* strip, int col0, int q, float a, float b, float c, float d) {
    const int lane = threadIdx.x & 63;
    const int n = col0 + 8 * q + 4 * (lane >> 5);
    *reinterpret_cast<uint2*>(strip + (lane & 31) * kStripStride + n * 2) = pack4(a, b, c, d);
}

// writes strip columns [col0, col0 + NC) of rows [0, rows_valid) to C (row stride ldc); columns >= cols_valid
// (a multiple of 4) are skipped.  NC = 32 or 64.  NT: streaming stores for results that this launch never reads
// again and that are written as whole 128-byte lines: they then do not displace the operand panels the workgroups of
// an XCD share through L2 (measured -1 to -2 % in the down, dX and weight-gradient kernels; the gate/up kernel, whose
// rows go out as 64-byte pieces, is 2.5 % slower with them and keeps ordinary stores).
// MASK = false: the caller knows that all 32 rows and NC columns are valid; the stores then stand outside any
// branch, and the compiler can tell how many of them are outstanding at a later wait (see the dAct epilogue).
// OFF32: a lane's address is a wave-uniform row group of C plus a fixed 32-bit offset (fewer address registers; it
// pays in the dAct epilogue, which is short of registers, and costs 1 to 5 % in the other kernels).
template <int NC, bool NT = false, bool MASK = true, bool OFF32 = false>
__device__ __forceinline__ void strip_flush(const char* strip, int col0, bf16_t* C, long ldc, int rows_valid,
                                            int cols_valid) {
    const int lane = threadIdx.x & 63;
    constexpr int LPR = NC / 4;          // lanes per row, 4 columns (8 bytes) each
    constexpr int RPI = 64 / LPR;        // rows per instruction
    const int c4 = (lane % LPR) * 4;
    const uint32_t o = (uint32_t)((lane / LPR) * (int)ldc + c4) * 2u;
#pragma unroll
    for (int it = 0; it < 32 / RPI; ++it) {
        const int r = it * RPI + lane / LPR;
        if (!MASK || (r < rows_valid && c4 < cols_valid)) {
            const uint2 v = *reinterpret_cast<const uint2*>(strip + r * kStripStride + (col0 + c4) * 2);
            bf16_t* dst = OFF32 ? reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(C + (long)(it * RPI) * ldc) + o)
                                : C + (long)r * ldc + c4;
            if (NT) {
                typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
                const u32x2_t w = {v.x, v.y};
                __builtin_nontemporal_store(w, reinterpret_cast<u32x2_t*>(dst));
            } else {
                *reinterpret_cast<uint2*>(dst) = v;
            }
        }
    }
}

// Tiles are handed out at run time.  Their cost is not uniform: the weight gradients' K is an expert's row count,
// and a row tile at the ragged end of a segment costs about three quarters of a full one, so a fixed share of
// tiles per workgroup leaves CUs idle at the end of a launch (and a tile count just above a multiple of the CU count
// costs a whole extra round).
// The tile list, longest experts first, is cut into groups of kQueueGroup consecutive tiles (neighbours share
// operand panels); group g belongs to the list of XCD g % 8, and each list has a counter.  A workgroup draws from
// its own XCD's list and, once that is empty, from the next XCD's, and so on round the ring; it stops after it
// has found all eight lists empty.  Only thread 0 touches the counters.
#ifndef XMOE_QUEUE_GROUP
#define XMOE_QUEUE_GROUP 16
#endif
constexpr int kQueueGroup = XMOE_QUEUE_GROUP;
#ifndef XMOE_WGRAD_BAND
#define XMOE_WGRAD_BAND 2
#endif
constexpr int kWgradBand = XMOE_WGRAD_BAND;   // tile rows per band of the weight-gradient tile numbering
__device__ __forceinline__ int queue_len(int total, int x) {
    const int ng = (total + kQueueGroup - 1) / kQueueGroup;
    return ((ng - x + kNumXcd - 1) / kNumXcd) * kQueueGroup;
}
struct TileQueue {
    int32_t* cnt;   // kNumXcd counters, zero at launch
    int total, victim, hops;
    // v: a value already drawn from cnt[victim], or -1.  Returns a tile index, or -1 when everything is taken.
    __device__ __forceinline__ int pop(int v) {
        for (;;) {
            if (v < 0) v = atomicAdd(&cnt[victim], 1);
            if (v < queue_len(total, victim)) {
                const int t = ((v / kQueueGroup) * kNumXcd + victim) * kQueueGroup + v % kQueueGroup;
                if (t < total) return t;
                v = -1;   // a hole in the last, partial group: draw again
                continue;
            }
            if (++hops >= kNumXcd) return -1;
            victim = (victim + 1) % kNumXcd;
            v = -1;
        }
    }
};

// A workgroup's walk over the tiles of a launch.  Workgroups are persistent (at most one per CU); thread 0 draws the
// next tile at the start of the current one (the atomic's latency passes during the main loop), resolves it after
// the main loop and hands the number over through LDS; everybody reads it behind the barrier that ends the tile.
// The two-slot hand-over buffer sits in the last 16 bytes of the CU's LDS: behind the four-stage ring and the index
// buffers, and inside the last unit of the five-unit ring, which a tile first refills behind its main loop's first
// barrier - no wave passes that barrier before it has read the slot; it is written after the main loop's final wait,
// when no load is in flight, and the epilogues' staging buffers end below it.
struct TileWalker {
    TileQueue q;
    int* slot;
    int it, drawn;
    // returns the first tile (or -1); counters: this launch's kNumXcd counters, zero at launch
    __device__ __forceinline__ int start(int32_t* counters, int total, char* smem) {
        q.cnt = counters;
        q.total = total;
        q.victim = blockIdx.x % kNumXcd;
        q.hops = 0;
        slot = reinterpret_cast<int*>(smem + kLdsBytes - 16);
        it = 0;
        drawn = -1;
        if (threadIdx.x == 0) slot[0] = q.pop(-1);
        __syncthreads();
        return __builtin_amdgcn_readfirstlane(slot[0]);
    }
    // at the start of a tile
    __device__ __forceinline__ void draw() {
        drawn = -1;
        if (threadIdx.x == 0) drawn = atomicAdd(&q.cnt[q.victim], 1);
    }
    // after the tile's main loop (the slot written here was last read before the barrier that ended the previous tile)
    __device__ __forceinline__ void hand_over() {
        // The draw's result is consumed under a branch (thread 0 only).  On the other path the compiler still counts
        // it as pending, and would wait for it - that is, for everything outstanding, the tile's result stores
        // included - where the register is next written: at the top of the next tile, in front of its first
        // requests.  A use by every lane here, where nothing is in flight, settles it.
        asm volatile("" ::"v"(drawn));
        if (threadIdx.x == 0) slot[(it + 1) & 1] = q.pop(drawn);
    }
    // ends the tile (every wave has left its staging strip before the next tile's loads land in the ring) and
    // returns the next one; the number is wave-uniform, so table look-ups that depend on it stay scalar loads
    __device__ __forceinline__ int next() {
        lds_done_and_barrier();
        ++it;
        return __builtin_amdgcn_readfirstlane(slot[it & 1]);
    }
};

// The weight gradients' tiles: experts in the order of `order` (longest first), tpe tiles each.  Dealt group by group
// round the XCDs, an expert's tiles would be spread over all of them and every L2 would fetch the expert's two operand
// panels (K rows of P and of Q) for itself.  Instead the queue numbers are mapped so that ONE list holds all tiles of an
// expert: list x has the experts at positions x, x+8, x+16, ... of `order`, one after the other (the lists stay
// balanced to within the stealing at the end, since neighbours in `order` have similar lengths).  The lists are
// padded to whole groups of equal number; the padding and the positions past E are holes without work.
// The host asks for this (one_xcd) where an expert's two panels are not much larger than an L2, which is where it pays:
// measured -2.4 % and -4.8 % on the backward launch of the 256-expert shapes (128 rows per expert, memory bound),
// -3.2 % at 128 experts of 384 rows, +1.6 % at 64 experts of 770 rows, whose 6.6 MB of panels are better off spread.
__device__ __forceinline__ int wgrad_queue_total(int E, int tpe, bool one_xcd) {
    if (!one_xcd) return E * tpe;
    const int per_list = ((E + kNumXcd - 1) / kNumXcd) * tpe;
    return ((per_list + kQueueGroup - 1) / kQueueGroup) * kQueueGroup * kNumXcd;
}
// queue number t -> position in `order` and tile of that expert; false: a hole
__device__ __forceinline__ bool wgrad_queue_tile(int t, int E, int tpe, bool one_xcd, int& pos, int& u) {
    if (!one_xcd) {
        pos = t / tpe;
        u = t - pos * tpe;
        return true;
    }
    const int g = t / kQueueGroup, x = g % kNumXcd;
    const int l = (g / kNumXcd) * kQueueGroup + t % kQueueGroup;   // number within list x
    pos = (l / tpe) * kNumXcd + x;
    u = l % tpe;
    return pos < E;
}

#ifndef XMOE_ROW_BAND
#define XMOE_ROW_BAND 4
#endif
constexpr int kRowBand = XMOE_ROW_BAND;   // row tiles per band of the row-GEMM tile numbering
struct RowTile {
    int e, row0, rows;   // expert, first row, valid rows (1..256)
    int col;             // column tile
};
// Tile t of a launch over (row tiles of all experts) x nt column tiles.  An expert's tiles occupy the range of t they
// have in row-major numbering (row tile * nt + column tile); inside it they are numbered band by band (kRowBand row
// tiles), and inside a band down the rows first.  The kQueueGroup consecutive tiles that the workgroups of an XCD take
// together then form a block of about 4 x 4 tiles (8 operand panels for 16 tiles) instead of a strip of one and a half
// rows (12 to 13 panels), whether the expert has three row tiles or thirty.
__device__ __forceinline__ RowTile get_tile(const int32_t* __restrict__ map, const int32_t* __restrict__ off, int t,
                                            int nt) {
    RowTile r;
    const int mt = t / nt;
    r.e = map[4 + 2 * mt];
    const int lo = off[r.e], hi = off[r.e + 1];
    if (kRowBand <= 1) {
        r.row0 = map[4 + 2 * mt + 1];
        r.col = t - mt * nt;
    } else {
        const int mt0 = mt - (map[4 + 2 * mt + 1] - lo) / TM;   // the expert's first row tile
        const int R = (hi - lo + TM - 1) / TM;                  // its row tiles
        const int local = t - mt0 * nt;
        const int band = local / (kRowBand * nt);
        const int in_band = local - band * kRowBand * nt;
        const int band_rows = R - band * kRowBand < kRowBand ? R - band * kRowBand : kRowBand;
        r.col = in_band / band_rows;
        r.row0 = lo + (band * kRowBand + in_band - r.col * band_rows) * TM;
    }
    r.rows = hi - r.row0 < TM ? hi - r.row0 : TM;
    return r;
}

__device__ __forceinline__ Operand row_op(const bf16_t* p, long ld, int rows) {
    Operand o;
    o.p_lo = o.p_hi = p;
    o.ld = ld;
    o.n_lo = o.n_hi = rows;
    o.k_valid = 0;
    o.gather = nullptr;
    o.gather_dma = nullptr;
    return o;
}
__device__ __forceinline__ Operand col_op(const bf16_t* p, long ld, int cols, int k_valid) {
    Operand o;
    o.p_lo = p;
    o.p_hi = p + 128;
    o.ld = ld;
    o.n_lo = cols < 128 ? cols : 128;
    o.n_hi = cols > 128 ? cols - 128 : 0;
    o.k_valid = k_valid;
    o.gather = nullptr;
    o.gather_dma = nullptr;
    return o;
}

// number of 32-row blocks of wave-row wm that contain valid rows
__device__ __forceinline__ int wave_mi_count(int rows) {
    const int wm = threadIdx.x >> 8;
    int r = rows - wm * 128;
    r = r < 0 ? 0 : (r > 128 ? 128 : r);
    return (r + 31) >> 5;
}

}  // namespace

// =========================================================================================================
// forward 1: G = Xd Wg, U = Xd Wu, A = silu(G) * U.   Block tile: 256 rows x (128 gate + 128 up columns).
// =========================================================================================================
// GATHER: xd is the token matrix x and row i of the expert input is x[row_index[i]] (the gather of dispatch fused
// into the operand load).
template <bool GATHER>
__global__ __launch_bounds__(512) void ffn_gateup_dma_kernel(const bf16_t* __restrict__ xd,
                                                             const int32_t* __restrict__ row_index,
                                                             const int32_t* __restrict__ off,
                                                             const int32_t* __restrict__ map, int d, int f,
                                                             const bf16_t* __restrict__ wg,
                                                             const bf16_t* __restrict__ wu, bf16_t* __restrict__ G,
                                                             bf16_t* __restrict__ U, bf16_t* __restrict__ A,
                                                             int32_t* __restrict__ counters, unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    const int nt = (f + 127) / 128;
    TileWalker tw;
    for (int t = tw.start(counters, map[0] * nt, smem); t >= 0; t = tw.next()) {
    tw.draw();
    const RowTile rt = get_tile(map, off, t, nt);
    const int n0 = rt.col * 128;
    const int ncols = f - n0 < 128 ? f - n0 : 128;
    Operand a = row_op(GATHER ? xd : xd + (long)rt.row0 * d, d, rt.rows);
    if (GATHER) a.gather = row_index + rt.row0;
    Operand b;
    b.p_lo = wg + (long)rt.e * d * f + n0;
    b.p_hi = wu + (long)rt.e * d * f + n0;
    b.ld = f;
    b.n_lo = b.n_hi = ncols;
    b.k_valid = d;
    f32x16_t acc[4][2];
    zero_acc(acc);
    const int mi_count = wave_mi_count(rt.rows);
    mainloop<false, true, true, GATHER>(acc, a, b, d, mi_count, smem);
    tw.hand_over();

    const int wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
    char* strip = smem + wave * kStripBytes;
    const int cols_valid = ncols - wn * 32;   // of this wave's 32 columns
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        float g[16], u[16], s[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            g[v] = acc[mi][0][v];
            u[v] = acc[mi][1][v];
            s[v] = g[v] * fast_sigmoid(g[v]) * u[v];
        }
        const int r0 = wm * 128 + mi * 32;
        const int rows_valid = rt.rows - r0;
        const long base = (long)(rt.row0 + r0) * f + n0 + wn * 32;
        strip_put(strip, 0, g);
        strip_put(strip, 32, u);
        strip_sync();
        strip_flush<32>(strip, 0, G + base, f, rows_valid, cols_valid);
        strip_flush<32>(strip, 32, U + base, f, rows_valid, cols_valid);
        strip_sync();
        strip_put(strip, 0, s);
        strip_sync();
        strip_flush<32>(strip, 0, A + base, f, rows_valid, cols_valid);
        strip_sync();
    }
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// forward 2: Y = A Wd          (K = f, N = d, weights "in x out" -> col tile)
// backward 1: dA = dY Wd^T     (K = d, N = f, weights K-contiguous -> row tile) + dG, dU, A in the epilogue
// =========================================================================================================
// DY_GATHER (backward 1 only): X is the [T, K] gradient of the layer's output and row i of dY is
// x_scale[i] * X[x_index[i]] (the backward of combine folded into this GEMM: dA = s * (dOut Wd^T), and the A that
// the weight-gradient kernel multiplies with the gathered dOut rows is written as s * A); x_scale NULL = 1.
// row_part (backward 1 only, may be NULL): partial sums of <unscaled row of dY, Y[row]> = sum_n P[row, n] A[row, n]
// with P the accumulator before the scale and A the unscaled activation - the gradient of the row's scale, i.e. of
// its combine weight, taken here so that nobody has to keep Y for it.  A wave writes the sum over its 64 columns of
// the rows it owns to row_part[(column tile * 4 + wave column) * row_part_ld + row]; the order of the additions is
// fixed, and a later kernel adds the partials of a row in ascending order.
template <bool DACT, bool DY_GATHER = false>
__global__ __launch_bounds__(512) void ffn_rowgemm_dma_kernel(const bf16_t* __restrict__ X,
                                                              const int32_t* __restrict__ x_index,
                                                              const float* __restrict__ x_scale,
                                                              const int32_t* __restrict__ off,
                                                              const int32_t* __restrict__ map, int K, int N,
                                                              const bf16_t* __restrict__ W, bf16_t* __restrict__ Y,
                                                              const bf16_t* __restrict__ G,
                                                              const bf16_t* __restrict__ U, bf16_t* __restrict__ dG,
                                                              bf16_t* __restrict__ dU, bf16_t* __restrict__ A,
                                                              float* __restrict__ row_part, long row_part_ld,
                                                              int32_t* __restrict__ counters, unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    const int nt = (N + TN - 1) / TN;
    TileWalker tw;
    for (int t = tw.start(counters, map[0] * nt, smem); t >= 0; t = tw.next()) {
    tw.draw();
    const RowTile rt = get_tile(map, off, t, nt);
    const int n0 = rt.col * TN;
    const int ncols = N - n0 < TN ? N - n0 : TN;
    Operand a = row_op(DY_GATHER ? X : X + (long)rt.row0 * K, K, rt.rows);
    if (DY_GATHER) a.gather = x_index + rt.row0;
    const bf16_t* We = W + (long)rt.e * K * N;
    f32x16_t acc[4][2];
    zero_acc(acc);
    const int wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
    // waves whose 64 columns lie past N have nothing to compute either
    const int mi_count = (wn * 64 < ncols) ? wave_mi_count(rt.rows) : 0;
    if (DACT) {
        Operand b = row_op(We + (long)n0 * K, K, ncols);   // Wd is [f, d]: its rows are the output columns
        mainloop<false, false, false, DY_GATHER>(acc, a, b, K, mi_count, smem);
    } else {
        Operand b = col_op(We + n0, N, ncols, K);          // Wd is [f, d]: k-rows, output columns contiguous
        mainloop<false, true, false>(acc, a, b, K, mi_count, smem);
    }
    tw.hand_over();
    char* strip = smem + wave * kStripBytes;
    const int lane = threadIdx.x & 63;
    const int cols_valid = ncols - wn * 64;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int r0 = wm * 128 + mi * 32;
        const int rows_valid = rt.rows - r0;
        const long base = (long)(rt.row0 + r0) * N + n0 + wn * 64;
        if (!DACT) {
            float x0[16], x1[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                x0[v] = acc[mi][0][v];
                x1[v] = acc[mi][1][v];
            }
            strip_put(strip, 0, x0);
            strip_put(strip, 32, x1);
            strip_sync();
            strip_flush<64, true>(strip, 0, Y + base, N, rows_valid, cols_valid);
            strip_sync();
        } else {
            // nothing here: the dAct epilogue is handled after the loop (it pipelines its G/U loads over all rounds)
        }
    }
    if (DACT) {
        // 8 rounds (mi, ni) of 32 x 32 outputs.  G and U of a round are fetched as full 64-byte row pieces (4 lanes
        // per row, 16 rows per instruction) while the previous round is computed and stored, then turned into the
        // accumulator layout through a wave-private LDS buffer (rows of 64 bytes, 16-byte chunks XOR-swizzled).
        const int m = lane & 31;
        char* inbuf = smem + 8 * kStripBytes + wave * kInBytes;   // G rows, then U rows
#ifndef XMOE_DACT_PF
#define XMOE_DACT_PF 1
#endif
        constexpr int PF = XMOE_DACT_PF;   // rounds of G / U fetched ahead
        // Two copies of the rounds.  FULL: every row and column of the wave's 128 x 64 block is valid, and no load or
        // store stands inside a branch.  That matters for more than the branches: the compiler can only leave memory
        // operations outstanding at a wait if it knows how many were issued, and with every load and store
        // conditional it waited for all of them (s_waitcnt vmcnt(0)) before each round's G and U were used - the
        // round's own stores and the G and U requested ahead for the next round included.
        const float* sc_base = x_scale ? x_scale + rt.row0 : &kOneF;
        const int sc_stride = x_scale ? 1 : 0;
        auto rounds = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr int NQ = PF + 1;   // buffers of a round's G / U
            uint4 gq[NQ][2], uq[NQ][2];
            const int frow = lane >> 2, fchunk = lane & 3;
            auto fetch = [&](int r, uint4 (&g2)[2], uint4 (&u2)[2]) {
                const int mi = r >> 1, ni = r & 1;
                const int r0 = wm * 128 + mi * 32;
                const int rows_valid = rt.rows - r0;
                const long base = (long)(rt.row0 + r0) * N + n0 + wn * 64 + ni * 32;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = 16 * i + frow;
                    g2[i] = make_uint4(0, 0, 0, 0);
                    u2[i] = make_uint4(0, 0, 0, 0);
                    if (FULL || (row < rows_valid && ni * 32 + fchunk * 8 < cols_valid)) {
                        // a wave-uniform group of 16 rows plus this lane's fixed 32-bit offset
                        const uint32_t o = (uint32_t)(frow * N + fchunk * 8) * 2u;
                        g2[i] = *reinterpret_cast<const uint4*>(
                            reinterpret_cast<const char*>(G + base + (long)(16 * i) * N) + o);
                        u2[i] = *reinterpret_cast<const uint4*>(
                            reinterpret_cast<const char*>(U + base + (long)(16 * i) * N) + o);
                    }
                }
            };
            // FULL: the four row blocks' scales first, ahead of every other request of the epilogue (requested where
            // they are used they would be the newest request each time, and waiting for the newest is waiting for
            // all).  No branch: without scales every lane reads a 1.  Read as global memory: through the selected
            // pointer it would be a flat load, which the compiler can only wait for by waiting for everything.
            float scv[4] = {1.0f, 1.0f, 1.0f, 1.0f};
            if (DY_GATHER && FULL) {
                typedef const __attribute__((address_space(1))) char* gchar_p;
                typedef const __attribute__((address_space(1))) float* gfloat_p;
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    scv[mi] = *(gfloat_p)((gchar_p)GLB_PTR(sc_base) +
                                          (uint32_t)((wm * 128 + mi * 32 + m) * sc_stride) * 4u);
            }
#pragma unroll
            for (int r = 0; r < PF; ++r) fetch(r, gq[r], uq[r]);
            float rowpart = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int mi = r >> 1, ni = r & 1;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = 16 * i + frow;
                    const int pos = (fchunk ^ ((row >> 2) & 3)) << 4;
                    *reinterpret_cast<uint4*>(inbuf + row * 64 + pos) = gq[r % NQ][i];
                    *reinterpret_cast<uint4*>(inbuf + 2048 + row * 64 + pos) = uq[r % NQ][i];
                }
                if (r + PF < 8) fetch(r + PF, gq[(r + PF) % NQ], uq[(r + PF) % NQ]);
                strip_sync();
                const int r0 = wm * 128 + mi * 32;
                const int rows_valid = rt.rows - r0;
                const long base = (long)(rt.row0 + r0) * N + n0 + wn * 64;
                uint2 gv[4], uv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {   // columns 8q + 4*(lane/32) .. +3 of row m: half (lane/32) of chunk q
                    const int off = m * 64 + ((q ^ ((m >> 2) & 3)) << 4) + 8 * (lane >> 5);
                    gv[q] = *reinterpret_cast<const uint2*>(inbuf + off);
                    uv[q] = *reinterpret_cast<const uint2*>(inbuf + 2048 + off);
                }
                float sc = 1.0f;   // DY_GATHER: the scale of this lane's row
                if (DY_GATHER && FULL)
                    sc = scv[mi];
                else if (DY_GATHER && x_scale && m < rows_valid)
                    sc = x_scale[rt.row0 + r0 + m];
                float part = 0.f;   // this lane's 16 columns of <unscaled dY row, Y row>
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t gw[2] = {gv[q].x, gv[q].y}, uw[2] = {uv[q].x, uv[q].y};
                    float dg[4], du[4], av[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t gb = (j & 1) ? (gw[j >> 1] & 0xffff0000u) : (gw[j >> 1] << 16);
                        const uint32_t ub = (j & 1) ? (uw[j >> 1] & 0xffff0000u) : (uw[j >> 1] << 16);
                        const float g = __uint_as_float(gb), u = __uint_as_float(ub);
                        const float pa = acc[mi][ni][4 * q + j];
                        const float da = DY_GATHER ? pa * sc : pa;
                        const float sg = fast_sigmoid(g);
                        const float sl = g * sg;
                        const float a1 = sl * u;
                        dg[j] = da * u * (sg * (1.0f + g * (1.0f - sg)));
                        du[j] = da * sl;
                        av[j] = DY_GATHER ? a1 * sc : a1;
                        part = fmaf(pa, a1, part);
                    }
                    strip_put4(strip, ni * 32, q, dg[0], dg[1], dg[2], dg[3]);
                    strip_put4(strip, 64 + ni * 32, q, du[0], du[1], du[2], du[3]);
                    strip_put4(strip, 128 + ni * 32, q, av[0], av[1], av[2], av[3]);
                }
                {   // the two column halves of the row block, then the lane pair of a row
                    rowpart = ni == 0 ? part : rowpart + part;
                    if (ni == 1) {
                        const float tot = rowpart + __shfl_xor(rowpart, 32, 64);
                        // (FULL: both lanes of a row hold the same total and both store it)
                        if (FULL || (lane < 32 && m < rows_valid))
                            *reinterpret_cast<float*>(
                                reinterpret_cast<char*>(row_part + (long)(rt.col * 4 + wn) * row_part_ld + rt.row0 + r0) +
                                (uint32_t)m * 4u) = tot;
                    }
                }
                if (ni == 1) {   // the row block's 64 columns of each output go out as whole 128-byte lines
                    strip_sync();
                    strip_flush<64, false, !FULL, true>(strip, 0, dG + base, N, rows_valid, cols_valid);
                    __builtin_amdgcn_sched_barrier(0);   // (keeps the staged rows of one output in registers at a time)
                    strip_flush<64, false, !FULL, true>(strip, 64, dU + base, N, rows_valid, cols_valid);
                    __builtin_amdgcn_sched_barrier(0);
                    strip_flush<64, false, !FULL, true>(strip, 128, A + base, N, rows_valid, cols_valid);
                    strip_sync();
                }
            }
        };
        if (rt.rows - wm * 128 >= 128 && cols_valid >= 64)
            rounds(std::true_type{});
        else
            rounds(std::false_type{});
    }
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// backward 2: dXd = dG Wg^T + dU Wu^T     (K = f twice, N = d; Wg, Wu [d, f]: rows are output columns)
// =========================================================================================================
// TWO = false: a single pair (the two-matrix expert: dXd = dH W1^T), dU and wu are not read
// one tile of it; t counts (row tiles of all experts) x column tiles
template <bool TWO>
__device__ __forceinline__ void dx_tile(int t, TileWalker& tw, char* smem, const bf16_t* __restrict__ dG,
                                        const bf16_t* __restrict__ dU, const int32_t* __restrict__ off,
                                        const int32_t* __restrict__ map, int d, int f,
                                        const bf16_t* __restrict__ wg, const bf16_t* __restrict__ wu,
                                        bf16_t* __restrict__ dXd) {
    const int nt = (d + TN - 1) / TN;
    const RowTile rt = get_tile(map, off, t, nt);
    const int n0 = rt.col * TN;
    const int ncols = d - n0 < TN ? d - n0 : TN;
    const int wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
    const int mi_count = (wn * 64 < ncols) ? wave_mi_count(rt.rows) : 0;
    f32x16_t acc[4][2];
    zero_acc(acc);
    {
        Operand a1 = row_op(dG + (long)rt.row0 * f, f, rt.rows);
        Operand b1 = row_op(wg + (long)rt.e * d * f + (long)n0 * f, f, ncols);
        Operand a2 = TWO ? row_op(dU + (long)rt.row0 * f, f, rt.rows) : a1;
        Operand b2 = TWO ? row_op(wu + (long)rt.e * d * f + (long)n0 * f, f, ncols) : b1;
        mainloop2<false, false, false, TWO>(acc, a1, b1, f, a2, b2, TWO ? f : 0, mi_count, smem);
    }
    tw.hand_over();
    char* strip = smem + wave * kStripBytes;
    const int cols_valid = ncols - wn * 64;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int r0 = wm * 128 + mi * 32;
        float x0[16], x1[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            x0[v] = acc[mi][0][v];
            x1[v] = acc[mi][1][v];
        }
        strip_put(strip, 0, x0);
        strip_put(strip, 32, x1);
        strip_sync();
        strip_flush<64, true>(strip, 0, dXd + (long)(rt.row0 + r0) * d + n0 + wn * 64, d, rt.rows - r0, cols_valid);
        strip_sync();
    }
}

template <bool TWO>
__global__ __launch_bounds__(512) void ffn_dx_dma_kernel(const bf16_t* __restrict__ dG, const bf16_t* __restrict__ dU,
                                                         const int32_t* __restrict__ off,
                                                         const int32_t* __restrict__ map, int d, int f,
                                                         const bf16_t* __restrict__ wg, const bf16_t* __restrict__ wu,
                                                         bf16_t* __restrict__ dXd, int32_t* __restrict__ counters, unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    const int nt = (d + TN - 1) / TN;
    TileWalker tw;
    for (int t = tw.start(counters, map[0] * nt, smem); t >= 0; t = tw.next()) {
        tw.draw();
        dx_tile<TWO>(t, tw, smem, dG, dU, off, map, d, f, wg, wu, dXd);
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// two-matrix expert, forward 1: H = Xd W1, A = act(H)      (K = d, N = f, weights "in x out" -> col tile)
// =========================================================================================================
// activation of the matrix-core epilogues: silu takes the hardware exp2 / reciprocal like the SwiGLU epilogues
// and gelu takes the error function from the rational approximation 7.1.26 of Abramowitz and Stegun
//   erf(x) = 1 - (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-x^2),  t = 1 / (1 + p x),  x >= 0,  |error| <= 1.5e-7,
// far below half a bf16 unit of the stored result; its exp(-x^2) with x = h / sqrt(2) is also the Gaussian density
// that the derivative needs.
__device__ __forceinline__ void fast_gelu_parts(float h, float& Phi, float& phi) {
    const float x = fabsf(h) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
    const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * x * x);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float erf_abs = 1.0f - poly * e;
    Phi = 0.5f * (1.0f + copysignf(erf_abs, h));
    phi = 0.39894228040143268f * e;
}
template <int ACT>
__device__ __forceinline__ float act_fast(float h) {
    if (ACT == XMOE_ACT_SILU) return h * fast_sigmoid(h);
    if (ACT == XMOE_ACT_GELU) {
        float Phi, phi;
        fast_gelu_parts(h, Phi, phi);
        return h * Phi;
    }
    return h;
}
template <int ACT>
__device__ __forceinline__ void act_fast_grad(float h, float& a, float& g) {
    if (ACT == XMOE_ACT_SILU) {
        const float sg = fast_sigmoid(h);
        a = h * sg;
        g = sg * (1.0f + h * (1.0f - sg));
    } else if (ACT == XMOE_ACT_GELU) {
        float Phi, phi;
        fast_gelu_parts(h, Phi, phi);
        a = h * Phi;
        g = Phi + h * phi;
    } else {
        a = h;
        g = 1.0f;
    }
}

template <bool GATHER, int ACT>
__global__ __launch_bounds__(512) void mlp2_up_dma_kernel(const bf16_t* __restrict__ xd,
                                                          const int32_t* __restrict__ row_index,
                                                          const int32_t* __restrict__ off,
                                                          const int32_t* __restrict__ map, int d, int f,
                                                          const bf16_t* __restrict__ w1, bf16_t* __restrict__ H,
                                                          bf16_t* __restrict__ A, int32_t* __restrict__ counters, unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    const int nt = (f + TN - 1) / TN;
    TileWalker tw;
    for (int t = tw.start(counters, map[0] * nt, smem); t >= 0; t = tw.next()) {
        tw.draw();
        const RowTile rt = get_tile(map, off, t, nt);
        const int n0 = rt.col * TN;
        const int ncols = f - n0 < TN ? f - n0 : TN;
        Operand a = row_op(GATHER ? xd : xd + (long)rt.row0 * d, d, rt.rows);
        if (GATHER) a.gather = row_index + rt.row0;
        Operand b = col_op(w1 + (long)rt.e * d * f + n0, f, ncols, d);
        f32x16_t acc[4][2];
        zero_acc(acc);
        const int wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
        const int mi_count = (wn * 64 < ncols) ? wave_mi_count(rt.rows) : 0;
        mainloop<false, true, false, GATHER>(acc, a, b, d, mi_count, smem);
        tw.hand_over();
        char* strip = smem + wave * kStripBytes;
        const int cols_valid = ncols - wn * 64;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int r0 = wm * 128 + mi * 32;
            const int rows_valid = rt.rows - r0;
            const long base = (long)(rt.row0 + r0) * f + n0 + wn * 64;
            float x0[16], x1[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                x0[v] = acc[mi][0][v];
                x1[v] = acc[mi][1][v];
            }
            strip_put(strip, 0, x0);
            strip_put(strip, 32, x1);
            strip_sync();
            strip_flush<64>(strip, 0, H + base, f, rows_valid, cols_valid);
            strip_sync();
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                x0[v] = act_fast<ACT>(x0[v]);
                x1[v] = act_fast<ACT>(x1[v]);
            }
            strip_put(strip, 0, x0);
            strip_put(strip, 32, x1);
            strip_sync();
            strip_flush<64>(strip, 0, A + base, f, rows_valid, cols_valid);
            strip_sync();
        }
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// two-matrix expert, backward 1: dA = dY W2^T (K = d, N = f; W2 [f, d]: its rows are the output columns), then
// dH = dA * act'(H) and A = act(H) in the epilogue
// =========================================================================================================
// DY_GATHER: as in ffn_rowgemm_dma_kernel (row i of dY is dy_scale[i] * dY[dy_index[i]]; A is written scaled)
template <int ACT, bool DY_GATHER>
__global__ __launch_bounds__(512) void mlp2_dact_dma_kernel(const bf16_t* __restrict__ dY,
                                                            const int32_t* __restrict__ dy_index,
                                                            const float* __restrict__ dy_scale,
                                                            const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ map, int d, int f,
                                                            const bf16_t* __restrict__ w2,
                                                            const bf16_t* __restrict__ H, bf16_t* __restrict__ dH,
                                                            bf16_t* __restrict__ A,
                                                            float* __restrict__ row_part, long row_part_ld,
                                                            int32_t* __restrict__ counters, unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    const int nt = (f + TN - 1) / TN;
    TileWalker tw;
    for (int t = tw.start(counters, map[0] * nt, smem); t >= 0; t = tw.next()) {
        tw.draw();
        const RowTile rt = get_tile(map, off, t, nt);
        const int n0 = rt.col * TN;
        const int ncols = f - n0 < TN ? f - n0 : TN;
        Operand a = row_op(DY_GATHER ? dY : dY + (long)rt.row0 * d, d, rt.rows);
        if (DY_GATHER) a.gather = dy_index + rt.row0;
        Operand b = row_op(w2 + (long)rt.e * f * d + (long)n0 * d, d, ncols);
        f32x16_t acc[4][2];
        zero_acc(acc);
        const int wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
        const int lane = threadIdx.x & 63;
        const int mi_count = (wn * 64 < ncols) ? wave_mi_count(rt.rows) : 0;
        mainloop<false, false, false, DY_GATHER>(acc, a, b, d, mi_count, smem);
        tw.hand_over();
        char* strip = smem + wave * kStripBytes;
        const int cols_valid = ncols - wn * 64;
        // 8 rounds (mi, ni) of 32 x 32 outputs.  H of a round is fetched as full 64-byte row pieces (4 lanes per
        // row, 16 rows per instruction) while the previous round is computed and stored, then turned into the
        // accumulator layout through a wave-private LDS buffer (rows of 64 bytes, 16-byte chunks XOR-swizzled).
        const int m = lane & 31;
        char* inbuf = smem + 8 * kStripBytes + wave * kInBytes;
        // two copies of the rounds, as in ffn_rowgemm_dma_kernel: FULL has no branch around any load or store
        const float* sc_base = dy_scale ? dy_scale + rt.row0 : &kOneF;
        const int sc_stride = dy_scale ? 1 : 0;
        auto rounds = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            uint4 hq[2][2];
            const int frow = lane >> 2, fchunk = lane & 3;
            auto fetch = [&](int r, uint4 (&h2)[2]) {
                const int mi = r >> 1, ni = r & 1;
                const int r0 = wm * 128 + mi * 32;
                const int rows_valid = rt.rows - r0;
                const long base = (long)(rt.row0 + r0) * f + n0 + wn * 64 + ni * 32;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = 16 * i + frow;
                    h2[i] = make_uint4(0, 0, 0, 0);
                    if (FULL || (row < rows_valid && ni * 32 + fchunk * 8 < cols_valid)) {
                        // a wave-uniform group of 16 rows plus this lane's fixed 32-bit offset
                        const uint32_t o = (uint32_t)(frow * f + fchunk * 8) * 2u;
                        h2[i] = *reinterpret_cast<const uint4*>(
                            reinterpret_cast<const char*>(H + base + (long)(16 * i) * f) + o);
                    }
                }
            };
            float scv[4] = {1.0f, 1.0f, 1.0f, 1.0f};   // FULL: the four row blocks' scales, requested first
            if (DY_GATHER && FULL) {
                typedef const __attribute__((address_space(1))) char* gchar_p;
                typedef const __attribute__((address_space(1))) float* gfloat_p;
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    scv[mi] = *(gfloat_p)((gchar_p)GLB_PTR(sc_base) +
                                          (uint32_t)((wm * 128 + mi * 32 + m) * sc_stride) * 4u);
            }
            fetch(0, hq[0]);
            float rowpart = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int mi = r >> 1, ni = r & 1;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int row = 16 * i + frow;
                    const int pos = (fchunk ^ ((row >> 2) & 3)) << 4;
                    *reinterpret_cast<uint4*>(inbuf + row * 64 + pos) = hq[r & 1][i];
                }
                if (r + 1 < 8) fetch(r + 1, hq[(r + 1) & 1]);
                strip_sync();
                const int r0 = wm * 128 + mi * 32;
                const int rows_valid = rt.rows - r0;
                const long base = (long)(rt.row0 + r0) * f + n0 + wn * 64;
                uint2 hv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q)   // columns 8q + 4*(lane/32) .. +3 of row m: half (lane/32) of chunk q
                    hv[q] = *reinterpret_cast<const uint2*>(inbuf + m * 64 + ((q ^ ((m >> 2) & 3)) << 4) + 8 * (lane >> 5));
                float sc = 1.0f;   // DY_GATHER: the scale of this lane's row
                if (DY_GATHER && FULL)
                    sc = scv[mi];
                else if (DY_GATHER && dy_scale && m < rows_valid)
                    sc = dy_scale[rt.row0 + r0 + m];
                float part = 0.f;   // this lane's 16 columns of <unscaled dY row, Y row> (see ffn_rowgemm_dma_kernel)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t hw[2] = {hv[q].x, hv[q].y};
                    float dh[4], av[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t hb = (j & 1) ? (hw[j >> 1] & 0xffff0000u) : (hw[j >> 1] << 16);
                        float a_, g_;
                        act_fast_grad<ACT>(__uint_as_float(hb), a_, g_);
                        const float pa = acc[mi][ni][4 * q + j];
                        dh[j] = DY_GATHER ? pa * sc * g_ : pa * g_;
                        av[j] = DY_GATHER ? a_ * sc : a_;
                        part = fmaf(pa, a_, part);
                    }
                    strip_put4(strip, ni * 32, q, dh[0], dh[1], dh[2], dh[3]);
                    strip_put4(strip, 64 + ni * 32, q, av[0], av[1], av[2], av[3]);
                }
                {
                    rowpart = ni == 0 ? part : rowpart + part;
                    if (ni == 1) {
                        const float tot = rowpart + __shfl_xor(rowpart, 32, 64);
                        if (FULL || (lane < 32 && m < rows_valid))
                            row_part[(long)(rt.col * 4 + wn) * row_part_ld + rt.row0 + r0 + m] = tot;
                    }
                }
                if (ni == 1) {
                    strip_sync();
                    strip_flush<64, false, !FULL, true>(strip, 0, dH + base, f, rows_valid, cols_valid);
                    strip_flush<64, false, !FULL, true>(strip, 64, A + base, f, rows_valid, cols_valid);
                    strip_sync();
                }
            }
        };
        if (rt.rows - wm * 128 >= 128 && cols_valid >= 64)
            rounds(std::true_type{});
        else
            rounds(std::false_type{});
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// weight gradients: dW_e[m, n] = sum over the expert's rows r of P[r, m] * Q[r, n]   (K = ragged row count; both
// operands are K-strided -> col tiles).  DUAL: two right-hand sides Q1, Q2 sharing P (dWg and dWu share Xd);
// the block then covers 128 columns of each.  An expert with no rows gets zeros.
// =========================================================================================================
// GATHER: P is a [T, M] matrix and row r of the expert's P is P[row_index[lo + r]].  QGATHER (not with DUAL): the
// same for Q1 through q_index (the gradient of the layer's output standing in for the rows of dY).
// one tile of it; t counts experts (in the order of `order`) x row tiles x column tiles
template <bool DUAL, bool GATHER, bool QGATHER>
__device__ __forceinline__ void wgrad_tile(int t, TileWalker& tw, char* smem, const bf16_t* __restrict__ P,
                                           const int32_t* __restrict__ row_index, const bf16_t* __restrict__ Q1,
                                           const bf16_t* __restrict__ Q2, const int32_t* __restrict__ q_index,
                                           const int32_t* __restrict__ row_index_dma,
                                           const int32_t* __restrict__ q_index_dma, const int32_t* __restrict__ off,
                                           const int32_t* __restrict__ order, int E, bool one_xcd, int M,
                                           int N, bf16_t* __restrict__ dW1, bf16_t* __restrict__ dW2) {
    constexpr int NB = DUAL ? 128 : TN;   // output columns per block and matrix
    const int mt = (M + TM - 1) / TM, nt = (N + NB - 1) / NB;
    int pos, u;
    if (!wgrad_queue_tile(t, E, mt * nt, one_xcd, pos, u)) {
        tw.hand_over();
        return;
    }
    const int e = order[pos];
    // Inside an expert the tiles are numbered band by band (kWgradBand tile rows), down the columns of a band, so
    // that the kQueueGroup consecutive tiles a group of workgroups takes form a 2 x 8 block of tiles rather than a
    // 1 x 16 strip: the operand that the strip would fetch once per tile is then fetched once per two tiles
    // (measured: bands of 2 beat bands of 1 and of 4 by 3 to 4 % on both the long and the short segments).
    const int band = u / (kWgradBand * nt);
    const int in_band = u - band * kWgradBand * nt;
    const int band_rows = mt - band * kWgradBand < kWgradBand ? mt - band * kWgradBand : kWgradBand;
    const int m0 = (band * kWgradBand + in_band % band_rows) * TM, n0 = (in_band / band_rows) * NB;
    const int lo = off[e], hi = off[e + 1];
    const int K = hi - lo;
    const int mrows = M - m0 < TM ? M - m0 : TM, ncols = N - n0 < NB ? N - n0 : NB;
    const int wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
    f32x16_t acc[4][2];
    zero_acc(acc);
    if (K > 0) {
        // GATHER: P is the token matrix and k-row r of the expert's P is P[row_index[lo + r]]
        Operand a = col_op(GATHER ? P + m0 : P + (long)lo * M + m0, M, mrows, K);
        if (GATHER) a.gather = row_index + lo, a.gather_dma = row_index_dma + lo;
        Operand b;
        if (DUAL) {
            b.p_lo = Q1 + (long)lo * N + n0;
            b.p_hi = Q2 + (long)lo * N + n0;
            b.ld = N;
            b.n_lo = b.n_hi = ncols;
            b.k_valid = K;
        } else {
            b = col_op(QGATHER ? Q1 + n0 : Q1 + (long)lo * N + n0, N, ncols, K);
            if (QGATHER) b.gather = q_index + lo, b.gather_dma = q_index_dma + lo;
        }
        // DUAL: the B tile is [Q1's 128 columns | Q2's 128 columns]; a wave takes 64 contiguous columns of ONE of
        // the two (waves 0, 1: Q1; waves 2, 3: Q2), so that it stores whole 128-byte lines of one matrix
        const int wcol = DUAL ? (wn & 1) * 64 : wn * 64;
        const int mi_count = (wcol < ncols) ? wave_mi_count(mrows) : 0;
        static_assert(!(DUAL && QGATHER), "the gathered right-hand side is a single matrix");
        mainloop<true, true, false, GATHER, QGATHER>(acc, a, b, K, mi_count, smem);
    }
    tw.hand_over();
    char* strip = smem + wave * kStripBytes;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int r0 = wm * 128 + mi * 32;
        float x0[16], x1[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            x0[v] = acc[mi][0][v];
            x1[v] = acc[mi][1][v];
        }
        strip_put(strip, 0, x0);
        strip_put(strip, 32, x1);
        strip_sync();
        if (DUAL) {
            const long o = (long)e * M * N + (long)(m0 + r0) * N + n0 + (wn & 1) * 64;
            strip_flush<64, true>(strip, 0, (wn < 2 ? dW1 : dW2) + o, N, mrows - r0, ncols - (wn & 1) * 64);
        } else {
            const long o = (long)e * M * N + (long)(m0 + r0) * N + n0 + wn * 64;
            strip_flush<64, true>(strip, 0, dW1 + o, N, mrows - r0, ncols - wn * 64);
        }
        strip_sync();
    }
}

template <bool DUAL, bool GATHER, bool QGATHER = false>
__global__ __launch_bounds__(512) void ffn_wgrad_dma_kernel(const bf16_t* __restrict__ P,
                                                            const int32_t* __restrict__ row_index,
                                                            const bf16_t* __restrict__ Q1,
                                                            const bf16_t* __restrict__ Q2,
                                                            const int32_t* __restrict__ q_index,
                                                            const int32_t* __restrict__ row_index_dma,
                                                            const int32_t* __restrict__ q_index_dma,
                                                            const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ order,
                                                            int32_t* __restrict__ counters, int E, int one_xcd,
                                                            int M, int N, bf16_t* __restrict__ dW1,
                                                            bf16_t* __restrict__ dW2,
                                                            unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    constexpr int NB = DUAL ? 128 : TN;
    const int mt = (M + TM - 1) / TM, nt = (N + NB - 1) / NB;
    TileWalker tw;
    for (int t = tw.start(counters, wgrad_queue_total(E, mt * nt, one_xcd), smem); t >= 0; t = tw.next()) {
        tw.draw();
        wgrad_tile<DUAL, GATHER, QGATHER>(t, tw, smem, P, row_index, Q1, Q2, q_index, row_index_dma, q_index_dma, off,
                                          order, E, one_xcd, M, N, dW1, dW2);
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// backward of the SwiGLU expert after dG, dU and A exist: dXd, dWd and dWg | dWu in ONE launch.  The three GEMMs
// are independent of each other, so a workgroup that finds dXd's tile queue empty goes straight on to dWd's and
// then to dWg | dWu's (each from the largest expert down) instead of idling until the launch ends: two of three
// launch tails and two launch gaps disappear.  The three walks are separate loops, each with the counters it has
// as a launch of its own, so each keeps the register allocation of its own kernel.
// =========================================================================================================
// SWIGLU = false: the two-matrix expert (dXd = dH W1^T, dW2 = A^T dY, dW1 = Xd^T dH; dG stands for dH, wg for W1,
// dWg for dW1; dU, wu and dWu are not used)
template <bool SWIGLU, bool GATHER, bool DY_GATHER>
__global__ __launch_bounds__(512) void ffn_bwd_rest_dma_kernel(
    const bf16_t* __restrict__ dG, const bf16_t* __restrict__ dU, const bf16_t* __restrict__ act,
    const bf16_t* __restrict__ dY, const int32_t* __restrict__ dy_index, const int32_t* __restrict__ dy_index_dma,
    const bf16_t* __restrict__ xd, const int32_t* __restrict__ row_index, const int32_t* __restrict__ row_index_dma,
    const int32_t* __restrict__ off, const int32_t* __restrict__ map, const int32_t* __restrict__ order,
    int32_t* __restrict__ cnt_dx, int32_t* __restrict__ cnt_wd, int32_t* __restrict__ cnt_wgu, int E, int one_xcd,
    int d, int f,
    const bf16_t* __restrict__ wg, const bf16_t* __restrict__ wu, bf16_t* __restrict__ dXd, bf16_t* __restrict__ dWd,
    bf16_t* __restrict__ dWg, bf16_t* __restrict__ dWu, unsigned long long* __restrict__ clk) {
    extern __shared__ __align__(16) char smem[];
    clock_note(clk, 0);
    TileWalker tw;
    for (int t = tw.start(cnt_dx, map[0] * ((d + TN - 1) / TN), smem); t >= 0; t = tw.next()) {
        tw.draw();
        dx_tile<SWIGLU>(t, tw, smem, dG, dU, off, map, d, f, wg, wu, dXd);
    }
    // a walk's start writes the hand-over slot that the last next() of the walk before it has just read
    __syncthreads();
    for (int t = tw.start(cnt_wd, wgrad_queue_total(E, ((f + TM - 1) / TM) * ((d + TN - 1) / TN), one_xcd), smem); t >= 0;
         t = tw.next()) {
        tw.draw();
        wgrad_tile<false, false, DY_GATHER>(t, tw, smem, act, nullptr, dY, nullptr, dy_index, nullptr, dy_index_dma,
                                            off, order, E, one_xcd, f, d, dWd, nullptr);
    }
    __syncthreads();
    constexpr int NB = SWIGLU ? 128 : TN;
    for (int t = tw.start(cnt_wgu, wgrad_queue_total(E, ((d + TM - 1) / TM) * ((f + NB - 1) / NB), one_xcd), smem); t >= 0;
         t = tw.next()) {
        tw.draw();
        wgrad_tile<SWIGLU, GATHER, false>(t, tw, smem, xd, row_index, dG, dU, nullptr, row_index_dma, nullptr, off,
                                          order, E, one_xcd, d, f, dWg, dWu);
    }
    clock_note(clk, 1);
}

// =========================================================================================================
// host side
// =========================================================================================================
bool ffn_dma_supported(const FfnArgs& a) {
    if (a.dt != XMOE_BF16) return false;
    if (a.d % 64 != 0 || a.f % 64 != 0) return false;
    const void* ptrs[] = {a.xd, a.wg, a.wu, a.wd, a.g, a.u, a.y, a.dy, a.dxd, a.dwg, a.dwu, a.dwd, a.act, a.dg, a.du};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return false;
    return true;
}

// Host-side state of this family, all of it set up once per device on the first call there (the calls themselves
// stay stateless: nothing below depends on an earlier call's arguments):
//   num_cu       compute units of the device, rounded down to a multiple of the XCD count (persistent grid size)
//   clock_probe  device address of g_clock_probe on that device
//   the raised dynamic-LDS limit of every kernel of the family
// Not synchronised: the first call on a device must not race with another call on the same device.
constexpr int kMaxDevices = 64;
struct DeviceState {
    int status = -1;   // -1: not initialised; else an xmoe_status
    int num_cu = 0;
    unsigned long long* clock_probe = nullptr;
};
static DeviceState g_dev[kMaxDevices];
static thread_local DeviceState* t_dev = nullptr;   // the device of the call in progress on this thread

// The backward's three independent GEMMs run as one launch unless the environment variable XMOE_BWD_MERGE is 0
// (for comparisons and for the per-kernel profiles); read once per process.
static bool bwd_merged() {
    static int v = -1;
    if (v < 0) {
        const char* e = getenv("XMOE_BWD_MERGE");
        v = (e && e[0] == '0') ? 0 : 1;
    }
    return v == 1;
}

// the work counters of a call's i-th row-GEMM launch (the schedule block holds, behind the sorted experts, kNumXcd
// counters for each of the two weight-gradient launches and then for each of the two row-GEMM launches)
static inline int32_t* row_counters(int32_t* sched, int E, int i) { return sched + E + (2 + i) * kNumXcd; }

// persistent launch: one workgroup per CU, but never more than there are tiles (host-side upper bound); a
// multiple of the XCD count
static inline unsigned round_up8(long v) {
    long g = (v + 7) / 8 * 8;
    const int num_cu = t_dev ? t_dev->num_cu : 0;
    if (num_cu > 0 && g > num_cu) g = num_cu;
    return (unsigned)(g < 8 ? 8 : g);
}

// the kernel's clock-probe slot while the launch profiler is on, else NULL
static inline unsigned long long* clock_slot(int slot) {
    return (prof_enabled() && t_dev && t_dev->clock_probe) ? t_dev->clock_probe + 4 * slot : nullptr;
}

template <class Kern>
static int allow_lds(Kern k, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                               bytes) == hipSuccess
               ? XMOE_OK
               : XMOE_ERR_HIP;
}
template <class Kern>
static int allow_big_lds(Kern k) {
    // the large-tile kernels use all 160 KiB of a CU's LDS, above the 64 KiB default limit
    return allow_lds(k, kLdsBytes);
}

static int init_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return XMOE_ERR_HIP;
    DeviceState& ds = g_dev[dev];
    t_dev = &ds;
    if (ds.status >= 0) return ds.status;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return ds.status = XMOE_ERR_HIP;
    ds.num_cu = prop.multiProcessorCount / kNumXcd * kNumXcd;
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_clock_probe)) != hipSuccess) return ds.status = XMOE_ERR_HIP;
    ds.clock_probe = static_cast<unsigned long long*>(sym);
    int st = XMOE_OK;
    if (st == XMOE_OK) st = allow_big_lds(ffn_gateup_dma_kernel<false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_gateup_dma_kernel<true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_rowgemm_dma_kernel<false, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_rowgemm_dma_kernel<true, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_rowgemm_dma_kernel<true, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_wgrad_dma_kernel<false, false, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_dx_dma_kernel<true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<true, false, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<true, false, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<true, true, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<true, true, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<false, false, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<false, false, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<false, true, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_bwd_rest_dma_kernel<false, true, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_dx_dma_kernel<false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_wgrad_dma_kernel<false, true>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_up_dma_kernel<false, XMOE_ACT_IDENTITY>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_up_dma_kernel<false, XMOE_ACT_GELU>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_up_dma_kernel<false, XMOE_ACT_SILU>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_up_dma_kernel<true, XMOE_ACT_IDENTITY>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_up_dma_kernel<true, XMOE_ACT_GELU>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_up_dma_kernel<true, XMOE_ACT_SILU>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_dact_dma_kernel<XMOE_ACT_IDENTITY, false>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_dact_dma_kernel<XMOE_ACT_IDENTITY, true>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_dact_dma_kernel<XMOE_ACT_GELU, false>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_dact_dma_kernel<XMOE_ACT_GELU, true>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_dact_dma_kernel<XMOE_ACT_SILU, false>);
    if (st == XMOE_OK) st = allow_big_lds(mlp2_dact_dma_kernel<XMOE_ACT_SILU, true>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_wgrad_dma_kernel<false, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_wgrad_dma_kernel<true, false>);
    if (st == XMOE_OK) st = allow_big_lds(ffn_wgrad_dma_kernel<true, true>);
    return ds.status = st;
}

// whether the weight gradients' tiles of an expert all go to one XCD: where its two panels (the mean number of rows
// of the d-wide and the f-wide operand) take at most 5.5 MiB - somewhat more than that XCD's 4 MiB of L2 still pays
// (measured: 2.5 MiB -2.4 %, 4.9 MiB -3.2 %, 5.1 MiB +-0, 6.6 MiB +1.6 % on the backward launch)
#ifndef XMOE_WGRAD_ONE_XCD_BYTES
#define XMOE_WGRAD_ONE_XCD_BYTES (11l << 19)
#endif
template <class Args>
static inline int wgrad_one_xcd(const Args& a) {
    return (long)(a.B / (a.E > 0 ? a.E : 1) + 1) * (a.d + a.f) * 2 <= XMOE_WGRAD_ONE_XCD_BYTES;
}

int ffn_fwd_dma(const FfnArgs& a, hipStream_t s) {
    int st = init_device();
    if (st != XMOE_OK) return st;
    const int max_tiles = ffn_max_tiles(a.B, a.E, TM);
    st = launch_tile_map(a.off, a.E, TM, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const bf16_t *xd = (const bf16_t*)a.xd, *wg = (const bf16_t*)a.wg, *wu = (const bf16_t*)a.wu,
                 *wd = (const bf16_t*)a.wd;
    const int ntg = (a.f + 127) / 128, ntd = (a.d + TN - 1) / TN;
    if (a.row_index)
        XMOE_LAUNCH(K_FFN_GATEUP_DMA, s,
                    hipLaunchKernelGGL(ffn_gateup_dma_kernel<true>, dim3(round_up8((long)max_tiles * ntg)), dim3(512),
                                       kLdsBytes, s, xd, a.row_index, a.off, a.map, a.d, a.f, wg, wu, (bf16_t*)a.g,
                                       (bf16_t*)a.u, (bf16_t*)a.act, row_counters(a.sched, a.E, 0), clock_slot(CS_GATEUP)));
    else
        XMOE_LAUNCH(K_FFN_GATEUP_DMA, s,
                    hipLaunchKernelGGL(ffn_gateup_dma_kernel<false>, dim3(round_up8((long)max_tiles * ntg)), dim3(512),
                                       kLdsBytes, s, xd, nullptr, a.off, a.map, a.d, a.f, wg, wu, (bf16_t*)a.g,
                                       (bf16_t*)a.u, (bf16_t*)a.act, row_counters(a.sched, a.E, 0), clock_slot(CS_GATEUP)));
    XMOE_LAUNCH(K_FFN_DOWN_DMA, s,
                hipLaunchKernelGGL((ffn_rowgemm_dma_kernel<false, false>), dim3(round_up8((long)max_tiles * ntd)), dim3(512),
                                   kLdsBytes, s, (const bf16_t*)a.act, nullptr, nullptr, a.off, a.map, a.f, a.d, wd,
                                   (bf16_t*)a.y, nullptr,
                                   nullptr, nullptr, nullptr, nullptr, (float*)nullptr, 0L, row_counters(a.sched, a.E, 1), clock_slot(CS_DOWN)));
    return XMOE_OK;
}

int ffn_bwd_dma(const FfnArgs& a, hipStream_t s) {
    int st = init_device();
    if (st != XMOE_OK) return st;
    const int max_tiles = ffn_max_tiles(a.B, a.E, TM);
    st = launch_tile_map(a.off, a.E, TM, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const bf16_t *xd = (const bf16_t*)a.xd, *wg = (const bf16_t*)a.wg, *wu = (const bf16_t*)a.wu,
                 *wd = (const bf16_t*)a.wd, *dy = (const bf16_t*)a.dy;
    bf16_t *dg = (bf16_t*)a.dg, *du = (bf16_t*)a.du, *act = (bf16_t*)a.act;
    const int ntf = (a.f + TN - 1) / TN, ntd = (a.d + TN - 1) / TN;
    if (a.dy_index)
        XMOE_LAUNCH(K_FFN_DACT_DMA, s,
                    hipLaunchKernelGGL((ffn_rowgemm_dma_kernel<true, true>), dim3(round_up8((long)max_tiles * ntf)),
                                       dim3(512), kLdsBytes, s, dy, a.dy_index, a.dy_scale, a.off, a.map, a.d, a.f, wd,
                                       nullptr, (const bf16_t*)a.g, (const bf16_t*)a.u, dg, du, act,
                                       a.row_part, (long)a.B, row_counters(a.sched, a.E, 0), clock_slot(CS_DACT)));
    else
        XMOE_LAUNCH(K_FFN_DACT_DMA, s,
                    hipLaunchKernelGGL((ffn_rowgemm_dma_kernel<true, false>), dim3(round_up8((long)max_tiles * ntf)),
                                       dim3(512), kLdsBytes, s, dy, nullptr, nullptr, a.off, a.map, a.d, a.f, wd,
                                       nullptr, (const bf16_t*)a.g, (const bf16_t*)a.u, dg, du, act,
                                       a.row_part, (long)a.B, row_counters(a.sched, a.E, 0), clock_slot(CS_DACT)));
    if (a.row_grad) {
        st = launch_row_grad_reduce(a.row_part, 4 * ntf, a.B, a.row_grad, s);
        if (st != XMOE_OK) return st;
    }
    const int mtf = (a.f + TM - 1) / TM, mtd = (a.d + TM - 1) / TM;
    const int ntf2 = (a.f + 127) / 128;
    if (bwd_merged()) {
        // dXd, dWd, dWg | dWu: one launch
        const long tiles = (long)max_tiles * ntd + (long)a.E * mtf * ntd + (long)a.E * mtd * ntf2;
        const dim3 grid(round_up8(tiles));
#define XMOE_REST(G, DYG)                                                                                             \
    XMOE_LAUNCH(K_FFN_BWD_REST_DMA, s,                                                                                \
                hipLaunchKernelGGL((ffn_bwd_rest_dma_kernel<true, G, DYG>), grid, dim3(512), kLdsBytes, s, dg, du,    \
                                   act, dy, a.dy_index, a.dy_index, xd, a.row_index, a.row_index, a.off, a.map,       \
                                   a.sched, row_counters(a.sched, a.E, 1), a.sched + a.E, a.sched + a.E + kNumXcd,    \
                                   a.E, wgrad_one_xcd(a), a.d, a.f, wg, wu, (bf16_t*)a.dxd, (bf16_t*)a.dwd, (bf16_t*)a.dwg,             \
                                   (bf16_t*)a.dwu, clock_slot(CS_BWD_REST)))
        if (a.row_index && a.dy_index) XMOE_REST(true, true);
        else if (a.row_index) XMOE_REST(true, false);
        else if (a.dy_index) XMOE_REST(false, true);
        else XMOE_REST(false, false);
#undef XMOE_REST
        return XMOE_OK;
    }
    XMOE_LAUNCH(K_FFN_DX_DMA, s,
                hipLaunchKernelGGL(ffn_dx_dma_kernel<true>, dim3(round_up8((long)max_tiles * ntd)), dim3(512), kLdsBytes, s, dg,
                                   du, a.off, a.map, a.d, a.f, wg, wu, (bf16_t*)a.dxd, row_counters(a.sched, a.E, 1), clock_slot(CS_DX)));
    // dWd [f, d] = A^T dY
    if (a.dy_index)
        XMOE_LAUNCH(K_FFN_WGRAD_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<false, false, true>),
                                       dim3(round_up8((long)a.E * mtf * ntd)), dim3(512), kLdsBytes, s, act, nullptr, dy,
                                       nullptr, a.dy_index, nullptr, a.dy_index, a.off, a.sched, a.sched + a.E, a.E, wgrad_one_xcd(a), a.f,
                                       a.d,
                                       (bf16_t*)a.dwd, nullptr, clock_slot(CS_WGRAD)));
    else
        XMOE_LAUNCH(K_FFN_WGRAD_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<false, false>), dim3(round_up8((long)a.E * mtf * ntd)),
                                       dim3(512), kLdsBytes, s, act, nullptr, dy, nullptr, nullptr, nullptr, nullptr, a.off,
                                       a.sched,
                                       a.sched + a.E, a.E, wgrad_one_xcd(a), a.f, a.d, (bf16_t*)a.dwd, nullptr, clock_slot(CS_WGRAD)));
    // dWg, dWu [d, f] = Xd^T dG, Xd^T dU in one launch
    if (a.row_index)
        XMOE_LAUNCH(K_FFN_WGRAD_DUAL_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<true, true>), dim3(round_up8((long)a.E * mtd * ntf2)),
                                       dim3(512), kLdsBytes, s, xd, a.row_index, dg, du, nullptr, a.row_index, nullptr, a.off,
                                       a.sched,
                                       a.sched + a.E + kNumXcd, a.E, wgrad_one_xcd(a), a.d, a.f, (bf16_t*)a.dwg, (bf16_t*)a.dwu, clock_slot(CS_WGRAD_DUAL)));
    else
        XMOE_LAUNCH(K_FFN_WGRAD_DUAL_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<true, false>), dim3(round_up8((long)a.E * mtd * ntf2)),
                                       dim3(512), kLdsBytes, s, xd, nullptr, dg, du, nullptr, nullptr, nullptr, a.off, a.sched,
                                       a.sched + a.E + kNumXcd, a.E, wgrad_one_xcd(a), a.d, a.f, (bf16_t*)a.dwg, (bf16_t*)a.dwu, clock_slot(CS_WGRAD_DUAL)));
    return XMOE_OK;
}

bool mlp2_dma_supported(const Mlp2Args& a) {
    if (a.dt != XMOE_BF16) return false;
    if (a.d % 64 != 0 || a.f % 64 != 0) return false;
    const void* ptrs[] = {a.xd, a.w1, a.w2, a.h, a.y, a.dy, a.dxd, a.dw1, a.dw2, a.a_buf, a.dh};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return false;
    return true;
}

int mlp2_fwd_dma(const Mlp2Args& a, hipStream_t s) {
    int st = init_device();
    if (st != XMOE_OK) return st;
    const int max_tiles = ffn_max_tiles(a.B, a.E, TM);
    st = launch_tile_map(a.off, a.E, TM, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const bf16_t *xd = (const bf16_t*)a.xd, *w1 = (const bf16_t*)a.w1, *w2 = (const bf16_t*)a.w2;
    const int ntf = (a.f + TN - 1) / TN, ntd = (a.d + TN - 1) / TN;
    const dim3 grid(round_up8((long)max_tiles * ntf));
    if (a.row_index) {
#define XMOE_CALL(ACT)                                                                                               \
    XMOE_LAUNCH(K_MLP2_UP_DMA, s,                                                                                    \
                hipLaunchKernelGGL((mlp2_up_dma_kernel<true, ACT>), grid, dim3(512), kLdsBytes, s, xd, a.row_index,  \
                                   a.off, a.map, a.d, a.f, w1, (bf16_t*)a.h, (bf16_t*)a.a_buf,              \
                                   row_counters(a.sched, a.E, 0), clock_slot(CS_MLP2_UP)))
        XMOE_DISPATCH_ACT(a.act, XMOE_CALL);
#undef XMOE_CALL
    } else {
#define XMOE_CALL(ACT)                                                                                               \
    XMOE_LAUNCH(K_MLP2_UP_DMA, s,                                                                                    \
                hipLaunchKernelGGL((mlp2_up_dma_kernel<false, ACT>), grid, dim3(512), kLdsBytes, s, xd, nullptr,     \
                                   a.off, a.map, a.d, a.f, w1, (bf16_t*)a.h, (bf16_t*)a.a_buf,              \
                                   row_counters(a.sched, a.E, 0), clock_slot(CS_MLP2_UP)))
        XMOE_DISPATCH_ACT(a.act, XMOE_CALL);
#undef XMOE_CALL
    }
    XMOE_LAUNCH(K_FFN_DOWN_DMA, s,
                hipLaunchKernelGGL((ffn_rowgemm_dma_kernel<false, false>), dim3(round_up8((long)max_tiles * ntd)), dim3(512),
                                   kLdsBytes, s, (const bf16_t*)a.a_buf, nullptr, nullptr, a.off, a.map, a.f, a.d, w2,
                                   (bf16_t*)a.y,
                                   nullptr, nullptr, nullptr, nullptr, nullptr, (float*)nullptr, 0L, row_counters(a.sched, a.E, 1), clock_slot(CS_DOWN)));
    return XMOE_OK;
}

int mlp2_bwd_dma(const Mlp2Args& a, hipStream_t s) {
    int st = init_device();
    if (st != XMOE_OK) return st;
    const int max_tiles = ffn_max_tiles(a.B, a.E, TM);
    st = launch_tile_map(a.off, a.E, TM, max_tiles, a.map, a.sched, s);
    if (st != XMOE_OK) return st;
    const bf16_t *xd = (const bf16_t*)a.xd, *w1 = (const bf16_t*)a.w1, *w2 = (const bf16_t*)a.w2,
                 *dy = (const bf16_t*)a.dy;
    bf16_t *dh = (bf16_t*)a.dh, *act = (bf16_t*)a.a_buf;
    const int ntf = (a.f + TN - 1) / TN, ntd = (a.d + TN - 1) / TN;
    const dim3 grid(round_up8((long)max_tiles * ntf));
    if (a.dy_index) {
#define XMOE_CALL(ACT)                                                                                              \
    XMOE_LAUNCH(K_MLP2_DACT_DMA, s,                                                                                 \
                hipLaunchKernelGGL((mlp2_dact_dma_kernel<ACT, true>), grid, dim3(512), kLdsBytes, s, dy, a.dy_index, \
                                   a.dy_scale, a.off, a.map, a.d, a.f, w2, (const bf16_t*)a.h, dh, act,            \
                                   a.row_part, (long)a.B, row_counters(a.sched, a.E, 0), clock_slot(CS_MLP2_DACT)))
        XMOE_DISPATCH_ACT(a.act, XMOE_CALL);
#undef XMOE_CALL
    } else {
#define XMOE_CALL(ACT)                                                                                              \
    XMOE_LAUNCH(K_MLP2_DACT_DMA, s,                                                                                 \
                hipLaunchKernelGGL((mlp2_dact_dma_kernel<ACT, false>), grid, dim3(512), kLdsBytes, s, dy, nullptr,  \
                                   nullptr, a.off, a.map, a.d, a.f, w2, (const bf16_t*)a.h, dh, act,               \
                                   a.row_part, (long)a.B, row_counters(a.sched, a.E, 0), clock_slot(CS_MLP2_DACT)))
        XMOE_DISPATCH_ACT(a.act, XMOE_CALL);
#undef XMOE_CALL
    }
    if (a.row_grad) {
        st = launch_row_grad_reduce(a.row_part, 4 * ntf, a.B, a.row_grad, s);
        if (st != XMOE_OK) return st;
    }
    const int mtf = (a.f + TM - 1) / TM, mtd = (a.d + TM - 1) / TM;
    if (bwd_merged()) {
        // dXd, dW2, dW1: one launch
        const long tiles = (long)max_tiles * ntd + (long)a.E * mtf * ntd + (long)a.E * mtd * ntf;
        const dim3 grid_rest(round_up8(tiles));
#define XMOE_REST(G, DYG)                                                                                             \
    XMOE_LAUNCH(K_FFN_BWD_REST_DMA, s,                                                                                \
                hipLaunchKernelGGL((ffn_bwd_rest_dma_kernel<false, G, DYG>), grid_rest, dim3(512), kLdsBytes, s, dh,  \
                                   nullptr, act, dy, a.dy_index, a.dy_index, xd, a.row_index, a.row_index, a.off,     \
                                   a.map, a.sched, row_counters(a.sched, a.E, 1), a.sched + a.E,                      \
                                   a.sched + a.E + kNumXcd, a.E, wgrad_one_xcd(a), a.d, a.f, w1, nullptr,             \
                                   (bf16_t*)a.dxd,                                                                    \
                                   (bf16_t*)a.dw2, (bf16_t*)a.dw1, nullptr, clock_slot(CS_BWD_REST)))
        if (a.row_index && a.dy_index) XMOE_REST(true, true);
        else if (a.row_index) XMOE_REST(true, false);
        else if (a.dy_index) XMOE_REST(false, true);
        else XMOE_REST(false, false);
#undef XMOE_REST
        return XMOE_OK;
    }
    XMOE_LAUNCH(K_FFN_DX_DMA, s,
                hipLaunchKernelGGL(ffn_dx_dma_kernel<false>, dim3(round_up8((long)max_tiles * ntd)), dim3(512),
                                   kLdsBytes, s, dh, nullptr, a.off, a.map, a.d, a.f, w1, nullptr, (bf16_t*)a.dxd,
                                   row_counters(a.sched, a.E, 1), clock_slot(CS_DX)));
    // dW2 [f, d] = A^T dY
    if (a.dy_index)
        XMOE_LAUNCH(K_FFN_WGRAD_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<false, false, true>),
                                       dim3(round_up8((long)a.E * mtf * ntd)), dim3(512), kLdsBytes, s, act, nullptr, dy,
                                       nullptr, a.dy_index, nullptr, a.dy_index, a.off, a.sched, a.sched + a.E, a.E, wgrad_one_xcd(a), a.f,
                                       a.d,
                                       (bf16_t*)a.dw2, nullptr, clock_slot(CS_WGRAD)));
    else
        XMOE_LAUNCH(K_FFN_WGRAD_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<false, false>), dim3(round_up8((long)a.E * mtf * ntd)),
                                       dim3(512), kLdsBytes, s, act, nullptr, dy, nullptr, nullptr, nullptr, nullptr, a.off,
                                       a.sched,
                                       a.sched + a.E, a.E, wgrad_one_xcd(a), a.f, a.d, (bf16_t*)a.dw2, nullptr, clock_slot(CS_WGRAD)));
    // dW1 [d, f] = Xd^T dH
    if (a.row_index)
        XMOE_LAUNCH(K_FFN_WGRAD_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<false, true>), dim3(round_up8((long)a.E * mtd * ntf)),
                                       dim3(512), kLdsBytes, s, xd, a.row_index, dh, nullptr, nullptr, a.row_index, nullptr,
                                       a.off, a.sched,
                                       a.sched + a.E + kNumXcd, a.E, wgrad_one_xcd(a), a.d, a.f, (bf16_t*)a.dw1, nullptr, clock_slot(CS_WGRAD)));
    else
        XMOE_LAUNCH(K_FFN_WGRAD_DMA, s,
                    hipLaunchKernelGGL((ffn_wgrad_dma_kernel<false, false>), dim3(round_up8((long)a.E * mtd * ntf)),
                                       dim3(512), kLdsBytes, s, xd, nullptr, dh, nullptr, nullptr, nullptr, nullptr, a.off,
                                       a.sched,
                                       a.sched + a.E + kNumXcd, a.E, wgrad_one_xcd(a), a.d, a.f, (bf16_t*)a.dw1, nullptr, clock_slot(CS_WGRAD)));
    return XMOE_OK;
}

}  // namespace xmoe

extern "C" int xmoe_prof_shader_clock(int kernel_id, double* ghz) {
    int slot = -1;
    switch (kernel_id) {
        case xmoe::K_FFN_GATEUP_DMA: slot = xmoe::CS_GATEUP; break;
        case xmoe::K_FFN_DOWN_DMA: slot = xmoe::CS_DOWN; break;
        case xmoe::K_FFN_DACT_DMA: slot = xmoe::CS_DACT; break;
        case xmoe::K_FFN_DX_DMA: slot = xmoe::CS_DX; break;
        case xmoe::K_FFN_WGRAD_DMA: slot = xmoe::CS_WGRAD; break;
        case xmoe::K_FFN_WGRAD_DUAL_DMA: slot = xmoe::CS_WGRAD_DUAL; break;
        case xmoe::K_FFN_BWD_REST_DMA: slot = xmoe::CS_BWD_REST; break;
        case xmoe::K_MLP2_UP_DMA: slot = xmoe::CS_MLP2_UP; break;
        case xmoe::K_MLP2_DACT_DMA: slot = xmoe::CS_MLP2_DACT; break;
        default: break;
    }
    if (!ghz) return XMOE_ERR_INVALID_ARG;
    *ghz = 0.0;
    if (slot < 0) return XMOE_OK;
    unsigned long long v[4];
    if (xmoe::init_device() != XMOE_OK || !xmoe::t_dev->clock_probe) return XMOE_ERR_HIP;
    if (hipMemcpy(v, xmoe::t_dev->clock_probe + 4 * slot, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess)
        return XMOE_ERR_HIP;
    if (v[3] > v[1] && v[2] > v[0]) *ghz = (double)(v[2] - v[0]) / ((double)(v[3] - v[1]) * 10.0);   // 100 MHz ticks
    return XMOE_OK;
}
