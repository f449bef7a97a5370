// Internal helpers shared by the HIP sources of libxmoe (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xmoe.h"

namespace xmoe {

// ---------------------------------------------------------------------------------------------------------
// kernel ids for the optional event profiler (names returned by xmoe_prof_kernel_name)
// ---------------------------------------------------------------------------------------------------------
enum KernelId : int {
    K_GATE_LOGITS = 0,
    K_ROUTE,
    K_ERI_HIST,
    K_ERI_SCAN,
    K_ERI_SCATTER,
    K_ERI_CAP,
    K_SHARED_SEGMENTS,
    K_DISPATCH,
    K_COMBINE,
    K_COMBINE_BWD,
    K_ROUTE_BWD,
    K_GATE_BWD_DW,
    K_GATE_BWD_DW_REDUCE,
    K_GATE_BWD_DX,
    K_TILE_MAP,
    K_ROW_GRAD_REDUCE,
    K_COMBINE_BWD_W,
    K_FFN_GATEUP_SIMT,
    K_FFN_DOWN_SIMT,
    K_FFN_DACT_SIMT,
    K_FFN_DX_SIMT,
    K_FFN_WGRAD_SIMT,
    K_FFN_GATEUP_DMA,
    K_FFN_DOWN_DMA,
    K_FFN_DACT_DMA,
    K_FFN_DX_DMA,
    K_FFN_WGRAD_DMA,
    K_FFN_WGRAD_DUAL_DMA,
    K_FFN_BWD_REST_DMA,
    K_MLP2_UP_SIMT,
    K_MLP2_DACT_SIMT,
    K_MLP2_UP_DMA,
    K_MLP2_DACT_DMA,
    K_RBD_MARK,
    K_RBD_COUNT,
    K_RBD_SCAN,
    K_RBD_SCATTER,
    K_RBD_MAP,
    K_RBD_ABS,
    K_PROF_COPY,
    K_COUNT
};

bool prof_enabled();   // the launch profiler of xmoe_prof_enable
void prof_begin(int kid, hipStream_t s);
void prof_end(int kid, hipStream_t s);

// Brackets one kernel launch with the profiler hooks and turns a launch error into XMOE_ERR_HIP.
#define XMOE_LAUNCH(kid, stream, ...)                              \
    do {                                                           \
        ::xmoe::prof_begin((kid), (stream));                       \
        __VA_ARGS__;                                               \
        ::xmoe::prof_end((kid), (stream));                         \
        if (hipGetLastError() != hipSuccess) return XMOE_ERR_HIP;  \
    } while (0)

// ---------------------------------------------------------------------------------------------------------
// element types: float32 and bfloat16 (stored as raw 16-bit patterns)
// ---------------------------------------------------------------------------------------------------------
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even float32 -> bfloat16 (NaN stays a NaN): the conversion instruction of gfx950
// (v_cvt_pk_bf16_f32), one instruction per two values
typedef __attribute__((ext_vector_type(2))) float xmoe_f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 xmoe_bf16x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const xmoe_f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, xmoe_bf16x2_t));
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float v) {
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return bf16_bits_to_float(v.bits); }

template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return bf16_t{float_to_bf16_bits(v)}; }

static inline size_t dtype_size(int dt) { return dt == XMOE_F32 ? 4 : 2; }
static inline bool dtype_ok(int dt) { return dt == XMOE_F32 || dt == XMOE_BF16; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr int kWave = 64;

// silu(g) = g * sigmoid(g) and its derivative, in float32
__device__ __forceinline__ float sigmoidf_(float g) { return 1.0f / (1.0f + expf(-g)); }
__device__ __forceinline__ float siluf_(float g) { return g * sigmoidf_(g); }

// activation of the two-matrix expert and its derivative, in float32 (ACT is an xmoe_act)
template <int ACT>
__device__ __forceinline__ float act_fwd(float h) {
    if (ACT == XMOE_ACT_GELU) return 0.5f * h * (1.0f + erff(h * 0.70710678118654752f));
    if (ACT == XMOE_ACT_SILU) return siluf_(h);
    return h;
}
// a = act(h), g = act'(h)
template <int ACT>
__device__ __forceinline__ void act_fwd_grad(float h, float& a, float& g) {
    if (ACT == XMOE_ACT_GELU) {
        const float Phi = 0.5f * (1.0f + erff(h * 0.70710678118654752f));
        a = h * Phi;
        g = Phi + h * (0.39894228040143268f * expf(-0.5f * h * h));
    } else if (ACT == XMOE_ACT_SILU) {
        const float sg = sigmoidf_(h);
        a = h * sg;
        g = sg * (1.0f + h * (1.0f - sg));
    } else {
        a = h;
        g = 1.0f;
    }
}
static inline bool act_ok(int act) { return act == XMOE_ACT_IDENTITY || act == XMOE_ACT_GELU || act == XMOE_ACT_SILU; }

// runs CALL(ACT) with the run-time activation code as a compile-time constant
#define XMOE_DISPATCH_ACT(act, CALL)                              \
    do {                                                           \
        if ((act) == XMOE_ACT_GELU) { CALL(XMOE_ACT_GELU); }       \
        else if ((act) == XMOE_ACT_SILU) { CALL(XMOE_ACT_SILU); }  \
        else { CALL(XMOE_ACT_IDENTITY); }                          \
    } while (0)

}  // namespace xmoe
