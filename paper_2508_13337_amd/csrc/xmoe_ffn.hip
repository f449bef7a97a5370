// Entry points of the expert MLP (paper: Listing 1 mlp(); Appendix B.4): argument checks, workspace carve-up,
// and the choice between the bf16 MFMA kernels (bf16 storage, d and f multiples of 64, 16-byte aligned operands)
// and the float32-ALU kernels (everything else).

#include "xmoe_ffn.h"

namespace xmoe {

static int check_common(int B, int E, int d, int f, int dt) {
    if (!dtype_ok(dt)) return XMOE_ERR_UNSUPPORTED;
    if (B < 0 || E < 1 || d < 1 || f < 1) return XMOE_ERR_INVALID_ARG;
    if (E > XMOE_MAX_EXPERTS) return XMOE_ERR_UNSUPPORTED;
    if ((long long)B * d >= (1ll << 40) || (long long)B * f >= (1ll << 40)) return XMOE_ERR_INVALID_ARG;
    return XMOE_OK;
}

}  // namespace xmoe

using namespace xmoe;

extern "C" {

int xmoe_expert_ffn_fwd(const void* xd, const int32_t* row_index, const int32_t* expert_offsets, int B, int E, int d,
                        int f, const void* wg,
                        const void* wu, const void* wd, void* g_save, void* u_save, void* y, int dt, void* ws,
                        size_t ws_bytes, void* stream) {
    int st = check_common(B, E, d, f, dt);
    if (st != XMOE_OK) return st;
    if (!expert_offsets || !wg || !wu || !wd) return XMOE_ERR_INVALID_ARG;
    if (B == 0) return XMOE_OK;
    if (!xd || !g_save || !u_save || !y) return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < ffn_fwd_ws_bytes(B, E, d, f, dt))
        return XMOE_ERR_WORKSPACE;
    FfnArgs a{};
    a.B = B; a.E = E; a.d = d; a.f = f; a.dt = dt;
    a.off = expert_offsets;
    a.xd = xd; a.wg = wg; a.wu = wu; a.wd = wd;
    a.row_index = row_index;
    a.g = g_save; a.u = u_save; a.y = y;
    char* p = (char*)ws;
    a.map = (int32_t*)p;
    a.sched = a.map + ffn_sched_offset(B, E);
    p += ffn_tilemap_bytes(B, E);
    a.act = p;
    hipStream_t s = (hipStream_t)stream;
    if (ffn_dma_supported(a)) return ffn_fwd_dma(a, s);
    return ffn_fwd_simt(a, s);
}

int xmoe_expert_ffn_bwd(const void* xd, const int32_t* row_index, const void* g_save, const void* u_save,
                        const void* dy, const int32_t* dy_row_index, const float* dy_row_scale,
                        float* dy_row_scale_grad,
                        const int32_t* expert_offsets, int B, int E, int d, int f, const void* wg, const void* wu,
                        const void* wd, void* dxd, void* dwg, void* dwu, void* dwd, int dt, void* ws,
                        size_t ws_bytes, void* stream) {
    int st = check_common(B, E, d, f, dt);
    if (st != XMOE_OK) return st;
    if (!expert_offsets || !wg || !wu || !wd || !dwg || !dwu || !dwd) return XMOE_ERR_INVALID_ARG;
    if (dy_row_scale && !dy_row_index) return XMOE_ERR_INVALID_ARG;
    if (B > 0 && (!xd || !g_save || !u_save || !dy || !dxd)) return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < ffn_bwd_ws_bytes(B, E, d, f, dt))
        return XMOE_ERR_WORKSPACE;
    FfnArgs a{};
    a.B = B; a.E = E; a.d = d; a.f = f; a.dt = dt;
    a.off = expert_offsets;
    a.xd = xd; a.wg = wg; a.wu = wu; a.wd = wd;
    a.row_index = row_index;
    a.g = const_cast<void*>(g_save); a.u = const_cast<void*>(u_save);
    a.dy = dy;
    a.dy_index = dy_row_index; a.dy_scale = dy_row_scale;
    a.dxd = dxd; a.dwg = dwg; a.dwu = dwu; a.dwd = dwd;
    char* p = (char*)ws;
    a.map = (int32_t*)p;
    a.sched = a.map + ffn_sched_offset(B, E);
    p += ffn_tilemap_bytes(B, E);
    a.dg = p;
    p += ffn_act_bytes(B, f, dt);
    a.du = p;
    p += ffn_act_bytes(B, f, dt);
    a.act = p;
    p += ffn_act_bytes(B, f, dt);
    a.row_grad = dy_row_scale_grad;
    a.row_part = (float*)p;   // the partial sums are always written (the matrix-core kernel has no branch for them)
    hipStream_t s = (hipStream_t)stream;
    if (ffn_dma_supported(a)) return ffn_bwd_dma(a, s);
    return ffn_bwd_simt(a, s);
}

int xmoe_expert_mlp2_fwd(const void* xd, const int32_t* row_index, const int32_t* expert_offsets, int B, int E,
                         int d, int f, const void* w1, const void* w2, int act, void* h_save, void* y, int dt,
                         void* ws, size_t ws_bytes, void* stream) {
    int st = check_common(B, E, d, f, dt);
    if (st != XMOE_OK) return st;
    if (!act_ok(act)) return XMOE_ERR_UNSUPPORTED;
    if (!expert_offsets || !w1 || !w2) return XMOE_ERR_INVALID_ARG;
    if (B == 0) return XMOE_OK;
    if (!xd || !h_save || !y) return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < mlp2_fwd_ws_bytes(B, E, d, f, dt))
        return XMOE_ERR_WORKSPACE;
    Mlp2Args a{};
    a.B = B; a.E = E; a.d = d; a.f = f; a.dt = dt; a.act = act;
    a.off = expert_offsets;
    a.xd = xd; a.w1 = w1; a.w2 = w2;
    a.row_index = row_index;
    a.h = h_save; a.y = y;
    char* p = (char*)ws;
    a.map = (int32_t*)p;
    a.sched = a.map + ffn_sched_offset(B, E);
    p += ffn_tilemap_bytes(B, E);
    a.a_buf = p;
    hipStream_t s = (hipStream_t)stream;
    if (mlp2_dma_supported(a)) return mlp2_fwd_dma(a, s);
    return mlp2_fwd_simt(a, s);
}

int xmoe_expert_mlp2_bwd(const void* xd, const int32_t* row_index, const void* h_save, const void* dy,
                         const int32_t* dy_row_index, const float* dy_row_scale, float* dy_row_scale_grad,
                         const int32_t* expert_offsets, int B, int E, int d, int f, const void* w1, const void* w2,
                         int act, void* dxd, void* dw1, void* dw2, int dt, void* ws, size_t ws_bytes, void* stream) {
    int st = check_common(B, E, d, f, dt);
    if (st != XMOE_OK) return st;
    if (!act_ok(act)) return XMOE_ERR_UNSUPPORTED;
    if (dy_row_scale && !dy_row_index) return XMOE_ERR_INVALID_ARG;
    if (!expert_offsets || !w1 || !w2 || !dw1 || !dw2) return XMOE_ERR_INVALID_ARG;
    if (B > 0 && (!xd || !h_save || !dy || !dxd)) return XMOE_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < mlp2_bwd_ws_bytes(B, E, d, f, dt))
        return XMOE_ERR_WORKSPACE;
    Mlp2Args a{};
    a.B = B; a.E = E; a.d = d; a.f = f; a.dt = dt; a.act = act;
    a.off = expert_offsets;
    a.xd = xd; a.w1 = w1; a.w2 = w2;
    a.row_index = row_index;
    a.h = const_cast<void*>(h_save);
    a.dy = dy;
    a.dy_index = dy_row_index; a.dy_scale = dy_row_scale;
    a.dxd = dxd; a.dw1 = dw1; a.dw2 = dw2;
    char* p = (char*)ws;
    a.map = (int32_t*)p;
    a.sched = a.map + ffn_sched_offset(B, E);
    p += ffn_tilemap_bytes(B, E);
    a.dh = p;
    p += ffn_act_bytes(B, f, dt);
    a.a_buf = p;
    p += ffn_act_bytes(B, f, dt);
    a.row_grad = dy_row_scale_grad;
    a.row_part = (float*)p;   // always written, as for the SwiGLU expert
    hipStream_t s = (hipStream_t)stream;
    if (mlp2_dma_supported(a)) return mlp2_bwd_dma(a, s);
    return mlp2_bwd_simt(a, s);
}

}  // extern "C"
