// Status strings, workspace sizing and the optional event profiler of libxmoe.
#include <vector>

#include "xmoe_internal.h"
#include "xmoe_sizes.h"

namespace xmoe {

namespace {
struct Sample {
    int kid;
    hipEvent_t start, stop;
};
struct Prof {
    bool on = false;
    std::vector<Sample> samples;
    std::vector<hipEvent_t> free_events;
    hipEvent_t pending_start = nullptr;
};
Prof g_prof;

const char* const kKernelNames[K_COUNT] = {
    "gate_logits_kernel",
    "route_kernel",
    "eri_hist_kernel",
    "eri_scan_kernel",
    "eri_scatter_kernel",
    "eri_cap_kernel",
    "shared_segments_kernel",
    "dispatch_kernel",
    "combine_kernel",
    "combine_bwd_kernel",
    "route_bwd_kernel",
    "gate_bwd_dw_kernel",
    "gate_bwd_dw_reduce_kernel",
    "gate_bwd_dx_kernel",
    "tile_map_kernel",
    "row_grad_reduce_kernel",
    "combine_bwd_weights_kernel",
    "ffn_gateup_simt_kernel",
    "ffn_down_simt_kernel",
    "ffn_dact_simt_kernel",
    "ffn_dx_simt_kernel",
    "ffn_wgrad_simt_kernel",
    "ffn_gateup_dma_kernel",
    "ffn_rowgemm_dma_kernel<false>",
    "ffn_rowgemm_dma_kernel<true>",
    "ffn_dx_dma_kernel",
    "ffn_wgrad_dma_kernel<false>",
    "ffn_wgrad_dma_kernel<true>",
    "ffn_bwd_rest_dma_kernel",
    "mlp2_up_simt_kernel",
    "mlp2_dact_simt_kernel",
    "mlp2_up_dma_kernel",
    "mlp2_dact_dma_kernel",
    "rbd_mark_kernel",
    "rbd_count_kernel",
    "rbd_scan_kernel",
    "rbd_scatter_kernel",
    "rbd_map_kernel",
    "rbd_absolute_kernel",
    "prof_copy_kernel",
};

hipEvent_t get_event() {
    if (!g_prof.free_events.empty()) {
        hipEvent_t e = g_prof.free_events.back();
        g_prof.free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

// A copy whose traffic is known exactly (bytes read + bytes written): the yardstick for hardware byte counters, and
// what a streaming kernel reaches on this GPU.  Every thread keeps four independent 16-byte loads in flight (lanes of
// a wave on consecutive 16-byte pieces, the four loads 4 KiB apart) and writes with streaming stores.
typedef __attribute__((ext_vector_type(4))) unsigned int prof_u32x4_t;
__global__ __launch_bounds__(256) void prof_copy_kernel(const prof_u32x4_t* __restrict__ src,
                                                        prof_u32x4_t* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 1024;
    for (size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x; base < n16; base += stride) {
        prof_u32x4_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (base + 256 * j < n16) v[j] = __builtin_nontemporal_load(src + base + 256 * j);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (base + 256 * j < n16) __builtin_nontemporal_store(v[j], dst + base + 256 * j);
    }
}

bool prof_enabled() { return g_prof.on; }

void prof_begin(int kid, hipStream_t s) {
    (void)kid;
    if (!g_prof.on) return;
    hipEvent_t e = get_event();
    g_prof.pending_start = e;
    if (e) (void)hipEventRecord(e, s);
}

void prof_end(int kid, hipStream_t s) {
    if (!g_prof.on) return;
    hipEvent_t st = g_prof.pending_start;
    g_prof.pending_start = nullptr;
    hipEvent_t e = get_event();
    if (!st || !e) return;
    (void)hipEventRecord(e, s);
    g_prof.samples.push_back(Sample{kid, st, e});
}

}  // namespace xmoe

using namespace xmoe;

extern "C" {

const char* xmoe_status_string(int status) {
    switch (status) {
        case XMOE_OK: return "XMOE_OK";
        case XMOE_ERR_INVALID_ARG: return "XMOE_ERR_INVALID_ARG: null pointer or size out of range";
        case XMOE_ERR_UNSUPPORTED: return "XMOE_ERR_UNSUPPORTED: dtype or size not supported";
        case XMOE_ERR_WORKSPACE: return "XMOE_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case XMOE_ERR_HIP: return "XMOE_ERR_HIP: HIP runtime error at kernel launch";
        default: return "unknown xmoe status";
    }
}

const char* xmoe_version(void) { return "xmoe 0.1 (gfx950)"; }

size_t xmoe_workspace_bytes(int op, int rows, int d, int E, int k, int f, int dt) {
    if (rows < 0 || d < 0 || E < 0 || k < 0 || f < 0 || !dtype_ok(dt)) return 0;
    switch (op) {
        case XMOE_WS_BUILD_ERI: return eri_ws_bytes(rows, E, k);
        case XMOE_WS_FFN_FWD: return ffn_fwd_ws_bytes(rows, E, d, f, dt);
        case XMOE_WS_FFN_BWD: return ffn_bwd_ws_bytes(rows, E, d, f, dt);
        case XMOE_WS_GATE_BWD: return gate_bwd_ws_bytes(rows, d, E);
        case XMOE_WS_BUILD_ERI_CAPPED: return eri_capped_ws_bytes(rows, E, k);
        case XMOE_WS_MLP2_FWD: return mlp2_fwd_ws_bytes(rows, E, d, f, dt);
        case XMOE_WS_MLP2_BWD: return mlp2_bwd_ws_bytes(rows, E, d, f, dt);
        case XMOE_WS_RBD_STAGE0: return rbd_ws_bytes(rows, k);
        default: return 0;
    }
}

void xmoe_prof_enable(int on) { g_prof.on = (on != 0); }

void xmoe_prof_reset(void) {
    for (auto& s : g_prof.samples) {
        g_prof.free_events.push_back(s.start);
        g_prof.free_events.push_back(s.stop);
    }
    g_prof.samples.clear();
}

int xmoe_prof_num_kernels(void) { return K_COUNT; }

const char* xmoe_prof_kernel_name(int kernel_id) {
    if (kernel_id < 0 || kernel_id >= K_COUNT) return "";
    return kKernelNames[kernel_id];
}

int xmoe_prof_get(int kernel_id, int* launches, double* total_ms) {
    if (kernel_id < 0 || kernel_id >= K_COUNT || !launches || !total_ms) return XMOE_ERR_INVALID_ARG;
    int n = 0;
    double ms = 0.0;
    for (auto& s : g_prof.samples) {
        if (s.kid != kernel_id) continue;
        if (hipEventSynchronize(s.stop) != hipSuccess) return XMOE_ERR_HIP;
        float t = 0.f;
        if (hipEventElapsedTime(&t, s.start, s.stop) != hipSuccess) return XMOE_ERR_HIP;
        ms += t;
        ++n;
    }
    *launches = n;
    *total_ms = ms;
    return XMOE_OK;
}

int xmoe_prof_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (bytes == 0) return XMOE_OK;
    if (!src || !dst || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15u) ||
        (reinterpret_cast<uintptr_t>(dst) & 15u))
        return XMOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 1023) / 1024;
    const unsigned grid = (unsigned)(want < 4096 ? want : 4096);
    XMOE_LAUNCH(K_PROF_COPY, s, hipLaunchKernelGGL(prof_copy_kernel, dim3(grid), dim3(256), 0, s,
                                                   (const prof_u32x4_t*)src, (prof_u32x4_t*)dst, n16));
    return XMOE_OK;
}

}  // extern "C"
