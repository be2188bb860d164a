// C ABI of the grouter library (see include/grouter.h): argument checks, workspace carving, launch order.
#include "../../include/grouter.h"

#include <mutex>
#include <vector>

#include "common.hpp"

using namespace grouter;

namespace {

thread_local int g_last_hip = 0;

struct TimedLaunch {
    int phase;
    hipEvent_t start, stop;
    bool owns_start;  // false when `start` is the previous entry's `stop` (phases chained inside one call)
};
// Timing state is shared by all host threads; g_timing_mu guards every access to it.
std::mutex g_timing_mu;
bool g_timing = false;
std::vector<TimedLaunch> g_pending;
std::vector<hipEvent_t> g_pool;
double g_ms[GROUTER_PH_COUNT];
int64_t g_launches[GROUTER_PH_COUNT];
constexpr size_t kMaxPending = 4096;

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Brackets one phase's launches with events when timing is on.  A phase that directly follows another one
// inside the same call passes that timer as `after`: the event that closed it also opens this one, so a
// chain of n phases costs n + 1 event records instead of 2 n.
struct PhaseTimer {
    TimedLaunch t{};
    hipStream_t s;
    bool on = false;
    bool closed = false;
    PhaseTimer(int phase, hipStream_t stream, PhaseTimer* after = nullptr) : s(stream) {
        // the phase before this one ends here whether or not this one is timed
        const bool chained = after && after->close();
        std::lock_guard<std::mutex> lock(g_timing_mu);
        if (!g_timing || g_pending.size() >= kMaxPending) return;
        // Events recorded while a stream is being captured become graph nodes and can never be read back.
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return;
        t.phase = phase;
        if (chained) {
            t.start = after->t.stop;
            t.owns_start = false;
            t.stop = take_event();
            on = t.stop != nullptr;
            return;
        }
        t.start = take_event();
        t.stop = take_event();
        t.owns_start = true;
        if (!t.start || !t.stop) {
            if (t.start) g_pool.push_back(t.start);
            if (t.stop) g_pool.push_back(t.stop);
            return;
        }
        on = hipEventRecord(t.start, s) == hipSuccess;
    }
    // records the closing event; true when the phase was timed and the event is usable as the next start
    bool close() {
        if (!on || closed) return on && closed;
        closed = true;
        if (hipEventRecord(t.stop, s) != hipSuccess) {
            on = false;
            return false;
        }
        std::lock_guard<std::mutex> lock(g_timing_mu);
        g_pending.push_back(t);
        return true;
    }
    ~PhaseTimer() { close(); }
};

int fail_hip(hipError_t e) {
    g_last_hip = (int)e;
    return GROUTER_ERR_HIP;
}

bool dims_ok(int64_t T, int k, int E) {
    if (T <= 0 || k <= 0 || E <= 0 || k > E || E > kMaxExperts) return false;
    if (T > (int64_t)0x7fffffff / k) return false;  // N = T*k must fit int32
    return true;
}

bool widths_ok(int64_t T, int k, int E, int d, int f) {
    if (!dims_ok(T, k, E) || d <= 0 || f <= 0 || (d % 8) || (f % 8)) return false;
    // The GEMM kernels address their operands through buffer descriptors with 32-bit byte offsets whose top
    // bit marks a masked lane: one expert's weight slab, and one expert's run of activation rows (at worst
    // all N = T*k rows), must each stay below 2^31 bytes.
    const uint64_t N = (uint64_t)T * (uint64_t)k;
    const uint64_t lim = 1ull << 31;
    if (N * (uint64_t)d * 2 >= lim || N * (uint64_t)f * 2 >= lim) return false;
    if ((uint64_t)d * (uint64_t)f * 2 >= lim) return false;
    return true;
}

struct CtxLayout {
    size_t ds_dg, ds_du, h, o, row_gate, total;   // ds_dg, ds_du: derivatives of silu(G) * U by G and by U
};
CtxLayout ctx_layout(int64_t T, int k, int d, int f) {
    const size_t N = (size_t)T * k;
    CtxLayout c{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    c.ds_dg = take(N * f * 2);
    c.ds_du = take(N * f * 2);
    c.h = take(N * f * 2);
    c.o = take(N * d * 2);
    c.row_gate = take(N * 4);
    c.total = o;
    return c;
}
struct FwdOnlyLayout {
    size_t h, o, row_gate, total;
};
FwdOnlyLayout fwd_only_layout(int64_t T, int k, int d, int f) {
    const size_t N = (size_t)T * k;
    FwdOnlyLayout c{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    c.h = take(N * f * 2);
    c.o = take(N * d * 2);
    c.row_gate = take(N * 4);
    c.total = o;
    return c;
}
struct BwdLayout {
    size_t dg, du, dxp, total;
};
BwdLayout bwd_layout(int64_t T, int k, int d, int f) {
    const size_t N = (size_t)T * k;
    BwdLayout c{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    c.dg = take(N * f * 2);
    c.du = take(N * f * 2);
    c.dxp = take(N * d * 2);
    c.total = o;
    return c;
}

bool aligned256(const void* p) { return ((uintptr_t)p & 255u) == 0; }
bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

extern "C" {

const char* grouter_strerror(int code) {
    switch (code) {
        case GROUTER_OK: return "ok";
        case GROUTER_ERR_INVALID_ARG: return "invalid argument";
        case GROUTER_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case GROUTER_ERR_INDEX_OUT_OF_RANGE: return "expert index out of range";
        case GROUTER_ERR_HIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

int grouter_last_hip_error(void) { return g_last_hip; }

size_t grouter_plan_bytes(int64_t T, int k, int E) {
    if (!dims_ok(T, k, E)) return 0;
    return make_plan_layout(T, k, E).total;
}

size_t grouter_ctx_bytes(int64_t T, int k, int d, int f) {
    if (!widths_ok(T, k, k, d, f)) return 0;
    return ctx_layout(T, k, d, f).total;
}

size_t grouter_fwd_only_bytes(int64_t T, int k, int d, int f) {
    if (!widths_ok(T, k, k, d, f)) return 0;
    return fwd_only_layout(T, k, d, f).total;
}

size_t grouter_bwd_scratch_bytes(int64_t T, int k, int d, int f) {
    if (!widths_ok(T, k, k, d, f)) return 0;
    return bwd_layout(T, k, d, f).total;
}

int grouter_plan_build(const void* topk_idx, int idx_dtype, int64_t T, int k, int E, void* plan_ws,
                       size_t plan_ws_bytes, void* stream) {
    if (!topk_idx || !plan_ws || !dims_ok(T, k, E)) return GROUTER_ERR_INVALID_ARG;
    if (idx_dtype != GROUTER_IDX_INT32 && idx_dtype != GROUTER_IDX_UINT8) return GROUTER_ERR_INVALID_ARG;
    if (idx_dtype == GROUTER_IDX_UINT8 && E > 256) return GROUTER_ERR_INVALID_ARG;
    if (!aligned256(plan_ws)) return GROUTER_ERR_INVALID_ARG;
    const PlanLayout L = make_plan_layout(T, k, E);
    if (plan_ws_bytes < L.total) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_PLAN, s);
    const hipError_t e = launch_plan_build(topk_idx, idx_dtype, L, plan_ws, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_plan_set_gates(void* plan_ws, int64_t T, int k, int E, const void* gate_w, void* stream) {
    if (!plan_ws || !gate_w || !dims_ok(T, k, E)) return GROUTER_ERR_INVALID_ARG;
    const PlanLayout L = make_plan_layout(T, k, E);
    const PlanView P = make_plan_view(plan_ws, L);
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_PLAN, s);
    const hipError_t e = launch_row_gates(P, (const bf16_t*)gate_w, (float*)((char*)plan_ws + L.off_row_gate), s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_plan_views(const void* plan_ws, int64_t T, int k, int E, const int32_t** counts,
                       const int32_t** offsets, const int32_t** row_to_src, const int32_t** src_to_row) {
    if (!plan_ws || !dims_ok(T, k, E)) return GROUTER_ERR_INVALID_ARG;
    const PlanView v = make_plan_view(plan_ws, make_plan_layout(T, k, E));
    if (counts) *counts = v.counts;
    if (offsets) *offsets = v.offsets;
    if (row_to_src) *row_to_src = v.row_to_src;
    if (src_to_row) *src_to_row = v.src_to_row;
    return GROUTER_OK;
}

int grouter_plan_status(const void* plan_ws, void* stream) {
    if (!plan_ws) return GROUTER_ERR_INVALID_ARG;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e);
    int32_t flags = 0;
    e = hipMemcpy(&flags, plan_ws, sizeof(flags), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(e);
    return (flags & 1) ? GROUTER_ERR_INDEX_OUT_OF_RANGE : GROUTER_OK;
}

int grouter_permute(const void* plan_ws, int64_t T, int k, int E, int d, const void* in, const void* gate_w,
                    void* out, void* stream) {
    if (!plan_ws || !in || !out || !dims_ok(T, k, E) || d <= 0 || (d % 8)) return GROUTER_ERR_INVALID_ARG;
    if (!aligned16(in) || !aligned16(out)) return GROUTER_ERR_INVALID_ARG;
    const PlanView P = make_plan_view(plan_ws, make_plan_layout(T, k, E));
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(gate_w ? GROUTER_PH_DO : GROUTER_PH_PERMUTE, s);
    const hipError_t e = launch_permute(P, d, (const bf16_t*)in, (const bf16_t*)gate_w, (bf16_t*)out, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_combine(const void* plan_ws, int64_t T, int k, int E, int d, const void* in, const void* gate_w,
                    void* out, void* stream) {
    if (!plan_ws || !in || !out || !dims_ok(T, k, E) || d <= 0 || (d % 8)) return GROUTER_ERR_INVALID_ARG;
    if (!aligned16(in) || !aligned16(out)) return GROUTER_ERR_INVALID_ARG;
    const PlanView P = make_plan_view(plan_ws, make_plan_layout(T, k, E));
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(gate_w ? GROUTER_PH_COMBINE : GROUTER_PH_DXREDUCE, s);
    const hipError_t e = launch_combine(P, d, (const bf16_t*)in, (const bf16_t*)gate_w, (bf16_t*)out, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_moe_fwd(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                    const void* gate_w, const void* W1, const void* W3, const void* W2, void* y, void* ctx_ws,
                    size_t ctx_ws_bytes, void* stream) {
    if (!plan_ws || !x || !W1 || !W3 || !W2 || !y || !ctx_ws) return GROUTER_ERR_INVALID_ARG;
    if (!widths_ok(T, k, E, d, f)) return GROUTER_ERR_INVALID_ARG;
    if (!aligned256(ctx_ws) || !aligned16(x) || !aligned16(W1) || !aligned16(W3) || !aligned16(W2) || !aligned16(y))
        return GROUTER_ERR_INVALID_ARG;
    const CtxLayout C = ctx_layout(T, k, d, f);
    if (ctx_ws_bytes < C.total) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    const PlanView P = make_plan_view(plan_ws, make_plan_layout(T, k, E));
    hipStream_t s = (hipStream_t)stream;
    char* c = (char*)ctx_ws;
    bf16_t* dSdG = (bf16_t*)(c + C.ds_dg);
    bf16_t* dSdU = (bf16_t*)(c + C.ds_du);
    bf16_t* H = (bf16_t*)(c + C.h);
    bf16_t* O = (bf16_t*)(c + C.o);
    const float* row_gate = P.row_gate;   // the plan's, unless this call brings gate weights of its own
    hipError_t e;
    PhaseTimer t_gateup(GROUTER_PH_GATEUP, s);
    if (gate_w) {
        e = launch_row_gates(P, (const bf16_t*)gate_w, (float*)(c + C.row_gate), s);
        if (e != hipSuccess) return fail_hip(e);
        row_gate = (const float*)(c + C.row_gate);
    }
    e = launch_gateup(P, d, f, (const bf16_t*)x, row_gate, (const bf16_t*)W1, (const bf16_t*)W3, dSdG, dSdU, H, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_down(GROUTER_PH_DOWN, s, &t_gateup);
    e = launch_down(P, d, f, H, (const bf16_t*)W2, O, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_combine(GROUTER_PH_COMBINE, s, &t_down);
    e = launch_combine(P, d, O, nullptr, (bf16_t*)y, s);  // the gate weights are already in H
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_moe_fwd_only(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                         const void* gate_w, const void* W1, const void* W3, const void* W2, void* y, void* ws,
                         size_t ws_bytes, void* stream) {
    if (!plan_ws || !x || !W1 || !W3 || !W2 || !y || !ws) return GROUTER_ERR_INVALID_ARG;
    if (!widths_ok(T, k, E, d, f)) return GROUTER_ERR_INVALID_ARG;
    if (!aligned256(ws) || !aligned16(x) || !aligned16(W1) || !aligned16(W3) || !aligned16(W2) || !aligned16(y))
        return GROUTER_ERR_INVALID_ARG;
    const FwdOnlyLayout C = fwd_only_layout(T, k, d, f);
    if (ws_bytes < C.total) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    const PlanView P = make_plan_view(plan_ws, make_plan_layout(T, k, E));
    hipStream_t s = (hipStream_t)stream;
    bf16_t* H = (bf16_t*)((char*)ws + C.h);
    bf16_t* O = (bf16_t*)((char*)ws + C.o);
    const float* row_gate = P.row_gate;   // the plan's, unless this call brings gate weights of its own
    hipError_t e;
    PhaseTimer t_gateup(GROUTER_PH_GATEUP, s);
    if (gate_w) {
        e = launch_row_gates(P, (const bf16_t*)gate_w, (float*)((char*)ws + C.row_gate), s);
        if (e != hipSuccess) return fail_hip(e);
        row_gate = (const float*)((char*)ws + C.row_gate);
    }
    e = launch_gateup(P, d, f, (const bf16_t*)x, row_gate, (const bf16_t*)W1, (const bf16_t*)W3, nullptr, nullptr, H, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_down(GROUTER_PH_DOWN, s, &t_gateup);
    e = launch_down(P, d, f, H, (const bf16_t*)W2, O, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_combine(GROUTER_PH_COMBINE, s, &t_down);
    e = launch_combine(P, d, O, nullptr, (bf16_t*)y, s);  // the gate weights are already in H
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

// ---- grouter_moe_fwd_only with its workspace in a static device array ---------------------------------
// Host code must not use the array's name as a device address: the address comes from hipGetSymbolAddress,
// once per device (every GPU holds its own copy), and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[GROUTER_STATIC_WS_BYTES];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ws[kMaxDevices] = {};

hipError_t static_ws_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ws[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_static_ws[dev] = p;
    }
    *out = g_static_ws[dev];
    return hipSuccess;
}
}  // namespace

size_t grouter_static_ws_bytes(void) { return (size_t)GROUTER_STATIC_WS_BYTES; }

int grouter_moe_fwd_only_static(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                                const void* gate_w, const void* W1, const void* W3, const void* W2, void* y,
                                void* stream) {
    if (!plan_ws || !x || !W1 || !W3 || !W2 || !y) return GROUTER_ERR_INVALID_ARG;
    if (!widths_ok(T, k, E, d, f)) return GROUTER_ERR_INVALID_ARG;
    if (fwd_only_layout(T, k, d, f).total > (size_t)GROUTER_STATIC_WS_BYTES) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    const hipError_t e = static_ws_of_current_device(&ws);
    if (e != hipSuccess) return fail_hip(e);
    // Every byte of H, O and the row gates that the kernels read is written earlier in the same call, so the
    // array needs no clearing between calls.
    return grouter_moe_fwd_only(plan_ws, T, k, E, d, f, x, gate_w, W1, W3, W2, y, ws, (size_t)GROUTER_STATIC_WS_BYTES, stream);
}

int grouter_moe_bwd(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                    const void* gate_w, const void* W1, const void* W3, const void* W2, const void* dY,
                    const void* ctx_ws, size_t ctx_ws_bytes, void* dX, void* dW1, void* dW3, void* dW2,
                    void* scratch_ws, size_t scratch_bytes, void* stream) {
    if (!plan_ws || !x || !W1 || !W3 || !W2 || !dY || !ctx_ws || !dX || !dW1 || !dW3 || !dW2 || !scratch_ws)
        return GROUTER_ERR_INVALID_ARG;
    if (!widths_ok(T, k, E, d, f)) return GROUTER_ERR_INVALID_ARG;
    if (!aligned256(ctx_ws) || !aligned256(scratch_ws) || !aligned16(x) || !aligned16(dY) || !aligned16(dX) || !aligned16(dW1) ||
        !aligned16(dW3) || !aligned16(dW2) || !aligned16(W1) || !aligned16(W3) || !aligned16(W2))
        return GROUTER_ERR_INVALID_ARG;
    const CtxLayout C = ctx_layout(T, k, d, f);
    if (ctx_ws_bytes < C.total) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    const BwdLayout B = bwd_layout(T, k, d, f);
    if (scratch_bytes < B.total) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    const PlanView P = make_plan_view(plan_ws, make_plan_layout(T, k, E));
    hipStream_t s = (hipStream_t)stream;
    const char* c = (const char*)ctx_ws;
    const bf16_t* dSdG = (const bf16_t*)(c + C.ds_dg);
    const bf16_t* dSdU = (const bf16_t*)(c + C.ds_du);
    const bf16_t* H = (const bf16_t*)(c + C.h);
    char* w = (char*)scratch_ws;
    bf16_t* dG = (bf16_t*)(w + B.dg);
    bf16_t* dU = (bf16_t*)(w + B.du);
    bf16_t* dXp = (bf16_t*)(w + B.dxp);
    hipError_t e;
    // dW2 needs nothing from dH and runs first, so that dG and dU are consumed by the two kernels right behind the one
    // that writes them (measured on the 8192-token, 64-expert training shape: dW2 -2 %, the others unchanged)
    PhaseTimer t_dw2(GROUTER_PH_DW2, s);
    e = launch_dw2(P, d, f, H, (const bf16_t*)dY, (bf16_t*)dW2, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_dh(GROUTER_PH_DH, s, &t_dw2);
    e = launch_dh(P, d, f, (const bf16_t*)dY, gate_w ? (const float*)(c + C.row_gate) : P.row_gate, (const bf16_t*)W2, dSdG, dSdU, dG, dU, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_dw13(GROUTER_PH_DW13, s, &t_dh);
    e = launch_dw13(P, d, f, (const bf16_t*)x, dG, dU, (bf16_t*)dW1, (bf16_t*)dW3, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_dxp(GROUTER_PH_DXP, s, &t_dw13);
    e = launch_dxp(P, d, f, dG, dU, (const bf16_t*)W1, (const bf16_t*)W3, dXp, s);
    if (e != hipSuccess) return fail_hip(e);
    PhaseTimer t_dx(GROUTER_PH_DXREDUCE, s, &t_dxp);
    e = launch_combine(P, d, dXp, nullptr, (bf16_t*)dX, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

namespace {
bool stats_dims_ok(int64_t n_outer, int64_t L, int k, int E, int idx_dtype) {
    if (idx_dtype != GROUTER_IDX_INT32 && idx_dtype != GROUTER_IDX_UINT8) return false;
    if (n_outer <= 0 || n_outer > 0x7fffffff || L <= 0 || k <= 0 || k > 64 || E <= 0 || E > kMaxExperts) return false;
    if (idx_dtype == GROUTER_IDX_UINT8 && E > 256) return false;
    if (L > (int64_t)0x7fffffff / k) return false;  // a sample's slot count fits int32
    return true;
}
}  // namespace

int grouter_affinity(const void* topk_idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                     double* entropy_bits, int64_t* loads, double* maxvio, void* stream) {
    if (!topk_idx || !counts || !entropy_bits || !loads || !maxvio) return GROUTER_ERR_INVALID_ARG;
    if (!stats_dims_ok(S, L, k, E, idx_dtype)) return GROUTER_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_AFFINITY, s);
    const hipError_t e = launch_affinity(topk_idx, idx_dtype, S, L, k, E, counts, entropy_bits, loads, maxvio, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_sample_placement(const void* topk_idx, int idx_dtype, int64_t S, int L, int k, int E,
                             const uint64_t* expert_nodes, int n_nodes, int32_t* comm, int32_t* best_node,
                             void* stream) {
    if (!topk_idx || !expert_nodes || !comm || !best_node) return GROUTER_ERR_INVALID_ARG;
    if (!stats_dims_ok(S, L, k, E, idx_dtype) || n_nodes <= 0 || n_nodes > 64) return GROUTER_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_PLACEMENT, s);
    const hipError_t e = launch_placement(topk_idx, idx_dtype, S, L, k, E, expert_nodes, n_nodes, comm, best_node, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_sample_stats(const void* topk_idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                         double* entropy_bits, int64_t* loads, double* maxvio, const uint64_t* expert_nodes, int n_nodes,
                         int32_t* comm, int32_t* best_node, void* stream) {
    if (!topk_idx || !counts || !entropy_bits || !loads || !maxvio || !expert_nodes || !comm || !best_node)
        return GROUTER_ERR_INVALID_ARG;
    if (!stats_dims_ok(S, L, k, E, idx_dtype) || n_nodes <= 0 || n_nodes > 64) return GROUTER_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_SAMPLE_STATS, s);
    const hipError_t e = launch_sample_stats(topk_idx, idx_dtype, S, L, k, E, counts, entropy_bits, loads, maxvio,
                                             expert_nodes, n_nodes, comm, best_node, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_coactivation(const void* topk_idx, int idx_dtype, int64_t T, int k, int E, int64_t* P, void* stream) {
    if (!topk_idx || !P) return GROUTER_ERR_INVALID_ARG;
    if (T <= 0 || k <= 0 || k > 64 || E <= 0 || E > 256) return GROUTER_ERR_INVALID_ARG;
    if (idx_dtype != GROUTER_IDX_INT32 && idx_dtype != GROUTER_IDX_UINT8) return GROUTER_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_COACT, s);
    const hipError_t e = launch_coactivation(topk_idx, idx_dtype, T, k, E, P, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_fold_groups(const int64_t* P, int E_S, int E_T, int32_t* group_of, void* stream) {
    if (!P || !group_of || E_S <= 0 || E_S > kMaxExperts || E_T <= 0 || E_T > E_S) return GROUTER_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_FOLD, s);
    const hipError_t e = launch_fold_groups(P, E_S, E_T, group_of, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_fold_weights(const float* W_s, const int32_t* group_of, int d, int E_S, int E_T, float* out,
                         void* stream) {
    if (!W_s || !group_of || !out || d <= 0 || E_S <= 0 || E_S > kMaxExperts || E_T <= 0 || E_T > E_S)
        return GROUTER_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    PhaseTimer tm(GROUTER_PH_FOLD, s);
    const hipError_t e = launch_fold_weights(W_s, group_of, d, E_S, E_T, out, s);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_mfma_probe(int mode, int iters, int workgroups, float* out, size_t out_elems, void* stream) {
    if (!out || mode < 0 || mode > 7 || iters <= 0 || (iters & 3) || workgroups <= 0 || workgroups > (1 << 20))
        return GROUTER_ERR_INVALID_ARG;
    if (out_elems < (size_t)workgroups * 256) return GROUTER_ERR_WORKSPACE_TOO_SMALL;
    const hipError_t e = launch_mfma_probe(mode, iters, workgroups, out, (hipStream_t)stream);
    return e == hipSuccess ? GROUTER_OK : fail_hip(e);
}

int grouter_timing_enable(int on) {
    std::lock_guard<std::mutex> lock(g_timing_mu);
    g_timing = on != 0;
    return GROUTER_OK;
}

int grouter_timing_read(double* ms, int64_t* launches) {
    std::lock_guard<std::mutex> lock(g_timing_mu);
    for (const TimedLaunch& t : g_pending) {
        hipError_t e = hipEventSynchronize(t.stop);
        float v = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&v, t.start, t.stop);
        if (e != hipSuccess) {  // give up on what is pending, but keep the events for later use
            for (const TimedLaunch& u : g_pending) {
                if (u.owns_start) g_pool.push_back(u.start);
                g_pool.push_back(u.stop);
            }
            g_pending.clear();
            return fail_hip(e);
        }
        g_ms[t.phase] += (double)v;
        g_launches[t.phase] += 1;
    }
    for (const TimedLaunch& u : g_pending) {
        if (u.owns_start) g_pool.push_back(u.start);
        g_pool.push_back(u.stop);
    }
    g_pending.clear();
    for (int p = 0; p < GROUTER_PH_COUNT; ++p) {
        if (ms) ms[p] = g_ms[p];
        if (launches) launches[p] = g_launches[p];
        g_ms[p] = 0.0;
        g_launches[p] = 0;
    }
    return GROUTER_OK;
}

const char* grouter_phase_name(int phase) {
    static const char* names[GROUTER_PH_COUNT] = {"plan", "permute", "gateup", "down", "combine", "dO",
                                                  "dH", "dW2", "dW13", "dXp", "dX_reduce", "affinity",
                                                  "placement", "coactivation", "fold", "sample_stats"};
    return (phase >= 0 && phase < GROUTER_PH_COUNT) ? names[phase] : "?";
}

}  // extern "C"
