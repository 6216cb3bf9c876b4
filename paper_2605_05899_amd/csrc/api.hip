// C-ABI entry points: argument validation and the enqueue sequence. No allocation, no copies, no
// synchronisation, except in the two measurement / debugging aids (stage timing, index checking) while they are
// switched on (see include/moe.h for the contract of every call).
#include <stdio.h>

#include <math.h>

#include <mutex>

#include "common.h"

using namespace vismoe;

// Scratch of moe_layer_forward_static: one array per GPU the library is loaded on, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)MOE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// A failed launch is exceptional: say which HIP error it was (the status code alone cannot carry it).
moe_status hip_status(hipError_t e, const char* where) {
    if (e == hipSuccess) return MOE_OK;
    fprintf(stderr, "libvismoe: %s: %s (%s)\n", where, hipGetErrorName(e), hipGetErrorString(e));
    return MOE_ERR_HIP;
}

#define VISMOE_TRY(expr, where)                       \
    do {                                              \
        const moe_status s_ = hip_status((expr), where); \
        if (s_ != MOE_OK) return s_;                  \
    } while (0)

// ---- optional stage timing (see moe.h)
struct StageTimer {
    bool enabled = false;
    hipEvent_t ev[MOE_N_STAGES][2];
    bool used[MOE_N_STAGES];
} g_timer;

void timer_reset() {
    if (g_timer.enabled)
        for (int i = 0; i < MOE_N_STAGES; ++i) g_timer.used[i] = false;
}
void timer_mark(int stage, int which, hipStream_t st) {
    if (!g_timer.enabled) return;
    (void)hipEventRecord(g_timer.ev[stage][which], st);
    if (which == 1) g_timer.used[stage] = true;
}

// ---- optional index checking (see moe.h)
struct IndexCheck {
    bool enabled = false;
    int* d_flag = nullptr;   // device word, set by the check kernels
    int* h_flag = nullptr;   // pinned host copy
} g_check;

__global__ void check_clear_kernel(int* flag) { *flag = 0; }

// flag |= any a[i] outside [lo, hi)
__global__ __launch_bounds__(256) void check_range_kernel(const int* __restrict__ a, long long n, int lo, int hi,
                                                          int* __restrict__ flag) {
    bool bad = false;
    for (long long i = blockIdx.x * 256ll + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const int v = a[i];
        bad |= v < lo || v >= hi;
    }
    if (bad) *flag = 1;
}

// flag |= offsets is not a non-decreasing sequence from 0 to total
__global__ __launch_bounds__(256) void check_offsets_kernel(const int* __restrict__ off, int G, int total,
                                                            int* __restrict__ flag) {
    bool bad = false;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < G; i += gridDim.x * 256) bad |= off[i + 1] < off[i];
    if (blockIdx.x == 0 && threadIdx.x == 0) bad |= off[0] != 0 || off[G] != total;
    if (bad) *flag = 1;
}

struct IndexChecker {
    hipStream_t st;
    bool active;
    explicit IndexChecker(hipStream_t s) : st(s), active(g_check.enabled) {
        if (active) hipLaunchKernelGGL(check_clear_kernel, dim3(1), dim3(1), 0, st, g_check.d_flag);
    }
    void range(const int* a, long long n, int lo, int hi) {
        if (!active || !a || n <= 0) return;
        const unsigned blocks = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
        hipLaunchKernelGGL(check_range_kernel, dim3(blocks), dim3(256), 0, st, a, n, lo, hi, g_check.d_flag);
    }
    void offsets(const int* off, int G, int total) {
        if (!active || !off) return;
        hipLaunchKernelGGL(check_offsets_kernel, dim3((G + 255) / 256), dim3(256), 0, st, off, G, total, g_check.d_flag);
    }
    // MOE_OK when checking is off or every entry was in range
    moe_status result() {
        if (!active) return MOE_OK;
        if (hipMemcpyAsync(g_check.h_flag, g_check.d_flag, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) {
            (void)hip_status(hipGetLastError(), "index check");
            return MOE_ERR_HIP;
        }
        return *g_check.h_flag ? MOE_ERR_INDEX : MOE_OK;
    }
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

moe_status check_config(const moe_config* c) {
    if (!c) return MOE_ERR_NULL;
    if (c->H <= 0 || c->I <= 0 || c->E <= 0 || c->k <= 0 || c->S < 0 || c->max_tokens < 0) return MOE_ERR_SHAPE;
    if (c->k > c->E) return MOE_ERR_SHAPE;
    if (c->E > kMaxE || c->k > kMaxK || c->S > kMaxS) return MOE_ERR_UNSUPPORTED;
    if (c->H % 64 != 0 || c->I % 64 != 0) return MOE_ERR_UNSUPPORTED;
    // int32 indexing of grouped rows and of per-expert weight offsets
    const long long rows = (long long)c->max_tokens * (c->k + c->S);
    if (rows > (1ll << 30) || (long long)c->H * c->I > (1ll << 30)) return MOE_ERR_UNSUPPORTED;
    // the tiled kernel addresses rows of x, of the intermediate and of the expert outputs by 32-bit byte offsets
    if (rows * (c->H > c->I ? c->H : c->I) * 2 >= (1ll << 32)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

moe_status check_tokens(const moe_config* c, int32_t T_in, const int32_t* keep_idx, int32_t T) {
    if (T < 0 || T_in < 0) return MOE_ERR_SHAPE;
    if (T > c->max_tokens) return MOE_ERR_SHAPE;
    if (!keep_idx && T != T_in) return MOE_ERR_SHAPE;
    if (T > 0 && T_in == 0) return MOE_ERR_SHAPE;
    if ((long long)T_in * c->H * 2 >= (1ll << 32)) return MOE_ERR_UNSUPPORTED;      // 32-bit byte offsets into x
    return MOE_OK;
}

moe_status check_ws(const void* ws) {
    if (!ws) return MOE_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return MOE_ERR_ALIGN;
    return MOE_OK;
}

// Weight-streaming kernel when groups are small on average, the LDS-tiled kernel otherwise.
#ifndef VISMOE_SKINNY_ROWS
#define VISMOE_SKINNY_ROWS 40
#endif
bool use_skinny(long long rows, int groups) { return rows <= (long long)VISMOE_SKINNY_ROWS * groups; }

struct WsPtrs {
    int* topk_ids; float* topk_w; int* offsets; int* sorted_token; int* inv_perm; int* n_tiles; int4* tile_map;
    int* hist; float* partial; bf16_t* hm; bf16_t* y;
};

WsPtrs ws_ptrs(const moe_config& c, void* ws) {
    const WsLayout L = ws_layout(c);
    char* b = static_cast<char*>(ws);
    WsPtrs w;
    w.topk_ids = reinterpret_cast<int*>(b + L.topk_ids);
    w.topk_w = reinterpret_cast<float*>(b + L.topk_w);
    w.offsets = reinterpret_cast<int*>(b + L.offsets);
    w.sorted_token = reinterpret_cast<int*>(b + L.sorted_token);
    w.inv_perm = reinterpret_cast<int*>(b + L.inv_perm);
    w.n_tiles = reinterpret_cast<int*>(b + L.n_tiles);
    w.tile_map = reinterpret_cast<int4*>(b + L.tile_map);
    w.hist = reinterpret_cast<int*>(b + L.hist);
    w.partial = reinterpret_cast<float*>(b + L.partial);
    w.hm = reinterpret_cast<bf16_t*>(b + L.hm);
    w.y = reinterpret_cast<bf16_t*>(b + L.y);
    return w;
}

// The two grouped GEMMs over `G` groups (`E_routed` routed + shared), `rows` grouped rows in total.
hipError_t run_ffn(const moe_config& c, const bf16_t* x, const int* keep_idx, int E_routed, int G, int rows,
                   const int* offsets, const int* sorted_token, const int4* tile_map, const int* n_tiles,
                   const bf16_t* w_gate, const bf16_t* w_up, const bf16_t* w_down, const bf16_t* ws_gate,
                   const bf16_t* ws_up, const bf16_t* ws_down, bf16_t* hm, bf16_t* y, hipStream_t st,
                   const bf16_t* const* slabs = nullptr) {
    const bool skinny = use_skinny(rows, G);
    GemmParams p{};
    p.slabs = slabs;                       // slab = [gate (I x H) | up (I x H) | down (H x I)]
    p.slab_off0 = 0;
    p.slab_off1 = (long long)c.I * c.H;
    p.A = x; p.lda = c.H; p.sorted_token = sorted_token; p.keep_idx = keep_idx;
    p.B0 = w_gate; p.B1 = w_up; p.Bs0 = ws_gate; p.Bs1 = ws_up;
    p.E = E_routed; p.G = G; p.b_stride = (long long)c.I * c.H;
    p.C = hm; p.ldc = c.I; p.K = c.H; p.N = c.I;
    p.offsets = offsets; p.tile_map = tile_map; p.n_tiles = n_tiles;
    p.n_ntiles = (c.I + 127) / 128;
    p.n_tall = (c.I + 255) / 256;
    timer_mark(2, 0, st);
    hipError_t e = launch_grouped_gemm(0, skinny, p, rows, st);
    timer_mark(2, 1, st);
    if (e != hipSuccess) return e;
    p.slab_off0 = 2ll * c.I * c.H;
    p.A = hm; p.lda = c.I; p.sorted_token = nullptr; p.keep_idx = nullptr;
    p.B0 = w_down; p.B1 = nullptr; p.Bs0 = ws_down; p.Bs1 = nullptr;
    p.C = y; p.ldc = c.H; p.K = c.I; p.N = c.H;
    p.n_ntiles = (c.H + 255) / 256;
    p.n_tall = (c.H + 255) / 256;
    timer_mark(3, 0, st);
    e = launch_grouped_gemm(1, skinny, p, rows, st);
    timer_mark(3, 1, st);
    return e;
}

}  // namespace

extern "C" {

size_t moe_workspace_bytes(const moe_config* cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    return ws_layout(*cfg).total;
}

const char* moe_status_string(moe_status st) {
    switch (st) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "a required pointer is NULL";
        case MOE_ERR_SHAPE: return "inconsistent sizes";
        case MOE_ERR_ALIGN: return "pointer not sufficiently aligned";
        case MOE_ERR_WORKSPACE: return "scratch memory too small for this config";
        case MOE_ERR_UNSUPPORTED: return "shape not supported by this build";
        case MOE_ERR_HIP: return "HIP kernel launch failed";
        case MOE_ERR_INDEX: return "an index array holds an entry out of range";
        case MOE_ERR_CACHE_FULL: return "no room: the expert cache cannot place a demanded expert";
    }
    return "unknown status";
}

moe_status moe_route(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                     const moe_bf16* w_router, int32_t* topk_ids, float* topk_w, void* ws, void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if ((s = check_tokens(cfg, T_in, keep_idx, T)) != MOE_OK) return s;
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !topk_ids || !topk_w) return MOE_ERR_NULL;
    if (!aligned16(x) || !aligned16(w_router) || !aligned16(topk_ids) || !aligned16(topk_w)) return MOE_ERR_ALIGN;
    (void)ws;
    IndexChecker chk((hipStream_t)stream);
    chk.range(keep_idx, T, 0, T_in);
    if ((s = chk.result()) != MOE_OK) return s;
    timer_reset();
    timer_mark(0, 0, (hipStream_t)stream);
    const hipError_t e = launch_route(*cfg, x, keep_idx, T, w_router, topk_ids, topk_w, (hipStream_t)stream);
    timer_mark(0, 1, (hipStream_t)stream);
    return hip_status(e, "route");
}

moe_status moe_dispatch(const moe_config* cfg, const int32_t* topk_ids, int32_t T, int32_t* expert_offsets,
                        int32_t* sorted_token, int32_t* inv_perm, void* ws, void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if (T < 0 || T > cfg->max_tokens) return MOE_ERR_SHAPE;
    if (!expert_offsets) return MOE_ERR_NULL;
    if ((s = check_ws(ws)) != MOE_OK) return s;
    if (T > 0 && (!topk_ids || !sorted_token || !inv_perm)) return MOE_ERR_NULL;
    const WsPtrs w = ws_ptrs(*cfg, ws);
    IndexChecker chk((hipStream_t)stream);
    chk.range(topk_ids, (long long)T * cfg->k, 0, cfg->E);
    if ((s = chk.result()) != MOE_OK) return s;
    // T == 0 still has a defined result: all-zero offsets
    timer_reset();
    timer_mark(1, 0, (hipStream_t)stream);
    const hipError_t e = launch_dispatch(*cfg, topk_ids, T, 0, expert_offsets, sorted_token, inv_perm, w.n_tiles,
                                         w.tile_map, w.hist, (hipStream_t)stream);
    timer_mark(1, 1, (hipStream_t)stream);
    return hip_status(e, "dispatch");
}

moe_status moe_expert_ffn(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                          const int32_t* expert_offsets, const int32_t* sorted_token, const moe_bf16* w_gate,
                          const moe_bf16* w_up, const moe_bf16* w_down, moe_bf16* y_sorted, void* ws, void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if ((s = check_tokens(cfg, T_in, keep_idx, T)) != MOE_OK) return s;
    if (T == 0) return MOE_OK;
    if (!x || !expert_offsets || !sorted_token || !w_gate || !w_up || !w_down || !y_sorted) return MOE_ERR_NULL;
    if ((s = check_ws(ws)) != MOE_OK) return s;
    if (!aligned16(x) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(y_sorted))
        return MOE_ERR_ALIGN;
    const WsPtrs w = ws_ptrs(*cfg, ws);
    hipStream_t st = (hipStream_t)stream;
    const int rows = T * cfg->k;
    IndexChecker chk(st);
    chk.range(keep_idx, T, 0, T_in);
    chk.offsets(expert_offsets, cfg->E, rows);
    chk.range(sorted_token, rows, 0, T);
    if ((s = chk.result()) != MOE_OK) return s;
    timer_reset();
    if (!use_skinny(rows, cfg->E))
        VISMOE_TRY(launch_tile_map(cfg->E, expert_offsets, tall_rows_for(rows, cfg->E, cfg->H, cfg->I), w.n_tiles, w.tile_map,
                                   st), "tile map");
    return hip_status(run_ffn(*cfg, x, keep_idx, cfg->E, cfg->E, rows, expert_offsets, sorted_token, w.tile_map,
                              w.n_tiles, w_gate, w_up, w_down, nullptr, nullptr, nullptr, w.hm, y_sorted, st),
                      "expert ffn");
}

moe_status moe_expert_ffn_slabs(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx,
                                int32_t T, const int32_t* expert_offsets, const int32_t* sorted_token,
                                const moe_bf16* const* slab_table, moe_bf16* y_sorted, int32_t* missing, void* ws,
                                void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if ((s = check_tokens(cfg, T_in, keep_idx, T)) != MOE_OK) return s;
    if (T == 0) return MOE_OK;
    if (!x || !expert_offsets || !sorted_token || !slab_table || !y_sorted || !missing) return MOE_ERR_NULL;
    if ((s = check_ws(ws)) != MOE_OK) return s;
    if (!aligned16(x) || !aligned16(y_sorted) || !aligned16(slab_table)) return MOE_ERR_ALIGN;
    const WsPtrs w = ws_ptrs(*cfg, ws);
    hipStream_t st = (hipStream_t)stream;
    const int rows = T * cfg->k;
    IndexChecker chk(st);
    chk.range(keep_idx, T, 0, T_in);
    chk.offsets(expert_offsets, cfg->E, rows);
    chk.range(sorted_token, rows, 0, T);
    if ((s = chk.result()) != MOE_OK) return s;
    timer_reset();
    VISMOE_TRY(launch_slab_report(cfg->E, expert_offsets, slab_table, missing, st), "slab report");
    if (!use_skinny(rows, cfg->E))
        VISMOE_TRY(launch_tile_map(cfg->E, expert_offsets, tall_rows_for(rows, cfg->E, cfg->H, cfg->I), w.n_tiles, w.tile_map,
                                   st), "tile map");
    return hip_status(run_ffn(*cfg, x, keep_idx, cfg->E, cfg->E, rows, expert_offsets, sorted_token, w.tile_map,
                              w.n_tiles, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, w.hm, y_sorted, st,
                              slab_table),
                      "expert ffn (slabs)");
}

moe_status moe_shared_ffn(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                          const moe_bf16* ws_gate, const moe_bf16* ws_up, const moe_bf16* ws_down,
                          moe_bf16* shared_out, void* ws, void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if (cfg->S < 1) return MOE_ERR_SHAPE;
    if ((s = check_tokens(cfg, T_in, keep_idx, T)) != MOE_OK) return s;
    if (T == 0) return MOE_OK;
    if (!x || !ws_gate || !ws_up || !ws_down || !shared_out) return MOE_ERR_NULL;
    if ((s = check_ws(ws)) != MOE_OK) return s;
    if (!aligned16(x) || !aligned16(ws_gate) || !aligned16(ws_up) || !aligned16(ws_down) || !aligned16(shared_out))
        return MOE_ERR_ALIGN;
    const WsPtrs w = ws_ptrs(*cfg, ws);
    hipStream_t st = (hipStream_t)stream;
    const int S = cfg->S, rows = S * T;
    IndexChecker chk(st);
    chk.range(keep_idx, T, 0, T_in);
    if ((s = chk.result()) != MOE_OK) return s;
    timer_reset();
    VISMOE_TRY(launch_shared_groups(T, S, w.offsets, w.sorted_token, st), "shared groups");
    if (!use_skinny(rows, S))
        VISMOE_TRY(launch_tile_map(S, w.offsets, tall_rows_for(rows, S, cfg->H, cfg->I), w.n_tiles, w.tile_map, st),
                   "tile map");
    VISMOE_TRY(run_ffn(*cfg, x, keep_idx, 0, S, rows, w.offsets, w.sorted_token, w.tile_map, w.n_tiles, nullptr, nullptr,
                       nullptr, ws_gate, ws_up, ws_down, w.hm, w.y, st), "shared ffn");
    timer_mark(4, 0, st);
    const hipError_t ce = launch_combine(nullptr, nullptr, nullptr, T, 0, cfg->H, w.y, S, (long long)T * cfg->H, shared_out, st);
    timer_mark(4, 1, st);
    return hip_status(ce, "shared sum");
}

moe_status moe_combine(const moe_config* cfg, const moe_bf16* y_sorted, const int32_t* inv_perm, const float* topk_w,
                       int32_t T, const moe_bf16* shared_out, moe_bf16* out, void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if (T < 0 || T > cfg->max_tokens) return MOE_ERR_SHAPE;
    if (T == 0) return MOE_OK;
    if (!y_sorted || !inv_perm || !topk_w || !out) return MOE_ERR_NULL;
    if (!aligned16(y_sorted) || !aligned16(out) || (shared_out && !aligned16(shared_out))) return MOE_ERR_ALIGN;
    IndexChecker chk((hipStream_t)stream);
    chk.range(inv_perm, (long long)T * cfg->k, 0, T * cfg->k);
    if ((s = chk.result()) != MOE_OK) return s;
    timer_reset();
    timer_mark(4, 0, (hipStream_t)stream);
    const hipError_t e = launch_combine(y_sorted, inv_perm, topk_w, T, cfg->k, cfg->H, shared_out, shared_out ? 1 : 0, 0,
                                        out, (hipStream_t)stream);
    timer_mark(4, 1, (hipStream_t)stream);
    return hip_status(e, "combine");
}

moe_status moe_layer_forward(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                             const moe_bf16* w_router, const moe_bf16* w_gate, const moe_bf16* w_up,
                             const moe_bf16* w_down, const moe_bf16* ws_gate, const moe_bf16* ws_up,
                             const moe_bf16* ws_down, moe_bf16* out, int32_t* topk_ids_opt, float* topk_w_opt,
                             void* ws, void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if ((s = check_tokens(cfg, T_in, keep_idx, T)) != MOE_OK) return s;
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !out) return MOE_ERR_NULL;
    const int S = cfg->S;
    if (S > 0 && (!ws_gate || !ws_up || !ws_down)) return MOE_ERR_NULL;
    if ((s = check_ws(ws)) != MOE_OK) return s;
    if (!aligned16(x) || !aligned16(w_router) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) ||
        !aligned16(out) || (S > 0 && (!aligned16(ws_gate) || !aligned16(ws_up) || !aligned16(ws_down))) ||
        (topk_ids_opt && !aligned16(topk_ids_opt)) || (topk_w_opt && !aligned16(topk_w_opt)))
        return MOE_ERR_ALIGN;
    const WsPtrs w = ws_ptrs(*cfg, ws);
    hipStream_t st = (hipStream_t)stream;
    int* ids = topk_ids_opt ? topk_ids_opt : w.topk_ids;
    float* gw = topk_w_opt ? topk_w_opt : w.topk_w;
    const int k = cfg->k, H = cfg->H;
    IndexChecker chk(st);
    chk.range(keep_idx, T, 0, T_in);
    if ((s = chk.result()) != MOE_OK) return s;

    timer_reset();
    if (sliced_route_ok(T, cfg->E)) {
        // K-sliced logits over many workgroups, a top-k kernel, then the dispatch (one workgroup for small batches)
        int n_slices = 0;
        timer_mark(0, 0, st);
        VISMOE_TRY(launch_route_partial(*cfg, x, keep_idx, T, w_router, w.partial, &n_slices, st), "route (logits)");
        timer_mark(0, 1, st);
        timer_mark(1, 0, st);
        VISMOE_TRY(launch_route_finish_dispatch(*cfg, w.partial, n_slices, T, S, ids, gw, w.offsets, w.sorted_token,
                                                w.inv_perm, w.n_tiles, w.tile_map, w.hist, st), "route (top-k) + dispatch");
        timer_mark(1, 1, st);
    } else {
        timer_mark(0, 0, st);
        VISMOE_TRY(launch_route(*cfg, x, keep_idx, T, w_router, ids, gw, st), "route");
        timer_mark(0, 1, st);
        timer_mark(1, 0, st);
        VISMOE_TRY(launch_dispatch(*cfg, ids, T, S, w.offsets, w.sorted_token, w.inv_perm, w.n_tiles, w.tile_map, w.hist,
                                   st), "dispatch");
        timer_mark(1, 1, st);
    }
    const int rows = T * (k + S);
    VISMOE_TRY(run_ffn(*cfg, x, keep_idx, cfg->E, cfg->E + S, rows, w.offsets, w.sorted_token, w.tile_map, w.n_tiles,
                       w_gate, w_up, w_down, ws_gate, ws_up, ws_down, w.hm, w.y, st), "expert ffn");
    // shared groups sit behind the T*k routed rows of y, one block of T rows per shared expert
    timer_mark(4, 0, st);
    const hipError_t ce =
        launch_combine(w.y, w.inv_perm, gw, T, k, H, w.y + (size_t)T * k * H, S, (long long)T * H, out, st);
    timer_mark(4, 1, st);
    return hip_status(ce, "combine");
}

// ---- the fused layer for callers that cannot allocate (see moe.h)
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, resolved on first use

moe_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return hip_status(hipGetLastError(), "static scratch: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return hip_status(e == hipSuccess ? hipErrorInvalidSymbol : e,
                                                       "static scratch: hipGetSymbolAddress");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace

size_t moe_static_scratch_bytes(void) { return kStaticScratchBytes; }

moe_status moe_layer_forward_static(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx,
                                    int32_t T, const moe_bf16* w_router, const moe_bf16* w_gate, const moe_bf16* w_up,
                                    const moe_bf16* w_down, const moe_bf16* ws_gate, const moe_bf16* ws_up,
                                    const moe_bf16* ws_down, moe_bf16* out, int32_t* topk_ids_opt, float* topk_w_opt,
                                    void* stream) {
    moe_status s = check_config(cfg);
    if (s != MOE_OK) return s;
    if (ws_layout(*cfg).total > kStaticScratchBytes) return MOE_ERR_WORKSPACE;
    void* ws = nullptr;
    if ((s = static_scratch(&ws)) != MOE_OK) return s;
    // Nothing in the workspace has to start at zero: every array in it is written by this call before it is read.
    return moe_layer_forward(cfg, x, T_in, keep_idx, T, w_router, w_gate, w_up, w_down, ws_gate, ws_up, ws_down, out,
                             topk_ids_opt, topk_w_opt, ws, stream);
}

moe_status moe_stage_timing_enable(int32_t enable) {
    if (enable && !g_timer.enabled) {
        for (int i = 0; i < MOE_N_STAGES; ++i)
            for (int j = 0; j < 2; ++j)
                if (hipEventCreate(&g_timer.ev[i][j]) != hipSuccess) return MOE_ERR_HIP;
        g_timer.enabled = true;
        timer_reset();
    } else if (!enable && g_timer.enabled) {
        g_timer.enabled = false;
        for (int i = 0; i < MOE_N_STAGES; ++i)
            for (int j = 0; j < 2; ++j) (void)hipEventDestroy(g_timer.ev[i][j]);
    }
    return MOE_OK;
}

moe_status moe_index_checks_enable(int32_t enable) {
    if (enable && !g_check.enabled) {
        if (hipMalloc(&g_check.d_flag, sizeof(int)) != hipSuccess) return MOE_ERR_HIP;
        if (hipHostMalloc(&g_check.h_flag, sizeof(int), hipHostMallocDefault) != hipSuccess) {
            (void)hipFree(g_check.d_flag);
            g_check.d_flag = nullptr;
            return MOE_ERR_HIP;
        }
        g_check.enabled = true;
    } else if (!enable && g_check.enabled) {
        g_check.enabled = false;
        (void)hipFree(g_check.d_flag);
        (void)hipHostFree(g_check.h_flag);
        g_check.d_flag = g_check.h_flag = nullptr;
    }
    return MOE_OK;
}

moe_status moe_stage_timing_read(float* ms_out) {
    if (!ms_out) return MOE_ERR_NULL;
    if (!g_timer.enabled) return MOE_ERR_SHAPE;
    for (int i = 0; i < MOE_N_STAGES; ++i) {
        ms_out[i] = 0.f;
        if (!g_timer.used[i]) continue;
        if (hipEventSynchronize(g_timer.ev[i][1]) != hipSuccess) return MOE_ERR_HIP;
        if (hipEventElapsedTime(&ms_out[i], g_timer.ev[i][0], g_timer.ev[i][1]) != hipSuccess) return MOE_ERR_HIP;
    }
    return MOE_OK;
}

size_t moe_compress_workspace_bytes(int32_t N, int32_t E) {
    if (N < 0 || N > (1 << 22)) return 0;
    return compress_workspace_bytes(N, E);
}

moe_status moe_token_compress(const float* attn, int32_t n_heads, int32_t N, const int32_t* prefix_topk_ids, int32_t L,
                              int32_t k, int32_t E, double alpha, double beta, float lambda, int32_t* keep_idx,
                              float* s_norm_opt, float* delta_opt, void* ws, void* stream) {
    if (N < 0 || n_heads < 1 || L < 1 || k < 1 || E < 1) return MOE_ERR_SHAPE;
    if (!(alpha >= 0.0) || !(beta >= alpha) || !(beta <= 1.0)) return MOE_ERR_SHAPE;
    if (E > kMaxE || N > (1 << 22)) return MOE_ERR_UNSUPPORTED;
    if (N == 0) return MOE_OK;
    const int K_core = (int)floor(alpha * (double)N), K_keep = (int)floor(beta * (double)N);
    if (K_keep == 0) return MOE_OK;
    if (!attn || !prefix_topk_ids || !keep_idx) return MOE_ERR_NULL;
    moe_status s = check_ws(ws);
    if (s != MOE_OK) return s;
    if (!aligned16(attn) || !aligned16(prefix_topk_ids) || !aligned16(keep_idx)) return MOE_ERR_ALIGN;
    return hip_status(launch_token_compress(attn, n_heads, N, prefix_topk_ids, L, k, E, K_core, K_keep, lambda, keep_idx,
                                            s_norm_opt, delta_opt, ws, (hipStream_t)stream),
                      "token_compress");
}

int32_t moe_compress_wide_min_tokens(int32_t n) { return compress_wide_min_tokens(n); }

size_t moe_mean_pool_workspace_bytes(int32_t D) {
    if (D < 8 || D % 8 != 0) return 0;
    return mean_pool_workspace_bytes(D);
}

moe_status moe_mean_pool(const moe_bf16* rows, int32_t n_rows, int32_t D, const int32_t* idx, int32_t K, float* out,
                         void* ws, void* stream) {
    if (n_rows < 0 || K < 0 || D < 8) return MOE_ERR_SHAPE;
    if (D % 8 != 0) return MOE_ERR_UNSUPPORTED;
    if (!idx && K > n_rows) return MOE_ERR_SHAPE;
    if (K > 0 && n_rows == 0) return MOE_ERR_SHAPE;
    if (K == 0) return MOE_OK;
    if (!rows || !out) return MOE_ERR_NULL;
    moe_status s = check_ws(ws);
    if (s != MOE_OK) return s;
    if (!aligned16(rows) || !aligned16(out)) return MOE_ERR_ALIGN;
    IndexChecker chk((hipStream_t)stream);
    chk.range(idx, K, 0, n_rows);
    if ((s = chk.result()) != MOE_OK) return s;
    return hip_status(launch_mean_pool(rows, D, idx, K, out, ws, (hipStream_t)stream), "mean pool");
}

moe_status moe_routing_histogram(const int32_t* ids, int64_t n, int32_t E, float* out, void* stream) {
    if (n < 0 || E < 1) return MOE_ERR_SHAPE;
    if (E > kMaxE) return MOE_ERR_UNSUPPORTED;
    if (!out || (n > 0 && !ids)) return MOE_ERR_NULL;
    return hip_status(launch_routing_histogram(ids, n, E, out, (hipStream_t)stream), "routing histogram");
}

moe_status moe_lookahead_target(const int32_t* future_ids, int32_t W, int64_t n, int32_t E, float gamma, float* g,
                                void* stream) {
    if (W < 0 || n < 0 || E < 1 || !(gamma > 0.f) || !(gamma <= 1.f)) return MOE_ERR_SHAPE;
    if (E > kMaxE) return MOE_ERR_UNSUPPORTED;
    if (!g || (W > 0 && n > 0 && !future_ids)) return MOE_ERR_NULL;
    return hip_status(launch_lookahead_target(future_ids, W, n, E, gamma, g, (hipStream_t)stream), "lookahead target");
}

size_t moe_predictor_workspace_bytes(int32_t D1, int32_t D2) {
    if (D1 < 4 || D2 < 4 || D1 % 4 != 0 || D2 % 4 != 0) return 0;
    return predictor_workspace_bytes(D1, D2);
}

moe_status moe_predictor_forward(const float* x, int32_t D, const float* W1, const float* s1, const float* t1, int32_t D1,
                                 const float* W2, const float* s2, const float* t2, int32_t D2, const float* Wo,
                                 int32_t E, int32_t B, float* y, int32_t* top, void* ws, void* stream) {
    if (D < 4 || D1 < 4 || D2 < 4 || E < 1 || B < 0 || B > E) return MOE_ERR_SHAPE;
    if (D % 4 != 0 || D1 % 4 != 0 || D2 % 4 != 0 || E > kMaxE) return MOE_ERR_UNSUPPORTED;
    if (!x || !W1 || !s1 || !t1 || !W2 || !s2 || !t2 || !Wo || !y || (B > 0 && !top)) return MOE_ERR_NULL;
    moe_status s = check_ws(ws);
    if (s != MOE_OK) return s;
    if (!aligned16(x) || !aligned16(W1) || !aligned16(W2) || !aligned16(Wo)) return MOE_ERR_ALIGN;
    return hip_status(launch_predictor_mlp(x, D, W1, s1, t1, D1, W2, s2, t2, D2, Wo, E, B, y, top, ws, (hipStream_t)stream),
                      "predictor mlp");
}

}  // extern "C"
