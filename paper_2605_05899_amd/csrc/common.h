// Internal declarations shared by the HIP sources of libvismoe (not part of the C-ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe.h"

namespace vismoe {

typedef uint16_t bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int kWave = 64;
constexpr int kMaxE = 512;
constexpr int kMaxK = 64;
constexpr int kMaxS = 8;

// Rows per M-tile of the tiled grouped GEMM; the tile map built by dispatch uses the same constant.
constexpr int kTileM = 256;
// A group of at most kTallM rows is computed as "tall" work units instead of a mostly empty M-tile: kTallM tokens
// against twice as many weight rows (see expert_ffn.hip).
constexpr int kTallM = 128;
// Groups of up to this many rows become tall units (at most kTallM; 0 switches the tall path off).
#ifndef VISMOE_TALL_ROWS
#define VISMOE_TALL_ROWS 128
#endif
constexpr int kTallRows = VISMOE_TALL_ROWS;
static_assert(kTallRows <= kTallM, "a tall unit holds at most kTallM token rows");
// Largest group that becomes a tall unit for a launch of `rows` grouped rows in G groups (0: none), decided from the
// sizes the host knows. Tall units are used when the mean group has at most kTallM rows (pruned prefill: most groups
// are then single, mostly empty M-tiles whose weight rows nothing else shares) and the launch has more work slots
// than the chip has CUs (below that, more and smaller workgroups finish sooner). With larger groups in the mix the
// long tall units only coarsen a schedule of four or five rounds: measured 5 % slower on the 228-rows-per-expert
// prefill, 11 % faster on the 66-rows-per-expert one.
static inline int tall_rows_for(long long rows, int G, int H, int I) {
    if (rows > (long long)kTallM * G) return 0;
    const long long entries = rows / kTileM + (G + 1) / 2;
    const long long slots0 = (I + 127) / 128, slots1 = (H + 255) / 256;
    return entries * (slots0 < slots1 ? slots0 : slots1) > 256 ? kTallRows : 0;
}
// Assignments ranked by one workgroup of the multi-block dispatch.
constexpr int kDispChunk = 1024;
// Largest T*k handled by the single-workgroup dispatch.
constexpr int kDispSmallMax = 8192;
// K-sliced router (decode, small or pruned prefill, mid-size prefill): the contraction is cut into at most
// kSmallSlices K groups (of four wave slices each) whose partial logits, T x padded E floats per group, go through
// the workspace. With few token blocks the one-kernel router leaves most CUs idle and every workgroup walks all of K
// alone (about 20 us whatever the batch); sliced over K the walk is a quarter as long on four times the workgroups.
constexpr int kSmallLogits = 262144;
constexpr int kSmallSlices = 4;
// Expert count padded to a power of two >= 32 (the fragment width) for the K-sliced router.
static inline int small_route_ep(int E) {
    int ep = 32;
    while (ep < E) ep <<= 1;
    return ep;
}
// The K-sliced router is used when its partial logits fit the workspace.
static inline bool sliced_route_ok(int T, int E) {
    return T > 0 && (long long)T * small_route_ep(E) <= kSmallLogits;
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace layout (byte offsets from the 256-byte aligned base), a pure function of the config.
struct WsLayout {
    size_t topk_ids;      // int32 [Tm*k]
    size_t topk_w;        // float [Tm*k]
    size_t offsets;       // int32 [E+S+1]   group offsets: routed experts, then one group per shared expert
    size_t sorted_token;  // int32 [Tm*(k+S)]
    size_t inv_perm;      // int32 [Tm*k]
    size_t n_tiles;       // int32 [2] (+pad): number of M-tiles and of tall row blocks in the tile map
    size_t tile_map;      // int4  [ceil(Tm*(k+S)/kTileM) + E + S]   (group, first row, end row of the group, 1 if tall)
    size_t hist;          // int32 [ceil(Tm*k/kDispChunk) * E]
    size_t partial;       // float [kSmallSlices * kSmallLogits]   K-slices of the small-batch router's logits
    size_t hm;            // bf16  [Tm*(k+S), I]   SwiGLU intermediate
    size_t y;             // bf16  [Tm*(k+S), H]   expert outputs in grouped order
    size_t total;
};

static inline WsLayout ws_layout(const moe_config& c) {
    WsLayout L;
    const size_t Tm = (size_t)c.max_tokens, k = (size_t)c.k, S = (size_t)c.S, E = (size_t)c.E;
    const size_t rows = Tm * (k + S);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.topk_ids = take(Tm * k * 4);
    L.topk_w = take(Tm * k * 4);
    L.offsets = take((E + S + 1) * 4);
    L.sorted_token = take(rows * 4);
    L.inv_perm = take(Tm * k * 4);
    L.n_tiles = take(4);
    L.tile_map = take(((rows + kTileM - 1) / kTileM + E + S) * 16);
    L.hist = take(((Tm * k + kDispChunk - 1) / kDispChunk) * E * 4);
    L.partial = take((size_t)kSmallSlices * kSmallLogits * 4);
    L.hm = take(rows * (size_t)c.I * 2);
    L.y = take(rows * (size_t)c.H * 2);
    L.total = o;
    return L;
}

// Arguments of the grouped GEMM kernels (both the MFMA-tiled one and the weight-streaming one).
// MODE 0: C[pos, n] = silu(A_row(pos) . B0[g][n]) * (A_row(pos) . B1[g][n]),  A rows gathered from x
// MODE 1: C[pos, n] = A[pos] . B0[g][n],                                      A = SwiGLU intermediate
struct GemmParams {
    const bf16_t* A;
    int lda;
    const int* sorted_token;  // MODE 0: grouped position -> compact token row
    const int* keep_idx;      // MODE 0: compact token row -> row of x (nullable)
    const bf16_t* B0;         // routed experts: gate (MODE 0) or down (MODE 1), [E, N, K]
    const bf16_t* B1;         // routed experts: up (MODE 0)
    const bf16_t* Bs0;        // shared experts, same roles, [S, N, K]
    const bf16_t* Bs1;
    int E;                    // groups >= E are shared experts
    int G;                    // number of groups
    long long b_stride;       // N*K
    bf16_t* C;
    int ldc;
    int K;
    int N;
    const int* offsets;       // [G+1]
    const int4* tile_map;     // (group, first row, end row of the group, 1 if tall): the M-tiles, then the tall row blocks
    const int* n_tiles;       // [0] number of M-tiles, [1] number of tall row blocks
    int n_ntiles;             // column tiles per M-tile
    int n_tall;               // column units per tall row block
    // Slab-addressed routed experts (nullable): slabs[e] is the device address of expert e's slab or NULL when the
    // expert is not resident; the operands of this GEMM start slab_off0 / slab_off1 elements into the slab.
    const bf16_t* const* slabs;
    long long slab_off0, slab_off1;
};

// Weight operands of group g. False when the group is a routed expert without a slab: its output rows are zeroed.
__device__ __forceinline__ bool group_weights(const GemmParams& p, int g, bool two, const bf16_t*& b0, const bf16_t*& b1) {
    if (g >= p.E) {
        b0 = p.Bs0 + (size_t)(g - p.E) * p.b_stride;
        b1 = two ? p.Bs1 + (size_t)(g - p.E) * p.b_stride : b0;
        return true;
    }
    if (p.slabs) {
        const bf16_t* s = p.slabs[g];
        if (!s) return false;
        b0 = s + p.slab_off0;
        b1 = two ? s + p.slab_off1 : b0;
        return true;
    }
    b0 = p.B0 + (size_t)g * p.b_stride;
    b1 = two ? p.B1 + (size_t)g * p.b_stride : b0;
    return true;
}

// Kernel launchers (host side, defined next to their kernels). All return hipGetLastError() of the launch.
hipError_t launch_route(const moe_config& c, const bf16_t* x, const int* keep_idx, int T, const bf16_t* w_router,
                        int* topk_ids, float* topk_w, hipStream_t st);
hipError_t launch_dispatch(const moe_config& c, const int* topk_ids, int T, int n_shared_groups, int* offsets,
                           int* sorted_token, int* inv_perm, int* n_tiles, int4* tile_map, int* hist, hipStream_t st);
hipError_t launch_tile_map(int G, const int* offsets, int tall_rows, int* n_tiles, int4* tile_map, hipStream_t st);
hipError_t launch_route_partial(const moe_config& c, const bf16_t* x, const int* keep_idx, int T, const bf16_t* w_router,
                                float* partial, int* n_slices_out, hipStream_t st);
hipError_t launch_route_finish_dispatch(const moe_config& c, const float* partial, int n_slices, int T, int S,
                                        int* topk_ids, float* topk_w, int* offsets, int* sorted_token, int* inv_perm,
                                        int* n_tiles, int4* tile_map, int* hist, hipStream_t st);
hipError_t launch_shared_groups(int T, int S, int* offsets, int* sorted_token, hipStream_t st);
hipError_t launch_grouped_gemm(int mode, bool skinny, const GemmParams& p, int max_rows, hipStream_t st);
hipError_t launch_slab_report(int E, const int* offsets, const bf16_t* const* slabs, int* missing, hipStream_t st);
hipError_t launch_combine(const bf16_t* y, const int* inv_perm, const float* topk_w, int T, int k, int H,
                          const bf16_t* extra, int n_extra, long long extra_stride, bf16_t* out, hipStream_t st);

size_t compress_workspace_bytes(int N, int E);
int compress_wide_min_tokens(int n);
hipError_t launch_token_compress(const float* attn, int n_heads, int N, const int* ids, int L, int k, int E, int K_core,
                                 int K_keep, float lambda, int* keep_idx, float* s_norm_out, float* delta_out, void* ws,
                                 hipStream_t st);

size_t mean_pool_workspace_bytes(int D);
hipError_t launch_mean_pool(const bf16_t* rows, int D, const int* idx, int K, float* out, void* ws, hipStream_t st);
hipError_t launch_routing_histogram(const int* ids, long long n, int E, float* out, hipStream_t st);
hipError_t launch_lookahead_target(const int* future_ids, int W, long long n, int E, float gamma, float* g, hipStream_t st);

size_t predictor_workspace_bytes(int D1, int D2);
hipError_t launch_predictor_mlp(const float* x, int D, const float* W1, const float* s1, const float* t1, int D1,
                                const float* W2, const float* s2, const float* t2, int D2, const float* Wo, int E, int B,
                                float* y, int* top, void* ws, hipStream_t st);

// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Two floats -> packed bf16x2, round-to-nearest-even (inputs finite).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    floatx2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// silu(a) = a / (1 + e^-a) with the hardware exp2 and reciprocal (about 1 ulp each; the result is rounded to bf16).
__device__ __forceinline__ float silu_f(float a) {
    return a * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * a));
}

}  // namespace vismoe
