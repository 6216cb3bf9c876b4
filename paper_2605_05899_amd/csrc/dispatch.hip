// Dispatch: the deterministic permutation of the T*k (token, slot) assignments into expert-grouped order.
// The paper leaves the layer's internals to its base runtime (Sec. 2.1); what is fixed here is that a group
// keeps ascending token order, which makes the permutation a pure function of the routing decision. So there is
// no arrival-order atomic anywhere: ranks come from wave ballots, per-wave counters in LDS and prefix sums.
//
// Large inputs: rank kernel (one workgroup per kDispChunk assignments) -> scatter kernel (prefix over chunks and
// experts recomputed by every workgroup, then the positions). Small inputs (T*k <= 8192): one workgroup does it all.
// The scatter step also emits the M-tile map of the tiled grouped GEMM and appends one group per shared expert
// (every token, identity order) behind the routed groups.
#include "common.h"
#include "topk.h"

namespace vismoe {

// Stable rank of each of a wave's elements among the wave's earlier elements with the same expert, on top of
// the wave's running per-expert counter `cnt` (LDS, this wave's own row). Returns the rank; updates cnt.
__device__ __forceinline__ int wave_rank_step(int e, bool valid, int nbits, int* cnt, int lane) {
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long bal = __ballot(valid && bit);
        peers &= bit ? bal : ~bal;
    }
    const unsigned long long lt = (1ull << lane) - 1ull;
    // every lane reads its counter, then (and only then) the first lane of each group of equal ids writes it back:
    // the wave barrier keeps the compiler from moving a write above another lane's read; in hardware the LDS
    // operations of one wave complete in issue order
    const int base = valid ? cnt[e] : 0;
    __builtin_amdgcn_wave_barrier();
    const int rank = base + __popcll(peers & lt);
    if (valid && (peers & lt) == 0) cnt[e] = base + __popcll(peers);
    __builtin_amdgcn_wave_barrier();
    return rank;
}

__device__ __forceinline__ int bits_for(int E) {
    int b = 1;
    while ((1 << b) < E) ++b;
    return b;
}

// Inclusive scan over the first n_valid of blockDim.x ints held one per thread (the rest must be zero; their result
// is unspecified); buf is LDS of blockDim.x ints. The scan itself is
// done by wave 0 alone, 64 values at a time with a running carry (two workgroup barriers in total instead of two per
// doubling step).
// Thread tid contributes at position pos (a permutation of the thread indices) and gets the sum up to that position.
__device__ __forceinline__ int block_inclusive_scan_at(int v, int pos, int* buf, int tid, int n_valid) {
    buf[pos] = v;
    __syncthreads();
    if (tid < 64) {
        int carry = 0;
        for (int base = 0; base < n_valid; base += 64) {     // entries at and beyond n_valid are zero and never used
            int x = buf[base + tid];
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int y = __shfl_up(x, off);
                if (tid >= off) x += y;
            }
            x += carry;
            buf[base + tid] = x;
            carry = __shfl(x, 63);
        }
    }
    __syncthreads();
    return buf[pos];
}
__device__ __forceinline__ int block_inclusive_scan(int v, int* buf, int tid, int n_valid) {
    return block_inclusive_scan_at(v, tid, buf, tid, n_valid);
}

// The work of a group of cnt rows: a group of at most tall_rows rows is one tall row block; any other group is cut
// into M-tiles of kTileM rows (the last one partial). Only whole groups go the tall way: the partial last M-tile of a
// larger group walks K in step with the group's other M-tiles and finds their weight rows in L2, which a tall unit,
// covering two column tiles at a pace of its own, would fetch from HBM again (measured: 30 us slower on the
// 512-rows-per-expert prefill when remainders were made tall).
__device__ __forceinline__ void group_tiles(int cnt, int tall_rows, int& n_mtiles, int& has_tall) {
    has_tall = (cnt > 0 && cnt <= tall_rows) ? 1 : 0;
    n_mtiles = has_tall ? 0 : (cnt + kTileM - 1) / kTileM;
}

// Tile map from per-group (offset, count), one group per thread (G <= blockDim.x): first the M-tiles of all groups,
// group-major, then the tall row blocks of all groups. n_tiles[0] and n_tiles[1] count the two parts.
__device__ void emit_tiles(int off, int cnt, int G, int tall_rows, int* s_scan, int* n_tiles, int4* tile_map) {
    const int tid = threadIdx.x;
    int tiles = 0, tall = 0;
    if (tid < G) group_tiles(cnt, tall_rows, tiles, tall);
    const int tinc = block_inclusive_scan(tiles, s_scan, tid, G);
    const int n_big = s_scan[G - 1];
    __syncthreads();
    const int ainc = block_inclusive_scan(tall, s_scan, tid, G);
    if (tid < G) {
        const int tfirst = tinc - tiles;
        for (int i = 0; i < tiles; ++i) tile_map[tfirst + i] = make_int4(tid, off + i * kTileM, off + cnt, 0);
        if (tall) tile_map[n_big + ainc - 1] = make_int4(tid, off, off + cnt, 1);
        if (tid == G - 1) {
            n_tiles[0] = n_big;
            n_tiles[1] = ainc;
        }
    }
    __syncthreads();
}

// Writes offsets[0..G], the tile maps and n_tiles from per-group counts (one group per thread, G <= blockDim.x).
// Groups [E, G) are the shared experts: T rows each.
__device__ void emit_offsets_and_tiles(int my_count, int G, int tall_rows, int* s_scan, int* offsets, int* n_tiles,
                                       int4* tile_map, int* s_off /*LDS [G+1] or null*/) {
    const int tid = threadIdx.x;
    const int cnt = (tid < G) ? my_count : 0;
    const int inc = block_inclusive_scan(cnt, s_scan, tid, G);
    const int off = inc - cnt;
    if (tid < G) {
        offsets[tid] = off;
        if (s_off) s_off[tid] = off;
        if (tid == G - 1) {
            offsets[G] = inc;
            if (s_off) s_off[G] = inc;
        }
    }
    __syncthreads();
    emit_tiles(off, cnt, G, tall_rows, s_scan, n_tiles, tile_map);
}

// ---------------------------------------------------------------- small path: one workgroup of 1024 threads
constexpr int kSmallWaves = 16, kSmallPerWave = kDispSmallMax / kSmallWaves, kSmallIter = kSmallPerWave / 64;

// The whole dispatch for T*k <= kDispSmallMax inside one workgroup of 1024 threads (512 assignments per wave in 8
// steps). LDS: s_cnt [16 * E], s_scan [1024], s_off [E + S + 1].
__device__ __forceinline__ void dispatch_small_body(const int* __restrict__ ids, int T, int k, int E, int S, int tall_rows,
                                                    int* __restrict__ offsets, int* __restrict__ sorted_token,
                                                    int* __restrict__ inv_perm, int* __restrict__ n_tiles,
                                                    int4* __restrict__ tile_map, int* s_cnt, int* s_scan, int* s_off) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = T * k, G = E + S, nbits = bits_for(E);

    // Each wave ranks one contiguous run of assignments, 64 at a time; the run length adapts to N so that small
    // batches are spread over all 16 waves instead of queueing up in the first one.
    const int per_wave = ((N + kSmallWaves * 64 - 1) / (kSmallWaves * 64)) * 64;
    const int iters = per_wave / 64;
    int my_e[kSmallIter], my_rank[kSmallIter];
#pragma unroll
    for (int it = 0; it < kSmallIter; ++it) {            // all loads first: one memory round trip, not eight
        const int idx = wave * per_wave + it * 64 + lane;
        my_e[it] = (it < iters && idx < N) ? ids[idx] : 0;
    }
    for (int i = tid; i < kSmallWaves * E; i += 1024) s_cnt[i] = 0;
    __syncthreads();

    int* cnt = s_cnt + wave * E;
#pragma unroll
    for (int it = 0; it < kSmallIter; ++it) {
        if (it < iters) {
            const int idx = wave * per_wave + it * 64 + lane;
            my_rank[it] = wave_rank_step(my_e[it], idx < N, nbits, cnt, lane);
        }
    }
    __syncthreads();
    // exclusive prefix of the per-wave counters over waves, per expert; the total is the group size
    int total = 0;
    if (tid < E) {
        for (int w = 0; w < kSmallWaves; ++w) {
            const int c = s_cnt[w * E + tid];
            s_cnt[w * E + tid] = total;
            total += c;
        }
    }
    const int my_count = (tid < E) ? total : T;     // shared groups hold every token
    __syncthreads();
    emit_offsets_and_tiles(my_count, G, tall_rows, s_scan, offsets, n_tiles, tile_map, s_off);

#pragma unroll
    for (int it = 0; it < kSmallIter; ++it) {
        const int idx = wave * per_wave + it * 64 + lane;
        if (it < iters && idx < N) {
            const int e = my_e[it];
            const int pos = s_off[e] + s_cnt[wave * E + e] + my_rank[it];
            inv_perm[idx] = pos;
            sorted_token[pos] = idx / k;
        }
    }
    for (int i = tid; i < S * T; i += 1024) sorted_token[N + i] = i % T;
}

__global__ __launch_bounds__(1024) void dispatch_small_kernel(const int* __restrict__ ids, int T, int k, int E, int S,
                                                              int tall_rows,
                                                              int* __restrict__ offsets, int* __restrict__ sorted_token,
                                                              int* __restrict__ inv_perm, int* __restrict__ n_tiles,
                                                              int4* __restrict__ tile_map) {
    __shared__ int s_cnt[kSmallWaves * kMaxE];
    __shared__ int s_scan[1024];
    __shared__ int s_off[kMaxE + kMaxS + 1];
    dispatch_small_body(ids, T, k, E, S, tall_rows, offsets, sorted_token, inv_perm, n_tiles, tile_map, s_cnt, s_scan,
                        s_off);
}

// ---------------------------------------------------------------- small batches: router finish, then dispatch
// Second half of the small-batch router. T/4 one-wave workgroups (four tokens each, one per 16-lane row): each sums
// the K-slices of its tokens' logits in slice order (a fixed order) and runs the top-k; the dispatch then runs as the
// single-workgroup kernel above. (One 1024-thread workgroup doing all three steps was 2.5 us slower on the 64-token
// decode batch: its 16 waves share the four SIMDs of one CU, and the top-k is instruction-bound.)
template <int EP>
__global__ __launch_bounds__(64) void route_topk_small_kernel(const float* __restrict__ partial, int n_slices, int T,
                                                              int k, int E, int norm_topk, int* __restrict__ topk_ids,
                                                              float* __restrict__ topk_w) {
    __shared__ float s_logit[4 * EP];
    const int lane = threadIdx.x;
    const int t_base = blockIdx.x * 4;
    const size_t n = (size_t)T * EP;
    constexpr int kPer = 4 * EP / 64;                 // logits per thread
    float v[kPer][kSmallSlices];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int i = lane + u * 64;                  // element of the workgroup's [4][EP] block
        const bool live = t_base + i / EP < T;
        const size_t g = (size_t)t_base * EP + i;
#pragma unroll
        for (int sl = 0; sl < kSmallSlices; ++sl) v[u][sl] = (live && sl < n_slices) ? partial[(size_t)sl * n + g] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        float acc = 0.f;
#pragma unroll
        for (int sl = 0; sl < kSmallSlices; ++sl) acc += v[u][sl];
        s_logit[lane + u * 64] = acc;
    }
    __syncthreads();
    const int row = lane >> 4, l16 = lane & 15;
    const int t = t_base + row, tc = min(t, T - 1);
    topk_row<EP / 16>(s_logit + row * EP, E, k, norm_topk, l16, t < T, topk_ids + (size_t)tc * k, topk_w + (size_t)tc * k);
}

hipError_t launch_route_finish_dispatch(const moe_config& c, const float* partial, int n_slices, int T, int S,
                                        int* topk_ids, float* topk_w, int* offsets, int* sorted_token, int* inv_perm,
                                        int* n_tiles, int4* tile_map, int* hist, hipStream_t st) {
#define VISMOE_RFD(EP)                                                                                              \
    hipLaunchKernelGGL(route_topk_small_kernel<EP>, dim3((T + 3) / 4), dim3(64), 0, st, partial, n_slices, T, c.k,  \
                       c.E, c.norm_topk, topk_ids, topk_w)
    const int ep = small_route_ep(c.E);
    if (ep == 32) VISMOE_RFD(32);
    else if (ep == 64) VISMOE_RFD(64);
    else if (ep == 128) VISMOE_RFD(128);
    else if (ep == 256) VISMOE_RFD(256);
    else VISMOE_RFD(512);
#undef VISMOE_RFD
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // one workgroup when the assignments fit it, the two-kernel dispatch otherwise
    return launch_dispatch(c, topk_ids, T, S, offsets, sorted_token, inv_perm, n_tiles, tile_map, hist, st);
}

// ---------------------------------------------------------------- large path
// Step 1: ranks inside a chunk of kDispChunk assignments (written to rank_tmp) and the chunk's histogram.
__global__ __launch_bounds__(256) void dispatch_rank_kernel(const int* __restrict__ ids, int N, int E,
                                                            int* __restrict__ rank_tmp, int* __restrict__ hist) {
    constexpr int NW = 4, PER_WAVE = kDispChunk / NW, ITER = PER_WAVE / 64;
    __shared__ int s_cnt[NW * kMaxE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nbits = bits_for(E);
    const int base = blockIdx.x * kDispChunk;

    for (int i = tid; i < NW * E; i += 256) s_cnt[i] = 0;
    __syncthreads();
    int my_e[ITER], my_rank[ITER];
    int* cnt = s_cnt + wave * E;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = base + wave * PER_WAVE + it * 64 + lane;
        const bool valid = idx < N;
        const int e = valid ? ids[idx] : 0;
        my_e[it] = e;
        my_rank[it] = wave_rank_step(e, valid, nbits, cnt, lane);
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256) {
        int total = 0;
        for (int w = 0; w < NW; ++w) {
            const int c = s_cnt[w * E + e];
            s_cnt[w * E + e] = total;
            total += c;
        }
        hist[(size_t)blockIdx.x * E + e] = total;
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = base + wave * PER_WAVE + it * 64 + lane;
        if (idx < N) rank_tmp[idx] = s_cnt[wave * E + my_e[it]] + my_rank[it];
    }
}

// Step 2: final positions. One workgroup per chunk (and the same 1024 assignments). Every workgroup first adds up,
// per expert, the histograms of all chunks (the group sizes) and of the chunks before its own (where its chunk's
// rows start inside each group): chunks are dealt to 1024 / E_pad thread groups whose partial sums meet in LDS, so a
// workgroup reads the whole chunk x expert table once, from L2, in a batch or two of independent loads. A scan over
// the group sizes gives the group offsets. That is redundant work in every workgroup and still cheaper than a
// launch of its own for the scan: the table is small and a launch costs microseconds. Workgroup 0 also writes the
// offsets and the tile map; the identity rows of the shared-expert groups are spread over all workgroups.
__global__ __launch_bounds__(1024) void dispatch_scatter_kernel(const int* __restrict__ ids, int T, int k, int E, int S,
                                                                int e_pad, int tall_rows, const int* __restrict__ hist,
                                                                int n_chunks, int* __restrict__ offsets,
                                                                int* __restrict__ n_tiles, int4* __restrict__ tile_map,
                                                                int* __restrict__ sorted_token,
                                                                int* __restrict__ inv_perm /* in: rank, out: position */) {
    __shared__ int s_scan[1024];
    __shared__ int s_part[2][1024];          // [total | before][thread group * e_pad + expert]
    __shared__ int s_base[kMaxE];            // group offset + rows of the earlier chunks, per expert
    const int tid = threadIdx.x;
    const int N = T * k, G = E + S;
    const int parts = 1024 / e_pad;          // e_pad: E rounded up to a power of two (at most 512): at least 2 groups
    {
        const int e = tid & (e_pad - 1), part = tid / e_pad;
        int tot = 0, before = 0;
        if (e < E) {
            for (int c0 = part; c0 < n_chunks; c0 += 16 * parts) {
                int h[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int c = c0 + u * parts;
                    h[u] = (c < n_chunks) ? hist[(size_t)c * E + e] : 0;
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    tot += h[u];
                    if (c0 + u * parts < (int)blockIdx.x) before += h[u];
                }
            }
        }
        s_part[0][tid] = tot;
        s_part[1][tid] = before;
    }
    __syncthreads();
    int my_count = 0, my_before = 0;
    if (tid < E) {
        for (int q = 0; q < parts; ++q) {
            my_count += s_part[0][q * e_pad + tid];
            my_before += s_part[1][q * e_pad + tid];
        }
    } else if (tid < G) {
        my_count = T;                        // shared groups hold every token
    }
    const int inc = block_inclusive_scan(my_count, s_scan, tid, G);
    const int off = inc - my_count;
    if (tid < E) s_base[tid] = off + my_before;
    if (blockIdx.x == 0) {
        if (tid < G) {
            offsets[tid] = off;
            if (tid == G - 1) offsets[G] = inc;
        }
        __syncthreads();
        emit_tiles(off, tid < G ? my_count : 0, G, tall_rows, s_scan, n_tiles, tile_map);
    }
    __syncthreads();
    const int idx = blockIdx.x * 1024 + tid;
    if (idx < N) {
        const int e = ids[idx];
        const int pos = s_base[e] + inv_perm[idx];
        inv_perm[idx] = pos;
        sorted_token[pos] = idx / k;
    }
    for (int i = blockIdx.x * 1024 + tid; i < S * T; i += gridDim.x * 1024) sorted_token[N + i] = i % T;
}

hipError_t launch_dispatch(const moe_config& c, const int* topk_ids, int T, int n_shared_groups, int* offsets,
                           int* sorted_token, int* inv_perm, int* n_tiles, int4* tile_map, int* hist, hipStream_t st) {
    const int N = T * c.k, S = n_shared_groups;
    const int tall_rows = tall_rows_for((long long)T * (c.k + S), c.E + S, c.H, c.I);
    if (N <= kDispSmallMax) {
        hipLaunchKernelGGL(dispatch_small_kernel, dim3(1), dim3(1024), 0, st, topk_ids, T, c.k, c.E, S, tall_rows, offsets,
                           sorted_token, inv_perm, n_tiles, tile_map);
        return hipGetLastError();
    }
    const int n_chunks = (N + kDispChunk - 1) / kDispChunk;
    static_assert(kDispChunk == 1024, "the scatter kernel places one chunk per 1024-thread workgroup");
    hipLaunchKernelGGL(dispatch_rank_kernel, dim3(n_chunks), dim3(256), 0, st, topk_ids, N, c.E, inv_perm, hist);
    hipLaunchKernelGGL(dispatch_scatter_kernel, dim3(n_chunks), dim3(1024), 0, st, topk_ids, T, c.k, c.E, S,
                       small_route_ep(c.E), tall_rows, hist, n_chunks, offsets, n_tiles, tile_map, sorted_token, inv_perm);
    return hipGetLastError();
}

// Tile map from existing offsets (used when the caller brings its own expert_offsets).
__global__ __launch_bounds__(1024) void tile_map_kernel(int G, const int* __restrict__ offsets, int tall_rows,
                                                        int* __restrict__ n_tiles,
                                                        int4* __restrict__ tile_map) {
    __shared__ int s_scan[1024];
    const int tid = threadIdx.x;
    int off = 0, cnt = 0;
    if (tid < G) {
        off = offsets[tid];
        cnt = offsets[tid + 1] - off;
    }
    emit_tiles(off, cnt, G, tall_rows, s_scan, n_tiles, tile_map);
}

hipError_t launch_tile_map(int G, const int* offsets, int tall_rows, int* n_tiles, int4* tile_map, hipStream_t st) {
    hipLaunchKernelGGL(tile_map_kernel, dim3(1), dim3(1024), 0, st, G, offsets, tall_rows, n_tiles, tile_map);
    return hipGetLastError();
}

// offsets[0..S] = s*T and sorted_token = identity per group: the group table of a shared-experts-only run.
__global__ void shared_groups_kernel(int T, int S, int* __restrict__ offsets, int* __restrict__ sorted_token) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx <= S) offsets[idx] = idx * T;
    if (idx < S * T) sorted_token[idx] = idx % T;
}

hipError_t launch_shared_groups(int T, int S, int* offsets, int* sorted_token, hipStream_t st) {
    const int total = S * T > S + 1 ? S * T : S + 1;
    hipLaunchKernelGGL(shared_groups_kernel, dim3((total + 255) / 256), dim3(256), 0, st, T, S, offsets, sorted_token);
    return hipGetLastError();
}

}  // namespace vismoe
