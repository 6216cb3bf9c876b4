/* moe.h -- C-ABI of the MI355X (gfx950) MoE-layer forward library (libvismoe.so).
 *
 * The layer is the sparse MoE feed-forward block of a vision-language MoE model (paper Sec. 2.1: every token
 * activates a small subset of the experts of a layer; Table 2: 128 experts / top-8, 72 experts / top-6 plus 2
 * shared experts). The paper treats the layer as a black box of its base runtime; the operation computed here is
 * the standard definition:
 *
 *   xt[j]      = x[keep_idx[j]]                       (retained-token stream after pruning: Sec. 3.2, Alg. 1
 *                                                      output I_keep; Sec. 3.4.1: later layers run compressed)
 *   logit[j,e] = <xt[j], w_router[e]>                 fp32 accumulation of exact bf16 products
 *   top-k by logit (ties to the lower expert), listed in descending logit order
 *   w[j,s]     = softmax(logit[j,:])[e_s], renormalised over the k selected when norm_topk != 0
 *   group e    = assignments (j,s) with e_s == e, in ascending j; expert_offsets = exclusive scan of group sizes
 *   y[pos]     = w_down[e] . ( silu(w_gate[e] . xt[j]) * (w_up[e] . xt[j]) )          (SwiGLU expert)
 *   out[j]     = sum_s w[j,s] * y[pos(j,s)]  +  sum over shared experts FFN_sh(xt[j])  (Sec. 3.4.1: shared
 *                                                      experts are always on, hit by every token)
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller (for instance torch tensors' data_ptr()).
 *     `cfg` is a HOST pointer. Nothing is retained after the call returns except what is written to the outputs
 *     and to the workspace.
 *   - bf16 is passed as uint16_t storage. Tensors are row-major with the innermost dimension contiguous;
 *     every base pointer must be 16-byte aligned. Weight matrices are "out x in": w_gate/w_up [E, I, H],
 *     w_down [E, H, I], w_router [E, H]; shared experts ws_gate/ws_up [S, I, H], ws_down [S, H, I].
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default stream). They never
 *     allocate, never copy between host and device and never synchronise.
 *   - The workspace `ws` is device memory of at least moe_workspace_bytes(cfg) bytes, 256-byte aligned, allocated
 *     once by the caller. Calls that share one workspace must be ordered on one stream; calls with distinct
 *     workspaces are independent.
 *   - With keep_idx == NULL, T must equal T_in. With keep_idx, output row j belongs to input row keep_idx[j] and
 *     all outputs are compact ([T, ...]); keep_idx may be unsorted and may repeat rows. Entries outside
 *     [0, T_in) are undefined behaviour (not checked on the device).
 *   - T == 0 returns MOE_OK without launching anything.
 *   - Errors are reported by return value only (no exceptions, no abort). On any status other than MOE_OK
 *     nothing has been launched, except MOE_ERR_HIP, which reports a failed launch (hipGetLastError) and may
 *     leave earlier kernels of the same call enqueued.
 *   - Supported shapes: 1 <= k <= min(E, 64); E <= 512; H and I multiples of 64; 0 <= S <= 8;
 *     T <= cfg->max_tokens. Anything else returns MOE_ERR_UNSUPPORTED / MOE_ERR_SHAPE.
 *   - Results are deterministic: the same inputs give bit-identical ids, permutation and outputs.
 */
#ifndef VISMOE_MOE_H
#define VISMOE_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t moe_bf16;

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    MOE_ERR_SHAPE = 2,       /* inconsistent sizes (k > E, T > max_tokens, T != T_in, ...)   */
    MOE_ERR_ALIGN = 3,       /* a base pointer is not 16-byte aligned (ws: 256-byte)         */
    MOE_ERR_WORKSPACE = 4,   /* the scratch memory at hand is too small for this config      */
    MOE_ERR_UNSUPPORTED = 5, /* valid layer, but outside the shapes this build supports      */
    MOE_ERR_HIP = 6,         /* a kernel launch failed                                       */
    MOE_ERR_INDEX = 7,       /* index checking is on and an index array holds an entry out of range */
    MOE_ERR_CACHE_FULL = 8   /* the expert cache cannot place a demanded expert: nothing is evictable */
} moe_status;

typedef struct {
    int32_t H;          /* hidden size                                             */
    int32_t I;          /* expert intermediate size                                */
    int32_t E;          /* routed experts                                          */
    int32_t k;          /* experts per token                                       */
    int32_t S;          /* shared experts (0 = none)                               */
    int32_t norm_topk;  /* != 0: gate weights renormalised over the k selected     */
    int32_t max_tokens; /* upper bound on T; sizes the workspace                   */
} moe_config;

/* Bytes of device workspace every other call needs for this config; 0 if the config is invalid. */
size_t moe_workspace_bytes(const moe_config* cfg);

/* Static, NUL-terminated description of a status code (host pointer, never freed). */
const char* moe_status_string(moe_status st);

/* Router: steps "logit", "top-k", "w" above.
 *   x [T_in, H] bf16, keep_idx [T] int32 or NULL, w_router [E, H] bf16
 *   -> topk_ids [T, k] int32 (descending logit), topk_w [T, k] fp32. */
moe_status moe_route(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                     const moe_bf16* w_router, int32_t* topk_ids, float* topk_w, void* ws, void* stream);

/* Dispatch: the permutation of the T*k assignments into expert-grouped order.
 *   topk_ids [T, k] (each row: k distinct experts in [0, E))
 *   -> expert_offsets [E+1] (exclusive scan of group sizes, last = T*k),
 *      sorted_token [T*k] (compact token row at each grouped position; ascending inside a group),
 *      inv_perm [T*k] (grouped position of assignment j*k+s). */
moe_status moe_dispatch(const moe_config* cfg, const int32_t* topk_ids, int32_t T, int32_t* expert_offsets,
                        int32_t* sorted_token, int32_t* inv_perm, void* ws, void* stream);

/* Routed experts: y_sorted[pos] = SwiGLU expert e(pos) applied to token sorted_token[pos].
 *   expert_offsets [E+1], sorted_token [T*k] as produced by moe_dispatch
 *   -> y_sorted [T*k, H] bf16. The SwiGLU intermediate lives in the workspace (bf16). */
moe_status moe_expert_ffn(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                          const int32_t* expert_offsets, const int32_t* sorted_token, const moe_bf16* w_gate,
                          const moe_bf16* w_up, const moe_bf16* w_down, moe_bf16* y_sorted, void* ws, void* stream);

/* Routed experts whose weights are addressed through a slab table (paper Sec. 3.4.2: the expert cache hands out
 * equal-sized slots, one expert per slot, carved once from a single region, so nothing is allocated at run time). Same
 * operation as moe_expert_ffn, except that expert e's weights are read from slab_table[e]:
 *   slab_table [E]  DEVICE array of DEVICE pointers (16-byte aligned each); NULL = expert e is not resident.
 *                   A slab is [ w_gate_e (I x H) | w_up_e (I x H) | w_down_e (H x I) ] bf16, contiguous.
 *   -> y_sorted [T*k, H] bf16; the rows of a non-resident expert are written as zeros.
 *   -> missing [E+1] int32 (device): missing[0] = number of experts that have at least one row but no slab,
 *      missing[1 .. missing[0]] = their ids in ascending order (the rest is left untouched). The caller reads it
 *      after the stream has caught up, fetches those experts and calls again.
 * The slabs and the table must stay valid until the call's work on `stream` has finished. */
moe_status moe_expert_ffn_slabs(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx,
                                int32_t T, const int32_t* expert_offsets, const int32_t* sorted_token,
                                const moe_bf16* const* slab_table, moe_bf16* y_sorted, int32_t* missing, void* ws,
                                void* stream);

/* Shared experts: shared_out[j] = sum_s FFN_s(xt[j]) for the S always-on experts (requires cfg->S >= 1).
 *   -> shared_out [T, H] bf16. */
moe_status moe_shared_ffn(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                          const moe_bf16* ws_gate, const moe_bf16* ws_up, const moe_bf16* ws_down,
                          moe_bf16* shared_out, void* ws, void* stream);

/* Combine: out[j] = sum_s topk_w[j,s] * y_sorted[inv_perm[j*k+s]] (+ shared_out[j] when not NULL), fp32
 * accumulation in ascending s, rounded once to bf16.   -> out [T, H] bf16. */
moe_status moe_combine(const moe_config* cfg, const moe_bf16* y_sorted, const int32_t* inv_perm, const float* topk_w,
                       int32_t T, const moe_bf16* shared_out, moe_bf16* out, void* stream);

/* The whole layer in one enqueue sequence: route -> dispatch -> grouped gate/up + SwiGLU -> grouped down
 * (shared experts ride along as S extra groups that every token belongs to) -> combine.
 *   ws_gate/ws_up/ws_down may be NULL iff cfg->S == 0.
 *   topk_ids_opt [T,k] / topk_w_opt [T,k]: optional copies of the routing decision (NULL to skip).
 *   -> out [T, H] bf16. */
moe_status moe_layer_forward(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx, int32_t T,
                             const moe_bf16* w_router, const moe_bf16* w_gate, const moe_bf16* w_up,
                             const moe_bf16* w_down, const moe_bf16* ws_gate, const moe_bf16* ws_up,
                             const moe_bf16* ws_down, moe_bf16* out, int32_t* topk_ids_opt, float* topk_w_opt,
                             void* ws, void* stream);

/* The same layer for callers that cannot allocate and have no workspace to hand over: code under HIP graph capture,
 * tight serving loops (decode steps), harnesses that forbid hipMalloc. Identical to moe_layer_forward (same kernels,
 * bit-identical results) except that the scratch memory is a static device array inside the library,
 * MOE_STATIC_SCRATCH_BYTES per GPU, which each GPU the library runs on holds until the process ends. The call
 * allocates nothing; the array's device address is looked up once per GPU on the first call there.
 *   - MOE_ERR_WORKSPACE when moe_workspace_bytes(cfg) exceeds moe_static_scratch_bytes(); nothing is launched.
 *     (cfg->max_tokens sizes the need: a 64-token decode batch of a 128-expert top-8 layer with H 2048, I 768
 *     needs 3.2 MB, a pruned 704-token prefill of a 64-expert top-6 layer with two shared experts 39 MB.)
 *   - Every call on a GPU uses that GPU's one array, which keeps the last call's contents (no call needs it
 *     cleared): calls that overlap on one GPU, on different streams or from different threads, race. Order them on
 *     one stream. */
#define MOE_STATIC_SCRATCH_BYTES (64u << 20)
size_t moe_static_scratch_bytes(void);
moe_status moe_layer_forward_static(const moe_config* cfg, const moe_bf16* x, int32_t T_in, const int32_t* keep_idx,
                                    int32_t T, const moe_bf16* w_router, const moe_bf16* w_gate, const moe_bf16* w_up,
                                    const moe_bf16* w_down, const moe_bf16* ws_gate, const moe_bf16* ws_up,
                                    const moe_bf16* ws_down, moe_bf16* out, int32_t* topk_ids_opt, float* topk_w_opt,
                                    void* stream);

/* Stage timing, a measurement aid for benchmarks (not part of the layer; no passage of the paper defines it).
 * While enabled, every call of the layer (the fused one and the per-step ones) brackets each stage it runs with a
 * pair of HIP events recorded on the call's stream:
 *   stage 0 route, 1 dispatch, 2 grouped gate/up + SwiGLU, 3 grouped down, 4 combine (for moe_shared_ffn: the sum
 *   over the shared experts).
 * moe_stage_timing_enable(1) creates the events (this one call allocates); (0) destroys them.
 * moe_stage_timing_read waits for the LAST call's events and writes the elapsed milliseconds of each stage to
 * ms_out (HOST pointer, MOE_N_STAGES floats; stages the last call did not run read 0). Timing state is
 * process-wide: use it from one thread and one stream at a time. */
#define MOE_N_STAGES 5
moe_status moe_stage_timing_enable(int32_t enable);
moe_status moe_stage_timing_read(float* ms_out);

/* Index checking, a debugging aid (not part of the layer; no passage of the paper defines it).
 * By default the index arrays a caller hands over are trusted: keep_idx (entries in [0, T_in)), topk_ids of
 * moe_dispatch ([0, E)), expert_offsets ([0] == 0, non-decreasing, [E] == T*k) and sorted_token ([0, T)) of
 * moe_expert_ffn / moe_expert_ffn_slabs, inv_perm of moe_combine ([0, T*k)) and idx of moe_mean_pool
 * ([0, n_rows)). An entry out of range is then an out-of-bounds access on the device.
 * While checking is enabled, each of these calls first runs a small kernel over its index arrays on the call's
 * stream and WAITS for it (the call becomes synchronous and must not be made under stream capture); when an entry
 * is out of range it returns MOE_ERR_INDEX and launches nothing else. moe_index_checks_enable(1) allocates one word
 * of device and of pinned host memory, which are kept until (0). The state is process-wide: use it from one thread
 * and one stream at a time. */
moe_status moe_index_checks_enable(int32_t enable);

/* ---- Affinity-aware token compression (paper Sec. 3.2, Alg. 1, Eq. 1-5): the producer of keep_idx.
 *
 * Data flow: (1) the saliency of each of the N visual tokens is the attention it receives, averaged over the heads
 * and rescaled min-max to [0, 1] (all-equal saliency rescales to 0); (2) the floor(alpha N) most salient tokens form
 * the core and are always kept; (3) each token carries the set of experts it was routed to in the L pinned-prefix
 * layers, as an E-bit mask (ids outside [0, E) are ignored), and the core's masks are OR-ed into one target mask;
 * (4) a token's novelty is the share of its own experts that are missing from the target mask (0 for an empty
 * mask); (5) tokens outside the core score saliency - lambda * novelty; (6) the floor(beta N) - floor(alpha N)
 * best-scoring of them are kept as well. Every selection takes the largest values with ties to the lower token
 * index; both floors are taken on the double-precision products.
 *
 * All score arithmetic is fp32 with one rounding per operation and the head sum in head order, so the selection
 * is reproducible bit for bit on a CPU.
 *   attn            [n_heads, N] float  attention received by each visual token, per head
 *   prefix_topk_ids [L, N, k] int32     top-k ids of each visual token in the L pinned-prefix layers (moe_route's
 *                                       topk_ids of those layers, stacked)
 *   -> keep_idx [floor(beta N)] int32, ascending token indices (positions in the visual-token array)
 *   -> s_norm_opt [N] float (rescaled saliency) and delta_opt [N] float (novelty; 0 for core tokens): optional,
 *      NULL to skip
 * `ws` needs moe_compress_workspace_bytes(N, E) bytes, 256-byte aligned. Limits: 1 <= E <= 512, n_heads >= 1,
 * L >= 1, k >= 1, 0 <= alpha <= beta <= 1, N <= 2^22; otherwise MOE_ERR_SHAPE / MOE_ERR_UNSUPPORTED. N == 0 or
 * K_keep == 0 returns MOE_OK without launching (no output is written, the optional ones included). Inputs must be finite. The other conventions (device
 * pointers, alignment, asynchronous on `stream`, no allocation, errors by return value) are those stated at the
 * top of this file. */
size_t moe_compress_workspace_bytes(int32_t N, int32_t E);
/* A tuning aid (no passage of the paper defines it). The compressor has two code paths with identical results: up to
 * a token count it runs the sequentially dependent part of Alg. 1 in one workgroup (two launches per call), from
 * that count on as a chain of twelve small launches spread over many compute units (about 65 us per call on an
 * MI355X whatever the token count up to 2^17; one workgroup costs about 25 us + 6.7 ns per token). The call sets the
 * count from which the second path is taken (0: always) and returns the previous one; a negative argument only reads
 * it. The setting is process-wide; the default is where the two paths cost the same on an MI355X. */
int32_t moe_compress_wide_min_tokens(int32_t n);
moe_status moe_token_compress(const float* attn, int32_t n_heads, int32_t N, const int32_t* prefix_topk_ids, int32_t L,
                              int32_t k, int32_t E, double alpha, double beta, float lambda, int32_t* keep_idx,
                              float* s_norm_opt, float* delta_opt, void* ws, void* stream);

/* ---- Features and training target of the lookahead predictor (paper Sec. 3.3.1, Eq. 6-7; Sec. 3.3.2, Eq. 9).
 * The predictor input x_l = [h^(r)_l ; h^(h)_l ; h^(v)] (Eq. 7) is a concatenation: point the three calls' outputs
 * at consecutive pieces of one buffer.
 *
 * moe_mean_pool: out[c] = (1/K) sum_i rows[idx[i], c]   (Eq. 6, MP over the retained tokens I_keep; used for the
 *   hidden-state summary h^(h)_l and for the visual summary h^(v)).
 *     rows [n_rows, D] bf16, D a multiple of 8; idx [K] int32 rows to pool, or NULL = the first K rows (after
 *     compression the retained visual tokens are the leading rows of the stream); entries outside [0, n_rows) are
 *     undefined behaviour. -> out [D] float. fp32 accumulation in a fixed order (deterministic); ws needs
 *     moe_mean_pool_workspace_bytes(D) bytes, 256-byte aligned. K == 0 returns MOE_OK and writes nothing.
 * moe_routing_histogram: out[e] = share of the n given activations that went to expert e (the routing history
 *   h^(r)_l: pass the top-k ids of the recent layers, any shape, flattened). ids outside [0, E) are not counted;
 *   all zeros when nothing is counted. -> out [E] float. E <= 512.
 * moe_lookahead_target: g[e] = max over 1 <= d <= W of gamma^(d-1) [e is activated at layer l+d]   (Eq. 9).
 *     future_ids [W, n] int32: the ids activated at layers l+1 .. l+W (n = T*k each); 0 < gamma <= 1;
 *     gamma^(d-1) is the fp32 product of d-1 factors. -> g [E] float (0 for experts the window does not touch). */
/* moe_predictor_forward: the bottleneck MLP of Eq. 8 at inference and the ordered candidate list of Sec. 3.3.2:
 *     a1 = max(0, s1 * (W1 x) + t1),  a2 = max(0, s2 * (W2 a1) + t2),  y = Wo a2,  top = the B largest entries of y
 *   (BN-ReLU-Dropout at inference: dropout is the identity, batch normalisation the per-feature affine map
 *   s = gamma / sqrt(var + eps), t = beta - s * mean, folded by the caller). All fp32, row-major:
 *   x [D], W1 [D1, D], s1/t1 [D1], W2 [D2, D1], s2/t2 [D2], Wo [E, D2]; D, D1, D2 multiples of 4; E <= 512;
 *   0 <= B <= E. -> y [E] float, top [B] int32 (descending y, ties to the lower expert; NULL allowed when B == 0).
 *   ws: moe_predictor_workspace_bytes(D1, D2) bytes, 256-byte aligned. The weights come from training (Sec. 3.3.3),
 *   which is outside this library. */
size_t moe_predictor_workspace_bytes(int32_t D1, int32_t D2);
moe_status moe_predictor_forward(const float* x, int32_t D, const float* W1, const float* s1, const float* t1, int32_t D1,
                                 const float* W2, const float* s2, const float* t2, int32_t D2, const float* Wo,
                                 int32_t E, int32_t B, float* y, int32_t* top, void* ws, void* stream);
size_t moe_mean_pool_workspace_bytes(int32_t D);
moe_status moe_mean_pool(const moe_bf16* rows, int32_t n_rows, int32_t D, const int32_t* idx, int32_t K, float* out,
                         void* ws, void* stream);
moe_status moe_routing_histogram(const int32_t* ids, int64_t n, int32_t E, float* out, void* stream);
moe_status moe_lookahead_target(const int32_t* future_ids, int32_t W, int64_t n, int32_t E, float gamma, float* g,
                                void* stream);

/* ---- Slab-based dynamic expert cache with a transfer and a compute stream (paper Sec. 3.4.2: equal-sized slots,
 * one expert each, carved once from the cache region; insertion driven by the lookahead predictions; eviction
 * guarded by the classes Required / Speculative / Expired. Sec. 3.4.3: transfers run on their own stream, and a
 * miss stalls the compute stream only on the expert concerned).
 *
 * Host-side object; it allocates no device memory (the caller hands over the pool) and launches no kernels: it
 * issues host-to-device copies on the transfer stream and event waits. An expert is (layer, expert), 0 <= layer <
 * n_layers, 0 <= expert < E; its image is slab_bytes bytes of PINNED host memory laid out as moe_expert_ffn_slabs
 * expects. Classes: 0 Required (listed by the latest prediction or demanded; its layer has not yet executed in this
 * pass), 1 Speculative (was Required, dropped by a newer prediction, layer not yet executed; still protected),
 * 2 Expired (its layer has executed). Only Expired experts are evicted, lowest priority first, ties to the lowest
 * (layer, expert); free slabs are taken lowest index first. Not thread-safe: one host thread drives a cache.
 *
 * moe_cache_create   pool = n_slabs * slab_bytes bytes of device memory, 256-byte aligned; slab_bytes % 16 == 0.
 * moe_cache_predict  the predictor's list for the lookahead window: n experts (each at most once) with priorities.
 *                    Required experts that are not listed become Speculative; listed residents become Required
 *                    with the new priority; listed absent experts are fetched in descending priority (ties:
 *                    ascending (layer, expert)) while slabs can be had, else refused (counted).
 *                    -> started_out [2n] (layer, expert) pairs whose copy was issued, in issue order (optional),
 *                       n_started.
 * moe_cache_acquire  before a layer runs: `needed` = the experts its tokens were routed to. Resident ones are hits;
 *                    the others are fetched on demand (ascending expert, priority 0). Writes the layer's slab
 *                    table (HOST array of E device pointers, NULL for experts not needed: copy it to the device
 *                    and pass it to moe_expert_ffn_slabs) and makes comp_stream wait for exactly those experts'
 *                    copies. MOE_ERR_CACHE_FULL when a demanded expert cannot be placed (nothing is Expired):
 *                    the misses placed before it stay resident as Required with their copies in flight
 *                    (missed_out / n_missed list them), the hits stay Required, no table is written and
 *                    comp_stream waits for nothing; the caller retries after a moe_cache_layer_done has made
 *                    experts evictable, or gives the cache more slabs.
 *                    -> missed_out [n] (optional), n_missed.
 * moe_cache_layer_done  after the layer's kernels are enqueued on comp_stream: its experts become Expired; a copy
 *                    that later reuses one of their slabs first waits for this point of comp_stream.
 * moe_cache_query    slab (-1 = absent), class, priority of one expert.
 * moe_cache_stats    out6 = hits, misses, prefetches, evictions, refused prefetches, bytes copied. */
typedef struct moe_expert_cache moe_expert_cache;
moe_status moe_cache_create(int32_t n_layers, int32_t E, size_t slab_bytes, int32_t n_slabs, void* device_pool,
                            moe_expert_cache** out);
void moe_cache_destroy(moe_expert_cache* cache);
moe_status moe_cache_predict(moe_expert_cache* cache, const int32_t* layers, const int32_t* experts,
                             const float* priorities, int32_t n, const void* const* host_src, void* trans_stream,
                             int32_t* started_out, int32_t* n_started);
moe_status moe_cache_acquire(moe_expert_cache* cache, int32_t layer, const int32_t* needed, int32_t n,
                             const void* const* host_src, void* trans_stream, void* comp_stream, const void** table_out,
                             int32_t* missed_out, int32_t* n_missed);
moe_status moe_cache_layer_done(moe_expert_cache* cache, int32_t layer, void* comp_stream);
moe_status moe_cache_query(const moe_expert_cache* cache, int32_t layer, int32_t expert, int32_t* slab, int32_t* cls,
                           float* priority);
moe_status moe_cache_stats(const moe_expert_cache* cache, int64_t* out6);

#ifdef __cplusplus
}
#endif
#endif /* VISMOE_MOE_H */
