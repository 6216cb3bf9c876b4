// Grouped expert FFN (paper Sec. 2.1: the sparse MoE feed-forward block; Table 2: per-expert weights; Sec.
// 3.4.1: shared experts run for every token). Two bf16 MFMA kernels, each in two modes:
//   MODE 0  hm[pos, i] = silu(x_row(pos) . Wg[g][i]) * (x_row(pos) . Wu[g][i])     rows gathered through sorted_token
//   MODE 1  y[pos, h]  = hm[pos] . Wd[g][h]
// Both are "NT" products: operand rows are contiguous along the contraction, so fragments load as 16-byte
// pieces. The MFMA is issued with the WEIGHT fragment as its first operand: the accumulator then holds, per
// lane, one token and 16 (or 4) consecutive output columns, which store as whole 16-byte words.
//
//  * ffn_tile_kernel   : 256 tokens x 256 weight rows per workgroup (4 waves of 128 x 128), K staged through two
//                        LDS stages in 64-wide slabs by direct-to-LDS loads (XOR-swizzled 16-byte chunks). For
//                        compute-bound shapes (prefill).
//  * ffn_skinny_kernel : weight-streaming; every wave owns 32 weight rows and feeds them from global memory
//                        straight into MFMA registers, tokens in 16-row fragments. For small ragged groups
//                        (decode, pruned prefill) where each weight byte is used a few times only.
#include "common.h"

namespace vismoe {

// ------------------------------------------------------------------------------------------------ tiled kernel
// Workgroup = 256 threads = 4 waves (one per SIMD), tile = 256 tokens x 256 weight rows (MODE 0: 128 gate + 128
// up rows, i.e. 128 output columns), K in 64-wide slabs. Wave (wm, wn) owns a 128 x 128 sub-tile: 4 token
// fragments x 4 weight fragments of 32 rows, 16 accumulators of 16 registers (the 256 accumulator registers live
// in AGPRs). The square wave tile keeps LDS traffic (128 B/clk/CU, shared by fragment reads and incoming slabs)
// below the MFMA time: 8 fragment reads feed 16 MFMAs.
//
// LDS is a ring of five 32 KB granules; a granule is the token half or the weight half of one K slab
// ([256 rows][64] bf16, rows of 128 B), so slab i occupies granules 2i and 2i+1 (ring slots (2i) % 5 and
// (2i+1) % 5) and three further granules are in flight while it is multiplied: one 64 KB slab in flight per CU is
// not enough to cover the L2/HBM latency. Granules arrive by direct-to-LDS loads (global_load_lds_dwordx4: lane l
// of a wave lands at base + 16*l, so one instruction fills 8 rows x 128 B). Rows are fetched in 128-byte pieces on
// purpose: with 64-byte pieces the L2 delivers about half the bandwidth (measured 16 vs 33 TB/s for L2-resident
// data). The 16-byte chunks of a row are XOR-swizzled with (row >> 1) & 7 by choosing which global chunk each
// lane fetches, which keeps the ds_read_b128 fragment reads free of bank conflicts.
//
// Schedule of one wave for slab i (4 k-steps of 16; fragments of the next k-step are read while the current one is
// multiplied): k-steps 0..2 | this wave's reads of slab i are complete and slab i+1 has landed: barrier | start
// refilling the granules of slab i | read the first fragments of slab i+1 | k-step 3. The loads of the following
// slabs are issued four per k-step, evenly, so that they never pile up in front of the wave's MFMAs.
// Token fragments past the end of the group are not multiplied (NT = number of live fragments of the wave).
constexpr int BM = kTileM;   // tokens per tile
constexpr int BK = 64;
static_assert(BM == 256, "tile map granularity and kernel tile must agree");

typedef __attribute__((address_space(3))) bf16_t lds_bf16;
typedef const __attribute__((address_space(3))) bf16x8* lds_frag_ptr;
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// LDS row m of a 32-row weight fragment holds weight row frag_perm(m): accumulator register i of lane
// (token, q) is then output column 16*q + i of the fragment.
__device__ __forceinline__ int frag_perm(int m) { return 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3); }

constexpr int kGranuleElems = 256 * BK;     // one granule: 256 rows x 64 bf16 = 32 KB

struct TileCtx {
    const bf16_t* a_base;     // MODE 0: x, MODE 1: hm
    const bf16_t* b_base[2];  // weight matrix feeding each half of the stage (MODE 0: gate / up; MODE 1: down twice)
    int a_off[8];             // element offsets of this lane's 8 token rows, already at its swizzled 16-byte chunk
    int b_off[8];             // ... and of its 8 weight rows
    int lds_blk;              // element offset of the first 1 KB block this wave fills (then +4 KB steps)
    int a_row, b_row[4];      // fragment row offsets (elements) for the reads; token fragments are 32 rows apart
    int key, q;
    int k_last;
};

struct Frags {
    bf16x8 x[4];              // token fragments
    bf16x8 w[4];              // weight fragments
};

// Half (4 of the 8 loads per lane) of the token rows of one K slab -> granule `wr`.
template <int HALF>
__device__ __forceinline__ void issue_tokens(lds_bf16* __restrict__ wr, int k0, const TileCtx& c) {
#pragma unroll
    for (int j = 4 * HALF; j < 4 * HALF + 4; ++j)
        __builtin_amdgcn_global_load_lds((gptr_t)(c.a_base + c.a_off[j] + k0), (lptr_t)(wr + c.lds_blk + j * 2048), 16, 0,
                                         0);
}
// Half of the weight rows of one K slab -> granule `wr`.
template <int HALF>
__device__ __forceinline__ void issue_weights(lds_bf16* __restrict__ wr, int k0, const TileCtx& c) {
#pragma unroll
    for (int j = 4 * HALF; j < 4 * HALF + 4; ++j)
        __builtin_amdgcn_global_load_lds((gptr_t)(c.b_base[j >> 2] + c.b_off[j] + k0), (lptr_t)(wr + c.lds_blk + j * 2048),
                                         16, 0, 0);
}

template <int NT>
__device__ __forceinline__ void read_frags(const lds_bf16* __restrict__ ga, const lds_bf16* __restrict__ gb, int ks,
                                           const TileCtx& c, Frags& f) {
    const int ch = ((ks * 2 + c.q) ^ c.key) * 8;
#pragma unroll
    for (int t = 0; t < NT; ++t) f.x[t] = *reinterpret_cast<lds_frag_ptr>(ga + c.a_row + t * 32 * BK + ch);
#pragma unroll
    for (int j = 0; j < 4; ++j) f.w[j] = *reinterpret_cast<lds_frag_ptr>(gb + c.b_row[j] + ch);
}

template <int NT>
__device__ __forceinline__ void mma_step(const Frags& f, floatx16 (&acc)[4][4]) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[j], f.x[t], acc[t][j], 0, 0, 0);
}

// Pin the instruction order of a k-step: 16 MFMAs with the 8 fragment reads and 4 slab loads spread between them.
// Left alone, the scheduler sinks the reads to just before their first use, where their latency is exposed: there
// is no second wave on the SIMD to hide it.
template <int NT>
__device__ __forceinline__ void pin_order() {
    if (NT == 0) return;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                   // DS read
        if (n & 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);        // VMEM read (direct-to-LDS load)
    }
}

// One slab i, held in granules (ca, cb). On entry f0 holds its k-step 0 fragments; (na, nb) hold slab i+1, `fa` is
// the fifth granule. The loads are spread evenly over the k-steps (4 per lane each) so that they never queue up
// in front of the MFMAs of the wave:
//     k-step 0: second half of the weights of slab i+1 -> nb      k-step 1, 2: tokens of slab i+2 -> fa
//     k-step 3 (after the barrier, when every wave is done with slab i): first half of the weights of slab i+2 -> ca
// The __restrict__ qualifiers matter: they let the compiler prove that fragment reads do not touch the granules
// being filled, so it does not wait for the loads in flight before every LDS read.
template <int NT>
__device__ __forceinline__ void slab_step(lds_bf16* __restrict__ ca, lds_bf16* __restrict__ cb,
                                          lds_bf16* __restrict__ na, lds_bf16* __restrict__ nb,
                                          lds_bf16* __restrict__ fa, int k1, int k2, const TileCtx& c, Frags& f0,
                                          Frags& f1, floatx16 (&acc)[4][4]) {
    issue_weights<1>(nb, k1, c);
    if (NT > 0) read_frags<NT>(ca, cb, 1, c, f1);
    mma_step<NT>(f0, acc);
    pin_order<NT>();
    __builtin_amdgcn_sched_barrier(0);
    issue_tokens<0>(fa, k2, c);
    if (NT > 0) read_frags<NT>(ca, cb, 2, c, f0);
    mma_step<NT>(f1, acc);
    pin_order<NT>();
    __builtin_amdgcn_sched_barrier(0);
    issue_tokens<1>(fa, k2, c);
    if (NT > 0) read_frags<NT>(ca, cb, 3, c, f1);
    mma_step<NT>(f0, acc);
    pin_order<NT>();
    __builtin_amdgcn_sched_barrier(0);
    // this wave's reads of (ca, cb) have returned: lgkmcnt(0); its share of slab i+1 has landed: all loads but the
    // newest 8 per lane (the tokens of slab i+2): vmcnt(8)
    __builtin_amdgcn_s_waitcnt(0x0078);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    issue_weights<0>(ca, k2, c);
    if (NT > 0) read_frags<NT>(na, nb, 0, c, f0);
    mma_step<NT>(f1, acc);
    pin_order<NT>();
    __builtin_amdgcn_sched_barrier(0);
}

// Epilogue of a wave's 128 x 128 sub-tile: lane = token r of fragment t; registers i = output columns 16*q + i of
// fragment j. MODE 0 applies SwiGLU to the gate (j = 0, 1) and up (j = 2, 3) sums of the same columns.
template <int MODE, int NT, int NJ = 4>
__device__ __forceinline__ void store_acc(const GemmParams& p, const floatx16 (&acc)[4][4], int m_first, int m_end,
                                          int n_first, int q) {
    const int r = threadIdx.x & 31;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int row = m_first + t * 32 + r;
        if (row >= m_end) continue;
        bf16_t* crow = p.C + (size_t)row * p.ldc;
        if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = n_first + j * 32 + 16 * q;
                if (col >= p.N) continue;
                uint32_t o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float h0 = silu_f(acc[t][j][2 * e]) * acc[t][j + 2][2 * e];
                    const float h1 = silu_f(acc[t][j][2 * e + 1]) * acc[t][j + 2][2 * e + 1];
                    o[e] = pack_bf16x2(h0, h1);
                }
                *reinterpret_cast<uint4*>(crow + col) = make_uint4(o[0], o[1], o[2], o[3]);
                *reinterpret_cast<uint4*>(crow + col + 8) = make_uint4(o[4], o[5], o[6], o[7]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int col = n_first + j * 32 + 16 * q;
                if (col >= p.N) continue;
                uint32_t o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = pack_bf16x2(acc[t][j][2 * e], acc[t][j][2 * e + 1]);
                *reinterpret_cast<uint4*>(crow + col) = make_uint4(o[0], o[1], o[2], o[3]);
                *reinterpret_cast<uint4*>(crow + col + 8) = make_uint4(o[4], o[5], o[6], o[7]);
            }
        }
    }
}

template <int MODE, int NT>
__device__ __forceinline__ void tile_body(const GemmParams& p, const TileCtx& c, lds_bf16* G0, lds_bf16* G1, lds_bf16* G2,
                                          lds_bf16* G3, lds_bf16* G4, int m_first, int m_end, int n_first) {
    floatx16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // Every slab step issues exactly 16 loads per lane (past the end of K it re-fetches the last slab into free
    // granules), so the main loop body has no branches and the loads in flight are the same on every path: with
    // conditional steps the compiler can no longer tell which loads are still in flight and waits for all of them
    // before each LDS read.
    const int KT = p.K / BK;
    auto slab_k = [&](int i) { return min(i * BK, c.k_last); };
    // (the weight halves of slab 0 and half of slab 1's were issued by the caller, ahead of the token gather)
    issue_tokens<0>(G0, 0, c);
    issue_tokens<1>(G0, 0, c);
    issue_tokens<0>(G2, slab_k(1), c);
    issue_tokens<1>(G2, slab_k(1), c);
    __builtin_amdgcn_s_waitcnt(0x0070 | 0x0008);   // vmcnt(8): slab 0 has landed, the tokens of slab 1 may be in flight
    __builtin_amdgcn_s_barrier();
    Frags f0, f1;
    if (NT > 0) read_frags<NT>(G0, G1, 0, c, f0);
    // slab i sits in ring slots (2i) % 5 and (2i+1) % 5: the pattern repeats every five slabs
#define VISMOE_SLAB(CA, CB, NA, NB, FA, I) slab_step<NT>(CA, CB, NA, NB, FA, slab_k((I) + 1), slab_k((I) + 2), c, f0, f1, acc)
    int i = 0;
    for (; i + 5 <= KT; i += 5) {
        VISMOE_SLAB(G0, G1, G2, G3, G4, i);
        VISMOE_SLAB(G2, G3, G4, G0, G1, i + 1);
        VISMOE_SLAB(G4, G0, G1, G2, G3, i + 2);
        VISMOE_SLAB(G1, G2, G3, G4, G0, i + 3);
        VISMOE_SLAB(G3, G4, G0, G1, G2, i + 4);
    }
    const int left = KT - i;
    if (left > 0) VISMOE_SLAB(G0, G1, G2, G3, G4, i);
    if (left > 1) VISMOE_SLAB(G2, G3, G4, G0, G1, i + 1);
    if (left > 2) VISMOE_SLAB(G4, G0, G1, G2, G3, i + 2);
    if (left > 3) VISMOE_SLAB(G1, G2, G3, G4, G0, i + 3);
#undef VISMOE_SLAB
    __builtin_amdgcn_s_waitcnt(0x0070);      // no load may still be writing LDS when the workgroup releases it

    store_acc<MODE, NT>(p, acc, m_first, m_end, n_first, c.q);
}

// ---------------------------------------------------------------------------------------------- tall work units
// A group of at most kTallM = 128 rows would fill an M-tile less than half while its workgroups still stream a full
// tile's weight rows. Such groups are computed as tall units instead: 128 tokens against 256 output columns (MODE 0:
// 256 gate + 256 up weight rows, half as many workgroups per group as M-tiles, the token rows read half as often;
// MODE 1: 256 down rows, as many workgroups as M-tiles but without the dead half of the token tile), each weight row
// still read once. The four waves sit side by side: every wave multiplies all 128 tokens with its own weight rows
// (MODE 0: 64 gate + 64 up, the same 4 x 4 fragments per wave as in an M-tile; MODE 1: 64 down rows, 4 x 2). A wave's weight rows are its private business (it requests them and is the only one to
// read them), the token rows are shared. LDS = ten 16 KB blocks: tokens of the slab being multiplied and of the next
// one, and per wave its weight rows of the two slabs. One barrier per slab: behind it every wave has finished with
// the current blocks and the next slab has landed, so the blocks just freed are requested again at once (slab i + 2)
// and stay in flight for a whole slab time.
constexpr int kTallBlockElems = kTallM * BK;      // 16 KB

struct TallCtx {
    const bf16_t* a_base;
    const bf16_t* b_base[2];   // the matrix feeding fragments 0, 1 and 2, 3 of the wave (MODE 0: gate / up)
    int a_off[4];              // element offsets of this lane's 4 token rows (rows 32 wave + 8 j + lane / 8), swizzled chunk
    int b_off[16];             // ... and of its 16 weight rows (rows 8 j + lane / 8 of the wave's block)
    int tok_blk;               // element offset of the 1 KB pieces this wave fills in a token block
    int a_row, b_row[4];
    int key, q, k_last;
};

__device__ __forceinline__ void tall_issue_tokens(lds_bf16* __restrict__ tok, int k0, const TallCtx& c) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
        __builtin_amdgcn_global_load_lds((gptr_t)(c.a_base + c.a_off[j] + k0), (lptr_t)(tok + c.tok_blk + j * 512), 16, 0, 0);
}
// NJ = weight fragments per wave: 4 in MODE 0 (64 gate + 64 up rows), 2 in MODE 1 (64 down rows).
// A tall unit is the only reader of its weight rows (one row block per group, one unit per column range), so in the
// gate/up launch they are requested with the non-temporal hint and do not displace the token rows and the
// intermediate from the caches: 160 -> 148 us on the pruned prefill. (In the down launch the same hint cost 4 us.)
constexpr int kCachePolicyNT = 2;           // the "nt" bit of a load's cache-policy operand
template <int NJ>
__device__ __forceinline__ void tall_issue_weights(lds_bf16* __restrict__ wts, int k0, const TallCtx& c) {
#pragma unroll
    for (int j = 0; j < 4 * NJ; ++j)
        __builtin_amdgcn_global_load_lds((gptr_t)(c.b_base[j / (2 * NJ)] + c.b_off[j] + k0), (lptr_t)(wts + j * 512), 16, 0,
                                         NJ == 4 ? kCachePolicyNT : 0);
}

// The MFMAs of token fragments [T0, T1) of a k-step.
template <int T0, int T1, int NJ>
__device__ __forceinline__ void mma_tall(const Frags& f, floatx16 (&acc)[4][4]) {
#pragma unroll
    for (int t = T0; t < T1; ++t)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[j], f.x[t], acc[t][j], 0, 0, 0);
}

template <int NT, int NJ>
__device__ __forceinline__ void tall_read(const lds_bf16* __restrict__ tok, const lds_bf16* __restrict__ wts, int ks,
                                          const TallCtx& c, Frags& f) {
    const int ch = ((ks * 2 + c.q) ^ c.key) * 8;
#pragma unroll
    for (int t = 0; t < NT; ++t) f.x[t] = *reinterpret_cast<lds_frag_ptr>(tok + c.a_row + t * 32 * BK + ch);
#pragma unroll
    for (int j = 0; j < NJ; ++j) f.w[j] = *reinterpret_cast<lds_frag_ptr>(wts + c.b_row[j] + ch);
}

// Instruction order of a tall k-step (or half of one): MFMAs with `reads` fragment reads and `loads` direct-to-LDS
// loads spread between them.
template <int MFMAS, int READS, int LOADS>
__device__ __forceinline__ void pin_tall() {
    if (MFMAS == 0) return;
    constexpr int M = MFMAS > 0 ? MFMAS : 1;
    constexpr int RP = (READS + M - 1) / M, LP = (LOADS + M - 1) / M;                    // per MFMA
#pragma unroll
    for (int n = 0; n < MFMAS; ++n) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                             // MFMA
        if (RP > 0 && n * RP < READS) __builtin_amdgcn_sched_group_barrier(0x100, RP, 0);    // DS read
        if (LP > 0 && n * LP < LOADS) __builtin_amdgcn_sched_group_barrier(0x020, LP, 0);    // direct-to-LDS load
    }
}

// One slab i held in (tc, wc); slab i + 1 has been requested into (tn, wn). On entry f0 holds the k-step 0 fragments.
// The wave's own weight block is requested again (slab i + 2) as soon as the wave has read its last fragments from
// it, before the barrier, so that loads are in flight while the waves wait for each other; the token block is shared
// and follows behind the barrier.
template <int NT, int NJ>
__device__ __forceinline__ void tall_step(lds_bf16* __restrict__ tc, lds_bf16* __restrict__ wc, lds_bf16* __restrict__ tn,
                                          lds_bf16* __restrict__ wn, int k2, const TallCtx& c, Frags& f0, Frags& f1,
                                          floatx16 (&acc)[4][4]) {
    if (NT > 0) tall_read<NT, NJ>(tc, wc, 1, c, f1);
    mma_tall<0, NT, NJ>(f0, acc);
    pin_tall<NJ * NT, NJ + NT, 0>();
    __builtin_amdgcn_sched_barrier(0);
    if (NT > 0) tall_read<NT, NJ>(tc, wc, 2, c, f0);
    mma_tall<0, NT, NJ>(f1, acc);
    pin_tall<NJ * NT, NJ + NT, 0>();
    __builtin_amdgcn_sched_barrier(0);
    if (NT > 0) tall_read<NT, NJ>(tc, wc, 3, c, f1);
    mma_tall<0, NT / 2, NJ>(f0, acc);
    pin_tall<NJ * NT / 2, NJ + NT, 0>();
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): this wave's reads of wc have returned
    tall_issue_weights<NJ>(wc, k2, c);
    mma_tall<NT / 2, NT, NJ>(f0, acc);
    pin_tall<NJ * NT / 2, 0, 4 * NJ>();
    __builtin_amdgcn_sched_barrier(0);
    // slab i + 1 has landed (this wave's share): all loads but the 4 NJ just issued
    __builtin_amdgcn_s_waitcnt(NJ == 4 ? 0x4F70 : 0x0F78);      // vmcnt(16) / vmcnt(8)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    tall_issue_tokens(tc, k2, c);
    if (NT > 0) tall_read<NT, NJ>(tn, wn, 0, c, f0);
    mma_tall<0, NT, NJ>(f1, acc);
    pin_tall<NJ * NT, NJ + NT, 4>();
    __builtin_amdgcn_sched_barrier(0);
}

template <int MODE, int NT>
__device__ __forceinline__ void tall_body(const GemmParams& p, const TallCtx& c, lds_bf16* T0, lds_bf16* T1, lds_bf16* W0,
                                          lds_bf16* W1, int m0, int m_end, int n_first) {
    constexpr int NJ = (MODE == 0) ? 4 : 2;
    floatx16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    const int KT = p.K / BK;
    auto slab_k = [&](int i) { return min(i * BK, c.k_last); };
    // every step requests one slab (past the end of K the last one again), so the loads in flight behind a wait are
    // the same on every path
    tall_issue_tokens(T0, 0, c);
    tall_issue_weights<NJ>(W0, 0, c);
    tall_issue_tokens(T1, slab_k(1), c);
    tall_issue_weights<NJ>(W1, slab_k(1), c);
    // slab 0 has landed, slab 1 (4 + 4 NJ loads) may be in flight: vmcnt(20) / vmcnt(12)
    __builtin_amdgcn_s_waitcnt(NJ == 4 ? 0x4074 : 0x007C);
    __builtin_amdgcn_s_barrier();
    Frags f0, f1;
    if (NT > 0) tall_read<NT, NJ>(T0, W0, 0, c, f0);
    int i = 0;
    for (; i + 2 <= KT; i += 2) {
        tall_step<NT, NJ>(T0, W0, T1, W1, slab_k(i + 2), c, f0, f1, acc);
        tall_step<NT, NJ>(T1, W1, T0, W0, slab_k(i + 3), c, f0, f1, acc);
    }
    if (i < KT) tall_step<NT, NJ>(T0, W0, T1, W1, slab_k(i + 2), c, f0, f1, acc);
    __builtin_amdgcn_s_waitcnt(0x0070);      // no load may still be writing LDS when the workgroup releases it
    store_acc<MODE, NT, NJ>(p, acc, m0, m_end, n_first, c.q);
}

template <int MODE>
__device__ __forceinline__ void tall_run(int nt, const GemmParams& p, const TallCtx& c, lds_bf16* T0, lds_bf16* T1,
                                         lds_bf16* W0, lds_bf16* W1, int m0, int m_end, int n_first) {
    if (nt == 4) tall_body<MODE, 4>(p, c, T0, T1, W0, W1, m0, m_end, n_first);
    else if (nt == 2) tall_body<MODE, 2>(p, c, T0, T1, W0, W1, m0, m_end, n_first);
    else tall_body<MODE, 0>(p, c, T0, T1, W0, W1, m0, m_end, n_first);
}

// One tall unit: column unit n_unit of the row block tm = (group, first row, end row).
template <int MODE>
__device__ __forceinline__ void tall_unit(const GemmParams& p, const int4 tm, int n_unit, lds_bf16* G0, lds_bf16* G1,
                                          lds_bf16* G2, lds_bf16* G3, lds_bf16* G4) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, q = lane >> 5;
    const int g = tm.x, m0 = tm.y, m_end = tm.z;            // 1 <= m_end - m0 <= kTallM
    constexpr int BNU = 256;                                // output columns per unit
    constexpr int BNW = BNU / 4;                            // ... per wave: 64 (MODE 0: 64 gate + 64 up weight rows)
    constexpr int NJ = (MODE == 0) ? 4 : 2;                 // weight fragments per wave
    const int n0 = n_unit * BNU;
    const int K = p.K, N = p.N;
    const bf16_t *b0, *b1;
    if (!group_weights(p, g, MODE == 0, b0, b1)) {
        // expert not resident: its part of the output is defined as zero (the caller is told which experts)
        const int rows = m_end - m0, cols = min(BNU, N - n0);
        for (int i = tid; i < rows * (cols / 8); i += 256) {
            const int rr = i / (cols / 8), cc = (i - rr * (cols / 8)) * 8;
            *reinterpret_cast<uint4*>(p.C + (size_t)(m0 + rr) * p.ldc + n0 + cc) = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    TallCtx c;
    c.q = q;
    c.key = (r >> 1) & 7;
    c.k_last = K - BK;
    c.a_base = p.A;
    c.b_base[0] = b0;
    c.b_base[1] = b1;
    c.tok_blk = wave * (32 * BK);
    const int lrow = lane >> 3, lpos = lane & 7;
    const int n_first = n0 + wave * BNW;                    // first output column of this wave
    // weight rows of the wave's private block: block row m = 32 f + rr holds, for fragment f,
    //   MODE 0: f = 0, 1 gate rows and f = 2, 3 up rows of output columns n_first + 32 (f & 1) + frag_perm(rr)
    //   MODE 1: f = 0, 1 down rows n_first + 32 f + frag_perm(rr)
    // Columns past N are clamped and never stored.
#pragma unroll
    for (int j = 0; j < 4 * NJ; ++j) {
        const int rr = 8 * (j & 3) + lrow, f = j >> 2;
        const int chunk = (lpos ^ ((rr >> 1) & 7)) * 8;
        const int col = (MODE == 0) ? n_first + 32 * (f & 1) + frag_perm(rr) : n_first + 32 * f + frag_perm(rr);
        c.b_off[j] = min(col, N - 1) * K + chunk;
    }
    // token rows 32 wave + 8 j + lrow of the block; rows past the end of the group repeat its last row
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int rr = 8 * j + lrow;
        const int chunk = (lpos ^ ((rr >> 1) & 7)) * 8;
        int arow = min(m0 + 32 * wave + rr, m_end - 1);
        if (MODE == 0) {
            arow = p.sorted_token[arow];
            if (p.keep_idx) arow = p.keep_idx[arow];
        }
        c.a_off[j] = arow * p.lda + chunk;
    }
    c.a_row = r * BK;
#pragma unroll
    for (int j = 0; j < NJ; ++j) c.b_row[j] = (32 * j + r) * BK;
    // LDS blocks. The compiler lets a fragment read overtake the loads in flight only when it can tell that they
    // touch different __shared__ arrays, so for every wave the blocks of one slab parity (tokens and its weights) and
    // those of the other parity must lie in different arrays, with pointers that are constants of the code path:
    //   G0 = [tokens even | wave 0 even]   G1 = [tokens odd | wave 0 odd]   G2 = [wave 1 even | wave 2 even]
    //   G3 = [wave 1 odd | wave 3 odd]     G4 = [wave 3 even | wave 2 odd]
    constexpr int HB = kTallBlockElems;
    // a wave whose columns all lie past N (last, ragged unit) multiplies nothing but keeps loading and synchronising;
    // one or three live token fragments run as two or four (the dead rows repeat the last live row)
    const int live = (m_end - m0 + 31) >> 5;
    const int nt = __builtin_amdgcn_readfirstlane(n_first >= N ? 0 : (live <= 2 ? 2 : 4));
    switch (wave) {
        case 0: tall_run<MODE>(nt, p, c, G0, G1, G0 + HB, G1 + HB, m0, m_end, n_first); break;
        case 1: tall_run<MODE>(nt, p, c, G0, G1, G2, G3, m0, m_end, n_first); break;
        case 2: tall_run<MODE>(nt, p, c, G0, G1, G2 + HB, G4 + HB, m0, m_end, n_first); break;
        default: tall_run<MODE>(nt, p, c, G0, G1, G4, G3 + HB, m0, m_end, n_first); break;
    }
}

template <int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void ffn_tile_kernel(const GemmParams p) {
    __shared__ __attribute__((aligned(1024))) bf16_t g0[kGranuleElems];
    __shared__ __attribute__((aligned(1024))) bf16_t g1[kGranuleElems];
    __shared__ __attribute__((aligned(1024))) bf16_t g2[kGranuleElems];
    __shared__ __attribute__((aligned(1024))) bf16_t g3[kGranuleElems];
    __shared__ __attribute__((aligned(1024))) bf16_t g4[kGranuleElems];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, q = lane >> 5;

    // Workgroups are spread over the 8 XCDs round-robin by the hardware; give each XCD one contiguous run of
    // the (group-major) list of M-tile work and one of the list of tall units, so that tiles sharing weights or
    // tokens share an L2 and both kinds of work are spread evenly over the XCDs.
    const int n_mt = p.n_tiles[0];
    const int n_work = n_mt * p.n_ntiles, n_tall_work = p.n_tiles[1] * p.n_tall;
    const int per_xcd = (n_work + 7) >> 3, per_xcd_tall = (n_tall_work + 7) >> 3;
    int slot = blockIdx.x >> 3;
    if (slot >= per_xcd + per_xcd_tall) return;
    // MODE 1 walks every XCD's run backwards: the rows of the intermediate that this XCD wrote last (in MODE 0, which
    // walks the same runs forwards) are read first, while they are still in its L2.
    if (MODE == 1) slot = per_xcd + per_xcd_tall - 1 - slot;
    lds_bf16* const G0 = (lds_bf16*)g0; lds_bf16* const G1 = (lds_bf16*)g1; lds_bf16* const G2 = (lds_bf16*)g2;
    lds_bf16* const G3 = (lds_bf16*)g3; lds_bf16* const G4 = (lds_bf16*)g4;
    // an XCD works through its tall units first (they take longest), then through its M-tiles (MODE 1: the other
    // way round)
    if (slot < per_xcd_tall) {
        const int unit = (blockIdx.x & 7) * per_xcd_tall + slot;
        if (unit >= n_tall_work) return;
        const int blk = unit / p.n_tall;
        tall_unit<MODE>(p, p.tile_map[n_mt + blk], unit - blk * p.n_tall, G0, G1, G2, G3, G4);
        return;
    }
    const int work = (blockIdx.x & 7) * per_xcd + slot - per_xcd_tall;
    if (work >= n_work) return;
    const int m_tile = work / p.n_ntiles, n_tile = work - m_tile * p.n_ntiles;
    const int4 tm = p.tile_map[m_tile];
    if (tm.w) {
        // a tall row block owns as many work slots as an M-tile and uses the first n_tall of them
        if (n_tile < p.n_tall) tall_unit<MODE>(p, tm, n_tile, G0, G1, G2, G3, G4);
        return;
    }
    const int g = tm.x, m0 = tm.y, m_end = tm.z;
    constexpr int BN = (MODE == 0) ? 128 : 256;     // output columns per tile
    const int n0 = n_tile * BN;
    const int K = p.K, N = p.N;
    const bf16_t *b0, *b1;
    if (!group_weights(p, g, MODE == 0, b0, b1)) {
        // expert not resident: its part of the output is defined as zero (the caller is told which experts)
        const int rows = min(BM, m_end - m0), cols = min(BN, N - n0);
        for (int i = tid; i < rows * (cols / 8); i += 256) {
            const int rr = i / (cols / 8), cc = (i - rr * (cols / 8)) * 8;
            *reinterpret_cast<uint4*>(p.C + (size_t)(m0 + rr) * p.ldc + n0 + cc) = make_uint4(0, 0, 0, 0);
        }
        return;
    }

    TileCtx c;
    c.q = q;
    c.key = (r >> 1) & 7;
    c.k_last = K - BK;
    c.lds_blk = wave * 512;
    c.a_base = p.A;
    const int lrow = lane >> 3, lpos = lane & 7;
    // load j of a slab fills the 1 KB block (4 j + wave) of each half of the stage = rows 32 j + 8 wave + lrow
    const int rr = wave * 8 + lrow;              // row within a 32-row fragment
    const int chunk = (lpos ^ ((rr >> 1) & 7)) * 8;
    // Order matters for the latency of a tile's start: the token-row lookups go out first, then the weight halves
    // of the first two slabs (which depend on nothing but the tile descriptor), and only then the dependent part
    // of the gather.
    int arow[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        arow[j] = min(m0 + 32 * j + rr, m_end - 1);
        if (MODE == 0) arow[j] = p.sorted_token[arow[j]];
    }
    // weight rows: stage rows [0,128) and [128,256) are the two halves (MODE 0: gate / up rows of the same 128
    // columns; MODE 1: columns [0,128) / [128,256) of the tile). Rows past N are clamped and never stored.
    c.b_base[0] = b0;
    c.b_base[1] = b1;
    const int pr = frag_perm(rr);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int col = (MODE == 0) ? n0 + 32 * (j & 3) + pr : n0 + 32 * j + pr;
        c.b_off[j] = min(col, N - 1) * K + chunk;
    }
    issue_weights<0>(G1, 0, c);
    issue_weights<1>(G1, 0, c);
    issue_weights<0>(G3, min(BK, c.k_last), c);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (MODE == 0 && p.keep_idx) arow[j] = p.keep_idx[arow[j]];
        c.a_off[j] = arow[j] * p.lda + chunk;
    }
    c.a_row = (wm * 128 + r) * BK;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (MODE == 0) c.b_row[j] = ((j >> 1) * 128 + wn * 64 + (j & 1) * 32 + r) * BK;   // j = 0,1 gate; 2,3 up
        else c.b_row[j] = (wn * 128 + j * 32 + r) * BK;
    }

    const int m_first = m0 + wm * 128;
    const int n_first = n0 + wn * ((MODE == 0) ? 64 : 128);
    const int live = m_end - m_first;            // rows of this wave's token slab that exist
    const int nt = __builtin_amdgcn_readfirstlane(live <= 0 ? 0 : min(4, (live + 31) >> 5));
    switch (nt) {
        case 4: tile_body<MODE, 4>(p, c, G0, G1, G2, G3, G4, m_first, m_end, n_first); break;
        case 3: tile_body<MODE, 3>(p, c, G0, G1, G2, G3, G4, m_first, m_end, n_first); break;
        case 2: tile_body<MODE, 2>(p, c, G0, G1, G2, G3, G4, m_first, m_end, n_first); break;
        case 1: tile_body<MODE, 1>(p, c, G0, G1, G2, G3, G4, m_first, m_end, n_first); break;
        default: tile_body<MODE, 0>(p, c, G0, G1, G2, G3, G4, m_first, m_end, n_first); break;
    }
}

// ----------------------------------------------------------------------------------------------- skinny kernel
// Workgroup = (column chunk, group); a wave owns 2 weight fragments of 16 rows of ONE weight matrix:
//   MODE 0: 64 hm columns per workgroup. Waves 0, 1 hold the gate rows of columns [0,32) and [32,64) of the chunk,
//           waves 2, 3 the up rows of the same columns; the up waves hand their sums to the gate waves through LDS,
//           which apply SwiGLU and store. A wave that streamed gate and up rows together would read two tensors at
//           equal offsets at the same time; when the two allocations sit at an unlucky distance those accesses
//           fight over the same DRAM banks (the same decode launch then took 155 instead of 144 us).
//   MODE 1: 32 down rows nb..nb+31 per wave, nb = chunk*128 + 32*w
// Lane (r = lane%16, q = lane/16) loads, per 64-wide k step, the 32 contiguous bytes k = 64*s + 16*q + [0,16) of
// its rows; the two MFMAs of a step contract the two 8-element halves (a consistent reordering of k).
template <int MODE, int MT>
__device__ __forceinline__ void skinny_pass(const GemmParams& p, const bf16_t* const (&w_src)[2], int m0, int m_end,
                                            int nb, int r, int q, int k_rot, floatx4 (*ex)[2][kWave]) {
    const int K = p.K;
    const bf16_t* x_src[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int row = min(m0 + t * 16 + r, m_end - 1);
        if (MODE == 0) {
            int tok = p.sorted_token[row];
            if (p.keep_idx) tok = p.keep_idx[tok];
            row = tok;
        }
        x_src[t] = p.A + (size_t)row * p.lda + q * 16;
    }
    floatx4 acc[MT][2];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int f = 0; f < 2; ++f) acc[t][f] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Every wave starts its walk through K at a different step and wraps around. If all waves of the chip read the
    // same offsets of their (4 KB apart) rows at the same time, the requests of a moment crowd into the few memory
    // channels those offsets map to, and how badly depends on where the weights happen to be allocated: on one box
    // the same decode launch took 137 to 180 us from allocation to allocation, and 144 us every time with the
    // staggered start. The order of the sum changes with the start, deterministically. (The tiled kernel does the
    // opposite on purpose: its workgroups share operands through L2 only while they walk K in step; staggering
    // them cost 24 %.)
    const int ksteps = K / 64;
#pragma unroll 4
    for (int s = 0; s < ksteps; ++s) {
        int ks = s + k_rot;
        if (ks >= ksteps) ks -= ksteps;
        const int k0 = ks * 64;
        bf16x8 wf[2][2], xf[MT][2];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int j = 0; j < 2; ++j) wf[f][j] = *reinterpret_cast<const bf16x8*>(w_src[f] + k0 + j * 8);
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j) xf[t][j] = *reinterpret_cast<const bf16x8*>(x_src[t] + k0 + j * 8);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int f = 0; f < 2; ++f)
                    acc[t][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[f][j], xf[t][j], acc[t][f], 0, 0, 0);
    }

    // D[m = weight row of the fragment, n = token]: lane holds token r, fragment rows 4q..4q+3.
    if (MODE == 0) {
        // up waves (2, 3) -> LDS -> gate waves (0, 1), which own the same columns and the same lane layout
        const int lane = threadIdx.x & (kWave - 1);
        const bool is_up = threadIdx.x >= 2 * kWave;
        if (is_up) {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int f = 0; f < 2; ++f) ex[t][f][lane] = acc[t][f];
        }
        __syncthreads();
        if (!is_up) {
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int row = m0 + t * 16 + r;
                if (row >= m_end) continue;
                bf16_t* crow = p.C + (size_t)row * p.ldc;
#pragma unroll
                for (int f = 0; f < 2; ++f) {
                    const floatx4 u = ex[t][f][lane];
                    float h[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) h[i] = silu_f(acc[t][f][i]) * u[i];
                    *reinterpret_cast<uint2*>(crow + nb + f * 16 + 4 * q) =
                        make_uint2(pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3]));
                }
            }
        }
        __syncthreads();          // the exchange buffer is free again for the next pass
        return;
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int row = m0 + t * 16 + r;
        if (row >= m_end) continue;
        bf16_t* crow = p.C + (size_t)row * p.ldc;
        // fragment f, row m <-> weight row nb + 8*(m>>2) + 4*f + (m&3): lane holds columns nb + 8q + [0, 8)
        *reinterpret_cast<uint4*>(crow + nb + 8 * q) =
            make_uint4(pack_bf16x2(acc[t][0][0], acc[t][0][1]), pack_bf16x2(acc[t][0][2], acc[t][0][3]),
                       pack_bf16x2(acc[t][1][0], acc[t][1][1]), pack_bf16x2(acc[t][1][2], acc[t][1][3]));
    }
}

template <int MODE>
__global__ __launch_bounds__(256) void ffn_skinny_kernel(const GemmParams p) {
    const int g = blockIdx.y;
    const int m_begin = p.offsets[g], m_end = p.offsets[g + 1];
    if (m_begin >= m_end) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    // exchange buffer of MODE 0: [gate wave 0 / 1][token fragment][weight fragment][lane]
    __shared__ floatx4 ex[(MODE == 0) ? 2 : 1][(MODE == 0) ? 4 : 1][2][kWave];
    const int nb_fill = (MODE == 0) ? blockIdx.x * 64 + wave * 16 : blockIdx.x * 128 + wave * 32;
    if (nb_fill >= p.N) return;           // N is a multiple of 64: all waves of a MODE 0 workgroup leave together

    const bf16_t *b0, *b1;
    if (!group_weights(p, g, MODE == 0, b0, b1)) {
        // expert not resident: this wave's columns of the group's rows are defined as zero
        constexpr int kCols = (MODE == 0) ? 16 : 32;
        for (int row = m_begin + lane; row < m_end; row += kWave)
#pragma unroll
            for (int c = 0; c < kCols; c += 8)
                *reinterpret_cast<uint4*>(p.C + (size_t)row * p.ldc + nb_fill + c) = make_uint4(0, 0, 0, 0);
        return;
    }
    const bf16_t* w_src[2];
    int nb;
    if (MODE == 0) {
        nb = blockIdx.x * 64 + (wave & 1) * 32;                  // first column of this wave's two fragments
        const bf16_t* mat = (wave >> 1) ? b1 : b0;              // waves 0, 1: gate; waves 2, 3: up
        w_src[0] = mat + (size_t)(nb + r) * p.K + q * 16;
        w_src[1] = mat + (size_t)(nb + 16 + r) * p.K + q * 16;
    } else {
        nb = nb_fill;
        const int wr = nb + 8 * (r >> 2) + (r & 3);
        w_src[0] = b0 + (size_t)wr * p.K + q * 16;
        w_src[1] = b0 + (size_t)(wr + 4) * p.K + q * 16;
    }
    const int k_rot = (int)((blockIdx.x * 5u + blockIdx.y * 11u + wave * 3u) % (unsigned)(p.K / 64));
    floatx4 (*exw)[2][kWave] = ex[(MODE == 0) ? (wave & 1) : 0];
    for (int m0 = m_begin; m0 < m_end; m0 += 64) {
        const int rows = m_end - m0;
        if (rows <= 16) skinny_pass<MODE, 1>(p, w_src, m0, m_end, nb, r, q, k_rot, exw);
        else if (rows <= 32) skinny_pass<MODE, 2>(p, w_src, m0, m_end, nb, r, q, k_rot, exw);
        else skinny_pass<MODE, 4>(p, w_src, m0, m_end, nb, r, q, k_rot, exw);
    }
}

// Experts that have rows but no slab, ascending: missing[0] = how many, missing[1..] = their ids. One wave.
__global__ __launch_bounds__(kWave) void slab_report_kernel(int E, const int* __restrict__ offsets,
                                                            const bf16_t* const* __restrict__ slabs, int* __restrict__ missing) {
    const int lane = threadIdx.x;
    int found = 0;
    for (int e0 = 0; e0 < E; e0 += kWave) {
        const int e = e0 + lane;
        const bool miss = e < E && offsets[e + 1] > offsets[e] && slabs[e] == nullptr;
        const unsigned long long m = __ballot(miss);
        if (miss) missing[1 + found + __popcll(m & ((1ull << lane) - 1ull))] = e;
        found += __popcll(m);
    }
    if (lane == 0) missing[0] = found;
}

hipError_t launch_slab_report(int E, const int* offsets, const bf16_t* const* slabs, int* missing, hipStream_t st) {
    hipLaunchKernelGGL(slab_report_kernel, dim3(1), dim3(kWave), 0, st, E, offsets, slabs, missing);
    return hipGetLastError();
}

hipError_t launch_grouped_gemm(int mode, bool skinny, const GemmParams& p, int max_rows, hipStream_t st) {
    if (skinny) {
        const dim3 block(256);
        if (mode == 0) {
            hipLaunchKernelGGL(ffn_skinny_kernel<0>, dim3((p.N + 63) / 64, p.G), block, 0, st, p);
        } else {
            hipLaunchKernelGGL(ffn_skinny_kernel<1>, dim3((p.N + 127) / 128, p.G), block, 0, st, p);
        }
        return hipGetLastError();
    }
    // worst-case number of M-tiles (every group may end in a partial tile) and of tall units (one row block per
    // group); each list is dealt to the 8 XCDs in equal runs
    const long long max_mtiles = (max_rows + BM - 1) / BM + p.G;
    const long long per_xcd = (max_mtiles * p.n_ntiles + 7) / 8 + ((long long)p.G * p.n_tall + 7) / 8;
    const long long blocks = per_xcd * 8;
    if (mode == 0) hipLaunchKernelGGL(ffn_tile_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(ffn_tile_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace vismoe
