// Affinity-aware token compression (paper Sec. 3.2, Alg. 1, Eq. 1-5): which visual tokens stay.
//
// Two kernels. compress_prepare_kernel is parallel over tokens: head-mean saliency, the token's E-bit multi-hot
// mask of active experts over the pinned-prefix layers (Eq. 3 works on exactly these masks) and its popcount, and
// per-workgroup minima / maxima of the saliency. compress_select_kernel is one workgroup of 1024 threads that runs
// the sequentially dependent rest: min-max normalisation, the core top-K (Eq. 1), the OR of the core tokens' masks
// (E_target), the marginal-expansion score (Eq. 2-4), the second top-K and the ascending index list (Eq. 5).
//
// From kWideMinTokens tokens on the same steps run as a chain of small kernels spread over all CUs (the "wide" path
// below): one workgroup walks N tokens at about 7 ns per token, the chain costs a fixed dozen launches.
//
// A top-K here is an exact radix select on order-preserving 32-bit keys (four 8-bit passes with an LDS histogram),
// followed by a rank among the keys equal to the threshold in token order, so that ties go to the lower index and
// the result does not depend on thread timing. Every floating-point step is a single correctly rounded fp32
// operation (no contraction into fma), in the order the CPU reference uses.
#include <atomic>

#include "common.h"

namespace vismoe {

constexpr int kSelThreads = 1024;
constexpr int kPrepThreads = 256;
constexpr int kMaxMaskWords = kMaxE / 32;

// Order-preserving map float -> uint32 (larger float = larger key); -0 is folded onto +0. Finite floats and
// infinities never map to 0, which is used as "below everything".
__device__ __forceinline__ uint32_t ordered_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kPrepThreads) void compress_prepare_kernel(const float* __restrict__ attn, int n_heads, int N,
                                                                        const int* __restrict__ ids, int L, int k, int E, int W,
                                                                        float* __restrict__ s, uint32_t* __restrict__ masks,
                                                                        int* __restrict__ cnt, float* __restrict__ part_min,
                                                                        float* __restrict__ part_max,
                                                                        uint32_t* __restrict__ clear, int n_clear) {
    __shared__ float s_min[kPrepThreads / kWave], s_max[kPrepThreads / kWave];
    const int i = blockIdx.x * kPrepThreads + threadIdx.x;
    // (the wide path's histograms and selection states start at zero)
    for (int c = i; c < n_clear; c += gridDim.x * kPrepThreads) clear[c] = 0u;
    const int ii = min(i, N - 1);          // lanes past the end repeat the last token, which changes no minimum
    // eight loads in flight at a time; the sum still runs in head order
    float sum = 0.f;
    for (int h0 = 0; h0 < n_heads; h0 += 8) {
        float a[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = attn[(size_t)min(h0 + u, n_heads - 1) * N + ii];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (h0 + u < n_heads) sum = __fadd_rn(sum, a[u]);
    }
    const float v = __fdiv_rn(sum, (float)n_heads);
    if (i < N) {
        s[i] = v;
        uint32_t m[kMaxMaskWords];
#pragma unroll
        for (int w = 0; w < kMaxMaskWords; ++w) m[w] = 0;
        for (int l = 0; l < L; ++l) {
            const int* row = ids + ((size_t)l * N + i) * k;
            for (int j0 = 0; j0 < k; j0 += 8) {          // eight ids in flight at a time
                int e8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) e8[u] = (j0 + u < k) ? row[j0 + u] : -1;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e8[u];
                    if ((unsigned)e < (unsigned)E) {
                        const uint32_t bit = 1u << (e & 31);
                        const int word = e >> 5;
#pragma unroll
                        for (int w = 0; w < kMaxMaskWords; ++w) m[w] |= (w == word) ? bit : 0u;     // stays in registers
                    }
                }
            }
        }
        int c = 0;
#pragma unroll
        for (int w = 0; w < kMaxMaskWords; ++w) {
            if (w < W) {
                masks[(size_t)i * W + w] = m[w];
                c += __popc(m[w]);
            }
        }
        cnt[i] = c;
    }
    float lo = v, hi = v;
    for (int o = 32; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) {
        s_min[wave] = lo;
        s_max[wave] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kPrepThreads / kWave; ++w) {
            lo = fminf(lo, s_min[w]);
            hi = fmaxf(hi, s_max[w]);
        }
        part_min[blockIdx.x] = lo;
        part_max[blockIdx.x] = hi;
    }
}

// Exclusive prefix sum of one int per thread over the workgroup; also returns the total.
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_sums, int& total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    int incl = v;
    for (int o = 1; o < kWave; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    __syncthreads();                       // wave_sums may still be read from an earlier call
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
    for (int w = 0; w < kSelThreads / kWave; ++w) {
        const int ws = wave_sums[w];
        if (w < wave) base += ws;
        tot += ws;
    }
    total = tot;
    return base + incl - v;
}

// The select kernel is one workgroup, so every pass over the N tokens is a chain of global-memory round trips unless
// several loads are in flight per thread: strided passes are unrolled eight-fold (the pointers are __restrict__, the
// compiler then issues the loads of a batch together), and the passes that need token order walk a contiguous range
// per thread in 16-byte pieces.
constexpr int kBatch = 8;

// The threads' contiguous ranges [b, e): `per` tokens each, a multiple of 4 so that every range starts on a 16-byte
// (keys) and 4-byte (flags) boundary.
__device__ __forceinline__ void my_range(int N, int& b, int& e) {
    const int per = ((N + kSelThreads - 1) / kSelThreads + 3) & ~3;
    b = min(N, (int)threadIdx.x * per);
    e = min(N, b + per);
}

// Marks with `bit` in flag[] the K entries of largest key (ties to the lower index) among keys that are not 0.
// Needs K <= number of non-zero keys. All threads of the workgroup call it.
__device__ void select_top(const uint32_t* __restrict__ key, int N, int K, uint8_t* __restrict__ flag, uint8_t bit,
                           uint32_t* hist, int* wave_sums, uint32_t* bcast) {
    if (K <= 0) return;
    uint32_t prefix = 0, known = 0;
    int remaining = K;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        __syncthreads();
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        for (int i0 = threadIdx.x; i0 < N; i0 += kBatch * kSelThreads) {
            uint32_t kk[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + u * kSelThreads;
                kk[u] = (i < N) ? key[i] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                if (kk[u] != 0 && (kk[u] & known) == prefix) atomicAdd(&hist[(kk[u] >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x < kWave) {
            // The digit at which the count of larger-or-equal keys first reaches `remaining`: lane l owns digits
            // 255 - 4l .. 252 - 4l; a wave scan gives the count of keys in all higher digits.
            const int l = threadIdx.x;
            uint32_t h[4], mine = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h[j] = hist[255 - 4 * l - j];
                mine += h[j];
            }
            uint32_t incl = mine;
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t t = __shfl_up(incl, o);
                if (l >= o) incl += t;
            }
            uint32_t above = incl - mine;
            if (above < (uint32_t)remaining && incl >= (uint32_t)remaining) {      // exactly one lane
                int j = 0;
                for (; j < 3; ++j) {
                    if (above + h[j] >= (uint32_t)remaining) break;
                    above += h[j];
                }
                bcast[0] = (uint32_t)(255 - 4 * l - j);
                bcast[1] = above;
            }
        }
        __syncthreads();
        prefix |= bcast[0] << shift;
        known |= 255u << shift;
        remaining -= (int)bcast[1];
    }
    // keys above the threshold are taken; of the keys equal to it, the first `remaining` in token order
    const uint32_t thr = prefix;
    int b, e;
    my_range(N, b, e);
    int eq = 0;
#pragma unroll 2
    for (int i = b; i < e; i += 4) {
        if (i + 4 <= e) {
            const uint4 k4 = *reinterpret_cast<const uint4*>(key + i);
            eq += (k4.x == thr) + (k4.y == thr) + (k4.z == thr) + (k4.w == thr);
        } else {
            for (int j = i; j < e; ++j) eq += (key[j] == thr);
        }
    }
    int total;
    int rank = block_exclusive_scan(eq, wave_sums, total);
#pragma unroll 2
    for (int i = b; i < e; i += 4) {
        if (i + 4 <= e) {
            const uint4 k4 = *reinterpret_cast<const uint4*>(key + i);
            const uint32_t kk[4] = {k4.x, k4.y, k4.z, k4.w};
            uint32_t f = *reinterpret_cast<const uint32_t*>(flag + i);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (kk[j] > thr || (kk[j] == thr && rank++ < remaining)) f |= (uint32_t)bit << (8 * j);
            *reinterpret_cast<uint32_t*>(flag + i) = f;
        } else {
            for (int j = i; j < e; ++j) {
                const uint32_t kk = key[j];
                if (kk > thr || (kk == thr && rank++ < remaining)) flag[j] |= bit;
            }
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kSelThreads) void compress_select_kernel(int N, int W, int K_core, int K_rem, float lambda,
                                                                      float* __restrict__ s, const uint32_t* __restrict__ masks,
                                                                      const int* __restrict__ cnt,
                                                                      const float* __restrict__ part_min,
                                                                      const float* __restrict__ part_max, int n_parts,
                                                                      uint32_t* __restrict__ key, uint8_t* __restrict__ flag,
                                                                      int* __restrict__ keep_idx, float* __restrict__ s_norm_out,
                                                                      float* __restrict__ delta_out) {
    __shared__ uint32_t hist[256];
    __shared__ int wave_sums[kSelThreads / kWave];
    __shared__ uint32_t bcast[2];
    __shared__ float red_min[kSelThreads / kWave], red_max[kSelThreads / kWave];
    __shared__ uint32_t target[kMaxMaskWords];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

    // ---- Normalize: minimum and maximum over the workgroups of the first kernel
    float lo = part_min[0], hi = part_max[0];
    for (int i = tid; i < n_parts; i += kSelThreads) {
        lo = fminf(lo, part_min[i]);
        hi = fmaxf(hi, part_max[i]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    if (lane == 0) {
        red_min[wave] = lo;
        red_max[wave] = hi;
    }
    if (tid < kMaxMaskWords) target[tid] = 0;
    __syncthreads();
    for (int w = 0; w < kSelThreads / kWave; ++w) {
        lo = fminf(lo, red_min[w]);
        hi = fmaxf(hi, red_max[w]);
    }
    const float range = __fsub_rn(hi, lo);
    for (int i0 = tid; i0 < N; i0 += kBatch * kSelThreads) {
        float v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u * kSelThreads;
            v[u] = (i < N) ? s[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u * kSelThreads;
            if (i < N) {
                const float st = (range > 0.f) ? __fdiv_rn(__fsub_rn(v[u], lo), range) : 0.f;
                s[i] = st;
                if (s_norm_out) s_norm_out[i] = st;
                key[i] = ordered_key(st);
                flag[i] = 0;
            }
        }
    }
    __syncthreads();

    // ---- I_core = TopK(s~, K_core)                                                              (Eq. 1)
    select_top(key, N, K_core, flag, 1, hist, wave_sums, bcast);

    // ---- E_target = union of the core tokens' expert sets, as a mask
    for (int i0 = tid; i0 < N; i0 += kBatch * kSelThreads) {
        uint8_t f[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u * kSelThreads;
            f[u] = (i < N) ? flag[i] : (uint8_t)0;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (f[u] & 1) {
                const int i = i0 + u * kSelThreads;
                for (int w = 0; w < W; ++w) {
                    const uint32_t m = masks[(size_t)i * W + w];
                    if (m) atomicOr(&target[w], m);
                }
            }
        }
    }
    __syncthreads();

    // ---- Delta_i and p_i for the tokens outside the core                                         (Eq. 2-4)
    for (int i0 = tid; i0 < N; i0 += 4 * kSelThreads) {
        uint8_t f[4];
        int c[4], fresh[4];
        float st[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + u * kSelThreads, N - 1);
            f[u] = flag[i];
            c[u] = cnt[i];
            st[u] = s[i];
            fresh[u] = 0;
            for (int w = 0; w < W; ++w) fresh[u] += __popc(masks[(size_t)i * W + w] & ~target[w]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kSelThreads;
            if (i < N) {
                float d = 0.f;
                if (f[u] & 1) {
                    key[i] = 0;                      // below every score: never selected again
                } else {
                    if (c[u] > 0) d = __fdiv_rn((float)fresh[u], (float)c[u]);
                    key[i] = ordered_key(__fsub_rn(st[u], __fmul_rn(lambda, d)));
                }
                if (delta_out) delta_out[i] = d;
            }
        }
    }
    __syncthreads();

    // ---- I_extra = TopK(p, K_keep - K_core) over the tokens outside the core                     (Eq. 5)
    select_top(key, N, K_rem, flag, 2, hist, wave_sums, bcast);

    // ---- I_keep in ascending token order
    int b, e;
    my_range(N, b, e);
    int n = 0;
#pragma unroll 2
    for (int i = b; i < e; i += 4) {
        if (i + 4 <= e) {
            const uint32_t f = *reinterpret_cast<const uint32_t*>(flag + i);
            n += ((f & 0xFFu) != 0) + ((f & 0xFF00u) != 0) + ((f & 0xFF0000u) != 0) + ((f & 0xFF000000u) != 0);
        } else {
            for (int j = i; j < e; ++j) n += (flag[j] != 0);
        }
    }
    int total;
    int at = block_exclusive_scan(n, wave_sums, total);
#pragma unroll 2
    for (int i = b; i < e; i += 4) {
        if (i + 4 <= e) {
            const uint32_t f = *reinterpret_cast<const uint32_t*>(flag + i);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((f >> (8 * j)) & 0xFFu) keep_idx[at++] = i + j;
        } else {
            for (int j = i; j < e; ++j)
                if (flag[j]) keep_idx[at++] = j;
        }
    }
}

// ------------------------------------------------------------------------------------------------ wide path
// The same algorithm as compress_select_kernel with every pass over the tokens spread over N / 4096 workgroups of
// 1024 threads (four consecutive tokens per thread). What one workgroup kept in LDS between passes lives in the
// workspace. A top-K is a radix select over three digits of the key (11, 11 and 10 bits): each pass builds the
// histogram of one digit (per workgroup in LDS first, then one global atomic per non-empty bin, so that a popular bin
// receives one update per workgroup and not one per token: updates of one address are served one after the other,
// about 50 ns each), and the NEXT pass starts by finding, in every workgroup again, the digit at which the count of
// larger keys reaches K. Token order matters in two places only, the rank among keys equal to the threshold and the
// position in the output list: a workgroup owns 4096 consecutive tokens, adds up the counts of the workgroups before
// it (written by the launch before) and scans its own. The core's expert set is OR-ed per workgroup and the
// workgroups' words are OR-ed by every workgroup of the scoring pass. Histogram and mask updates are integer
// operations whose result does not depend on their order, so the output is the same bit for bit as that of the
// single-workgroup kernel.
constexpr int kWideThreads = 1024, kWidePer = 4, kWideTokens = kWideThreads * kWidePer;
constexpr int kDigit1Shift = 21, kDigit2Shift = 10;             // digits: key >> 21 | (key >> 10) & 2047 | key & 1023
constexpr int kBins1 = 2048, kBins2 = 2048, kBins3 = 1024;
constexpr int kSelHist = kBins1 + kBins2 + kBins3;              // ints of histogram per selection
constexpr uint32_t kNoDigit = 0xFFFFFFFFu;                      // "nothing is selected": matches no key
#ifndef VISMOE_WIDE_MIN_TOKENS
#define VISMOE_WIDE_MIN_TOKENS 7168
#endif
constexpr int kWideMinTokens = VISMOE_WIDE_MIN_TOKENS;
static std::atomic<int> g_wide_min{kWideMinTokens};
int compress_wide_min_tokens(int n) {
    return n < 0 ? g_wide_min.load() : g_wide_min.exchange(n);
}
// selection state, written by workgroup 0 of the pass that decides it and read by the passes after it:
// [0] digit 1, [1] keys still to take below it, [2] digit 2, [3] keys still to take, [4] threshold key, [5] how many
// of the keys equal to the threshold are taken (the first ones in token order)
constexpr int kSelState = 8;

struct WideLds {
    uint32_t hist[kBins1];
    int wave_sums[kWideThreads / kWave];
    uint32_t pick[2];
    uint32_t target[kMaxMaskWords];
};

// The digit d of `hist` (nbins bins, a power of two of at most 2 x 1024) at which the number of keys with a larger
// digit first reaches `want`: above < want <= above + hist[d]. Returns d and want - above to all threads; kNoDigit
// and 0 when want <= 0 or want exceeds the number of keys. All 1024 threads call it.
__device__ __forceinline__ void wide_decide(const uint32_t* __restrict__ hist, int nbins, int want, WideLds& L,
                                            uint32_t& digit, int& left) {
    const int tid = threadIdx.x, per = nbins / kWideThreads;           // 2 or 1 bins per thread, walked downwards
    const int first = nbins - per * (tid + 1);
    const int h1 = (int)hist[first + per - 1], h0 = per == 2 ? (int)hist[first] : 0;
    if (tid == 0) {
        L.pick[0] = kNoDigit;
        L.pick[1] = 0u;
    }
    int total;
    const int above = block_exclusive_scan(h1 + h0, L.wave_sums, total);       // (synchronises: pick is set)
    if (want > 0 && above < want && above + h1 + h0 >= want) {                 // exactly one thread
        const bool upper = above + h1 >= want;
        L.pick[0] = (uint32_t)(upper ? first + per - 1 : first);
        L.pick[1] = (uint32_t)(want - (upper ? above : above + h1));
    }
    __syncthreads();
    digit = L.pick[0];
    left = (int)L.pick[1];
    __syncthreads();                         // pick may be set again by the next call
}

__device__ __forceinline__ void wide_hist_clear(WideLds& L) {
    for (int i = threadIdx.x; i < kBins1; i += kWideThreads) L.hist[i] = 0u;
    __syncthreads();
}
// One global update per non-empty bin of the workgroup's histogram.
__device__ __forceinline__ void wide_hist_flush(WideLds& L, int nbins, uint32_t* __restrict__ hist) {
    __syncthreads();
    for (int i = threadIdx.x; i < nbins; i += kWideThreads) {
        const uint32_t c = L.hist[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// Sum of one int per thread over the workgroup, returned to all threads.
__device__ __forceinline__ int wide_block_sum(int v, WideLds& L) {
    int total;
    (void)block_exclusive_scan(v, L.wave_sums, total);
    return total;
}
// Sum of cnt[0 .. blockIdx.x): what the workgroups before this one contributed.
__device__ __forceinline__ int wide_before(const int* __restrict__ cnt, WideLds& L) {
    int v = 0;
    for (int w = threadIdx.x; w < (int)blockIdx.x; w += kWideThreads) v += cnt[w];
    return wide_block_sum(v, L);
}

// Min-max normalisation, keys of the first selection and the histogram of their first digits.
__global__ __launch_bounds__(kWideThreads) void wide_norm_kernel(int N, float* __restrict__ s,
                                                                 const float* __restrict__ part_min,
                                                                 const float* __restrict__ part_max, int n_parts,
                                                                 uint32_t* __restrict__ key, uint8_t* __restrict__ flag,
                                                                 float* __restrict__ s_norm_out, uint32_t* __restrict__ hist1) {
    __shared__ WideLds L;
    __shared__ float red_min[kWideThreads / kWave], red_max[kWideThreads / kWave];
    const int tid = threadIdx.x;
    float lo = part_min[0], hi = part_max[0];
    for (int i = tid; i < n_parts; i += kWideThreads) {
        lo = fminf(lo, part_min[i]);
        hi = fmaxf(hi, part_max[i]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    if ((tid & (kWave - 1)) == 0) {
        red_min[tid / kWave] = lo;
        red_max[tid / kWave] = hi;
    }
    wide_hist_clear(L);                      // (synchronises)
    for (int w = 0; w < kWideThreads / kWave; ++w) {
        lo = fminf(lo, red_min[w]);
        hi = fmaxf(hi, red_max[w]);
    }
    const float range = __fsub_rn(hi, lo);
    const int i0 = (blockIdx.x * kWideThreads + tid) * kWidePer;
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        const int i = i0 + j;
        if (i < N) {
            const float st = (range > 0.f) ? __fdiv_rn(__fsub_rn(s[i], lo), range) : 0.f;
            s[i] = st;
            if (s_norm_out) s_norm_out[i] = st;
            const uint32_t k = ordered_key(st);
            key[i] = k;
            flag[i] = 0;
            atomicAdd(&L.hist[k >> kDigit1Shift], 1u);
        }
    }
    wide_hist_flush(L, kBins1, hist1);
}

// Second pass of a selection: decides digit 1 from its histogram (want = K), then the histogram of the second
// digits of the keys that carry it.
__global__ __launch_bounds__(kWideThreads) void wide_digit2_kernel(int N, const uint32_t* __restrict__ key, int K,
                                                                   const uint32_t* __restrict__ hist1,
                                                                   uint32_t* __restrict__ state, uint32_t* __restrict__ hist2) {
    __shared__ WideLds L;
    uint32_t d1;
    int left;
    wide_decide(hist1, kBins1, K, L, d1, left);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[0] = d1;
        state[1] = (uint32_t)left;
    }
    wide_hist_clear(L);
    const int i0 = (blockIdx.x * kWideThreads + threadIdx.x) * kWidePer;
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        const int i = i0 + j;
        if (i < N) {
            const uint32_t k = key[i];
            if (k != 0u && (k >> kDigit1Shift) == d1) atomicAdd(&L.hist[(k >> kDigit2Shift) & (kBins2 - 1)], 1u);
        }
    }
    wide_hist_flush(L, kBins2, hist2);
}

// Third pass: decides digit 2, then the histogram of the last digits of the keys that carry digits 1 and 2.
__global__ __launch_bounds__(kWideThreads) void wide_digit3_kernel(int N, const uint32_t* __restrict__ key,
                                                                   const uint32_t* __restrict__ hist2,
                                                                   uint32_t* __restrict__ state, uint32_t* __restrict__ hist3) {
    __shared__ WideLds L;
    const uint32_t d1 = state[0];
    uint32_t d2;
    int left;
    wide_decide(hist2, kBins2, (int)state[1], L, d2, left);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[2] = d2;
        state[3] = (uint32_t)left;
    }
    const uint32_t prefix = (d1 == kNoDigit || d2 == kNoDigit) ? kNoDigit : ((d1 << (kDigit1Shift - kDigit2Shift)) | d2);
    wide_hist_clear(L);
    const int i0 = (blockIdx.x * kWideThreads + threadIdx.x) * kWidePer;
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        const int i = i0 + j;
        if (i < N) {
            const uint32_t k = key[i];
            if (k != 0u && (k >> kDigit2Shift) == prefix) atomicAdd(&L.hist[k & (kBins3 - 1)], 1u);
        }
    }
    wide_hist_flush(L, kBins3, hist3);
}

// Fourth pass: decides the last digit, i.e. the threshold key and how many of the keys equal to it are taken; per
// workgroup, the number of keys equal to the threshold.
__global__ __launch_bounds__(kWideThreads) void wide_count_eq_kernel(int N, const uint32_t* __restrict__ key,
                                                                     const uint32_t* __restrict__ hist3,
                                                                     uint32_t* __restrict__ state, int* __restrict__ wg_eq) {
    __shared__ WideLds L;
    const uint32_t d1 = state[0], d2 = state[2];
    uint32_t d3;
    int take;
    wide_decide(hist3, kBins3, (int)state[3], L, d3, take);
    const bool none = d1 == kNoDigit || d2 == kNoDigit || d3 == kNoDigit;
    const uint32_t thr = none ? kNoDigit : ((d1 << kDigit1Shift) | (d2 << kDigit2Shift) | d3);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[4] = thr;
        state[5] = none ? 0u : (uint32_t)take;
    }
    const int i0 = (blockIdx.x * kWideThreads + threadIdx.x) * kWidePer;
    int eq = 0;
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        const int i = i0 + j;
        if (i < N && key[i] == thr) ++eq;
    }
    const int t = wide_block_sum(eq, L);
    if (threadIdx.x == 0) wg_eq[blockIdx.x] = t;
}

// Marks with `bit` the keys above the threshold and the first state[5] keys equal to it, in token order. With
// `wg_target`: ORs the masks of the tokens marked by this workgroup into its 16 words there (the core's expert set).
// With `wg_keep`: counts, per workgroup, the tokens that carry any mark.
__global__ __launch_bounds__(kWideThreads) void wide_mark_kernel(int N, int W, const uint32_t* __restrict__ key,
                                                                 const uint32_t* __restrict__ state,
                                                                 const int* __restrict__ wg_eq, uint8_t* __restrict__ flag,
                                                                 uint8_t bit, const uint32_t* __restrict__ masks,
                                                                 uint32_t* __restrict__ wg_target, int* __restrict__ wg_keep) {
    __shared__ WideLds L;
    const int tid = threadIdx.x;
    const uint32_t thr = state[4];
    const int take_eq = (int)state[5];
    const int i0 = (blockIdx.x * kWideThreads + tid) * kWidePer;
    uint32_t k[kWidePer];
    int eq = 0;
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        k[j] = (i0 + j < N) ? key[i0 + j] : 0u;
        eq += (k[j] != 0u && k[j] == thr) ? 1 : 0;
    }
    if (tid < kMaxMaskWords) L.target[tid] = 0u;
    const int before = wide_before(wg_eq, L);
    int total;
    int rank = before + block_exclusive_scan(eq, L.wave_sums, total);
    uint8_t f[kWidePer];
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) f[j] = (i0 + j < N) ? flag[i0 + j] : (uint8_t)0;
    int kept = 0;
    bool marked[kWidePer];
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        const bool is_eq = k[j] != 0u && k[j] == thr;
        marked[j] = k[j] != 0u && (k[j] > thr || (is_eq && rank < take_eq));        // (k is 0 past the end)
        if (marked[j]) {
            f[j] |= bit;
            flag[i0 + j] = f[j];
        }
        if (is_eq) ++rank;
        kept += f[j] != 0 ? 1 : 0;
    }
    if (wg_target) {
        // masks of the marked tokens: OR-ed over the thread's tokens, over the wave by a butterfly, and once per wave
        // into the workgroup's words
        for (int w = 0; w < W; ++w) {
            uint32_t m = 0u;
#pragma unroll
            for (int j = 0; j < kWidePer; ++j)
                if (marked[j]) m |= masks[(size_t)(i0 + j) * W + w];
            for (int o = 32; o > 0; o >>= 1) m |= __shfl_xor(m, o);
            if ((tid & (kWave - 1)) == 0 && m) atomicOr(&L.target[w], m);
        }
    }
    if (wg_target) {
        __syncthreads();
        if (tid < kMaxMaskWords) wg_target[(size_t)blockIdx.x * kMaxMaskWords + tid] = L.target[tid];
    }
    if (wg_keep) {
        const int t = wide_block_sum(kept, L);
        if (tid == 0) wg_keep[blockIdx.x] = t;
    }
}

// Novelty and score of the tokens outside the core (Eq. 2-4), keys of the second selection and the histogram of
// their first digits. The target set is the OR of the words the marking pass left per workgroup.
__global__ __launch_bounds__(kWideThreads) void wide_score_kernel(int N, int W, float lambda, const float* __restrict__ s,
                                                                  const uint32_t* __restrict__ masks,
                                                                  const int* __restrict__ cnt,
                                                                  const uint32_t* __restrict__ wg_target, int n_wg,
                                                                  const uint8_t* __restrict__ flag, uint32_t* __restrict__ key,
                                                                  float* __restrict__ delta_out, uint32_t* __restrict__ hist1) {
    __shared__ WideLds L;
    const int tid = threadIdx.x;
    if (tid < kMaxMaskWords) L.target[tid] = 0u;
    wide_hist_clear(L);                      // (synchronises)
    for (int i = tid; i < n_wg * kMaxMaskWords; i += kWideThreads) {
        const uint32_t m = wg_target[i];
        if (m) atomicOr(&L.target[i & (kMaxMaskWords - 1)], m);
    }
    __syncthreads();
    const int i0 = (blockIdx.x * kWideThreads + tid) * kWidePer;
    // all loads of the thread's four tokens are independent of each other (rows past the end repeat the last token)
    int ii[kWidePer], c[kWidePer], fresh[kWidePer];
    uint8_t f[kWidePer];
    float st[kWidePer];
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        ii[j] = min(i0 + j, N - 1);
        f[j] = flag[ii[j]];
        c[j] = cnt[ii[j]];
        st[j] = s[ii[j]];
        fresh[j] = 0;
    }
    for (int w = 0; w < W; ++w) {
        const uint32_t tw = ~L.target[w];
#pragma unroll
        for (int j = 0; j < kWidePer; ++j) fresh[j] += __popc(masks[(size_t)ii[j] * W + w] & tw);
    }
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        const int i = i0 + j;
        if (i >= N) continue;
        float d = 0.f;
        uint32_t k = 0;                      // core tokens: below every score, never selected again
        if (!(f[j] & 1)) {
            if (c[j] > 0) d = __fdiv_rn((float)fresh[j], (float)c[j]);
            k = ordered_key(__fsub_rn(st[j], __fmul_rn(lambda, d)));
            atomicAdd(&L.hist[k >> kDigit1Shift], 1u);
        }
        key[i] = k;
        if (delta_out) delta_out[i] = d;
    }
    wide_hist_flush(L, kBins1, hist1);
}

// The marked tokens in ascending order.
__global__ __launch_bounds__(kWideThreads) void wide_write_kernel(int N, const uint8_t* __restrict__ flag,
                                                                  const int* __restrict__ wg_keep, int n_out,
                                                                  int* __restrict__ keep_idx) {
    __shared__ WideLds L;
    const int i0 = (blockIdx.x * kWideThreads + threadIdx.x) * kWidePer;
    bool kept[kWidePer];
    int n = 0;
#pragma unroll
    for (int j = 0; j < kWidePer; ++j) {
        kept[j] = i0 + j < N && flag[i0 + j] != 0;
        n += kept[j] ? 1 : 0;
    }
    const int before = wide_before(wg_keep, L);
    int total;
    int at = before + block_exclusive_scan(n, L.wave_sums, total);
#pragma unroll
    for (int j = 0; j < kWidePer; ++j)
        if (kept[j]) {
            if (at < n_out) keep_idx[at] = i0 + j;
            ++at;
        }
}

// Workspace of the compressor: s [N] float, key [N] u32, cnt [N] int, masks [N, W] u32, minima / maxima per
// workgroup of the first kernel, flag [N] u8; for the wide path the histograms and states of the two selections and,
// per workgroup, two counts and the words of the core's expert set.
struct CompressWs {
    size_t s, key, cnt, masks, part_min, part_max, flag, hist, state, wg_eq, wg_keep, wg_target, total;
};
static CompressWs compress_ws(int N, int E) {
    CompressWs L;
    const size_t n = (size_t)N, W = (size_t)(E + 31) / 32, parts = (n + kPrepThreads - 1) / kPrepThreads;
    const size_t wgs = (n + kWideTokens - 1) / kWideTokens;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.s = take(n * 4);
    L.key = take(n * 4);
    L.cnt = take(n * 4);
    L.masks = take(n * W * 4);
    L.part_min = take(parts * 4);
    L.part_max = take(parts * 4);
    L.flag = take(n);
    // hist and state are contiguous: the first kernel clears them together
    L.hist = take((size_t)2 * kSelHist * 4);
    L.state = take(2 * kSelState * 4);
    L.wg_eq = take(wgs * 4);
    L.wg_keep = take(wgs * 4);
    L.wg_target = take(wgs * kMaxMaskWords * 4);
    L.total = o;
    return L;
}

size_t compress_workspace_bytes(int N, int E) {
    if (N < 0 || E < 1 || E > kMaxE) return 0;
    return compress_ws(N > 0 ? N : 1, E).total;
}

hipError_t launch_token_compress(const float* attn, int n_heads, int N, const int* ids, int L, int k, int E, int K_core,
                                 int K_keep, float lambda, int* keep_idx, float* s_norm_out, float* delta_out, void* ws,
                                 hipStream_t st) {
    const CompressWs lay = compress_ws(N, E);
    char* b = static_cast<char*>(ws);
    float* s = reinterpret_cast<float*>(b + lay.s);
    uint32_t* key = reinterpret_cast<uint32_t*>(b + lay.key);
    int* cnt = reinterpret_cast<int*>(b + lay.cnt);
    uint32_t* masks = reinterpret_cast<uint32_t*>(b + lay.masks);
    float* pmin = reinterpret_cast<float*>(b + lay.part_min);
    float* pmax = reinterpret_cast<float*>(b + lay.part_max);
    uint8_t* flag = reinterpret_cast<uint8_t*>(b + lay.flag);
    const int W = (E + 31) / 32, parts = (N + kPrepThreads - 1) / kPrepThreads;
    const bool wide_path = N >= g_wide_min.load();
    uint32_t* hist = reinterpret_cast<uint32_t*>(b + lay.hist);
    uint32_t* state = reinterpret_cast<uint32_t*>(b + lay.state);
    const int n_clear = wide_path ? (int)((lay.state + 2 * kSelState * 4 - lay.hist) / 4) : 0;
    hipLaunchKernelGGL(compress_prepare_kernel, dim3(parts), dim3(kPrepThreads), 0, st, attn, n_heads, N, ids, L, k, E, W, s,
                       masks, cnt, pmin, pmax, hist, n_clear);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (!wide_path) {
        hipLaunchKernelGGL(compress_select_kernel, dim3(1), dim3(kSelThreads), 0, st, N, W, K_core, K_keep - K_core, lambda,
                           s, masks, cnt, pmin, pmax, parts, key, flag, keep_idx, s_norm_out, delta_out);
        return hipGetLastError();
    }
    int* wg_eq = reinterpret_cast<int*>(b + lay.wg_eq);
    int* wg_keep = reinterpret_cast<int*>(b + lay.wg_keep);
    uint32_t* wg_target = reinterpret_cast<uint32_t*>(b + lay.wg_target);
    const int wgs = (N + kWideTokens - 1) / kWideTokens;
    const dim3 grid(wgs), block(kWideThreads);
#define VISMOE_WIDE(KERNEL, ...)                                      \
    hipLaunchKernelGGL(KERNEL, grid, block, 0, st, __VA_ARGS__);      \
    if ((e = hipGetLastError()) != hipSuccess) return e
    // I_core (Eq. 1); the marked tokens' masks give the target set
    uint32_t *h1 = hist, *h2 = hist + kBins1, *h3 = hist + kBins1 + kBins2;
    VISMOE_WIDE(wide_norm_kernel, N, s, pmin, pmax, parts, key, flag, s_norm_out, h1);
    VISMOE_WIDE(wide_digit2_kernel, N, key, K_core, h1, state, h2);
    VISMOE_WIDE(wide_digit3_kernel, N, key, h2, state, h3);
    VISMOE_WIDE(wide_count_eq_kernel, N, key, h3, state, wg_eq);
    VISMOE_WIDE(wide_mark_kernel, N, W, key, state, wg_eq, flag, (uint8_t)1, masks, wg_target, (int*)nullptr);
    // scores (Eq. 2-4) and I_extra (Eq. 5)
    h1 += kSelHist; h2 += kSelHist; h3 += kSelHist;
    uint32_t* state2 = state + kSelState;
    VISMOE_WIDE(wide_score_kernel, N, W, lambda, s, masks, cnt, wg_target, wgs, flag, key, delta_out, h1);
    VISMOE_WIDE(wide_digit2_kernel, N, key, K_keep - K_core, h1, state2, h2);
    VISMOE_WIDE(wide_digit3_kernel, N, key, h2, state2, h3);
    VISMOE_WIDE(wide_count_eq_kernel, N, key, h3, state2, wg_eq);
    VISMOE_WIDE(wide_mark_kernel, N, W, key, state2, wg_eq, flag, (uint8_t)2, masks, (uint32_t*)nullptr, wg_keep);
    VISMOE_WIDE(wide_write_kernel, N, flag, wg_keep, K_keep, keep_idx);
#undef VISMOE_WIDE
    return hipSuccess;
}

}  // namespace vismoe
