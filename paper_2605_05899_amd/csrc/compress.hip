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
                                                                        float* __restrict__ part_max) {
    __shared__ float s_min[kPrepThreads / kWave], s_max[kPrepThreads / kWave];
    const int i = blockIdx.x * kPrepThreads + threadIdx.x;
    const int ii = min(i, N - 1);          // lanes past the end repeat the last token, which changes no minimum
    float sum = 0.f;
    for (int h = 0; h < n_heads; ++h) sum = __fadd_rn(sum, attn[(size_t)h * N + ii]);
    const float v = __fdiv_rn(sum, (float)n_heads);
    if (i < N) {
        s[i] = v;
        uint32_t m[kMaxMaskWords];
#pragma unroll
        for (int w = 0; w < kMaxMaskWords; ++w) m[w] = 0;
        for (int l = 0; l < L; ++l) {
            const int* row = ids + ((size_t)l * N + i) * k;
            for (int j = 0; j < k; ++j) {
                const int e = row[j];
                if ((unsigned)e < (unsigned)E) {
                    const uint32_t bit = 1u << (e & 31);
                    const int word = e >> 5;
#pragma unroll
                    for (int w = 0; w < kMaxMaskWords; ++w) m[w] |= (w == word) ? bit : 0u;     // stays in registers
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
// The same algorithm as compress_select_kernel with every pass over the tokens spread over N / 256 workgroups.
// What one workgroup kept in LDS between passes lives in the workspace: two 65 536-bin histograms per selection (a
// top-K is a radix select with two 16-bit digits here), the selection state, the target mask, and one count per
// workgroup for the two places where token order matters (the rank among keys equal to the threshold, the position
// in the output list): a workgroup owns 256 consecutive tokens, adds up the counts of the workgroups before it and
// scans its own. Histogram and mask updates are integer atomics, whose result does not depend on their order, so
// the output is the same bit for bit as that of the single-workgroup kernel.
constexpr int kWideThreads = 256;
constexpr int kWideBins = 65536;
#ifndef VISMOE_WIDE_MIN_TOKENS
#define VISMOE_WIDE_MIN_TOKENS 12288
#endif
constexpr int kWideMinTokens = VISMOE_WIDE_MIN_TOKENS;
static std::atomic<int> g_wide_min{kWideMinTokens};
int compress_wide_min_tokens(int n) {
    return n < 0 ? g_wide_min.load() : g_wide_min.exchange(n);
}
// selection state: [0] high digit of the threshold, [1] keys still to take below it, [2] threshold key, [3] how many
// of the keys equal to the threshold are taken (the first ones in token order)
constexpr int kSelState = 4;

__global__ __launch_bounds__(kWideThreads) void wide_zero_kernel(uint32_t* __restrict__ p, int n) {
    for (int i = blockIdx.x * kWideThreads + threadIdx.x; i < n; i += gridDim.x * kWideThreads) p[i] = 0u;
}

// Sum of one int per thread over the workgroup, returned to all threads. red: LDS, one int per wave.
__device__ __forceinline__ int wide_block_sum(int v, int* red) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();                       // red may still be read from an earlier call
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    int t = 0;
    for (int w = 0; w < kWideThreads / kWave; ++w) t += red[w];
    return t;
}
// Exclusive prefix of one int per thread over the workgroup (thread order). red: LDS, one int per wave.
__device__ __forceinline__ int wide_block_prefix(int v, int* red) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    int incl = v;
    for (int o = 1; o < kWave; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    __syncthreads();
    if (lane == kWave - 1) red[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += red[w];
    return base + incl - v;
}
// Sum of cnt[0 .. blockIdx.x): what the workgroups before this one contributed.
__device__ __forceinline__ int wide_before(const int* __restrict__ cnt, int* red) {
    int v = 0;
    for (int w = threadIdx.x; w < (int)blockIdx.x; w += kWideThreads) v += cnt[w];
    return wide_block_sum(v, red);
}

// Min-max normalisation, keys of the first selection and the histogram of their high digits.
__global__ __launch_bounds__(kWideThreads) void wide_norm_kernel(int N, float* __restrict__ s,
                                                                 const float* __restrict__ part_min,
                                                                 const float* __restrict__ part_max, int n_parts,
                                                                 uint32_t* __restrict__ key, uint8_t* __restrict__ flag,
                                                                 float* __restrict__ s_norm_out, uint32_t* __restrict__ hist_hi) {
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
    __syncthreads();
    for (int w = 0; w < kWideThreads / kWave; ++w) {
        lo = fminf(lo, red_min[w]);
        hi = fmaxf(hi, red_max[w]);
    }
    const float range = __fsub_rn(hi, lo);
    const int i = blockIdx.x * kWideThreads + tid;
    if (i < N) {
        const float st = (range > 0.f) ? __fdiv_rn(__fsub_rn(s[i], lo), range) : 0.f;
        s[i] = st;
        if (s_norm_out) s_norm_out[i] = st;
        const uint32_t k = ordered_key(st);
        key[i] = k;
        flag[i] = 0;
        atomicAdd(&hist_hi[k >> 16], 1u);
    }
}

// One digit of the radix select, one workgroup of 1024 threads: the digit d at which the number of keys with a
// larger digit first reaches `want` (the count of keys in larger digits is `above` < want <= above + hist[d]).
// stage 0 (high digit): want = K;          writes state[0] = d, state[1] = want - above
// stage 1 (low digit):  want = state[1];   writes state[2] = (state[0] << 16) | d, state[3] = want - above
// want <= 0, or more than there are keys: nothing is selected (threshold above every key, take none).
__global__ __launch_bounds__(kSelThreads) void wide_decide_kernel(const uint32_t* __restrict__ hist, int stage, int K,
                                                                  uint32_t* __restrict__ state) {
    __shared__ int wave_sums[kSelThreads / kWave];
    __shared__ int found;
    const int tid = threadIdx.x;
    const int want = stage == 0 ? K : (int)state[1];
    if (tid == 0) found = 0;
    // thread t owns the 64 bins 65535 - 64 t .. 65472 - 64 t, walked downwards
    constexpr int kPer = kWideBins / kSelThreads;
    const uint32_t* mine = hist + (kWideBins - kPer * (tid + 1));
    uint32_t h[kPer];
#pragma unroll
    for (int j = 0; j < kPer; j += 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(mine + j);
        h[j] = v.x; h[j + 1] = v.y; h[j + 2] = v.z; h[j + 3] = v.w;
    }
    int sum = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) sum += (int)h[j];
    int total;
    int above = block_exclusive_scan(sum, wave_sums, total);
    if (want > 0 && above < want && above + sum >= want) {           // exactly one thread
        int j = kPer - 1;
        for (; j > 0; --j) {
            if (above + (int)h[j] >= want) break;
            above += (int)h[j];
        }
        const uint32_t d = (uint32_t)(kWideBins - kPer * (tid + 1) + j);
        if (stage == 0) {
            state[0] = d;
            state[1] = (uint32_t)(want - above);
        } else {
            state[2] = (state[0] << 16) | d;
            state[3] = (uint32_t)(want - above);
        }
        found = 1;
    }
    __syncthreads();
    if (tid == 0 && !found) {
        if (stage == 0) {
            state[0] = 0xFFFFFFFFu;          // matches no key's high digit
            state[1] = 0u;
        } else {
            state[2] = 0xFFFFFFFFu;
            state[3] = 0u;
        }
    }
}

// Histogram of the low digits of the keys whose high digit is the threshold's.
__global__ __launch_bounds__(kWideThreads) void wide_hist_lo_kernel(int N, const uint32_t* __restrict__ key,
                                                                    const uint32_t* __restrict__ state,
                                                                    uint32_t* __restrict__ hist_lo) {
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    if (i >= N) return;
    const uint32_t k = key[i];
    if (k != 0 && (k >> 16) == state[0]) atomicAdd(&hist_lo[k & 0xFFFFu], 1u);
}

// Per workgroup, the number of keys equal to the threshold.
__global__ __launch_bounds__(kWideThreads) void wide_count_eq_kernel(int N, const uint32_t* __restrict__ key,
                                                                     const uint32_t* __restrict__ state,
                                                                     int* __restrict__ wg_eq) {
    __shared__ int red[kWideThreads / kWave];
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    const uint32_t thr = state[2];
    const int eq = (i < N && key[i] == thr && thr != 0u) ? 1 : 0;
    const int t = wide_block_sum(eq, red);
    if (threadIdx.x == 0) wg_eq[blockIdx.x] = t;
}

// Marks with `bit` the keys above the threshold and the first state[3] keys equal to it, in token order. With
// `target`: ORs the masks of the marked tokens into it (the core's expert set). With `wg_keep`: counts, per
// workgroup, the tokens that carry any mark.
__global__ __launch_bounds__(kWideThreads) void wide_mark_kernel(int N, int W, const uint32_t* __restrict__ key,
                                                                 const uint32_t* __restrict__ state,
                                                                 const int* __restrict__ wg_eq, uint8_t* __restrict__ flag,
                                                                 uint8_t bit, const uint32_t* __restrict__ masks,
                                                                 uint32_t* __restrict__ target, int* __restrict__ wg_keep) {
    __shared__ int red[kWideThreads / kWave];
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    const uint32_t thr = state[2];
    const int take_eq = (int)state[3];
    const uint32_t k = (i < N) ? key[i] : 0u;
    const int eq = (i < N && k == thr && thr != 0u) ? 1 : 0;
    const int rank = wide_before(wg_eq, red) + wide_block_prefix(eq, red);
    uint8_t f = 0;
    if (i < N) {
        f = flag[i];
        if (k != 0u && (k > thr || (eq && rank < take_eq))) {
            f |= bit;
            flag[i] = f;
            if (target)
                for (int w = 0; w < W; ++w) {
                    const uint32_t m = masks[(size_t)i * W + w];
                    if (m) atomicOr(&target[w], m);
                }
        }
    }
    if (wg_keep) {
        const int t = wide_block_sum(f != 0 ? 1 : 0, red);
        if (threadIdx.x == 0) wg_keep[blockIdx.x] = t;
    }
}

// Novelty and score of the tokens outside the core (Eq. 2-4), keys of the second selection and the histogram of
// their high digits.
__global__ __launch_bounds__(kWideThreads) void wide_score_kernel(int N, int W, float lambda, const float* __restrict__ s,
                                                                  const uint32_t* __restrict__ masks,
                                                                  const int* __restrict__ cnt,
                                                                  const uint32_t* __restrict__ target,
                                                                  const uint8_t* __restrict__ flag, uint32_t* __restrict__ key,
                                                                  float* __restrict__ delta_out, uint32_t* __restrict__ hist_hi) {
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    if (i >= N) return;
    float d = 0.f;
    uint32_t k = 0;                          // core tokens: below every score, never selected again
    if (!(flag[i] & 1)) {
        int fresh = 0;
        for (int w = 0; w < W; ++w) fresh += __popc(masks[(size_t)i * W + w] & ~target[w]);
        const int c = cnt[i];
        if (c > 0) d = __fdiv_rn((float)fresh, (float)c);
        k = ordered_key(__fsub_rn(s[i], __fmul_rn(lambda, d)));
        atomicAdd(&hist_hi[k >> 16], 1u);
    }
    key[i] = k;
    if (delta_out) delta_out[i] = d;
}

// The marked tokens in ascending order.
__global__ __launch_bounds__(kWideThreads) void wide_write_kernel(int N, const uint8_t* __restrict__ flag,
                                                                  const int* __restrict__ wg_keep, int n_out,
                                                                  int* __restrict__ keep_idx) {
    __shared__ int red[kWideThreads / kWave];
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    const int kept = (i < N && flag[i] != 0) ? 1 : 0;
    const int at = wide_before(wg_keep, red) + wide_block_prefix(kept, red);
    if (kept && at < n_out) keep_idx[at] = i;
}

// Workspace of the compressor: s [N] float, key [N] u32, cnt [N] int, masks [N, W] u32, minima / maxima per
// workgroup of the first kernel, flag [N] u8; for the wide path four histograms, the two selection states, the
// target mask and two counts per workgroup.
struct CompressWs {
    size_t s, key, cnt, masks, part_min, part_max, flag, hist, state, target, wg_eq, wg_keep, total;
};
static CompressWs compress_ws(int N, int E) {
    CompressWs L;
    const size_t n = (size_t)N, W = (size_t)(E + 31) / 32, parts = (n + kPrepThreads - 1) / kPrepThreads;
    const size_t wgs = (n + kWideThreads - 1) / kWideThreads;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.s = take(n * 4);
    L.key = take(n * 4);
    L.cnt = take(n * 4);
    L.masks = take(n * W * 4);
    L.part_min = take(parts * 4);
    L.part_max = take(parts * 4);
    L.flag = take(n);
    // hist, state and target are contiguous: one kernel clears them
    L.hist = take((size_t)4 * kWideBins * 4);
    L.state = take(2 * kSelState * 4);
    L.target = take(kMaxMaskWords * 4);
    L.wg_eq = take(wgs * 4);
    L.wg_keep = take(wgs * 4);
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
    hipLaunchKernelGGL(compress_prepare_kernel, dim3(parts), dim3(kPrepThreads), 0, st, attn, n_heads, N, ids, L, k, E, W, s,
                       masks, cnt, pmin, pmax);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (N < g_wide_min.load()) {
        hipLaunchKernelGGL(compress_select_kernel, dim3(1), dim3(kSelThreads), 0, st, N, W, K_core, K_keep - K_core, lambda,
                           s, masks, cnt, pmin, pmax, parts, key, flag, keep_idx, s_norm_out, delta_out);
        return hipGetLastError();
    }
    uint32_t* hist = reinterpret_cast<uint32_t*>(b + lay.hist);
    uint32_t* state = reinterpret_cast<uint32_t*>(b + lay.state);
    uint32_t* target = reinterpret_cast<uint32_t*>(b + lay.target);
    int* wg_eq = reinterpret_cast<int*>(b + lay.wg_eq);
    int* wg_keep = reinterpret_cast<int*>(b + lay.wg_keep);
    const int wgs = (N + kWideThreads - 1) / kWideThreads;
    const dim3 wide(wgs), wt(kWideThreads), one(1), sel(kSelThreads);
    const int n_clear = (int)((lay.target + kMaxMaskWords * 4 - lay.hist) / 4);
#define VISMOE_WIDE(KERNEL, GRID, BLOCK, ...)                        \
    hipLaunchKernelGGL(KERNEL, GRID, BLOCK, 0, st, __VA_ARGS__);     \
    if ((e = hipGetLastError()) != hipSuccess) return e
    VISMOE_WIDE(wide_zero_kernel, dim3(256), wt, hist, n_clear);
    VISMOE_WIDE(wide_norm_kernel, wide, wt, N, s, pmin, pmax, parts, key, flag, s_norm_out, hist);
    // I_core (Eq. 1); the marked tokens' masks give the target set
    VISMOE_WIDE(wide_decide_kernel, one, sel, hist, 0, K_core, state);
    VISMOE_WIDE(wide_hist_lo_kernel, wide, wt, N, key, state, hist + kWideBins);
    VISMOE_WIDE(wide_decide_kernel, one, sel, hist + kWideBins, 1, K_core, state);
    VISMOE_WIDE(wide_count_eq_kernel, wide, wt, N, key, state, wg_eq);
    VISMOE_WIDE(wide_mark_kernel, wide, wt, N, W, key, state, wg_eq, flag, (uint8_t)1, masks, target, (int*)nullptr);
    // scores (Eq. 2-4) and I_extra (Eq. 5)
    uint32_t* state2 = state + kSelState;
    VISMOE_WIDE(wide_score_kernel, wide, wt, N, W, lambda, s, masks, cnt, target, flag, key, delta_out, hist + 2 * kWideBins);
    VISMOE_WIDE(wide_decide_kernel, one, sel, hist + 2 * kWideBins, 0, K_keep - K_core, state2);
    VISMOE_WIDE(wide_hist_lo_kernel, wide, wt, N, key, state2, hist + 3 * kWideBins);
    VISMOE_WIDE(wide_decide_kernel, one, sel, hist + 3 * kWideBins, 1, K_keep - K_core, state2);
    VISMOE_WIDE(wide_count_eq_kernel, wide, wt, N, key, state2, wg_eq);
    VISMOE_WIDE(wide_mark_kernel, wide, wt, N, W, key, state2, wg_eq, flag, (uint8_t)2, masks, (uint32_t*)nullptr, wg_keep);
    VISMOE_WIDE(wide_write_kernel, wide, wt, N, flag, wg_keep, K_keep, keep_idx);
#undef VISMOE_WIDE
    return hipSuccess;
}

}  // namespace vismoe
