// Feature construction of the lookahead predictor (paper Sec. 3.3.1, Eq. 6-7) and its decayed target (Sec. 3.3.2,
// Eq. 9): mean pooling over the retained tokens, a routing histogram, and the windowed target score.
#include "common.h"
#include "topk.h"

namespace vismoe {

// ------------------------------------------------------------------------------------------------ mean pooling
// out[c] = (1/K) sum over the K selected rows of rows[., c]                                             (Eq. 6, MP)
// HBM-bound: K rows of D bf16 are read once. Workgroup b of kPoolBlocks walks rows b, b + NB, ... with eight rows in
// flight per thread (at a few thousand rows the call is a handful of memory round trips, so their number is what
// counts); a thread owns 8 consecutive columns (one 16-byte load per row) and the four waves of a workgroup own
// consecutive 512-column pieces, so a row is read in whole 1 KB segments. The partial sums of the workgroups go to the workspace and a
// second kernel adds them in workgroup order: the result does not depend on timing.
constexpr int kPoolBlocks = 64;
constexpr int kPoolRows = 8;            // rows a thread keeps in flight
constexpr int kPoolCols = 256 * 8;      // columns one workgroup covers per pass

__global__ __launch_bounds__(256) void mean_pool_partial_kernel(const bf16_t* __restrict__ rows, int D,
                                                                const int* __restrict__ idx, int K, int nb,
                                                                float* __restrict__ partial) {
    const int b = blockIdx.x;
    for (int c0 = threadIdx.x * 8; c0 < D; c0 += kPoolCols) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        int i = b;
        for (; i + (kPoolRows - 1) * nb < K; i += kPoolRows * nb) {
            int r[kPoolRows];
#pragma unroll
            for (int u = 0; u < kPoolRows; ++u) r[u] = idx ? idx[i + u * nb] : i + u * nb;
            uint4 v[kPoolRows];
#pragma unroll
            for (int u = 0; u < kPoolRows; ++u) v[u] = *reinterpret_cast<const uint4*>(rows + (size_t)r[u] * D + c0);
#pragma unroll
            for (int u = 0; u < kPoolRows; ++u) {
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[2 * j] += bf16_bits_to_float(w[j] & 0xFFFFu);
                    acc[2 * j + 1] += bf16_bits_to_float(w[j] >> 16);
                }
            }
        }
        for (; i < K; i += nb) {
            const int r = idx ? idx[i] : i;
            const uint4 v = *reinterpret_cast<const uint4*>(rows + (size_t)r * D + c0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[2 * j] += bf16_bits_to_float(w[j] & 0xFFFFu);
                acc[2 * j + 1] += bf16_bits_to_float(w[j] >> 16);
            }
        }
        float4* dst = reinterpret_cast<float4*>(partial + (size_t)b * D + c0);
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

__global__ __launch_bounds__(256) void mean_pool_finish_kernel(const float* __restrict__ partial, int D, int nb, int K,
                                                               float* __restrict__ out) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= D) return;
    float s = 0.f;
#pragma unroll 16
    for (int b = 0; b < nb; ++b) s += partial[(size_t)b * D + c];
    out[c] = __fdiv_rn(s, (float)K);
}

size_t mean_pool_workspace_bytes(int D) { return (size_t)kPoolBlocks * (size_t)D * 4; }

hipError_t launch_mean_pool(const bf16_t* rows, int D, const int* idx, int K, float* out, void* ws, hipStream_t st) {
    float* partial = static_cast<float*>(ws);
    const int nb = K < kPoolBlocks ? K : kPoolBlocks;
    hipLaunchKernelGGL(mean_pool_partial_kernel, dim3(nb), dim3(256), 0, st, rows, D, idx, K, nb, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mean_pool_finish_kernel, dim3((D + 255) / 256), dim3(256), 0, st, partial, D, nb, K, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------- routing histogram
// out[e] = (number of the n given activations that went to expert e) / (number that went to any expert in [0, E)).
// One workgroup: counts in LDS (integer atomics: the result is order-independent), eight loads in flight per thread.
__global__ __launch_bounds__(1024) void routing_histogram_kernel(const int* __restrict__ ids, long long n, int E,
                                                                 float* __restrict__ out) {
    __shared__ int cnt[kMaxE];
    __shared__ int wave_tot[1024 / kWave];
    for (int e = threadIdx.x; e < E; e += 1024) cnt[e] = 0;
    __syncthreads();
    int mine = 0;
    for (long long i0 = threadIdx.x; i0 < n; i0 += 8 * 1024) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const long long i = i0 + u * 1024;
            v[u] = (i < n) ? ids[i] : -1;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if ((unsigned)v[u] < (unsigned)E) {
                atomicAdd(&cnt[v[u]], 1);
                ++mine;
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
    if ((threadIdx.x & (kWave - 1)) == 0) wave_tot[threadIdx.x / kWave] = mine;
    __syncthreads();
    int total = 0;
    for (int w = 0; w < 1024 / kWave; ++w) total += wave_tot[w];
    for (int e = threadIdx.x; e < E; e += 1024) out[e] = total > 0 ? __fdiv_rn((float)cnt[e], (float)total) : 0.f;
}

hipError_t launch_routing_histogram(const int* ids, long long n, int E, float* out, hipStream_t st) {
    hipLaunchKernelGGL(routing_histogram_kernel, dim3(1), dim3(1024), 0, st, ids, n, E, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------- lookahead target
// g[e] = max over 1 <= d <= W of gamma^(d-1) [e in E_{l+d}]                                               (Eq. 9)
// future_ids [W, n]: the ids activated at layers l+1 .. l+W. One workgroup; per layer the active experts are flagged
// in LDS (every writer stores the same 1), then g is raised to gamma^(d-1), an fp32 product of d-1 factors.
__global__ __launch_bounds__(1024) void lookahead_target_kernel(const int* __restrict__ future_ids, int W, long long n, int E,
                                                                float gamma, float* __restrict__ g) {
    __shared__ uint8_t active[kMaxE];
    __shared__ float gs[kMaxE];
    for (int e = threadIdx.x; e < E; e += 1024) gs[e] = 0.f;
    float decay = 1.f;
    for (int d = 0; d < W; ++d) {
        for (int e = threadIdx.x; e < E; e += 1024) active[e] = 0;
        __syncthreads();
        const int* row = future_ids + (size_t)d * n;
        for (long long i0 = threadIdx.x; i0 < n; i0 += 8 * 1024) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const long long i = i0 + u * 1024;
                v[u] = (i < n) ? row[i] : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if ((unsigned)v[u] < (unsigned)E) active[v[u]] = 1;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < E; e += 1024)
            if (active[e]) gs[e] = fmaxf(gs[e], decay);
        decay = __fmul_rn(decay, gamma);
        __syncthreads();
    }
    for (int e = threadIdx.x; e < E; e += 1024) g[e] = gs[e];
}

hipError_t launch_lookahead_target(const int* future_ids, int W, long long n, int E, float gamma, float* g, hipStream_t st) {
    hipLaunchKernelGGL(lookahead_target_kernel, dim3(1), dim3(1024), 0, st, future_ids, W, n, E, gamma, g);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------- predictor MLP
// z = psi(W2 psi(W1 x)), y = Wo z                                                                       (Eq. 8)
// with psi = BN-ReLU at inference: a -> max(0, s a + t) per feature (dropout is the identity, batch normalisation an
// affine map the caller has folded into s and t). Three matrix-vector products, HBM-bound on W1; one wave per output
// row, lanes stride over the columns in 16-byte loads, fp32 sums combined by a fixed butterfly (deterministic).
__global__ __launch_bounds__(256) void gemv_affine_kernel(const float* __restrict__ W, const float* __restrict__ x,
                                                          const float* __restrict__ s, const float* __restrict__ t, int rows,
                                                          int cols, int relu, float* __restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int row = blockIdx.x * 4 + threadIdx.x / kWave;
    if (row >= rows) return;
    const float* w = W + (size_t)row * cols;
    float acc = 0.f;
    for (int c = lane * 4; c < cols; c += kWave * 4) {
        const float4 a = *reinterpret_cast<const float4*>(w + c);
        const float4 b = *reinterpret_cast<const float4*>(x + c);
        acc += a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) {
        float v = s ? s[row] * acc + t[row] : acc;
        if (relu) v = fmaxf(v, 0.f);
        out[row] = v;
    }
}

// Maximum / minimum over the wave: inside each 16-lane row by DPP steps, across the four rows through scalar
// registers. (A butterfly of cross-lane shuffles goes through the LDS crossbar, about a hundred cycles per step:
// with twelve of them in each of the B rounds this kernel took 10.8 us for B = 20.)
__device__ __forceinline__ float wave_max_f(float v) {
    v = row_max(v);
    const int b = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ int wave_min_i(int v) {
    v = row_min(v);
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// The B highest entries of y[0..E), descending, ties to the lower index (the ordered prefetch candidates). One wave.
__global__ __launch_bounds__(kWave) void top_b_kernel(const float* __restrict__ y, int E, int B, int* __restrict__ top) {
    const int lane = threadIdx.x;
    constexpr int kPer = kMaxE / kWave;
    float v[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int e = lane + kWave * j;
        v[j] = (e < E) ? y[e] : -INFINITY;
    }
    for (int b = 0; b < B; ++b) {
        float best = -INFINITY;
#pragma unroll
        for (int j = 0; j < kPer; ++j) best = fmaxf(best, v[j]);
        best = wave_max_f(best);
        int bi = 0x7fffffff;
#pragma unroll
        for (int j = kPer - 1; j >= 0; --j)
            if (v[j] == best && lane + kWave * j < E) bi = lane + kWave * j;
        bi = wave_min_i(bi);
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (lane + kWave * j == bi) v[j] = -INFINITY;
        if (lane == 0) top[b] = bi;
    }
}

hipError_t launch_predictor_mlp(const float* x, int D, const float* W1, const float* s1, const float* t1, int D1,
                                const float* W2, const float* s2, const float* t2, int D2, const float* Wo, int E, int B,
                                float* y, int* top, void* ws, hipStream_t st) {
    float* a1 = static_cast<float*>(ws);
    float* a2 = a1 + ((D1 + 63) / 64) * 64;
    hipLaunchKernelGGL(gemv_affine_kernel, dim3((D1 + 3) / 4), dim3(256), 0, st, W1, x, s1, t1, D1, D, 1, a1);
    hipLaunchKernelGGL(gemv_affine_kernel, dim3((D2 + 3) / 4), dim3(256), 0, st, W2, (const float*)a1, s2, t2, D2, D1, 1, a2);
    hipLaunchKernelGGL(gemv_affine_kernel, dim3((E + 3) / 4), dim3(256), 0, st, Wo, (const float*)a2, (const float*)nullptr,
                       (const float*)nullptr, E, D2, 0, y);
    if (B > 0) hipLaunchKernelGGL(top_b_kernel, dim3(1), dim3(kWave), 0, st, (const float*)y, E, B, top);
    return hipGetLastError();
}

size_t predictor_workspace_bytes(int D1, int D2) { return (size_t)(((D1 + 63) / 64) * 64 + ((D2 + 63) / 64) * 64) * 4; }

}  // namespace vismoe
