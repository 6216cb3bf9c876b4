// Weighted combine: out[j] = sum_s w[j,s] * y[inv_perm[j*k+s]] + sum of the shared-expert rows of token j,
// fp32 accumulation in ascending s, one rounding to bf16 (the last step of the MoE feed-forward block of
// paper Sec. 2.1; the shared-expert term is Sec. 3.4.1's always-on experts).
// One workgroup per (token, 1024-column slab); every lane moves 16-byte pieces, so each y row is read as
// whole cache lines.
#include <type_traits>

#include "common.h"

namespace vismoe {

__global__ __launch_bounds__(128) void combine_kernel(const bf16_t* __restrict__ y, const int* __restrict__ inv_perm,
                                                      const float* __restrict__ topk_w, int k, int H,
                                                      const bf16_t* __restrict__ extra, int n_extra,
                                                      long long extra_stride, bf16_t* __restrict__ out) {
    const int t = blockIdx.x;
    const int col = (blockIdx.y * 128 + threadIdx.x) * 8;
    if (col >= H) return;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    auto fma_piece = [&](const uint4& v, float w) {
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += w * __uint_as_float(u[i] << 16);
            acc[2 * i + 1] += w * __uint_as_float(u[i] & 0xffff0000u);
        }
    };
    auto fma_row = [&](const bf16_t* row, float w) { fma_piece(*reinterpret_cast<const uint4*>(row + col), w); };
    // N rows at a time: all positions, then all row pieces are requested before the first is used, so that a token's
    // rows are in flight together; the sum still runs in ascending s
    auto batch = [&](auto n_tag, int s0) {
        constexpr int N = decltype(n_tag)::value;
        int pos[N];
        float w[N];
        uint4 v[N];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            pos[i] = inv_perm[(size_t)t * k + s0 + i];
            w[i] = topk_w[(size_t)t * k + s0 + i];
        }
#pragma unroll
        // every element of y is read exactly once: loads marked non-temporal (the 268 MB of the video prefill otherwise
        // push their way through the caches; 55.7 -> 49.3 us on that workload, no change on the small ones)
        for (int i = 0; i < N; ++i) {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(y + (size_t)pos[i] * H + col));
            v[i] = make_uint4(t.x, t.y, t.z, t.w);
        }
#pragma unroll
        for (int i = 0; i < N; ++i) fma_piece(v[i], w[i]);
    };
    int s = 0;
    for (; s + 8 <= k; s += 8) batch(std::integral_constant<int, 8>{}, s);
    if (s + 4 <= k) { batch(std::integral_constant<int, 4>{}, s); s += 4; }
    if (s + 2 <= k) { batch(std::integral_constant<int, 2>{}, s); s += 2; }
    if (s < k) batch(std::integral_constant<int, 1>{}, s);
    for (int s = 0; s < n_extra; ++s) fma_row(extra + (size_t)s * extra_stride + (size_t)t * H, 1.0f);
    uint4 o;
    o.x = pack_bf16x2(acc[0], acc[1]);
    o.y = pack_bf16x2(acc[2], acc[3]);
    o.z = pack_bf16x2(acc[4], acc[5]);
    o.w = pack_bf16x2(acc[6], acc[7]);
    *reinterpret_cast<uint4*>(out + (size_t)t * H + col) = o;
}

hipError_t launch_combine(const bf16_t* y, const int* inv_perm, const float* topk_w, int T, int k, int H,
                          const bf16_t* extra, int n_extra, long long extra_stride, bf16_t* out, hipStream_t st) {
    const dim3 grid(T, (H + 1023) / 1024), block(128);
    hipLaunchKernelGGL(combine_kernel, grid, block, 0, st, y, inv_perm, topk_w, k, H, extra, n_extra, extra_stride,
                       out);
    return hipGetLastError();
}

}  // namespace vismoe
