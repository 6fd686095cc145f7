// Kernel group (1): stride sums of the keys (inner sum of the importance equation, Sec. 3.2).
//
//   Ksum[b][g][j][c] = sum_{s=0}^{S-1} K[b][g][j*S + s][c]          (fp32, contiguous)
//
// HBM-bound: K is read exactly once with 16-byte loads (a row of d elements is covered by
// consecutive lanes, so every wave instruction reads whole 256-byte segments) and the fp32 sums
// are written once.  The 1/S of the mean is folded into the score scale by the consumer.
#include "rr_common.hpp"

namespace rr {

template <typename T>
__global__ void __launch_bounds__(256)
k_stride_sum(Geom g, const T* __restrict__ K, int S, int Ls, float* __restrict__ Ksum) {
    constexpr int V = Elem<T>::kVec;
    const int chunks = g.d / V;
    const long long total = (long long)g.batch * g.Hkv * Ls * chunks;
    long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % chunks);
    long long r = idx / chunks;
    const int j = (int)(r % Ls);
    r /= Ls;
    const int kv = (int)(r % g.Hkv);
    const int b = (int)(r / g.Hkv);
    const T* src = K + b * g.ksb + kv * g.ksh + (long long)j * S * g.ksl + c * V;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    // strides that are not complete within the real length do not exist (Sec. 3.1: floor(L/S) of them): zeros
    const int nkeys = (j + 1) * S <= g.Lr ? S : 0;
    for (int s = 0; s < nkeys; ++s) {
        float v[V];
        Elem<T>::load16(src + s * g.ksl, v);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += v[i];
    }
    float* dst = Ksum + (((long long)(b * g.Hkv + kv) * Ls + j) * g.d + c * V);
#pragma unroll
    for (int i = 0; i < V; i += 4) {
        f32x4 o = {acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
        *reinterpret_cast<f32x4*>(dst + i) = o;
    }
}

hipError_t launch_stride_sum(const Geom& g, int dtype, const void* K, int S, float* Ksum, hipStream_t st) {
    const int Ls = g.L / S;
    const int V = dtype == RR_BF16 ? 8 : 4;
    const long long total = (long long)g.batch * g.Hkv * Ls * (g.d / V);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == RR_BF16)
        hipLaunchKernelGGL(k_stride_sum<bf16_t>, dim3(blocks), dim3(256), 0, st, g, (const bf16_t*)K, S, Ls, Ksum);
    else
        hipLaunchKernelGGL(k_stride_sum<float>, dim3(blocks), dim3(256), 0, st, g, (const float*)K, S, Ls, Ksum);
    return hipGetLastError();
}

}  // namespace rr
