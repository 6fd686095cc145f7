// Kernel group (3), generic form: causal block-sparse attention (Sec. 2.1) in fp32 on the
// vector ALUs, for every shape the MFMA kernel does not take (fp32 tensors, d != 128, B != 128).
//
// One workgroup per (batch, head, query block m).  The query block, the running output and one
// key/value block at a time live in LDS as fp32; each of the four waves takes four query rows at
// a time and walks them over the staged block with an online softmax: lane j scores key j (and
// j+64) against the four rows, the wave reduces max and sum, lane c then accumulates output
// column c (c+64, ...) of the four rows.  Token causality (j <= i) is applied inside the diagonal block only.
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kRows = 4;                 // query rows a wave works on at a time

template <typename T>
__global__ void __launch_bounds__(kThreads)
k_attn_generic(Geom g, AttnArgs a, float scale) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int B = a.B, d = g.d, Nb = a.Nb;
    const int dk = d + 1;                                    // padded key rows: lane j reads row j
    float* Qs = reinterpret_cast<float*>(lds);               // [B][d]
    float* Os = Qs + B * d;                                  // [B][d]
    float* Ks = Os + B * d;                                  // [B][d+1]
    float* Vs = Ks + B * dk;                                 // [B][d]
    float* Ps = Vs + B * d;                                  // [kWaves][kRows][B]
    float* Ms = Ps + kWaves * kRows * B;                     // [B] running max
    float* Lsum = Ms + B;                                    // [B] running denominator

    const int t = threadIdx.x, w = t >> 6, lane = t & 63;
    const int Nbq = g.Lq / B;                         // rows of the launch (chunked prefill: the last query blocks)
    const int m = Nb - 1 - (int)blockIdx.x;
    const int mq = m - (Nb - Nbq);
    const int h = blockIdx.y, b = blockIdx.z;
    const int kv = h / g.G;
    const long long row_id = ((long long)b * g.Hq + h) * Nbq + mq;
    // row x of the block (position m B + x) is row mq B + x - qoff of Q and O: a step that starts inside its
    // first block has no rows for the first qoff positions of that block
    const long long row0 = (long long)mq * B - g.qoff;
    const T* Q = reinterpret_cast<const T*>(a.Q) + b * g.qsb + h * g.qsh + row0 * g.qsl;
    const T* K = reinterpret_cast<const T*>(a.K) + b * g.ksb + kv * g.ksh;
    const T* V = reinterpret_cast<const T*>(a.V) + b * g.ksb + kv * g.ksh;
    T* O = reinterpret_cast<T*>(a.O) + b * g.qsb + h * g.qsh + row0 * g.qsl;
    const float NEG_INF = -__builtin_huge_valf();
    constexpr int VEC = Elem<T>::kVec;
    const int chunks = d / VEC;

    // rows that do not exist (past the real length, in front of the step) are computed on a copy of the nearest
    // real row and not stored: the real rows of this block are x = rows_lo .. rows_q - 1 (at least one)
    const int rows_lo = mq == 0 ? g.qoff : 0;
    const int rows_q = (int)min((long long)B, (long long)(g.Lr - g.q0) - row0);
    for (int idx = t; idx < B * chunks; idx += kThreads) {
        const int r = idx / chunks, c = (idx - r * chunks) * VEC;
        float v[VEC];
        Elem<T>::load16(Q + (long long)max(min(r, rows_q - 1), rows_lo) * g.qsl + c, v);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { Qs[r * d + c + i] = v[i]; Os[r * d + c + i] = 0.f; }
    }
    for (int r = t; r < B; r += kThreads) { Ms[r] = NEG_INF; Lsum[r] = 0.f; }

    // a caller-made list is not trusted with addresses: count held to [0, m+1], entries to [0, m]
    int first = (!a.row_list && a.seq_first) ? a.seq_first[m] : 0;   // dense walk of packed sequences
    first = first < 0 ? 0 : (first > m ? m : first);
    int count = a.row_list ? a.row_count[row_id] : (m + 1 - first);
    count = count < 0 ? 0 : (count > m + 1 ? m + 1 : count);
    const int32_t* list = a.row_list ? a.row_list + row_id * Nb : nullptr;

    for (int it = 0; it < count; ++it) {
        int n = list ? list[it] : first + it;
        n = n < 0 ? 0 : (n > m ? m : n);
        __syncthreads();                                      // previous block fully consumed
        for (int idx = t; idx < B * chunks; idx += kThreads) {
            const int r = idx / chunks, c = (idx - r * chunks) * VEC;
            float kvv[VEC], vv[VEC];
            const long long krow = min(n * B + r, g.Lr - 1);   // keys past the real length: only in the diagonal block, masked there
            Elem<T>::load16(K + krow * g.ksl + c, kvv);
            Elem<T>::load16(V + krow * g.ksl + c, vv);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { Ks[r * dk + c + i] = kvv[i]; Vs[r * d + c + i] = vv[i]; }
        }
        __syncthreads();
        const bool diag = (n == m);
        // four query rows at a time per wave: every key / value element read from LDS feeds four FMAs
        float* P = Ps + w * (kRows * B);
        for (int r0 = kRows * w; r0 < B; r0 += kRows * kWaves) {
            float mx[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) mx[u] = NEG_INF;
            for (int j = lane; j < B; j += 64) {
                float s[kRows];
#pragma unroll
                for (int u = 0; u < kRows; ++u) s[u] = 0.f;
                const float* k = Ks + j * dk;
                for (int c = 0; c < d; ++c) {
                    const float kc = k[c];
#pragma unroll
                    for (int u = 0; u < kRows; ++u) s[u] = fmaf(Qs[min(r0 + u, B - 1) * d + c], kc, s[u]);
                }
#pragma unroll
                for (int u = 0; u < kRows; ++u) {
                    float v = s[u] * scale;
                    if (diag && j > r0 + u) v = NEG_INF;      // token causality inside the diagonal block
                    P[u * B + j] = v;
                    mx[u] = fmaxf(mx[u], v);
                }
            }
            float alpha[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int r = min(r0 + u, B - 1);
                mx[u] = wave_max(mx[u]);
                const float m_old = Ms[r];
                const float m_new = fmaxf(m_old, mx[u]);      // finite: key 0 of a block is visible to every row
                float lsum = 0.f;
                for (int j = lane; j < B; j += 64) {
                    const float p = expf(P[u * B + j] - m_new);
                    P[u * B + j] = p;
                    lsum += p;
                }
                lsum = wave_sum(lsum);
                alpha[u] = expf(m_old - m_new);               // exp(-inf) = 0 on the first block
                if (lane == 0 && r0 + u < B) { Ms[r] = m_new; Lsum[r] = Lsum[r] * alpha[u] + lsum; }
            }
            for (int c = lane; c < d; c += 64) {
                float acc[kRows];
#pragma unroll
                for (int u = 0; u < kRows; ++u) acc[u] = Os[min(r0 + u, B - 1) * d + c] * alpha[u];
                for (int j = 0; j < B; ++j) {
                    const float vj = Vs[j * d + c];
#pragma unroll
                    for (int u = 0; u < kRows; ++u) acc[u] = fmaf(P[u * B + j], vj, acc[u]);
                }
#pragma unroll
                for (int u = 0; u < kRows; ++u)
                    if (r0 + u < B) Os[(r0 + u) * d + c] = acc[u];
            }
        }
    }
    __syncthreads();
    for (int idx = rows_lo * d + t; idx < rows_q * d; idx += kThreads) {
        const int r = idx / d, c = idx - r * d;
        const float l = Lsum[r];
        Elem<T>::store1(O + (long long)r * g.qsl + c, l > 0.f ? Os[idx] / l : 0.f);
    }
    if (a.lse) {
        float* lse = a.lse + ((long long)b * g.Hq + h) * (g.Lr - g.q0) + row0;
        for (int r = rows_lo + t; r < rows_q; r += kThreads) lse[r] = Lsum[r] > 0.f ? Ms[r] + logf(Lsum[r]) : NEG_INF;
    }
}

size_t attn_generic_lds(int B, int d) {
    return sizeof(float) * ((size_t)B * d * 3 + (size_t)B * (d + 1) + (size_t)kWaves * kRows * B + 2 * (size_t)B);
}

}  // namespace

bool attn_generic_fits(int B, int d) { return attn_generic_lds(B, d) <= 150 * 1024; }

hipError_t launch_attn_generic(const Geom& g, int dtype, const AttnArgs& a, hipStream_t st) {
    const size_t lds = attn_generic_lds(a.B, g.d);
    const float scale = (float)(1.0 / sqrt((double)g.d));
    dim3 grid(g.Lq / a.B, g.Hq, g.batch);
    hipError_t e;
    if (dtype == RR_BF16) {
        e = allow_dynamic_lds((const void*)k_attn_generic<bf16_t>, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_attn_generic<bf16_t>, grid, dim3(kThreads), lds, st, g, a, scale);
    } else {
        e = allow_dynamic_lds((const void*)k_attn_generic<float>, lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_attn_generic<float>, grid, dim3(kThreads), lds, st, g, a, scale);
    }
    return hipGetLastError();
}

}  // namespace rr
