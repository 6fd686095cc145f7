// Block selection accuracy of a block mask against full attention (appendix "Block Selection
// Accuracy Analysis"): for a query i the ground truth K*_i is a smallest set of key positions whose
// causal softmax attention sums to >= tau (taken by descending attention, equal values by smaller
// position first), the prediction K_i is every position j <= i of the key blocks the mask selects
// for the query's block row; precision_i = |K_i n K*_i| / |K_i|, recall_i = |K_i n K*_i| / |K*_i|,
// averaged over the sampled queries i = step-1, 2 step-1, ...; F1 from the two averages.
//
// A diagnostic, not part of the prefill path.  One workgroup per sampled query: the attention row
// is computed in fp32 into a workspace row, the threshold value of K*_i is found by bisection on
// the bit pattern of the (positive) attention values -- the largest value t whose upper set
// {A >= t} still holds mass >= tau -- and the few ties at t are resolved by position.
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kThreads = 256;

// sum of one float per thread over the workgroup, same order every time; `buf` holds 4 floats
__device__ __forceinline__ float block_sum(float v, float* buf) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
    __syncthreads();
    return (buf[0] + buf[1]) + (buf[2] + buf[3]);
}
__device__ __forceinline__ float block_max(float v, float* buf) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(buf[0], buf[1]), fmaxf(buf[2], buf[3]));
}
__device__ __forceinline__ int block_sum_int(int v, int* buf) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
    __syncthreads();
    return buf[0] + buf[1] + buf[2] + buf[3];
}

struct AccArgs {
    const void* Q; const void* K;
    const int32_t* row_count; const int32_t* row_list;
    float* rows;          // [batch*Hq*ns][L] attention rows (scratch)
    float2* per_query;    // [batch*Hq*ns] (precision_i, recall_i)
    int B, Nb, step, ns;
    float tau, scale;
};

template <typename T>
__global__ void __launch_bounds__(kThreads)
k_accuracy_rows(Geom g, AccArgs a) {
    __shared__ float q[256];
    __shared__ float redf[4];
    __shared__ int redi[4];
    __shared__ int tie_pos;
    const int t = threadIdx.x;
    const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int i = g.q0 + (s + 1) * a.step - 1;          // the query position inside the context
    const int n = i + 1;                                // causal row length
    const int m = i / a.B;
    const int kv = h / g.G;
    const long long sample = ((long long)b * g.Hq + h) * a.ns + s;
    float* A = a.rows + sample * g.L;
    const T* Qp = reinterpret_cast<const T*>(a.Q) + b * g.qsb + h * g.qsh + (long long)(i - g.q0) * g.qsl;
    const T* Kp = reinterpret_cast<const T*>(a.K) + b * g.ksb + kv * g.ksh;
    for (int c = t; c < g.d; c += kThreads) q[c] = Elem<T>::load1(Qp + c);
    __syncthreads();

    // ---- scores, maximum, denominator, attention values ----
    float lmax = -__builtin_huge_valf();
    for (int j = t; j < n; j += kThreads) {
        const T* kr = Kp + (long long)j * g.ksl;
        float acc = 0.f;
        for (int c = 0; c < g.d; c += Elem<T>::kVec) {
            float kvv[8];
            Elem<T>::load16(kr + c, kvv);
#pragma unroll
            for (int e = 0; e < Elem<T>::kVec; ++e) acc = fmaf(q[c + e], kvv[e], acc);
        }
        acc *= a.scale;
        A[j] = acc;
        lmax = fmaxf(lmax, acc);
    }
    const float M = block_max(lmax, redf);
    float lz = 0.f;
    for (int j = t; j < n; j += kThreads) lz += expf(A[j] - M);
    const float Z = block_sum(lz, redf);
    for (int j = t; j < n; j += kThreads) A[j] = expf(A[j] - M) / Z;      // each thread rereads its own writes

    // ---- threshold of K*: the largest value t with mass{A >= t} >= tau ----
    auto mass_ge = [&](unsigned bits) {
        float ls = 0.f;
        for (int j = t; j < n; j += kThreads) {
            const float v = A[j];
            if (__float_as_uint(v) >= bits) ls += v;
        }
        return block_sum(ls, redf);
    };
    unsigned lo = 0u, hi = 0x7F800000u;                 // mass_ge(hi) = 0 < tau
    const bool reachable = mass_ge(0u) >= a.tau;       // else (tau ~ 1 and rounding): every position
    if (reachable) {
        while (hi - lo > 1u) {
            const unsigned mid = lo + ((hi - lo) >> 1);
            if (mass_ge(mid) >= a.tau) lo = mid; else hi = mid;
        }
    }
    const float thr = __uint_as_float(lo);
    float lgt = 0.f;
    int cgt = 0, ceq = 0;
    for (int j = t; j < n; j += kThreads) {
        const float v = A[j];
        if (v > thr) { lgt += v; ++cgt; }
        else if (v == thr) ++ceq;
    }
    const float mass_gt = block_sum(lgt, redf);
    const int cnt_gt = block_sum_int(cgt, redi);
    const int n_eq = block_sum_int(ceq, redi);
    // ties needed: the smallest c with mass_gt + c * thr >= tau
    int c = n_eq;
    if (reachable && thr > 0.f) {
        c = (int)ceilf((a.tau - mass_gt) / thr);
        c = c < 1 ? 1 : (c > n_eq ? n_eq : c);
        while (c > 1 && mass_gt + (float)(c - 1) * thr >= a.tau) --c;
        while (c < n_eq && mass_gt + (float)c * thr < a.tau) ++c;
    }
    const int star = cnt_gt + c;

    // position of the c-th tie (ties beyond it are not in K*); all ties are in when c == n_eq
    int last_tie = n;                                   // ties at positions <= last_tie count
    if (c < n_eq) {
        if (t == 0) tie_pos = n;
        int seen = 0;
        for (int j0 = 0; j0 < n; j0 += kThreads) {      // chunks in position order
            const int j = j0 + t;
            const int flag = (j < n && A[j] == thr) ? 1 : 0;
            // inclusive rank of this tie inside the chunk
            int incl = flag;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int up = __shfl_up(incl, o);
                if ((t & 63) >= o) incl += up;
            }
            __syncthreads();
            if ((t & 63) == 63) redi[t >> 6] = incl;
            __syncthreads();
            int before = seen;
            for (int w = 0; w < (t >> 6); ++w) before += redi[w];
            if (flag && before + incl == c) tie_pos = j;
            seen += redi[0] + redi[1] + redi[2] + redi[3];
            if (seen >= c) break;                       // uniform: every thread has the same `seen`
        }
        __syncthreads();
        last_tie = tie_pos;
    }

    // ---- predicted set: positions j <= i of the selected blocks of row (h, m) ----
    const int Nbq = g.Lq / a.B;
    const long long row_id = ((long long)b * g.Hq + h) * Nbq + (m - (a.Nb - Nbq));
    int cnt = a.row_count[row_id];                       // held to [0, m+1], entries to [0, m]: no stray reads
    cnt = cnt < 0 ? 0 : (cnt > m + 1 ? m + 1 : cnt);
    const int32_t* list = a.row_list + row_id * a.Nb;
    int linter = 0, lpred = 0;
    for (int idx = t; idx < cnt * a.B; idx += kThreads) {
        int blk = list[idx / a.B];
        blk = blk < 0 ? 0 : (blk > m ? m : blk);
        const int j = blk * a.B + idx % a.B;
        if (j <= i) {
            ++lpred;
            const float v = A[j];
            if (v > thr || (v == thr && j <= last_tie)) ++linter;
        }
    }
    const int inter = block_sum_int(linter, redi);
    const int pred = block_sum_int(lpred, redi);
    if (t == 0)
        a.per_query[sample] = make_float2(pred > 0 ? (float)inter / (float)pred : 0.f, (float)inter / (float)star);
}

// mean precision, mean recall and their F1 per (batch, head)
__global__ void __launch_bounds__(kThreads)
k_accuracy_reduce(const float2* __restrict__ per_query, int ns, float* __restrict__ out) {
    __shared__ float redf[4];
    const long long bh = blockIdx.x;
    float lp = 0.f, lr = 0.f;
    for (int s = threadIdx.x; s < ns; s += kThreads) {
        const float2 v = per_query[bh * ns + s];
        lp += v.x;
        lr += v.y;
    }
    const float p = block_sum(lp, redf) / (float)ns;
    const float r = block_sum(lr, redf) / (float)ns;
    if (threadIdx.x == 0) {
        out[bh * 3 + 0] = p;
        out[bh * 3 + 1] = r;
        out[bh * 3 + 2] = (p + r > 0.f) ? 2.f * p * r / (p + r) : 0.f;
    }
}

}  // namespace

size_t accuracy_rows_bytes(const Geom& g, int step) {
    return (size_t)g.batch * g.Hq * (g.Lq / step) * g.L * sizeof(float);
}
size_t accuracy_per_query_bytes(const Geom& g, int step) {
    return (size_t)g.batch * g.Hq * (g.Lq / step) * sizeof(float2);
}

hipError_t launch_selection_accuracy(const Geom& g, int dtype, const void* Q, const void* K,
                                     const int32_t* row_count, const int32_t* row_list, int B, float tau, int step,
                                     float* rows, float2* per_query, float* out, hipStream_t st) {
    AccArgs a;
    a.Q = Q; a.K = K; a.row_count = row_count; a.row_list = row_list;
    a.rows = rows; a.per_query = per_query;
    a.B = B; a.Nb = g.L / B; a.step = step; a.ns = g.Lq / step;
    a.tau = tau;
    a.scale = (float)(1.0 / sqrt((double)g.d));
    dim3 grid(a.ns, g.Hq, g.batch);
    if (dtype == RR_BF16) hipLaunchKernelGGL(k_accuracy_rows<bf16_t>, grid, dim3(kThreads), 0, st, g, a);
    else hipLaunchKernelGGL(k_accuracy_rows<float>, grid, dim3(kThreads), 0, st, g, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_accuracy_reduce, dim3(g.batch * g.Hq), dim3(kThreads), 0, st, per_query, a.ns, out);
    return hipGetLastError();
}

}  // namespace rr
