// Kernel group (2), generic form: one workgroup per (batch, query head h, query block m) runs
// the whole of Sec. 3.2-3.3 for that row of the block mask without materialising the stride
// score matrix:
//
//   A  scores of the R = B/S sampled queries of block m (Sec. 3.1 positions) against the stride
//      sums of every causal key stride, in chunks; per (sampled query r, key block n) the chunk
//      is reduced at once to a softmax partial (max, sum of exp) -- the "state".
//   B  row maxima and denominators of the causal stride softmax from the state.
//   C  block mass S[m][n] = sum_r state[r][n] rescaled to the row's max / denominator, and its
//      fraction of the row total.
//   D  Top-tau: bitonic sort of (mass descending, index ascending), prefix sum, first prefix
//      reaching tau; the last query block keeps every block when protection is on.
//   E  dense mask row, ascending compacted list and count.
//
// Works for any S | B | L, any d (multiple of 4 for fp32 rows), any group size; fp32 throughout.
// The MFMA path covers the benchmark shapes; this one covers everything else and is the
// reference point inside the library.
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kThreads = 256;
constexpr size_t kLdsBudget = 150 * 1024;     // of the 160 KB a workgroup can address

struct EstPlan {
    int Rp;          // R rounded up to a multiple of 8 (zero rows appended)
    int CH;          // key strides per chunk (multiple of R)
    int NbP2;        // power of two >= Nb
    int state_in_lds;
    unsigned off_qs, off_sc, off_state, off_keys, off_frac, off_flags, off_scan, off_rows, total;
};

// `pre`: the softmax state was already produced (MFMA score kernel) and lies in the workspace
// in [n][r] order; the plan then holds the selection buffers only.
__host__ EstPlan make_plan(const Geom& g, int S, int B, bool pre = false) {
    EstPlan p;
    const int R = B / S, Nb = g.L / B;
    p.Rp = (R + 7) / 8 * 8;
    int cap = 8192 / R;
    if (cap > 256) cap = 256;
    p.CH = cap / R * R;
    if (p.CH < R) p.CH = R;
    p.NbP2 = 1;
    while (p.NbP2 < Nb) p.NbP2 <<= 1;
    unsigned o = 0;
    auto take = [&](size_t bytes) { unsigned at = o; o += (unsigned)((bytes + 15) / 16 * 16); return at; };
    p.off_qs = take(pre ? 0 : (size_t)p.Rp * g.d * 4);
    p.off_sc = take(pre ? 0 : (size_t)R * p.CH * 4);
    p.off_keys = take((size_t)p.NbP2 * 8);
    p.off_frac = take((size_t)p.NbP2 * 4);
    p.off_flags = take((size_t)p.NbP2 * 4);
    p.off_scan = take((size_t)kThreads * 4 * 2);
    p.off_rows = take((size_t)R * 8 + 64);
    // the softmax state stays in LDS when it fits beside the rest, else it lives in the workspace
    p.state_in_lds = (!pre && o + (size_t)R * Nb * sizeof(float2) <= kLdsBudget) ? 1 : 0;
    p.off_state = take(p.state_in_lds ? (size_t)R * Nb * 8 : 0);
    p.total = o;
    return p;
}

// exclusive prefix sum of one value per thread over the 256 threads of the workgroup;
// `buf` holds 2 * 256 words; returns the exclusive prefix and writes the total to *total.
template <typename V>
__device__ V block_exclusive_scan(V v, V* buf, V* total) {
    const int t = threadIdx.x;
    V* a = buf;
    V* b = buf + kThreads;
    a[t] = v;
    __syncthreads();
    for (int o = 1; o < kThreads; o <<= 1) {
        V x = a[t];
        if (t >= o) x += a[t - o];
        b[t] = x;
        __syncthreads();
        V* tmp = a; a = b; b = tmp;
    }
    V incl = a[t];
    *total = a[kThreads - 1];
    __syncthreads();
    return incl - v;
}

// kExt = false compiles the packed-sequence table and the cut diagonal stride out (the plain method).
template <typename T, bool kExt>
__global__ void __launch_bounds__(kThreads)
k_estimate_generic(Geom g, EstimateArgs a, EstPlan p, float scale) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int32_t* const seq_first = kExt ? a.seq_first : nullptr;
    const bool diag_token = kExt && a.diag_token != 0;
    float* qs = reinterpret_cast<float*>(lds + p.off_qs);
    float* sc = reinterpret_cast<float*>(lds + p.off_sc);
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(lds + p.off_keys);
    float* frac = reinterpret_cast<float*>(lds + p.off_frac);
    int* flags = reinterpret_cast<int*>(lds + p.off_flags);
    float* scanbuf = reinterpret_cast<float*>(lds + p.off_scan);
    float* rowM = reinterpret_cast<float*>(lds + p.off_rows);
    float* rowZ = rowM + a.R;                        // reciprocal of the denominator of each sampled query
    int* misc = reinterpret_cast<int*>(rowZ + a.R);

    const int t = threadIdx.x;
    const int m = a.Nb - 1 - (int)blockIdx.x;      // heaviest rows first; the grid covers the Lq/B query blocks
    const int h = blockIdx.y, b = blockIdx.z;
    const int kv = h / g.G;
    const int R = a.R, S = a.S, Nb = a.Nb, d = g.d, CH = p.CH;
    const int Ls = g.L / S;
    const int Nbq = g.Lq / a.B;                      // rows of the mask (chunked prefill: < Nb)
    const long long row_id = ((long long)b * g.Hq + h) * Nbq + (m - (Nb - Nbq));
    // packed sequences: row m sees the key blocks nlo .. m of its own sequence; it is that sequence's last
    // query block when the next block starts another one.  A malformed table only gives a wrong row.
    int nlo = seq_first ? seq_first[m] : 0;
    nlo = nlo < 0 ? 0 : (nlo > m ? m : nlo);
    const bool last_of_seq = (m == Nb - 1) || (seq_first && seq_first[m + 1] == m + 1);
    const int mcnt = m + 1 - nlo;                  // causal key blocks of the row
    // sampled queries of this block that exist: its strides that are complete within the real length
    // (fewer than R only in a partial last block; none at all: the row has no estimate and keeps every block)
    int Rv = g.Lr / S - m * R;
    Rv = Rv < 0 ? 0 : (Rv > R ? R : Rv);

    float2* state = p.state_in_lds ? reinterpret_cast<float2*>(lds + p.off_state)
                                   : a.state_ws + row_id * R * Nb;
    const bool pre = a.state_precomputed != 0;     // state already in the workspace, [n][r] order
    auto sidx = [&](int r, int n) -> long long {
        return pre ? (long long)n * R + r : (long long)r * Nb + n;
    };
    const float NEG_INF = -__builtin_huge_valf();

    if (!pre) {

    // ---- sampled queries of this block: position (m*R + r)*S + S-1-(h mod S), Sec. 3.1 ----
    const T* Q = reinterpret_cast<const T*>(a.Q) + b * g.qsb + h * g.qsh;
    const int off = S - 1 - ((a.off_hmul * h + a.off_add) % S);
    for (int idx = t; idx < p.Rp * d; idx += kThreads) {
        const int r = idx / d, c = idx - r * d;
        float v = 0.f;
        if (r < Rv) v = Elem<T>::load1(Q + ((long long)(m * R + r) * S + off - g.q0) * g.qsl + c);
        qs[idx] = v;
    }
    __syncthreads();

    // ---- A: stride scores, reduced per (sampled query, key block) to (max, sum exp) ----
    const float* Ksum = a.Ksum + ((long long)(b * g.Hkv + kv) * Ls) * d;
    const int nstr = (m + 1) * R;
    for (int c0 = nlo * R; c0 < nstr; c0 += CH) {
        if (t < CH && c0 + t < nstr) {
            const int j = c0 + t;
            const float* kp = Ksum + (long long)j * d;
            for (int r0 = 0; r0 < p.Rp; r0 += 8) {
                float acc[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc[u] = 0.f;
                for (int dc = 0; dc < d; dc += 4) {
                    const f32x4 k4 = *reinterpret_cast<const f32x4*>(kp + dc);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const f32x4 q4 = *reinterpret_cast<const f32x4*>(qs + (r0 + u) * d + dc);
                        acc[u] = fmaf(q4[0], k4[0], acc[u]);
                        acc[u] = fmaf(q4[1], k4[1], acc[u]);
                        acc[u] = fmaf(q4[2], k4[2], acc[u]);
                        acc[u] = fmaf(q4[3], k4[3], acc[u]);
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = r0 + u;
                    if (r < R) {
                        const int i = m * R + r;                  // query stride index
                        sc[r * CH + t] = (j <= i) ? acc[u] * scale : NEG_INF;   // causal at stride level
                    }
                }
            }
        }
        __syncthreads();
        if (diag_token && t < Rv) {
            // alternative reading of the diagonal stride: the query at position i*S + off is scored against
            // the keys i*S .. i*S + off of its own stride only (the default sums the whole stride)
            const int i = m * R + t;
            if (i >= c0 && i < c0 + CH) {
                const T* Kd = reinterpret_cast<const T*>(a.K) + b * g.ksb + kv * g.ksh + (long long)i * S * g.ksl;
                float acc = 0.f;
                for (int s = 0; s <= off; ++s)
                    for (int c = 0; c < d; ++c) acc = fmaf(qs[t * d + c], Elem<T>::load1(Kd + (long long)s * g.ksl + c), acc);
                sc[t * CH + (i - c0)] = acc * scale;
            }
        }
        if (diag_token) __syncthreads();
        const int nbc = CH / R;
        for (int pidx = t; pidx < R * nbc; pidx += kThreads) {
            const int nbl = pidx / R, r = pidx - nbl * R;
            const int n = c0 / R + nbl;
            if (n <= m) {
                const float* s = sc + r * CH + nbl * R;
                float mx = NEG_INF;
                for (int jj = 0; jj < R; ++jj) mx = fmaxf(mx, s[jj]);
                float e = 0.f;
                for (int jj = 0; jj < R; ++jj) e += expf(s[jj] - mx);   // exp(-inf) = 0 for masked strides
                state[(long long)r * Nb + n] = make_float2(mx, e);
            }
        }
        __syncthreads();
    }
    }  // !pre

    // ---- B: row maximum and denominator of the causal stride softmax ----
    if (pre) {
        // the score kernel already reduced every sampled query's row
        if (t < Rv) {
            const float2 ms = a.rowstat[row_id * R + t];
            rowM[t] = ms.x;
            rowZ[t] = 1.0f / ms.y;                  // phase C multiplies by the reciprocal
        }
    } else {
        const int w = t >> 6, lane = t & 63;
        for (int r = w; r < R; r += kThreads / 64) {
            float mx = NEG_INF;
            for (int n = nlo + lane; n <= m; n += 64) mx = fmaxf(mx, state[(long long)r * Nb + n].x);
            mx = wave_max(mx);
            float z = 0.f;
            for (int n = nlo + lane; n <= m; n += 64) {
                const float2 v = state[(long long)r * Nb + n];
                z += v.y * expf(v.x - mx);
            }
            z = wave_sum(z);
            if (lane == 0) { rowM[r] = mx; rowZ[r] = 1.0f / z; }
        }
    }
    __syncthreads();

    // ---- C: block mass and its fraction of the row total ----
    float part = 0.f;
    for (int n = nlo + t; n <= m; n += kThreads) {
        float mass = 0.f;
        for (int r = 0; r < Rv; ++r) {
            const float2 v = state[sidx(r, n)];
            // hardware exp2 of the scaled difference and a multiply: this line runs R times per key block
            mass += v.y * __builtin_amdgcn_exp2f((v.x - rowM[r]) * 1.4426950408889634f) * rowZ[r];
        }
        frac[n] = mass;
        part += mass;
    }
    part = wave_sum(part);
    if ((t & 63) == 0) scanbuf[t >> 6] = part;
    __syncthreads();
    const float total = scanbuf[0] + scanbuf[1] + scanbuf[2] + scanbuf[3];
    __syncthreads();
    for (int n = nlo + t; n <= m; n += kThreads) frac[n] = Rv > 0 ? frac[n] / total : 0.f;
    __syncthreads();
    if (a.block_mass) {
        float* bm = a.block_mass + row_id * Nb;
        for (int n = t; n < Nb; n += kThreads) bm[n] = (n >= nlo && n <= m) ? frac[n] : 0.f;
    }

    // ---- D: Top-tau ----
    const bool keep_all = (a.tau >= 1.0f) || (a.protect_last && last_of_seq) || Rv == 0;
    if (keep_all) {
        for (int n = t; n < Nb; n += kThreads) flags[n] = (n >= nlo && n <= m) ? 1 : 0;
        __syncthreads();
    } else {
        // sorted position i holds key block nlo + i before the sort
        int P2 = 1;
        while (P2 < mcnt) P2 <<= 1;
        for (int i = t; i < P2; i += kThreads) {
            unsigned long long key = ~0ull;
            if (i < mcnt) key = ((unsigned long long)(~__float_as_uint(frac[nlo + i])) << 32) | (unsigned)(nlo + i);
            keys[i] = key;
        }
        __syncthreads();
        for (int k = 2; k <= P2; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                // one compare-exchange per loop trip: pair p is (i, i + j) with bit j of i clear; every lane works,
                // and the exchange is two selects instead of a divergent branch
                for (int p2 = t; p2 < (P2 >> 1); p2 += kThreads) {
                    const int i = ((p2 & ~(j - 1)) << 1) | (p2 & (j - 1));
                    const int x = i | j;
                    const unsigned long long ka = keys[i], kb = keys[x];
                    const bool sw = (ka > kb) == ((i & k) == 0);
                    keys[i] = sw ? kb : ka;
                    keys[x] = sw ? ka : kb;
                }
                __syncthreads();
            }
        }
        // inclusive prefix of the sorted fractions; thread t owns a contiguous segment
        const int seg = (P2 + kThreads - 1) / kThreads;
        const int lo = t * seg;
        float local = 0.f;
        for (int i = lo; i < lo + seg && i < mcnt; ++i) local += __uint_as_float(~(unsigned)(keys[i] >> 32));
        float dummy;
        float run = block_exclusive_scan<float>(local, scanbuf, &dummy);
        if (t == 0) misc[0] = mcnt;                      // keep all if tau is never reached
        __syncthreads();
        // smallest prefix length reaching tau.  The minimum over all threads, not "the thread that
        // sees the crossing": a thread's starting value comes from the tree-ordered scan while its
        // neighbour's last value is a sequential sum, so the two can round to different sides of tau.
        for (int i = lo; i < lo + seg && i < mcnt; ++i) {
            run += __uint_as_float(~(unsigned)(keys[i] >> 32));
            if (run >= a.tau) { atomicMin(&misc[0], i + 1); break; }
        }
        for (int n = t; n < Nb; n += kThreads) flags[n] = 0;
        __syncthreads();
        const int kstar = misc[0];
        for (int i = t; i < kstar; i += kThreads) flags[(unsigned)(keys[i] & 0xFFFFFFFFu)] = 1;
        __syncthreads();
    }

    // sink / recent blocks are added after the selection (a union)
    if (a.sink_blocks > 0 || a.recent_blocks > 0) {
        for (int n = nlo + t; n <= m; n += kThreads)
            if (n - nlo < a.sink_blocks || n > m - a.recent_blocks) flags[n] = 1;
        __syncthreads();
    }

    // ---- E: outputs ----
    if (a.dense) {
        uint8_t* row = a.dense + row_id * Nb;
        for (int n = t; n < Nb; n += kThreads) row[n] = (uint8_t)flags[n];
    }
    {
        const int seg = (m + 1 + kThreads - 1) / kThreads;
        const int lo = t * seg;
        int cnt = 0;
        for (int n = lo; n < lo + seg && n <= m; ++n) cnt += flags[n];
        int total_cnt;
        int pos = block_exclusive_scan<int>(cnt, reinterpret_cast<int*>(scanbuf), &total_cnt);
        int32_t* list = a.row_list + row_id * Nb;
        for (int n = lo; n < lo + seg && n <= m; ++n)
            if (flags[n]) list[pos++] = n;
        if (t == 0) a.row_count[row_id] = total_cnt;
    }
}

}  // namespace

bool estimate_generic_fits(const Geom& g, int S, int B, bool state_precomputed) {
    return make_plan(g, S, B, state_precomputed).total <= kLdsBudget;
}

size_t estimate_generic_state_bytes(const Geom& g, int S, int B) {
    const EstPlan p = make_plan(g, S, B);
    if (p.state_in_lds) return 0;
    return (size_t)g.batch * g.Hq * (g.Lq / B) * (B / S) * (g.L / B) * sizeof(float2);
}

hipError_t launch_estimate_generic(const Geom& g, int dtype, const EstimateArgs& a, hipStream_t st) {
    const EstPlan p = make_plan(g, a.S, a.B, a.state_precomputed != 0);
    const float scale = (float)(1.0 / ((double)a.S * sqrt((double)g.d)));
    dim3 grid(g.Lq / a.B, g.Hq, g.batch);
    const bool ext = a.seq_first != nullptr || a.diag_token != 0;
    auto launch = [&](auto kernel) -> hipError_t {
        hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.total);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), p.total, st, g, a, p, scale);
        return hipGetLastError();
    };
    if (dtype == RR_BF16) return ext ? launch(k_estimate_generic<bf16_t, true>) : launch(k_estimate_generic<bf16_t, false>);
    return ext ? launch(k_estimate_generic<float, true>) : launch(k_estimate_generic<float, false>);
}

}  // namespace rr
