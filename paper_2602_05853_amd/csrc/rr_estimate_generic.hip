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
//   D  Top-tau by one wavefront (rr_select.hpp: threshold bisection instead of a sort), the last query
//      block keeps every block when protection is on; dense mask row, ascending list and count.
//
// Works for any S | B | L, any d (multiple of 4 for fp32 rows), any group size; fp32 throughout.
// The MFMA path covers the benchmark shapes; this one covers everything else and is the
// reference point inside the library.  k_select_rows is the selection stage of the MFMA path: the same
// phase D on block masses that the MFMA kernel left in the workspace.
#include "rr_common.hpp"
#include "rr_select.hpp"

namespace rr {

namespace {

constexpr int kThreads = 256;
constexpr size_t kLdsBudget = 150 * 1024;     // of the 160 KB a workgroup can address

struct EstPlan {
    int Rp;          // R rounded up to a multiple of 8 (zero rows appended)
    int CH;          // key strides per chunk (multiple of R)
    int NbP2;        // power of two >= Nb
    int state_in_lds;
    unsigned off_qs, off_sc, off_state, off_frac, off_scan, off_rows, total;
};

__host__ EstPlan make_plan(const Geom& g, int S, int B) {
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
    p.off_qs = take((size_t)p.Rp * g.d * 4);
    p.off_sc = take((size_t)R * p.CH * 4);
    p.off_frac = take((size_t)p.NbP2 * 4);
    p.off_scan = take(64);
    p.off_rows = take((size_t)R * 8 + 64);
    // the softmax state stays in LDS when it fits beside the rest, else it lives in the workspace
    p.state_in_lds = (o + (size_t)R * Nb * sizeof(float2) <= kLdsBudget) ? 1 : 0;
    p.off_state = take(p.state_in_lds ? (size_t)R * Nb * 8 : 0);
    p.total = o;
    return p;
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
    float* frac = reinterpret_cast<float*>(lds + p.off_frac);
    float* scanbuf = reinterpret_cast<float*>(lds + p.off_scan);
    float* rowM = reinterpret_cast<float*>(lds + p.off_rows);
    float* rowZ = rowM + a.R;                        // reciprocal of the denominator of each sampled query

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
    // ... and whose sampled position is not in front of the step's first query (a step that starts inside this
    // block): the sampled queries of the row are r = R0 .. Rv - 1
    const int off = S - 1 - ((a.off_hmul * h + a.off_add) % S);
    int R0 = g.q0 - off - m * R * S;
    R0 = R0 <= 0 ? 0 : (R0 + S - 1) / S;
    R0 = R0 > R ? R : R0;

    float2* state = p.state_in_lds ? reinterpret_cast<float2*>(lds + p.off_state)
                                   : a.state_ws + row_id * R * Nb;
    const float NEG_INF = -__builtin_huge_valf();

    // ---- sampled queries of this block: position (m*R + r)*S + S-1-(h mod S), Sec. 3.1 ----
    const T* Q = reinterpret_cast<const T*>(a.Q) + b * g.qsb + h * g.qsh;
    for (int idx = t; idx < p.Rp * d; idx += kThreads) {
        const int r = idx / d, c = idx - r * d;
        float v = 0.f;
        if (r >= R0 && r < Rv) v = Elem<T>::load1(Q + ((long long)(m * R + r) * S + off - g.q0) * g.qsl + c);
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
        if (diag_token && t >= R0 && t < Rv) {
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

    // ---- B: row maximum and denominator of the causal stride softmax ----
    {
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
        for (int r = R0; r < Rv; ++r) {
            const float2 v = state[(long long)r * Nb + n];
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
    for (int n = nlo + t; n <= m; n += kThreads) frac[n] = Rv > R0 ? frac[n] / total : 0.f;
    __syncthreads();
    if (a.block_mass) {
        float* bm = a.block_mass + row_id * Nb;
        for (int n = t; n < Nb; n += kThreads) bm[n] = (n >= nlo && n <= m) ? frac[n] : 0.f;
    }

    // ---- D: Top-tau, union with sink / recent blocks, outputs: one wavefront ----
    if (t < 64) {
        SelectRow r;
        r.nlo = nlo; r.m = m; r.Nb = Nb;
        r.tau = a.tau;
        r.keep_all = (a.tau >= 1.0f) || (a.protect_last && last_of_seq) || Rv <= R0;
        r.sink_blocks = a.sink_blocks; r.recent_blocks = a.recent_blocks;
        r.dense = a.dense ? a.dense + row_id * Nb : nullptr;
        r.list = a.row_list + row_id * Nb;
        r.count = a.row_count + row_id;
        select_row_wave(RowInLds(frac, nlo, m, t), r, t);
    }
}

// Selection stage of the MFMA path: one wavefront per mask row.  mass[row][n] holds the block masses
// (Sec. 3.3 block-importance equation: stride-softmax probabilities summed over the R x R strides of a
// block pair) for nlo <= n <= m; the row total normalises them, then phase D as above.
// NCH > 0: rows of up to 64 * NCH key blocks, held in registers; NCH = 0: any length, through LDS.
template <bool kExt, int NCH>
__global__ void __launch_bounds__(kThreads)
k_select_rows(Geom g, EstimateArgs a, const float* __restrict__ mass, long long rows) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int32_t* const seq_first = kExt ? a.seq_first : nullptr;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int Nb = a.Nb, Nbq = g.Lq / a.B;
    // heaviest rows (largest m) first; the four rows of a workgroup are neighbours in m
    const long long slot = (long long)blockIdx.x * (kThreads / 64) + w;
    if (slot >= rows) return;
    const int mq = Nbq - 1 - (int)(slot % Nbq);
    const long long bh = slot / Nbq;
    const long long row_id = bh * Nbq + mq;
    const int m = mq + (Nb - Nbq);
    int nlo = seq_first ? seq_first[m] : 0;
    nlo = nlo < 0 ? 0 : (nlo > m ? m : nlo);
    const bool last_of_seq = (m == Nb - 1) || (seq_first && seq_first[m + 1] == m + 1);
    const float* src = mass + row_id * Nb;
    // a row without a sampled query (a last block without one complete stride, a decode step that holds none of
    // its block's sampled positions) has no estimate, and nothing was written to its row of the workspace
    bool has_strides;
    {
        const int h = (int)(bh % g.Hq);
        const int off = a.S - 1 - ((a.off_hmul * h + a.off_add) % a.S);
        int r_hi = g.Lr / a.S - m * a.R;                       // strides of the block complete within the length
        r_hi = r_hi > a.R ? a.R : r_hi;
        int r_lo = g.q0 - off - m * a.R * a.S;                 // sampled positions not in front of the step
        r_lo = r_lo <= 0 ? 0 : (r_lo + a.S - 1) / a.S;
        has_strides = r_lo < r_hi;
    }
    SelectRow r;
    r.nlo = nlo; r.m = m; r.Nb = Nb;
    r.tau = a.tau;
    r.keep_all = (a.tau >= 1.0f) || (a.protect_last && last_of_seq);
    r.sink_blocks = a.sink_blocks; r.recent_blocks = a.recent_blocks;
    r.dense = a.dense ? a.dense + row_id * Nb : nullptr;
    r.list = a.row_list + row_id * Nb;
    r.count = a.row_count + row_id;
    float* bm = a.block_mass ? a.block_mass + row_id * Nb : nullptr;
    if (NCH > 0) {
        // the row fits in registers: 64 * NCH >= Nb
        RowInRegs<(NCH > 0 ? NCH : 1)> row;
        float part = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int n = 64 * c + lane;
            row.v[c] = (has_strides && n >= nlo && n <= m) ? src[n] : 0.f;
            part += row.v[c];
        }
        const float total = wave_sum_fixed(part);
        const bool estimated = total > 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            row.v[c] = estimated ? row.v[c] / total : 0.f;
            if (bm && 64 * c + lane < Nb) bm[64 * c + lane] = row.v[c];
        }
        r.keep_all = r.keep_all || !estimated;
        select_row_wave(row, r, lane);
    } else {
        float* frac = reinterpret_cast<float*>(lds) + (size_t)w * ((Nb + 63) / 64 * 64);
        float part = 0.f;
        for (int n = nlo + lane; n <= m; n += 64) {
            const float v = has_strides ? src[n] : 0.f;
            frac[n] = v;
            part += v;
        }
        const float total = wave_sum_fixed(part);
        const bool estimated = total > 0.f;
        for (int n = nlo + lane; n <= m; n += 64) frac[n] = estimated ? frac[n] / total : 0.f;
        if (bm)
            for (int n = lane; n < Nb; n += 64) bm[n] = (n >= nlo && n <= m) ? frac[n] : 0.f;
        r.keep_all = r.keep_all || !estimated;
        select_row_wave(RowInLds(frac, nlo, m, lane), r, lane);
    }
}

}  // namespace

bool estimate_generic_fits(const Geom& g, int S, int B) {
    return make_plan(g, S, B).total <= kLdsBudget;
}

size_t estimate_generic_state_bytes(const Geom& g, int S, int B) {
    const EstPlan p = make_plan(g, S, B);
    if (p.state_in_lds) return 0;
    return (size_t)g.batch * g.Hq * (g.Lq / B) * (B / S) * (g.L / B) * sizeof(float2);
}

hipError_t launch_estimate_generic(const Geom& g, int dtype, const EstimateArgs& a, hipStream_t st) {
    const EstPlan p = make_plan(g, a.S, a.B);
    const float scale = (float)(1.0 / ((double)a.S * sqrt((double)g.d)));
    dim3 grid(g.Lq / a.B, g.Hq, g.batch);
    const bool ext = a.seq_first != nullptr || a.diag_token != 0;
    auto launch = [&](auto kernel) -> hipError_t {
        hipError_t e = allow_dynamic_lds((const void*)kernel, p.total);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), p.total, st, g, a, p, scale);
        return hipGetLastError();
    };
    if (dtype == RR_BF16) return ext ? launch(k_estimate_generic<bf16_t, true>) : launch(k_estimate_generic<bf16_t, false>);
    return ext ? launch(k_estimate_generic<float, true>) : launch(k_estimate_generic<float, false>);
}

hipError_t launch_select_rows(const Geom& g, const EstimateArgs& a, const float* mass, hipStream_t st) {
    const long long rows = (long long)g.batch * g.Hq * (g.Lq / a.B);
    const int nch = a.Nb <= 256 ? 4 : (a.Nb <= 512 ? 8 : (a.Nb <= 1024 ? 16 : 0));
    const unsigned lds_bytes = nch ? 0u : (unsigned)((kThreads / 64) * ((a.Nb + 63) / 64 * 64) * sizeof(float));
    const dim3 grid((unsigned)((rows + kThreads / 64 - 1) / (kThreads / 64)));
    auto launch = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 48 * 1024) {
            hipError_t e = allow_dynamic_lds((const void*)kernel, lds_bytes);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds_bytes, st, g, a, mass, rows);
        return hipGetLastError();
    };
    const bool ext = a.seq_first != nullptr;
    switch (nch) {
        case 4: return ext ? launch(k_select_rows<true, 4>) : launch(k_select_rows<false, 4>);
        case 8: return ext ? launch(k_select_rows<true, 8>) : launch(k_select_rows<false, 8>);
        case 16: return ext ? launch(k_select_rows<true, 16>) : launch(k_select_rows<false, 16>);
        default: return ext ? launch(k_select_rows<true, 0>) : launch(k_select_rows<false, 0>);
    }
}

}  // namespace rr
