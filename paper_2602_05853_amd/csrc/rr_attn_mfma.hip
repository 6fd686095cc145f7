// Kernel group (3), MFMA form: causal block-sparse flash attention (Sec. 2.1) for bf16 tensors
// with d = 128 and B = 128 on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// One workgroup (4 waves) per (batch, head, query block m); it walks the compacted ascending
// list of selected key blocks of that row (or every n <= m for the dense baseline).
//
// The products are formed transposed, S^T = K Q^T and O^T = V^T P^T, so that a lane always owns
// one QUERY (MFMA column = lane % 32):
//   * the softmax statistics of a query (running max, denominator, rescale factor) are per-lane
//     scalars; the only cross-lane step is one exchange with lane ^ 32;
//   * the fp32 S^T accumulator registers, rounded to bf16, already ARE the B operand of the
//     second product -- P never goes through LDS.  The k-index order inside an MFMA is free as
//     long as both operands agree, so V^T is laid out in LDS in exactly the key order in which
//     the S^T accumulators hold the keys (0-3, 8-11 | 4-7, 12-15 of every 16).
//
// Wave w works on queries 64*(w & 1) .. +63 and on keys 64*(w >> 1) .. +63 of every key block
// (each LDS operand fragment feeds two MFMAs); the two key halves are merged once at the end.
// K tiles are staged row-major, V tiles transposed (d-major) through registers; both use an XOR
// swizzle of their 16-byte chunks so that LDS writes and MFMA operand reads are conflict-free,
// and both are double-buffered: global loads of block it+1 are in flight while block it is
// being multiplied.
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kThreads = 256;
constexpr int kTileBytes = 128 * 256;                // one 128 x 128 bf16 tile
constexpr int kLdsBytes = 4 * kTileBytes;            // K and V^T, two stages each
constexpr int kXchgFloats = 132;                     // per lane: 128 accumulators + 2 max + 2 sum
constexpr int kOutRowBytes = 264;                    // 128 bf16 + 8 bytes of padding

__device__ __forceinline__ int k_swz(int key, int chunk) { return key * 256 + ((chunk ^ (key & 15)) << 4); }
__device__ __forceinline__ int v_swz(int drow, int chunk) {
    return drow * 256 + ((chunk ^ ((drow & 15) ^ ((drow >> 4) & 7))) << 4);
}

// workgroup id -> (batch, head, query block).  Workgroups are dealt to the 8 XCDs round-robin, so
// id % 8 picks the XCD: every XCD is given whole KV groups (its L2 then holds one KV head's keys
// and values), the heads of a group sit next to each other, and rows go heaviest (largest m) first.
__device__ __forceinline__ bool decode_block(int bid, const Geom& g, int Nb, int& b, int& h, int& m) {
    const int NG = g.batch * g.Hkv, G = g.G;
    int mr, grp, hl;
    if ((NG & 7) == 0) {
        const int x = bid & 7, s = bid >> 3, per = (NG >> 3) * G;
        mr = s / per;
        const int r = s - mr * per;
        grp = x + 8 * (r / G);
        hl = r % G;
    } else if (8 % NG == 0) {
        const int k = 8 / NG, x = bid & 7, s = bid >> 3;
        grp = x % NG;
        const int q = s / G;
        hl = s - q * G;
        mr = q * k + x / NG;
    } else {
        mr = bid / (NG * G);
        const int r = bid - mr * NG * G;
        grp = r / G;
        hl = r - grp * G;
    }
    if (mr >= Nb) return false;
    m = Nb - 1 - mr;
    b = grp / g.Hkv;
    h = (grp - b * g.Hkv) * G + hl;
    return true;
}

__host__ unsigned grid_size(const Geom& g, int Nb) {
    const int NG = g.batch * g.Hkv;
    if ((NG & 7) != 0 && 8 % NG == 0) {
        const int k = 8 / NG;
        return 8u * g.G * ((Nb + k - 1) / k);
    }
    return (unsigned)NG * g.G * Nb;
}

__global__ void __launch_bounds__(kThreads)
k_attn_mfma_bf16(Geom g, AttnArgs a, float scale_log2, float scale) {
    extern __shared__ __align__(16) unsigned char lds[];
    int b, h, m;
    if (!decode_block(blockIdx.x, g, a.Nb, b, h, m)) return;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int qi = w & 1, ki = w >> 1;
    const int l32 = lane & 31, gsel = lane >> 5;
    const int kv = h / g.G;
    const long long row_id = ((long long)b * g.Hq + h) * a.Nb + m;
    const unsigned short* Qp = reinterpret_cast<const unsigned short*>(a.Q) + b * g.qsb + h * g.qsh;
    const unsigned short* Kp = reinterpret_cast<const unsigned short*>(a.K) + b * g.ksb + kv * g.ksh;
    const unsigned short* Vp = reinterpret_cast<const unsigned short*>(a.V) + b * g.ksb + kv * g.ksh;
    const float NEG_INF = -__builtin_huge_valf();

    const int count = a.row_list ? a.row_count[row_id] : (m + 1);
    const int32_t* list = a.row_list ? a.row_list + row_id * a.Nb : nullptr;

    // ---- Q^T operand: this lane's query, d = 16*kc + 8*gsel .. +7, for both 32-query subtiles ----
    bf16x8 qf[2][8];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const long long row = (long long)m * 128 + 64 * qi + 32 * qt + l32;
#pragma unroll
        for (int kc = 0; kc < 8; ++kc)
            qf[qt][kc] = *reinterpret_cast<const bf16x8*>(Qp + row * g.qsl + 16 * kc + 8 * gsel);
    }

    f32x16 acc[4][2];                                  // O^T: [32-row d tile][32-query subtile]
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[dt][qt][r] = 0.f;
    float m_run[2] = {NEG_INF, NEG_INF};               // running max of the raw dot products
    float l_run[2] = {0.f, 0.f};                       // this lane's part of the denominator

    // ---- staging: thread (dc, rb) moves 8 x 16 bytes of K and of V per block ----
    const int dc = tid & 15, rb = tid >> 4;
    u32x4 stg[8];                                      // K and V take turns in these registers
    // keys of V chunk rb in the order the S^T accumulators hold them
    const int vbase = 32 * (rb >> 2) + 16 * ((rb >> 1) & 1) + 4 * (rb & 1);

    auto gload_k = [&](int n) {
        const unsigned short* kb = Kp + (long long)n * 128 * g.ksl + 8 * dc;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            stg[i] = *reinterpret_cast<const u32x4*>(kb + (long long)(rb + 16 * i) * g.ksl);
    };
    auto gload_v = [&](int n) {
        const unsigned short* vb = Vp + (long long)n * 128 * g.ksl + 8 * dc;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            stg[i] = *reinterpret_cast<const u32x4*>(vb + (long long)(vbase + 8 * (i >> 2) + (i & 3)) * g.ksl);
    };
    auto lds_store_k = [&](int stage) {
        unsigned char* ks = lds + stage * kTileBytes;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<u32x4*>(ks + k_swz(rb + 16 * i, dc)) = stg[i];
    };
    auto lds_store_v = [&](int stage) {
        unsigned char* vs = lds + (2 + stage) * kTileBytes;
        // 8 keys x 8 d  ->  8 d rows x 8 keys
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            u32x4 o;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const unsigned x = stg[2 * p][j >> 1], y = stg[2 * p + 1][j >> 1];
                o[p] = (j & 1) ? __builtin_amdgcn_perm(y, x, 0x07060302u)
                               : __builtin_amdgcn_perm(y, x, 0x05040100u);
            }
            *reinterpret_cast<u32x4*>(vs + v_swz(8 * dc + j, rb)) = o;
        }
    };

    if (count > 0) {
        const int n0 = list ? list[0] : 0;
        gload_k(n0);
        lds_store_k(0);
        gload_v(n0);
        lds_store_v(0);
    }
    __syncthreads();

    for (int it = 0; it < count; ++it) {
        const int n = list ? list[it] : it;
        const bool more = it + 1 < count;
        const int n_next = more ? (list ? list[it + 1] : it + 1) : 0;
        if (more) gload_k(n_next);                     // lands while S^T and the softmax run

        const bool diag = (n == m);
        const bool active = !(diag && ki > qi);        // upper-right quarter of the diagonal block: nothing visible
        const unsigned char* ks = lds + (it & 1) * kTileBytes;
        const unsigned char* vs = lds + (2 + (it & 1)) * kTileBytes;
        bf16x8 pf[2][2][2];                            // [qt][t][c]: P^T operand, keys in accumulator order
        if (active) {

            // ---- S^T = K Q^T for 64 keys x 64 queries ----
            f32x16 s[2][2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[t][qt][r] = 0.f;
#pragma unroll
            for (int kc = 0; kc < 8; ++kc) {
                bf16x8 kf[2];
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    kf[t] = *reinterpret_cast<const bf16x8*>(ks + k_swz(64 * ki + 32 * t + l32, 2 * kc + gsel));
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt)
                        s[t][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[qt][kc], s[t][qt], 0, 0, 0);
            }

            // ---- online softmax; a lane owns query column l32 of each subtile ----
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                if (diag && ki == qi) {
                    const int qloc = 32 * qt + l32;
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int kloc = 32 * t + 8 * (r >> 2) + 4 * gsel + (r & 3);
                            if (kloc > qloc) s[t][qt][r] = NEG_INF;
                        }
                }
                float mx = NEG_INF;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][qt][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[qt], mx);
                const float m_use = (m_new == NEG_INF) ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((m_run[qt] - m_use) * scale_log2);   // 0 while the running max is -inf
                const float mb = m_use * scale_log2;
                float psum = 0.f;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(s[t][qt][r], scale_log2, -mb));
                        psum += p;
                        pf[qt][t][r >> 3][r & 7] = (__bf16)p;
                    }
                l_run[qt] = l_run[qt] * alpha + psum;
                m_run[qt] = m_new;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[dt][qt][r] *= alpha;
                }
            }

        }
        if (more) {                                    // K regs -> LDS, then V of the next block lands during PV
            lds_store_k((it + 1) & 1);
            gload_v(n_next);
        }
        if (active) {
            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        const bf16x8 vf = *reinterpret_cast<const bf16x8*>(
                            vs + v_swz(32 * dt + l32, 4 * (2 * ki + t) + 2 * c + gsel));
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt)
                            acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][t][c], acc[dt][qt], 0, 0, 0);
                    }
        }

        if (more) lds_store_v((it + 1) & 1);
        __syncthreads();
    }

    // ---- merge the two key halves of every query, normalise, write ----
    float l_tot[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) l_tot[qt] = l_run[qt] + __shfl_xor(l_run[qt], 32);

    float* xch = reinterpret_cast<float*>(lds) + qi * (kXchgFloats * 64);
    if (ki == 1) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[((dt * 2 + qt) * 16 + r) * 64 + lane] = acc[dt][qt][r];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            xch[(128 + qt) * 64 + lane] = m_run[qt];
            xch[(130 + qt) * 64 + lane] = l_tot[qt];
        }
    }
    __syncthreads();
    if (ki == 0) {
        unsigned char* ost = lds + 2 * kXchgFloats * 64 * 4 + qi * (64 * kOutRowBytes);
        float* lse = a.lse ? a.lse + ((long long)b * g.Hq + h) * g.L + (long long)m * 128 + 64 * qi : nullptr;
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            const float m1 = xch[(128 + qt) * 64 + lane], l1 = xch[(130 + qt) * 64 + lane];
            const float m0 = m_run[qt], l0 = l_tot[qt];
            const float mm = fmaxf(m0, m1);
            const float a0 = (m0 == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f((m0 - mm) * scale_log2);
            const float a1 = (m1 == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f((m1 - mm) * scale_log2);
            const float l = l0 * a0 + l1 * a1;
            const float inv = l > 0.f ? 1.0f / l : 0.f;
            const float w0 = a0 * inv, w1 = a1 * inv;
            if (lse && gsel == 0) lse[32 * qt + l32] = l > 0.f ? mm * scale + logf(l) : NEG_INF;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    unsigned int pk[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int r0 = 4 * rg + 2 * e;
                        const float v0 = acc[dt][qt][r0] * w0 + xch[((dt * 2 + qt) * 16 + r0) * 64 + lane] * w1;
                        const float v1 = acc[dt][qt][r0 + 1] * w0 + xch[((dt * 2 + qt) * 16 + r0 + 1) * 64 + lane] * w1;
                        pk[e] = f32_to_bf16_bits(v0) | (f32_to_bf16_bits(v1) << 16);
                    }
                    u32x2 o = {pk[0], pk[1]};
                    *reinterpret_cast<u32x2*>(ost + (32 * qt + l32) * kOutRowBytes + 2 * (32 * dt + 8 * rg + 4 * gsel)) = o;
                }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        unsigned short* Op = reinterpret_cast<unsigned short*>(a.O) + b * g.qsb + h * g.qsh +
                             ((long long)m * 128 + 64 * qi) * g.qsl;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int idx = lane + 64 * k, row = idx >> 4, ch = idx & 15;
            const u32x2 lo = *reinterpret_cast<const u32x2*>(ost + row * kOutRowBytes + 16 * ch);
            const u32x2 hi = *reinterpret_cast<const u32x2*>(ost + row * kOutRowBytes + 16 * ch + 8);
            u32x4 o = {lo[0], lo[1], hi[0], hi[1]};
            *reinterpret_cast<u32x4*>(Op + (long long)row * g.qsl + 8 * ch) = o;
        }
    }
}

}  // namespace

hipError_t launch_attn_mfma_bf16(const Geom& g, const AttnArgs& a, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)k_attn_mfma_bf16,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const double sc = 1.0 / sqrt((double)g.d);
    const float scale = (float)sc, scale_log2 = (float)(sc * 1.4426950408889634);
    hipLaunchKernelGGL(k_attn_mfma_bf16, dim3(grid_size(g, a.Nb)), dim3(kThreads), kLdsBytes, st,
                       g, a, scale_log2, scale);
    return hipGetLastError();
}

}  // namespace rr
