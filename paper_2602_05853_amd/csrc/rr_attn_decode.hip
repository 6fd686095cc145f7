// Attention of a very short step (one or two new tokens) against a long context: the decode-stage use of the
// path (the paper's "Future Work"; its experiments decode densely, Sec. 4.1).  bf16, d = 128, B = 128.
//
// Such a step has G * T query rows per KV head (T tokens, G query heads), far too few for a 128-row matrix tile,
// and its cost is reading K and V once.  So: no matrix instructions, no LDS staging.  One workgroup takes a
// range of key blocks of ONE KV head and serves all G * T rows from the same loaded keys (the GQA sharing);
// a wavefront reads four keys per load instruction (16 lanes x 16 bytes = one key row), every lane keeps the
// 8 channels of its chunk, the dot products are finished with butterflies inside the 16 lanes (DPP).  Each
// group of 16 lanes runs its own online softmax over the keys it sees; the 16 streams of a workgroup are merged
// at the end and the part's normalised output and log-sum-exp go to the workspace.  A second kernel merges the
// parts (the softmax over the selected keys is one sum, Sec. 2.1, so parts combine exactly up to rounding).
//
// Sparse steps walk the union of the rows' block lists: a key block is loaded when any row of the KV head
// selected it, and a row skips the blocks it did not select (its scores are masked), so every row still sees
// exactly the blocks of its own list.
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kDecThreads = 256;
constexpr int kDecMaxRows = 8;          // G * T
constexpr int kDecMaxTokens = 2;
constexpr int kDecMaxParts = 256;
constexpr int kDecBlock = 128;

struct DecodeArgs {
    AttnArgs a;
    int T;              // query positions of the step
    int nblocks;        // key blocks 0 .. nblocks-1 reach the last query
    int len;            // key blocks per part
    float scale_log2;   // log2(e) / sqrt(d)
};

template <int CTRL>
__device__ __forceinline__ float dec_dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// sum over the 16 lanes of a DPP row; every lane gets it
__device__ __forceinline__ float row16_sum(float v) {
    v += dec_dpp<0xB1>(v);      // quad_perm [1,0,3,2]
    v += dec_dpp<0x4E>(v);      // quad_perm [2,3,0,1]
    v += dec_dpp<0x141>(v);     // row_half_mirror
    v += dec_dpp<0x140>(v);     // row_mirror
    return v;
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// 8-channel dot product of two packed bf16 chunks, fp32 accumulation (v_dot2c_f32_bf16).  The pairs are taken
// from the whole vector with shuffles: bit-casting single 32-bit elements picked by a loop index made the
// compiler use the first pair four times.
__device__ __forceinline__ float dot8(const bf16x8& a, const bf16x8& b) {
    float s = 0.f;
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), s, false);
    return s;
}

__device__ __forceinline__ void unpack8(const u32x4& x, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(x[i] << 16);
        f[2 * i + 1] = __uint_as_float(x[i] & 0xFFFF0000u);
    }
}

// RM: rows the instantiation carries (the smallest of 1, 2, 4, 8 that holds G * T); rows beyond G * T repeat row
// 0 and are never stored.
template <int RM>
__global__ void __launch_bounds__(kDecThreads, 2)
k_attn_decode(Geom g, DecodeArgs da) {
    __shared__ float s_m[4][RM], s_l[4][RM];
    __shared__ float s_o[4][RM][128];
    const AttnArgs& a = da.a;
    const int part = blockIdx.x, kv = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int kq = lane >> 4, c = lane & 15;
    const int T = da.T, R = g.G * T;
    const int Nbq = g.Lq / kDecBlock, m_first = (g.L - g.Lq) / kDecBlock;
    const long long nrows = (long long)g.batch * g.Hq * T;
    const float NEG_INF = -__builtin_huge_valf();

    const unsigned short* Qp = reinterpret_cast<const unsigned short*>(a.Q);
    const unsigned short* Kp = reinterpret_cast<const unsigned short*>(a.K) + b * g.ksb + kv * g.ksh + c * 8;
    const unsigned short* Vp = reinterpret_cast<const unsigned short*>(a.V) + b * g.ksb + kv * g.ksh + c * 8;

    bf16x8 q[RM];
    int qpos[RM], mrow[RM], cnt[RM], lpos[RM], cur[RM];     // cur: the list entry at lpos, read one block ahead
    const int32_t* list[RM];
    const int n_lo = part * da.len;
    const int n_hi = n_lo + da.len < da.nblocks ? n_lo + da.len : da.nblocks;
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        const int rr = r < R ? r : 0;
        const int hl = rr / T, t = rr - hl * T, h = kv * g.G + hl;
        q[r] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Qp + b * g.qsb + h * g.qsh + (long long)t * g.qsl + c * 8));
        qpos[r] = g.q0 + t;
        mrow[r] = qpos[r] / kDecBlock;
        list[r] = nullptr;
        cnt[r] = 0;
        lpos[r] = 0;
        cur[r] = 0x7fffffff;
        if (a.row_list) {
            const long long rid = ((long long)b * g.Hq + h) * Nbq + (mrow[r] - m_first);
            int cn = a.row_count[rid];
            cn = cn < 0 ? 0 : (cn > a.Nb ? a.Nb : cn);
            cnt[r] = cn;
            list[r] = a.row_list + rid * a.Nb;
        }
    }
    // Where the part starts in every row's list: the number of entries below n_lo, counted by the whole workgroup
    // at once (a binary search would be a chain of dependent loads per row, longer than the part's real work).
    if (a.row_list && n_lo > 0) {
        __shared__ int s_below[4][RM];
        int below[RM], most = 0;
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            below[r] = 0;
            most = cnt[r] > most ? cnt[r] : most;
        }
        for (int j = tid; j < most; j += kDecThreads) {
#pragma unroll
            for (int r = 0; r < RM; ++r) {                  // the loads of all rows together, none predicated
                const int e = list[r][j < cnt[r] ? j : 0];
                below[r] += (j < cnt[r] && e < n_lo) ? 1 : 0;
            }
        }
#pragma unroll
        for (int r = 0; r < RM; ++r) {
#pragma unroll
            for (int sft = 32; sft >= 1; sft >>= 1) below[r] += __shfl_xor(below[r], sft);
            if (lane == 0) s_below[wv][r] = below[r];
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RM; ++r) lpos[r] = s_below[0][r] + s_below[1][r] + s_below[2][r] + s_below[3][r];
    }
    if (a.row_list) {
#pragma unroll
        for (int r = 0; r < RM; ++r)
            if (lpos[r] < cnt[r]) cur[r] = list[r][lpos[r]];
    }

    float mref[RM], lsum[RM], acc[RM][8];
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        mref[r] = NEG_INF;
        lsum[r] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    }

    for (int n = n_lo; n < n_hi; ++n) {
        bool sel[RM];
        bool any = false;
        if (a.row_list) {
            // Block n is in a row's list when the entry the row stands at equals n.  The entry for the next trip
            // is requested here, for every row without a branch or a wait in between, and first looked at in the
            // next trip, so its latency hides behind this block's work.  (An entry below n cannot occur in an
            // ascending list; were one there, it is passed over, one per trip.)
            int nxt[RM];
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                sel[r] = cur[r] == n;
                lpos[r] += cur[r] <= n ? 1 : 0;
                const int idx = lpos[r] < cnt[r] ? lpos[r] : 0;           // always inside the row's Nb entries
                nxt[r] = list[r][idx];
            }
#pragma unroll
            for (int r = 0; r < RM; ++r) cur[r] = lpos[r] < cnt[r] ? nxt[r] : 0x7fffffff;
        } else {
#pragma unroll
            for (int r = 0; r < RM; ++r) sel[r] = true;
        }
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            sel[r] = sel[r] && n <= mrow[r] && r < R;
            any = any || sel[r];
        }
        if (!any) continue;                               // the same in every lane of the workgroup
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            // four keys per lane group: key index, clamped for the loads to the positions that exist
            u32x4 kk[4], vv[4];
            int kidx[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kidx[i] = n * kDecBlock + wv * 32 + half * 16 + 4 * i + kq;
                const int kc = kidx[i] < g.Lr ? kidx[i] : g.Lr - 1;
                kk[i] = *reinterpret_cast<const u32x4*>(Kp + (long long)kc * g.ksl);
                vv[i] = *reinterpret_cast<const u32x4*>(Vp + (long long)kc * g.ksl);
            }
            float sc[RM][4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bf16x8 kb = __builtin_bit_cast(bf16x8, kk[i]);
#pragma unroll
                for (int r = 0; r < RM; ++r) {
                    const float d = row16_sum(dot8(kb, q[r]));
                    sc[r][i] = (sel[r] && kidx[i] <= qpos[r]) ? d * da.scale_log2 : NEG_INF;
                }
            }
            float p[RM][4];
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                const float mx = fmaxf(fmaxf(sc[r][0], sc[r][1]), fmaxf(sc[r][2], sc[r][3]));
                const float mnew = fmaxf(mref[r], mx);
                if (mnew == NEG_INF) {                     // nothing visible so far
#pragma unroll
                    for (int i = 0; i < 4; ++i) p[r][i] = 0.f;
                    continue;
                }
                const float alpha = __builtin_amdgcn_exp2f(mref[r] - mnew);    // mref = -inf: 0
                mref[r] = mnew;
                float ps = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p[r][i] = __builtin_amdgcn_exp2f(sc[r][i] - mnew);         // masked: 0
                    ps += p[r][i];
                }
                lsum[r] = lsum[r] * alpha + ps;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[r][e] *= alpha;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float vf[8];
                unpack8(vv[i], vf);
#pragma unroll
                for (int r = 0; r < RM; ++r) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][e] = fmaf(p[r][i], vf[e], acc[r][e]);
                }
            }
        }
    }

    // the four lane groups of the wavefront: to one reference, then summed (every lane ends with the totals)
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        float mall = fmaxf(mref[r], __shfl_xor(mref[r], 16));
        mall = fmaxf(mall, __shfl_xor(mall, 32));
        const float f = mref[r] == NEG_INF ? 0.f : __builtin_amdgcn_exp2f(mref[r] - mall);
        float l = lsum[r] * f;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        lsum[r] = l;
        mref[r] = mall;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float o = acc[r][e] * f;
            o += __shfl_xor(o, 16);
            o += __shfl_xor(o, 32);
            acc[r][e] = o;
        }
        if (kq == 0) {
            if (c == 0) { s_m[wv][r] = mall; s_l[wv][r] = l; }
#pragma unroll
            for (int e = 0; e < 8; ++e) s_o[wv][r][c * 8 + e] = acc[r][e];
        }
    }
    __syncthreads();
    // the four wavefronts: the part's normalised output and its natural-log sum of exponentials
    for (int idx = tid; idx < RM * 128; idx += kDecThreads) {
        const int r = idx >> 7, e = idx & 127;
        if (r >= R) continue;
        float mall = NEG_INF;
#pragma unroll
        for (int w = 0; w < 4; ++w) mall = fmaxf(mall, s_m[w][r]);
        float tot = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = s_m[w][r] == NEG_INF ? 0.f : __builtin_amdgcn_exp2f(s_m[w][r] - mall);
            tot = fmaf(s_l[w][r], f, tot);
            o = fmaf(s_o[w][r][e], f, o);
        }
        // rows of this instantiation are (hl, t) pairs in the order of the set-up loop
        const int hl = r / T, t = r - hl * T;
        const long long row = ((long long)b * g.Hq + kv * g.G + hl) * T + t;
        a.part_O[((long long)part * nrows + row) * 128 + e] = tot > 0.f ? o / tot : 0.f;
        if (e == 0) a.part_lse[(long long)part * nrows + row] = tot > 0.f ? mall * 0.6931471805599453f + logf(tot) : NEG_INF;
    }
}

// One workgroup per query row: O = sum_p w_p O_p / sum_p w_p with w_p = exp(lse_p - max), rounded once.
__global__ void __launch_bounds__(kDecThreads)
k_attn_decode_combine(Geom g, AttnArgs a, int T) {
    __shared__ float s_w[kDecMaxParts];
    __shared__ float s_red[4];
    __shared__ float s_o[4][128];
    const long long nrows = (long long)g.batch * g.Hq * T;
    const long long row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int P = a.nsplit;
    const float NEG_INF = -__builtin_huge_valf();
    const float l = tid < P ? a.part_lse[(long long)tid * nrows + row] : NEG_INF;
    float mx = l;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s));
    if (lane == 0) s_red[wv] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    const float w = (tid < P && l != NEG_INF) ? expf(l - mx) : 0.f;
    if (tid < kDecMaxParts) s_w[tid] = w;
    __syncthreads();
    // wavefront wv takes the parts p = wv, wv + 4, ..; a lane two channels
    float den = 0.f, o0 = 0.f, o1 = 0.f;
    for (int p = wv; p < P; p += 4) {
        const float wp = s_w[p];
        if (wp == 0.f) continue;
        const float2 v = *reinterpret_cast<const float2*>(a.part_O + ((long long)p * nrows + row) * 128 + 2 * lane);
        den += wp;
        o0 = fmaf(wp, v.x, o0);
        o1 = fmaf(wp, v.y, o1);
    }
    __syncthreads();
    if (lane == 0) s_red[wv] = den;
    s_o[wv][2 * lane] = o0;
    s_o[wv][2 * lane + 1] = o1;
    __syncthreads();
    if (wv == 0) {
        den = s_red[0] + s_red[1] + s_red[2] + s_red[3];
        o0 = s_o[0][2 * lane] + s_o[1][2 * lane] + s_o[2][2 * lane] + s_o[3][2 * lane];
        o1 = s_o[0][2 * lane + 1] + s_o[1][2 * lane + 1] + s_o[2][2 * lane + 1] + s_o[3][2 * lane + 1];
        const float inv = den > 0.f ? 1.0f / den : 0.f;
        const long long bh = row / T, t = row - bh * T;
        const int b = (int)(bh / g.Hq), h = (int)(bh - (long long)b * g.Hq);
        unsigned short* O = reinterpret_cast<unsigned short*>(a.O) + b * g.qsb + h * g.qsh + t * g.qsl;
        *reinterpret_cast<unsigned*>(O + 2 * lane) = f32_to_bf16_bits(o0 * inv) | (f32_to_bf16_bits(o1 * inv) << 16);
        if (a.lse && lane == 0) a.lse[row] = den > 0.f ? mx + logf(den) : NEG_INF;
    }
}

}  // namespace

// Parts of a decode-sized step, 0 when the step is not one: at most kDecMaxTokens positions and kDecMaxRows
// rows per KV head.  The launch is sized to what the chip holds at once -- two workgroups per compute unit (the
// kernel is compiled to at most 256 registers per lane for that; eight rows need 244) -- because a second round
// of workgroups costs more than longer parts save; measured at 128K tokens, one new token, 32 / 8 heads: 256
// workgroups 143 us, 384 132, 512 112, 768 115, 1024 125-133, 2048 144; two tokens (eight rows): 256 227 us,
// 512 166.  A part is at least two key blocks long.
int attn_decode_parts(const Geom& g, int B) {
    if (B != kDecBlock || g.d != 128) return 0;
    const int T = g.Lr - g.q0;
    if (T < 1 || T > kDecMaxTokens || g.G * T > kDecMaxRows) return 0;
    const int nblocks = (g.Lr - 1) / kDecBlock + 1;
    const long long groups = (long long)g.batch * g.Hkv, target = 512;
    long long P = (target + groups - 1) / groups;
    if (P > (nblocks + 1) / 2) P = (nblocks + 1) / 2;
    if (P > kDecMaxParts) P = kDecMaxParts;
    return P < 1 ? 1 : (int)P;
}

size_t attn_decode_bytes(const Geom& g, int B) {
    const int P = attn_decode_parts(g, B);
    if (P < 1) return 0;
    const size_t rows = (size_t)g.batch * g.Hq * (size_t)(g.Lr - g.q0);
    return (size_t)P * rows * 128 * sizeof(float) + (size_t)P * rows * sizeof(float);
}

// expects a.nsplit = attn_decode_parts(g, a.B) >= 1 and a.part_O / a.part_lse of attn_decode_bytes
hipError_t launch_attn_decode(const Geom& g, const AttnArgs& a, hipStream_t st) {
    const int T = g.Lr - g.q0, R = g.G * T;
    if (a.nsplit < 1 || a.nsplit > kDecMaxParts || !a.part_O || !a.part_lse || T < 1 || T > kDecMaxTokens || R > kDecMaxRows ||
        g.batch > 65535 || g.Hkv > 65535)
        return hipErrorInvalidValue;
    DecodeArgs da;
    da.a = a;
    da.T = T;
    da.nblocks = (g.Lr - 1) / kDecBlock + 1;
    da.len = (da.nblocks + a.nsplit - 1) / a.nsplit;
    da.scale_log2 = (float)(1.4426950408889634 / sqrt((double)g.d));
    const dim3 grid((unsigned)a.nsplit, (unsigned)g.Hkv, (unsigned)g.batch);
    if (R <= 1) hipLaunchKernelGGL(k_attn_decode<1>, grid, dim3(kDecThreads), 0, st, g, da);
    else if (R <= 2) hipLaunchKernelGGL(k_attn_decode<2>, grid, dim3(kDecThreads), 0, st, g, da);
    else if (R <= 4) hipLaunchKernelGGL(k_attn_decode<4>, grid, dim3(kDecThreads), 0, st, g, da);
    else hipLaunchKernelGGL(k_attn_decode<8>, grid, dim3(kDecThreads), 0, st, g, da);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long nrows = (long long)g.batch * g.Hq * T;
    hipLaunchKernelGGL(k_attn_decode_combine, dim3((unsigned)nrows), dim3(kDecThreads), 0, st, g, a, T);
    return hipGetLastError();
}

}  // namespace rr
