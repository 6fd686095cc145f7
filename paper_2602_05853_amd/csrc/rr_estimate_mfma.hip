// Kernel group (2), MFMA form of the estimation (importance equation, causal stride softmax and block
// mass, Sec. 3.2-3.3) for bf16 tensors with d = 128 and B/S in {4,8,16,32}.
//
// Exactness.  The stride sums of K are fp32 and must not be rounded to bf16 (that would move
// logits by ~1e-2 and flip far more blocks than the parity margin excuses).  Each fp32 sum is
// instead split exactly into three bf16 terms hi + mid + lo (3 x 8 mantissa bits); Q is bf16
// already, so three bf16 MFMAs with fp32 accumulation reproduce the fp32 products exactly and only
// the accumulation order differs from a plain fp32 dot product.
//
// Work split.  One workgroup per (batch, KV head, group of MB consecutive query blocks).  Its
// "rows" are the sampled queries (Sec. 3.1 positions) of all G query heads of the KV head in those
// blocks, up to 256 of them: this is the GQA sharing -- every staged tile of split stride sums is
// used by all heads of the group.  Wave w owns rows 64w .. 64w+63 as two MFMA column tiles; a
// tile of 32 key strides is the M dimension.  The products are formed transposed (S^T = Ksum Q^T)
// so that a lane owns one sampled query and the softmax statistics of a query are per-lane scalars.
//
// Two sweeps, nothing but the block mass leaves the chip.  The block mass needs every probability
// divided by its query's softmax denominator, which is only known once the query has seen all its
// key strides.  Instead of parking per-(query, key block) partial sums in memory until then, the
// workgroup walks its key tiles twice with the queries held in registers: sweep 1 accumulates each
// query's denominator against a lazily moved reference (no maximum in the common path: the
// reference only moves when a tile's sum of exponentials exceeds 2^10), sweep 2 recomputes the
// scores, forms exp(score - reference) / denominator, sums it over the strides of each key block
// (in-lane and one exchange with lane ^ 32) and over the R sampled queries of a query block (R
// neighbouring lanes, DPP butterfly), and writes one fp32 block mass per (head, query block, key
// block).  The matrix work doubles; the traffic to memory drops by 2 R and the per-row selection
// (k_select_rows) reads R times less.
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kThreads = 256;
constexpr int kTileStrides = 32;
constexpr int kPlaneBytes = kTileStrides * 256;        // 32 strides x 128 bf16
constexpr int kTileBytes = 3 * kPlaneBytes;            // hi, mid, lo
constexpr int kLdsBytes = 2 * kTileBytes;              // double buffered

// ---- stride sums, split into three bf16 planes: Ksp[p][b][kv][j][c], j < LsCap ----
__global__ void __launch_bounds__(256)
k_stride_sum_split(Geom g, const unsigned short* __restrict__ K, int S, int Ls, int j0, int LsCap,
                   unsigned short* __restrict__ Ksp) {
    // strides j0 .. Ls-1 (the ones in front are kept from an earlier call); rows of LsCap strides per (batch, KV head)
    const int chunks = g.d / 8, span = Ls - j0;
    const long long total = (long long)g.batch * g.Hkv * span * chunks;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % chunks);
    long long r = idx / chunks;
    const int j = j0 + (int)(r % span);
    r /= span;
    const int kv = (int)(r % g.Hkv);
    const int b = (int)(r / g.Hkv);
    const unsigned short* src = K + b * g.ksb + kv * g.ksh + (long long)j * S * g.ksl + c * 8;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    // strides that are not complete within the real length do not exist (Sec. 3.1: floor(L/S) of them): zeros
    const int nkeys = (j + 1) * S <= g.Lr ? S : 0;
    for (int s = 0; s < nkeys; ++s) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(src + s * g.ksl);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += __uint_as_float(v[i] << 16);
            acc[2 * i + 1] += __uint_as_float(v[i] & 0xFFFF0000u);
        }
    }
    const long long plane = (long long)g.batch * g.Hkv * LsCap * g.d;
    const long long at = (((long long)(b * g.Hkv + kv) * LsCap + j) * g.d + c * 8);
    unsigned int part[3][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float x = acc[i];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const unsigned int bits = f32_to_bf16_bits(x);
            part[p][i] = bits;
            x -= __uint_as_float(bits << 16);              // exact: the remainder has fewer bits
        }
    }
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        u32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = part[p][2 * i] | (part[p][2 * i + 1] << 16);
        *reinterpret_cast<u32x4*>(Ksp + p * plane + at) = o;
    }
}

// The value lane ^ 32 holds, through the vector ALU (v_permlane32_swap: the upper half of one operand and
// the lower half of the other change places) instead of a round trip through LDS: the tile loop needs it
// five times per query and would otherwise wait for the LDS latency each time.
__device__ __forceinline__ float lane_xor32(float v, bool upper) {
    const unsigned a = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);   // r[0] = (lo, lo), r[1] = (hi, hi)
    return __uint_as_float(upper ? r[0] : r[1]);
}

__device__ __forceinline__ int swz(int row, int chunk) { return row * 256 + ((chunk ^ (row & 15)) << 4); }

struct ScoreArgs {
    const unsigned short* Q;
    const unsigned short* K;        // the keys themselves (diag_token only)
    int diag_token;                 // 1: a query's own stride is cut at the query's position
    const unsigned short* Ksp;      // [3][batch][Hkv][LsCap][128]
    int LsCap;                      // strides the planes are laid out for (>= Ls)
    float* mass;                    // [batch*Hq*Nbq][Nb]: block mass of (row, key block), written for n <= m
    int S, R, Nb, Ls, MB;           // MB query blocks per workgroup
    int off_hmul, off_add;          // sampled offset = S - 1 - ((off_hmul * h + off_add) mod S)
    const int32_t* seq_first;       // packed sequences: first block of the sequence of block m, or nullptr
    float scale_log2;               // log2(e) / (S sqrt(d))
    // Key split: with few workgroups (short contexts, steps) the key tiles of a workgroup's rows are shared out
    // among nsplit workgroups and the two sweeps become two launches.  mode 1: sweep 1 over the own chunk, the
    // softmax state (reference, sum) of every sampled query goes to stats; mode 2: the states of all chunks are
    // combined, then sweep 2 over the own chunk (every key block belongs to exactly one chunk).  mode 0, nsplit
    // 1: both sweeps in one launch.
    float2* stats;                  // [pair][group][nsplit][256]
    int nsplit, mode;
};

// butterfly steps among neighbouring lanes through DPP (no LDS round trip): after xor1 and xor2 all four
// lanes of a quad hold the quad's sum, so "the other quad" / "the other half row" may be reached by mirroring
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// sum over the R lanes l, l^1, .. of an aligned group of R neighbouring lanes; every lane gets the result
template <int R>
__device__ __forceinline__ float group_sum(float v) {
    v += dpp_get<0xB1>(v);                          // quad_perm [1,0,3,2]
    v += dpp_get<0x4E>(v);                          // quad_perm [2,3,0,1]
    if (R >= 8) v += dpp_get<0x141>(v);             // row_half_mirror: lane i <- lane 7 - i
    if (R >= 16) v += dpp_get<0x140>(v);            // row_mirror: lane i <- lane 15 - i
    if (R >= 32) v += __shfl_xor(v, 16);
    return v;
}

constexpr float kLazySum = 1024.0f;                 // a tile's 16-term sum above 2^10 moves the reference

// kExt = false compiles the packed-sequence table and the cut diagonal stride out (the plain method).
// Three workgroups per compute unit (48 KB of LDS and at most 168 registers per lane each): the plain form needs
// 148 registers; the kExt form would take 190 and spills 17-18 of them, which still measured faster than running
// it two to a compute unit.
template <int R, bool kExt>
__global__ void __launch_bounds__(kThreads, 3)
k_stride_mass_mfma(Geom g, ScoreArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int32_t* const seq_first = kExt ? a.seq_first : nullptr;
    const bool diag_token = kExt && a.diag_token != 0;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, gsel = lane >> 5;
    const int Nbq = g.Lq / (a.R * a.S);                            // query blocks (chunked prefill: the last Nbq)
    const int mfirst = a.Nb - Nbq;
    const int ngroups = (Nbq + a.MB - 1) / a.MB;
    // Launch order: the heaviest groups of ALL (batch, KV head) pairs first.  A group's work grows with its
    // position (the last one walks every key tile, a third of the kernel's duration on its own), so a launch
    // that went KV head by KV head would start half of the heaviest workgroups late and end with a few of
    // them running alone.  Consecutive workgroups go to consecutive XCDs: with the KV head as the fastest
    // index every XCD keeps reading the stride sums of the same few KV heads.
    const int pairs = g.Hkv * g.batch;
    const int chunk = (int)blockIdx.x % a.nsplit, wg = (int)blockIdx.x / a.nsplit;
    const int rank = wg / pairs, pr = wg - rank * pairs;
    const int mg = ngroups - 1 - rank;
    const int b = pr / g.Hkv, kv = pr - b * g.Hkv;
    const int m0 = mfirst + mg * a.MB;
    const int mb = min(a.MB, a.Nb - m0);                           // query blocks in this group
    const int GR = g.G * R;
    const int NR = mb * GR;                                        // rows of this workgroup

    // ---- this lane's two sampled queries (one per column tile) ----
    bf16x8 qf[2][8];
    int qi_stride[2];                 // query stride index m*R + r, or -1 for a padding row
    int q_lo[2];                      // first key stride the query may see (start of its sequence)
    float* mass_row[2];               // block masses of the query's (head, query block), or nullptr for rows past the group
    int q_m[2];
    float diag_raw[2] = {0.f, 0.f};   // diag_token: Q . (keys of the own stride up to the query), unscaled
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int q = 64 * wv + 32 * nt + l32;
        const bool in_group = q < NR;
        const int ml = in_group ? q / GR : 0;
        const int rem = in_group ? q - ml * GR : 0;
        const int hl = rem / R, r = rem - hl * R;
        const int h = kv * g.G + hl, m = m0 + ml;
        const long long pos = (long long)(m * R + r) * a.S + (a.S - 1 - ((a.off_hmul * h + a.off_add) % a.S)) - g.q0;   // Sec. 3.1
        // a stride of a partial last block that is not complete within the real length has no sampled query;
        // neither has one whose sampled position lies in front of the step's first query
        const bool valid = in_group && (m * R + r + 1) * a.S <= g.Lr && pos >= 0;
        qi_stride[nt] = valid ? m * R + r : -1;
        q_m[nt] = m;
        {
            int first = (seq_first && in_group) ? seq_first[m] : 0;
            first = first < 0 ? 0 : (first > m ? m : first);      // a malformed table only gives a wrong row
            q_lo[nt] = first * R;
        }
        mass_row[nt] = in_group ? a.mass + (((long long)b * g.Hq + h) * Nbq + (m - mfirst)) * a.Nb : nullptr;
        const unsigned short* qp = a.Q + b * g.qsb + h * g.qsh + pos * g.qsl + 8 * gsel;
#pragma unroll
        for (int kc = 0; kc < 8; ++kc) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (valid) v = *reinterpret_cast<const u32x4*>(qp + 16 * kc);
            qf[nt][kc] = __builtin_bit_cast(bf16x8, v);
        }
        if (diag_token) {
            // this lane holds elements 16 kc + 8 gsel .. +7 of the query; lane ^ 32 holds the others
            const int off = a.S - 1 - ((a.off_hmul * h + a.off_add) % a.S);
            const unsigned short* kp = a.K + b * g.ksb + kv * g.ksh + (long long)(m * R + r) * a.S * g.ksl + 8 * gsel;
            float acc = 0.f;
            if (valid) {
                for (int s = 0; s <= off; ++s) {
#pragma unroll
                    for (int kc = 0; kc < 8; ++kc) {
                        const u32x4 kx = *reinterpret_cast<const u32x4*>(kp + (long long)s * g.ksl + 16 * kc);
                        const u32x4 qx = __builtin_bit_cast(u32x4, qf[nt][kc]);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            acc = fmaf(__uint_as_float(qx[e] << 16), __uint_as_float(kx[e] << 16), acc);
                            acc = fmaf(__uint_as_float(qx[e] & 0xFFFF0000u), __uint_as_float(kx[e] & 0xFFFF0000u), acc);
                        }
                    }
                }
            }
            diag_raw[nt] = acc + __shfl_xor(acc, 32);
        }
    }
    // last key stride any row of this wave may see (wave-uniform)
    int wave_last = max(qi_stride[0], qi_stride[1]);
    wave_last = max(wave_last, __shfl_xor(wave_last, 1));
#pragma unroll
    for (int o = 2; o < 64; o <<= 1) wave_last = max(wave_last, __shfl_xor(wave_last, o));
    wave_last = __builtin_amdgcn_readfirstlane(wave_last);
    // first key stride at which some row of this wave needs the causal mask
    int wave_first = qi_stride[0] < 0 ? 0x7fffffff : qi_stride[0];
    wave_first = min(wave_first, qi_stride[1] < 0 ? 0x7fffffff : qi_stride[1]);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) wave_first = min(wave_first, __shfl_xor(wave_first, o));
    wave_first = __builtin_amdgcn_readfirstlane(wave_first);
    // packed sequences: the range of sequence starts among the rows of this wave (both 0 otherwise)
    int lo_min = 0, lo_max = 0;
    if (kExt) {
        lo_min = min(qi_stride[0] < 0 ? 0x7fffffff : q_lo[0], qi_stride[1] < 0 ? 0x7fffffff : q_lo[1]);
        lo_max = max(qi_stride[0] < 0 ? 0 : q_lo[0], qi_stride[1] < 0 ? 0 : q_lo[1]);
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            lo_min = min(lo_min, __shfl_xor(lo_min, o));
            lo_max = max(lo_max, __shfl_xor(lo_max, o));
        }
        lo_min = __builtin_amdgcn_readfirstlane(lo_min);
        lo_max = __builtin_amdgcn_readfirstlane(lo_max);
    }

    const int last_stride = (m0 + mb) * R - 1;                     // of the whole workgroup
    const int ntiles = last_stride / kTileStrides + 1;
    int tile0 = 0;                                                 // packed sequences: nothing before block m0's sequence is seen
    if (seq_first) {
        int first = seq_first[m0];
        first = first < 0 ? 0 : (first > m0 ? m0 : first);
        tile0 = first * R / kTileStrides;
    }
    const int span = ntiles - tile0;                               // tiles per sweep
    const long long plane = (long long)g.batch * g.Hkv * a.LsCap * g.d;
    const unsigned short* kbase = a.Ksp + ((long long)(b * g.Hkv + kv) * a.LsCap) * g.d;

    // ---- staging: 3 planes x 32 strides x 256 bytes, copied global -> LDS directly, 1 KB (4 strides) per wave
    // instruction, 6 instructions per wave and tile.  The LDS side of such a copy is lane-contiguous, so the
    // swizzle is applied on the global side: lane (r4, c) of row 4 rg + r4 fetches chunk c ^ (row & 15).
    // Rows past the last stride (last tile only) read the last row: never used unmasked.
    const int r4 = lane >> 4, c16 = lane & 15;
    const int wvu = __builtin_amdgcn_readfirstlane(wv);            // the wave index, known to be the same in every lane
    auto issue_tile = [&](int jt, int buf) {
        const int lim = a.Ls - 1 - jt * kTileStrides;              // last row of the tile that exists (>= 0)
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const int q = wvu + 4 * i;                             // 1 KB piece of the tile: plane q / 8, row group q % 8
            const int p = q >> 3, row = 4 * (q & 7) + r4;
            const unsigned long long srcv = (unsigned long long)(kbase + p * plane + (long long)jt * kTileStrides * g.d);
            // wave-uniform: into scalar registers (readfirstlane yields an int: through unsigned, or the low word
            // is sign-extended over the high one)
            const unsigned src_hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(srcv >> 32));
            const unsigned src_lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)srcv);
            const unsigned short* src =
                reinterpret_cast<const unsigned short*>(((unsigned long long)src_hi << 32) | (unsigned long long)src_lo);
            const unsigned off = 2u * ((unsigned)min(row, lim) * 128u + 8u * (unsigned)(c16 ^ (row & 15)));
            const unsigned dst = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)lds) +
                                 (unsigned)(buf * kTileBytes + p * kPlaneBytes + (q & 7) * 1024);
            asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                         :: "v"(off), "s"(src), "s"(__builtin_amdgcn_readfirstlane(dst)) : "memory");
        }
    };
    auto wait_copies = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    // steps t of this workgroup: [0, span) is sweep 1, [span, 2 span) sweep 2; a split workgroup has its chunk
    // of one of them
    int t_begin = 0, t_end = 2 * span;
    if (a.nsplit > 1) {
        const int len = (span + a.nsplit - 1) / a.nsplit;
        const int c_lo = min(span, chunk * len), c_hi = min(span, c_lo + len);
        t_begin = (a.mode == 1 ? 0 : span) + c_lo;
        t_end = (a.mode == 1 ? 0 : span) + c_hi;
        if (a.mode == 2 && t_begin >= t_end) return;               // no key block of these rows is in this chunk
    }
    auto tile_of = [&](int t) { return tile0 + (t >= span ? t - span : t); };
    float2* const my_stats = a.stats ? a.stats + (((long long)pr * ngroups + mg) * a.nsplit) * 256 : nullptr;

    if (t_begin < t_end) issue_tile(tile_of(t_begin), t_begin & 1);
    // The sampled queries must be complete in their registers before the tile loop: the compiler's waits for
    // ordinary loads count only the loads it knows, and inside the loop they would stall on the tile copies.
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int kc = 0; kc < 8; ++kc) asm volatile("" : "+v"(qf[nt][kc]));
    wait_copies();
    __syncthreads();

    const float NEG_INF = -__builtin_huge_valf();
    // Softmax state of this lane's share (the strides 8k + 4 gsel .. +3 of every tile) of its two queries, in
    // log2 units: reference U (lazily moved) and sum of 2^(score - U).  Rows that do not exist score 0
    // everywhere (zero query): a finite reference keeps them off the slow path.
    float U[2], Z[2] = {0.f, 0.f}, nbq[2] = {0.f, 0.f}, invZ[2] = {0.f, 0.f};
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) U[nt] = qi_stride[nt] >= 0 ? NEG_INF : 0.f;

    if (a.nsplit > 1 && a.mode == 2) {
        // the softmax state of a query over ALL key strides: its states in the chunks, brought to one reference
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const float2* sq = my_stats + 64 * wv + 32 * nt + l32;
            float um = NEG_INF;
            for (int c = 0; c < a.nsplit; ++c) {
                const float2 s2 = sq[c * 256];
                if (s2.y > 0.f) um = fmaxf(um, s2.x);
            }
            float z = 0.f;
            for (int c = 0; c < a.nsplit; ++c) {
                const float2 s2 = sq[c * 256];
                if (s2.y > 0.f) z += s2.y * __builtin_amdgcn_exp2f(s2.x - um);
            }
            nbq[nt] = (um == NEG_INF) ? 0.f : -um;
            invZ[nt] = (qi_stride[nt] >= 0 && z > 0.f) ? 1.0f / z : 0.f;
        }
    }

    // step t: tile tile_of(t) of sweep t / span, in LDS buffer t & 1
    for (int t = t_begin; t < t_end; ++t) {
        const bool sweep2 = t >= span;
        const int jt = tile_of(t);
        const bool more = t + 1 < t_end;
        if (more) issue_tile(tile_of(t + 1), (t + 1) & 1);          // its last readers passed the barrier of step t - 1
        if (t == span && a.nsplit == 1) {
            // between the sweeps: the two lanes of a query hold disjoint strides; combine their states
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const float oU = lane_xor32(U[nt], gsel != 0), oZ = lane_xor32(Z[nt], gsel != 0);
                const float um = fmaxf(U[nt], oU);
                const float use = (um == NEG_INF) ? 0.f : um;
                const float z = Z[nt] * __builtin_amdgcn_exp2f(U[nt] - use) + oZ * __builtin_amdgcn_exp2f(oU - use);
                nbq[nt] = -use;
                invZ[nt] = (qi_stride[nt] >= 0 && z > 0.f) ? 1.0f / z : 0.f;
            }
        }
        const int j0 = jt * kTileStrides;
        if (j0 <= wave_last && j0 + kTileStrides > lo_min) {
            const unsigned char* tile = lds + (t & 1) * kTileBytes;
            f32x16 s[2];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[nt][i] = 0.f;
#pragma unroll
            for (int kc = 0; kc < 8; ++kc) {
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(tile + p * kPlaneBytes + swz(l32, 2 * kc + gsel));
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nt][kc], s[nt], 0, 0, 0);
                }
            }
            if (diag_token && j0 + kTileStrides - 1 >= wave_first) {
                // the tile may hold a query's own stride: put the cut score in its place
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (j0 + 8 * (i >> 2) + 4 * gsel + (i & 3) == qi_stride[nt]) s[nt][i] = diag_raw[nt];
            }
            const bool need_mask = j0 + kTileStrides - 1 > wave_first || j0 < lo_max;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int iq = qi_stride[nt];
                const int jlo = q_lo[nt];
                if (need_mask) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int j = j0 + 8 * (i >> 2) + 4 * gsel + (i & 3);
                        // causal at stride level (also kills padding rows), and inside the query's own sequence
                        if (j > iq || j < jlo) s[nt][i] = NEG_INF;
                    }
                }
                if (!sweep2) {
                    // ---- sweep 1: denominator against the lazy reference ----
                    const float nb = -U[nt];
                    float sum = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(s[nt][i], a.scale_log2, nb));
                    // a reference of -inf (nothing seen yet) gives inf or nan and lands here as well
                    const bool move = !(sum <= kLazySum);
                    if (__any(move)) {
                        if (move) {
                            float mx = NEG_INF;
#pragma unroll
                            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[nt][i]);
                            const float top = (mx == NEG_INF) ? NEG_INF : mx * a.scale_log2;
                            const float nu = fmaxf(U[nt], top);
                            const float use = (nu == NEG_INF) ? 0.f : nu;
                            Z[nt] *= __builtin_amdgcn_exp2f(U[nt] - use);      // 0 while the reference is -inf
                            U[nt] = nu;
                            sum = 0.f;
#pragma unroll
                            for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(s[nt][i], a.scale_log2, -use));
                        }
                    }
                    Z[nt] += sum;
                } else {
                    // ---- sweep 2: probabilities, summed per key block and over the R queries of a query block ----
                    const float nb = nbq[nt];
                    float e[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(fmaf(s[nt][i], a.scale_log2, nb));
                    constexpr int NBL = (R == 4) ? 4 : kTileStrides / R;       // blocks this lane has a share of
                    constexpr int RPB = 16 / NBL;                               // registers per block
                    const int r = l32 & (R - 1);                                // the query's index inside its block
                    const int m = q_m[nt];
                    const int nlo = jlo / R;
                    float out = 0.f;                                            // the block mass this lane writes
#pragma unroll
                    for (int k = 0; k < NBL; ++k) {
                        float sum = 0.f;
#pragma unroll
                        for (int i = 0; i < RPB; ++i) sum += e[k * RPB + i];
                        // R = 4: a lane holds whole blocks (strides 8k + 4 gsel .. +3 are block 2k + gsel of the
                        // tile); else a block is R/2 consecutive registers here and in lane ^ 32
                        if (R != 4) sum += lane_xor32(sum, gsel != 0);
                        const float tot = group_sum<R>(sum * invZ[nt]);
                        if (r == k) out = tot;
                    }
                    // lane r writes block r of the tile (R = 4: block 2 r + gsel): neighbouring lanes, neighbouring words
                    const int n = (R == 4) ? jt * 8 + 2 * r + gsel : jt * NBL + r;
                    const bool writer = (R == 4) ? true : (gsel == 0 && r < NBL);
                    if (writer && mass_row[nt] && n <= m && n >= nlo) mass_row[nt][n] = out;
                }
            }
        }
        wait_copies();
        __syncthreads();
    }
    if (a.nsplit > 1 && a.mode == 1) {
        // the state of each query over this chunk (the two lanes of a query combined), for the second launch
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const float oU = lane_xor32(U[nt], gsel != 0), oZ = lane_xor32(Z[nt], gsel != 0);
            const float um = fmaxf(U[nt], oU);
            const float use = (um == NEG_INF) ? 0.f : um;
            const float z = Z[nt] * __builtin_amdgcn_exp2f(U[nt] - use) + oZ * __builtin_amdgcn_exp2f(oU - use);
            if (gsel == 0) my_stats[chunk * 256 + 64 * wv + 32 * nt + l32] = make_float2(use, z);
        }
    }
}

}  // namespace

size_t estimate_mfma_ksplit_bytes(const Geom& g, int S) {
    return (size_t)3 * g.batch * g.Hkv * (g.L / S) * g.d * sizeof(unsigned short);
}
// Key split (ScoreArgs::nsplit).  Measured on the 128K workload's generator at 8K .. 128K tokens and on steps:
// a launch of fewer than 1024 workgroups gains from being split into about three times as many (never fewer
// than 768, never more than 1536: beyond that the repeated set-up of a workgroup -- its queries, its first
// tile -- costs more than the idle compute units did), each chunk at least 8 key tiles long.  From 1024
// workgroups on (128K tokens with 8 KV heads) two launches and one are level, and it stays one.
int estimate_mfma_splits(const Geom& g, int S, int B) {
    const int R = B / S, Nbq = g.Lq / B;
    int MB = 256 / (g.G * R);
    if (MB > Nbq) MB = Nbq;
    const long long wgs = (long long)((Nbq + MB - 1) / MB) * g.Hkv * g.batch;
    const int tiles = (g.L / S + kTileStrides - 1) / kTileStrides;
    if (wgs >= 1024) return 1;
    long long target = 3 * wgs;
    target = target < 768 ? 768 : (target > 1536 ? 1536 : target);
    long long P = (target + wgs - 1) / wgs;
    if (P > tiles / 8) P = tiles / 8;
    if (P > 64) P = 64;
    return P < 1 ? 1 : (int)P;
}
size_t estimate_mfma_stats_bytes(const Geom& g, int S, int B) {
    const int P = estimate_mfma_splits(g, S, B);
    if (P <= 1) return 0;
    const int R = B / S, Nbq = g.Lq / B;
    int MB = 256 / (g.G * R);
    if (MB > Nbq) MB = Nbq;
    return (size_t)((Nbq + MB - 1) / MB) * g.Hkv * g.batch * P * 256 * sizeof(float2);
}
size_t estimate_mfma_mass_bytes(const Geom& g, int B) {
    return (size_t)g.batch * g.Hq * (g.Lq / B) * (g.L / B) * sizeof(float);
}
bool estimate_mfma_supported(const Geom& g, int dtype, int S, int B) {
    const int R = B / S;
    return dtype == RR_BF16 && g.d == 128 && (R == 4 || R == 8 || R == 16 || R == 32) && g.G * R <= 256;
}

hipError_t launch_stride_mass_mfma(const Geom& g, const void* Q, const void* K, int S, int B, int off_hmul,
                                   int off_add, int diag_token, const int32_t* seq_first, unsigned short* ksplit,
                                   int ls_cap, int ls_valid, float* mass, float2* stats, hipStream_t st) {
    const int Ls = g.L / S, R = B / S, Nb = g.L / B;
    if (ls_cap < Ls || ls_valid < 0) return hipErrorInvalidValue;
    const int j0 = ls_valid < Ls ? ls_valid : Ls;
    if (j0 < Ls) {
        const long long total = (long long)g.batch * g.Hkv * (Ls - j0) * (g.d / 8);
        hipLaunchKernelGGL(k_stride_sum_split, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g,
                           (const unsigned short*)K, S, Ls, j0, ls_cap, ksplit);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    ScoreArgs a;
    a.Q = (const unsigned short*)Q;
    a.Ksp = ksplit;
    a.LsCap = ls_cap;
    a.mass = mass;
    a.off_hmul = off_hmul;
    a.off_add = off_add;
    a.seq_first = seq_first;
    a.K = (const unsigned short*)K;
    a.diag_token = diag_token;
    a.S = S; a.R = R; a.Nb = Nb; a.Ls = Ls;
    a.MB = 256 / (g.G * R);
    const int Nbq = g.Lq / B;
    if (a.MB > Nbq) a.MB = Nbq;
    const double sc = 1.0 / ((double)S * sqrt((double)g.d));
    a.scale_log2 = (float)(sc * 1.4426950408889634);
    const int ngroups = (Nbq + a.MB - 1) / a.MB;
    a.nsplit = stats ? estimate_mfma_splits(g, S, B) : 1;
    a.stats = a.nsplit > 1 ? stats : nullptr;
    dim3 grid((unsigned)ngroups * g.Hkv * g.batch * a.nsplit);
    const bool ext = seq_first != nullptr || diag_token != 0;
#define RR_LAUNCH_MASS(RV)                                                                          \
    do {                                                                                            \
        if (ext) hipLaunchKernelGGL((k_stride_mass_mfma<RV, true>), grid, dim3(kThreads), kLdsBytes, st, g, a);  \
        else hipLaunchKernelGGL((k_stride_mass_mfma<RV, false>), grid, dim3(kThreads), kLdsBytes, st, g, a);     \
    } while (0)
    // one launch, or (key split) the first sweep and then the second
    for (int pass = (a.nsplit > 1 ? 1 : 0); pass <= (a.nsplit > 1 ? 2 : 0); ++pass) {
        a.mode = pass;
        switch (R) {
            case 4: RR_LAUNCH_MASS(4); break;
            case 8: RR_LAUNCH_MASS(8); break;
            case 16: RR_LAUNCH_MASS(16); break;
            case 32: RR_LAUNCH_MASS(32); break;
            default: return hipErrorInvalidValue;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
#undef RR_LAUNCH_MASS
    return hipSuccess;
}

}  // namespace rr
