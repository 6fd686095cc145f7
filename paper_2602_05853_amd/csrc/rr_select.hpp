// Adaptive Top-tau selection (Sec. 3.3) of one query-block row by ONE wavefront, shared by the
// estimate kernels.  Input: the row's block-mass fractions in LDS (each row sums to 1).  Output: the
// dense 0/1 row, the ascending list of selected key blocks and their count.
//
// The definition ranks the key blocks by mass (ties: smaller index first) and keeps the shortest prefix
// whose cumulative mass reaches tau.  No sort is needed for that: with g(t) = sum of the fractions >= t,
// the mass of the last kept block is the largest t with g(t) >= tau, and g is a step function whose
// steps sit at the row's own values, so a bisection over the 31 value bits of a non-negative float finds
// it exactly.  Everything above that value is kept, and of the blocks equal to it the first few in index
// order, as many as the cumulative sum still needs.  g is evaluated with one fixed summation order
// (per lane ascending, then a fixed lane tree), which makes it monotone in t in floating point as well.
#pragma once
#include "rr_common.hpp"

namespace rr {

struct SelectRow {
    int nlo, m, Nb;                  // candidates are the key blocks nlo .. m; the row has Nb entries
    float tau;
    bool keep_all;                   // tau = 1, a protected last query block, or a row without an estimate
    int sink_blocks, recent_blocks;  // added after the selection (a union)
    uint8_t* dense;                  // [Nb] or nullptr
    int32_t* list;                   // [Nb]
    int32_t* count;                  // [1]
};

// sum over the wavefront in a fixed order; every lane gets the result
__device__ __forceinline__ float wave_sum_fixed(float v) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// Row access.  chunk c of a row holds key blocks 64 c .. 64 c + 63, lane l the block 64 c + l; at(c) returns
// this lane's fraction of chunk c, 0 for a block outside the candidates nlo .. m.
//   RowInLds   any row length: the fractions stay in LDS and are read again on every pass
//   RowInRegs  rows of up to 64 * NCH key blocks held in registers (loops over c are unrolled, so the
//              register index is static)
struct RowInLds {
    const float* frac; int nlo, m, lane, c0, c1;
    __device__ __forceinline__ RowInLds(const float* f, int nlo_, int m_, int lane_)
        : frac(f), nlo(nlo_), m(m_), lane(lane_), c0(nlo_ >> 6), c1((m_ >> 6) + 1) {}
    __device__ __forceinline__ float at(int c) const {
        const int n = 64 * c + lane;
        return (n >= nlo && n <= m) ? frac[n] : 0.f;
    }
    template <typename F> __device__ __forceinline__ void for_chunks(F&& f) const {
        for (int c = c0; c < c1; ++c) f(c, at(c));
    }
};
template <int NCH>
struct RowInRegs {
    float v[NCH];
    template <typename F> __device__ __forceinline__ void for_chunks(F&& f) const {
#pragma unroll
        for (int c = 0; c < NCH; ++c) f(c, v[c]);
    }
};

// Called by all 64 lanes of one wavefront.
template <typename Row>
__device__ __forceinline__ void select_row_wave(const Row& row, const SelectRow& r, int lane) {
    const int nlo = r.nlo, m = r.m;
    float tstar = 0.f;                                      // mass of the last kept block
    int ties_kept = 0;                                      // how many blocks equal to it are kept
    bool all = r.keep_all;
    if (!all) {
        auto g = [&](float t) {
            float s = 0.f;
            row.for_chunks([&](int, float f) { s += (f >= t) ? f : 0.f; });
            return wave_sum_fixed(s);
        };
        if (!(g(0.f) >= r.tau)) {
            all = true;                                     // the whole row does not reach tau (rounding): keep it
        } else {
            unsigned lo = 0u, hi = 0x7f800001u;             // g(lo) >= tau > g(hi)
            while (hi - lo > 1u) {
                const unsigned mid = lo + ((hi - lo) >> 1);
                if (g(__uint_as_float(mid)) >= r.tau) lo = mid; else hi = mid;
            }
            tstar = __uint_as_float(lo);                    // > 0: the positive entries alone already reach tau
            float above = 0.f;
            int nties = 0;
            row.for_chunks([&](int, float f) {
                above += (f > tstar) ? f : 0.f;
                nties += (f == tstar) ? 1 : 0;
            });
            above = wave_sum_fixed(above);
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) nties += __shfl_xor(nties, o);
            float run = above;
            do { run += tstar; ++ties_kept; } while (run < r.tau && ties_kept < nties);
        }
    }
    // flags -> ascending list, count, dense row
    int pos = 0, tie_seen = 0;
    row.for_chunks([&](int c, float f) {
        const int n = 64 * c + lane;
        const bool cand = n >= nlo && n <= m;
        const bool tie = cand && !all && f == tstar;
        const unsigned long long tb = __ballot(tie);
        const int rank = tie_seen + __popcll(tb & ((1ull << lane) - 1ull));
        tie_seen += __popcll(tb);
        const bool sel = cand && (all || f > tstar || (tie && rank < ties_kept) ||
                                  n - nlo < r.sink_blocks || n > m - r.recent_blocks);
        const unsigned long long sb = __ballot(sel);
        if (sel) r.list[pos + __popcll(sb & ((1ull << lane) - 1ull))] = n;
        pos += __popcll(sb);
        if (r.dense && n < r.Nb) r.dense[n] = sel ? 1 : 0;
    });
    if (lane == 0) *r.count = pos;
    // dense entries of the chunks that hold no candidate
    if (r.dense) {
        const int c0 = nlo >> 6, c1 = (m >> 6) + 1;
        for (int n = lane; n < r.Nb; n += 64) {
            const int c = n >> 6;
            if (c < c0 || c >= c1) r.dense[n] = 0;
        }
    }
}

}  // namespace rr
