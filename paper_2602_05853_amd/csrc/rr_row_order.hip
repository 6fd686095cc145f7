// Scheduling hint for the sparse attention launch: per (batch, KV head) the rows (hl, m) of its G
// query heads in the order their workgroups should start.
//
// Balance.  Workgroups are handed to the XCDs round-robin in launch order and a workgroup cannot start
// before the one launched ahead of it: rows of very different length next to each other (Top-tau
// keeps anything from a handful of blocks to all of them, Sec. 3.3) leave compute units idle, rows of
// equal length side by side do not.  Rows are therefore sorted by count class (count / 8), heaviest
// class first.
// Locality.  Inside a class rows go by descending query block, the G heads of a query block together:
// such neighbours select many of the same key blocks and walk them at the same pace.  Within every
// run of 8 G sorted rows the launch ranks are transposed, so that G consecutive sorted rows get ranks 8
// apart and meet in the L2 of one XCD.  The order is a pure function of the counts (deterministic).
//
// One workgroup per (batch, KV head): keys (class << 15 | (Nb-1-m) * G + hl) are sorted in LDS with a
// bitonic network.  G * Nb <= 32768 rows (the caller checks).
#include "rr_common.hpp"

namespace rr {

namespace {

constexpr int kSortThreads = 1024;
constexpr int kCountShift = 3;      // rows whose counts differ by less than 8 blocks form one class

__global__ void __launch_bounds__(kSortThreads)
k_row_order(Geom g, int Nb, int P2, const int32_t* __restrict__ row_count, int32_t* __restrict__ row_order,
            int32_t* __restrict__ queue) {
    extern __shared__ unsigned int keys[];
    const int t = threadIdx.x;
    const int kv = blockIdx.x, b = blockIdx.y;
    // the row counters of the attention launch that will follow this order start from zero
    if (queue && kv == 0 && b == 0 && t < RR_QUEUE_WORDS) queue[t] = 0;
    const int Nbq = g.Lq / (g.L / Nb);                  // rows per head (chunked prefill: the last Nbq query blocks)
    const int N = g.G * Nbq;
    const int32_t* cnt = row_count + ((long long)b * g.Hq + (long long)kv * g.G) * Nbq;   // G heads, contiguous
    for (int i = t; i < P2; i += kSortThreads) {
        unsigned int key = 0xFFFFFFFFu;
        if (i < N) {
            int c = cnt[i];
            c = c < 0 ? 0 : (c > Nb ? Nb : c);
            const int hl = i / Nbq, m = i - hl * Nbq;
            const unsigned f = (unsigned)(Nbq - 1 - m) * g.G + hl;            // m descending, then head
            key = (((unsigned)(Nb - c) >> kCountShift) << 15) | f;
        }
        keys[i] = key;
    }
    __syncthreads();
    for (int k = 2; k <= P2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            // one compare-exchange per loop trip: pair p is (i, i + j) with bit j of i clear
            for (int p = t; p < (P2 >> 1); p += kSortThreads) {
                const int i = ((p & ~(j - 1)) << 1) | (p & (j - 1));
                const int x = i | j;
                const unsigned int ka = keys[i], kb = keys[x];
                const bool sw = (ka > kb) == ((i & k) == 0);
                keys[i] = sw ? kb : ka;
                keys[x] = sw ? ka : kb;
            }
            __syncthreads();
        }
    }
    int32_t* out = row_order + ((long long)b * g.Hkv + kv) * N;
    // Rows that are neighbours in the sorted sequence (same count class, same or adjacent query block, the
    // G heads of one KV head) share many key blocks and walk them at the same pace.  Workgroups go to the
    // XCDs round-robin in launch order, so within every run of 8 G sorted rows the launch order is
    // transposed: G consecutive sorted rows get ranks 8 apart and meet in the L2 of one XCD.
    const int C = g.G;
    const int full = N / (8 * C) * (8 * C);
    for (int i = t; i < N; i += kSortThreads) {
        const unsigned f = keys[i] & 0x7FFFu;
        const int mr = f / g.G, hl = f - mr * g.G;
        int rank = i;
        if (C > 1 && i < full) {
            const int base = i / (8 * C) * (8 * C), w = i - base;
            rank = base + 8 * (w % C) + w / C;
        }
        out[rank] = hl * Nbq + (Nbq - 1 - mr);
    }
}

// dense 0/1 rows -> count and ascending list, one wave per (batch, head, row); entries above the
// diagonal are ignored.  Lanes scan 64 columns at a time, the rank of a set column is the count of set
// columns before it (ballot + popcount).
__global__ void __launch_bounds__(256)
k_mask_from_dense(long long rows, int Nb, int Nbq, const uint8_t* __restrict__ dense, int32_t* __restrict__ row_count,
                  int32_t* __restrict__ row_list) {
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    const int m = (Nb - Nbq) + (int)(row % Nbq);
    const uint8_t* src = dense + row * Nb;
    int32_t* dst = row_list + row * Nb;
    int count = 0;
    for (int n0 = 0; n0 <= m; n0 += 64) {
        const int n = n0 + lane;
        const bool set = n <= m && src[n] != 0;
        const unsigned long long bal = __ballot(set);
        if (set) dst[count + __popcll(bal & ((1ull << lane) - 1ull))] = n;
        count += __popcll(bal);
    }
    if (lane == 0) row_count[row] = count;
}

}  // namespace

hipError_t launch_mask_from_dense(const Geom& g, int Nb, const uint8_t* dense, int32_t* row_count, int32_t* row_list,
                                  hipStream_t st) {
    const int Nbq = g.Lq / (g.L / Nb);
    const long long rows = (long long)g.batch * g.Hq * Nbq;
    hipLaunchKernelGGL(k_mask_from_dense, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, rows, Nb, Nbq, dense,
                       row_count, row_list);
    return hipGetLastError();
}

hipError_t launch_row_order(const Geom& g, int Nb, const int32_t* row_count, int32_t* row_order, int32_t* queue,
                            hipStream_t st) {
    const int N = g.G * (g.Lq / (g.L / Nb));
    if (N > kMaxOrderedRows) return hipErrorInvalidValue;
    int P2 = 1;
    while (P2 < N) P2 <<= 1;
    const size_t lds = (size_t)P2 * sizeof(unsigned int);
    hipError_t e = allow_dynamic_lds((const void*)k_row_order, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_row_order, dim3(g.Hkv, g.batch), dim3(kSortThreads), lds, st, g, Nb, P2, row_count, row_order, queue);
    return hipGetLastError();
}

}  // namespace rr
