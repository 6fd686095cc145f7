// Kernel group (3), MFMA form: causal block-sparse flash attention (Sec. 2.1) for bf16 tensors
// with d = 128 and B = 128 on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// One workgroup (8 waves, two per SIMD) per (batch, head, query block m); it walks the compacted
// ascending list of selected key blocks of that row (or every n <= m for the dense baseline).
//
// Transposed products.  S^T = K Q^T and O^T = V^T P^T, so a lane always owns one QUERY (MFMA
// column = lane % 32): the softmax statistics of a query are per-lane scalars, and the fp32 S^T
// accumulators, rounded to bf16, already ARE the B operand of the second product -- P never goes
// through LDS.  The k-index order inside an MFMA is free as long as both operands agree, so V^T
// is laid out in LDS in exactly the key order in which the S^T accumulators hold the keys
// (0-3, 8-11 | 4-7, 12-15 of every 16).
//
// Work split.  Wave w owns the 32 queries 32*(w % 4) .. +31 and keys 64*(w / 4) .. +63 of every key
// block (NQT = 1 subtile of 32 queries per wave; the code is written for NQT subtiles, NQT = 2 being
// four waves of 64 queries whose LDS fragments feed two MFMAs each).  The two key halves of a query
// are merged once at the end.  A wave's 64 keys are taken in two steps of 32.  Measured on MI355X
// both splits run at the same speed: under this kernel the chip is power limited (the clock drops
// from 2.39 GHz to 1.98-2.2 GHz); the 8-wave split needs 11 % fewer cycles but reads twice as much
// from LDS.  It is kept because it leaves half the registers free (128 + 104 of 512 per lane).
//
// Software pipeline.  On this chip the vector ALU instructions of a SIMD do not run in the shadow
// of its MFMAs for more than a few cycles per MFMA (measured: 32 MFMAs + the softmax of 32 scores
// take 1320 cycles against 975 for the MFMAs alone, with one or two waves per SIMD alike), but LDS
// reads, tile copies and scalar work do, so the steps are skewed: phase j issues the MFMAs of
// PV(step j-1) and QK(step j+1) interleaved with the softmax of step j, one element per
// MFMA slot.  The softmax itself is pipelined over the slots (scale, exp2, bf16 rounding and row sum of
// an element sit in four different slots), so that a wave never issues a vector instruction right behind
// the one that produces its operand.  The running maximum is lazy: P is taken relative to a reference that is only moved
// (with a rescale of O^T and the denominator) when a new maximum exceeds it by 2^8, which keeps the
// common path branch-free and exact (all terms of a row share the reference).
//
// Staging.  K and V tiles go global -> LDS directly (global_load_lds, 16 bytes per lane, no
// staging registers), row-major, double-buffered one key block ahead.  K fragments are plain
// 16-byte LDS reads; V^T fragments come out of the row-major V tile through the transposing LDS
// read (ds_read_b64_tr_b16: within 16 lanes, lane 4e+q supplies four consecutive d of key e and
// lane 4q+c receives element c of all four keys).  Each tile has its own XOR swizzle of the
// 16-byte chunks so that these reads are bank-conflict-free.
// The diagonal block (token-causal mask) is handled after the pipeline by a plain masked pass that skips
// the steps no query of the wave can see; its tile is fetched by the pipeline's last two copy slots.
//
// Lengths.  When the real length ends inside the last block (kRagged), that block is the only partial
// tile: it is read by the diagonal pass alone, through copies whose source rows stop at the last real
// position; query rows past the length work on a copy of the last real row and are not stored.
#include "rr_common.hpp"

#include <atomic>
#include <type_traits>

namespace rr {

namespace {

constexpr int NQT = 1;                               // 32-query subtiles per wave
constexpr int kQWaves = 128 / (32 * NQT);            // waves along the queries
constexpr int kWaves = 2 * kQWaves;                  // x 2 key halves
constexpr int kThreads = 64 * kWaves;
constexpr int kRowsPerWave = 128 / kWaves;           // tile rows each wave copies
constexpr int kCopies = kRowsPerWave / 4;            // copy instructions per wave and tile (4 rows each)
constexpr int kTileBytes = 128 * 256;                // one 128 x 128 bf16 tile
constexpr int kLdsBytes = 4 * kTileBytes;            // K and V^T, two stages each
constexpr int kXchgFloats = 66 * NQT;                // per lane: 64 accumulators + max + sum per subtile
constexpr int kOutRowBytes = 264;                    // 128 bf16 + 8 bytes of padding
constexpr float kLazyLog2 = 8.0f;                    // move the softmax reference when exceeded by 2^8
constexpr float kLazySum = 256.0f;                   // = 2^kLazyLog2: a lane's 16-term sum above it triggers the move

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
typedef __attribute__((address_space(3))) int lds_int_t;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr_t;

__device__ __forceinline__ int k_swz(int key, int chunk) { return key * 256 + ((chunk ^ (key & 15)) << 4); }
__device__ __forceinline__ int v_swz(int key, int chunk) { return key * 256 + ((chunk ^ ((key & 7) << 1)) << 4); }

// workgroup id -> (batch, head, query block).  Workgroups are dealt to the 8 XCDs round-robin
// (id % 8 picks the XCD) and start in id order.  When Nb is a multiple of 8 the KV groups are
// taken `gi` at a time GPU-wide, so that the keys and values in use stay cache resident and L2 misses of
// the sparse walk stay off HBM (gi = 1 at 128K tokens, where one group's K and V are 64 MB);
// XCD x takes the rows with rank = x (mod 8), the query heads of a group back to back, rows heaviest
// (largest m) first.  Otherwise XCDs are given whole KV groups where the counts allow it.
// Interleaving.  Inside a set of gi groups the launch goes rank by rank, not group by group: every group's
// heaviest row, then every group's second, ...  Taken one after the other, each group would end with a tail
// of light rows that leaves compute units idle while the next group's heavy rows have not started; with few
// rows per compute unit (short contexts) those tails were a quarter of the launch.  The position of a group
// inside a rank rotates with the rank, so that an XCD is not always handed the same (perhaps heaviest) group.
// Ordered launches: the entry of the caller-supplied row order (rows of each KV group, heaviest first) that
// launch rank `bid` stands for, with the batch index and the first query head of its KV group.  Sets of gi
// groups, rank by rank inside a set, the group's position rotating with the rank.
__device__ __forceinline__ int order_entry_of(int bid, const Geom& g, int Nb, const int32_t* order, int gi,
                                              int& b, int& h0) {
    const int N = g.G * Nb;
    const int set = bid / (gi * N), r = bid - set * (gi * N);
    const int rank = r / gi;
    const int grp = set * gi + (r - rank * gi + rank) % gi;
    b = grp / g.Hkv;
    h0 = (grp - b * g.Hkv) * g.G;
    return order[(long long)grp * N + rank];
}

__device__ __forceinline__ bool decode_block(int bid, const Geom& g, int Nb, const int32_t* order, int a_interleave,
                                             int& b, int& h, int& m) {
    const int NG = g.batch * g.Hkv, G = g.G;
    int mr, grp, hl;
    if (order) {
        const int v = order_entry_of(bid, g, Nb, order, a_interleave, b, h);
        if ((unsigned)v >= (unsigned)(G * Nb)) return false;
        hl = v / Nb;
        m = v - hl * Nb;
        h += hl;
        return true;
    }
    if ((Nb & 7) == 0) {
        // one KV group after the other GPU-wide (its keys and values then fit the memory-side
        // cache); XCD x takes the rows with rank = x mod 8, the heads of a group back to back
        const int x = bid & 7, s = bid >> 3;
        hl = s % G;
        const int q = s / G, nb8 = Nb >> 3, gi = a_interleave;
        const int set = q / (gi * nb8), q2 = q - set * (gi * nb8);
        const int level = q2 / gi;                        // eight ranks of every group of the set, then the next eight
        grp = set * gi + (q2 - level * gi);
        // the residue an XCD takes rotates with the head: rows that are heavy in every head (the
        // protected last row keeps all blocks) are then spread over the XCDs instead of piling up on one
        mr = level * 8 + ((x + grp * G + hl) & 7);
    } else if ((NG & 7) == 0) {
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

__host__ unsigned grid_size(const Geom& g, int Nb, bool ordered) {
    const int NG = g.batch * g.Hkv;
    if (ordered) return (unsigned)NG * g.G * Nb;
    if ((Nb & 7) == 0) return (unsigned)NG * g.G * Nb;
    if ((NG & 7) != 0 && 8 % NG == 0) {
        const int k = 8 / NG;
        return 8u * g.G * ((Nb + k - 1) / k);
    }
    return (unsigned)NG * g.G * Nb;
}

#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// The MFMAs are one-instruction asm statements so that the register class of every operand is
// fixed by hand: O^T and the Q^T operand live in the accumulation registers (only the matrix
// pipe touches them), S^T lands in ordinary vector registers because the softmax reads it with
// vector ALU instructions.  (Left to itself the compiler puts every MFMA result in accumulation
// registers and copies S^T out and back around each instruction.)
// The compiler does not see inside these statements and adds no wait states for them.  The code
// keeps the distances itself: inside the pipeline a result is only reused as the accumulator of
// the next MFMA of its chain (which the matrix pipe interlocks) or, for S^T, read by vector
// instructions a whole phase and a barrier later; wherever else vector instructions touch a
// result, a settle statement comes first.
#define RR_MFMA_TEXT "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
__device__ __forceinline__ void mfma_pv(f32x16& acc, const bf16x8& vt, const bf16x8& pt) {
    asm volatile(RR_MFMA_TEXT : "+a"(acc) : "v"(vt), "v"(pt));
}
__device__ __forceinline__ void mfma_qk(f32x16& s, const bf16x8& k, const bf16x8& qt) {
    asm volatile(RR_MFMA_TEXT : "+v"(s) : "v"(k), "a"(qt));
}
__device__ __forceinline__ void mfma_qk_first(f32x16& s, const bf16x8& k, const bf16x8& qt) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(k), "a"(qt));
}
// Idle issue cycles longer than the tail of the last MFMA, then the values pass through empty
// asm statements: whatever reads them afterwards depends on those statements and therefore
// cannot be scheduled in front of the idle cycles.
__device__ __forceinline__ void mfma_settle_s(f32x16 (&s)[NQT]) {
    if constexpr (NQT == 2) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(s[0]), "+v"(s[NQT - 1]));
    else asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(s[0]));
}
__device__ __forceinline__ void mfma_settle_acc(f32x16 (&acc)[4][NQT]) {
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15");
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) asm volatile("" : "+a"(acc[dt][qt]));
}

// Per-wave state and operand addressing.
struct Wave {
    const lds_byte_t* lds;
    int lane, l32, gsel, qi, ki;
    float sl2;                         // log2(e) / sqrt(d)
    bf16x8 qf[NQT][8];                 // Q^T operand: [32-query subtile][16-wide d chunk]
    f32x16 acc[4][NQT];                // O^T: [32-row d tile][32-query subtile]
    float mref[NQT];                   // softmax reference of the lane's queries, log2 units
    float lsum[NQT];                   // this lane's part of the denominators
    // Per-lane LDS byte addresses.  The XOR swizzle makes the chunk part of an address
    // base ^ (32 * kc) for K and base ^ (64 * dt) for V.
    unsigned ka0;                      // K: row (64 ki + lane%32), chunk gsel, swizzled
    unsigned va0;                      // V: keys 4 gsel + (lane%16)/4 of the wave's half, d tile 0
    // ... and all of them, so that the hot loop forms no address: the chunk part is kaddr[kc] = ka0 ^ 32 kc,
    // vaddr[dt] = va0 ^ 64 dt; buffer, subtile and key-chunk selection ride in the instruction's immediate
    // offset (the loop is unrolled over the buffer parity for that).
    unsigned kaddr[8];
    unsigned vaddr[4];

    __device__ __forceinline__ void init_addresses() {
        const unsigned lds0 = (unsigned)(uintptr_t)lds;       // LDS addresses are 32 bits
        ka0 = lds0 + k_swz(64 * ki + l32, gsel);
        const int s16 = lane & 15, dhalf = (lane >> 4) & 1;
        const int key = 64 * ki + 4 * gsel + (s16 >> 2);
        va0 = lds0 + 2 * kTileBytes + 8 * (s16 & 1) + v_swz(key, 2 * dhalf + ((s16 & 3) >> 1));
#pragma unroll
        for (int kc = 0; kc < 8; ++kc) kaddr[kc] = ka0 ^ (32u * kc);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) vaddr[dt] = va0 ^ (64u * dt);
    }
    __device__ __forceinline__ unsigned ka(int kc) const { return ka0 ^ (32u * kc); }
    __device__ __forceinline__ unsigned va(int dt) const { return va0 ^ (64u * dt); }
    __device__ __forceinline__ bf16x8 kfrag_at(unsigned at, int buf, int t) const {
        return *(const lds_bf16x8_t*)(uintptr_t)(at + (unsigned)(buf * kTileBytes + t * 32 * 256));
    }
    // fragment reads of the pipeline: address register + compile-time byte offset
    template <int OFF>
    __device__ __forceinline__ bf16x8 kfrag_imm(int kc) const {
        return *(const lds_bf16x8_t*)(uintptr_t)(kaddr[kc] + (unsigned)OFF);
    }
    template <int OFF>
    __device__ __forceinline__ bf16x8 vfrag_imm(int u) const { return vfrag_at(vaddr[u >> 1] + (unsigned)OFF, 0, 0, u); }
    __device__ __forceinline__ bf16x8 kfrag(int buf, int t, int kc) const { return kfrag_at(ka(kc), buf, t); }
    // V^T operand (32 d rows x 16 keys) of d tile u >> 1 and 16-key chunk u & 1 of subtile t: two
    // transposing reads, keys {4g..4g+3} and {8+4g..8+4g+3} of the chunk (accumulator order).
    __device__ __forceinline__ bf16x8 vfrag(int buf, int t, int u) const { return vfrag_at(va(u >> 1), buf, t, u); }
    __device__ __forceinline__ bf16x8 vfrag_at(unsigned at, int buf, int t, int u) const {
        const unsigned p = at + (unsigned)(buf * kTileBytes + t * 32 * 256 + (u & 1) * 16 * 256);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)(uintptr_t)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)(uintptr_t)(p + 8 * 256));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    }
};

// S^T of one 32-key step, nothing overlapped (pipeline prologue and the diagonal block).
__device__ __forceinline__ void qk_step(const Wave& w, int buf, int t, f32x16 (&s)[NQT]) {
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) {
        const bf16x8 kf = w.kfrag(buf, t, kc);
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            if (kc == 0) mfma_qk_first(s[qt], kf, w.qf[qt][kc]);
            else mfma_qk(s[qt], kf, w.qf[qt][kc]);
        }
    }
    mfma_settle_s(s);
}

// O^T += V^T P^T of one 32-key step, nothing overlapped.
__device__ __forceinline__ void pv_step(Wave& w, int buf, int t, const bf16x8 (&p)[NQT][2]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const bf16x8 vf = w.vfrag(buf, t, u);
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) mfma_pv(w.acc[u >> 1][qt], vf, p[qt][u & 1]);
    }
    mfma_settle_acc(w.acc);
}

// exp2 of the 32 scores of a step against the current reference; fills P, returns sums and maxima.
__device__ __forceinline__ void exp_all(const Wave& w, const f32x16 (&s)[NQT], bf16x8 (&p)[NQT][2],
                                        float (&psum)[NQT], float (&mx)[NQT]) {
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const float nb = -w.mref[qt];
        psum[qt] = 0.f;
        mx[qt] = -__builtin_huge_valf();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float e = __builtin_amdgcn_exp2f(fmaf(s[qt][r], w.sl2, nb));
            psum[qt] += e;
            mx[qt] = fmaxf(mx[qt], s[qt][r]);
            p[qt][r >> 3][r & 7] = (__bf16)e;
        }
    }
}

// Moves the softmax reference of the lane's queries up to the new maximum, rescales O^T and the
// denominator, and recomputes P of the step at hand.  Rare; entered by the whole wave.
__device__ __forceinline__ void move_reference(Wave& w, const f32x16 (&s)[NQT], bf16x8 (&p)[NQT][2],
                                               float (&psum)[NQT], float (&mx)[NQT]) {
    mfma_settle_acc(w.acc);                             // O^T is about to be read by vector instructions
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        float top = mx[qt] * w.sl2;
        top = fmaxf(top, __shfl_xor(top, 32));
        const float nref = fmaxf(w.mref[qt], top);
        const float use = (nref == -__builtin_huge_valf()) ? 0.f : nref;
        const float alpha = __builtin_amdgcn_exp2f(w.mref[qt] - use);   // 0 while the reference is -inf
        w.mref[qt] = nref;
        w.lsum[qt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.acc[dt][qt][r] *= alpha;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float e = __builtin_amdgcn_exp2f(fmaf(s[qt][r], w.sl2, -use));
            sum += e;
            p[qt][r >> 3][r & 7] = (__bf16)e;
        }
        psum[qt] = sum;
    }
    mfma_settle_acc(w.acc);                             // ... and was written by them
}

__device__ __forceinline__ void finish_softmax(Wave& w, const f32x16 (&s)[NQT], bf16x8 (&p)[NQT][2],
                                               float (&psum)[NQT], float (&mx)[NQT], bool valid = true) {
    if (!valid) return;                                 // a fill phase of the pipeline: nothing to keep
    bool need = false;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) need = need || (mx[qt] * w.sl2 > w.mref[qt] + kLazyLog2);
    if (__any(need)) move_reference(w, s, p, psum, mx);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) w.lsum[qt] += psum[qt];
}

// Global -> LDS copies of one 128 x 128 bf16 tile, kCopies instructions per wave (4 rows each), issued
// as asm statements: the compiler would otherwise make every later LDS read wait for them (it
// cannot tell that the reads go to the other buffer), which turns the prefetch into a blocking
// copy.  The kernel waits for them itself (wait_vm) before the barrier that hands a buffer over.
// Lane l lands in LDS slot (row l/16 of the group, physical chunk l%16) and therefore fetches
// logical chunk (l%16) ^ swizzle(row); the per-lane byte offsets of the 8 row groups are kept in
// registers, the tile origin is wave-uniform.
struct Stager {
    const unsigned short* Kp;
    const unsigned short* Vp;
    long long ksl;
    unsigned lds0;                     // LDS address of the buffers
    int wv;                            // wave index, uniform
    unsigned koff[kCopies];            // K: byte offset of this lane's 16 bytes in row group i
    unsigned voff[kCopies];            // V: same with the V swizzle

    __device__ __forceinline__ void init(int lane) {
        const int r4 = lane >> 4, c = lane & 15;
#pragma unroll
        for (int i = 0; i < kCopies; ++i) {
            const int row = 4 * i + r4;                    // row inside the wave's rows (16 | rows per wave: swizzle period)
            koff[i] = 2u * ((unsigned)(row * ksl) + 8u * (c ^ (row & 15)));
            voff[i] = 2u * ((unsigned)(row * ksl) + 8u * (c ^ ((row & 7) << 1)));
        }
    }
    // one of the copies of a tile: row group i of this wave's rows
    __device__ __forceinline__ void issue_one(const unsigned short* wave_src, unsigned wave_dst,
                                              const unsigned (&off)[kCopies], int i) const {
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(off[i]), "s"(wave_src), "s"(wave_dst + 4 * i * 256) : "memory");
    }
    __device__ __forceinline__ const unsigned short* k_src(int n) const { return Kp + ((long long)n * 128 + kRowsPerWave * wv) * ksl; }
    __device__ __forceinline__ const unsigned short* v_src(int n) const { return Vp + ((long long)n * 128 + kRowsPerWave * wv) * ksl; }
    __device__ __forceinline__ unsigned k_dst(int buf) const { return lds0 + buf * kTileBytes + kRowsPerWave * wv * 256; }
    __device__ __forceinline__ unsigned v_dst(int buf) const { return lds0 + (2 + buf) * kTileBytes + kRowsPerWave * wv * 256; }
    // A tile whose last rows lie past the real length (`rows` real rows, 1 <= rows < 128): those LDS rows get a
    // copy of the last real row (finite, and masked by token causality wherever a real query meets them).
    // Offsets are formed on the spot from the tile origin: this path runs once per launch row at most.
    __device__ __forceinline__ void issue_partial(const unsigned short* base, int n, unsigned dst, bool is_v, int rows,
                                                  int lane) const {
        const unsigned short* tile = base + (long long)n * 128 * ksl;
        const int r4 = lane >> 4, c = lane & 15;
#pragma unroll
        for (int i = 0; i < kCopies; ++i) {
            const int row = 4 * i + r4;                      // LDS row inside the wave's rows: decides the swizzle
            const int src_row = min(kRowsPerWave * wv + row, rows - 1);
            const unsigned sw = is_v ? ((row & 7) << 1) : (row & 15);
            const unsigned off = 2u * ((unsigned)(src_row * ksl) + 8u * (c ^ sw));
            asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                         :: "v"(off), "s"(tile), "s"(dst + 4 * i * 256) : "memory");
        }
    }
    __device__ __forceinline__ void issue_k(int n, int buf) const {
#pragma unroll
        for (int i = 0; i < kCopies; ++i) issue_one(k_src(n), k_dst(buf), koff, i);
    }
    __device__ __forceinline__ void issue_v(int n, int buf) const {
#pragma unroll
        for (int i = 0; i < kCopies; ++i) issue_one(v_src(n), v_dst(buf), voff, i);
    }
};

__device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// One pipeline phase: the MFMAs of PV(step j-1) [V^T fragments from LDS base vbase, operand pprev]
// and of QK(step j+1) [K fragments from kbase, result snext] interleaved with the exp2 / sum /
// max / bf16 rounding of step j [scores scur -> pcur], one element per MFMA slot, and (kFetch)
// with the wave's global -> LDS copies of the prefetched K and V tiles, one every other slot, so the
// copies never queue up in front of the arithmetic.  `valid` is false for the two fill phases at either end of a
// row, whose softmax is thrown away.
template <bool kFetch, int VOFF, int KOFF>
__device__ __forceinline__ void phase(Wave& w, const f32x16 (&scur)[NQT], f32x16 (&snext)[NQT],
                                      const bf16x8 (&pprev)[NQT][2], bf16x8 (&pcur)[NQT][2],
                                      bool valid, const Stager& st,
                                      const unsigned short* k_src, unsigned k_dst,
                                      const unsigned short* v_src, unsigned v_dst) {
    // The empty asm statements emit nothing.  Being ordered among themselves and with the MFMA
    // statements, they keep the compiler from sinking the softmax arithmetic out of the MFMA
    // shadow or hoisting all operand reads to the top.
    bf16x8 vf[2], kf[2];
    vf[0] = w.template vfrag_imm<VOFF>(0);
    kf[0] = w.template kfrag_imm<KOFF>(0);
    float psum[NQT], nb[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) { psum[qt] = 0.f; nb[qt] = -w.mref[qt]; }
    bf16x2 ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;
    // Softmax of step j, software pipelined over the MFMA slots so that no vector instruction waits for the
    // one in front of it: stage A (scale and shift of element k) runs at step k, B (its exp2) at step k + 1,
    // C (rounding the pair (2j, 2j+1) to bf16, which is what PV will use) at step 2j + 3, D (adding the pair to
    // the row sum) at step 2j + 4.
    constexpr int NE = 16 * NQT;
    float tq[NE], ev[NE];
    auto step = [&](int sidx) {
        if (sidx >= 1 && sidx - 1 < NE) {                           // B
            ev[sidx - 1] = __builtin_amdgcn_exp2f(tq[sidx - 1]);
            asm volatile("" : "+v"(ev[sidx - 1]));
        }
        if (sidx < NE) {                                            // A
            tq[sidx] = fmaf(scur[sidx >> 4][sidx & 15], w.sl2, nb[sidx >> 4]);
            asm volatile("" : "+v"(tq[sidx]));
        }
        if (sidx >= 3 && (sidx & 1) && (sidx - 3) / 2 < NE / 2) {   // C
            const int j = (sidx - 3) / 2, eq = (2 * j) >> 4, er = (2 * j) & 15;
            bf16x2 pr;
            pr[0] = (__bf16)ev[2 * j];
            pr[1] = (__bf16)ev[2 * j + 1];
            pcur[eq][er >> 3][er & 7] = pr[0];
            pcur[eq][er >> 3][(er & 7) + 1] = pr[1];
            asm volatile("" : "+v"(pcur[eq][er >> 3]));
        }
        if (sidx >= 4 && !(sidx & 1) && (sidx - 4) / 2 < NE / 2) {  // D
            const int j = (sidx - 4) / 2, eq = (2 * j) >> 4, er = (2 * j) & 15;
            bf16x2 pr;
            pr[0] = pcur[eq][er >> 3][er & 7];
            pr[1] = pcur[eq][er >> 3][(er & 7) + 1];
            psum[eq] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum[eq], false);   // sums what PV will use
            asm volatile("" : "+v"(psum[eq]));
        }
    };
    // The scores of this step were completed by the last QK MFMA of the previous phase (an asm statement, so the
    // compiler adds no wait states for it); a vector instruction may read them 11 wait states after that MFMA
    // was issued.  The previous phase ends with a PV MFMA, which the matrix pipe accepts 8 wait states after
    // the QK one; the operand reads above and this statement add the rest whatever the compiler puts in
    // between.  The scores pass through the statement, so nothing that reads them can be scheduled in front.
    {
        f32x16& first = const_cast<f32x16&>(scur[0]);
        if constexpr (NQT == 2) asm volatile("s_nop 2" : "+v"(first), "+v"(const_cast<f32x16&>(scur[NQT - 1])));
        else asm volatile("s_nop 2" : "+v"(first));
    }
    // four steps run ahead of the first MFMA: they fill the softmax pipeline and cover the latency of the first
    // operand reads
    step(0);
    step(1);
    step(2);
    step(3);
    SCHED_FENCE();
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        // operand fragments of the next group are requested one group (4 MFMA slots) ahead
        if (u < 7) {
            vf[(u + 1) & 1] = w.template vfrag_imm<VOFF>(u + 1);
            kf[(u + 1) & 1] = w.template kfrag_imm<KOFF>(u + 1);
        }
#pragma unroll
        for (int sl = 0; sl < 2 * NQT; ++sl) {
            const int qt = sl >> 1;
            // QK before PV: the phase then ends with a PV product, and the scores of the next step are complete
            // one MFMA earlier
            if ((sl & 1) == 0) {
                if (u == 0) mfma_qk_first(snext[qt], kf[0], w.qf[qt][0]);
                else mfma_qk(snext[qt], kf[u & 1], w.qf[qt][u]);
            } else {
                mfma_pv(w.acc[u >> 1][qt], vf[u & 1], pprev[qt][u & 1]);
            }
            if constexpr (NQT == 2) {
                if (kFetch && sl == 0) st.issue_one(k_src, k_dst, st.koff, u);
                if (kFetch && sl == 2) st.issue_one(v_src, v_dst, st.voff, u);
            } else {
                if (kFetch && sl == 0 && (u & 1) == 0) st.issue_one(k_src, k_dst, st.koff, u >> 1);
                if (kFetch && sl == 0 && (u & 1) == 1) st.issue_one(v_src, v_dst, st.voff, u >> 1);
            }
            step(2 * NQT * u + sl + 4);
            SCHED_FENCE();
        }
    }
    // A score more than 2^8 above the reference makes its term, hence the lane's sum of 16 terms,
    // exceed 2^8 (the first step of a row, whose reference is -inf, gives +inf): the sum is the
    // trigger, the maximum itself is only computed on the rare path.
    if (valid) {
        bool need = false;
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) need = need || !(psum[qt] <= kLazySum);
        if (__any(need)) {
            float mx[NQT];
#pragma unroll
            for (int qt = 0; qt < NQT; ++qt) {
                mx[qt] = -__builtin_huge_valf();
#pragma unroll
                for (int r = 0; r < 16; ++r) mx[qt] = fmaxf(mx[qt], scur[qt][r]);
            }
            move_reference(w, scur, pcur, psum, mx);
        }
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) w.lsum[qt] += psum[qt];
    }
}

// Row queue of the persistent form: one counter per XCD, each on a cache line of its own, and one count of the
// workgroups that have left.  All zero between launches.
constexpr int kQueueStride = 16;                       // int32 words between counters
constexpr int kQueueDone = 8 * kQueueStride;

// The kernel's arguments as one struct, so that the persistent form can read them again from the kernel
// argument segment whenever it needs them instead of keeping ~50 scalar registers alive across its row loop
// (which pushed scalars into vector registers and those into scratch memory).
struct AttnKernelArgs {
    Geom g;
    AttnArgs a;
    float scale_log2;
};
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) AttnKernelArgs* kernarg_ptr_t;
#else
typedef const AttnKernelArgs* kernarg_ptr_t;           // the host pass only parses the kernel
#endif
// the argument segment (the struct is the first and only argument, at offset 0); `fresh` hides from the compiler
// that it is the pointer it already knows, so that loads through it are made where they are written
template <bool kFresh>
__device__ __forceinline__ kernarg_ptr_t kernel_args() {
#if defined(__HIP_DEVICE_COMPILE__)
    kernarg_ptr_t p = (kernarg_ptr_t)__builtin_amdgcn_kernarg_segment_ptr();
    if (kFresh) asm volatile("" : "+s"(p));
    return p;
#else
    return nullptr;
#endif
}

template <bool kRagged, bool kPersist>
__global__ void __launch_bounds__(kThreads)
k_attn_mfma_bf16(AttnKernelArgs kernel_arguments) {
    // kRagged: the real length ends inside the last block (g.Lr < g.L) or the queries start inside their first
    // block (g.qoff > 0): clamped Q rows, a clamped copy of the partial diagonal tile, predicated stores.  Compiled apart so that the plain launch carries none of it
    // (both forms run at the same rate).
    //
    // kPersist (sparse launches with a row order and a queue): one workgroup per compute unit that takes row after
    // row.  Workgroup i starts with launch rank i and then draws ranks x + 8 t (x = i mod 8, the XCD the
    // dispatcher gave it) from the counter of its XCD, so that every rank keeps the XCD the order was made for
    // while the compute units of an XCD share its rows dynamically, and the next row is looked up while the
    // current one is merged and stored.
    (void)kernel_arguments;
    extern __shared__ __align__(16) unsigned char lds_generic[];
    lds_byte_t* lds = (lds_byte_t*)lds_generic;
    const bool draws = threadIdx.x == 0;                    // the lane that talks to the row queue
    const float NEG_INF = -__builtin_huge_valf();

    // ---- the next row of a persistent workgroup ----
    // Fetched in five steps, each needing what the one before it loaded: (1) a ticket from the XCD's counter,
    // published to the other waves through LDS, (2) the rank it stands for and that rank's entry of the row
    // order, (3) the row, its count and its first list entries, (4) its last list entry, (5) done.  They are
    // placed in the tail of the current row: the ticket travels during the diagonal pass, the order entry during
    // the merge, count and first entries during the output stores; only the last entry is waited for.  The ticket
    // is deliberately NOT drawn earlier (say, at the
    // start of the row, which would hide all five steps): a workgroup that claims its next row a whole row
    // ahead starts it out of step with the rows queued around it, which were ordered to walk the same key
    // blocks at the same time on one XCD; measured, the early draw cost 2-3 % at 32K-128K tokens.
    struct NextRow {
        int rank;           // launch rank, or -1 when the queue is empty
        int order_entry;    // as loaded
        bool live;          // the order entry names a row
        int b, h, mq;
        int count_raw, e0, e1, elast;
    } nx;
    nx.rank = -1; nx.live = false; nx.order_entry = 0;
    nx.b = nx.h = nx.mq = 0; nx.count_raw = nx.e0 = nx.e1 = nx.elast = 0;
    const int xcd = (int)blockIdx.x & 7;
    volatile lds_int_t* const ticket_slot = (volatile lds_int_t*)(lds + kLdsBytes);
    int ticket = 0;                                         // lane 0 of wave 0
    auto draw_issue = [&]() {
        if (draws) ticket = atomicAdd(kernel_args<true>()->a.queue + kQueueStride * xcd, 1);
    };
    auto draw_publish = [&]() {                             // readable after the next workgroup barrier
        if (draws) *ticket_slot = ticket;
    };
    auto step_order = [&](long long rank) {                 // (2); rank = workgroup index for the first row
        const kernarg_ptr_t ka = kernel_args<true>();
        const Geom g = ka->g;
        const int Nbq = g.Lq >> 7;
        nx.live = false;
        // (a queue that did not start from zero can only make the launch skip rows: a rank outside the launch ends it)
        if (rank >= 0 && rank < (long long)g.batch * g.Hq * Nbq) {
            int pb, ph;
            nx.rank = (int)rank;
            nx.order_entry = order_entry_of((int)rank, g, Nbq, ka->a.row_order, ka->a.interleave, pb, ph);
            nx.b = __builtin_amdgcn_readfirstlane(pb);
            nx.h = __builtin_amdgcn_readfirstlane(ph);
        } else {
            nx.rank = -1;
        }
    };
    auto step_rank = [&]() {
        const int t = __builtin_amdgcn_readfirstlane(*ticket_slot);
        step_order(((long long)((int)gridDim.x >> 3) + t) * 8 + xcd);
    };
    auto step_row = [&]() {                                 // (3)
        if (nx.rank < 0) return;
        const kernarg_ptr_t ka = kernel_args<true>();
        const int Nbq = ka->g.Lq >> 7;
        const int v = __builtin_amdgcn_readfirstlane(nx.order_entry);
        nx.live = (unsigned)v < (unsigned)(ka->g.G * Nbq);
        if (!nx.live) return;
        const int hl = v / Nbq;
        nx.mq = v - hl * Nbq;
        nx.h += hl;                                         // step_order left the group's first head here
        const long long rid = ((long long)nx.b * ka->g.Hq + nx.h) * Nbq + nx.mq;
        const int32_t* lp = ka->a.row_list + rid * ka->a.Nb;
        nx.count_raw = ka->a.row_count[rid];
        nx.e0 = lp[0];
        nx.e1 = lp[ka->a.Nb > 1 ? 1 : 0];
    };
    auto step_last = [&]() {                                // (4)
        if (nx.rank < 0 || !nx.live) return;
        const kernarg_ptr_t ka = kernel_args<true>();
        const int Nbq = ka->g.Lq >> 7;
        // loaded values are the same in every lane: from here on they live in scalar registers
        nx.count_raw = __builtin_amdgcn_readfirstlane(nx.count_raw);
        nx.e0 = __builtin_amdgcn_readfirstlane(nx.e0);
        nx.e1 = __builtin_amdgcn_readfirstlane(nx.e1);
        const int m = nx.mq + (ka->a.Nb - Nbq);
        int c = nx.count_raw;
        c = c < 0 ? 0 : (c > m + 1 ? m + 1 : c);
        const long long rid = ((long long)nx.b * ka->g.Hq + nx.h) * Nbq + nx.mq;
        int it = c > 0 ? c - 1 : 0;
        it = it < ka->a.Nb - 1 ? it : ka->a.Nb - 1;
        nx.elast = ka->a.row_list[rid * ka->a.Nb + it];
    };
    auto step_done = [&]() {                                // (5)
        if (nx.rank >= 0 && nx.live) nx.elast = __builtin_amdgcn_readfirstlane(nx.elast);
    };
    if (kPersist) {
        // the first row: rank = workgroup index, the same steps, each waiting for its loads
        step_order((long long)blockIdx.x);
        step_row(); step_last(); step_done();
    }

  constexpr bool kSplit = kRagged && !kPersist;          // the one instantiation that also serves split launches
  for (;;) {
    // (The persistent form reads its arguments again for every row, and derives everything that depends on the
    // lane from a thread index the compiler takes for a new value each time: hoisted out of the row loop, the
    // lane's fragment, exchange and staging addresses stayed alive through all of it and spilled.)
    int tid = threadIdx.x;
    if (kPersist) asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const kernarg_ptr_t kargs = kernel_args<kPersist>();
    const Geom g = kargs->g;
    const AttnArgs a = kargs->a;
    const float scale_log2 = kargs->scale_log2;
    // rows of the launch: the Lq / 128 query blocks of the call (chunked prefill: the last ones of the context)
    const int Nbq = g.Lq >> 7;
    int b, h, mq;
    bool have_row;
    int pf_count = 0, pf_e0 = 0, pf_e1 = 0, pf_elast = 0;
    if (kPersist) {
        if (nx.rank < 0) break;                             // the queue is empty: leave
        have_row = nx.live;
        b = nx.b; h = nx.h; mq = nx.mq;
        pf_count = nx.count_raw; pf_e0 = nx.e0; pf_e1 = nx.e1; pf_elast = nx.elast;
    }
    // split launches: which share of the row's block list this workgroup walks
    int part = kSplit ? (int)blockIdx.x % a.nsplit : 0;
    bool split = kSplit && a.nsplit > 1;
    const bool planned = kSplit && a.split_len > 0;
    int plan_slot = -1;                                     // planned launches: where this part's result goes
    if (!kPersist) {
        // A planned launch has one workgroup per slot the plan could have used and one per row.  The slots in use
        // come first (the parts of the cut rows: the longest items of the launch), then the rows (a cut row's own
        // workgroup leaves at once), and the workgroups of unused slots last, where they leave while the others finish.
        const int grid_rows = planned ? (int)gridDim.x - a.split_budget : 0;
        const int used = planned ? __builtin_amdgcn_readfirstlane(*a.plan_total) : 0;
        if (planned && (int)blockIdx.x < used) {
            plan_slot = (int)blockIdx.x;
            const int rid = __builtin_amdgcn_readfirstlane(a.plan_items[plan_slot]);
            if ((unsigned)rid >= (unsigned)(g.batch * g.Hq * Nbq)) return;
            part = plan_slot - __builtin_amdgcn_readfirstlane(a.plan_row[rid]);
            if (part < 0) return;
            mq = rid % Nbq;
            const int bh = rid / Nbq;
            h = bh % g.Hq;
            b = bh / g.Hq;
            have_row = true;
        } else {
            const int rank = (int)blockIdx.x - used;
            if (planned && rank >= grid_rows) return;
            have_row = decode_block(kSplit && !planned ? rank / a.nsplit : rank, g, Nbq, a.row_order, a.interleave, b, h, mq);
            if (planned) part = 0;
        }
        if (!have_row) return;
    }
   if (have_row) {
    // the same for every lane: keep them (and all the addresses derived from them) in scalar registers
    b = __builtin_amdgcn_readfirstlane(b);
    h = __builtin_amdgcn_readfirstlane(h);
    mq = __builtin_amdgcn_readfirstlane(mq);
    const int m = mq + (a.Nb - Nbq);                    // query block inside the context: causal limit of the row

    Wave w;
    w.lds = lds;
    w.qi = wv % kQWaves; w.ki = wv / kQWaves;
    w.lane = lane; w.l32 = lane & 31; w.gsel = lane >> 5;
    w.sl2 = scale_log2;
    w.init_addresses();
    const int qi = w.qi, ki = w.ki, l32 = w.l32, gsel = w.gsel;
    const int kv = h / g.G;
    const long long row_id = ((long long)b * g.Hq + h) * Nbq + mq;
    const unsigned short* Qp = reinterpret_cast<const unsigned short*>(a.Q) + b * g.qsb + h * g.qsh;
    Stager st;
    st.Kp = reinterpret_cast<const unsigned short*>(a.K) + b * g.ksb + kv * g.ksh;
    st.Vp = reinterpret_cast<const unsigned short*>(a.V) + b * g.ksb + kv * g.ksh;
    st.ksl = g.ksl;
    st.lds0 = (unsigned)(uintptr_t)lds;
    st.wv = wv;
    st.init(lane);

    // a caller-made list is not trusted with addresses: the count is held to [0, m+1] and entries to [0, m]
    // (a list that breaks the contract gives a wrong row, never an access outside K and V)
    // the dense walk starts at block 0, or (packed sequences) at the first block of the row's sequence
    int first_in = (!a.row_list && a.seq_first) ? a.seq_first[m] : 0;
    first_in = first_in < 0 ? 0 : (first_in > m ? m : first_in);
    const int first = __builtin_amdgcn_readfirstlane(first_in);
    int count_in = kPersist ? pf_count : (a.row_list ? a.row_count[row_id] : (m + 1 - first));
    count_in = count_in < 0 ? 0 : (count_in > m + 1 ? m + 1 : count_in);
    int count = __builtin_amdgcn_readfirstlane(count_in);
    // a split launch: entries [list_lo, list_lo + count) of the row's list are this workgroup's; the diagonal
    // block (always the last entry) belongs to the part that holds the end of the list
    int list_lo = 0;
    bool last_part = true;
    if (planned) {
        // the plan decides: a row without slots is an ordinary row that stores its own result
        const int base = __builtin_amdgcn_readfirstlane(a.plan_row[row_id]);
        split = base >= 0;
        if (split != (plan_slot >= 0)) return;              // a cut row is computed by its slots' workgroups only
        if (split && plan_slot != base + part) return;
    }
    if (split) {
        const int len = planned ? a.split_len : (count + a.nsplit - 1) / a.nsplit;
        list_lo = min(count, part * len);
        const int hi = min(count, list_lo + len);
        last_part = hi == count;
        count = hi - list_lo;
    }
    const int32_t* list = a.row_list ? a.row_list + row_id * a.Nb + list_lo : nullptr;
    // entry `it` of the row's block list (clamped: entries are read ahead of their use); the value is
    // the same in every lane, block_at() moves it to a scalar register
    const int tile_rows = g.Lr - m * 128;               // real rows of block m; < 128 only for a partial last block
    const bool partial = kRagged && tile_rows < 128;
    auto clamp_block = [&](int n) { return n < 0 ? 0 : (n > m ? m : n); };
    auto block_raw = [&](int it) {
        it = it < a.Nb - 1 - list_lo ? it : a.Nb - 1 - list_lo;
        return clamp_block(list ? list[it] : first + list_lo + it);
    };
    // the entries a row needs before its first tile: the first two and the last (the persistent form has them
    // already)
    const int e0_raw = kPersist ? clamp_block(pf_e0) : block_raw(0);
    const int e1_raw = kPersist ? clamp_block(pf_e1) : block_raw(1);
    const int elast_raw = kPersist ? clamp_block(pf_elast) : block_raw(count > 0 ? count - 1 : 0);
    // the diagonal block, if listed, is the last entry; it is taken after the pipelined blocks
    const bool has_diag = last_part && count > 0 && __builtin_amdgcn_readfirstlane(elast_raw) == m;
    const int cnt = count - (has_diag ? 1 : 0);

    // ---- Q^T operand: this lane's query, d = 16*kc + 8*gsel .. +7, for both 32-query subtiles ----
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        // (query rows that do not exist -- past the real length, or in front of a step that starts inside its
        // first block -- work on a copy of the nearest real row)
        int row_in = mq * 128 + 32 * NQT * qi + 32 * qt + l32;
        if (kRagged) row_in = max(min(row_in - g.qoff, g.Lr - g.q0 - 1), 0);
        const long long row = row_in;
#pragma unroll
        for (int kc = 0; kc < 8; ++kc)
            w.qf[qt][kc] = *reinterpret_cast<const bf16x8*>(Qp + row * g.qsl + 16 * kc + 8 * gsel);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.acc[dt][qt][r] = 0.f;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) { w.mref[qt] = NEG_INF; w.lsum[qt] = 0.f; }

    f32x16 sa[NQT], sb[NQT];
    bf16x8 pa[NQT][2], pb[NQT][2];

    if (cnt > 0) {
        // Steps j = 2 i + t over the pipelined blocks i; K(i) sits in K buffer i & 1, V(i) in V
        // buffer i & 1.  Iteration i runs phases 2i+1 and 2i+2, which use K(i+1) and V(i), and
        // fetches K(i+2) and V(i+1) behind its barrier.  The same code also fills and drains the
        // pipeline: iteration -1 computes S(0) and the softmax of step 0 (its PV products use a
        // zero P against the K(0) tile, which is there and finite), iteration cnt-1 finishes the
        // last PV products (its QK products read whatever the idle K buffer holds and are
        // never used).
        {
            int n0 = __builtin_amdgcn_readfirstlane(e0_raw);
            if (partial && n0 == m && m > 0) n0 = m - 1;    // see whole_tile below
            st.issue_k(n0, 0);
        }
        wait_vm();
        // The Q^T operand must be complete in its registers here.  Its loads may target the accumulation
        // registers directly, and their first reader would then be an MFMA inside the tile loop: the compiler
        // places its waits for the eight loads there (vmcnt(7) .. vmcnt(0) in front of successive MFMAs), and
        // on every later trip those same waits stall on the tile copies in flight instead -- 6 % of the launch.
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
            for (int kc = 0; kc < 8; ++kc) asm volatile("" : "+a"(w.qf[qt][kc]));
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e) { pa[qt][c][e] = (__bf16)0.f; pb[qt][c][e] = (__bf16)0.f; }
        // The copies being unconditional, the pipeline fetches two entries past its last block.  With a whole
        // diagonal tile selected those fetches are that tile (list entry cnt): its K and V are then in
        // LDS (buffers cnt & 1) when the masked pass below starts.  Otherwise the last tile is fetched again.
        const int last_entry = (has_diag && !partial) ? cnt : cnt - 1;
        auto entry_raw = [&](int it) { return block_raw(it < last_entry ? it : last_entry); };
        // A partial block m is only ever read by the diagonal pass, whose copies stay inside the real length:
        // an entry of a malformed list that names it in the middle of the row is moved to block m - 1.
        // Applied to the scalar copy of an entry, where it is consumed: touching the loaded value any earlier
        // would move the wait for the list load, and with it a stall, into the middle of the iteration.
        auto whole_tile = [&](int n) { return (partial && n == m && m > 0) ? m - 1 : n; };
        int n1 = whole_tile(__builtin_amdgcn_readfirstlane(e0_raw));            // list entries i+1 and i+2
        int n2 = whole_tile(__builtin_amdgcn_readfirstlane(last_entry >= 1 ? e1_raw : e0_raw));
        // One iteration; P = i & 1 is a compile-time constant (the loop is unrolled over it) so that every LDS
        // offset is an immediate.  `fill` marks iteration -1, which only starts the pipeline: it computes S(0),
        // S(1) and the softmax of step 0; its PV products multiply whatever the idle V buffer holds and are
        // thrown away by clearing O^T afterwards.  (The fill must stay an ordinary trip of the one loop: peeled
        // off, the compiler knows O^T to be zero there, builds the accumulator tuples of the asm MFMAs from
        // copies and moves the results right behind each MFMA without the wait states an MFMA result needs.)
        auto iteration = [&](int i, auto parity, bool fill) {
            constexpr int P = decltype(parity)::value;
            constexpr int KO = (P ^ 1) * kTileBytes;                       // K buffer (i + 1) & 1
            constexpr int VO = P * kTileBytes;                             // V buffer i & 1
            __syncthreads();
            // list entry i+3, wanted at the end of this iteration: requested first, so that it is
            // back long before the wait for the tile copies (loads complete in order)
            const int n3_raw = entry_raw(i + 3);
            // phase 2i+1: softmax(2i+1) | PV(2i) QK(2i+2) | fetch K(i+2) and V(i+1)
            phase<true, VO, KO>(w, sb, sa, pa, pb, !fill, st, st.k_src(n2), st.k_dst(P),
                                         st.v_src(n1), st.v_dst(P ^ 1));
            // phase 2i+2: softmax(2i+2) | PV(2i+1) QK(2i+3)
            phase<false, VO + 32 * 256, KO + 32 * 256>(w, sa, sb, pb, pa, i + 1 < cnt, st, nullptr, 0, nullptr, 0);
            if (fill) {
                mfma_settle_acc(w.acc);
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) w.acc[dt][qt][r] = 0.f;
                mfma_settle_acc(w.acc);
            }
            wait_vm();
            n1 = n2;
            n2 = whole_tile(__builtin_amdgcn_readfirstlane(n3_raw));
        };
        using std::integral_constant;
        for (int i = -1; i < cnt; i += 2) {
            iteration(i, integral_constant<int, 1>{}, i < 0);
            if (i + 1 < cnt) iteration(i + 1, integral_constant<int, 0>{}, false);
        }
        mfma_settle_acc(w.acc);
    }

    if (kPersist) draw_issue();                             // (1): the ticket is back when the diagonal pass is done
    if (has_diag) {
        // ---- diagonal block: token-causal mask, no overlap ----
        __syncthreads();                                    // the pipeline is done; its last copies have landed
        int dbuf = 0;
        if (cnt > 0 && !partial) {
            dbuf = cnt & 1;                                 // fetched by the last two iterations of the pipeline
        } else {
            if (partial) {
                st.issue_partial(st.Kp, m, st.k_dst(0), false, tile_rows, lane);
                st.issue_partial(st.Vp, m, st.v_dst(0), true, tile_rows, lane);
            } else {
                st.issue_k(m, 0);
                st.issue_v(m, 0);
            }
            wait_vm();
            __syncthreads();
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int kbase = 64 * ki + 32 * t;             // first key of this wave's step, inside the block
            const int qbase = 32 * NQT * qi;                // first query of this wave
            if (kbase <= qbase + 32 * NQT - 1) {            // else no key of the step precedes any query of the wave
                qk_step(w, dbuf, t, sa);
                if (kbase + 31 > qbase) {
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int kabs = kbase + 8 * (r >> 2) + 4 * gsel + (r & 3);
                            if (kabs > qbase + 32 * qt + l32) sa[qt][r] = NEG_INF;
                        }
                }
                float psum[NQT], mx[NQT];
                exp_all(w, sa, pa, psum, mx);
                finish_softmax(w, sa, pa, psum, mx);
                pv_step(w, dbuf, t, pa);
            }
        }
    }
    if (kPersist) draw_publish();
    __syncthreads();
    if (kPersist) step_rank();                              // (2): the order entry arrives during the merge

    // ---- merge the two key halves of every query, normalise, write ----
    float l_tot[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) l_tot[qt] = w.lsum[qt] + __shfl_xor(w.lsum[qt], 32);

    float* xch = reinterpret_cast<float*>(lds_generic) + qi * (kXchgFloats * 64);
    if (ki == 1) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[((dt * NQT + qt) * 16 + r) * 64 + lane] = w.acc[dt][qt][r];
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            xch[(64 * NQT + qt) * 64 + lane] = w.mref[qt];
            xch[(65 * NQT + qt) * 64 + lane] = l_tot[qt];
        }
    }
    __syncthreads();
    if (ki == 0) {
        unsigned char* ost = lds_generic + kQWaves * kXchgFloats * 64 * 4 + qi * (32 * NQT * kOutRowBytes);
        // row of Q / O of this wave's first query (negative in front of a step that starts inside its first
        // block), and the rows of the wave that exist: rows_lo <= x < rows_q (may be empty in the ragged form)
        const long long wrow0 = (long long)mq * 128 + 32 * NQT * qi - (kRagged ? g.qoff : 0);
        const int rows_q = kRagged ? (int)min((long long)(32 * NQT), (long long)(g.Lr - g.q0) - wrow0) : 32 * NQT;
        const int rows_lo = kRagged ? (int)max(0ll, -wrow0) : 0;
        // a split launch writes its part's result (normalised over the part's own blocks) and lse to the
        // workspace, rows contiguous; the merge kernel weighs the parts by their lse
        const long long rows_call = g.Lr - g.q0;
        float* lse_base = split ? a.part_lse + (long long)part * g.batch * g.Hq * rows_call : a.lse;
        float* lse = lse_base ? lse_base + ((long long)b * g.Hq + h) * rows_call + wrow0 : nullptr;
        if (planned && split) lse = a.part_lse + (long long)plan_slot * 128 + 32 * NQT * qi;   // a slot holds a whole tile
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            const float m1 = xch[(64 * NQT + qt) * 64 + lane], l1 = xch[(65 * NQT + qt) * 64 + lane];
            const float m0 = w.mref[qt], l0 = l_tot[qt];
            const float mm = fmaxf(m0, m1);
            const float a0 = (m0 == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(m0 - mm);
            const float a1 = (m1 == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(m1 - mm);
            const float l = l0 * a0 + l1 * a1;
            const float inv = l > 0.f ? 1.0f / l : 0.f;
            const float w0 = a0 * inv, w1 = a1 * inv;
            if (lse && gsel == 0 && 32 * qt + l32 < rows_q && 32 * qt + l32 >= rows_lo) lse[32 * qt + l32] = l > 0.f ? mm * 0.6931471805599453f + logf(l) : NEG_INF;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r0 = 4 * rg + e;
                        v[e] = w.acc[dt][qt][r0] * w0 + xch[((dt * NQT + qt) * 16 + r0) * 64 + lane] * w1;
                    }
                    if (split) {
                        // a part's result stays fp32 (the merge rounds once, at the end): straight from the
                        // registers, 16 bytes per lane
                        const int q = 32 * qt + l32;
                        if (q < rows_q && q >= rows_lo) {
                            float* dst = planned
                                ? a.part_O + ((long long)plan_slot * 128 + 32 * NQT * qi + q) * g.d + 32 * dt + 8 * rg + 4 * gsel
                                : a.part_O + (((long long)part * g.batch * g.Hq + (long long)b * g.Hq + h) * rows_call +
                                              wrow0 + q) * g.d + 32 * dt + 8 * rg + 4 * gsel;
                            *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                        }
                    } else {
                        u32x2 o = {f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16),
                                   f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16)};
                        *reinterpret_cast<u32x2*>(ost + (32 * qt + l32) * kOutRowBytes + 2 * (32 * dt + 8 * rg + 4 * gsel)) = o;
                    }
                }
        }
        if (kPersist) step_row();                           // (3): the order entry came in during the merge
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        unsigned short* Op = reinterpret_cast<unsigned short*>(a.O) + b * g.qsb + h * g.qsh + wrow0 * g.qsl;
#pragma unroll
        for (int k = 0; k < 8 * NQT; ++k) {
            const int idx = lane + 64 * k, row = idx >> 4, ch = idx & 15;
            const u32x2 lo = *reinterpret_cast<const u32x2*>(ost + row * kOutRowBytes + 16 * ch);
            const u32x2 hi = *reinterpret_cast<const u32x2*>(ost + row * kOutRowBytes + 16 * ch + 8);
            u32x4 o = {lo[0], lo[1], hi[0], hi[1]};
            if (!split && row < rows_q && row >= rows_lo) *reinterpret_cast<u32x4*>(Op + (long long)row * g.qsl + 8 * ch) = o;
        }
        if (kPersist) step_last();                          // (4): count and first entries came in during the stores
    } else if (kPersist) {
        step_row();                                         // the waves that only handed their half over: (3), (4)
        step_last();
    }
   }  // have_row
    if (!kPersist) break;
    // what is left of the look-ahead (all of it after a rank without a row).  The barrier keeps the next row's
    // tile copies behind this row's last reads of the exchange and staging areas.
    if (!have_row) { draw_issue(); draw_publish(); }
    __syncthreads();
    if (!have_row) { step_rank(); step_row(); step_last(); }
    step_done();                                            // (5)
  }
    if (kPersist && draws) {
        // every workgroup has drawn its last (empty) ticket before it counts itself out: the last one out
        // leaves the queue as it found it
        int32_t* const queue = kernel_args<true>()->a.queue;
        const int gone = atomicAdd(queue + kQueueDone, 1);
        if (gone == (int)gridDim.x - 1) {
#pragma unroll
            for (int x = 0; x < 8; ++x) queue[kQueueStride * x] = 0;
            queue[kQueueDone] = 0;
        }
    }
}

}  // namespace

// KV groups launched interleaved: the largest divisor of the number of groups that keeps K and V of the set
// within 32 MB, the L2 capacity of the chip (8 XCDs x 4 MB).  Measured on the 128K-token workload's generator at
// other lengths: 8 groups at 8K tokens (32 MB) +24 %, 4 at 16K +7 %, 2 at 32K +5 %; sets of 64 MB and 128 MB
// lose 2-6 % at 32K-128K (their rows no longer find each other's tiles in L2), so 64K tokens and more keep
// one group at a time.
#ifndef RR_INTERLEAVE_BYTES
#define RR_INTERLEAVE_BYTES (32ll << 20)
#endif
int interleave_groups(const Geom& g) {
    const long long per_group = 2ll * g.L * g.d * 2;               // K and V of one KV head, bf16
    const int NG = g.batch * g.Hkv;
    int gi = 1;
    for (int c = 1; c <= NG && c <= 64; ++c)
        if (NG % c == 0 && c * per_group <= RR_INTERLEAVE_BYTES) gi = c;
    return gi;
}

constexpr int kPersistMaxBlocks = 256;                 // contexts up to 32K tokens

// workgroups of a persistent launch: one per compute unit (a workgroup's tile buffers fill the LDS of one), a
// multiple of 8 so that workgroup i sits on XCD i mod 8
int persistent_workgroups() {
    static std::atomic<int> cached[64];                    // zero-initialised; per device, written once
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        n = n / 8 * 8;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// ---- split launches: merge of the parts ----
// Every part holds softmax attention over its own key blocks, O_p and lse_p = log of its sum of exponentials; over
// all blocks O = sum_p exp(lse_p - lse) O_p with lse = log sum_p exp(lse_p) (Sec. 2.1: the softmax is one sum
// over the selected keys).  One wavefront per query row, a lane two channels of d = 128.
__global__ void __launch_bounds__(256)
k_attn_combine(Geom g, AttnArgs a) {
    const long long rows_call = g.Lr - g.q0;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long nrows = (long long)g.batch * g.Hq * rows_call;
    if (row >= nrows) return;
    const int lane = threadIdx.x & 63;
    const long long bh = row / rows_call, r = row - bh * rows_call;
    const int b = (int)(bh / g.Hq), h = (int)(bh - (long long)b * g.Hq);
    const float NEG_INF = -__builtin_huge_valf();
    float mx = NEG_INF;
    for (int p = 0; p < a.nsplit; ++p) mx = fmaxf(mx, a.part_lse[(long long)p * nrows + row]);
    float den = 0.f, o0 = 0.f, o1 = 0.f;
    if (mx != NEG_INF) {
        for (int p = 0; p < a.nsplit; ++p) {
            const float l = a.part_lse[(long long)p * nrows + row];
            if (l == NEG_INF) continue;                       // a part without a block
            const float wgt = expf(l - mx);
            const float2 v = *reinterpret_cast<const float2*>(a.part_O + ((long long)p * nrows + row) * g.d + 2 * lane);
            den += wgt;
            o0 = fmaf(wgt, v.x, o0);
            o1 = fmaf(wgt, v.y, o1);
        }
    }
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    unsigned short* O = reinterpret_cast<unsigned short*>(a.O) + b * g.qsb + h * g.qsh + r * g.qsl;
    *reinterpret_cast<unsigned*>(O + 2 * lane) = f32_to_bf16_bits(o0 * inv) | (f32_to_bf16_bits(o1 * inv) << 16);
    if (a.lse && lane == 0) a.lse[row] = den > 0.f ? mx + logf(den) : NEG_INF;
}

// ---- planned launches (chunks of a long prompt): the plan and the merge ----
// One workgroup walks the rows in launch order, gives every row longer than split_len entries one slot per part
// (a prefix sum, so the longest rows, which start first, are served first when the slots run out) and lists the
// slots' rows.
constexpr int kPlanThreads = 1024;
__global__ void __launch_bounds__(kPlanThreads)
k_split_plan(Geom g, AttnArgs a, int grid_rows) {
    __shared__ int s_scan[kPlanThreads];
    __shared__ int s_base, s_used, s_cut;
    const int t = threadIdx.x;
    const int Nbq = g.Lq >> 7;
    const int rows_total = g.batch * g.Hq * Nbq;
    for (int i = t; i < rows_total; i += kPlanThreads) a.plan_row[i] = -1;
    if (t == 0) { s_base = 0; s_used = 0; s_cut = 0; }
    __syncthreads();
    for (int start = 0; start < grid_rows; start += kPlanThreads) {
        const int rank = start + t;
        int parts = 0, rid = -1;
        if (rank < grid_rows) {
            int b, h, mq;
            if (decode_block(rank, g, Nbq, a.row_order, a.interleave, b, h, mq)) {
                const int m = mq + (a.Nb - Nbq);
                rid = (b * g.Hq + h) * Nbq + mq;
                int count = a.row_list ? a.row_count[rid] : m + 1;
                count = count < 0 ? 0 : (count > m + 1 ? m + 1 : count);      // as the attention kernel holds it
                if (count > a.split_len) parts = (count + a.split_len - 1) / a.split_len;
            }
        }
        // the parts (at most 4096 rows x 32 < 2^18), and above them the number of rows with parts (at most 2^12)
        s_scan[t] = parts | (parts > 0 ? 1 << 18 : 0);
        __syncthreads();
        for (int off = 1; off < kPlanThreads; off <<= 1) {
            const int v = t >= off ? s_scan[t - off] : 0;
            __syncthreads();
            s_scan[t] += v;
            __syncthreads();
        }
        const int incl = s_base + s_scan[t];
        const int first = (incl & 0x3FFFF) - parts, nth = (incl >> 18) - 1;      // slots and cut rows in front of this row
        if (parts > 0 && first + parts <= a.split_budget) {
            a.plan_row[rid] = first;
            for (int p = 0; p < parts; ++p) a.plan_items[first + p] = rid;
            a.plan_cut[nth] = rid;                             // the cut rows, in launch order (all in front fit as well)
            atomicMax(&s_used, first + parts);
            atomicMax(&s_cut, nth + 1);
        }
        __syncthreads();
        if (t == 0) s_base += s_scan[kPlanThreads - 1];
        __syncthreads();
    }
    if (t == 0) { a.plan_total[0] = s_used; a.plan_total[1] = s_cut; }
}

// The cut rows: O = sum_p exp(lse_p - lse) O_p over the row's parts, rounded once.  A wavefront per query row
// (blockIdx.x: which cut row, blockIdx.y picks four of its tile's 128), a lane two channels; the parts' lse values are read by one lane each, so
// that nothing in the merge is a chain of dependent loads.  At most 64 parts per row.
__global__ void __launch_bounds__(256)
k_attn_combine_plan(Geom g, AttnArgs a) {
    const int Nbq = g.Lq >> 7;
    if ((int)blockIdx.x >= a.plan_total[1]) return;                      // blockIdx.x: which of the cut rows
    const int rid = a.plan_cut[blockIdx.x];
    if ((unsigned)rid >= (unsigned)(g.batch * g.Hq * Nbq)) return;
    const int base = a.plan_row[rid];
    if (base < 0) return;
    const int mq = rid % Nbq, bh = rid / Nbq, h = bh % g.Hq, b = bh / g.Hq;
    const int m = mq + (a.Nb - Nbq);
    int count = a.row_list ? a.row_count[rid] : m + 1;
    count = count < 0 ? 0 : (count > m + 1 ? m + 1 : count);
    int parts = (count + a.split_len - 1) / a.split_len;
    parts = parts > 64 ? 64 : parts;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const long long rows_call = g.Lr - g.q0;
    const float NEG_INF = -__builtin_huge_valf();
    const int x = 4 * (int)blockIdx.y + wv;                              // query row of the tile
    const long long r = (long long)mq * 128 + x - g.qoff;               // row of Q / O
    if (r < 0 || r >= rows_call) return;
    const float l = lane < parts ? a.part_lse[(long long)(base + lane) * 128 + x] : NEG_INF;
    float mx = l;
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mx = fmaxf(mx, __shfl_xor(mx, sft));
    const float wgt = (lane < parts && l != NEG_INF) ? expf(l - mx) : 0.f;
    float den = wgt;
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) den += __shfl_xor(den, sft);
    float o0 = 0.f, o1 = 0.f;
    const float* src = a.part_O + ((long long)base * 128 + x) * g.d + 2 * lane;
#pragma unroll 4
    for (int p = 0; p < parts; ++p) {
        const float wp = __shfl(wgt, p);
        const float2 v = *reinterpret_cast<const float2*>(src + (long long)p * 128 * g.d);
        o0 = fmaf(wp, v.x, o0);
        o1 = fmaf(wp, v.y, o1);
    }
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    unsigned short* O = reinterpret_cast<unsigned short*>(a.O) + b * g.qsb + h * g.qsh + r * g.qsl;
    *reinterpret_cast<unsigned*>(O + 2 * lane) = f32_to_bf16_bits(o0 * inv) | (f32_to_bf16_bits(o1 * inv) << 16);
    if (a.lse && lane == 0) a.lse[((long long)b * g.Hq + h) * rows_call + r] = den > 0.f ? mx + logf(den) : NEG_INF;
}

int attn_mfma_plan_len(const Geom& g, int B, int* budget) {
    // A chunk of a long prompt: many rows, most of them short, a few nearly as long as the context, and the launch
    // takes as long as its longest row (measured at 128K, tau 0.9: 1.1 ms for chunks of 512 to 2048 tokens whose
    // blocks are 0.15-0.19 ms of matrix work).  Parts of 64 list entries, 128 where the launch has more than 2048 rows
    // (measured: 32 / 64 / 128 entries are level up to 4096 tokens, 64 is best at 8192, 128 at 16384; what remains
    // above the matrix work is memory traffic: the rows of such a launch share few tiles in L2).
    if (budget) *budget = 0;
    if (B != 128 || g.d != 128) return 0;
    const int Nb = g.L / B, Nbq = g.Lq / B;
    const long long rows = (long long)g.batch * g.Hq * Nbq;
    if (Nbq < 2 || Nb < 128 || g.q0 <= 0 || rows > 4096) return 0;
    int len = rows <= 2048 ? 64 : 128;
    if (len < (Nb + 31) / 32) len = (Nb + 31) / 32;                     // at most 32 parts per row
    if (Nb <= len) return 0;
    // slots: several times what the rows of such chunks were seen to need (300-1000 at 128K), between 512 and 2048
    // (34-135 MB of partial results); the workgroups of unused slots run last and cost nothing measurable
    if (budget) *budget = (int)(4 * rows < 512 ? 512 : (4 * rows > 2048 ? 2048 : 4 * rows));
    return len;
}
namespace {
size_t plan_align(size_t x) { return (x + 255) / 256 * 256; }
}
size_t attn_mfma_plan_bytes(const Geom& g, int B) {
    int budget = 0;
    if (attn_mfma_plan_len(g, B, &budget) <= 0) return 0;
    const size_t rows = (size_t)g.batch * g.Hq * (size_t)(g.Lq / B);
    return 256 + plan_align(rows * 4) + plan_align((size_t)budget * 4) + plan_align((size_t)budget / 2 * 4) +
           plan_align((size_t)budget * 128 * 4) + (size_t)budget * 128 * g.d * 4;
}
void attn_mfma_plan_pointers(const Geom& g, int B, void* workspace, AttnArgs* a) {
    int budget = 0;
    a->split_len = attn_mfma_plan_len(g, B, &budget);
    a->split_budget = budget;
    const size_t rows = (size_t)g.batch * g.Hq * (size_t)(g.Lq / B);
    unsigned char* p = static_cast<unsigned char*>(workspace);
    a->plan_total = reinterpret_cast<int32_t*>(p);
    p += 256;
    a->plan_row = reinterpret_cast<int32_t*>(p);
    p += plan_align(rows * 4);
    a->plan_items = reinterpret_cast<int32_t*>(p);
    p += plan_align((size_t)budget * 4);
    a->plan_cut = reinterpret_cast<int32_t*>(p);                    // a cut row has two parts or more
    p += plan_align((size_t)budget / 2 * 4);
    a->part_lse = reinterpret_cast<float*>(p);
    p += plan_align((size_t)budget * 128 * 4);
    a->part_O = reinterpret_cast<float*>(p);
    a->nsplit = 1;
}

int attn_mfma_splits(const Geom& g, int B) {
    // few rows, all of them deep inside the context (a step, not a prefill: even the first row has 16 causal
    // blocks or more): bring the launch to about two workgroups per compute unit (measured at a 128K context:
    // 512 workgroups 0.32 ms for a dense one-token step, 1024 workgroups 0.42 ms), every part at least 8 blocks
    // long
    const int Nb = g.L / B, Nbq = g.Lq / B;
    const long long rows = (long long)g.batch * g.Hq * Nbq;
    if (rows >= 512 || Nb - Nbq + 1 < 16) return 1;
    long long P = (512 + rows - 1) / rows;
    if (P > Nb / 8) P = Nb / 8;
    if (P > 32) P = 32;
    return P < 1 ? 1 : (int)P;
}
size_t attn_mfma_split_bytes(const Geom& g, int B) {
    const int P = attn_mfma_splits(g, B);
    if (P <= 1) return 0;
    const size_t rows = (size_t)g.batch * g.Hq * (size_t)(g.Lr - g.q0);
    return (size_t)P * rows * g.d * sizeof(float) + (size_t)P * rows * sizeof(float);
}
hipError_t launch_attn_combine(const Geom& g, const AttnArgs& a, hipStream_t st) {
    const long long nrows = (long long)g.batch * g.Hq * (g.Lr - g.q0);
    hipLaunchKernelGGL(k_attn_combine, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, st, g, a);
    return hipGetLastError();
}

hipError_t launch_attn_mfma_bf16(const Geom& g, const AttnArgs& a_in, hipStream_t st) {
    AttnArgs a = a_in;
    a.interleave = interleave_groups(g);
    if (a.nsplit < 1 || !a.part_O || !a.part_lse) a.nsplit = 1;
    const bool planned = a.split_len > 0 && a.split_budget > 0 && a.plan_total && a.plan_row && a.plan_items && a.plan_cut &&
                         a.part_O && a.part_lse;
    if (!planned) { a.split_len = 0; a.split_budget = 0; } else a.nsplit = 1;
    const bool ragged = g.Lr != g.L || g.qoff != 0 || a.nsplit > 1 || planned;   // split launches use the ragged instantiation
    const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)g.d));
    const long long rows = (long long)g.batch * g.Hq * (g.Lq / 128);
    const int cus = persistent_workgroups();
    // Persistent workgroups pay where rows are short, i.e. where the start of a row is a visible share of it:
    // measured on the 128K workload's generator at other lengths, +15 % at 8K tokens, +9 % at 16K, +2 % at 32K,
    // level or slightly behind from 64K on (there the launch is limited by power, not by the gaps between rows).
    const bool persist = a.row_order != nullptr && a.queue != nullptr && cus >= 8 && a.Nb <= kPersistMaxBlocks &&
                         a.nsplit == 1 && !planned;
    const unsigned grid_rows = grid_size(g, g.Lq / 128, a.row_order != nullptr);
    dim3 grid(grid_rows * (unsigned)a.nsplit + (planned ? (unsigned)a.split_budget : 0u));
    if (planned) {
        hipLaunchKernelGGL(k_split_plan, dim3(1), dim3(kPlanThreads), 0, st, g, a, (int)grid_rows);
        const hipError_t pe = hipGetLastError();
        if (pe != hipSuccess) return pe;
    }
    if (persist) grid = dim3((unsigned)(rows < cus ? (rows + 7) / 8 * 8 : cus));
    const int lds_bytes = kLdsBytes + (persist ? 16 : 0);
    auto launch = [&](auto kernel) -> hipError_t {
        hipError_t e = allow_dynamic_lds((const void*)kernel, lds_bytes);
        if (e != hipSuccess) return e;
        AttnKernelArgs ka;
        ka.g = g;
        ka.a = a;
        ka.scale_log2 = scale_log2;
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds_bytes, st, ka);
        return hipGetLastError();
    };
    if (persist) return ragged ? launch(k_attn_mfma_bf16<true, true>) : launch(k_attn_mfma_bf16<false, true>);
    const hipError_t e = ragged ? launch(k_attn_mfma_bf16<true, false>) : launch(k_attn_mfma_bf16<false, false>);
    if (e != hipSuccess) return e;
    if (planned) {
        const long long rows_total = (long long)g.batch * g.Hq * (g.Lq / 128);
        const long long cut_max = rows_total < a.split_budget / 2 ? rows_total : a.split_budget / 2;
        hipLaunchKernelGGL(k_attn_combine_plan, dim3((unsigned)cut_max, 32), dim3(256), 0, st, g, a);
        return hipGetLastError();
    }
    if (a.nsplit == 1) return e;
    return launch_attn_combine(g, a, st);
}

}  // namespace rr
