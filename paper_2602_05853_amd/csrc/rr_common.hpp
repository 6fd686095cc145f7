// Shared declarations of the RRAttention HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "rr_attn.h"

namespace rr {

// Geometry handed to every kernel: strides in elements, head dimension contiguous.
struct Geom {
    int batch, L, Hq, Hkv, d, G;
    int Lq, q0;                 // queries are the last positions of the context: row r of Q is token q0 + r
    // A step may start inside a block (decode steps, unaligned chunks): its first query block then begins
    // qoff positions before q0.  After pad_to_blocks Lq counts from that block's first position, so that
    // Lq / B is the number of query-block rows; the positions in front of q0 have no row in Q or O (loads are
    // clamped to row 0, stores predicated).
    int qoff;
    // The kernels walk whole blocks: once the block size is known the entry points round L and Lq up to
    // multiples of it (pad_to_blocks) and keep the real number of positions here.  Positions >= Lr exist in no
    // tensor: their rows are never stored, and a load that would touch one reads row Lr - 1 instead.
    int Lr;
    long long qsb, qsh, qsl;
    long long ksb, ksh, ksl;
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

// ---- element access in fp32, whatever the storage type --------------------------------
struct bf16_t { unsigned short bits; };

__device__ __forceinline__ float bf16_bits_to_f32(unsigned int bits16) {
    return __uint_as_float(bits16 << 16);
}
// round-to-nearest-even fp32 -> bf16 bit pattern (inputs here are finite)
__device__ __forceinline__ unsigned int f32_to_bf16_bits(float x) {
    unsigned int u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kVec = 4;   // elements per 16-byte load
    __device__ static __forceinline__ void load16(const float* p, float* out) {
        f32x4 v = *reinterpret_cast<const f32x4*>(p);
        out[0] = v[0]; out[1] = v[1]; out[2] = v[2]; out[3] = v[3];
    }
    __device__ static __forceinline__ float load1(const float* p) { return *p; }
    __device__ static __forceinline__ void store1(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int kVec = 8;
    __device__ static __forceinline__ void load16(const bf16_t* p, float* out) {
        u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(v[i] << 16);
            out[2 * i + 1] = __uint_as_float(v[i] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ float load1(const bf16_t* p) { return bf16_bits_to_f32(p->bits); }
    __device__ static __forceinline__ void store1(bf16_t* p, float v) {
        p->bits = (unsigned short)f32_to_bf16_bits(v);
    }
};

// ---- wavefront (64 lanes) reductions ---------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---- launchers (one per kernel group), defined in their own .hip files -------------------
// (1) stride sums of K: Ksum[b][g][j][c] = sum_{s<S} K[b][g][j*S+s][c], fp32, contiguous.
hipError_t launch_stride_sum(const Geom& g, int dtype, const void* K, int S, float* Ksum, hipStream_t st);

// (2) fused stride scores -> causal softmax state -> block mass -> Top-tau -> mask/list.
struct EstimateArgs {
    const void* Q;
    const void* K;            // the keys themselves: read only with diag_token
    const float* Ksum;        // [batch][Hkv][Ls][d]
    float2* state_ws;         // global softmax state when it does not fit in LDS, else nullptr
    int S, B, R, Nb;
    float tau;
    int protect_last;
    int diag_token;           // 1: in a sampled query's own stride only keys up to the query's position are summed
    int off_hmul, off_add;    // sampled offset = S - 1 - ((off_hmul * h + off_add) mod S)
    int sink_blocks, recent_blocks;
    const int32_t* seq_first; // packed sequences: [Nb] first block of the sequence of block m; nullptr = one sequence
    uint8_t* dense;
    int32_t* row_count;
    int32_t* row_list;
    float* block_mass;
};
size_t estimate_generic_state_bytes(const Geom& g, int S, int B);   // 0 when LDS suffices
bool estimate_generic_fits(const Geom& g, int S, int B);   // LDS plan within the CU's 160 KB
bool attn_generic_fits(int B, int d);
hipError_t launch_estimate_generic(const Geom& g, int dtype, const EstimateArgs& a, hipStream_t st);

// (2') MFMA form for bf16, d = 128, B/S in {4,8,16,32}: split stride sums, then scores -> stride softmax ->
// block mass [batch*Hq*Nbq][Nb] in two sweeps; launch_select_rows then does Top-tau on those rows
// (only a's selection parameters and output arrays are read).
bool estimate_mfma_supported(const Geom& g, int dtype, int S, int B);
size_t estimate_mfma_ksplit_bytes(const Geom& g, int S);
size_t estimate_mfma_mass_bytes(const Geom& g, int B);
size_t estimate_mfma_stats_bytes(const Geom& g, int S, int B);   // per-chunk softmax states of the key split; 0 without one
hipError_t launch_stride_mass_mfma(const Geom& g, const void* Q, const void* K, int S, int B, int off_hmul,
                                   int off_add, int diag_token, const int32_t* seq_first, unsigned short* ksplit,
                                   int ls_cap, int ls_valid, float* mass, float2* stats, hipStream_t st);
// (ksplit holds rows of ls_cap >= L / S strides per (batch, KV head); the first ls_valid strides are kept as they are)
hipError_t launch_select_rows(const Geom& g, const EstimateArgs& a, const float* mass, hipStream_t st);

// (2'') rows of every KV head sorted by descending row_count: order[b][kv][rank] = hl * Nb + m.  A queue
// (rr_mask.queue, RR_QUEUE_WORDS words) given with it is zeroed.
hipError_t launch_row_order(const Geom& g, int Nb, const int32_t* row_count, int32_t* row_order, int32_t* queue,
                            hipStream_t st);

// (4) diagnostic: precision / recall / F1 of a mask against full attention.
size_t accuracy_rows_bytes(const Geom& g, int step);
size_t accuracy_per_query_bytes(const Geom& g, int step);
hipError_t launch_selection_accuracy(const Geom& g, int dtype, const void* Q, const void* K,
                                     const int32_t* row_count, const int32_t* row_list, int B, float tau, int step,
                                     float* rows, float2* per_query, float* out, hipStream_t st);

// caller-made masks: dense 0/1 matrix -> row_count / row_list
hipError_t launch_mask_from_dense(const Geom& g, int Nb, const uint8_t* dense, int32_t* row_count, int32_t* row_list,
                                  hipStream_t st);

// (3) attention over per-row block lists (row_list == nullptr: every block n <= m).
struct AttnArgs {
    const void* Q; const void* K; const void* V; void* O; float* lse;
    const int32_t* row_count; const int32_t* row_list;
    int B, Nb;
    const int32_t* seq_first;   // dense walk of packed sequences: row m takes blocks seq_first[m] .. m; nullptr = 0 .. m
    const int32_t* row_order;   // optional launch order of the rows per KV head (MFMA kernel only)
    int interleave;             // MFMA kernel: KV groups whose rows are launched interleaved (a divisor of batch * Hkv)
    int32_t* queue;             // MFMA kernel, with row_order: row counters of the persistent form (rr_mask.queue), or nullptr
    // MFMA kernel, launches of few rows (steps): the block list of a row is shared out among nsplit workgroups;
    // part p writes its own attention output and lse to part_O / part_lse ([nsplit][batch][Hq][rows][d] and
    // [nsplit][batch][Hq][rows], fp32, rows = the query positions of the call) and a second kernel merges them
    int nsplit;
    float* part_O; float* part_lse;
    // MFMA kernel, chunks of a long prompt (many rows, a few of them very long): rows longer than split_len list
    // entries are cut into parts of split_len entries.  A plan made on the device before the launch gives every such
    // row a run of slots (one per part) in part_O / part_lse, here laid out [slot][128 query rows][d] and
    // [slot][128]: plan_row[row] = first slot or -1 (the row is computed whole and stored directly), plan_items[slot]
    // = row, plan_cut[k] = the k-th cut row, plan_total[0] = slots in use (at most split_budget; rows that no longer
    // fit stay whole), plan_total[1] = cut rows.  The launch has one workgroup per slot and one per row.
    // split_len = 0: off.
    int split_len, split_budget;
    int32_t* plan_total; int32_t* plan_row; int32_t* plan_items; int32_t* plan_cut;
};
// split of a launch with few rows, and the bytes its partial results need; 1 / 0 when the launch is not split
int attn_mfma_splits(const Geom& g, int B);
size_t attn_mfma_split_bytes(const Geom& g, int B);
// chunks of a long prompt: length of a row part (0: the launch is not planned), slots of the plan, bytes of plan and
// partial results, and the pointers into a workspace of that size
int attn_mfma_plan_len(const Geom& g, int B, int* budget);
size_t attn_mfma_plan_bytes(const Geom& g, int B);
void attn_mfma_plan_pointers(const Geom& g, int B, void* workspace, AttnArgs* a);
hipError_t launch_attn_combine(const Geom& g, const AttnArgs& a, hipStream_t st);
// Decode-sized steps (one or two positions, at most 8 rows per KV head; bf16, d = 128, B = 128): parts of the
// launch (0: not such a step), bytes of its partial results, and the launch itself (a.nsplit parts, a.part_O /
// a.part_lse laid out as above), which also merges the parts into a.O / a.lse.
int attn_decode_parts(const Geom& g, int B);
size_t attn_decode_bytes(const Geom& g, int B);
hipError_t launch_attn_decode(const Geom& g, const AttnArgs& a, hipStream_t st);
constexpr int kMaxOrderedRows = 32768;   // G * Nb up to which a row order is produced and used
hipError_t launch_attn_generic(const Geom& g, int dtype, const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_mfma_bf16(const Geom& g, const AttnArgs& a, hipStream_t st);

// Raises a kernel's dynamic-LDS limit on the current device to at least `bytes`.  The limit is per (kernel,
// device) and only ever grows, so the runtime is asked once per pair and size, not on every launch.
hipError_t allow_dynamic_lds(const void* kernel, size_t bytes);

}  // namespace rr
