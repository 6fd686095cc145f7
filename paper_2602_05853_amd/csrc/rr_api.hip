// C ABI of the library (see include/rr_attn.h): argument checks on the host, then launches.
#include "rr_common.hpp"

#include <mutex>

namespace rr {
bool attn_generic_fits(int B, int d);
}

// Scratch of rr_estimate_static.  In host code this name is only a handle for hipGetSymbolAddress: the
// array's device address differs per GPU and is looked up once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[RR_STATIC_SCRATCH_BYTES];

namespace rr {

hipError_t allow_dynamic_lds(const void* kernel, size_t bytes) {
    struct Granted { const void* kernel; int device; size_t bytes; };
    static std::mutex mu;
    static Granted table[256];
    static int used = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    Granted* slot = nullptr;
    for (int i = 0; i < used; ++i)
        if (table[i].kernel == kernel && table[i].device == dev) { slot = &table[i]; break; }
    if (slot && slot->bytes >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    if (!slot && used < 256) slot = &table[used++];      // a full table only costs the repeated call
    if (slot) *slot = Granted{kernel, dev, bytes};
    return hipSuccess;
}

}  // namespace rr

namespace {

using namespace rr;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_shape(const rr_shape* s, Geom* g) {
    if (!s) return RR_ERR_NULL;
    if (s->dtype != RR_BF16 && s->dtype != RR_F32) return RR_ERR_DTYPE;
    if (s->batch < 1 || s->L < 1 || s->Hq < 1 || s->Hkv < 1 || s->d < 8) return RR_ERR_SHAPE;
    if (s->Hq % s->Hkv) return RR_ERR_SHAPE;
    if (s->d % 8 || s->d > 256) return RR_ERR_SHAPE;
    const int64_t row = s->dtype == RR_BF16 ? 8 : 4;          // elements per 16 bytes
    const int64_t st[6] = {s->q_stride_b, s->q_stride_h, s->q_stride_l,
                           s->kv_stride_b, s->kv_stride_h, s->kv_stride_l};
    for (int i = 0; i < 6; ++i)
        if (st[i] < 0 || st[i] % row) return RR_ERR_SHAPE;
    if (s->q_stride_l < s->d || s->kv_stride_l < s->d) return RR_ERR_SHAPE;
    g->batch = s->batch; g->L = s->L; g->Hq = s->Hq; g->Hkv = s->Hkv; g->d = s->d;
    g->G = s->Hq / s->Hkv;
    if (s->Lq < 0 || s->Lq > s->L) return RR_ERR_SHAPE;
    g->Lq = s->Lq ? s->Lq : s->L;
    g->q0 = g->L - g->Lq;
    g->qoff = 0;
    g->Lr = g->L;
    g->qsb = s->q_stride_b; g->qsh = s->q_stride_h; g->qsl = s->q_stride_l;
    g->ksb = s->kv_stride_b; g->ksh = s->kv_stride_h; g->ksl = s->kv_stride_l;
    return RR_OK;
}

// L rounded up, and the start of the query rows rounded down, to whole blocks of B
int pad_to_blocks(Geom* g, int B) {
    if (B < 1) return RR_ERR_SHAPE;
    const long long Lp = ((long long)g->Lr + B - 1) / B * B;
    if (Lp > 0x7fffffffLL) return RR_ERR_SHAPE;
    g->L = (int)Lp;
    g->qoff = g->q0 % B;
    g->Lq = g->L - (g->q0 - g->qoff);
    return RR_OK;
}

// expects pad_to_blocks(g, B)
int check_blocks(const Geom& g, int S, int B) {
    if (S < 1 || B < 1 || B % S || g.L % B || g.Lq % B) return RR_ERR_SHAPE;
    if (B / S > 128 || B > 128) return RR_ERR_SHAPE;
    if (g.L / B > 8192) return RR_ERR_SHAPE;
    return RR_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool use_mfma_attn(const Geom& g, int dtype, int B) { return dtype == RR_BF16 && g.d == 128 && B == 128; }

size_t ksum_bytes(const Geom& g, int S) {
    return align_up((size_t)g.batch * g.Hkv * (g.L / S) * g.d * sizeof(float), 256);
}

int run_attn(const rr_shape* shape, const void* Q, const void* K, const void* V, int B,
             const int32_t* row_count, const int32_t* row_list, const int32_t* row_order, int32_t* queue,
             const int32_t* seq_first, void* O, float* lse, void* stream, void* workspace = nullptr,
             size_t workspace_bytes = 0) {
    Geom g;
    int rc = check_shape(shape, &g);
    if (rc != RR_OK) return rc;
    if (!Q || !K || !V || !O) return RR_ERR_NULL;
    if (B < 1 || B > 128 || pad_to_blocks(&g, B) != RR_OK) return RR_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return RR_ERR_SHAPE;
    AttnArgs a;
    a.Q = Q; a.K = K; a.V = V; a.O = O; a.lse = lse;
    a.row_count = row_count; a.row_list = row_list;
    a.B = B; a.Nb = g.L / B;
    if (seq_first && g.q0 != 0) return RR_ERR_PARAM;          // packed sequences and a query chunk do not combine
    a.seq_first = seq_first;
    a.row_order = (row_list && (long long)g.G * (g.Lq / B) <= kMaxOrderedRows) ? row_order : nullptr;
    a.queue = a.row_order ? queue : nullptr;
    a.interleave = 1;
    a.nsplit = 1;
    a.part_O = nullptr;
    a.part_lse = nullptr;
    a.split_len = 0;
    a.split_budget = 0;
    a.plan_total = nullptr;
    a.plan_row = nullptr;
    a.plan_items = nullptr;
    a.plan_cut = nullptr;
    bool decode = false;
    if (workspace && use_mfma_attn(g, shape->dtype, B) && !seq_first && attn_decode_parts(g, B) >= 1) {
        // one or two new positions: the kernel that reads K and V once per KV head for all its query heads
        const size_t need = attn_decode_bytes(g, B);
        if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RR_ERR_WORKSPACE;
        a.nsplit = attn_decode_parts(g, B);
        const size_t rows = (size_t)g.batch * g.Hq * (size_t)(g.Lr - g.q0);
        a.part_O = reinterpret_cast<float*>(workspace);
        a.part_lse = a.part_O + (size_t)a.nsplit * rows * g.d;
        decode = true;
    } else if (workspace && use_mfma_attn(g, shape->dtype, B) && !seq_first && attn_mfma_plan_len(g, B, nullptr) > 0) {
        // a chunk of a long prompt: the few very long rows are cut into parts after a plan made on the device
        const size_t need = attn_mfma_plan_bytes(g, B);
        if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RR_ERR_WORKSPACE;
        attn_mfma_plan_pointers(g, B, workspace, &a);
    } else if (workspace && use_mfma_attn(g, shape->dtype, B) && !seq_first) {
        // a launch of few rows with a workspace: the block list of every row is shared out among several workgroups
        const size_t need = attn_mfma_split_bytes(g, B);
        if (need) {
            if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RR_ERR_WORKSPACE;
            a.nsplit = attn_mfma_splits(g, B);
            const size_t rows = (size_t)g.batch * g.Hq * (size_t)(g.Lr - g.q0);
            a.part_O = reinterpret_cast<float*>(workspace);
            a.part_lse = a.part_O + (size_t)a.nsplit * rows * g.d;
        }
    }
    hipError_t e;
    if (decode) {
        e = launch_attn_decode(g, a, (hipStream_t)stream);
    } else if (use_mfma_attn(g, shape->dtype, B)) {
        e = launch_attn_mfma_bf16(g, a, (hipStream_t)stream);
    } else {
        if (!attn_generic_fits(B, g.d)) return RR_ERR_SHAPE;
        e = launch_attn_generic(g, shape->dtype, a, (hipStream_t)stream);
    }
    return e == hipSuccess ? RR_OK : RR_ERR_LAUNCH;
}

// Device address of `scratch` on the current device; looked up on the first call per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RR_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RR_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RR_OK;
}

}  // namespace

#define RR_API __attribute__((visibility("default")))

extern "C" {

RR_API int rr_version(void) { return 500; }

RR_API const char* rr_status_string(int status) {
    switch (status) {
        case RR_OK: return "ok";
        case RR_ERR_NULL: return "a required pointer is NULL";
        case RR_ERR_SHAPE: return "unsupported or inconsistent shape";
        case RR_ERR_DTYPE: return "unsupported dtype";
        case RR_ERR_PARAM: return "parameter out of range";
        case RR_ERR_WORKSPACE: return "workspace missing or too small";
        case RR_ERR_LAUNCH: return "HIP launch failed";
        case RR_ERR_SCRATCH_LIMIT: return "geometry needs more scratch than RR_STATIC_SCRATCH_BYTES";
        default: return "unknown status";
    }
}

RR_API size_t rr_workspace_bytes(const rr_shape* shape, int S, int B) {
    Geom g;
    if (check_shape(shape, &g) != RR_OK || pad_to_blocks(&g, B) != RR_OK || check_blocks(g, S, B) != RR_OK) return 0;
    if (estimate_mfma_supported(g, shape->dtype, S, B))
        return align_up(estimate_mfma_ksplit_bytes(g, S), 256) + align_up(estimate_mfma_mass_bytes(g, B), 256) +
               align_up(estimate_mfma_stats_bytes(g, S, B), 256);
    return ksum_bytes(g, S) + align_up(estimate_generic_state_bytes(g, S, B), 256);
}

RR_API int rr_estimate(const rr_shape* shape, const void* Q, const void* K, int S, int B, float tau,
                uint32_t flags, void* workspace, size_t workspace_bytes, rr_mask* out,
                void* hip_stream) {
    const rr_estimate_opts opts = {flags, RR_OFFSET_HEAD, 0, 0, 0, nullptr, 0, 0};
    return rr_estimate_ex(shape, Q, K, S, B, tau, &opts, workspace, workspace_bytes, out, hip_stream);
}

RR_API int rr_estimate_static(const rr_shape* shape, const void* Q, const void* K, int S, int B, float tau,
                       uint32_t flags, rr_mask* out, void* hip_stream) {
    const size_t need = rr_workspace_bytes(shape, S, B);
    // need == 0 is an invalid geometry: rr_estimate below names the reason without touching the scratch
    if (need > RR_STATIC_SCRATCH_BYTES) return RR_ERR_SCRATCH_LIMIT;
    void* ptr = nullptr;
    if (need) {
        const int rc = static_scratch(&ptr);
        if (rc != RR_OK) return rc;
    }
    return rr_estimate(shape, Q, K, S, B, tau, flags, ptr, need ? (size_t)RR_STATIC_SCRATCH_BYTES : 0, out, hip_stream);
}

RR_API int rr_estimate_ex(const rr_shape* shape, const void* Q, const void* K, int S, int B, float tau,
                   const rr_estimate_opts* opts, void* workspace, size_t workspace_bytes, rr_mask* out,
                   void* hip_stream) {
    if (!opts) return RR_ERR_NULL;
    const uint32_t flags = opts->flags;
    if (opts->offset_mode < RR_OFFSET_HEAD || opts->offset_mode > RR_OFFSET_HYBRID) return RR_ERR_PARAM;
    if (opts->layer < 0 || opts->layer > (1 << 20) || opts->sink_blocks < 0 || opts->recent_blocks < 0) return RR_ERR_PARAM;
    const int off_hmul = (opts->offset_mode == RR_OFFSET_HEAD || opts->offset_mode == RR_OFFSET_HYBRID) ? 1 : 0;
    const int off_add = (opts->offset_mode == RR_OFFSET_LAYER || opts->offset_mode == RR_OFFSET_HYBRID) ? opts->layer : 0;
    Geom g;
    int rc = check_shape(shape, &g);
    if (rc != RR_OK) return rc;
    if (!Q || !K || !out || !out->row_count || !out->row_list) return RR_ERR_NULL;
    rc = pad_to_blocks(&g, B);
    if (rc != RR_OK) return rc;
    rc = check_blocks(g, S, B);
    if (rc != RR_OK) return rc;
    if (!(tau > 0.f) || tau > 1.f) return RR_ERR_PARAM;
    if (flags & ~(RR_FLAG_PROTECT_LAST | RR_FLAG_DIAGONAL_TOKEN)) return RR_ERR_PARAM;
    const int diag_token = (flags & RR_FLAG_DIAGONAL_TOKEN) ? 1 : 0;
    if (out->Nb != g.L / B || out->B != B) return RR_ERR_PARAM;
    if (opts->seq_first && g.q0 != 0) return RR_ERR_PARAM;    // packed sequences and a query chunk do not combine
    if (!aligned16(Q) || !aligned16(K)) return RR_ERR_SHAPE;
    const bool mfma = estimate_mfma_supported(g, shape->dtype, S, B);
    if (!mfma && !estimate_generic_fits(g, S, B)) return RR_ERR_SHAPE;
    size_t need = rr_workspace_bytes(shape, S, B);
    // stride sums kept from call to call: laid out for ksum_capacity positions, at the front of the workspace
    int ls_cap = g.L / S, ls_valid = 0;
    size_t planes = mfma ? align_up(estimate_mfma_ksplit_bytes(g, S), 256) : 0;
    if (opts->ksum_capacity != 0 || opts->ksum_valid != 0) {
        if (opts->ksum_capacity < g.L || opts->ksum_capacity % B || opts->ksum_valid < 0 || opts->ksum_valid > g.Lr ||
            opts->seq_first)
            return RR_ERR_PARAM;
        if (mfma) {
            Geom gc = g;
            gc.L = opts->ksum_capacity;
            need += align_up(estimate_mfma_ksplit_bytes(gc, S), 256) - planes;
            planes = align_up(estimate_mfma_ksplit_bytes(gc, S), 256);
            ls_cap = gc.L / S;
            ls_valid = opts->ksum_valid / S;                 // whole strides only: the one that was incomplete is redone
        }
    }
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return RR_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)hip_stream;
    unsigned char* wsb = reinterpret_cast<unsigned char*>(workspace);
    EstimateArgs a;
    a.Q = Q;
    a.K = K;
    a.S = S; a.B = B; a.R = B / S; a.Nb = g.L / B;
    a.tau = tau;
    a.protect_last = (flags & RR_FLAG_PROTECT_LAST) ? 1 : 0;
    a.diag_token = diag_token;
    a.off_hmul = off_hmul; a.off_add = off_add;
    a.sink_blocks = opts->sink_blocks; a.recent_blocks = opts->recent_blocks;
    a.seq_first = opts->seq_first;
    a.dense = out->dense; a.row_count = out->row_count; a.row_list = out->row_list;
    a.block_mass = out->block_mass;
    a.Ksum = nullptr;
    a.state_ws = nullptr;
    if (mfma) {
        // split stride sums -> block masses in the workspace (two sweeps on the matrix cores) -> Top-tau per row
        unsigned short* ksplit = reinterpret_cast<unsigned short*>(wsb);
        float* mass = reinterpret_cast<float*>(wsb + planes);
        float2* stats = reinterpret_cast<float2*>(reinterpret_cast<unsigned char*>(mass) +
                                                  align_up(estimate_mfma_mass_bytes(g, B), 256));
        if (launch_stride_mass_mfma(g, Q, K, S, B, off_hmul, off_add, diag_token, opts->seq_first, ksplit, ls_cap,
                                    ls_valid, mass, estimate_mfma_stats_bytes(g, S, B) ? stats : nullptr, st) != hipSuccess)
            return RR_ERR_LAUNCH;
        if (launch_select_rows(g, a, mass, st) != hipSuccess) return RR_ERR_LAUNCH;
    } else {
        float* Ksum = reinterpret_cast<float*>(wsb);
        if (launch_stride_sum(g, shape->dtype, K, S, Ksum, st) != hipSuccess) return RR_ERR_LAUNCH;
        a.Ksum = Ksum;
        a.state_ws = estimate_generic_state_bytes(g, S, B) ? reinterpret_cast<float2*>(wsb + ksum_bytes(g, S)) : nullptr;
        if (launch_estimate_generic(g, shape->dtype, a, st) != hipSuccess) return RR_ERR_LAUNCH;
    }
    if (out->row_order && (long long)g.G * (g.Lq / B) <= kMaxOrderedRows)
        if (launch_row_order(g, a.Nb, out->row_count, out->row_order, out->queue, st) != hipSuccess) return RR_ERR_LAUNCH;
    return RR_OK;
}

RR_API int rr_sparse_attn(const rr_shape* shape, const void* Q, const void* K, const void* V,
                   const rr_mask* mask, void* O, float* lse, void* hip_stream) {
    if (!mask || !mask->row_count || !mask->row_list) return RR_ERR_NULL;
    if (shape && mask->B > 0 && mask->Nb != (shape->L + mask->B - 1) / mask->B) return RR_ERR_PARAM;
    return run_attn(shape, Q, K, V, mask->B, mask->row_count, mask->row_list, mask->row_order, mask->queue, nullptr, O, lse,
                    hip_stream);
}

RR_API int rr_mask_from_dense(const rr_shape* shape, rr_mask* mask, void* hip_stream) {
    Geom g;
    int rc = check_shape(shape, &g);
    if (rc != RR_OK) return rc;
    if (!mask || !mask->dense || !mask->row_count || !mask->row_list) return RR_ERR_NULL;
    if (mask->B < 1 || pad_to_blocks(&g, mask->B) != RR_OK || mask->Nb != g.L / mask->B) return RR_ERR_PARAM;
    hipStream_t st = (hipStream_t)hip_stream;
    if (launch_mask_from_dense(g, mask->Nb, mask->dense, mask->row_count, mask->row_list, st) != hipSuccess)
        return RR_ERR_LAUNCH;
    if (mask->row_order && (long long)g.G * (g.Lq / mask->B) <= kMaxOrderedRows)
        if (launch_row_order(g, mask->Nb, mask->row_count, mask->row_order, mask->queue, st) != hipSuccess) return RR_ERR_LAUNCH;
    return RR_OK;
}

RR_API size_t rr_accuracy_workspace_bytes(const rr_shape* shape, int step) {
    Geom g;
    if (check_shape(shape, &g) != RR_OK || step < 1 || g.Lq % step) return 0;
    return align_up(accuracy_rows_bytes(g, step), 256) + align_up(accuracy_per_query_bytes(g, step), 256);
}

RR_API int rr_selection_accuracy(const rr_shape* shape, const void* Q, const void* K, const rr_mask* mask,
                          float tau, int step, void* workspace, size_t workspace_bytes, float* out,
                          void* hip_stream) {
    Geom g;
    int rc = check_shape(shape, &g);
    if (rc != RR_OK) return rc;
    if (!Q || !K || !mask || !mask->row_count || !mask->row_list || !out) return RR_ERR_NULL;
    if (mask->B < 1 || g.L % mask->B || g.Lq % mask->B || mask->Nb != g.L / mask->B) return RR_ERR_PARAM;
    if (!(tau > 0.f) || !(tau < 1.f) || step < 1 || g.Lq % step) return RR_ERR_PARAM;
    if (!aligned16(Q) || !aligned16(K)) return RR_ERR_SHAPE;
    const size_t need = rr_accuracy_workspace_bytes(shape, step);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return RR_ERR_WORKSPACE;
    unsigned char* wsb = reinterpret_cast<unsigned char*>(workspace);
    float* rows = reinterpret_cast<float*>(wsb);
    float2* per_query = reinterpret_cast<float2*>(wsb + align_up(accuracy_rows_bytes(g, step), 256));
    const hipError_t e = launch_selection_accuracy(g, shape->dtype, Q, K, mask->row_count, mask->row_list, mask->B, tau,
                                                   step, rows, per_query, out, (hipStream_t)hip_stream);
    return e == hipSuccess ? RR_OK : RR_ERR_LAUNCH;
}

RR_API int rr_dense_attn(const rr_shape* shape, const void* Q, const void* K, const void* V, int B,
                  void* O, float* lse, void* hip_stream) {
    return run_attn(shape, Q, K, V, B, nullptr, nullptr, nullptr, nullptr, nullptr, O, lse, hip_stream);
}

RR_API size_t rr_attn_workspace_bytes(const rr_shape* shape, int B) {
    Geom g;
    if (check_shape(shape, &g) != RR_OK || B < 1 || B > 128 || pad_to_blocks(&g, B) != RR_OK) return 0;
    if (!use_mfma_attn(g, shape->dtype, B)) return 0;
    if (attn_decode_parts(g, B) >= 1) return align_up(attn_decode_bytes(g, B), 256);
    if (attn_mfma_plan_len(g, B, nullptr) > 0) return align_up(attn_mfma_plan_bytes(g, B), 256);
    return align_up(attn_mfma_split_bytes(g, B), 256);
}

RR_API int rr_sparse_attn_ws(const rr_shape* shape, const void* Q, const void* K, const void* V, const rr_mask* mask,
                             void* O, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!mask || !mask->row_count || !mask->row_list) return RR_ERR_NULL;
    if (shape && mask->B > 0 && mask->Nb != (shape->L + mask->B - 1) / mask->B) return RR_ERR_PARAM;
    return run_attn(shape, Q, K, V, mask->B, mask->row_count, mask->row_list, mask->row_order, mask->queue, nullptr, O, lse,
                    hip_stream, workspace, workspace_bytes);
}

RR_API int rr_dense_attn_ws(const rr_shape* shape, const void* Q, const void* K, const void* V, int B, void* O, float* lse,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run_attn(shape, Q, K, V, B, nullptr, nullptr, nullptr, nullptr, nullptr, O, lse, hip_stream, workspace,
                    workspace_bytes);
}

RR_API int rr_dense_attn_packed(const rr_shape* shape, const void* Q, const void* K, const void* V, int B,
                         const int32_t* seq_first, void* O, float* lse, void* hip_stream) {
    if (!seq_first) return RR_ERR_NULL;
    return run_attn(shape, Q, K, V, B, nullptr, nullptr, nullptr, nullptr, seq_first, O, lse, hip_stream);
}

}  // extern "C"
