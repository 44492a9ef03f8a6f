// C ABI of the library: argument validation on the host, then the kernel launchers.
// Every entry point either enqueues all of its work on `stream` or (non-zero status) nothing.
#include "../../include/specmoe.h"
#include "common.h"

#include <limits.h>

#include <mutex>

using namespace specmoe;

namespace {

inline bool bad_dtype(int dt) { return dt != SPECMOE_F32 && dt != SPECMOE_BF16; }
inline size_t esize(int dt) { return dt == SPECMOE_F32 ? 4 : 2; }
inline int dev(hipError_t e) { return e == hipSuccess ? SPECMOE_OK : SPECMOE_ERR_DEVICE; }
inline bool pairs_overflow(int T, int k) { return (long long)T * k > (long long)INT_MAX / 2; }

}  // namespace

extern "C" {

int moe_route_topk(const void* x, const void* w_router, const float* router_bias, int T,
                   int d_model, int E, int k, int renorm, int dtype, int32_t* topk_idx,
                   float* topk_w, void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (T < 0 || d_model < 1 || E < 1 || E > SPECMOE_MAX_EXPERTS || k < 1 || k > E ||
        k > SPECMOE_MAX_TOPK || pairs_overflow(T, k))
        return SPECMOE_ERR_SHAPE;
    if (T == 0) return SPECMOE_OK;
    if (!x || !w_router || !topk_idx || !topk_w) return SPECMOE_ERR_NULL;
    return dev(launch_route_topk(x, w_router, router_bias, T, d_model, E, k, renorm, dtype,
                                 topk_idx, topk_w, (hipStream_t)stream));
}

int moe_permute(const void* x, const int32_t* topk_idx, int T, int d_model, int E, int k,
                int dtype, void* x_perm, int32_t* expert_offsets, int32_t* row_src,
                int32_t* row_of, void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (T < 0 || d_model < 1 || E < 1 || E > SPECMOE_MAX_EXPERTS || k < 1 || k > E ||
        k > SPECMOE_MAX_TOPK || pairs_overflow(T, k))
        return SPECMOE_ERR_SHAPE;
    if (!expert_offsets) return SPECMOE_ERR_NULL;
    if (T > 0 && (!topk_idx || !row_src || !row_of)) return SPECMOE_ERR_NULL;
    if (T > 0 && x_perm && !x) return SPECMOE_ERR_NULL;
    return dev(launch_permute(x, topk_idx, T, d_model, E, k, dtype, x_perm, expert_offsets,
                              row_src, row_of, (hipStream_t)stream));
}

size_t moe_grouped_swiglu_workspace_bytes(int n_rows, int d_model, int d_ff, int E, int dtype) {
    if (bad_dtype(dtype) || n_rows < 0 || d_model < 1 || d_ff < 1 || E < 1) return 0;
    size_t h = (size_t)n_rows * (size_t)d_ff * esize(dtype);
    return (h + 255) / 256 * 256 + 256;      // never 0 for valid arguments
}

static int check_expert_shapes(int n_rows, int d_model, int d_ff, int E, int dtype) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (n_rows < 0 || d_model < 1 || d_ff < 1 || E < 1 || E > SPECMOE_MAX_EXPERTS)
        return SPECMOE_ERR_SHAPE;
    if (dtype == SPECMOE_BF16 && (d_model % 64 != 0 || d_ff % 64 != 0)) return SPECMOE_ERR_SHAPE;
    return SPECMOE_OK;
}

int moe_expert_up_swiglu(const void* x_perm, const int32_t* expert_offsets, const void* w_gate,
                         const void* w_up, int n_rows, int d_model, int d_ff, int E, int dtype,
                         void* h, void* stream) {
    const int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (n_rows == 0) return SPECMOE_OK;
    if (!x_perm || !expert_offsets || !w_gate || !w_up || !h) return SPECMOE_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == SPECMOE_F32)
        return dev(launch_expert_up_f32((const float*)x_perm, expert_offsets, (const float*)w_gate,
                                        (const float*)w_up, n_rows, d_model, d_ff, E, (float*)h, s));
    return dev(launch_expert_up_bf16((const bf16_t*)x_perm, expert_offsets, (const bf16_t*)w_gate,
                                     (const bf16_t*)w_up, n_rows, d_model, d_ff, E, (bf16_t*)h, s));
}

int moe_expert_up_swiglu_gather(const void* x, const int32_t* row_src, int T, int k,
                                const int32_t* expert_offsets, const void* w_gate,
                                const void* w_up, int n_rows, int d_model, int d_ff, int E,
                                int dtype, void* h, void* stream) {
    const int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (T < 0 || k < 1 || k > SPECMOE_MAX_TOPK || pairs_overflow(T, k) ||
        (long long)n_rows > (long long)T * k)
        return SPECMOE_ERR_SHAPE;
    // the gathered loads address a token row through a 32-bit byte offset
    if ((unsigned long long)T * (unsigned long long)d_model * esize(dtype) >= (1ull << 32))
        return SPECMOE_ERR_SHAPE;
    if (n_rows == 0) return SPECMOE_OK;
    if (!x || !row_src || !expert_offsets || !w_gate || !w_up || !h) return SPECMOE_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == SPECMOE_F32)
        return dev(launch_expert_up_f32((const float*)x, expert_offsets, (const float*)w_gate,
                                        (const float*)w_up, n_rows, d_model, d_ff, E, (float*)h, s,
                                        row_src, k));
    return dev(launch_expert_up_bf16((const bf16_t*)x, expert_offsets, (const bf16_t*)w_gate,
                                     (const bf16_t*)w_up, n_rows, d_model, d_ff, E, (bf16_t*)h, s,
                                     row_src, k));
}

int moe_expert_down(const void* h, const int32_t* expert_offsets, const void* w_down, int n_rows,
                    int d_model, int d_ff, int E, int dtype, void* y_perm, void* stream) {
    const int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (n_rows == 0) return SPECMOE_OK;
    if (!h || !expert_offsets || !w_down || !y_perm) return SPECMOE_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == SPECMOE_F32)
        return dev(launch_expert_down_f32((const float*)h, expert_offsets, (const float*)w_down,
                                          n_rows, d_model, d_ff, E, (float*)y_perm, s));
    return dev(launch_expert_down_bf16((const bf16_t*)h, expert_offsets, (const bf16_t*)w_down,
                                       n_rows, d_model, d_ff, E, (bf16_t*)y_perm, s));
}

int moe_grouped_swiglu(const void* x_perm, const int32_t* expert_offsets, const void* w_gate,
                       const void* w_up, const void* w_down, int n_rows, int d_model, int d_ff,
                       int E, int dtype, void* y_perm, void* workspace, size_t workspace_bytes,
                       void* stream) {
    int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (n_rows == 0) return SPECMOE_OK;
    if (!x_perm || !expert_offsets || !w_gate || !w_up || !w_down || !y_perm || !workspace)
        return SPECMOE_ERR_NULL;
    if (workspace_bytes < moe_grouped_swiglu_workspace_bytes(n_rows, d_model, d_ff, E, dtype) ||
        ((uintptr_t)workspace & 255u) != 0)
        return SPECMOE_ERR_WORKSPACE;
    st = moe_expert_up_swiglu(x_perm, expert_offsets, w_gate, w_up, n_rows, d_model, d_ff, E,
                              dtype, workspace, stream);
    if (st != SPECMOE_OK) return st;
    return moe_expert_down(workspace, expert_offsets, w_down, n_rows, d_model, d_ff, E, dtype,
                           y_perm, stream);
}

int moe_pack_weights(const void* w, int E, int n_rows, int n_cols, int dtype, void* w_packed,
                     void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (dtype != SPECMOE_BF16) return SPECMOE_ERR_DTYPE;
    if (E < 1 || E > SPECMOE_MAX_EXPERTS || n_rows < 16 || n_cols < 32 || n_rows % 16 != 0 ||
        n_cols % 32 != 0)
        return SPECMOE_ERR_SHAPE;
    if (!w || !w_packed) return SPECMOE_ERR_NULL;
    const size_t bytes = (size_t)E * n_rows * n_cols * 2;
    const uintptr_t a = (uintptr_t)w, b = (uintptr_t)w_packed;
    if (((a | b) & 15u) != 0 || (a < b + bytes && b < a + bytes)) return SPECMOE_ERR_SHAPE;
    return dev(launch_pack_tiles((const bf16_t*)w, (long long)E * n_rows, n_cols,
                                 (bf16_t*)w_packed, (hipStream_t)stream));
}

size_t moe_packed_h_bytes(int n_rows, int d_ff, int E) {
    if (n_rows < 0 || d_ff < 1 || E < 1) return 0;
    return ((size_t)(n_rows / 16) + (size_t)E) * 16 * (size_t)d_ff * 2;
}

int moe_expert_up_swiglu_gather_packed(const void* x, const int32_t* row_src, int T, int k,
                                       const int32_t* expert_offsets, const void* w_gate_packed,
                                       const void* w_up_packed, int n_rows, int d_model, int d_ff,
                                       int E, int dtype, void* h_packed, size_t h_packed_bytes,
                                       void* x_packed_workspace, size_t x_packed_workspace_bytes,
                                       void* stream) {
    const int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (dtype != SPECMOE_BF16) return SPECMOE_ERR_DTYPE;
    if (row_src) {
        if (T < 0 || k < 1 || k > SPECMOE_MAX_TOPK || pairs_overflow(T, k) ||
            (long long)n_rows > (long long)T * k)
            return SPECMOE_ERR_SHAPE;
        if ((unsigned long long)T * (unsigned long long)d_model * 2 >= (1ull << 32))
            return SPECMOE_ERR_SHAPE;
    }
    if (n_rows == 0) return SPECMOE_OK;
    if (!x || !expert_offsets || !w_gate_packed || !w_up_packed || !h_packed)
        return SPECMOE_ERR_NULL;
    if (h_packed_bytes < moe_packed_h_bytes(n_rows, d_ff, E) || ((uintptr_t)h_packed & 15u) != 0)
        return SPECMOE_ERR_WORKSPACE;
    if (x_packed_workspace) {
        const int sp = moe_permute_rows_packed(x, row_src, T, k, expert_offsets, n_rows, d_model, E,
                                               dtype, x_packed_workspace,
                                               x_packed_workspace_bytes, stream);
        if (sp != SPECMOE_OK) return sp;
        return moe_expert_up_swiglu_packed(x_packed_workspace, x_packed_workspace_bytes,
                                           expert_offsets, w_gate_packed, w_up_packed, n_rows,
                                           d_model, d_ff, E, dtype, h_packed, h_packed_bytes, 0,
                                           stream);
    }
    return dev(launch_expert_up_bf16_packed((const bf16_t*)x, expert_offsets,
                                            (const bf16_t*)w_gate_packed,
                                            (const bf16_t*)w_up_packed, n_rows, d_model, d_ff, E,
                                            (bf16_t*)h_packed, (hipStream_t)stream, row_src,
                                            row_src ? k : 1));
}

int moe_permute_rows_packed(const void* x, const int32_t* row_src, int T, int k,
                            const int32_t* expert_offsets, int n_rows, int d_model, int E,
                            int dtype, void* x_packed, size_t x_packed_bytes, void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (dtype != SPECMOE_BF16) return SPECMOE_ERR_DTYPE;
    if (n_rows < 0 || d_model < 1 || d_model % 64 != 0 || E < 1 || E > SPECMOE_MAX_EXPERTS)
        return SPECMOE_ERR_SHAPE;
    if (row_src) {
        if (T < 0 || k < 1 || k > SPECMOE_MAX_TOPK || pairs_overflow(T, k) ||
            (long long)n_rows > (long long)T * k)
            return SPECMOE_ERR_SHAPE;
    }
    if (n_rows == 0) return SPECMOE_OK;
    if (!x || !expert_offsets || !x_packed) return SPECMOE_ERR_NULL;
    if (x_packed_bytes < moe_packed_h_bytes(n_rows, d_model, E) ||
        ((uintptr_t)x_packed & 15u) != 0 || ((uintptr_t)x & 15u) != 0)
        return SPECMOE_ERR_WORKSPACE;
    return dev(launch_gather_pack_rows((const bf16_t*)x, row_src, row_src ? k : 1, expert_offsets,
                                       n_rows, E, d_model, (bf16_t*)x_packed,
                                       (hipStream_t)stream));
}

int moe_expert_up_swiglu_packed(const void* x_packed, size_t x_packed_bytes,
                                const int32_t* expert_offsets, const void* w_gate_packed,
                                const void* w_up_packed, int n_rows, int d_model, int d_ff, int E,
                                int dtype, void* h, size_t h_bytes, int h_row_major,
                                void* stream) {
    const int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (dtype != SPECMOE_BF16) return SPECMOE_ERR_DTYPE;
    if (n_rows == 0) return SPECMOE_OK;
    if (!x_packed || !expert_offsets || !w_gate_packed || !w_up_packed || !h)
        return SPECMOE_ERR_NULL;
    const size_t h_need = h_row_major ? (size_t)n_rows * (size_t)d_ff * 2
                                      : moe_packed_h_bytes(n_rows, d_ff, E);
    if (h_bytes < h_need || ((uintptr_t)h & 15u) != 0 ||
        x_packed_bytes < moe_packed_h_bytes(n_rows, d_model, E) || ((uintptr_t)x_packed & 15u) != 0)
        return SPECMOE_ERR_WORKSPACE;
    return dev(launch_expert_up_bf16_packed_x(
        (const bf16_t*)x_packed, expert_offsets, (const bf16_t*)w_gate_packed,
        (const bf16_t*)w_up_packed, n_rows, d_model, d_ff, E, (bf16_t*)h, h_row_major != 0,
        (hipStream_t)stream));
}

int moe_expert_down_packed(const void* h_packed, const int32_t* expert_offsets,
                           const void* w_down_packed, int n_rows, int d_model, int d_ff, int E,
                           int dtype, void* y_perm, void* stream) {
    const int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (dtype != SPECMOE_BF16) return SPECMOE_ERR_DTYPE;
    if (n_rows == 0) return SPECMOE_OK;
    if (!h_packed || !expert_offsets || !w_down_packed || !y_perm) return SPECMOE_ERR_NULL;
    return dev(launch_expert_down_bf16_packed((const bf16_t*)h_packed, expert_offsets,
                                              (const bf16_t*)w_down_packed, n_rows, d_model, d_ff,
                                              E, (bf16_t*)y_perm, (hipStream_t)stream));
}

// Scratch of moe_grouped_swiglu_static: one copy per GPU, held until the process ends.
static __device__ __align__(256) unsigned char scratch[SPECMOE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU (0 = unknown)

// Device address of the scratch array on the current GPU.  The array's name is only a
// host-side handle; the address comes from hipGetSymbolAddress, once per device.
int scratch_address(void** out) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices)
        return SPECMOE_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return SPECMOE_ERR_DEVICE;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return SPECMOE_OK;
}
}  // namespace

int moe_grouped_swiglu_static(const void* x_perm, const int32_t* expert_offsets,
                              const void* w_gate, const void* w_up, const void* w_down,
                              int n_rows, int d_model, int d_ff, int E, int dtype, void* y_perm,
                              void* stream) {
    int st = check_expert_shapes(n_rows, d_model, d_ff, E, dtype);
    if (st != SPECMOE_OK) return st;
    if (n_rows == 0) return SPECMOE_OK;
    if (!x_perm || !expert_offsets || !w_gate || !w_up || !w_down || !y_perm)
        return SPECMOE_ERR_NULL;
    if ((unsigned long long)n_rows * (unsigned long long)d_ff * esize(dtype) >
        (unsigned long long)SPECMOE_STATIC_SCRATCH_BYTES)
        return SPECMOE_ERR_WORKSPACE;
    void* h = nullptr;
    st = scratch_address(&h);
    if (st != SPECMOE_OK) return st;
    st = moe_expert_up_swiglu(x_perm, expert_offsets, w_gate, w_up, n_rows, d_model, d_ff, E,
                              dtype, h, stream);
    if (st != SPECMOE_OK) return st;
    return moe_expert_down(h, expert_offsets, w_down, n_rows, d_model, d_ff, E, dtype, y_perm,
                           stream);
}

int moe_combine(const void* y_perm, const int32_t* row_of, const float* topk_w,
                const void* residual, int T, int d_model, int k, int dtype, void* out,
                void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (T < 0 || d_model < 1 || k < 1 || k > SPECMOE_MAX_TOPK || pairs_overflow(T, k))
        return SPECMOE_ERR_SHAPE;
    if (T == 0) return SPECMOE_OK;
    if (!y_perm || !row_of || !topk_w || !out) return SPECMOE_ERR_NULL;
    return dev(launch_combine(y_perm, row_of, topk_w, residual, T, d_model, k, dtype, out,
                              (hipStream_t)stream));
}

int spec_accept(const int32_t* draft_ids, const int32_t* target_ids, int B, int gamma,
                int32_t* accept_len, int32_t* out_tokens, void* stream) {
    if (B < 0 || gamma < 0 || (long long)B * (gamma + 1ll) > INT_MAX) return SPECMOE_ERR_SHAPE;
    if (B == 0) return SPECMOE_OK;
    if (!target_ids || !accept_len || !out_tokens || (gamma > 0 && !draft_ids))
        return SPECMOE_ERR_NULL;
    return dev(launch_spec_accept(draft_ids, target_ids, B, gamma, accept_len, out_tokens,
                                  (hipStream_t)stream));
}

int moe_hot_experts(const int32_t* expert_offsets, int E, int n_hot, int32_t* hot_ids,
                    int32_t* hot_counts, void* stream) {
    if (E < 1 || E > SPECMOE_MAX_EXPERTS || n_hot < 0 || n_hot > E) return SPECMOE_ERR_SHAPE;
    if (n_hot == 0) return SPECMOE_OK;
    if (!expert_offsets || !hot_ids) return SPECMOE_ERR_NULL;
    return dev(launch_hot_experts(expert_offsets, E, n_hot, hot_ids, hot_counts,
                                  (hipStream_t)stream));
}

size_t moe_affinity_table_workspace_bytes(int E) {
    if (E < 1 || E > SPECMOE_MAX_EXPERTS) return 0;
    return affinity_workspace_bytes(E);
}

int moe_affinity_table(const void* w_gate, const void* w_up, const void* w_down, int E,
                       int d_model, int d_ff, int dtype, float* affinity, void* workspace,
                       size_t workspace_bytes, void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (E < 1 || E > SPECMOE_MAX_EXPERTS || d_model < 1 || d_ff < 1) return SPECMOE_ERR_SHAPE;
    // 16-byte loads: one expert matrix must be a whole number of 16-byte chunks
    if (((size_t)d_model * d_ff * esize(dtype)) % 16 != 0) return SPECMOE_ERR_SHAPE;
    if (!w_gate || !w_up || !w_down || !affinity || !workspace) return SPECMOE_ERR_NULL;
    if ((((uintptr_t)w_gate | (uintptr_t)w_up | (uintptr_t)w_down) & 15u) != 0 ||
        ((uintptr_t)workspace & 7u) != 0)
        return SPECMOE_ERR_SHAPE;
    if (workspace_bytes < affinity_workspace_bytes(E)) return SPECMOE_ERR_WORKSPACE;
    return dev(launch_affinity_table(w_gate, w_up, w_down, E, d_model, d_ff, dtype, affinity,
                                     workspace, (hipStream_t)stream));
}

int moe_nearest_draft_expert(const float* affinity, int E, const int32_t* draft_ids, int n_draft,
                             int32_t* remap, void* stream) {
    if (E < 1 || E > SPECMOE_MAX_EXPERTS || n_draft < 1 || n_draft > E) return SPECMOE_ERR_SHAPE;
    if (!affinity || !draft_ids || !remap) return SPECMOE_ERR_NULL;
    return dev(launch_nearest_draft(affinity, E, draft_ids, n_draft, remap, (hipStream_t)stream));
}

int moe_route_topk_draft(const void* x, const void* w_router, const float* router_bias, int T,
                         int d_model, int E, int k, int renorm, int dtype, const int32_t* remap,
                         int32_t* topk_idx, float* topk_w, void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (T < 0 || d_model < 1 || E < 1 || E > SPECMOE_MAX_EXPERTS || k < 1 || k > E ||
        k > SPECMOE_MAX_TOPK || pairs_overflow(T, k))
        return SPECMOE_ERR_SHAPE;
    if (!remap) return SPECMOE_ERR_NULL;
    if (T == 0) return SPECMOE_OK;
    if (!x || !w_router || !topk_idx || !topk_w) return SPECMOE_ERR_NULL;
    return dev(launch_route_topk(x, w_router, router_bias, T, d_model, E, k, renorm, dtype,
                                 topk_idx, topk_w, (hipStream_t)stream, remap));
}

int spec_accept_sample(const int32_t* draft_ids, const float* p_draft, const float* p_target,
                       const float* u_accept, const float* u_sample, int B, int gamma, int V,
                       int32_t* accept_len, int32_t* out_tokens, void* stream) {
    if (B < 0 || gamma < 0 || gamma > SPECMOE_MAX_GAMMA || V < 1) return SPECMOE_ERR_SHAPE;
    if ((long long)B * (gamma + 1) > INT_MAX / 2) return SPECMOE_ERR_SHAPE;
    if (B == 0) return SPECMOE_OK;
    if (!p_target || !u_sample || !accept_len || !out_tokens) return SPECMOE_ERR_NULL;
    if (gamma > 0 && (!draft_ids || !p_draft || !u_accept)) return SPECMOE_ERR_NULL;
    return dev(launch_spec_accept_sample(draft_ids, p_draft, p_target, u_accept, u_sample, B,
                                         gamma, V, accept_len, out_tokens, (hipStream_t)stream));
}

int spec_greedy_tokens(const void* logits, int R, int V, int dtype, int32_t* tokens,
                       void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (R < 0 || V < 1) return SPECMOE_ERR_SHAPE;
    if (R == 0) return SPECMOE_OK;
    if (!logits || !tokens) return SPECMOE_ERR_NULL;
    return dev(launch_greedy_tokens(logits, R, V, dtype, tokens, (hipStream_t)stream));
}

int moe_active_expert_bytes(const int32_t* expert_offsets, int E, long long bytes_per_expert,
                            long long* out_bytes, void* stream) {
    if (E < 1 || E > SPECMOE_MAX_EXPERTS || bytes_per_expert < 0) return SPECMOE_ERR_SHAPE;
    if (!expert_offsets || !out_bytes) return SPECMOE_ERR_NULL;
    return dev(launch_active_expert_bytes(expert_offsets, E, bytes_per_expert, out_bytes,
                                          (hipStream_t)stream));
}

int moe_rmsnorm(const void* x, const void* gain, int T, int d_model, float eps, int dtype,
                void* out, void* stream) {
    if (bad_dtype(dtype)) return SPECMOE_ERR_DTYPE;
    if (T < 0 || d_model < 1 || !(eps >= 0.f)) return SPECMOE_ERR_SHAPE;
    if (T == 0) return SPECMOE_OK;
    if (!x || !gain || !out) return SPECMOE_ERR_NULL;
    return dev(launch_rmsnorm(x, gain, T, d_model, eps, dtype, out, (hipStream_t)stream));
}

const char* specmoe_status_string(int status) {
    switch (status) {
        case SPECMOE_OK: return "ok";
        case SPECMOE_ERR_NULL: return "a required pointer is NULL";
        case SPECMOE_ERR_SHAPE: return "invalid or unsupported shape";
        case SPECMOE_ERR_DTYPE: return "unknown dtype";
        case SPECMOE_ERR_WORKSPACE: return "workspace too small or misaligned";
        case SPECMOE_ERR_DEVICE: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

int specmoe_abi_version(void) { return 8; }

}  // extern "C"
