// C-ABI entry points of libsage: host-side validation, then kernel launches.
#include "../../include/sage.h"
#include "sage_internal.h"
#include <cmath>
#include <mutex>

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_shape(int B, int H, int N, int D) {
    if (B <= 0 || H <= 0 || N <= 0 || D <= 0) return SAGE_ERR_SHAPE;
    if (N > (1 << 23)) return SAGE_ERR_SHAPE;
    if ((long long)B * H > 65535) return SAGE_ERR_SHAPE;          // slabs are a grid dimension of the pre-pass
    // B*H*N*D must stay below 2^62 (N*N*B*H for the dump is the caller's concern)
    long double elems = (long double)B * H * (long double)N * D;
    if (elems > 4.0e18L) return SAGE_ERR_SHAPE;
    if (D != 64 && D != 128) return SAGE_ERR_UNSUPPORTED;
    return SAGE_OK;
}

// tokens per scale: 1 = per-token quantizer, else a per-block one
bool quant_block_ok(int b) { return b == 1 || b == 32 || b == 64 || b == 128; }

}  // namespace

#ifndef SAGE_SOURCE_HASH
#define SAGE_SOURCE_HASH "unknown"
#endif

extern "C" {

const char* sage_source_hash(void) {
    // the marker stays in the binary, so that the hash can also be read from the file without loading it
    static const char tagged[] = "SAGE_SOURCE_HASH=" SAGE_SOURCE_HASH;
    return tagged + sizeof("SAGE_SOURCE_HASH=") - 1;
}

float sage_default_sm_scale(int D) { return D > 0 ? 1.0f / std::sqrt((float)D) : 0.0f; }

const char* sage_status_string(int status) {
    switch (status) {
        case SAGE_OK: return "SAGE_OK";
        case SAGE_ERR_NULL: return "SAGE_ERR_NULL: a required pointer is NULL";
        case SAGE_ERR_SHAPE: return "SAGE_ERR_SHAPE: B, H, N, D out of range";
        case SAGE_ERR_UNSUPPORTED: return "SAGE_ERR_UNSUPPORTED: head dimension or block size not covered";
        case SAGE_ERR_WORKSPACE: return "SAGE_ERR_WORKSPACE: workspace too small";
        case SAGE_ERR_ALIGN: return "SAGE_ERR_ALIGN: pointer alignment";
        case SAGE_ERR_LAUNCH: return "SAGE_ERR_LAUNCH: HIP launch failed";
        case SAGE_ERR_VALUE: return "SAGE_ERR_VALUE: sm_scale must be finite and positive";
        case SAGE_ERR_SCRATCH: return "SAGE_ERR_SCRATCH: the shape needs more scratch than the library's static buffer holds";
        default: return "SAGE_ERR_UNKNOWN";
    }
}

namespace {
int quant_q_impl(const void* q_f16, const float* cs, const float* sn, bool rope, int8_t* q_i8, float* q_scale,
                 int B, int H, int N, int D, float sm_scale, int block_q, void* stream) {
    if (!q_f16 || !q_i8 || !q_scale || (rope && (!cs || !sn))) return SAGE_ERR_NULL;
    if (int e = check_shape(B, H, N, D)) return e;
    if (!quant_block_ok(block_q)) return SAGE_ERR_UNSUPPORTED;
    if (!std::isfinite(sm_scale) || !(sm_scale > 0.0f)) return SAGE_ERR_VALUE;
    if (!aligned(q_f16, 16) || !aligned(q_i8, 16) || !aligned(q_scale, 4)) return SAGE_ERR_ALIGN;
    if (rope && (!aligned(cs, 16) || !aligned(sn, 16))) return SAGE_ERR_ALIGN;
    hipError_t e = sage::launch_quant_q(q_f16, q_i8, q_scale, B * H, N, D, sm_scale, block_q,
                                        rope ? cs : nullptr, rope ? sn : nullptr, (hipStream_t)stream);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}

int smooth_quant_k_impl(const void* k_f16, const float* cs, const float* sn, bool rope, int8_t* k_i8,
                        float* k_scale, float* k_mean, void* workspace, size_t workspace_bytes,
                        int B, int H, int N, int D, int block_k, void* stream) {
    if (!k_f16 || !k_i8 || !k_scale || (rope && (!cs || !sn))) return SAGE_ERR_NULL;      // k_mean is optional
    if (int e = check_shape(B, H, N, D)) return e;
    if (!quant_block_ok(block_k)) return SAGE_ERR_UNSUPPORTED;
    const size_t need = sage_smooth_quant_k_workspace(B, H, N, D);
    if (need > 0 && !workspace) return SAGE_ERR_NULL;
    if (workspace_bytes < need) return SAGE_ERR_WORKSPACE;
    if (!aligned(k_f16, 16) || !aligned(k_i8, 16) || !aligned(k_scale, 4) || !aligned(k_mean, 4) ||
        !aligned(workspace, 8))
        return SAGE_ERR_ALIGN;
    if (rope && (!aligned(cs, 16) || !aligned(sn, 16))) return SAGE_ERR_ALIGN;
    hipError_t e = sage::launch_smooth_quant_k(k_f16, k_i8, k_scale, k_mean, (long long*)workspace,
                                               B * H, N, D, block_k, rope ? cs : nullptr, rope ? sn : nullptr,
                                               (hipStream_t)stream);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}
}  // namespace

int sage_quant_q(const void* q_f16, int8_t* q_i8, float* q_scale,
                 int B, int H, int N, int D, float sm_scale, int block_q, void* stream) {
    return quant_q_impl(q_f16, nullptr, nullptr, false, q_i8, q_scale, B, H, N, D, sm_scale, block_q, stream);
}

int sage_rope_quant_q(const void* q_f16, const float* rope_cos, const float* rope_sin, int8_t* q_i8, float* q_scale,
                      int B, int H, int N, int D, float sm_scale, int block_q, void* stream) {
    return quant_q_impl(q_f16, rope_cos, rope_sin, true, q_i8, q_scale, B, H, N, D, sm_scale, block_q, stream);
}

size_t sage_smooth_quant_k_workspace(int B, int H, int N, int D) {
    if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || (long long)B * H > 65535) return 0;
    return (size_t)sage::plan_colsum(B * H, N).parts * B * H * D * sizeof(long long);
}

int sage_smooth_quant_k(const void* k_f16, int8_t* k_i8, float* k_scale, float* k_mean,
                        void* workspace, size_t workspace_bytes,
                        int B, int H, int N, int D, int block_k, void* stream) {
    return smooth_quant_k_impl(k_f16, nullptr, nullptr, false, k_i8, k_scale, k_mean, workspace, workspace_bytes,
                               B, H, N, D, block_k, stream);
}

// ---- sage_smooth_quant_k for callers that cannot allocate: the partial column sums live in a
// file-scope device array instead of a caller-supplied workspace.
namespace {
constexpr size_t SCRATCH_BYTES = SAGE_NOALLOC_SCRATCH_BYTES;
constexpr int SCRATCH_MAX_DEVICES = 64;
__device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];
// Every device holds its own copy of the array at its own address; `scratch` itself is only a
// host-side handle and must never be handed to a kernel or a copy.
void* scratch_addr[SCRATCH_MAX_DEVICES];
std::mutex scratch_mutex;

// Device address of this device's copy of `scratch` (looked up once per device), or null on error.
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SCRATCH_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_addr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        scratch_addr[dev] = p;
    }
    return scratch_addr[dev];
}
}  // namespace

int sage_smooth_quant_k_noalloc(const void* k_f16, int8_t* k_i8, float* k_scale, float* k_mean,
                                int B, int H, int N, int D, int block_k, void* stream) {
    if (int e = check_shape(B, H, N, D)) return e;
    const size_t need = sage_smooth_quant_k_workspace(B, H, N, D);
    if (need > SCRATCH_BYTES) return SAGE_ERR_SCRATCH;
    void* ws = nullptr;
    if (need > 0) {
        ws = scratch_on_current_device();
        if (ws == nullptr) return SAGE_ERR_LAUNCH;
    }
    return smooth_quant_k_impl(k_f16, nullptr, nullptr, false, k_i8, k_scale, k_mean, ws, need, B, H, N, D, block_k, stream);
}

int sage_quant_qk(const void* q_f16, const void* k_f16, int8_t* q_i8, float* q_scale,
                  int8_t* k_i8, float* k_scale, float* k_mean, void* workspace, size_t workspace_bytes,
                  int B, int H, int Nq, int Nkv, int D, float sm_scale, int block_q, int block_k, void* stream) {
    if (!q_f16 || !k_f16 || !q_i8 || !q_scale || !k_i8 || !k_scale) return SAGE_ERR_NULL;      // k_mean is optional
    if (int e = check_shape(B, H, Nq, D)) return e;
    if (int e = check_shape(B, H, Nkv, D)) return e;
    if (!quant_block_ok(block_q) || !quant_block_ok(block_k)) return SAGE_ERR_UNSUPPORTED;
    if (!std::isfinite(sm_scale) || !(sm_scale > 0.0f)) return SAGE_ERR_VALUE;
    const size_t need = sage_smooth_quant_k_workspace(B, H, Nkv, D);
    if (need > 0 && !workspace) return SAGE_ERR_NULL;
    if (workspace_bytes < need) return SAGE_ERR_WORKSPACE;
    if (!aligned(q_f16, 16) || !aligned(q_i8, 16) || !aligned(q_scale, 4) || !aligned(k_f16, 16) || !aligned(k_i8, 16) ||
        !aligned(k_scale, 4) || !aligned(k_mean, 4) || !aligned(workspace, 8))
        return SAGE_ERR_ALIGN;
    hipError_t e = sage::launch_quant_qk(q_f16, k_f16, q_i8, q_scale, k_i8, k_scale, k_mean, (long long*)workspace,
                                         B * H, Nq, Nkv, D, sm_scale, block_q, block_k, (hipStream_t)stream);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}

int sage_rope_smooth_quant_k(const void* k_f16, const float* rope_cos, const float* rope_sin,
                             int8_t* k_i8, float* k_scale, float* k_mean,
                             void* workspace, size_t workspace_bytes,
                             int B, int H, int N, int D, int block_k, void* stream) {
    return smooth_quant_k_impl(k_f16, rope_cos, rope_sin, true, k_i8, k_scale, k_mean, workspace, workspace_bytes,
                               B, H, N, D, block_k, stream);
}

namespace {
// The six attention entry points differ in the second product (v is V in fp16, or V^^T in INT8 with
// v_scale), in whether the two lengths may differ, and in whether the keys are cut into chunks
// (split: n_splits requested chunks and a workspace; otherwise one chunk, no workspace).
int attn_impl(bool pv_int8, bool split, const int8_t* q_i8, const float* q_scale, const int8_t* k_i8,
              const float* k_scale, const void* v, const float* v_scale, void* o_f16,
              void* workspace, size_t workspace_bytes, int B, int H, int Nq, int Nkv, int D, int causal,
              float sm_scale, int block_q, int block_k, int n_splits, void* stream) {
    if (!q_i8 || !q_scale || !k_i8 || !k_scale || !v || !o_f16 || (pv_int8 && !v_scale)) return SAGE_ERR_NULL;
    if (int e = check_shape(B, H, Nq, D)) return e;
    if (int e = check_shape(B, H, Nkv, D)) return e;
    if (causal && Nq > Nkv) return SAGE_ERR_UNSUPPORTED;        // a query before the first key would see nothing
    if (!quant_block_ok(block_q)) return SAGE_ERR_UNSUPPORTED;
    if (block_k != 1 && block_k != 64 && block_k != 128) return SAGE_ERR_UNSUPPORTED;
    if (split && n_splits < 0) return SAGE_ERR_VALUE;
    if (!std::isfinite(sm_scale) || !(sm_scale > 0.0f)) return SAGE_ERR_VALUE;
    // (slab, chunk) pairs are counted in an int by the kernels
    if (split && (long long)B * H * sage_attn_split_count(B, H, Nq, Nkv, causal, n_splits) > (1ll << 30)) return SAGE_ERR_SHAPE;
    const size_t need = split ? sage_attn_split_workspace(B, H, Nq, Nkv, D, causal, n_splits) : 0;
    if (need > 0 && !workspace) return SAGE_ERR_NULL;
    if (workspace_bytes < need) return SAGE_ERR_WORKSPACE;
    if (!aligned(q_i8, 16) || !aligned(k_i8, 16) || !aligned(v, 16) || !aligned(o_f16, 16) ||
        !aligned(q_scale, 4) || !aligned(k_scale, 4) || (pv_int8 && !aligned(v_scale, 16)) ||
        (need > 0 && !aligned(workspace, 16)))
        return SAGE_ERR_ALIGN;
    const int c = causal ? 1 : 0, BH = B * H;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (pv_int8) {
        const int8_t* vt = (const int8_t*)v;
        e = split ? sage::launch_attn_pv8_split(q_i8, q_scale, k_i8, k_scale, vt, v_scale, o_f16, workspace, BH, Nq, Nkv, D, c,
                                                block_q, block_k, n_splits, st)
                  : sage::launch_attn_pv8(q_i8, q_scale, k_i8, k_scale, vt, v_scale, o_f16, BH, Nq, Nkv, D, c, block_q, block_k, st);
    } else {
        e = split ? sage::launch_attn_split(q_i8, q_scale, k_i8, k_scale, v, o_f16, workspace, BH, Nq, Nkv, D, c,
                                            block_q, block_k, n_splits, st)
                  : sage::launch_attn(q_i8, q_scale, k_i8, k_scale, v, o_f16, nullptr, BH, Nq, Nkv, D, c, block_q, block_k, st);
    }
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}
}  // namespace

int sage_attn_split_count(int B, int H, int Nq, int Nkv, int causal, int n_splits) {
    if (B <= 0 || H <= 0 || Nq <= 0 || Nkv <= 0 || n_splits < 0) return 0;
    if (causal && Nq > Nkv) return 0;
    return sage::plan_split(B * H, Nq, Nkv, causal ? 1 : 0, n_splits).n_splits;
}

size_t sage_attn_split_workspace(int B, int H, int Nq, int Nkv, int D, int causal, int n_splits) {
    const int n = sage_attn_split_count(B, H, Nq, Nkv, causal, n_splits);
    if (n <= 1 || D <= 0) return 0;
    return (size_t)n * B * H * Nq * ((size_t)D * 2 + 4);
}

int sage_attn_fwd(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                  const void* v_f16, void* o_f16, int B, int H, int N, int D, int causal,
                  float sm_scale, int block_q, int block_k, void* stream) {
    return attn_impl(false, false, q_i8, q_scale, k_i8, k_scale, v_f16, nullptr, o_f16, nullptr, 0,
                     B, H, N, N, D, causal, sm_scale, block_q, block_k, 1, stream);
}

int sage_attn_cross_fwd(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                        const void* v_f16, void* o_f16, int B, int H, int Nq, int Nkv, int D, int causal,
                        float sm_scale, int block_q, int block_k, void* stream) {
    return attn_impl(false, false, q_i8, q_scale, k_i8, k_scale, v_f16, nullptr, o_f16, nullptr, 0,
                     B, H, Nq, Nkv, D, causal, sm_scale, block_q, block_k, 1, stream);
}

int sage_attn_cross_split_fwd(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                              const void* v_f16, void* o_f16, void* workspace, size_t workspace_bytes,
                              int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                              int block_q, int block_k, int n_splits, void* stream) {
    return attn_impl(false, true, q_i8, q_scale, k_i8, k_scale, v_f16, nullptr, o_f16, workspace, workspace_bytes,
                     B, H, Nq, Nkv, D, causal, sm_scale, block_q, block_k, n_splits, stream);
}

int sage_attn_pv_int8_fwd(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                          const int8_t* v_i8t, const float* v_scale, void* o_f16,
                          int B, int H, int N, int D, int causal, float sm_scale,
                          int block_q, int block_k, void* stream) {
    return attn_impl(true, false, q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, o_f16, nullptr, 0,
                     B, H, N, N, D, causal, sm_scale, block_q, block_k, 1, stream);
}

int sage_attn_pv_int8_cross_fwd(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                                const int8_t* v_i8t, const float* v_scale, void* o_f16,
                                int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                                int block_q, int block_k, void* stream) {
    return attn_impl(true, false, q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, o_f16, nullptr, 0,
                     B, H, Nq, Nkv, D, causal, sm_scale, block_q, block_k, 1, stream);
}

int sage_attn_pv_int8_cross_split_fwd(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                                      const int8_t* v_i8t, const float* v_scale, void* o_f16,
                                      void* workspace, size_t workspace_bytes,
                                      int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                                      int block_q, int block_k, int n_splits, void* stream) {
    return attn_impl(true, true, q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, o_f16, workspace, workspace_bytes,
                     B, H, Nq, Nkv, D, causal, sm_scale, block_q, block_k, n_splits, stream);
}

size_t sage_quant_v_workspace(int B, int H, int N, int D) {
    (void)N;
    if (B <= 0 || H <= 0 || D <= 0) return 0;
    return (size_t)B * H * D * sizeof(unsigned);
}

int sage_quant_v_pitch(int N) { return N <= 0 ? 0 : 64 * ((N + 63) / 64); }

int sage_quant_v(const void* v_f16, int8_t* v_i8t, float* v_scale, void* workspace, size_t workspace_bytes,
                 int B, int H, int N, int D, void* stream) {
    if (!v_f16 || !v_i8t || !v_scale || !workspace) return SAGE_ERR_NULL;
    if (int e = check_shape(B, H, N, D)) return e;
    if (workspace_bytes < sage_quant_v_workspace(B, H, N, D)) return SAGE_ERR_WORKSPACE;
    if (!aligned(v_f16, 16) || !aligned(v_i8t, 16) || !aligned(v_scale, 16) || !aligned(workspace, 4))
        return SAGE_ERR_ALIGN;
    hipError_t e = sage::launch_quant_v(v_f16, v_i8t, v_scale, (unsigned*)workspace, B * H, N, D, (hipStream_t)stream);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}

int sage_microbench(int kind, int waves_per_simd, int workgroups, int iters,
                    const int32_t* data, uint64_t* out, void* stream) {
    if (!data || !out) return SAGE_ERR_NULL;
    if (kind < 0 || kind > 20 || (waves_per_simd != 1 && waves_per_simd != 2)) return SAGE_ERR_UNSUPPORTED;
    if (kind == 5 && waves_per_simd != 2) return SAGE_ERR_UNSUPPORTED;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return SAGE_ERR_SHAPE;
    if (!aligned(data, 16) || !aligned(out, 8)) return SAGE_ERR_ALIGN;
    hipError_t e = sage::launch_microbench(kind, waves_per_simd, workgroups, iters, (const int*)data,
                                           (unsigned long long*)out, (hipStream_t)stream);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}

int sage_attn_qk_i32_debug(const int8_t* q_i8, const int8_t* k_i8, int32_t* s_i32,
                           int B, int H, int N, int D, int block_q, int block_k, int wg_rows, void* stream) {
    if (!q_i8 || !k_i8 || !s_i32) return SAGE_ERR_NULL;
    if (int e = check_shape(B, H, N, D)) return e;
    if (!quant_block_ok(block_q)) return SAGE_ERR_UNSUPPORTED;
    if (block_k != 1 && block_k != 64 && block_k != 128) return SAGE_ERR_UNSUPPORTED;
    if (wg_rows != 0 && wg_rows != 128 && wg_rows != 256) return SAGE_ERR_UNSUPPORTED;
    if (!aligned(q_i8, 16) || !aligned(k_i8, 16) || !aligned(s_i32, 4)) return SAGE_ERR_ALIGN;
    // scales are not read by the dump path; pass the tensor pointers as placeholders of valid memory
    hipError_t e = sage::launch_attn(q_i8, (const float*)q_i8, k_i8, (const float*)k_i8, nullptr, nullptr, s_i32,
                                     B * H, N, N, D, 0, block_q, block_k, (hipStream_t)stream, wg_rows);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}

int sage_attn_clock_debug(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                          const void* v_f16, void* o_f16, uint64_t* clocks,
                          int B, int H, int N, int D, int causal, int block_q, int block_k, void* stream) {
    if (!q_i8 || !q_scale || !k_i8 || !k_scale || !v_f16 || !o_f16 || !clocks) return SAGE_ERR_NULL;
    if (int e = check_shape(B, H, N, D)) return e;
    if (D != 128 || !quant_block_ok(block_q) || (block_k != 64 && block_k != 128)) return SAGE_ERR_UNSUPPORTED;
    if (!aligned(q_i8, 16) || !aligned(k_i8, 16) || !aligned(v_f16, 16) || !aligned(o_f16, 16) ||
        !aligned(q_scale, 4) || !aligned(k_scale, 4) || !aligned(clocks, 8))
        return SAGE_ERR_ALIGN;
    hipError_t e = sage::launch_attn_clocks(q_i8, q_scale, k_i8, k_scale, v_f16, o_f16, (unsigned long long*)clocks,
                                            B * H, N, causal ? 1 : 0, block_q, block_k, (hipStream_t)stream);
    return e == hipSuccess ? SAGE_OK : SAGE_ERR_LAUNCH;
}

}  // extern "C"
