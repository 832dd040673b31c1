// Internal launch interface between the translation units of libmassv_verify.
// Every function only enqueues on `st` and returns a massv_status.
#pragma once

#include "common.h"
#include <hip/hip_ext.h>

namespace massv {

// ---- one-shot kernel timing hook (api.hip) ----
// massv_trace_kernel() arms a request on the calling thread; the next launch of that kernel goes out
// through hipExtLaunchKernelGGL with the caller's two events, which then carry the kernel's own begin
// and end timestamps (the same clock a profiler's kernel trace reports), and the request is disarmed.
struct TraceRequest { int kid; hipEvent_t start, stop; };
TraceRequest& trace_request();

template <typename K, typename... Args>
inline void launch_traced(int kid, K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
    TraceRequest& t = trace_request();
    if (kid >= 0 && t.kid == kid) {
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, t.start, t.stop, 0, args...);
        t.kid = -1;
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
    }
}

// ---- small row-wise kernels (elementwise.hip) ----
// y[m,:] = x[m,:] * g / sqrt(mean(x[m,:]^2) + eps)
int launch_rmsnorm(const void* x, const void* g, void* y, int M, int H, float eps, hipStream_t st);      // fp32 rows
// bf16 only: same, output in operand order (packed_index); g == nullptr re-lays the rows out without normalising.
int launch_rmsnorm_packed(const void* x, const void* g, void* y, int M, int H, float eps, hipStream_t st);
// Rotates the q and k heads of qkv[M][(n_q+2n_kv)*d] by pos[m], writes q to
// q_out[M][n_q][d] and the k / v rows of token (b,i) to cache row kv_len[b]+i.
// q_norm / k_norm [d] (nullptr = none): RMSNorm of every query / key head before the rotation.
int launch_rope_append(const void* qkv, const int32_t* pos, const int32_t* kv_len, void* q_out,
                       void* k_cache, void* v_cache, const void* q_norm, const void* k_norm, float eps,
                       const massv_attn_desc& a, float theta, hipStream_t st);
// bf16: sums the K slabs of the q/k/v projection's partial sums [slabs][Mp][(n_q+2n_kv)*d], adds the biases
// (nullptr = none), normalises the q / k heads (q_norm, k_norm; nullptr = no), rotates q and k, writes q to
// q_out[M][n_q][d] and k / v to their cache rows.
int launch_qkv_finish(const float* partial, int n_slabs, size_t slab_stride, const void* bq, const void* bk,
                      const void* bv, const int32_t* pos, const int32_t* kv_len, void* q_out, void* k_cache,
                      void* v_cache, const void* q_norm, const void* k_norm, float eps,
                      const massv_attn_desc& a, float theta, hipStream_t st);
// bf16: y[m,:] = sum over slabs of partial[s][m,:]; r = base + (post ? rmsnorm(y, post) : y) with base = h_in (fp32
// rows) when given, else x; r is written to h_out (fp32) when given, else to x (bf16); if ln != nullptr also
// rmsnorm(r, ln) in operand order to xn_packed.
int launch_residual_finish(const float* partial, int n_slabs, size_t slab_stride, void* x, const float* h_in, float* h_out,
                           const void* post, const void* ln, void* xn_packed, int M, int H, float eps, hipStream_t st);
// fp32: x[m,:] += rmsnorm(y[m,:], g).
int launch_postnorm_residual(void* x, const void* y, const void* g, int M, int H, float eps, hipStream_t st);

// ---- projections (gemm.hip) ----
// One linear map Y = X W^T over M rows.  Up to three weight matrices that share
// X are applied in one launch; their outputs are laid side by side in Y
// ([M][n0+n1+n2]).
enum Epilogue {
    EPI_STORE = 0,      // f32 only: y = acc (+ bias)
    EPI_RESIDUAL = 1,   // f32 only: y = acc + residual (residual may alias y)
    EPI_GATED = 2,      // two matrices (gate, up) of equal size: y = act(gate) * up (bf16: y in operand order)
    EPI_LOGITS = 3,     // y = acc stored as float32 [M][N]
    EPI_PARTIAL = 4,    // bf16 only: fp32 partial sums y[slab][16*ceil(M/16)][N], one slab per K range;
                        // bias / residual are applied by the kernel that sums the slabs
    EPI_ARGMAX = 5,     // bf16 only: nothing is stored but, per row and workgroup, the largest output and its
                        // (lowest) column: y is RowPartial[M][groups]
    EPI_LOGITS_STATS = 6 // bf16 only: EPI_LOGITS, and stats[M][groups] receives per row and workgroup the largest
                        // output, its lowest column and the sum of exp((x - largest) / T) over the workgroup's columns
};
// Maximum, first arg-max and sum of exponentials of one piece of a logit row (pieces are merged by accept_decide_kernel).
struct RowPartial { float m; int arg; double s; };
struct GemmPlan { int nt, slabs, groups; };
// Greedy accept chain from per-piece row partials: part[row][C] for the B*(gamma+1) target rows (accept.hip).
int launch_accept_decide_greedy(const RowPartial* part, int C, const int32_t* draft_tokens, int B, int gamma, int V,
                                int32_t* n_accepted, int32_t* out_tokens, hipStream_t st);
// log2(e)/T split in two floats (d*hi + d*lo is d*log2(e)/T to about 1 ulp) and 1/T: how every kernel that forms
// exp((x - max)/T) scales its exponent.
struct TempScale { float hi, lo; double inv; };
TempScale temp_scale(float temperature);
// The accept rule at T > 0 with the target rows' statistics already formed by the vocabulary projection
// (part_t[B*(gamma+1)][C_t], written by an EPI_LOGITS_STATS launch): pass 1 runs over the draft rows only.
// ws: accept_prestats_bytes(B, gamma, V) bytes.
size_t accept_prestats_bytes(int B, int gamma, int V);
int launch_accept_prestats(const float* target_logits, const RowPartial* part_t, int C_t, const float* draft_logits,
                           const int32_t* draft_tokens, const float* uniforms, float temperature, int B, int gamma, int V,
                           int32_t* n_accepted, int32_t* out_tokens, void* ws, hipStream_t st);
struct GemmArgs {
    const void* x;            // f32: [M][K] row-major; bf16: operand order (packed_index), packed_elems(M,K) elements
    const void* w[3];         // [n_i][K]
    const void* bias[3];      // [n_i] or nullptr
    int n[3];                 // rows of each matrix (0 = unused)
    const void* residual;     // EPI_RESIDUAL: [M][n0]
    void* y;
    void* stats;              // EPI_LOGITS_STATS: RowPartial[M][groups]
    float temperature;        // EPI_LOGITS_STATS: T > 0 of the exponentials
    void* scratch;            // f32 + EPI_GATED only: [M][2*n0] floats
    int M, K;
    int epilogue, act, dtype;
    int kid;                  // massv_kernel_id bracketed by a pending trace request
};
int launch_gemm(const GemmArgs& g, hipStream_t st);
// bf16: tile count per wave and number of K slabs launch_gemm will use; bytes of the EPI_PARTIAL output.
GemmPlan gemm_plan(const GemmArgs& g);
size_t gemm_partial_bytes(const GemmArgs& g);
// Whether launch_gemm can run this problem (host-side shape check only).
int gemm_supported(const GemmArgs& g);

// ---- attention (attention.hip) ----
size_t attention_workspace(const massv_attn_desc& a);
int check_attn_desc(const massv_attn_desc* a);
// out_packed (bf16 only): write out[B*Q][n_q*d] in operand order for the output projection.
int launch_attention(const massv_attn_desc& a, const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* kv_len, void* out, void* ws, bool out_packed, hipStream_t st);

}  // namespace massv
