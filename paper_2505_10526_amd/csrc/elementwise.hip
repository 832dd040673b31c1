// Row-wise kernels of the decoder layer: RMSNorm, rotary embedding with KV
// append, cache and weight packing.  All traffic here is a few
// hundred KB per call; the kernels are written for clarity and coalescing,
// the math is fp32 (angles in double).
#include "kernels.h"

namespace massv {

// ---------------------------------------------------------------------------
// RMSNorm: one workgroup per row.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256)
void rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ g, T* __restrict__ y, int H, float eps) {
    const int m = blockIdx.x, tid = threadIdx.x;
    const T* xr = x + (size_t)m * H;
    float ss = 0.f;
    for (int k = tid; k < H; k += 256) { float v = ldf(xr + k); ss += v * v; }
    ss = wave_sum(ss);
    __shared__ float part[4];
    if ((tid & 63) == 0) part[tid >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float rstd = 1.0f / sqrtf(tot / (float)H + eps);
    T* yr = y + (size_t)m * H;
    for (int k = tid; k < H; k += 256) stf(yr + k, ldf(xr + k) * rstd * ldf(g + k));
}

// bf16 rows -> RMSNorm -> operand-order output (see packed_index).  g == nullptr: no
// normalisation, the row is only re-laid out.  H % 8 == 0.
__global__ __launch_bounds__(1024)
void rmsnorm_pack_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ g, bf16_t* __restrict__ y,
                         int H, float eps, int mt_count) {
    const int m = blockIdx.x, tid = threadIdx.x;
    const bf16x8* xr = reinterpret_cast<const bf16x8*>(x + (size_t)m * H);
    const int groups = H / 8;
    float rstd = 1.f;
    if (g) {
        float ss = 0.f;
        for (int k8 = tid; k8 < groups; k8 += 1024) {
            const bf16x8 v = xr[k8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float f = (float)v[e]; ss += f * f; }
        }
        ss = wave_sum(ss);
        __shared__ float part[16];
        if ((tid & 63) == 0) part[tid >> 6] = ss;
        __syncthreads();
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) tot += part[w];
        rstd = 1.0f / sqrtf(tot / (float)H + eps);
    }
    for (int k8 = tid; k8 < groups; k8 += 1024) {
        bf16x8 v = xr[k8];
        if (g) {
            const bf16x8 gv = reinterpret_cast<const bf16x8*>(g)[k8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = (bf16_t)((float)v[e] * rstd * (float)gv[e]);
        }
        *reinterpret_cast<bf16x8*>(y + packed_index(m, k8 * 8, mt_count)) = v;
    }
}

int launch_rmsnorm_packed(const void* x, const void* g, void* y, int M, int H, float eps, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_pack_kernel, dim3(M), dim3(1024), 0, st, (const bf16_t*)x, (const bf16_t*)g, (bf16_t*)y,
                       H, eps, (M + 15) / 16);
    return launch_status();
}

int launch_rmsnorm(const void* x, const void* g, void* y, int M, int H, float eps, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(M), dim3(256), 0, st, (const float*)x, (const float*)g, (float*)y, H, eps);
    return launch_status();
}

// Sum of one float per thread over a workgroup of at most 256 threads (every thread must call it).
__device__ inline float block_sum_256(float v, float* red /* [4] shared */) {
    v = wave_sum(v);
    __syncthreads();                                  // red may still be read from a previous call
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < (int)(blockDim.x + 63) / 64; ++w) t += red[w];
    return t;
}

// ---------------------------------------------------------------------------
// Rotary embedding + KV append.  grid = (M, n_q + 2 n_kv); thread j < d/2 owns
// the pair (j, j + d/2) of one head of one token.
// ---------------------------------------------------------------------------
__device__ inline size_t v_cache_index(size_t bg, int l_max, int d, int j, int c) {
    return ((bg * (size_t)(l_max / MASSV_V_BLOCK) + (size_t)(j / MASSV_V_BLOCK)) * d + c) * MASSV_V_BLOCK + (j % MASSV_V_BLOCK);
}

template <typename T>
__global__ void rope_append_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ pos,
                                   const int32_t* __restrict__ kv_len, T* __restrict__ q_out,
                                   T* __restrict__ k_cache, T* __restrict__ v_cache,
                                   const T* __restrict__ q_norm, const T* __restrict__ k_norm, float eps,
                                   int Q, int n_q, int n_kv, int d, int l_max, double log2_theta) {
    const int m = blockIdx.x, head = blockIdx.y, j = threadIdx.x;
    const int half = d / 2;
    const bool live = j < half;
    const int b = m / Q, i = m % Q;
    const int width = (n_q + 2 * n_kv) * d;
    const T* src = qkv + (size_t)m * width + (size_t)head * d;
    float x1 = live ? ldf(src + j) : 0.f, x2 = live ? ldf(src + j + half) : 0.f;
    const T* hn = head < n_q ? q_norm : head < n_q + n_kv ? k_norm : nullptr;
    if (hn) {                                            // uniform over the workgroup: RMSNorm of the head
        __shared__ float red[4];
        const float ss = block_sum_256(x1 * x1 + x2 * x2, red);
        const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
        if (live) { x1 *= rstd * ldf(hn + j); x2 *= rstd * ldf(hn + j + half); }
    }
    if (!live) return;
    int row = kv_len[b];
    row = (row < 0 ? 0 : row) + i;
    if (head < n_q + n_kv) {
        const double ang = (double)pos[m] * exp2(-2.0 * (double)j / (double)d * log2_theta);
        double sn, cs;
        sincos(ang, &sn, &cs);
        const float y1 = (float)((double)x1 * cs - (double)x2 * sn);
        const float y2 = (float)((double)x2 * cs + (double)x1 * sn);
        if (head < n_q) {
            T* dst = q_out + ((size_t)m * n_q + head) * d;
            stf(dst + j, y1); stf(dst + j + half, y2);
        } else if (row < l_max) {
            const int g = head - n_q;
            T* dst = k_cache + (((size_t)b * n_kv + g) * l_max + row) * d;
            stf(dst + j, y1); stf(dst + j + half, y2);
        }
    } else if (row < l_max) {
        const int g = head - n_q - n_kv;
        const size_t bg = (size_t)b * n_kv + g;
        stf(v_cache + v_cache_index(bg, l_max, d, row, j), x1);
        stf(v_cache + v_cache_index(bg, l_max, d, row, j + half), x2);
    }
}

int launch_rope_append(const void* qkv, const int32_t* pos, const int32_t* kv_len, void* q_out,
                       void* k_cache, void* v_cache, const void* q_norm, const void* k_norm, float eps,
                       const massv_attn_desc& a, float theta, hipStream_t st) {
    const int M = a.batch * a.n_query;
    dim3 grid(M, a.n_q_heads + 2 * a.n_kv_heads), block(a.head_dim / 2 < 64 ? 64 : a.head_dim / 2);
    const double l2t = log2((double)theta);
    if (a.dtype == MASSV_F32)
        hipLaunchKernelGGL(rope_append_kernel<float>, grid, block, 0, st, (const float*)qkv, pos, kv_len, (float*)q_out,
                           (float*)k_cache, (float*)v_cache, (const float*)q_norm, (const float*)k_norm, eps,
                           a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, l2t);
    else
        hipLaunchKernelGGL(rope_append_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)qkv, pos, kv_len, (bf16_t*)q_out,
                           (bf16_t*)k_cache, (bf16_t*)v_cache, (const bf16_t*)q_norm, (const bf16_t*)k_norm, eps,
                           a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, l2t);
    return launch_status();
}

// Prompt pass (paper Section 2.2): the same rotation and append for a block of L_q new positions per sequence, of
// which the first n_new[b] exist.  One, or three rotary position ids per row: with three (temporal, height, width,
// the numbering the Qwen2.5-VL family gives image positions) pair j turns by the id of the section it falls in --
// pairs [0, s_t) temporal, [s_t, s_th) height, the rest width -- at its own frequency theta^(-2j/d).
// grid = (B * L_q, n_q + 2 n_kv); thread j < d/2 owns the pair (j, j + d/2).  bf16 keys go to the blocked cache.
template <typename T>
__global__ void rope_rows_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ pos, int n_pos, size_t pos_stride,
                                 int s_t, int s_th, const int32_t* __restrict__ kv_len, const int32_t* __restrict__ n_new,
                                 T* __restrict__ q_out, T* __restrict__ k_cache, T* __restrict__ v_cache,
                                 const T* __restrict__ q_norm, const T* __restrict__ k_norm, float eps,
                                 int Lq, int n_q, int n_kv, int d, int l_max, double log2_theta) {
    const int m = blockIdx.x, head = blockIdx.y, j = threadIdx.x;
    const int half = d / 2;
    const bool live = j < half;
    const int b = m / Lq, i = m % Lq;
    int L0 = kv_len[b]; L0 = L0 < 0 ? 0 : L0;
    int n = n_new[b]; n = n < 0 ? 0 : (n > Lq ? Lq : n);
    if (L0 + n > l_max) n = l_max - L0 > 0 ? l_max - L0 : 0;
    if (i >= n) return;                                  // uniform over the workgroup
    const int width = (n_q + 2 * n_kv) * d;
    const T* src = qkv + (size_t)m * width + (size_t)head * d;
    float x1 = live ? ldf(src + j) : 0.f, x2 = live ? ldf(src + j + half) : 0.f;
    const T* hn = head < n_q ? q_norm : head < n_q + n_kv ? k_norm : nullptr;
    if (hn) {                                            // uniform over the workgroup: RMSNorm of the head
        __shared__ float red[4];
        const float ss = block_sum_256(x1 * x1 + x2 * x2, red);
        const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
        if (live) { x1 *= rstd * ldf(hn + j); x2 *= rstd * ldf(hn + j + half); }
    }
    if (!live) return;
    const int row = L0 + i;
    if (head < n_q + n_kv) {
        const int comp = n_pos == 1 ? 0 : (j < s_t ? 0 : j < s_th ? 1 : 2);
        const double ang = (double)pos[(size_t)comp * pos_stride + m] * exp2(-2.0 * (double)j / (double)d * log2_theta);
        double sn, cs;
        sincos(ang, &sn, &cs);
        const float y1 = (float)((double)x1 * cs - (double)x2 * sn);
        const float y2 = (float)((double)x2 * cs + (double)x1 * sn);
        if (head < n_q) {
            T* dst = q_out + ((size_t)m * n_q + head) * d;
            stf(dst + j, y1); stf(dst + j + half, y2);
        } else {
            const size_t bg = (size_t)b * n_kv + (head - n_q);
            if constexpr (sizeof(T) == 2) {
                stf(k_cache + k_cache_index(bg, l_max, d, row, j), y1);
                stf(k_cache + k_cache_index(bg, l_max, d, row, j + half), y2);
            } else {
                T* dst = k_cache + (bg * l_max + row) * d;
                stf(dst + j, y1); stf(dst + j + half, y2);
            }
        }
    } else {
        const size_t bg = (size_t)b * n_kv + (head - n_q - n_kv);
        stf(v_cache + v_cache_index(bg, l_max, d, row, j), x1);
        stf(v_cache + v_cache_index(bg, l_max, d, row, j + half), x2);
    }
}

// bf16 path: the q/k/v projection leaves fp32 partial sums per K slab; this kernel sums them, adds the
// bias, optionally normalises the query / key head, applies the rotary embedding and scatters q / k / v.
// Grid (heads, rows): consecutive workgroups read adjacent pieces of one row of partial sums (with rows as the
// fast index the 28-layer step measured 11 us slower).
__global__ void qkv_finish_kernel(const float* __restrict__ partial, int n_slabs, size_t slab_stride,
                                  const bf16_t* __restrict__ bq, const bf16_t* __restrict__ bk,
                                  const bf16_t* __restrict__ bv, const int32_t* __restrict__ pos,
                                  const int32_t* __restrict__ kv_len, bf16_t* __restrict__ q_out,
                                  bf16_t* __restrict__ k_cache, bf16_t* __restrict__ v_cache,
                                  const bf16_t* __restrict__ q_norm, const bf16_t* __restrict__ k_norm, float eps,
                                  int Q, int n_q, int n_kv, int d, int l_max, double log2_theta) {
    const int m = blockIdx.y, head = blockIdx.x, j = threadIdx.x;
    const int half = d / 2;
    const bf16_t* hn = head < n_q ? q_norm : head < n_q + n_kv ? k_norm : nullptr;
    if (j >= half && !hn) return;                        // with a head norm every thread reaches the block sum
    const bool live = j < half;
    const int b = m / Q, i = m % Q;
    const int width = (n_q + 2 * n_kv) * d;
    const size_t col = (size_t)head * d + (live ? j : 0);
    float x1 = 0.f, x2 = 0.f;
    for (int s0 = 0; s0 < n_slabs; s0 += 8) {           // 8 slabs' loads in flight at once; summed in slab order
        float t1[8], t2[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = s0 + u < n_slabs;
            const float* p = partial + (size_t)(ok ? s0 + u : 0) * slab_stride + (size_t)m * width + col;
            t1[u] = ok ? p[0] : 0.f; t2[u] = ok ? p[half] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) { x1 += t1[u]; x2 += t2[u]; }
    }
    const bf16_t* bias = head < n_q ? bq : head < n_q + n_kv ? bk : bv;
    if (bias && live) {
        const int hb = head < n_q ? head : head < n_q + n_kv ? head - n_q : head - n_q - n_kv;
        x1 += (float)bias[hb * d + j]; x2 += (float)bias[hb * d + j + half];
    }
    if (hn) {                                            // uniform over the workgroup: RMSNorm of the head
        __shared__ float red[4];
        if (!live) { x1 = 0.f; x2 = 0.f; }
        const float ss = block_sum_256(x1 * x1 + x2 * x2, red);
        const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
        if (!live) return;
        x1 *= rstd * (float)hn[j]; x2 *= rstd * (float)hn[j + half];
    }
    int row = kv_len[b];
    row = (row < 0 ? 0 : row) + i;
    if (head < n_q + n_kv) {
        const double ang = (double)pos[m] * exp2(-2.0 * (double)j / (double)d * log2_theta);
        double sn, cs;
        sincos(ang, &sn, &cs);
        const float y1 = (float)((double)x1 * cs - (double)x2 * sn);
        const float y2 = (float)((double)x2 * cs + (double)x1 * sn);
        if (head < n_q) {
            bf16_t* dst = q_out + ((size_t)m * n_q + head) * d;
            dst[j] = (bf16_t)y1; dst[j + half] = (bf16_t)y2;
        } else if (row < l_max) {
            const size_t bg = (size_t)b * n_kv + (head - n_q);
            k_cache[k_cache_index(bg, l_max, d, row, j)] = (bf16_t)y1;
            k_cache[k_cache_index(bg, l_max, d, row, j + half)] = (bf16_t)y2;
        }
    } else if (row < l_max) {
        const size_t bg = (size_t)b * n_kv + (head - n_q - n_kv);
        v_cache[v_cache_index(bg, l_max, d, row, j)] = (bf16_t)x1;
        v_cache[v_cache_index(bg, l_max, d, row, j + half)] = (bf16_t)x2;
    }
}

int launch_qkv_finish(const float* partial, int n_slabs, size_t slab_stride, const void* bq, const void* bk,
                      const void* bv, const int32_t* pos, const int32_t* kv_len, void* q_out, void* k_cache,
                      void* v_cache, const void* q_norm, const void* k_norm, float eps,
                      const massv_attn_desc& a, float theta, hipStream_t st) {
    const int M = a.batch * a.n_query;
    dim3 grid(a.n_q_heads + 2 * a.n_kv_heads, M), block(a.head_dim / 2 < 64 ? 64 : a.head_dim / 2);
    hipLaunchKernelGGL(qkv_finish_kernel, grid, block, 0, st, partial, n_slabs, slab_stride, (const bf16_t*)bq,
                       (const bf16_t*)bk, (const bf16_t*)bv, pos, kv_len, (bf16_t*)q_out, (bf16_t*)k_cache,
                       (bf16_t*)v_cache, (const bf16_t*)q_norm, (const bf16_t*)k_norm, eps,
                       a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, log2((double)theta));
    return launch_status();
}

// bf16 path: residual add of a projection's partial sums, optionally followed by RMSNorm into operand
// order.  One workgroup of 1024 threads per row; a thread owns one group of 8 consecutive features
// (H <= 8192), so a row's loads are all in flight at once.
constexpr int kFinishThreads = 1024;

// Sum of one float per thread over the kFinishThreads threads of a workgroup (every thread calls it).
__device__ inline float finish_block_sum(float v, float* part /* [kFinishThreads / kWave] shared */) {
    v = wave_sum(v);
    __syncthreads();                                  // part may still be read from a previous call
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kFinishThreads / kWave; ++w) tot += part[w];
    return tot;
}

// post != nullptr: the projection's output row is RMS-normalised with these gains before it is added.
// The row the sum is added to comes from h_in (fp32) when given, else from x (bf16); the result goes to h_out (fp32)
// when given, else to x (rounded to bf16).  A layer uses both: the stream between its attention block and its MLP
// block stays in fp32 (one rounding of the residual stream per layer, at the layer's output, instead of two).
__global__ __launch_bounds__(kFinishThreads)
void residual_finish_kernel(const float* __restrict__ partial, int n_slabs, size_t slab_stride,
                            bf16_t* __restrict__ x, const float* __restrict__ h_in, float* __restrict__ h_out,
                            const bf16_t* __restrict__ post, const bf16_t* __restrict__ ln,
                            bf16_t* __restrict__ xn, int H, float eps, int mt_count) {
    const int m = blockIdx.x, tid = threadIdx.x;
    const int k8 = tid;
    const bool live = k8 < H / 8;
    __shared__ float part[kFinishThreads / kWave];
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float add[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float ss = 0.f;
    if (live) {
        if (h_in) {
            const floatx4* hp = reinterpret_cast<const floatx4*>(h_in + (size_t)m * H + k8 * 8);
            const floatx4 a = hp[0], b = hp[1];
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
        } else {
            const bf16x8 xv = *reinterpret_cast<const bf16x8*>(x + (size_t)m * H + k8 * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = (float)xv[e];
        }
        for (int s0 = 0; s0 < n_slabs; s0 += 8) {              // 8 slabs' loads in flight at once; summed in slab order
            floatx4 p0[8], p1[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool ok = s0 + u < n_slabs;
                const floatx4* p = reinterpret_cast<const floatx4*>(partial + (size_t)(ok ? s0 + u : 0) * slab_stride +
                                                                    (size_t)m * H + k8 * 8);
                p0[u] = ok ? p[0] : floatx4{0.f, 0.f, 0.f, 0.f};
                p1[u] = ok ? p[1] : floatx4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) { add[e] += p0[u][e]; add[4 + e] += p1[u][e]; }
        }
    }
    if (post) {                                                // uniform over the grid
        float sy = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sy += add[e] * add[e];
        const float rstd_y = 1.0f / sqrtf(finish_block_sum(sy, part) / (float)H + eps);
        if (live) {
            const bf16x8 gv = *reinterpret_cast<const bf16x8*>(post + k8 * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) add[e] *= rstd_y * (float)gv[e];
        }
    }
    if (live) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { v[e] += add[e]; ss += v[e] * v[e]; }
        if (h_out) {
            floatx4* hp = reinterpret_cast<floatx4*>(h_out + (size_t)m * H + k8 * 8);
            hp[0] = floatx4{v[0], v[1], v[2], v[3]};
            hp[1] = floatx4{v[4], v[5], v[6], v[7]};
        } else {
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[e];
            *reinterpret_cast<bf16x8*>(x + (size_t)m * H + k8 * 8) = o;
        }
    }
    if (!ln) return;
    const float rstd = 1.0f / sqrtf(finish_block_sum(ss, part) / (float)H + eps);
    if (live) {
        const bf16x8 gv = *reinterpret_cast<const bf16x8*>(ln + k8 * 8);
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)(v[e] * rstd * (float)gv[e]);
        *reinterpret_cast<bf16x8*>(xn + packed_index(m, k8 * 8, mt_count)) = o;
    }
}

int launch_residual_finish(const float* partial, int n_slabs, size_t slab_stride, void* x, const float* h_in, float* h_out,
                           const void* post, const void* ln, void* xn_packed, int M, int H, float eps, hipStream_t st) {
    if (H % 8 || H > 8 * kFinishThreads) return MASSV_EUNSUPPORTED;
    hipLaunchKernelGGL(residual_finish_kernel, dim3(M), dim3(kFinishThreads), 0, st, partial, n_slabs, slab_stride,
                       (bf16_t*)x, h_in, h_out, (const bf16_t*)post, (const bf16_t*)ln, (bf16_t*)xn_packed, H, eps, (M + 15) / 16);
    return launch_status();
}

// fp32 path: x += rmsnorm(y, g) row by row (the block-output norm); one workgroup per row.
__global__ __launch_bounds__(256)
void postnorm_residual_kernel(float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g,
                              int H, float eps) {
    const int m = blockIdx.x, tid = threadIdx.x;
    const float* yr = y + (size_t)m * H;
    float ss = 0.f;
    for (int k = tid; k < H; k += 256) ss += yr[k] * yr[k];
    __shared__ float red[4];
    const float rstd = 1.0f / sqrtf(block_sum_256(ss, red) / (float)H + eps);
    for (int k = tid; k < H; k += 256) x[(size_t)m * H + k] += yr[k] * rstd * g[k];
}

int launch_postnorm_residual(void* x, const void* y, const void* g, int M, int H, float eps, hipStream_t st) {
    hipLaunchKernelGGL(postnorm_residual_kernel, dim3(M), dim3(256), 0, st, (float*)x, (const float*)y, (const float*)g, H, eps);
    return launch_status();
}

// ---------------------------------------------------------------------------
// Row-major values -> blocked value cache.  One thread per destination element
// (writes coalesced).
// ---------------------------------------------------------------------------
template <typename T>
__global__ void v_pack_kernel(const T* __restrict__ src, T* __restrict__ dst, size_t total, int l_max, int d) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total) return;
    const int jj = (int)(o % MASSV_V_BLOCK);
    const size_t t1 = o / MASSV_V_BLOCK;
    const int c = (int)(t1 % d);
    const size_t t2 = t1 / d;
    const int blk = (int)(t2 % (l_max / MASSV_V_BLOCK));
    const size_t bg = t2 / (l_max / MASSV_V_BLOCK);
    const int j = blk * MASSV_V_BLOCK + jj;
    dst[o] = src[(bg * l_max + j) * d + c];
}

// Row-major bf16 W[N][K] -> streaming layout: one thread per 16-byte destination chunk.
__global__ void weight_pack_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, size_t chunks, int K) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= chunks) return;
    const int lane = (int)(o % 64);
    const size_t t2 = o / 64;
    const int ksteps = K / 32;
    const int ks = (int)(t2 % ksteps);
    const size_t tile = t2 / ksteps;
    const size_t n = tile * 16 + (lane % 16);
    const int k = ks * 32 + (lane / 16) * 8;
    *reinterpret_cast<bf16x8*>(dst + o * 8) = *reinterpret_cast<const bf16x8*>(src + n * K + k);
}

// Embedding rows gathered as 4-byte words: one workgroup per output row.
__global__ __launch_bounds__(256)
void embed_tokens_kernel(const uint32_t* __restrict__ table, const int* __restrict__ tokens,
                         uint32_t* __restrict__ x, int words, int V) {
    const int m = blockIdx.x, tok = tokens[m];
    const bool ok = tok >= 0 && tok < V;
    const uint32_t* src = table + (size_t)(ok ? tok : 0) * words;
    uint32_t* dst = x + (size_t)m * words;
    for (int i = threadIdx.x; i < words; i += blockDim.x) dst[i] = ok ? src[i] : 0u;
}

}  // namespace massv

using namespace massv;

extern "C" int massv_rope_append(const massv_attn_desc* desc, const void* qkv, const int32_t* pos, int32_t n_pos,
                                 const int32_t* sections, float rope_theta, const void* q_norm, const void* k_norm,
                                 float norm_eps, const int32_t* kv_len, const int32_t* n_new, void* q_out,
                                 void* k_cache, void* v_cache, void* stream) {
    if (!desc) return MASSV_EINVAL;
    // the descriptor rules of verify_attention, except that the row count per KV head is not limited
    massv_attn_desc one = *desc;
    one.n_query = 1;
    const int rc = check_attn_desc(&one);
    if (rc != MASSV_OK) return rc;
    if (desc->n_query < 1 || desc->n_query > desc->l_max) return MASSV_EINVAL;
    if (!qkv || !pos || !kv_len || !n_new || !q_out || !k_cache || !v_cache) return MASSV_EINVAL;
    if (!(rope_theta > 0.f) || isinf(rope_theta) || !(norm_eps >= 0.f)) return MASSV_EINVAL;
    if (n_pos != 1 && n_pos != 3) return MASSV_EINVAL;
    int s_t = 0, s_th = 0;
    if (n_pos == 3) {
        if (!sections) return MASSV_EINVAL;
        if (sections[0] < 0 || sections[1] < 0 || sections[2] < 0) return MASSV_EINVAL;
        if ((int64_t)sections[0] + sections[1] + sections[2] != desc->head_dim / 2) return MASSV_EINVAL;
        s_t = sections[0]; s_th = sections[0] + sections[1];
    }
    const massv_attn_desc& a = *desc;
    if (a.head_dim > 512) return MASSV_EUNSUPPORTED;
    const int64_t M = (int64_t)a.batch * a.n_query;
    if (M > 0x7fffffff || a.n_q_heads + 2 * a.n_kv_heads > 65535) return MASSV_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)M, a.n_q_heads + 2 * a.n_kv_heads), block(a.head_dim / 2 < 64 ? 64 : a.head_dim / 2);
    const double l2t = log2((double)rope_theta);
    if (a.dtype == MASSV_F32)
        hipLaunchKernelGGL(rope_rows_kernel<float>, grid, block, 0, st, (const float*)qkv, pos, n_pos, (size_t)M, s_t, s_th,
                           kv_len, n_new, (float*)q_out, (float*)k_cache, (float*)v_cache, (const float*)q_norm,
                           (const float*)k_norm, norm_eps, a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, l2t);
    else
        hipLaunchKernelGGL(rope_rows_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)qkv, pos, n_pos, (size_t)M, s_t, s_th,
                           kv_len, n_new, (bf16_t*)q_out, (bf16_t*)k_cache, (bf16_t*)v_cache, (const bf16_t*)q_norm,
                           (const bf16_t*)k_norm, norm_eps, a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, l2t);
    return launch_status();
}

extern "C" int massv_rmsnorm(const void* x, const void* gain, void* y, int32_t M, int32_t H, float eps, int32_t dtype,
                             void* stream) {
    if (!x || !gain || !y || M < 1 || H < 1 || !(eps >= 0.f)) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MASSV_F32)
        hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(M), dim3(256), 0, st, (const float*)x, (const float*)gain, (float*)y, H, eps);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(M), dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)gain, (bf16_t*)y, H, eps);
    return launch_status();
}

extern "C" int massv_embed_tokens(const void* table, const int32_t* tokens, void* x,
                                  int32_t M, int32_t H, int32_t V, int32_t dtype, void* stream) {
    if (!table || !tokens || !x || M < 1 || H < 1 || V < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    const size_t row_bytes = (size_t)H * (dtype == MASSV_F32 ? 4 : 2);
    if (row_bytes % 4) return MASSV_EUNSUPPORTED;
    hipLaunchKernelGGL(embed_tokens_kernel, dim3(M), dim3(256), 0, (hipStream_t)stream,
                       (const uint32_t*)table, tokens, (uint32_t*)x, (int)(row_bytes / 4), V);
    return launch_status();
}

extern "C" int massv_weight_pack(const void* src, void* dst, int32_t N, int32_t K, int32_t dtype, void* stream) {
    if (!src || !dst || N < 1 || K < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MASSV_F32)
        return hipMemcpyAsync(dst, src, (size_t)N * K * 4, hipMemcpyDeviceToDevice, st) == hipSuccess ? MASSV_OK : MASSV_ELAUNCH;
    if (N % 16 || K % 32) return MASSV_EUNSUPPORTED;
    const size_t chunks = (size_t)N * K / 8;
    const size_t blocks = (chunks + 255) / 256;
    if (blocks > 0x7fffffffu) return MASSV_EUNSUPPORTED;
    hipLaunchKernelGGL(weight_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t*)src, (bf16_t*)dst, chunks, K);
    return launch_status();
}

// Row-major keys -> blocked bf16 key cache; one thread per destination element.
__global__ void k_pack_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, size_t total, int l_max, int d) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total) return;
    const size_t per_block = (size_t)32 * d;
    const size_t blk_all = o / per_block;                       // block index over all (b, g)
    const int r = (int)(o % per_block);
    const int e = r & 7, slot = (r >> 3) & 15, chunk_all = r >> 7;              // chunk_all = half * (d/8) + chunk
    const int half = chunk_all / (d >> 3), chunk = chunk_all % (d >> 3);
    const int jj = (slot >> 2) * 8 + half * 4 + (slot & 3);
    dst[o] = src[(blk_all * 32 + jj) * d + chunk * 8 + e];      // blocks of one (b, g) are consecutive in both
}

extern "C" int massv_k_cache_pack(const void* src, void* dst, int32_t batch, int32_t n_kv_heads,
                                  int32_t l_max, int32_t head_dim, int32_t dtype, void* stream) {
    if (!src || !dst || batch < 1 || n_kv_heads < 1 || l_max < 1 || head_dim < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    const size_t total = (size_t)batch * n_kv_heads * l_max * head_dim;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MASSV_F32) {
        if (hipMemcpyAsync(dst, src, total * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return MASSV_ELAUNCH;
        return MASSV_OK;
    }
    if (l_max % 32 || head_dim % 8) return MASSV_EINVAL;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffu) return MASSV_EUNSUPPORTED;
    hipLaunchKernelGGL(k_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t*)src, (bf16_t*)dst, total, l_max, head_dim);
    return launch_status();
}

extern "C" int massv_v_cache_pack(const void* src, void* dst, int32_t batch, int32_t n_kv_heads,
                                  int32_t l_max, int32_t head_dim, int32_t dtype, void* stream) {
    if (!src || !dst || batch < 1 || n_kv_heads < 1 || l_max < 1 || head_dim < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    if (l_max % MASSV_V_BLOCK) return MASSV_EINVAL;
    const size_t total = (size_t)batch * n_kv_heads * l_max * head_dim;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffu) return MASSV_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MASSV_F32)
        hipLaunchKernelGGL(v_pack_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)src, (float*)dst, total, l_max, head_dim);
    else
        hipLaunchKernelGGL(v_pack_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t*)src, (bf16_t*)dst, total, l_max, head_dim);
    return launch_status();
}
