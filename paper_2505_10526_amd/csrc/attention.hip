// verify_attention: grouped-query causal attention of the Q = gamma+1 new
// positions over the KV cache (paper Section 2.1: one parallel forward scores
// every drafted position; query i sees cache rows [0, kv_len + i]).
//
// bf16 path (the one that matters): the cost is one pass over the cached K and
// V of every (sequence, KV head), so the kernel is built as an HBM stream.
//   * The G*Q query rows that share a KV head are stacked as the 16-row tiles
//     of the matrix instruction, so each K / V element is fetched once for all
//     of them (G*Q = 42 for 28/4 heads and gamma = 5).
//   * Scores are formed transposed, S^T = K Q^T with v_mfma_f32_16x16x32_bf16:
//     the A operand is a 16-key x 32-dim tile of K that every lane loads
//     straight from HBM with one 16-byte load -- the key cache is stored in
//     that operand order, so a wave's load is one contiguous 1 KB and can
//     carry the non-temporal hint (with row-major keys a load touched 16 half
//     lines: 93.4 -> 91.1 us on the 8192-key shape) -- the B operand is Q held
//     in registers for the whole kernel.  The result leaves each lane holding, for
//     one query row, 4 consecutive keys of the 32-key block per instruction.
//     Choosing the 16 keys of a tile as {8c + 4t + i} makes the two tiles of a
//     block hand lane group c exactly keys 8c..8c+7 -- the operand order the
//     second product needs -- so probabilities never move between lanes.
//   * O^T += V^T P^T takes V^T tiles (16 dims x 32 keys) as the A operand.  The
//     value cache stores each block of 32 keys dim-major, so that tile is again
//     one 16-byte load per lane, contiguous over the wave.  No LDS staging and
//     no transposes are needed; LDS is used only to merge the waves of a
//     workgroup at the end.
//   * A workgroup (4 waves) owns one (sequence, KV head, split of the key
//     range); its waves take 32-key blocks round-robin, keep a running
//     (max, sum, O) in registers with the usual streaming softmax, and are
//     merged through LDS.  Splits are merged by a second small kernel in fixed
//     order.  Only the blocks holding the new positions pay for the causal
//     mask.
// f32 path: a plain one-workgroup-per-(b, head, query) kernel for the small
// fp32 configuration.
#include "kernels.h"

#include <atomic>

namespace massv {

constexpr int kAttnWaves = 4;
constexpr int kAttnThreads = kAttnWaves * kWave;
constexpr int kBlk = MASSV_V_BLOCK;            // keys per block

__device__ inline size_t v_index(size_t bg, int l_max, int d, int j, int c) {
    return ((bg * (size_t)(l_max / kBlk) + (size_t)(j / kBlk)) * d + c) * kBlk + (j % kBlk);
}

__device__ inline int clamp_total(int kv_len, int Q, int l_max) {
    int n = (kv_len < 0 ? 0 : kv_len) + Q;
    return n > l_max ? l_max : n;
}

// ---------------------------------------------------------------------------
// generic kernel (any dtype, any d <= 256): grid (Q, n_q, B), 256 threads.
// Keys are taken 256 at a time: thread t scores key t, the tile's weights go
// through LDS, thread c accumulates output column c.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256)
void attention_generic_kernel(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
                              const int32_t* __restrict__ kv_len, T* __restrict__ out,
                              int Q, int n_q, int n_kv, int d, int l_max, float scale, int window) {
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int G = n_q / n_kv, g = h / G;
    const size_t bg = (size_t)b * n_kv + g;
    int L = kv_len[b]; L = L < 0 ? 0 : L;
    int n_vis = L + i + 1;
    if (n_vis > l_max) n_vis = l_max;
    const int lo = (window > 0 && n_vis > window) ? n_vis - window : 0;      // first row of the sliding window
    __shared__ float qs[256];
    __shared__ float w[256];
    __shared__ float red[4];
    const T* qr = q + (((size_t)b * Q + i) * n_q + h) * d;
    if (tid < d) qs[tid] = ldf(qr + tid);
    __syncthreads();
    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
    for (int j0 = lo; j0 < n_vis; j0 += 256) {
        const int j = j0 + tid;
        float s = -INFINITY;
        if (j < n_vis) {
            const T* kr = kc + (bg * l_max + j) * d;
            float dot = 0.f;
            for (int c = 0; c < d; ++c) dot += qs[c] * ldf(kr + c);
            s = dot * scale;
        }
        float mx = wave_max(s);
        if ((tid & 63) == 0) red[tid >> 6] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float m_new = fmaxf(m_run, mx);                 // finite: key j0 is visible
        const float p = (j < n_vis) ? expf(s - m_new) : 0.f;
        w[tid] = p;
        float ps = wave_sum(p);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = ps;
        __syncthreads();
        ps = red[0] + red[1] + red[2] + red[3];
        const float alpha = expf(m_run - m_new);
        l_run = l_run * alpha + ps;
        acc *= alpha;
        if (tid < d) {
            const int cnt = (n_vis - j0) < 256 ? (n_vis - j0) : 256;
            for (int t = 0; t < cnt; ++t) acc += w[t] * ldf(vc + v_index(bg, l_max, d, j0 + t, tid));
        }
        m_run = m_new;
        __syncthreads();
    }
    if (tid < d) stf(out + (((size_t)b * Q + i) * n_q + h) * d + tid, acc / l_run);
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.
// ---------------------------------------------------------------------------
// Two merge buffers of [16 MT][D + 4] floats (plus the small per-wave tables) within the 160 KB of LDS of a CU?
// (Always, for the tile shapes built; above 64 KB the kernel's limit is raised once per device.)
__host__ __device__ constexpr bool attn_tree_merge(int D, int MT) {
    return 2 * MT * 16 * (D + 4) * (int)sizeof(float) + 4096 <= 160 * 1024;
}

__device__ inline float xor16_max(float v) {        // over the 4 lane groups that share a query row
    v = fmaxf(v, __shfl_xor(v, 16, kWave));
    return fmaxf(v, __shfl_xor(v, 32, kWave));
}
__device__ inline float xor16_sum(float v) {
    v += __shfl_xor(v, 16, kWave);
    return v + __shfl_xor(v, 32, kWave);
}

struct AttnParams {
    const bf16_t* q; const bf16_t* kc; const bf16_t* vc; const int32_t* kv_len;
    bf16_t* out;                 // used when n_split == 1
    float* part_o; float* part_ml;   // [B][n_kv][S][rows_pad][D], [B][n_kv][S][rows_pad][2]
    int Q, n_q, n_kv, l_max, n_split;
    int window;                  // 0: all rows; W > 0: a query at row r sees rows r-W+1 .. r
    int out_mt;                  // > 0: out is written in operand order with this many row tiles
    float scale_log2;            // scale * log2(e)
};

template <int D, int MT>
__global__ __launch_bounds__(kAttnThreads)
void attention_mfma_kernel(AttnParams p) {
    // Two K/V register sets (the next block's loads fly while this one is used) only where they fit:
    // with 3-4 row tiles at d = 128 a second set (or even a second K set alone) cost more in register
    // shuffling than it hid -- the plain loop measured 95 us, K double-buffering 101 us, full double
    // buffering 124 us on the 56-row, 8192-key shape.
    constexpr bool PREFETCH = (D * MT <= 256) && (D <= 128);
    constexpr int KS = D / 32;          // k-steps of the score product
    constexpr int NT = D / 16;          // 16-dim tiles of the output
    constexpr int ROWS = MT * 16;
    constexpr int LDS_STRIDE = D + 4;   // floats per row in the merge buffer (keeps float4 stores conflict-light)
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int lr = lane % 16, lc = lane / 16;
    const int G = p.n_q / p.n_kv, rows = G * p.Q;
    const size_t bg = (size_t)b * p.n_kv + g;
    int L = p.kv_len[b]; L = L < 0 ? 0 : L;
    const int n_total = clamp_total(L, p.Q, p.l_max);
    const int n_blocks = (n_total + kBlk - 1) / kBlk;
    // sliding window: the first query (row L) sees rows from L-W+1 on and later queries start higher, so
    // blocks below that row are skipped altogether; blocks that hold a row below the LAST query's window
    // start (row L+Q-W) need the lower mask
    const int W = p.window;
    const int blk_lo = (W > 0 && L + 1 > W) ? (L + 1 - W) / kBlk : 0;
    const int low_mask_end = (W > 0) ? L + p.Q - W : 0;         // rows below it are outside some query's window
    const int per = (n_blocks - blk_lo + p.n_split - 1) / p.n_split;
    const int blk_begin = blk_lo + split * per;
    const int blk_end = (blk_begin + per < n_blocks) ? blk_begin + per : n_blocks;
    const int first_masked_blk = L / kBlk;      // blocks before it hold cached positions only

    // ---- Q operand: lane (lr, lc) holds Q[row = 16 mt + lr][32 ks + 8 lc .. +8] ----
    // (kept in registers for the whole kernel; operand tiles in LDS measured no gain)
    extern __shared__ float s_dyn[];             // [ROWS][LDS_STRIDE] merge buffer(s)
    bf16x8 qreg[MT][KS];
    int qi[MT];                                 // query position of this lane's row in tile mt (clamped)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r = mt * 16 + lr;
        const int i = r / G, hh = r % G;
        qi[mt] = i < p.Q ? i : p.Q - 1;
        const bf16_t* qr = p.q + (((size_t)b * p.Q + (i < p.Q ? i : 0)) * p.n_q + g * G + hh) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (r < rows) v = *reinterpret_cast<const bf16x8*>(qr + ks * 32 + lc * 8);
            qreg[mt][ks] = v;
        }
    }

    floatx4 acc[MT][NT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY; l_run[mt] = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const bf16_t* kbase = p.kc + bg * (size_t)p.l_max * D;
    const bf16_t* vbase = p.vc + bg * (size_t)p.l_max * D;

    // ---- loads of one 32-key block: K tile t holds keys {8c + 4t + i}; lane lr = 4c + i.  The key cache keeps
    // each (tile, k-step) operand as 64 consecutive 16-byte pieces in lane order (k_cache_index) ----
    auto load_k = [&](int blk, bf16x8 (&kreg)[2][KS]) {
        const bf16_t* kb = kbase + (size_t)blk * kBlk * D + lane * 8;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kreg[t][ks] = ldg_stream(reinterpret_cast<const bf16x8*>(kb + (t * KS + ks) * 512));
    };
    auto load_v = [&](int blk, bf16x8 (&vreg)[NT]) {
        const bf16_t* vb = vbase + (size_t)blk * D * kBlk + lc * 8;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            vreg[nt] = ldg_stream(reinterpret_cast<const bf16x8*>(vb + (size_t)(nt * 16 + lr) * kBlk));
    };
    auto load_block = [&](int blk, bf16x8 (&kreg)[2][KS], bf16x8 (&vreg)[NT]) {
        load_k(blk, kreg);
        load_v(blk, vreg);
    };

    // One 32-key block.  Instruction count matters here: at 56-64 stacked rows the kernel was issuing
    // VALU / MFMA instructions half of the time.  Hence
    //   * all score products first, k-step outermost, so the 2*MT accumulators form independent chains;
    //   * the exponent uses ONE fma per score (s*c - m) and the raw v_exp_f32;
    //   * the running reference exponent m of a row is only raised when the block's maximum exceeds it
    //     by more than kLazy (probabilities then stay <= 2^kLazy, harmless in bf16 / fp32): the common
    //     block needs no cross-lane maximum and no rescaling of the output accumulators.  The result
    //     acc / l does not depend on which reference is used.
    constexpr float kLazy = 8.0f;
    // Score product of one block: S^T tile pairs, lane holds keys 8 lc + (0..7) of query row 16 mt + lr.
    auto block_scores = [&](bf16x8 (&kreg)[2][KS], floatx4 (&s0)[MT], floatx4 (&s1)[MT]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { s0[mt] = floatx4{0.f, 0.f, 0.f, 0.f}; s1[mt] = floatx4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 qv = qreg[mt][ks];
                s0[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[0][ks], qv, s0[mt], 0, 0, 0);
                s1[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[1][ks], qv, s1[mt], 0, 0, 0);
            }
    };
    // Mask, streaming softmax and O^T += V^T P^T of one block, from its scores.
    auto block_finish = [&](int blk, floatx4 (&s0)[MT], floatx4 (&s1)[MT], bf16x8 (&vreg)[NT]) {
        const bool tail = (blk + 1) * kBlk > n_total;         // block reaches past the valid rows
        if (tail) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (blk * kBlk + lc * 8 + e >= n_total) vreg[nt][e] = (bf16_t)0.f;
        }
        const bool masked = blk >= first_masked_blk || blk * kBlk < low_mask_end;

        bf16x8 pv[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float sv[8] = {s0[mt][0], s0[mt][1], s0[mt][2], s0[mt][3], s1[mt][0], s1[mt][1], s1[mt][2], s1[mt][3]};
            if (masked) {
                const int last_visible = L + qi[mt];
                const int first_visible = W > 0 ? last_visible - W + 1 : 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = blk * kBlk + lc * 8 + e;
                    if (key > last_visible || key < first_visible) sv[e] = -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
            mx *= p.scale_log2;                                // scale > 0: the maximum commutes with it
            if (__any(mx > m_run[mt] + kLazy)) {               // some row of this tile needs a new reference
                mx = xor16_max(mx);
                if (mx > m_run[mt] + kLazy) {
                    const float alpha = __builtin_amdgcn_exp2f(m_run[mt] - mx);     // m_run = -inf gives 0
                    l_run[mt] *= alpha;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] *= alpha;
                    m_run[mt] = mx;
                }
            }
            const float neg_m = (m_run[mt] == -INFINITY) ? 0.f : -m_run[mt];
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(sv[e], p.scale_log2, neg_m));
                ps += pe;
                pv[mt][e] = (bf16_t)pe;
            }
            l_run[mt] += ps;
        }
        // ---- O^T += V^T P^T ----
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vreg[nt], pv[mt], acc[mt][nt], 0, 0, 0);
    };

    auto process_block = [&](int blk, bf16x8 (&kreg)[2][KS], bf16x8 (&vreg)[NT]) {
        floatx4 s0[MT], s1[MT];
        block_scores(kreg, s0, s1);
        block_finish(blk, s0, s1, vreg);
    };

    // The wave's blocks are blk_begin + wave, + 4, ...; the loads of the next one are in flight while
    // the current one is processed (two register sets), unless the tile shape leaves no registers.
    if constexpr (PREFETCH) {
        bf16x8 kc[2][KS], vc[NT], kn[2][KS], vn[NT];
        int blk = blk_begin + wave;
        if (blk < blk_end) load_block(blk, kc, vc);
#pragma unroll 1
        for (; blk < blk_end; blk += kAttnWaves) {
            const int nb = blk + kAttnWaves;
            if (nb < blk_end) load_block(nb, kn, vn);
            process_block(blk, kc, vc);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kc[t][ks] = kn[t][ks];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) vc[nt] = vn[nt];
        }
    } else if constexpr (D <= 128) {
        // One register set, refilled in halves: the key registers are free once the scores are formed, so the next
        // block's keys are requested before the softmax and the second product; its values right after that
        // (long-context shape 91.9 -> 90.9 us; at d = 256 the longer live ranges spill, so that shape keeps the
        // plain loop below).
        bf16x8 k0[2][KS], v0[NT];
        int blk = blk_begin + wave;
        if (blk < blk_end) load_block(blk, k0, v0);
        for (; blk < blk_end; blk += kAttnWaves) {
            const int nb = blk + kAttnWaves;
            floatx4 s0[MT], s1[MT];
            block_scores(k0, s0, s1);
            if (nb < blk_end) load_k(nb, k0);
            block_finish(blk, s0, s1, v0);
            if (nb < blk_end) load_v(nb, v0);
        }
    } else {
        bf16x8 k0[2][KS], v0[NT];
        for (int blk = blk_begin + wave; blk < blk_end; blk += kAttnWaves) {
            load_block(blk, k0, v0);
            process_block(blk, k0, v0);
        }
    }

    // ---- merge the waves of the workgroup ----
    __shared__ float s_m[kAttnWaves][ROWS];
    __shared__ float s_l[kAttnWaves][ROWS];
    __shared__ float s_lt[ROWS];
    float* s_o = s_dyn;                          // [ROWS][LDS_STRIDE]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const float l = xor16_sum(l_run[mt]);
        if (lc == 0) { s_m[wave][mt * 16 + lr] = m_run[mt]; s_l[wave][mt * 16 + lr] = l; }
    }
    __syncthreads();
    float m_tot[MT], l_tot[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r = mt * 16 + lr;
        float m = s_m[0][r];
#pragma unroll
        for (int w = 1; w < kAttnWaves; ++w) m = fmaxf(m, s_m[w][r]);
        const float m_safe = (m == -INFINITY) ? 0.f : m;
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) l += s_l[w][r] * exp2f(s_m[w][r] - m_safe);
        const float f = exp2f(m_run[mt] - m_safe);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] *= f;
        m_tot[mt] = m; l_tot[mt] = l;
        if (wave == 0 && lc == 0) s_lt[r] = l;
    }
    // Where two merge buffers fit in LDS the four waves are summed as (w0 + w2) + (w1 + w3): waves 0 and 1 store
    // side by side, waves 2 and 3 add to them side by side, the readers below add the two buffers.  (One buffer with
    // the waves taking turns took 3.6 us of an 11 us launch.)  Otherwise the waves add into one buffer in turn.
    constexpr bool TREE = attn_tree_merge(D, MT);
    float* s_o2 = s_o + ROWS * LDS_STRIDE;
    auto merge_store = [&](float* buf, bool add) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float* dst = buf + (mt * 16 + lr) * LDS_STRIDE + nt * 16 + lc * 4;
                floatx4 v = acc[mt][nt];
                if (add) v += *reinterpret_cast<floatx4*>(dst);
                *reinterpret_cast<floatx4*>(dst) = v;
            }
    };
    if constexpr (TREE) {
        if (wave < 2) merge_store(wave == 0 ? s_o : s_o2, false);
        __syncthreads();
        if (wave >= 2) merge_store(wave == 2 ? s_o : s_o2, true);
        __syncthreads();
    } else {
        for (int w = 0; w < kAttnWaves; ++w) {
            if (wave == w) merge_store(s_o, w > 0);
            __syncthreads();
        }
    }
    auto merged = [&](int r, int c4) -> floatx4 {
        floatx4 v = *reinterpret_cast<const floatx4*>(s_o + r * LDS_STRIDE + c4 * 4);
        if constexpr (TREE) v += *reinterpret_cast<const floatx4*>(s_o2 + r * LDS_STRIDE + c4 * 4);
        return v;
    };

    // ---- write: final output if there is one split, else the partial ----
    if (p.n_split == 1) {
        for (int idx = tid; idx < rows * (D / 4); idx += kAttnThreads) {
            const int r = idx / (D / 4), c4 = idx % (D / 4);
            const int i = r / G, hh = r % G;
            const floatx4 v = merged(r, c4);
            const float inv = 1.0f / s_lt[r];
            bf16x4 o = {(bf16_t)(v[0] * inv), (bf16_t)(v[1] * inv), (bf16_t)(v[2] * inv), (bf16_t)(v[3] * inv)};
            const int mrow = b * p.Q + i, col = (g * G + hh) * D + c4 * 4;
            bf16_t* dst = p.out_mt > 0 ? p.out + packed_index(mrow, col, p.out_mt)
                                       : p.out + (size_t)mrow * p.n_q * D + col;
            *reinterpret_cast<bf16x4*>(dst) = o;
        }
    } else {
        const size_t slot = (bg * p.n_split + split) * ROWS;
        for (int idx = tid; idx < rows * (D / 4); idx += kAttnThreads) {
            const int r = idx / (D / 4), c4 = idx % (D / 4);
            *reinterpret_cast<floatx4*>(p.part_o + (slot + r) * D + c4 * 4) = merged(r, c4);
        }
        if (wave == 0 && lc == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float* ml = p.part_ml + (slot + mt * 16 + lr) * 2;
                ml[0] = m_tot[mt]; ml[1] = l_tot[mt];
            }
        }
    }
}

// Merge of the key-range splits.  D/4 threads own one output row (4 features each); a 128-thread
// workgroup handles 512/D rows (64, 256 and 512 threads measured 2-6 us slower per 28-layer step).  Splits are taken 8 at a time with all their loads in flight, in split
// order (deterministic).
constexpr int kCombineThreads = 128;
template <int D>
__global__ __launch_bounds__(kCombineThreads)
void attention_combine_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                              bf16_t* __restrict__ out, int Q, int n_q, int n_kv, int n_split, int rows_pad,
                              int out_mt, int total_rows) {
    constexpr int TPR = D / 4;                       // threads per row
    const int row_id = blockIdx.x * (kCombineThreads / TPR) + threadIdx.x / TPR, t = threadIdx.x % TPR;
    if (row_id >= total_rows) return;
    const int h = row_id % n_q, i = (row_id / n_q) % Q, b = row_id / (n_q * Q);
    const int G = n_q / n_kv, g = h / G, r = i * G + (h % G);
    const size_t slot0 = ((size_t)b * n_kv + g) * n_split * rows_pad;
    float m = -INFINITY, l = 0.f;
    floatx4 o = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < n_split; s0 += 8) {
        float ms[8], ls[8];
        floatx4 os[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = s0 + u < n_split;
            const size_t row = slot0 + (size_t)(ok ? s0 + u : 0) * rows_pad + r;
            ms[u] = ok ? part_ml[row * 2] : -INFINITY;
            ls[u] = ok ? part_ml[row * 2 + 1] : 0.f;
            os[u] = *reinterpret_cast<const floatx4*>(part_o + row * D + t * 4);
        }
        float mb = m;
#pragma unroll
        for (int u = 0; u < 8; ++u) mb = fmaxf(mb, ms[u]);
        if (mb == -INFINITY) continue;               // no split so far saw a visible key for this row
        const float keep = exp2f(m - mb);             // m = -inf gives 0
        l *= keep; o *= keep; m = mb;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (ms[u] == -INFINITY) continue;         // that split's sums may be uninitialised
            const float w = exp2f(ms[u] - m);
            l += ls[u] * w;
            o += os[u] * w;
        }
    }
    const float inv = 1.0f / l;
    bf16x4 ob = {(bf16_t)(o[0] * inv), (bf16_t)(o[1] * inv), (bf16_t)(o[2] * inv), (bf16_t)(o[3] * inv)};
    const int mrow = b * Q + i, col = h * D + t * 4;
    bf16_t* dst = out_mt > 0 ? out + packed_index(mrow, col, out_mt) : out + (size_t)mrow * n_q * D + col;
    *reinterpret_cast<bf16x4*>(dst) = ob;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int rows_pad_of(const massv_attn_desc& a) {
    const int rows = (a.n_q_heads / a.n_kv_heads) * a.n_query;
    return (rows + 15) / 16 * 16;
}

// Number of key-range splits: enough workgroups to give every CU one, but no
// split shorter than one block per wave.
static int n_split_of(const massv_attn_desc& a) {
    const int pairs = a.batch * a.n_kv_heads;
    const int max_blocks = a.l_max / kBlk;
    int s = (256 + pairs - 1) / pairs;
    const int cap = (max_blocks + kAttnWaves - 1) / kAttnWaves;
    if (s > cap) s = cap;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return s;
}

int check_attn_desc(const massv_attn_desc* a) {
    if (!a) return MASSV_EINVAL;
    if (a->batch < 1 || a->n_query < 1 || a->n_q_heads < 1 || a->n_kv_heads < 1 || a->head_dim < 2) return MASSV_EINVAL;
    if (a->n_q_heads % a->n_kv_heads) return MASSV_EINVAL;
    if (a->l_max < kBlk || a->l_max % kBlk) return MASSV_EINVAL;
    if (a->n_query > a->l_max) return MASSV_EINVAL;
    if (!(a->scale >= 0.f) || isinf(a->scale)) return MASSV_EINVAL;
    if (a->window < 0) return MASSV_EINVAL;
    if (a->dtype != MASSV_F32 && a->dtype != MASSV_BF16) return MASSV_EINVAL;
    if (a->head_dim % 2) return MASSV_EINVAL;
    if (a->batch > 65535 || a->n_q_heads > 65535) return MASSV_EUNSUPPORTED;
    if (a->dtype == MASSV_F32) {
        if (a->head_dim > 256) return MASSV_EUNSUPPORTED;
    } else {
        if (a->head_dim != 64 && a->head_dim != 128 && a->head_dim != 256) return MASSV_EUNSUPPORTED;
        if (rows_pad_of(*a) > MASSV_MAX_ROWS) return MASSV_EUNSUPPORTED;
        if (a->head_dim == 256 && rows_pad_of(*a) > 32) return MASSV_EUNSUPPORTED;
    }
    return MASSV_OK;
}

size_t attention_workspace(const massv_attn_desc& a) {
    if (a.dtype == MASSV_F32) return 256;
    const size_t slots = (size_t)a.batch * a.n_kv_heads * n_split_of(a) * rows_pad_of(a);
    return align_up(slots * a.head_dim * sizeof(float), 256) + align_up(slots * 2 * sizeof(float), 256);
}

template <int D, int MT>
static int launch_mfma(const massv_attn_desc& a, AttnParams p, hipStream_t st) {
    const size_t lds = (size_t)MT * 16 * (D + 4) * sizeof(float) * (attn_tree_merge(D, MT) ? 2 : 1);
    if (lds > 48 * 1024) {                       // more dynamic LDS than a kernel may use by default
        static std::atomic<bool> ready[64];       // zero-initialised; calls may come from several threads
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MASSV_ELAUNCH;
        if (!ready[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute((const void*)attention_mfma_kernel<D, MT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds) != hipSuccess) return MASSV_ELAUNCH;
            ready[dev].store(true, std::memory_order_release);
        }
    }
    launch_traced(MASSV_K_ATTENTION, attention_mfma_kernel<D, MT>, dim3(p.n_split, a.n_kv_heads, a.batch),
                  dim3(kAttnThreads), lds, st, p);
    if (p.n_split > 1)
    {
        const int total_rows = a.batch * a.n_query * a.n_q_heads, rows_per_wg = kCombineThreads / (D / 4);
        launch_traced(MASSV_K_ATTN_COMBINE, attention_combine_kernel<D>, dim3((total_rows + rows_per_wg - 1) / rows_per_wg),
                      dim3(kCombineThreads), 0, st, (const float*)p.part_o, (const float*)p.part_ml, p.out, a.n_query,
                      a.n_q_heads, a.n_kv_heads, p.n_split, MT * 16, p.out_mt, total_rows);
    }
    return launch_status();
}

template <int D>
static int launch_mfma_d(const massv_attn_desc& a, AttnParams p, int mt, hipStream_t st) {
    switch (mt) {
        case 1: return launch_mfma<D, 1>(a, p, st);
        case 2: return launch_mfma<D, 2>(a, p, st);
        case 3: if constexpr (D <= 128) return launch_mfma<D, 3>(a, p, st); else return MASSV_EUNSUPPORTED;
        case 4: if constexpr (D <= 128) return launch_mfma<D, 4>(a, p, st); else return MASSV_EUNSUPPORTED;
    }
    return MASSV_EUNSUPPORTED;
}

int launch_attention(const massv_attn_desc& a, const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* kv_len, void* out, void* ws, bool out_packed, hipStream_t st) {
    const float scale = a.scale > 0.f ? a.scale : 1.0f / sqrtf((float)a.head_dim);
    if (a.dtype == MASSV_F32) {
        hipLaunchKernelGGL(attention_generic_kernel<float>, dim3(a.n_query, a.n_q_heads, a.batch), dim3(256), 0, st,
                           (const float*)q, (const float*)k_cache, (const float*)v_cache, kv_len, (float*)out,
                           a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, scale, a.window);
        return launch_status();
    }
    AttnParams p;
    p.q = (const bf16_t*)q; p.kc = (const bf16_t*)k_cache; p.vc = (const bf16_t*)v_cache; p.kv_len = kv_len;
    p.out = (bf16_t*)out;
    p.Q = a.n_query; p.n_q = a.n_q_heads; p.n_kv = a.n_kv_heads; p.l_max = a.l_max;
    p.n_split = n_split_of(a);
    p.window = a.window;
    p.out_mt = out_packed ? (a.batch * a.n_query + 15) / 16 : 0;
    p.scale_log2 = scale * 1.4426950408889634f;
    const int rp = rows_pad_of(a);
    const size_t slots = (size_t)a.batch * a.n_kv_heads * p.n_split * rp;
    p.part_o = (float*)ws;
    p.part_ml = (float*)((char*)ws + align_up(slots * a.head_dim * sizeof(float), 256));
    const int mt = rp / 16;
    switch (a.head_dim) {
        case 64: return launch_mfma_d<64>(a, p, mt, st);
        case 128: return launch_mfma_d<128>(a, p, mt, st);
        case 256: return launch_mfma_d<256>(a, p, mt, st);
    }
    return MASSV_EUNSUPPORTED;
}

}  // namespace massv

using namespace massv;

extern "C" size_t massv_verify_attention_workspace(const massv_attn_desc* desc) {
    if (check_attn_desc(desc) != MASSV_OK) return 0;
    return attention_workspace(*desc);
}

extern "C" int massv_verify_attention(const massv_attn_desc* desc, const void* q, const void* k_cache,
                                      const void* v_cache, const int32_t* kv_len, void* out,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_attn_desc(desc);
    if (rc != MASSV_OK) return rc;
    if (!q || !k_cache || !v_cache || !kv_len || !out) return MASSV_EINVAL;
    if (!workspace || workspace_bytes < attention_workspace(*desc)) return MASSV_EWORKSPACE;
    return launch_attention(*desc, q, k_cache, v_cache, kv_len, out, workspace, false, (hipStream_t)stream);
}
