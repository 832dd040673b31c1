// prefill_attention: attention of the prompt pass that fills the cache (paper Section 2.2: the projected image
// features enter the sequence ahead of the text tokens, and the language model conditions on all of them).  Same
// definition as verify_attention -- the query at cache row r sees rows 0 .. r -- but with hundreds to thousands
// of new positions per sequence instead of gamma+1, so the work is a dense contraction and the matrix cores are
// the roof, not HBM.
//
// bf16 kernel:
//   * The caches are read in the library's blocked layouts; a wave's operands of both products are 16-byte loads per
//     lane straight into registers, no LDS staging and no transposes.
//   * The G query heads that share a KV head are stacked with the positions into rows (row = position * G + head),
//     so every key / value tile fetched serves all G heads.
//   * A wave owns RT tiles of 32 stacked rows (64 rows for d <= 128) for the whole key range: Q stays in registers
//     as the B operand of v_mfma_f32_32x32x16_bf16, scores are formed transposed (S^T = K Q^T) so that the
//     probabilities already sit in the operand layout of O^T += V^T P^T, and the streaming softmax keeps
//     (reference, sum, O) in registers.  Nothing is merged between waves; each writes its own rows.
//   * The four waves of a workgroup take neighbouring row ranges, so they walk the same key blocks at nearly
//     the same time and share them through the CU's vector cache; workgroups of one (sequence, KV head) pair
//     have linear ids congruent modulo the pair count, which (8 dies, round-robin dispatch) puts them on one
//     die whenever the pair count is a multiple of 8, so the pair's keys and values are fetched into one L2.
//   * Only blocks that cross some row's first or last visible key pay for masks.
// Measured and dropped at 8 x 2048 positions, d = 128 (the shipped kernel: 285-304 us):
//   the 16x16x32 instruction with 4 tiles of 16 rows, 336-376 us (a lone wave issues one of those only every ~31
//   cycles, and twice as many are needed); two key / value register sets with Q re-read from LDS, 489 us; 32 rows
//   per wave with two waves per SIMD and operands loaded per wave, 343-378 us (the vector cache cannot feed twice
//   the operand traffic); eight waves of 32 rows with the blocks staged once per workgroup in LDS by direct
//   global->LDS loads (ring of 4 stages of 2 blocks, one barrier per stage), 283-313 us and no better on four
//   other shapes: the barrier re-aligns the two waves of a SIMD, which then want the same unit at the same time.
// fp32: the plain one-workgroup-per-(position, head) kernel below, for the small configuration.
#include "kernels.h"

#include <type_traits>

namespace massv {

constexpr int kPfWaves = 4;
constexpr int kPfThreads = kPfWaves * kWave;
constexpr int kPfBlk = MASSV_V_BLOCK;

struct PrefillParams {
    const bf16_t* q; const bf16_t* kc; const bf16_t* vc;
    const int32_t* kv_len; const int32_t* n_new; const int32_t* n_bidir;     // n_bidir may be null
    bf16_t* out;
    int Lq, n_q, n_kv, l_max, window, n_tiles;
    float scale_log2;            // scale * log2(e)
};

// One past the last row visible to the query at cache row r: r + 1, or the end of the leading block of m rows
// that attends within itself when r lies inside it (never beyond the rows that exist, `total`).
__host__ __device__ inline int pf_hi(int r, int m, int total) {
    if (r < m) { const int e = m < total ? m : total; return e > r + 1 ? e : r + 1; }
    return r + 1;
}
__host__ __device__ inline int pf_lo(int r, int W) { return (W > 0 && r + 1 > W) ? r + 1 - W : 0; }

// max(a, b, c) in one instruction.  (fmaxf nests compile to a canonicalising self-maximum per operand plus the
// maximum itself: 11 instructions for 8 scores instead of 4; operands here are never NaN -- masked scores are -inf.)
__device__ inline float pf_max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// ---------------------------------------------------------------------------
// A lone wave per SIMD gets a 32x32x16 matrix instruction out every ~40 cycles (against ~31 for the 16x16x32 form
// that does half the work).  A wave owns RT tiles of 32 stacked rows.
//   S^T tile (32 key slots x 32 rows): lane l holds row l % 32 and the slots 8 (v / 4) + 4 (l / 32) + v % 4, v = 0..15.
//   Key slot rho of a block carries key 16 (g / 2) + 8 h + 4 (g % 2) + r (rho = 8 g + 4 h + r), so that the lane's
//   values v = 8 t .. 8 t + 7 are the keys 16 t + 8 (l / 32) + (0..7): as they stand they are the B operand of step t
//   of O^T += V^T P^T, whose A operand is then one 16-byte load of 8 consecutive keys of one dim.
// ---------------------------------------------------------------------------
__device__ inline float pf_xor32_max(float v) { return fmaxf(v, __shfl_xor(v, 32, kWave)); }

template <int D, int RT>
__global__ __launch_bounds__(kPfThreads)
void prefill_attention_kernel(PrefillParams p) {
    constexpr int KS = D / 16;          // 16-wide k-steps of the score product
    constexpr int NT = D / 32;          // 32-dim tiles of the output
    constexpr int RW = RT * 32;         // stacked rows per wave
    const int pair = blockIdx.x, b = pair / p.n_kv, g = pair % p.n_kv;
    const int tile = p.n_tiles - 1 - (int)blockIdx.y;                 // the longest key ranges are started first
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lr = lane % 32, hh = lane / 32;
    const int G = p.n_q / p.n_kv;
    int L = p.kv_len[b]; L = L < 0 ? 0 : L;
    int n = p.n_new[b]; n = n < 0 ? 0 : (n > p.Lq ? p.Lq : n);
    if (L + n > p.l_max) n = p.l_max - L > 0 ? p.l_max - L : 0;
    const int rows = n * G;
    const int r0 = (tile * kPfWaves + wave) * RW;                     // first stacked row of this wave
    if (r0 >= rows) return;                                            // (no barriers below: waves are independent)
    const int total = L + n;
    const int m_bidir = p.n_bidir ? p.n_bidir[b] : 0;
    const int W = p.window;
    const size_t bg = (size_t)b * p.n_kv + g;

    // ---- rows of this wave: position, visible key range; Q operand in registers ----
    bf16x8 qreg[RT][KS];
    int hi_row[RT], lo_row[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        int r = r0 + rt * 32 + lr;
        if (r >= rows) r = rows - 1;                                   // padding rows repeat the last one; never stored
        const int i = r / G, qh = r % G;
        hi_row[rt] = pf_hi(L + i, m_bidir, total);
        lo_row[rt] = pf_lo(L + i, W);
        const bf16_t* qr = p.q + (((size_t)b * p.Lq + i) * p.n_q + g * G + qh) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qreg[rt][ks] = *reinterpret_cast<const bf16x8*>(qr + ks * 16 + hh * 8);
    }
    const int i_first = r0 / G;
    const int r_last = (r0 + RW - 1 < rows - 1) ? r0 + RW - 1 : rows - 1;
    const int i_last = r_last / G;
    const int min_hi = pf_hi(L + i_first, m_bidir, total), max_hi = pf_hi(L + i_last, m_bidir, total);
    const int min_lo = pf_lo(L + i_first, W), max_lo = pf_lo(L + i_last, W);
    const int blk_begin = min_lo / kPfBlk, blk_end = (max_hi + kPfBlk - 1) / kPfBlk;

    floatx16 acc[RT][NT];
    float m_run[RT], l_run[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        m_run[rt] = -INFINITY; l_run[rt] = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[rt][nt][e] = 0.f;
    }

    // key slot lr = 8 g + 4 h + r of a block -> key 16 (g / 2) + 8 h + 4 (g % 2) + r, which the blocked key cache
    // keeps in its half g % 2 (bit 2 of the key) at place 4 (2 (g / 2) + h) + r; the lane's 8 dims are chunk
    // 2 ks + hh of that half
    const int sg = lr / 8, sh = (lr / 4) % 2, sr = lr % 4;
    const bf16_t* kbase = p.kc + bg * (size_t)p.l_max * D + (size_t)(sg % 2) * (D * 16) + hh * 128 + ((2 * (sg / 2) + sh) * 4 + sr) * 8;
    const bf16_t* vbase = p.vc + bg * (size_t)p.l_max * D + (size_t)lr * kPfBlk + hh * 8;
    auto load_k = [&](int blk, bf16x8 (&kreg)[KS]) {
        const bf16_t* kb = kbase + (size_t)blk * kPfBlk * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[ks] = *reinterpret_cast<const bf16x8*>(kb + ks * 256);
    };
    // value operand (nt, t): dim 32 nt + lr, keys 16 t + 8 hh + (0..7) of the block
    auto load_v = [&](int blk, bf16x8 (&vreg)[NT][2]) {
        const bf16_t* vb = vbase + (size_t)blk * D * kPfBlk;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                vreg[nt][t] = *reinterpret_cast<const bf16x8*>(vb + (size_t)(nt * 32) * kPfBlk + t * 16);
    };

    constexpr float kLazy = 8.0f;       // a row's reference exponent is raised only when exceeded by 2^8
    // ---- pieces of one block for one row tile ----
    // S^T tile: KS matrix instructions
    auto s_tile = [&](bf16x8 (&kr)[KS], int rt, floatx16& sc) {
#pragma unroll
        for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[ks], qreg[rt][ks], sc, 0, 0, 0);
    };
    // O^T += V^T P^T: 2 NT matrix instructions
    auto pv_tile = [&](int rt, bf16x8 (&vr)[NT][2], bf16x8 (&pv)[2]) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[rt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[nt][t], pv[t], acc[rt][nt], 0, 0, 0);
    };
    // values of rows past the valid length may hold anything: zero them (last block only)
    auto v_clean = [&](int blk, bf16x8 (&vr)[NT][2]) {
        const int key0 = blk * kPfBlk + hh * 8;
        if ((blk + 1) * kPfBlk > total) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (key0 + 16 * t + e >= total) vr[nt][t][e] = (bf16_t)0.f;
        }
    };
    // first half of the streaming softmax: masks, the lane's maximum, and (rarely) a raised reference with the
    // accumulators rescaled.  Value v of the lane is key key0 + 16 (v / 8) + v % 8.
    auto soft_max = [&](int rt, int blk, floatx16& sc) {
        const int key0 = blk * kPfBlk + hh * 8;
        const bool masked = (blk + 1) * kPfBlk > min_hi || blk * kPfBlk < max_lo;
        if (masked) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = key0 + 16 * (v / 8) + v % 8;
                if (key >= hi_row[rt] || key < lo_row[rt]) sc[v] = -INFINITY;
            }
        }
        float mx = pf_max3(pf_max3(pf_max3(sc[0], sc[1], sc[2]), pf_max3(sc[3], sc[4], sc[5]), pf_max3(sc[6], sc[7], sc[8])),
                           pf_max3(pf_max3(sc[9], sc[10], sc[11]), pf_max3(sc[12], sc[13], sc[14]), sc[15]), sc[15]);
        mx *= p.scale_log2;
        if (__any(mx > m_run[rt] + kLazy)) {
            mx = pf_xor32_max(mx);
            if (mx > m_run[rt] + kLazy) {
                const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - mx);     // m_run = -inf gives 0
                l_run[rt] *= alpha;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    // keeps the copies out of the accumulation registers inside this rare branch
                    asm volatile("" : "+a"(acc[rt][nt]));
                    acc[rt][nt] *= alpha;
                }
                m_run[rt] = mx;
            }
        }
    };
    // second half: probabilities relative to the reference, their sum, and the bf16 operand of the second product
    auto soft_exp = [&](int rt, const floatx16& sc, bf16x8 (&pv)[2]) {
        const float neg_m = (m_run[rt] == -INFINITY) ? 0.f : -m_run[rt];
        float ps = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float pe = __builtin_amdgcn_exp2f(fmaf(sc[v], p.scale_log2, neg_m));
            ps += pe;
            pv[v / 8][v % 8] = (bf16_t)pe;
        }
        l_run[rt] += ps;
    };

    if constexpr (RT == 2) {
        // Two row tiles A and B leapfrog, so that the vector arithmetic of one tile's softmax is issued between the
        // matrix instructions of the other tile (one wave per SIMD: a matrix instruction holds the wave's issue for
        // about 18 of the 40 cycles it needs, the rest is free for independent vector instructions -- but only if
        // the instruction stream alternates, since a wave issues in order):
        //   step 1 of block i:  exponentials of (B, i)      between   O_A += V_i P_A,i   and   S_A,i+1 = K_i+1 Q_A
        //   step 2 of block i:  exponentials of (A, i + 1)  between   O_B += V_i P_B,i   and   S_B,i+1 = K_i+1 Q_B
        // Keys are held two blocks ahead and values one block ahead, in two register sets each.
        // A step is two halves of 8 score values each: the first next to the KS matrix instructions of the other
        // tile's next scores, the second next to the 2 NT matrix instructions of the other tile's second product.
        // One key set and one value set: the keys of block i + 2 are requested as soon as the scores of block i + 1
        // are formed (middle of step 2), the values of block i + 1 at the end of step 2; each has the other half of
        // the work before it is needed.
        auto exps = [&](int rv, const floatx16& sv, bf16x8& po, int v0, float neg_m, float& ps) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(sv[v0 + e], p.scale_log2, neg_m));
                ps += pe;
                po[e] = (bf16_t)pe;
            }
        };
        auto order = [&](auto n_mfma) {            // the order asked of the scheduler for one half
            constexpr int N = decltype(n_mfma)::value, VP = 8 / N;
#pragma unroll
            for (int m = 0; m < N; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2 * VP, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, VP, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2 * VP, 0);
            }
        };
        // first half: tile rv's values 0..7, tile rm's scores of the block whose keys kq holds
        auto half_s = [&](int rv, const floatx16& sv, bf16x8 (&pvo)[2], float neg_m, float& ps, int rm, bf16x8 (&kq)[KS], floatx16& sm) {
            __builtin_amdgcn_sched_barrier(0);
            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                sm = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kq[ks], qreg[rm][ks], ks == 0 ? zero : sm, 0, 0, 0);
            exps(rv, sv, pvo[0], 0, neg_m, ps);
            order(std::integral_constant<int, KS>{});
            // (the probabilities are first needed a step later; without a use here the compiler moves their
            // arithmetic down to that step, away from the matrix instructions it is meant to sit between)
            asm volatile("" : "+v"(pvo[0]), "+v"(ps));
            __builtin_amdgcn_sched_barrier(0);
        };
        // second half: tile rv's values 8..15, tile rm's second product with the values vq holds
        auto half_pv = [&](int rv, const floatx16& sv, bf16x8 (&pvo)[2], float neg_m, float& ps, int rm, bf16x8 (&pm)[2], bf16x8 (&vq)[NT][2]) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[rm][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[nt][t], pm[t], acc[rm][nt], 0, 0, 0);
            exps(rv, sv, pvo[1], 8, neg_m, ps);
            order(std::integral_constant<int, 2 * NT>{});
            asm volatile("" : "+v"(pvo[1]), "+v"(ps));
            __builtin_amdgcn_sched_barrier(0);
        };
        const int nb = blk_end - blk_begin;
        bf16x8 kq[KS], vq[NT][2];
        floatx16 sA, sB;
        bf16x8 pA[2], pB[2];
        if (nb > 0) {
            load_k(blk_begin, kq);
            s_tile(kq, 0, sA);
            s_tile(kq, 1, sB);
            if (nb > 1) load_k(blk_begin + 1, kq);
            load_v(blk_begin, vq);                     // keys before values, the order the loop requests them in
            soft_max(0, blk_begin, sA);
            soft_exp(0, sA, pA);
        }
        // entering block i: kq holds the keys of block i + 1, vq the values of block i, pA tile A's probabilities
        // and sB tile B's scores of block i
        for (int i = 0; i + 1 < nb; ++i) {
            const int blk = blk_begin + i;
            v_clean(blk, vq);
            soft_max(1, blk, sB);
            {
                const float neg_m = (m_run[1] == -INFINITY) ? 0.f : -m_run[1];
                float ps = 0.f;
                half_s(1, sB, pB, neg_m, ps, 0, kq, sA);
                half_pv(1, sB, pB, neg_m, ps, 0, pA, vq);
                l_run[1] += ps;
            }
            soft_max(0, blk + 1, sA);
            {
                const float neg_m = (m_run[0] == -INFINITY) ? 0.f : -m_run[0];
                float ps = 0.f;
                half_s(0, sA, pA, neg_m, ps, 1, kq, sB);
                if (i + 2 < nb) load_k(blk + 2, kq);
                half_pv(0, sA, pA, neg_m, ps, 1, pB, vq);
                load_v(blk + 1, vq);
                l_run[0] += ps;
            }
        }
        if (nb > 0) {                                  // the last block: nothing follows tile A's second product
            const int blk = blk_end - 1;
            v_clean(blk, vq);
            soft_max(1, blk, sB);
            const float neg_m = (m_run[1] == -INFINITY) ? 0.f : -m_run[1];
            float ps = 0.f;
            exps(1, sB, pB[0], 0, neg_m, ps);
            half_pv(1, sB, pB, neg_m, ps, 0, pA, vq);
            l_run[1] += ps;
            pv_tile(1, vq, pB);
        }
    } else {
        bf16x8 k0[KS], v0[NT][2];
        floatx16 sc;
        bf16x8 pv[2];
        for (int blk = blk_begin; blk < blk_end; ++blk) {
            load_k(blk, k0); load_v(blk, v0);
            s_tile(k0, 0, sc);
            v_clean(blk, v0);
            soft_max(0, blk, sc);
            soft_exp(0, sc, pv);
            pv_tile(0, v0, pv);
        }
    }

    // ---- write this wave's rows: lane holds dims 32 nt + 8 (v / 4) + 4 hh + v % 4 of row 32 rt + lr ----
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const float l = l_run[rt] + __shfl_xor(l_run[rt], 32, kWave);
        const int r = r0 + rt * 32 + lr;
        if (r >= rows) continue;
        const float inv = 1.0f / l;                        // every row sees at least its own key
        const int i = r / G, qh = r % G;
        bf16_t* dst = p.out + (((size_t)b * p.Lq + i) * p.n_q + g * G + qh) * D + hh * 4;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const floatx16& v = acc[rt][nt];
                bf16x4 o = {(bf16_t)(v[4 * q4] * inv), (bf16_t)(v[4 * q4 + 1] * inv), (bf16_t)(v[4 * q4 + 2] * inv), (bf16_t)(v[4 * q4 + 3] * inv)};
                *reinterpret_cast<bf16x4*>(dst + nt * 32 + q4 * 8) = o;
            }
    }
}

// ---------------------------------------------------------------------------
// fp32: grid (L_q, n_q, B), 256 threads; keys 256 at a time (thread t scores key t, thread c accumulates column c).
// Row-major fp32 keys, blocked values.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void prefill_generic_kernel(const float* __restrict__ q, const float* __restrict__ kc, const float* __restrict__ vc,
                            const int32_t* __restrict__ kv_len, const int32_t* __restrict__ n_new,
                            const int32_t* __restrict__ n_bidir, float* __restrict__ out,
                            int Lq, int n_q, int n_kv, int d, int l_max, float scale, int window) {
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int G = n_q / n_kv, g = h / G;
    const size_t bg = (size_t)b * n_kv + g;
    int L = kv_len[b]; L = L < 0 ? 0 : L;
    int n = n_new[b]; n = n < 0 ? 0 : (n > Lq ? Lq : n);
    if (L + n > l_max) n = l_max - L > 0 ? l_max - L : 0;
    if (i >= n) return;                                    // uniform over the workgroup
    const int hi = pf_hi(L + i, n_bidir ? n_bidir[b] : 0, L + n), lo = pf_lo(L + i, window);
    __shared__ float qs[256];
    __shared__ float w[256];
    __shared__ float red[4];
    const float* qr = q + (((size_t)b * Lq + i) * n_q + h) * d;
    if (tid < d) qs[tid] = qr[tid];
    __syncthreads();
    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
    for (int j0 = lo; j0 < hi; j0 += 256) {
        const int j = j0 + tid;
        float s = -INFINITY;
        if (j < hi) {
            const float* kr = kc + (bg * l_max + j) * d;
            float dot = 0.f;
            for (int c = 0; c < d; ++c) dot += qs[c] * kr[c];
            s = dot * scale;
        }
        float mx = wave_max(s);
        if ((tid & 63) == 0) red[tid >> 6] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float m_new = fmaxf(m_run, mx);              // finite: key j0 is visible
        const float pe = (j < hi) ? expf(s - m_new) : 0.f;
        w[tid] = pe;
        float ps = wave_sum(pe);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = ps;
        __syncthreads();
        ps = red[0] + red[1] + red[2] + red[3];
        const float alpha = expf(m_run - m_new);
        l_run = l_run * alpha + ps;
        acc *= alpha;
        if (tid < d) {
            const int cnt = (hi - j0) < 256 ? (hi - j0) : 256;
            for (int t = 0; t < cnt; ++t) {
                const int jj = j0 + t;
                acc += w[t] * vc[((bg * (size_t)(l_max / kPfBlk) + (size_t)(jj / kPfBlk)) * d + tid) * kPfBlk + (jj % kPfBlk)];
            }
        }
        m_run = m_new;
        __syncthreads();
    }
    if (tid < d) out[(((size_t)b * Lq + i) * n_q + h) * d + tid] = acc / l_run;
}

template <int D, int RT>
static int launch_prefill(const massv_attn_desc& a, PrefillParams p, hipStream_t st) {
    const int rows_max = a.n_query * (a.n_q_heads / a.n_kv_heads);
    const int per_wg = kPfWaves * RT * 32;
    p.n_tiles = (rows_max + per_wg - 1) / per_wg;
    if (p.n_tiles > 65535) return MASSV_EUNSUPPORTED;
    launch_traced(MASSV_K_PREFILL_ATTENTION, prefill_attention_kernel<D, RT>, dim3(a.batch * a.n_kv_heads, p.n_tiles),
                  dim3(kPfThreads), 0, st, p);
    return launch_status();
}

}  // namespace massv

using namespace massv;

extern "C" int massv_prefill_attention(const massv_attn_desc* desc, const void* q, const void* k_cache,
                                       const void* v_cache, const int32_t* kv_len, const int32_t* n_new,
                                       const int32_t* n_bidir, void* out, void* stream) {
    if (!desc) return MASSV_EINVAL;
    // the descriptor rules of verify_attention, except that the row count per KV head is not limited
    massv_attn_desc one = *desc;
    one.n_query = 1;
    const int rc = check_attn_desc(&one);
    if (rc != MASSV_OK) return rc;
    if (desc->n_query < 1 || desc->n_query > desc->l_max) return MASSV_EINVAL;
    if (!q || !k_cache || !v_cache || !kv_len || !n_new || !out) return MASSV_EINVAL;
    if ((int64_t)desc->batch * desc->n_kv_heads > 0x7fffffff) return MASSV_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const massv_attn_desc& a = *desc;
    const float scale = a.scale > 0.f ? a.scale : 1.0f / sqrtf((float)a.head_dim);
    if (a.dtype == MASSV_F32) {
        if (a.n_query > 65535) return MASSV_EUNSUPPORTED;
        hipLaunchKernelGGL(prefill_generic_kernel, dim3(a.n_query, a.n_q_heads, a.batch), dim3(256), 0, st,
                           (const float*)q, (const float*)k_cache, (const float*)v_cache, kv_len, n_new, n_bidir,
                           (float*)out, a.n_query, a.n_q_heads, a.n_kv_heads, a.head_dim, a.l_max, scale, a.window);
        return launch_status();
    }
    PrefillParams p;
    p.q = (const bf16_t*)q; p.kc = (const bf16_t*)k_cache; p.vc = (const bf16_t*)v_cache;
    p.kv_len = kv_len; p.n_new = n_new; p.n_bidir = n_bidir;
    p.out = (bf16_t*)out;
    p.Lq = a.n_query; p.n_q = a.n_q_heads; p.n_kv = a.n_kv_heads; p.l_max = a.l_max; p.window = a.window;
    p.n_tiles = 0;
    p.scale_log2 = scale * 1.4426950408889634f;
    switch (a.head_dim) {
        case 64: return launch_prefill<64, 2>(a, p, st);
        case 128: return launch_prefill<128, 2>(a, p, st);
        case 256: return launch_prefill<256, 1>(a, p, st);
    }
    return MASSV_EUNSUPPORTED;
}
