// spec_accept: vocabulary-wide softmax statistics and the sequential
// accept / reject / resample rule of speculative decoding (paper Section 2.1).
//
// The work is a stream over the logits, bound by HBM bandwidth:
//   pass 1  accept_stats   every target row (and, at T > 0, every draft row) is
//                          cut into chunks of 1024 logits; one WAVE per (row,
//                          chunk) produces {max, first arg-max, sum exp} with
//                          shuffles only -- no LDS, no barriers, waves retire
//                          independently.
//           accept_decide  one workgroup per sequence merges the chunk partials
//                          (a wave per row); lane i of its first wave tests
//                          draft i, the first failure ends the chain.
//   pass 2  residual_mass  (T > 0) re-reads the ONE target/draft row pair per
//                          sequence the final token is drawn from and sums
//                          max(p - q, 0) and p per chunk,
//           residual_pick  finds the chunk, then the token, where the running
//                          sum first exceeds uniform * total.
// Sums that decide a token are carried in double so that the result does not
// depend on how the vocabulary was cut into chunks.
#include "kernels.h"

#include <limits.h>
#include <atomic>

namespace massv {

constexpr int kAccThreads = 128;                          // 2 waves, one chunk each (64: 73 us, 128: 66 us, 256: 67 us,
                                                          // 1024: 75 us for the sampling call on the long-context shape)
constexpr int kAccPerLane = 16;                           // 4 float4 loads per lane
constexpr int kAccChunk = kWave * kAccPerLane;            // 1024 logits per wave
constexpr int kMaxGamma = 15;

struct SeqSel { int n; int bonus; int pad0; int pad1; double m_t, s_t, m_d, s_d; };
struct ChunkMass { double r, p; };


// 2^x by the hardware instruction alone: x <= 0 here, results below the smallest normal number flush to
// zero (a probability under 2^-126 of the row's largest), no range handling needed.
__device__ inline float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// d is a logit minus the row maximum (<= 0, possibly -inf for padding or a
// zero-probability token); clamping to the largest finite value keeps
// (-inf) * lo from producing NaN, the result still underflows exp to 0.
__device__ inline float scaled(float d, TempScale ts) {
    d = fmaxf(d, -3.0e38f);
    return fmaf(d, ts.lo, d * ts.hi);
}

// Coalesced read of one chunk by one wave: x[j*4+e] is element base + (j*64 + lane)*4 + e;
// out-of-range elements read as -inf.
__device__ inline void load_chunk(const float* __restrict__ row, int V, int base, int lane, int vec,
                                  float (&x)[kAccPerLane]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int idx = base + (j * kWave + lane) * 4;
        if (vec && idx + 3 < V) {
            float4 v = ldg_stream(reinterpret_cast<const float4*>(row + idx));
            x[j * 4 + 0] = v.x; x[j * 4 + 1] = v.y; x[j * 4 + 2] = v.z; x[j * 4 + 3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[j * 4 + e] = (idx + e < V) ? row[idx + e] : -INFINITY;
        }
    }
}

__device__ inline int chunk_index(int base, int lane, int k) {
    return base + ((k >> 2) * kWave + lane) * 4 + (k & 3);
}

// (value, index) ordering: larger value first, then smaller index.
__device__ inline void argmax_merge(float& v, int& i, float ov, int oi) {
    if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// (maximum, lowest index of it) over the wave by the six moves of the wave reductions; a lane without a source
// merges with itself.
template <int CTRL, int ROW_MASK>
__device__ inline void dpp_argmax_step(float& m, int& am) {
    const float om = dpp_move<CTRL, ROW_MASK>(m, m);
    const int oi = dpp_move<CTRL, ROW_MASK>(am, am);
    argmax_merge(m, am, om, oi);
}
__device__ inline void wave_argmax(float& m, int& am) {       // result in every lane
    dpp_argmax_step<kDppShr1, 0xf>(m, am);
    dpp_argmax_step<kDppShr2, 0xf>(m, am);
    dpp_argmax_step<kDppShr4, 0xf>(m, am);
    dpp_argmax_step<kDppShr8, 0xf>(m, am);
    dpp_argmax_step<kDppBcast15, 0xa>(m, am);
    dpp_argmax_step<kDppBcast31, 0xc>(m, am);
    m = lane_value(m, kWave - 1);
    am = __builtin_amdgcn_readlane(am, kWave - 1);
}

__global__ __launch_bounds__(kAccThreads)
void accept_stats_kernel(const float* __restrict__ target, const float* __restrict__ draft,
                         int n_target_rows, int V, int C, TempScale ts, int greedy, int vec,
                         RowPartial* __restrict__ part) {
    const int lane = threadIdx.x % kWave;
    const int c = blockIdx.x * (kAccThreads / kWave) + threadIdx.x / kWave, r = blockIdx.y;
    if (c >= C) return;                                      // whole wave leaves together
    const float* row = (r < n_target_rows) ? target + (size_t)r * V
                                           : draft + (size_t)(r - n_target_rows) * V;
    const int base = c * kAccChunk;
    float x[kAccPerLane];
    load_chunk(row, V, base, lane, vec, x);

    float m = x[0];
    int am = chunk_index(base, lane, 0);
#pragma unroll
    for (int k = 1; k < kAccPerLane; ++k)
        if (x[k] > m) { m = x[k]; am = chunk_index(base, lane, k); }
    wave_argmax(m, am);
    double s = 0.0;
    if (!greedy) {
        float acc = 0.f;
        if (m > -INFINITY) {
#pragma unroll
            for (int k = 0; k < kAccPerLane; ++k) acc += exp2_raw(scaled(x[k] - m, ts));
        }
        s = wave_sum((double)acc);
    }
    if (lane == 0) {
        RowPartial p; p.m = m; p.arg = am; p.s = s;
        part[(size_t)r * C + c] = p;
    }
}

constexpr int kDecideThreads = 1024;                      // 16 waves: one row of the sequence each

__global__ __launch_bounds__(kDecideThreads)
void accept_decide_kernel(const float* __restrict__ target, const float* __restrict__ draft,
                          const int* __restrict__ tokens, const float* __restrict__ uniforms,
                          int B, int gamma, int V, double inv_t, float scale2, int greedy,
                          const RowPartial* __restrict__ part_t, int C_t, const RowPartial* __restrict__ part_d, int C_d,
                          SeqSel* __restrict__ sel, int* __restrict__ n_accepted, int* __restrict__ out_tokens) {
    const int b = blockIdx.x, tid = threadIdx.x, Q = gamma + 1;
    const int wave = tid / kWave, lane = tid % kWave;
    __shared__ double row_m[2 * kMaxGamma + 1], row_s[2 * kMaxGamma + 1];
    __shared__ int row_arg[2 * kMaxGamma + 1];
    const int nrows = greedy ? Q : Q + gamma;
    // wave 0, lane i examines draft i: its token and the two logits at that token do not depend on the
    // statistics, so their loads are issued before the merge below and are back when it is done
    int tok = 0;
    bool in_range = false;
    float lt_f = 0.f, ld_f = 0.f, u_f = 0.f;
    if (wave == 0 && lane < gamma) {
        tok = tokens[b * gamma + lane];
        in_range = (tok >= 0 && tok < V);
        if (in_range && !greedy) {
            lt_f = target[((size_t)b * Q + lane) * V + tok];
            ld_f = draft[((size_t)b * gamma + lane) * V + tok];
            u_f = uniforms[b * Q + lane];
        }
    }
    // one wave per row: lanes take the row's partials (part_t[B*Q][C_t] for target rows, part_d[B*gamma][C_d] for
    // draft rows), merged by a fixed shuffle tree
    for (int t = wave; t < nrows; t += kDecideThreads / kWave) {
        const int C = (t < Q) ? C_t : C_d;
        const RowPartial* p = (t < Q) ? part_t + (size_t)(b * Q + t) * C_t : part_d + (size_t)(b * gamma + (t - Q)) * C_d;
        float m = -INFINITY; int am = INT_MAX;
        double s = 0.0;
        if (C <= 4 * kWave) {                       // the usual case: every partial is loaded once, all loads in flight
            RowPartial own[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = lane + j * kWave;
                own[j].m = -INFINITY; own[j].arg = INT_MAX; own[j].s = 0.0;
                if (c < C) own[j] = p[c];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) argmax_merge(m, am, own[j].m, own[j].arg);      // ascending c, as below
            wave_argmax(m, am);
            if (!greedy) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (own[j].m > -INFINITY) s += own[j].s * (double)exp2f((own[j].m - m) * scale2);
                s = wave_sum(s);
            }
        } else {
            for (int c = lane; c < C; c += kWave) argmax_merge(m, am, p[c].m, p[c].arg);
            wave_argmax(m, am);
            if (!greedy) {
                for (int c = lane; c < C; c += kWave)
                    if (p[c].m > -INFINITY) s += p[c].s * (double)exp2f((p[c].m - m) * scale2);
                s = wave_sum(s);
            }
        }
        if (lane == 0) { row_m[t] = (double)m; row_s[t] = s; row_arg[t] = (am == INT_MAX) ? 0 : am; }
    }
    __syncthreads();
    if (wave != 0) return;

    // all comparisons in parallel, then the first failure ends the chain
    bool ok = true;
    if (lane < gamma) {
        if (!in_range) {
            ok = false;
        } else if (greedy) {
            ok = (tok == row_arg[lane]);
        } else {
            const double p = exp(((double)lt_f - row_m[lane]) * inv_t) / row_s[lane];
            const double q = exp(((double)ld_f - row_m[Q + lane]) * inv_t) / row_s[Q + lane];
            ok = (p >= q) || ((double)u_f * q < p);
        }
    }
    const unsigned long long fail = __ballot(!ok);
    const int n = fail ? __ffsll((long long)fail) - 1 : gamma;      // gamma <= 15 < 64
    if (lane < n) out_tokens[b * Q + lane] = tok;
    if (lane != 0) return;
    n_accepted[b] = n;
    for (int i = n + 1; i < Q; ++i) out_tokens[b * Q + i] = -1;
    if (greedy) {
        out_tokens[b * Q + n] = row_arg[n];
    } else {
        SeqSel s;
        s.n = n; s.bonus = (n == gamma); s.pad0 = s.pad1 = 0;
        s.m_t = row_m[n]; s.s_t = row_s[n];
        s.m_d = s.bonus ? 0.0 : row_m[Q + n];
        s.s_d = s.bonus ? 1.0 : row_s[Q + n];
        sel[b] = s;
    }
}

// Unnormalised-to-normalised probability of one logit in double.  The product is rounded on its own
// (never fused into a following subtraction), so that equal logits under equal statistics give
// exactly equal probabilities and p - q is exactly zero there.
__device__ inline double prob_of(float logit, double m, double inv_s, TempScale ts) {
#pragma clang fp contract(off)
    const double p = (double)exp2_raw(scaled(logit - (float)m, ts)) * inv_s;
    return p;
}

__global__ __launch_bounds__(kAccThreads)
void residual_mass_kernel(const float* __restrict__ target, const float* __restrict__ draft,
                          int gamma, int V, int C, TempScale ts, int vec,
                          const SeqSel* __restrict__ sel, ChunkMass* __restrict__ mass) {
    const int lane = threadIdx.x % kWave, Q = gamma + 1;
    const int c = blockIdx.x * (kAccThreads / kWave) + threadIdx.x / kWave, b = blockIdx.y;
    if (c >= C) return;
    const SeqSel s = sel[b];
    const int base = c * kAccChunk;
    float xt[kAccPerLane], xd[kAccPerLane];
    load_chunk(target + ((size_t)b * Q + s.n) * V, V, base, lane, vec, xt);
    if (!s.bonus) load_chunk(draft + ((size_t)b * gamma + s.n) * V, V, base, lane, vec, xd);
    const double inv_st = 1.0 / s.s_t, inv_sd = 1.0 / s.s_d;
    double sr = 0.0, sp = 0.0;
#pragma unroll
    for (int k = 0; k < kAccPerLane; ++k) {
        const double p = prob_of(xt[k], s.m_t, inv_st, ts);
        sp += p;
        if (!s.bonus) {
            const double q = prob_of(xd[k], s.m_d, inv_sd, ts);
            sr += fmax(p - q, 0.0);
        }
    }
    sr = wave_sum(sr); sp = wave_sum(sp);
    if (lane == 0) {
        ChunkMass m; m.r = sr; m.p = sp;
        mass[(size_t)b * C + c] = m;
    }
}

constexpr int kPickPerLane = kAccChunk / kWave;                // 16 consecutive logits per lane when locating the token

// One wave per sequence, no LDS and no barriers: the lanes own consecutive runs of chunks, then consecutive
// runs of tokens of the chosen chunk, so "first index whose running mass exceeds the threshold" is the first
// lane that found one.
__global__ __launch_bounds__(kWave)
void residual_pick_kernel(const float* __restrict__ target, const float* __restrict__ draft,
                          const float* __restrict__ uniforms, int gamma, int V, int C, TempScale ts, int vec,
                          const SeqSel* __restrict__ sel, const ChunkMass* __restrict__ mass,
                          int* __restrict__ out_tokens) {
    const int b = blockIdx.x, lane = threadIdx.x, Q = gamma + 1;
    // the selection record, the uniform and the chunk masses are independent loads: one round trip
    const SeqSel s = sel[b];
    const float u_res = uniforms[b * Q + gamma];

    // ---- which chunk: every lane owns `per` consecutive chunks ----
    const ChunkMass* m = mass + (size_t)b * C;
    const int per = (C + kWave - 1) / kWave;
    double my_r = 0.0, my_p = 0.0;
    for (int i = 0; i < per; ++i) { const int c = lane * per + i; if (c < C) { my_r += m[c].r; my_p += m[c].p; } }
    const double incl_r = wave_scan_incl(my_r), incl_p = wave_scan_incl(my_p);
    const double tot_r = lane_value(incl_r, kWave - 1), tot_p = lane_value(incl_p, kWave - 1);
    const int use_p = s.bonus || !(tot_r > 0.0);
    const double total = use_p ? tot_p : tot_r;
    const double thr = (double)u_res * total;
    int found = -1, lastpos = -1;
    double ahead_found = 0.0, ahead_last = 0.0;                // mass ahead of that chunk
    {
        double run = (use_p ? incl_p - my_p : incl_r - my_r);  // mass ahead of this lane's chunks
        for (int i = 0; i < per; ++i) {
            const int c = lane * per + i;
            if (c >= C) break;
            const double v = use_p ? m[c].p : m[c].r;
            if (v > 0.0) { lastpos = c; ahead_last = run; }
            if (run + v > thr) { found = c; ahead_found = run; break; }
            run += v;
        }
    }
    // the first lane that crossed the threshold; else (rounding at u -> 1) the last chunk with any mass; else chunk 0
    const unsigned long long hit = __ballot(found >= 0), any = __ballot(lastpos >= 0);
    int chunk = 0;
    double prefix = 0.0;
    if (hit) {
        const int src = __ffsll((long long)hit) - 1;
        chunk = __builtin_amdgcn_readlane(found, src); prefix = lane_value(ahead_found, src);
    } else if (any) {
        const int src = 63 - __clzll((long long)any);
        chunk = __builtin_amdgcn_readlane(lastpos, src); prefix = lane_value(ahead_last, src);
    }

    // ---- which token inside the chunk: every lane owns 16 consecutive tokens ----
    const int base = chunk * kAccChunk + lane * kPickPerLane;
    const float* trow = target + ((size_t)b * Q + s.n) * V;
    const float* drow = s.bonus ? trow : draft + ((size_t)b * gamma + s.n) * V;      // never read when bonus
    const double inv_st = 1.0 / s.s_t, inv_sd = 1.0 / s.s_d;
    float xt[kPickPerLane], xd[kPickPerLane];
#pragma unroll
    for (int j = 0; j < kPickPerLane / 4; ++j) {
        const int idx = base + j * 4;
        if (vec && idx + 3 < V) {
            const float4 a = *reinterpret_cast<const float4*>(trow + idx);
            xt[j * 4 + 0] = a.x; xt[j * 4 + 1] = a.y; xt[j * 4 + 2] = a.z; xt[j * 4 + 3] = a.w;
            if (!use_p) {
                const float4 d = *reinterpret_cast<const float4*>(drow + idx);
                xd[j * 4 + 0] = d.x; xd[j * 4 + 1] = d.y; xd[j * 4 + 2] = d.z; xd[j * 4 + 3] = d.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                xt[j * 4 + e] = (idx + e < V) ? trow[idx + e] : -INFINITY;
                if (!use_p) xd[j * 4 + e] = (idx + e < V) ? drow[idx + e] : -INFINITY;
            }
        }
    }
    double r[kPickPerLane];
    double tot = 0.0;
#pragma unroll
    for (int k = 0; k < kPickPerLane; ++k) {
        double v = 0.0;
        if (base + k < V) {
            const double p = prob_of(xt[k], s.m_t, inv_st, ts);
            v = use_p ? p : fmax(p - prob_of(xd[k], s.m_d, inv_sd, ts), 0.0);
        }
        r[k] = v; tot += v;
    }
    double run = wave_scan_incl(tot) - tot + prefix;
    int first = INT_MAX, last = -1;
#pragma unroll
    for (int k = 0; k < kPickPerLane; ++k) {
        run += r[k];
        if (r[k] > 0.0) last = base + k;
        if (first == INT_MAX && run > thr && base + k < V) first = base + k;
    }
    const unsigned long long hit2 = __ballot(first != INT_MAX), any2 = __ballot(last >= 0);
    int token = 0;
    if (hit2) token = __builtin_amdgcn_readlane(first, __ffsll((long long)hit2) - 1);
    else if (any2) token = __builtin_amdgcn_readlane(last, 63 - __clzll((long long)any2));
    if (lane == 0) out_tokens[b * Q + s.n] = token;
}

static inline int n_chunks(int V) { return (V + kAccChunk - 1) / kAccChunk; }

struct AcceptLayout { size_t part, sel, mass, total; };
static AcceptLayout accept_layout(int B, int gamma, int V) {
    AcceptLayout l;
    const size_t C = n_chunks(V), rows = (size_t)B * (2 * gamma + 1);
    l.part = 0;
    l.sel = align_up(l.part + rows * C * sizeof(RowPartial), 256);
    l.mass = align_up(l.sel + (size_t)B * sizeof(SeqSel), 256);
    l.total = align_up(l.mass + (size_t)B * C * sizeof(ChunkMass), 256);
    return l;
}


// ---- total variation distance between the two distributions of a row (paper Section 6) ----
struct RowStat { double m, s; };

// One wave per row: the chunk partials of pass 1 merged into the row's maximum and sum of exponentials.
__global__ __launch_bounds__(kAccThreads)
void tvd_rowstat_kernel(const RowPartial* __restrict__ part, int n_rows, int C, float scale2,
                        RowStat* __restrict__ stat) {
    const int lane = threadIdx.x % kWave;
    const int r = blockIdx.x * (kAccThreads / kWave) + threadIdx.x / kWave;
    if (r >= n_rows) return;
    const RowPartial* p = part + (size_t)r * C;
    float m = -INFINITY;
    for (int c = lane; c < C; c += kWave) m = fmaxf(m, p[c].m);
    m = wave_max(m);
    double s = 0.0;
    for (int c = lane; c < C; c += kWave)
        if (p[c].m > -INFINITY) s += p[c].s * (double)exp2f((p[c].m - m) * scale2);
    s = wave_sum(s);
    if (lane == 0) { RowStat o; o.m = (double)m; o.s = s; stat[r] = o; }
}

// One wave per (row, chunk): sum of |p - q| over the chunk's 1024 tokens, in double.
__global__ __launch_bounds__(kAccThreads)
void tvd_chunk_kernel(const float* __restrict__ target, const float* __restrict__ draft,
                      int rows, int V, int C, TempScale ts, int vec,
                      const RowStat* __restrict__ stat, double* __restrict__ chunk_abs) {
    const int lane = threadIdx.x % kWave;
    const int c = blockIdx.x * (kAccThreads / kWave) + threadIdx.x / kWave, r = blockIdx.y;
    if (c >= C) return;
    const RowStat st = stat[r], sd = stat[rows + r];
    const int base = c * kAccChunk;
    float xt[kAccPerLane], xd[kAccPerLane];
    load_chunk(target + (size_t)r * V, V, base, lane, vec, xt);
    load_chunk(draft + (size_t)r * V, V, base, lane, vec, xd);
    const double inv_st = 1.0 / st.s, inv_sd = 1.0 / sd.s;
    double a = 0.0;
#pragma unroll
    for (int k = 0; k < kAccPerLane; ++k)
        a += fabs(prob_of(xt[k], st.m, inv_st, ts) - prob_of(xd[k], sd.m, inv_sd, ts));
    a = wave_sum(a);
    if (lane == 0) chunk_abs[(size_t)r * C + c] = a;
}

// One wave per row: chunk sums added in a fixed order, halved.
__global__ __launch_bounds__(kAccThreads)
void tvd_final_kernel(const double* __restrict__ chunk_abs, int rows, int C, double* __restrict__ tvd) {
    const int lane = threadIdx.x % kWave;
    const int r = blockIdx.x * (kAccThreads / kWave) + threadIdx.x / kWave;
    if (r >= rows) return;
    double a = 0.0;
    for (int c = lane; c < C; c += kWave) a += chunk_abs[(size_t)r * C + c];
    a = wave_sum(a);
    if (lane == 0) tvd[r] = 0.5 * a;
}

struct TvdLayout { size_t part, stat, chunk, total; };
static TvdLayout tvd_layout(int rows, int V) {
    TvdLayout l;
    const size_t C = n_chunks(V);
    l.part = 0;
    l.stat = align_up(l.part + 2 * (size_t)rows * C * sizeof(RowPartial), 256);
    l.chunk = align_up(l.stat + 2 * (size_t)rows * sizeof(RowStat), 256);
    l.total = align_up(l.chunk + (size_t)rows * C * sizeof(double), 256);
    return l;
}

TempScale temp_scale(float temperature) {
    TempScale ts;
    ts.inv = 1.0 / (double)temperature;
    const double k2 = ts.inv * 1.4426950408889634074;      // log2(e) / T
    ts.hi = (float)k2;
    ts.lo = (float)(k2 - (double)ts.hi);
    return ts;
}

}  // namespace massv

using namespace massv;

extern "C" size_t massv_spec_accept_workspace(int32_t B, int32_t gamma, int32_t V) {
    if (B < 1 || gamma < 0 || gamma > kMaxGamma || V < 1) return 0;
    return accept_layout(B, gamma, V).total;
}

// Argument checks shared by the two entry points (everything except the scratch space).
static int check_accept_args(const float* target_logits, const float* draft_logits, const int32_t* draft_tokens,
                             const float* uniforms, float temperature, int32_t B, int32_t gamma, int32_t V,
                             const int32_t* n_accepted, const int32_t* out_tokens) {
    if (B < 1 || gamma < 0 || V < 1) return MASSV_EINVAL;
    if (!(temperature >= 0.f) || isinf(temperature)) return MASSV_EINVAL;     // also catches NaN
    if (!target_logits || !n_accepted || !out_tokens) return MASSV_EINVAL;
    if (gamma > 0 && !draft_tokens) return MASSV_EINVAL;
    const int greedy = (temperature == 0.f);
    if (!greedy && (!uniforms || (gamma > 0 && !draft_logits))) return MASSV_EINVAL;
    if (gamma > kMaxGamma) return MASSV_EUNSUPPORTED;
    if ((size_t)B * (2 * gamma + 1) > 65535) return MASSV_EUNSUPPORTED;       // grid.y limit of pass 1
    return MASSV_OK;
}

// The four launches of one call; `workspace` holds accept_layout(B, gamma, V).total bytes.
static int run_accept(const float* target_logits, const float* draft_logits, const int32_t* draft_tokens,
                      const float* uniforms, float temperature, int32_t B, int32_t gamma, int32_t V,
                      int32_t* n_accepted, int32_t* out_tokens, void* workspace, hipStream_t st) {
    const AcceptLayout lay = accept_layout(B, gamma, V);
    const int greedy = (temperature == 0.f);
    char* ws = (char*)workspace;
    RowPartial* part = (RowPartial*)(ws + lay.part);
    SeqSel* sel = (SeqSel*)(ws + lay.sel);
    ChunkMass* mass = (ChunkMass*)(ws + lay.mass);
    const int C = n_chunks(V), Q = gamma + 1;
    TempScale ts; ts.hi = 1.f; ts.lo = 0.f; ts.inv = 1.0;
    if (!greedy) ts = temp_scale(temperature);
    const int vec = (V % 4 == 0) && ((uintptr_t)target_logits % 16 == 0) &&
                    (greedy || (uintptr_t)draft_logits % 16 == 0);
    const int rows = greedy ? B * Q : B * (Q + gamma);

    launch_traced(MASSV_K_ACCEPT_STATS, accept_stats_kernel, dim3((C + kAccThreads / kWave - 1) / (kAccThreads / kWave), rows), dim3(kAccThreads), 0, st,
                  target_logits, draft_logits, B * Q, V, C, ts, greedy, vec, part);
    hipLaunchKernelGGL(accept_decide_kernel, dim3(B), dim3(kDecideThreads), 0, st,
                       target_logits, draft_logits, draft_tokens, uniforms, B, gamma, V, ts.inv,
                       ts.hi, greedy, (const RowPartial*)part, C, (const RowPartial*)(part + (size_t)B * Q * C), C,
                       sel, n_accepted, out_tokens);
    if (!greedy) {
        launch_traced(MASSV_K_RESIDUAL_MASS, residual_mass_kernel, dim3((C + kAccThreads / kWave - 1) / (kAccThreads / kWave), B), dim3(kAccThreads), 0, st,
                      target_logits, draft_logits, gamma, V, C, ts, vec, (const SeqSel*)sel, mass);
        hipLaunchKernelGGL(residual_pick_kernel, dim3(B), dim3(kWave), 0, st,
                           target_logits, draft_logits, uniforms, gamma, V, C, ts, vec, sel, mass, out_tokens);
    }
    return launch_status();
}

extern "C" int massv_spec_accept(const float* target_logits, const float* draft_logits,
                                 const int32_t* draft_tokens, const float* uniforms,
                                 float temperature, int32_t B, int32_t gamma, int32_t V,
                                 int32_t* n_accepted, int32_t* out_tokens,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_accept_args(target_logits, draft_logits, draft_tokens, uniforms, temperature, B, gamma, V,
                                     n_accepted, out_tokens);
    if (rc != MASSV_OK) return rc;
    if (!workspace || workspace_bytes < accept_layout(B, gamma, V).total) return MASSV_EWORKSPACE;
    return run_accept(target_logits, draft_logits, draft_tokens, uniforms, temperature, B, gamma, V, n_accepted,
                      out_tokens, workspace, (hipStream_t)stream);
}

// ---- the same call for callers that cannot allocate: scratch space inside the library ----
// A fixed array in device memory replaces the workspace argument.  Each GPU the library is used on holds its own
// copy of the array at its own address for the life of the process; the address is asked for once per device, with
// that device current, and kept.  In host code the array's name is only a handle for that query, never an address.
constexpr size_t kStaticScratchBytes = MASSV_SPEC_ACCEPT_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::atomic<void*> scratch_ptr[64];        // per device; zero-initialised

static int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MASSV_ELAUNCH;
    void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {                                   // two threads may both ask; they get the same answer
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MASSV_ELAUNCH;
        scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return MASSV_OK;
}

extern "C" size_t massv_spec_accept_static_limit(void) { return kStaticScratchBytes; }

extern "C" int massv_spec_accept_static(const float* target_logits, const float* draft_logits,
                                        const int32_t* draft_tokens, const float* uniforms,
                                        float temperature, int32_t B, int32_t gamma, int32_t V,
                                        int32_t* n_accepted, int32_t* out_tokens, void* stream) {
    int rc = check_accept_args(target_logits, draft_logits, draft_tokens, uniforms, temperature, B, gamma, V,
                               n_accepted, out_tokens);
    if (rc != MASSV_OK) return rc;
    if (accept_layout(B, gamma, V).total > kStaticScratchBytes) return MASSV_EUNSUPPORTED;   // use massv_spec_accept
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != MASSV_OK) return rc;
    // nothing has to start at zero: every record the later kernels read is written by an earlier kernel of this call
    return run_accept(target_logits, draft_logits, draft_tokens, uniforms, temperature, B, gamma, V, n_accepted,
                      out_tokens, ws, (hipStream_t)stream);
}

namespace massv {
// Target statistics come with the logits (one partial per row and workgroup of the vocabulary projection): pass 1
// streams the draft rows only; the rest of the call is the same four-kernel chain.
struct PrestatsLayout { size_t part_d, sel, mass, total; };
static PrestatsLayout prestats_layout(int B, int gamma, int V) {
    PrestatsLayout l;
    const size_t C = n_chunks(V);
    l.part_d = 0;
    l.sel = align_up(l.part_d + (size_t)B * gamma * C * sizeof(RowPartial), 256);
    l.mass = align_up(l.sel + (size_t)B * sizeof(SeqSel), 256);
    l.total = align_up(l.mass + (size_t)B * C * sizeof(ChunkMass), 256);
    return l;
}
size_t accept_prestats_bytes(int B, int gamma, int V) { return prestats_layout(B, gamma, V).total; }

int launch_accept_prestats(const float* target_logits, const RowPartial* part_t, int C_t, const float* draft_logits,
                           const int32_t* draft_tokens, const float* uniforms, float temperature, int B, int gamma, int V,
                           int32_t* n_accepted, int32_t* out_tokens, void* workspace, hipStream_t st) {
    const PrestatsLayout lay = prestats_layout(B, gamma, V);
    char* ws = (char*)workspace;
    RowPartial* part_d = (RowPartial*)(ws + lay.part_d);
    SeqSel* sel = (SeqSel*)(ws + lay.sel);
    ChunkMass* mass = (ChunkMass*)(ws + lay.mass);
    const int C = n_chunks(V);
    const TempScale ts = temp_scale(temperature);
    const int vec = (V % 4 == 0) && ((uintptr_t)target_logits % 16 == 0) && (gamma == 0 || (uintptr_t)draft_logits % 16 == 0);
    const int wpb = kAccThreads / kWave;
    if (gamma > 0)
        launch_traced(MASSV_K_ACCEPT_STATS, accept_stats_kernel, dim3((C + wpb - 1) / wpb, B * gamma), dim3(kAccThreads), 0, st,
                      (const float*)nullptr, draft_logits, 0, V, C, ts, 0, vec, part_d);
    hipLaunchKernelGGL(accept_decide_kernel, dim3(B), dim3(kDecideThreads), 0, st,
                       target_logits, draft_logits, draft_tokens, uniforms, B, gamma, V, ts.inv, ts.hi, 0,
                       part_t, C_t, (const RowPartial*)part_d, C, sel, n_accepted, out_tokens);
    launch_traced(MASSV_K_RESIDUAL_MASS, residual_mass_kernel, dim3((C + wpb - 1) / wpb, B), dim3(kAccThreads), 0, st,
                  target_logits, draft_logits, gamma, V, C, ts, vec, (const SeqSel*)sel, mass);
    hipLaunchKernelGGL(residual_pick_kernel, dim3(B), dim3(kWave), 0, st,
                       target_logits, draft_logits, uniforms, gamma, V, C, ts, vec, sel, mass, out_tokens);
    return launch_status();
}

int launch_accept_decide_greedy(const RowPartial* part, int C, const int32_t* draft_tokens, int B, int gamma, int V,
                                int32_t* n_accepted, int32_t* out_tokens, hipStream_t st) {
    hipLaunchKernelGGL(accept_decide_kernel, dim3(B), dim3(kDecideThreads), 0, st, (const float*)nullptr, (const float*)nullptr,
                       draft_tokens, (const float*)nullptr, B, gamma, V, 1.0, 1.f, 1, part, C, (const RowPartial*)nullptr, 0,
                       (SeqSel*)nullptr, n_accepted, out_tokens);
    return launch_status();
}

__global__ void commit_tokens_kernel(const int* __restrict__ n_accepted, const int* __restrict__ out_tokens,
                                     int* __restrict__ kv_len, int* __restrict__ last_token, int B, int gamma) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int n = n_accepted[b];
    n = n < 0 ? 0 : (n > gamma ? gamma : n);
    if (last_token) last_token[b] = out_tokens[b * (gamma + 1) + n];
    kv_len[b] += n + 1;
}
}  // namespace massv

extern "C" int massv_commit_tokens(const int32_t* n_accepted, const int32_t* out_tokens, int32_t* kv_len,
                                   int32_t* last_token, int32_t B, int32_t gamma, void* stream) {
    if (!n_accepted || !out_tokens || !kv_len || B < 1 || gamma < 0) return MASSV_EINVAL;
    hipLaunchKernelGGL(commit_tokens_kernel, dim3((B + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       n_accepted, out_tokens, kv_len, last_token, B, gamma);
    return launch_status();
}

extern "C" size_t massv_spec_tvd_workspace(int32_t rows, int32_t V) {
    if (rows < 1 || rows > 32767 || V < 1) return 0;
    return tvd_layout(rows, V).total;
}

extern "C" int massv_spec_tvd(const float* target_logits, const float* draft_logits, float temperature,
                              int32_t rows, int32_t V, double* tvd,
                              void* workspace, size_t workspace_bytes, void* stream) {
    if (rows < 1 || V < 1) return MASSV_EINVAL;
    if (!(temperature > 0.f) || isinf(temperature)) return MASSV_EINVAL;      // also catches NaN
    if (!target_logits || !draft_logits || !tvd) return MASSV_EINVAL;
    if (rows > 32767) return MASSV_EUNSUPPORTED;                              // grid.y limit of pass 1
    const TvdLayout lay = tvd_layout(rows, V);
    if (!workspace || workspace_bytes < lay.total) return MASSV_EWORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    RowPartial* part = (RowPartial*)(ws + lay.part);
    RowStat* stat = (RowStat*)(ws + lay.stat);
    double* chunk_abs = (double*)(ws + lay.chunk);
    const int C = n_chunks(V);
    const TempScale ts = temp_scale(temperature);
    const int vec = (V % 4 == 0) && ((uintptr_t)target_logits % 16 == 0) && ((uintptr_t)draft_logits % 16 == 0);
    const int wpb = kAccThreads / kWave;

    hipLaunchKernelGGL(accept_stats_kernel, dim3((C + wpb - 1) / wpb, 2 * rows), dim3(kAccThreads), 0, st,
                       target_logits, draft_logits, rows, V, C, ts, 0, vec, part);
    hipLaunchKernelGGL(tvd_rowstat_kernel, dim3((2 * rows + wpb - 1) / wpb), dim3(kAccThreads), 0, st,
                       (const RowPartial*)part, 2 * rows, C, ts.hi, stat);
    hipLaunchKernelGGL(tvd_chunk_kernel, dim3((C + wpb - 1) / wpb, rows), dim3(kAccThreads), 0, st,
                       target_logits, draft_logits, rows, V, C, ts, vec, (const RowStat*)stat, chunk_abs);
    hipLaunchKernelGGL(tvd_final_kernel, dim3((rows + wpb - 1) / wpb), dim3(kAccThreads), 0, st,
                       (const double*)chunk_abs, rows, C, tvd);
    return launch_status();
}
