// Projections of the verify forward: Y[M][N] = X[M][K] W[N][K]^T with M = B*(gamma+1)
// rows (6 .. 64).  At these row counts every weight byte is used for only M
// multiply-adds, far below the machine balance, so the kernels are weight
// STREAMERS: the job is to pull W through HBM once at full bandwidth; the
// matrix cores only have to keep up.
//
// bf16 kernel (gemm_stream_kernel), shaped by measurements on MI355X:
//   * v_mfma_f32_16x16x32_bf16 with W as the A operand (16 output features x
//     32 k) and X as the B operand (32 k x 16 rows): every lane's W operand is
//     one 16-byte global load.  W is kept in the library's streaming layout
//     (massv_weight_pack): per 16-feature tile, the operands of consecutive
//     k-steps lie back to back, so a wave's load is a contiguous 1 KB of whole
//     cache lines and a tile is one sequential stream.  That allows the
//     non-temporal hint; measured against row-major W (64-byte pieces of 16
//     rows per load) the same kernel went from 4.4 to 5.2 TB/s on the gate/up
//     shape.
//   * X comes from L2, and those reads -- not HBM -- were the first limiter.
//     Two remedies: X is kept in operand order (packed_index) so a wave reads it
//     as contiguous 1 KB blocks, and a wave owns NT = 4..10 feature tiles per
//     chunk so that each X block it loads is used NT times.
//   * Each of the wave's NT tiles has its own register slot: right after the
//     matrix instructions of tile t for chunk c have been issued, the loads of
//     tile t for the wave's next chunk go out.  This keeps about NT-1 tile
//     loads (4 KB each) in flight per wave with ONE set of W registers; X is
//     double-buffered.
//   * A workgroup is 4 waves that split its K range in interleaved chunks of
//     four 32-element steps (so the workgroup reads contiguous 16 KB runs of
//     a tile; giving each wave one contiguous quarter instead measured 1%
//     slower on the whole step) with the ragged last round dealt evenly, and
//     are summed through LDS in wave order (deterministic).
//   * The grid is sized to at most one workgroup per CU (256) wherever
//     possible: with a register-heavy streaming kernel a second partial round
//     of workgroups costs as much as a full one.  Wide outputs (gate/up,
//     lm_head) choose NT for that; narrow outputs (q/k/v, O, down) split K
//     over gridDim.y slabs, write fp32 partial sums and leave the slab sum to
//     the row-wise kernel that follows anyway (bias + rotary + cache append,
//     residual + RMSNorm).
//   * Epilogues: fp32 partial sums, act(gate)*up for interleaved gate/up tiles
//     (written in operand order for the down projection), fp32 logits.
// f32 kernel: one wave per output feature, plain FMAs, for the small fp32
// configuration.
#include "kernels.h"

#include <limits.h>
#include <atomic>

namespace massv {

constexpr int kGemmWaves = 4;            // waves per workgroup (K split)
constexpr int kCUs = 256;

struct GemmDev {
    const bf16_t* x;
    const bf16_t* w[3];
    int tiles[3];            // 16-feature tiles per matrix
    void* y;
    void* stats;             // EPI_LOGITS_STATS: RowPartial[M][gridDim.x]
    float ts_hi, ts_lo;      // EPI_LOGITS_STATS: log2(e)/T in two floats
    int M, K, ldy;           // ldy: elements per output row
    int act;
    int unit_base, unit_rem; // balanced split of the tile units over gridDim.x: the first unit_rem workgroups own unit_base+1
    size_t slab_stride;      // elements between the partial sums of consecutive K slabs
};

// Gated-MLP activations through the hardware exp2 and reciprocal (about 1e-6 relative error, the result is
// rounded to bf16): the library versions with exact division and tanhf made the projection's epilogue a few
// thousand instructions long, 3 us of a 46 us launch.  0.5 (1 + tanh(u)) is sigmoid(2u).
__device__ inline float fast_sigmoid(float x) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ inline float gemm_act(float x, int act) {
    if (act == MASSV_ACT_SILU) return x * fast_sigmoid(x);
    const float c = 0.7978845608028654f;
    return x * fast_sigmoid(2.0f * c * (x + 0.044715f * x * x * x));
}

// 2^(d * log2(e)/T) for d <= 0 (a logit minus a running maximum; -inf and NaN from -inf - -inf give 0).
__device__ inline float exp2_scaled(float d, float hi, float lo) {
    d = fmaxf(d, -3.0e38f);
    return __builtin_amdgcn_exp2f(fmaf(d, lo, d * hi));
}

__device__ inline bf16x8 ld8(const bf16_t* p, bool ok) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    return ok ? *reinterpret_cast<const bf16x8*>(p) : z;
}
__device__ inline bf16x8 ld8_stream(const bf16_t* p, bool ok) {      // weights: read once, whole lines
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    return ok ? ldg_stream(reinterpret_cast<const bf16x8*>(p)) : z;
}


// Tiles of LDS reduced per round: at most 128 KB of fp32 fragments at a time -- one round for every shape built
// (10 tiles x 3 row tiles x 4 waves = 120 KB); rounds of 48 KB cost two more barrier pairs per launch.
template <int MT, int NT>
struct ReduceGroup {
    static constexpr int kMax = 128 / (MT * kGemmWaves);
    static constexpr int raw = (NT < kMax) ? NT : kMax;
    static constexpr int value = (raw >= 2) ? (raw / 2) * 2 : 1;     // even, so gate/up pairs stay together
};

template <int MT, int NT, int EPI>
__global__ __launch_bounds__(kGemmWaves * kWave)
void gemm_stream_kernel(GemmDev g) {
    constexpr int WK = kGemmWaves;
    constexpr bool gated = (EPI == EPI_GATED);
    extern __shared__ floatx4 red[];                 // [WK][GRP*MT][64]
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int lr = lane % 16, lc = lane / 16;
    const int K = g.K;

    // ---- the NT feature tiles of this workgroup ----
    const bf16_t* wrow[NT];
    bool nvalid[NT];
    int ocol[NT];
    // a unit is one tile (a gate/up tile pair for the gated epilogue); units are dealt to the workgroups
    // as evenly as possible, so a workgroup may own fewer than its NT tile slots
    constexpr int UT = gated ? 2 : 1;
    // split-K launches: the slab is the fast grid index, so that the workgroups of one slab -- which read the same
    // piece of X -- have linear indices that are congruent modulo the slab count and fall on the same XCDs
    constexpr bool SLAB_FAST = (EPI == EPI_PARTIAL);
    const int bx = SLAB_FAST ? blockIdx.y : blockIdx.x;
    const int n_slabs = SLAB_FAST ? gridDim.x : gridDim.y;
    const int unit0 = bx * g.unit_base + (bx < g.unit_rem ? bx : g.unit_rem);
    const int n_units = g.unit_base + (bx < g.unit_rem ? 1 : 0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int t = unit0 * UT + nt;
        const bool owned = nt < n_units * UT;
        int seg, local;
        if (gated) {                                  // tiles alternate gate, up of one 16-feature group
            seg = t & 1; local = t >> 1;
            nvalid[nt] = owned && local < g.tiles[0];
            ocol[nt] = local * 16;
        } else {
            if (t < g.tiles[0]) { seg = 0; local = t; }
            else if (t < g.tiles[0] + g.tiles[1]) { seg = 1; local = t - g.tiles[0]; }
            else { seg = 2; local = t - g.tiles[0] - g.tiles[1]; }
            nvalid[nt] = owned && t < g.tiles[0] + g.tiles[1] + g.tiles[2];
            ocol[nt] = t * 16;
        }
        if (!nvalid[nt]) { seg = 0; local = 0; }
        wrow[nt] = g.w[seg] + (size_t)local * (K / 32) * 512 + lane * 8;      // tile `local` of the streaming layout
    }
    // X in operand order: the B operand of (k-step ks, row tile mt) is the 1 KB block ((ks*MT + mt)*64 + lane)*8
    const bf16_t* xlane = g.x + (size_t)lane * 8;

    floatx4 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    // K is dealt in 32-element MFMA steps.  The steps of the launch are split evenly over the gridDim.y slabs.  Inside
    // a slab the waves take chunks of four steps in turn (so the workgroup reads contiguous 16 KB runs of a tile), and
    // the last, incomplete round of 16 steps is split evenly: no wave does more than one step above the average.
    const int n_steps = K / 32;
    const int sb = n_steps / n_slabs, sr = n_steps % n_slabs;
    const int by = SLAB_FAST ? blockIdx.x : blockIdx.y;
    const int s_begin = by * sb + (by < sr ? by : sr);
    const int s_count = sb + (by < sr ? 1 : 0);
    const int rounds = s_count / (4 * WK);
    const int tail = s_count - rounds * 4 * WK;
    const int tb = tail / WK, tr = tail % WK;
    const int t_len = tb + (wave < tr ? 1 : 0);                              // 0..4 steps
    const int t_k0 = s_begin + rounds * 4 * WK + wave * tb + (wave < tr ? wave : tr);
    const int n_it = rounds + (t_len > 0 ? 1 : 0);
    auto k0_of = [&](int it) { return it < rounds ? s_begin + (it * WK + wave) * 4 : t_k0; };
    auto cnt_of = [&](int it) { return it < rounds ? 4 : t_len; };

    bf16x8 a[NT][4];
    bf16x8 xb[2][MT][4];
    auto wload = [&](int nt, int k0, int cnt) {
#pragma unroll
        for (int j = 0; j < 4; ++j) a[nt][j] = ld8_stream(wrow[nt] + (size_t)(k0 + j) * 512, nvalid[nt] && j < cnt);
    };
    auto xload = [&](int buf, int k0, int cnt) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                xb[buf][mt][j] = ld8(xlane + (size_t)((k0 + j) * MT + mt) * 512, j < cnt);
    };
    if (n_it > 0) {
        xload(0, k0_of(0), cnt_of(0));
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wload(nt, k0_of(0), cnt_of(0));
    }
    int par = 0;
    for (int it = 0; it < n_it; ++it, par ^= 1) {
        const bool more = it + 1 < n_it;
        const int nx = k0_of(it + 1), ncnt = cnt_of(it + 1);
        if (more) { if (par) xload(0, nx, ncnt); else xload(1, nx, ncnt); }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[nt][j], par ? xb[1][mt][j] : xb[0][mt][j],
                                                                         acc[nt][mt], 0, 0, 0);
            if (more) wload(nt, nx, ncnt);            // refill this tile's slot for the wave's next four steps
        }
    }

    // EPI_ARGMAX, EPI_LOGITS_STATS: largest summed output (and its lowest column) seen by this lane for row
    // 16 mt + lr; EPI_LOGITS_STATS: also the sum of exp((x - largest)/T) over what the lane has seen (rescaled
    // whenever the largest moves)
    constexpr bool STATS = (EPI == EPI_LOGITS_STATS);
    float best_v[MT], sum_e[MT];
    int best_i[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { best_v[mt] = -INFINITY; best_i[mt] = INT_MAX; sum_e[mt] = 0.f; }

    // ---- sum the waves through LDS in wave order, GRP tiles per round ----
    constexpr int GRP = ReduceGroup<MT, NT>::value;
    for (int g0 = 0; g0 < NT; g0 += GRP) {
        if (g0) __syncthreads();
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (nt >= g0 && nt < g0 + GRP)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    red[(wave * GRP * MT + (nt - g0) * MT + mt) * kWave + lane] = acc[nt][mt];
        __syncthreads();
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (nt < g0 || nt >= g0 + GRP) continue;
            if (gated && (nt & 1)) continue;                    // the up tile is consumed with its gate tile
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int item = gated ? ((nt - g0) / 2) * MT + mt : (nt - g0) * MT + mt;
                if (item % WK != wave || !nvalid[nt]) continue;  // items are dealt round-robin to the waves
                const int f = (nt - g0) * MT + mt;
                floatx4 s = red[f * kWave + lane];
                for (int w = 1; w < WK; ++w) s += red[(w * GRP * MT + f) * kWave + lane];
                const int m = mt * 16 + lr;
                const int col = ocol[nt] + lc * 4;               // 4 consecutive output features
                if (gated) {
                    constexpr int UP = (NT > 1) ? MT : 0;        // fragment of the paired up tile
                    floatx4 u = red[(f + UP) * kWave + lane];
                    for (int w = 1; w < WK; ++w) u += red[(w * GRP * MT + f + UP) * kWave + lane];
                    if (m < g.M) {
                        bf16x4 o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[i] = (bf16_t)(gemm_act(s[i], g.act) * u[i]);
                        *reinterpret_cast<bf16x4*>((bf16_t*)g.y + packed_index(m, col, MT)) = o;
                    }
                } else if (EPI == EPI_ARGMAX || STATS) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {                 // ascending columns: a tie keeps the lower one
                        if constexpr (STATS) {
                            if (s[i] > best_v[mt]) sum_e[mt] = sum_e[mt] * exp2_scaled(best_v[mt] - s[i], g.ts_hi, g.ts_lo) + 1.f;
                            else sum_e[mt] += exp2_scaled(s[i] - best_v[mt], g.ts_hi, g.ts_lo);
                        }
                        if (s[i] > best_v[mt] || (s[i] == best_v[mt] && col + i < best_i[mt])) { best_v[mt] = s[i]; best_i[mt] = col + i; }
                    }
                    if (STATS && m < g.M) *reinterpret_cast<floatx4*>((float*)g.y + (size_t)m * g.ldy + col) = s;
                } else if (m < g.M) {
                    float* dst = (float*)g.y + (EPI == EPI_PARTIAL ? (size_t)by * g.slab_stride : 0) +
                                 (size_t)m * g.ldy + col;
                    *reinterpret_cast<floatx4*>(dst) = s;
                }
            }
        }
    }
    if constexpr (EPI == EPI_ARGMAX || STATS) {
        // lanes of the four column groups of a row, then the four waves, then one record per row and workgroup
        __syncthreads();                                         // the reduction buffer is free
        float* bv = reinterpret_cast<float*>(red);               // [WK][MT*16]
        int* bi = reinterpret_cast<int*>(bv + WK * MT * 16);
        float* bs = reinterpret_cast<float*>(bi + WK * MT * 16);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float v = best_v[mt], se = sum_e[mt]; int i = best_i[mt];
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                const float ov = __shfl_xor(v, o, kWave);
                const int oi = __shfl_xor(i, o, kWave);
                if constexpr (STATS) {
                    const float os = __shfl_xor(se, o, kWave);
                    const float mn = fmaxf(v, ov);
                    se = (mn == -INFINITY) ? 0.f : se * exp2_scaled(v - mn, g.ts_hi, g.ts_lo) + os * exp2_scaled(ov - mn, g.ts_hi, g.ts_lo);
                }
                if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
            }
            if (lc == 0) { bv[wave * MT * 16 + mt * 16 + lr] = v; bi[wave * MT * 16 + mt * 16 + lr] = i; bs[wave * MT * 16 + mt * 16 + lr] = se; }
        }
        __syncthreads();
        if (tid < MT * 16 && tid < g.M) {
            float v = bv[tid]; int i = bi[tid];
            for (int w = 1; w < WK; ++w) {
                const float ov = bv[w * MT * 16 + tid]; const int oi = bi[w * MT * 16 + tid];
                if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
            }
            RowPartial r; r.m = v; r.arg = i; r.s = 0.0;
            if constexpr (STATS) {                               // wave order, in double
                for (int w = 0; w < WK; ++w)
                    if (bv[w * MT * 16 + tid] > -INFINITY)
                        r.s += (double)bs[w * MT * 16 + tid] * (double)exp2_scaled(bv[w * MT * 16 + tid] - v, g.ts_hi, g.ts_lo);
            }
            reinterpret_cast<RowPartial*>(STATS ? g.stats : g.y)[(size_t)tid * gridDim.x + blockIdx.x] = r;
        }
    }
}

// ---------------------------------------------------------------------------
// f32 kernel: grid (N, ceil(M/8)), one wave per output feature and 8 rows.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kWave)
void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
                     const float* residual, float* y, int M, int K, int ldy, int col0) {
    const int n = blockIdx.x, m0 = blockIdx.y * 8, lane = threadIdx.x;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float* wr = w + (size_t)n * K;
    for (int k = lane; k < K; k += kWave) {
        const float wv = wr[k];
#pragma unroll
        for (int r = 0; r < 8; ++r)
            if (m0 + r < M) acc[r] += x[(size_t)(m0 + r) * K + k] * wv;
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const float s = wave_sum(acc[r]);
        if (lane == 0 && m0 + r < M) {
            const size_t o = (size_t)(m0 + r) * ldy + col0 + n;
            float v = s + (bias ? bias[n] : 0.f);
            if (residual) v += residual[o];
            y[o] = v;
        }
    }
}

__global__ void gated_rows_f32_kernel(const float* __restrict__ gu, float* __restrict__ h, int M, int F, int act) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)M * F) return;
    const size_t m = i / F, f = i % F;
    const float gv = gu[m * 2 * F + f], uv = gu[m * 2 * F + F + f];
    float a;
    if (act == MASSV_ACT_SILU) a = gv / (1.0f + expf(-gv));
    else a = 0.5f * gv * (1.0f + tanhf(0.7978845608028654f * (gv + 0.044715f * gv * gv * gv)));
    h[i] = a * uv;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int n_total(const GemmArgs& g) { return g.n[0] + g.n[1] + g.n[2]; }

int gemm_supported(const GemmArgs& g) {
    if (g.M < 1 || g.K < 1 || g.n[0] < 1) return MASSV_EINVAL;
    if (g.epilogue == EPI_GATED && (g.n[1] != g.n[0] || g.n[2] != 0)) return MASSV_EINVAL;
    if (g.dtype == MASSV_F32)
        return (g.epilogue == EPI_PARTIAL || g.epilogue == EPI_ARGMAX || g.epilogue == EPI_LOGITS_STATS) ? MASSV_EINVAL : MASSV_OK;
    if (g.epilogue == EPI_LOGITS_STATS && (!g.stats || !(g.temperature > 0.f))) return MASSV_EINVAL;
    if (g.epilogue == EPI_STORE || g.epilogue == EPI_RESIDUAL) return MASSV_EINVAL;   // bf16 goes through partial sums
    if (g.M > MASSV_MAX_ROWS) return MASSV_EUNSUPPORTED;
    if (g.K % 32) return MASSV_EUNSUPPORTED;
    for (int s = 0; s < 3; ++s)
        if (g.n[s] % 16) return MASSV_EUNSUPPORTED;
    return MASSV_OK;
}

// Narrow outputs (fewer than 256 workgroups at full K): K is cut into slabs and the slab sums are left to the
// row-wise kernel that follows.  Tiles per wave and slabs are chosen by an estimate of the launch plus its share of
// that kernel, in microseconds, fitted to sweeps of the three split projections of the 7B-shaped layer (M = 48):
//   weights at 6.5 TB/s, stretched when fewer than 256 workgroups pull them;
//   X, re-read from L2 once per workgroup column: (T / nt) * K/32 * MT KB, at 14 TB/s;
//   0.8 us per MB of partial sums (written here, read back by the next kernel).
// Measured against the earlier rule "as many slabs as fill 256 workgroups, largest tile count": q/k/v (8 tiles, 7
// slabs) -> (4, 3) -1.9 us, output projection (7, 7) -> (4, 4) -1.0 us, down projection (7, 8) unchanged.
static GemmPlan plan_split(const GemmArgs& g, int mt, int T) {
    GemmPlan best = {0, 1, 0};
    const int n_steps = g.K / 32;
    int max_slabs = n_steps / kGemmWaves; if (max_slabs < 1) max_slabs = 1; if (max_slabs > 32) max_slabs = 32;   // a step per wave at least
    const double w_us = (double)n_total(g) * g.K * 2.0 / 6.5e6;
    const double slab_us = (double)(mt * 16) * n_total(g) * 4.0 / 1e6 * 0.8;
    static const int cand[] = {8, 7, 4};
    double best_t = 1e30;
    for (int nt : cand) {
        if (mt == 4 && nt > 4) continue;                       // register budget of four row tiles
        const int groups = (T + nt - 1) / nt;
        if (groups >= kCUs) continue;
        const double x_us = (double)groups * n_steps * mt * 1024.0 / 1e6 * 0.07;
        for (int slabs = 1; slabs <= max_slabs && groups * slabs <= kCUs; ++slabs) {
            const double t = w_us * (1.0 + 0.44 * ((double)kCUs / (groups * slabs) - 1.0)) + x_us + slabs * slab_us;
            if (t < best_t) { best_t = t; best.nt = nt; best.slabs = slabs; best.groups = groups; }
        }
    }
    return best;
}

// Tiles per wave and K slabs for one launch.  T: 16-feature tiles to produce.
//   wide output  (>= 256 groups): slabs = 1, NT chosen so that the last round of workgroups is as full as possible;
//   narrow output with the partial-sum epilogue: plan_split; the kernel deals the K/32 steps evenly over the slabs.
GemmPlan gemm_plan(const GemmArgs& g) {
    GemmPlan best = {0, 1, 0};
    if (g.dtype != MASSV_BF16) return best;
    const int mt = (g.M + 15) / 16;
    const int T = (g.epilogue == EPI_GATED) ? 2 * (g.n[0] / 16) : n_total(g) / 16;
    if (g.epilogue == EPI_PARTIAL && (T + 3) / 4 < kCUs) return plan_split(g, mt, T);
    // wide output (or a partial-sum output wide enough for 256 workgroups at full K): one slab
    static const int cand_partial[] = {8, 7, 4}, cand_gated[] = {10, 8, 4}, cand_logits[] = {10, 8, 4};
    const int* cand = g.epilogue == EPI_GATED ? cand_gated : (g.epilogue == EPI_LOGITS || g.epilogue == EPI_ARGMAX || g.epilogue == EPI_LOGITS_STATS) ? cand_logits : cand_partial;
    double best_score = -1.0;
    for (int i = 0; i < 3; ++i) {
        int nt = cand[i];
        if (mt == 4 && nt > 4) continue;                       // register budget of four row tiles
        const int ut = (g.epilogue == EPI_GATED) ? 2 : 1;      // tiles per unit
        int groups = (T + nt - 1) / nt;
        if (groups < kCUs) {                                    // one round: spread the units over as many CUs as there are
            const int units = T / ut;                           // (never a partial-sum launch: those went to plan_split)
            groups = units < kCUs ? units : kCUs;
        }
        const int rounds = (groups + kCUs - 1) / kCUs;
        if (rounds > 1 && rounds * kCUs <= T / ut) groups = rounds * kCUs;     // full rounds: the units are dealt evenly over them
        const double eff = (double)T / ((double)nt * rounds * kCUs);
        const double score = eff + 0.004 * nt;                 // near ties go to the larger tile count (less X traffic)
        if (score > best_score) { best_score = score; best.nt = nt; best.slabs = 1; best.groups = groups; }
    }
    return best;
}

size_t gemm_partial_bytes(const GemmArgs& g) {
    if (g.dtype != MASSV_BF16 || g.epilogue != EPI_PARTIAL) return 0;
    const GemmPlan p = gemm_plan(g);
    return (size_t)p.slabs * ((g.M + 15) / 16 * 16) * n_total(g) * sizeof(float);
}

template <int MT, int NT, int EPI>
static int launch_stream(const GemmDev& d, const GemmPlan& p, int kid, hipStream_t st) {
    constexpr int GRP = ReduceGroup<MT, NT>::value;
    const size_t lds = (size_t)kGemmWaves * GRP * MT * kWave * sizeof(floatx4);
    if (lds > 48 * 1024) {                       // more dynamic LDS than a kernel may use by default
        static std::atomic<bool> ready[64];       // zero-initialised; calls may come from several threads
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MASSV_ELAUNCH;
        if (!ready[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute((const void*)gemm_stream_kernel<MT, NT, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds) != hipSuccess) return MASSV_ELAUNCH;
            ready[dev].store(true, std::memory_order_release);
        }
    }
    const dim3 grid = (EPI == EPI_PARTIAL) ? dim3(p.slabs, p.groups) : dim3(p.groups, p.slabs);
    launch_traced(kid, gemm_stream_kernel<MT, NT, EPI>, grid, dim3(kGemmWaves * kWave), lds, st, d);
    return MASSV_OK;
}

template <int MT, int EPI>
static int launch_stream_nt(const GemmDev& d, const GemmPlan& p, int kid, hipStream_t st) {
    switch (p.nt) {
        case 4: return launch_stream<MT, 4, EPI>(d, p, kid, st);
        case 7: if constexpr (EPI == EPI_PARTIAL && MT <= 3) return launch_stream<MT, 7, EPI>(d, p, kid, st); break;
        case 8: if constexpr (MT <= 3) return launch_stream<MT, 8, EPI>(d, p, kid, st); break;
        case 10: if constexpr (EPI != EPI_PARTIAL && MT <= 3) return launch_stream<MT, 10, EPI>(d, p, kid, st); break;
    }
    return MASSV_EUNSUPPORTED;
}

template <int EPI>
static int launch_stream_epi(const GemmDev& d, int M, const GemmPlan& p, int kid, hipStream_t st) {
    switch ((M + 15) / 16) {
        case 1: return launch_stream_nt<1, EPI>(d, p, kid, st);
        case 2: return launch_stream_nt<2, EPI>(d, p, kid, st);
        case 3: return launch_stream_nt<3, EPI>(d, p, kid, st);
        case 4: return launch_stream_nt<4, EPI>(d, p, kid, st);
    }
    return MASSV_EUNSUPPORTED;
}

int launch_gemm(const GemmArgs& g, hipStream_t st) {
    const int rc = gemm_supported(g);
    if (rc != MASSV_OK) return rc;
    const int N = n_total(g);
    if (g.dtype == MASSV_F32) {
        const bool gated = g.epilogue == EPI_GATED;
        float* y = gated ? (float*)g.scratch : (float*)g.y;
        const int ldy = gated ? 2 * g.n[0] : N;
        int col = 0;
        for (int s = 0; s < 3; ++s) {
            if (!g.n[s]) continue;
            const float* res = (g.epilogue == EPI_RESIDUAL) ? (const float*)g.residual : nullptr;
            hipLaunchKernelGGL(gemm_f32_kernel, dim3(g.n[s], (g.M + 7) / 8), dim3(kWave), 0, st,
                               (const float*)g.x, (const float*)g.w[s], (const float*)g.bias[s], res, y, g.M, g.K, ldy, col);
            col += g.n[s];
        }
        if (gated) {
            const size_t n = (size_t)g.M * g.n[0];
            hipLaunchKernelGGL(gated_rows_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                               (const float*)g.scratch, (float*)g.y, g.M, g.n[0], g.act);
        }
        return launch_status();
    }
    const GemmPlan p = gemm_plan(g);
    GemmDev d;
    d.x = (const bf16_t*)g.x;
    for (int s = 0; s < 3; ++s) { d.w[s] = (const bf16_t*)g.w[s]; d.tiles[s] = g.n[s] / 16; }
    d.y = g.y;
    d.stats = g.stats;
    d.ts_hi = 1.f; d.ts_lo = 0.f;
    if (g.epilogue == EPI_LOGITS_STATS) { const TempScale ts = temp_scale(g.temperature); d.ts_hi = ts.hi; d.ts_lo = ts.lo; }
    d.M = g.M; d.K = g.K;
    d.ldy = (g.epilogue == EPI_GATED) ? g.n[0] : N;
    d.act = g.act;
    {
        const int ut = (g.epilogue == EPI_GATED) ? 2 : 1;
        const int units = ((g.epilogue == EPI_GATED) ? 2 * d.tiles[0] : N / 16) / ut;
        d.unit_base = units / p.groups;
        d.unit_rem = units % p.groups;
        if ((d.unit_base + (d.unit_rem ? 1 : 0)) * ut > p.nt) return MASSV_EUNSUPPORTED;     // cannot happen with gemm_plan's groups
    }
    d.slab_stride = (size_t)((g.M + 15) / 16 * 16) * N;
    int rc2 = MASSV_EUNSUPPORTED;
    switch (g.epilogue) {
        case EPI_PARTIAL: rc2 = launch_stream_epi<EPI_PARTIAL>(d, g.M, p, g.kid, st); break;
        case EPI_GATED: rc2 = launch_stream_epi<EPI_GATED>(d, g.M, p, g.kid, st); break;
        case EPI_LOGITS: rc2 = launch_stream_epi<EPI_LOGITS>(d, g.M, p, g.kid, st); break;
        case EPI_ARGMAX: rc2 = launch_stream_epi<EPI_ARGMAX>(d, g.M, p, g.kid, st); break;
        case EPI_LOGITS_STATS: rc2 = launch_stream_epi<EPI_LOGITS_STATS>(d, g.M, p, g.kid, st); break;
    }
    if (rc2 != MASSV_OK) return rc2;
    return launch_status();
}

}  // namespace massv
