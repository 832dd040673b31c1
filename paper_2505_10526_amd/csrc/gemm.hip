// Projections of the verify forward: Y[M][N] = X[M][K] W[N][K]^T with M = B*(gamma+1)
// rows (6 .. 64).  At these row counts every weight byte is used for only M
// multiply-adds, far below the machine balance, so the kernels are weight
// STREAMERS: the job is to pull W through HBM once at full bandwidth; the
// matrix cores only have to keep up.
//
// bf16 kernel (gemm_skinny_kernel):
//   * v_mfma_f32_16x16x32_bf16 with W as the A operand (16 output features x
//     32 k) and X as the B operand (32 k x 16 rows): every lane's operand is one
//     16-byte global load from a row of W (or X); four lanes cover 64
//     contiguous bytes of a row and the four k-steps of a chunk cover 256.
//   * A wave owns NT feature tiles x all MT row tiles; the WK waves of a
//     workgroup split K in interleaved 128-element chunks (so the workgroup
//     reads contiguous row segments) and are summed through LDS in wave order
//     (deterministic).  WK is raised for the projections with few output
//     features (O, down) so that the grid still fills 256 CUs without a
//     second pass over HBM partials.
//   * Loads of the next chunk are issued before the matrix instructions of the
//     current one (two register buffers).
//   * X (M x K bf16, at most a few MB) is re-read by every workgroup from L2.  It
//     is kept in operand order (packed_index) so that these reads are contiguous
//     1 KB blocks; its producers (RMSNorm, attention, the gated epilogue) write
//     that order directly.
//   * Epilogues: bias + store, residual add, act(gate)*up for interleaved
//     gate/up tiles, fp32 logits.
// f32 kernel: one wave per output feature, plain FMAs, for the small fp32
// configuration.
#include "kernels.h"

namespace massv {

struct GemmDev {
    const bf16_t* x;
    const bf16_t* w[3];
    const bf16_t* bias[3];
    int tiles[3];            // 16-feature tiles per matrix
    const bf16_t* residual;
    void* y;
    int M, K, ldy;           // ldy: elements per output row
    int act;
};

__device__ inline float gemm_act(float x, int act) {
    if (act == MASSV_ACT_SILU) return x / (1.0f + __expf(-x));
    const float c = 0.7978845608028654f;
    return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}

__device__ inline bf16x8 ld8(const bf16_t* p, bool ok) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    return ok ? *reinterpret_cast<const bf16x8*>(p) : z;
}

template <int MT, int NT, int WK, int EPI>
__global__ __launch_bounds__(WK * kWave)
void gemm_skinny_kernel(GemmDev g) {
    extern __shared__ floatx4 red[];                 // [WK][NT*MT][64]
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int lr = lane % 16, lc = lane / 16;
    const int K = g.K;
    constexpr bool gated = (EPI == EPI_GATED);

    // ---- which feature tiles this workgroup owns ----
    const bf16_t* wrow[NT];
    bool nvalid[NT];
    int seg_of[NT], ocol[NT], wfeat[NT];             // matrix, output column of the tile, first feature within its matrix
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int seg, local;
        if (gated) {
            seg = nt & 1;
            local = blockIdx.x * (NT / 2) + nt / 2;
            nvalid[nt] = local < g.tiles[0];
            ocol[nt] = local * 16;
        } else {
            const int t = blockIdx.x * NT + nt;
            if (t < g.tiles[0]) { seg = 0; local = t; }
            else if (t < g.tiles[0] + g.tiles[1]) { seg = 1; local = t - g.tiles[0]; }
            else { seg = 2; local = t - g.tiles[0] - g.tiles[1]; }
            nvalid[nt] = t < g.tiles[0] + g.tiles[1] + g.tiles[2];
            ocol[nt] = t * 16;
        }
        if (!nvalid[nt]) { seg = 0; local = 0; }
        seg_of[nt] = seg; wfeat[nt] = local * 16;
        wrow[nt] = g.w[seg] + (size_t)(local * 16 + lr) * K + lc * 8;
    }
    // X is stored in operand order: the B operand of (k-step ks, row tile mt) is the 1 KB block
    // ((ks * MT + mt) * 64 + lane) * 8.
    const bf16_t* xlane = g.x + (size_t)lane * 8;

    floatx4 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int n_chunks = (K + 127) / 128;
    bf16x8 a0[NT][4], b0[MT][4], a1[NT][4], b1[MT][4];

#define MASSV_GEMM_LOAD(A, B, CH)                                                         \
    {                                                                                     \
        const int k0 = (CH) * 128;                                                        \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                   \
            const bool kok = k0 + j * 32 < K;                                             \
            _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                             \
                A[nt][j] = ld8(wrow[nt] + k0 + j * 32, kok && nvalid[nt]);                \
            _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                             \
                B[mt][j] = ld8(xlane + (size_t)(((CH) * 4 + j) * MT + mt) * 512, kok);    \
        }                                                                                 \
    }
#define MASSV_GEMM_MMA(A, B)                                                              \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                         \
        _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                 \
            _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                             \
                acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[nt][j], B[mt][j], acc[nt][mt], 0, 0, 0);

    int ch = wave;
    if (ch < n_chunks) MASSV_GEMM_LOAD(a0, b0, ch)
    while (ch < n_chunks) {
        if (ch + WK < n_chunks) MASSV_GEMM_LOAD(a1, b1, ch + WK)
        MASSV_GEMM_MMA(a0, b0)
        ch += WK;
        if (ch >= n_chunks) break;
        if (ch + WK < n_chunks) MASSV_GEMM_LOAD(a0, b0, ch + WK)
        MASSV_GEMM_MMA(a1, b1)
        ch += WK;
    }
#undef MASSV_GEMM_LOAD
#undef MASSV_GEMM_MMA

    // ---- sum the K-splits of the workgroup through LDS, in wave order ----
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) red[(wave * NT * MT + nt * MT + mt) * kWave + lane] = acc[nt][mt];
    __syncthreads();

#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (gated && (nt & 1)) continue;                 // the up tile is consumed with its gate tile
            const int item = gated ? (nt / 2) * MT + mt : nt * MT + mt;
            if (item % WK != wave || !nvalid[nt]) continue;  // items are dealt round-robin to the waves
            floatx4 s = red[(nt * MT + mt) * kWave + lane];
            for (int w = 1; w < WK; ++w) s += red[(w * NT * MT + nt * MT + mt) * kWave + lane];
            const int m = mt * 16 + lr;
            const int col = ocol[nt] + lc * 4;               // 4 consecutive output features
            if (gated) {
                constexpr int NTU = (NT > 1) ? 1 : 0;        // NT >= 2 whenever the epilogue is gated
                const int nu = nt + NTU;
                floatx4 u = red[(nu * MT + mt) * kWave + lane];
                for (int w = 1; w < WK; ++w) u += red[(w * NT * MT + nu * MT + mt) * kWave + lane];
                if (m < g.M) {
                    bf16x4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = (bf16_t)(gemm_act(s[i], g.act) * u[i]);
                    *reinterpret_cast<bf16x4*>((bf16_t*)g.y + packed_index(m, col, MT)) = o;
                }
            } else if (m < g.M) {
                if (EPI == EPI_LOGITS) {
                    *reinterpret_cast<floatx4*>((float*)g.y + (size_t)m * g.ldy + col) = s;
                } else {
                    const bf16_t* bias = g.bias[seg_of[nt]];
                    if (bias) {
                        const bf16x4 bv = *reinterpret_cast<const bf16x4*>(bias + wfeat[nt] + lc * 4);
#pragma unroll
                        for (int i = 0; i < 4; ++i) s[i] += (float)bv[i];
                    }
                    if (EPI == EPI_RESIDUAL) {
                        const bf16x4 rv = *reinterpret_cast<const bf16x4*>(g.residual + (size_t)m * g.ldy + col);
#pragma unroll
                        for (int i = 0; i < 4; ++i) s[i] += (float)rv[i];
                    }
                    bf16x4 o = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
                    *reinterpret_cast<bf16x4*>((bf16_t*)g.y + (size_t)m * g.ldy + col) = o;
                }
            }
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
    if (g.dtype == MASSV_F32) return MASSV_OK;
    if (g.M > MASSV_MAX_ROWS) return MASSV_EUNSUPPORTED;
    if (g.K % 32) return MASSV_EUNSUPPORTED;
    for (int s = 0; s < 3; ++s)
        if (g.n[s] % 16) return MASSV_EUNSUPPORTED;
    return MASSV_OK;
}

template <int MT, int NT, int WK, int EPI>
static void launch_skinny(const GemmDev& d, int work_tiles, hipStream_t st) {
    constexpr int per_wg = (EPI == EPI_GATED) ? NT / 2 : NT;
    const int grid = (work_tiles + per_wg - 1) / per_wg;
    const size_t lds = (size_t)WK * NT * MT * kWave * sizeof(floatx4);
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, WK, EPI>), dim3(grid), dim3(WK * kWave), lds, st, d);
}

// Tile shape per launch.  work_tiles: 16-feature tiles (tile PAIRS for the gated
// epilogue).  Wide outputs give each wave 4 or 2 tiles so that X is re-read
// less; narrow outputs (O, down) keep one tile per wave and raise the number of
// waves that split K until the grid holds about 2048 waves.
template <int MT, int EPI>
static void launch_skinny_mt(const GemmDev& d, int work_tiles, hipStream_t st) {
    constexpr bool gated = (EPI == EPI_GATED);
    const int chunks = (d.K + 127) / 128;
    int nt = 1;
    if (gated) nt = (work_tiles / 2 >= 448 && MT <= 3) ? 4 : 2;
    else if (work_tiles / 4 >= 448 && MT <= 3) nt = 4;
    else if (work_tiles / 2 >= 448) nt = 2;
    if (nt == 4) { launch_skinny<MT, 4, 4, EPI>(d, work_tiles, st); return; }
    if (nt == 2) { launch_skinny<MT, 2, 4, EPI>(d, work_tiles, st); return; }
    if constexpr (!gated) {
        if constexpr (MT <= 2) {                      // 16 waves leave 128 VGPRs each: enough for two row tiles
            if (work_tiles * 8 < 2048 && chunks >= 32) { launch_skinny<MT, 1, 16, EPI>(d, work_tiles, st); return; }
        }
        launch_skinny<MT, 1, 8, EPI>(d, work_tiles, st);
    }
}

template <int EPI>
static int launch_skinny_epi(const GemmDev& d, int M, int work_tiles, hipStream_t st) {
    switch ((M + 15) / 16) {
        case 1: launch_skinny_mt<1, EPI>(d, work_tiles, st); break;
        case 2: launch_skinny_mt<2, EPI>(d, work_tiles, st); break;
        case 3: launch_skinny_mt<3, EPI>(d, work_tiles, st); break;
        case 4: launch_skinny_mt<4, EPI>(d, work_tiles, st); break;
        default: return MASSV_EUNSUPPORTED;
    }
    return MASSV_OK;
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
    GemmDev d;
    d.x = (const bf16_t*)g.x;
    for (int s = 0; s < 3; ++s) {
        d.w[s] = (const bf16_t*)g.w[s];
        d.bias[s] = (const bf16_t*)g.bias[s];
        d.tiles[s] = g.n[s] / 16;
    }
    d.residual = (const bf16_t*)g.residual;
    d.y = g.y;
    d.M = g.M; d.K = g.K;
    d.ldy = (g.epilogue == EPI_GATED) ? g.n[0] : N;
    d.act = g.act;
    const int work = (g.epilogue == EPI_GATED) ? d.tiles[0] : N / 16;
    int rc2 = MASSV_EUNSUPPORTED;
    trace_begin(g.kid, st);
    switch (g.epilogue) {
        case EPI_STORE: rc2 = launch_skinny_epi<EPI_STORE>(d, g.M, work, st); break;
        case EPI_RESIDUAL: rc2 = launch_skinny_epi<EPI_RESIDUAL>(d, g.M, work, st); break;
        case EPI_GATED: rc2 = launch_skinny_epi<EPI_GATED>(d, g.M, work, st); break;
        case EPI_LOGITS: rc2 = launch_skinny_epi<EPI_LOGITS>(d, g.M, work, st); break;
    }
    trace_end(g.kid, st);
    if (rc2 != MASSV_OK) return rc2;
    return launch_status();
}

}  // namespace massv
