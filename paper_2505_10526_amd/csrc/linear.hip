// massv_linear: Y = act(X W^T + bias) for prefill-sized inputs (hundreds to thousands of rows), the compute-bound
// counterpart of the verify projections: the multimodal projector that maps the vision encoder's features into
// the language model's embedding space (paper Section 3.1) and the projections of an image-token prefill.
//
// One workgroup of four waves owns a 256-feature x 256-row tile of Y; each wave a 128 x 128 quarter held as 4 x 4
// accumulators of v_mfma_f32_32x32x16_bf16 (all 256 accumulation registers).  A single wave per SIMD cannot issue
// the 16x16x32 form back to back (measured 31 cycles per instruction against 16), the 32x32x16 form it can.
// Both operands arrive in operand order (W: the streaming layout of massv_weight_pack; X: re-laid out by
// linear_pack_kernel), so every global load and every LDS access is a contiguous 1 KB per wave.
// Pipeline per 64-wide k-step (four quarter-steps of 16 matrix instructions):
//   * the tile of step ks+2 is requested from global memory into one of two register sets,
//   * the tile of step ks+1 (requested a whole step earlier) moves to the other LDS buffer, one write per
//     instruction slot, while quarters 1 and 2 are multiplied,
//   * LDS reads of the next quarter's fragments are interleaved one per two matrix instructions (a burst of
//     reads in front of the matrix instructions left the matrix pipe idle a third of the time),
//   * the one barrier of the step sits in the middle of quarter 3 with matrix instructions queued on both sides.
// The matrix instruction is issued through inline assembly with the accumulator tied as input and output: with
// the builtin the register allocator separates the two whenever an accumulator is updated twice in one loop body
// and then has to shuffle 256 accumulator registers every iteration.
#include "kernels.h"

#include <atomic>

namespace massv {

constexpr int kLinTile = 256;            // rows / features per workgroup
constexpr int kLinGroupM = 8;            // row tiles per scheduling group
constexpr size_t kLinLds = 2 * 2 * 2 * 16 * 64 * sizeof(bf16x8);      // [buf][k32 sub-step][W|X][tile16 * 64 + lane] = 128 KB

template <int ACT>
__device__ inline float linear_act(float v) {
    if constexpr (ACT == MASSV_LIN_SILU) return v / (1.0f + expf(-v));
    else if constexpr (ACT == MASSV_LIN_GELU_TANH) return 0.5f * v * (1.0f + tanhf(0.7978845608028654f * (v + 0.044715f * v * v * v)));
    else if constexpr (ACT == MASSV_LIN_GELU_ERF) return 0.5f * v * (1.0f + erff(v * 0.7071067811865476f));
    else return v;
}

// Row-major X[M][K] -> operand order [ceil(M/16)][K/32][64][8]; rows beyond M are zero.  One thread per 16-byte chunk.
__global__ void linear_pack_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, size_t chunks, int M, int K) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= chunks) return;
    const int lane = (int)(o % 64);
    const size_t t2 = o / 64;
    const int ksteps = K / 32;
    const int ks = (int)(t2 % ksteps);
    const size_t m = (t2 / ksteps) * 16 + (lane % 16);
    const int k = ks * 32 + (lane / 16) * 8;
    bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (m < (size_t)M) v = *reinterpret_cast<const bf16x8*>(src + m * K + k);
    *reinterpret_cast<bf16x8*>(dst + o * 8) = v;
}

template <int ACT>
__global__ __launch_bounds__(256)
void linear_tile_kernel(const bf16_t* __restrict__ xpk, const bf16_t* __restrict__ wpk, const bf16_t* __restrict__ bias,
                        bf16_t* __restrict__ y, int M, int N, int K, int tiles_m, int tiles_n) {
    extern __shared__ bf16x8 lds_raw[];
    bf16x8 (*lds)[2][2][16 * 64] = reinterpret_cast<bf16x8 (*)[2][2][16 * 64]>(lds_raw);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wy = wave / 2, wx = wave % 2;
    // Workgroup -> tile.  Consecutive workgroup ids go to different compute dies, each with its own L2: every die
    // gets a contiguous range of logical ids, and logical ids walk the tile grid in groups of kLinGroupM row tiles,
    // so that the workgroups running together on a die share their W and X strips.
    const int total = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int per = total / 8;
        if (per * 8 == total) pid = (pid % 8) * per + pid / 8;
    }
    const int in_group = kLinGroupM * tiles_n;
    const int first_m = (pid / in_group) * kLinGroupM;
    const int gsz = (tiles_m - first_m) < kLinGroupM ? (tiles_m - first_m) : kLinGroupM;
    const int tm = first_m + (pid % in_group) % gsz;
    const int tn = (pid % in_group) / gsz;

    const int KS = K / 32, KS2 = K / 64, lastk = KS2 - 1;
    const int n16 = N / 16, m16 = (M + 15) / 16;
    // wave w stages feature tiles and row tiles 4w .. 4w+3; out-of-range tiles read a valid one instead (their
    // results are never stored)
    const bf16x8* wsrc[4];
    const bf16x8* xsrc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        int T = tn * 16 + 4 * wave + t; T = T < n16 ? T : n16 - 1;
        wsrc[t] = reinterpret_cast<const bf16x8*>(wpk + ((size_t)T * KS) * 512) + lane;
        int U = tm * 16 + 4 * wave + t; U = U < m16 ? U : m16 - 1;
        xsrc[t] = reinterpret_cast<const bf16x8*>(xpk + ((size_t)U * KS) * 512) + lane;
    }
    bf16x8 gA[16], gB[16];
    auto gload = [&](int ks, bf16x8 (&g)[16]) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                g[u * 8 + t] = wsrc[t][(size_t)(2 * ks + u) * 64];
                g[u * 8 + 4 + t] = xsrc[t][(size_t)(2 * ks + u) * 64];
            }
    };
    // n-th of the 16 staged 1 KB pieces of a k-step -> LDS
    auto lstore1 = [&](int buf, const bf16x8 (&g)[16], int n) {
        const int u = n / 8, r = n % 8, t = r % 4;
        lds[buf][u][r < 4 ? 0 : 1][(4 * wave + t) * 64 + lane] = g[n];
    };

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand fragment (32 rows x 16 k) out of the 16-row x 32-k tiles in LDS: lane l takes row l % 32 and k chunk
    // l / 32 of half h, i.e. unit (tile16 = 2 i + (l % 32) / 16, lane' = l % 16 + 16 (2 h + l / 32))
    const int frag_off = ((lane % 32) / 16) * 64 + (lane % 16) + 16 * (lane / 32);
    bf16x8 wf[2][4], xf[2][4];
    // fragment f of quarter-step s (s = 2 u + h): f < 4 a feature fragment, else a row fragment
    auto load_frag = [&](int buf, int s, int f, bf16x8 (&w)[4], bf16x8 (&x4)[4]) {
        if (f < 4) w[f] = lds[buf][s / 2][0][(8 * wy + 2 * f) * 64 + frag_off + 32 * (s % 2)];
        else x4[f - 4] = lds[buf][s / 2][1][(8 * wx + 2 * (f - 4)) * 64 + frag_off + 32 * (s % 2)];
    };
    auto mfma = [&](floatx16& c, bf16x8 a, bf16x8 b) {
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    };

    gload(0, gA);
    gload(1 < KS2 ? 1 : lastk, gB);
#pragma unroll
    for (int n = 0; n < 16; ++n) lstore1(0, gA, n);
    __syncthreads();
#pragma unroll
    for (int f = 0; f < 8; ++f) load_frag(0, 0, f, wf[0], xf[0]);

    // step ks: g_free held tile ks (already in LDS) and receives tile ks+2; g_next holds tile ks+1.  Loads past the
    // end re-read the last tile and what they bring is never multiplied.
    auto step = [&](int ks, bf16x8 (&g_free)[16], const bf16x8 (&g_next)[16]) {
        const int buf = ks & 1;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            if (s4 == 0) gload(ks + 2 < KS2 ? ks + 2 : lastk, g_free);
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                __builtin_amdgcn_sched_barrier(0);
                if (s4 < 3) load_frag(buf, s4 + 1, p, wf[(s4 + 1) % 2], xf[(s4 + 1) % 2]);
                if (s4 == 1 || s4 == 2) lstore1(buf ^ 1, g_next, (s4 - 1) * 8 + p);
                if (s4 == 3 && p == 4) __syncthreads();
                if (s4 == 3 && p >= 4) {                        // the next step's first fragments (set 0 is free)
                    load_frag(buf ^ 1, 0, 2 * (p - 4), wf[0], xf[0]);
                    load_frag(buf ^ 1, 0, 2 * (p - 4) + 1, wf[0], xf[0]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int idx = 2 * p + t, j = idx / 4, i = idx % 4;
                    mfma(acc[i][j], wf[s4 % 2][i], xf[s4 % 2][j]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int ks = 0;
    for (; ks + 1 < KS2; ks += 2) {
        step(ks, gA, gB);
        step(ks + 1, gB, gA);
    }
    if (ks < KS2) step(ks, gA, gB);
    // The matrix instructions above are assembly the compiler cannot see into: it does not know that their results
    // arrive up to 16 passes (64 cycles) after issue, so it inserts no wait before the epilogue reads the
    // accumulators.  The wait is written here -- 4 x 16 idle cycles -- and tied to the data: the two statements take
    // every accumulator as an in/out operand, so neither a matrix instruction nor an accumulator read can be
    // scheduled across them (two statements because one takes at most 30 operands; volatile keeps their order).
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15"
                 : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]),
                   "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
    asm volatile("" : "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]),
                      "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3]));

    // epilogue: lane holds features 32 i + 8 g + 4 (lane / 32) + r (g, r = 0..3) of row 32 j + lane % 32
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int m = tm * kLinTile + 128 * wx + 32 * j + lane % 32;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int n = tn * kLinTile + 128 * wy + 32 * i + 8 * g4 + 4 * (lane / 32);
                if (n >= N) continue;
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = acc[i][j][4 * g4 + r];
                if (bias) {
                    const bf16x4 bv = *reinterpret_cast<const bf16x4*>(bias + n);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] += (float)bv[r];
                }
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (bf16_t)linear_act<ACT>(v[r]);
                *reinterpret_cast<bf16x4*>(y + (size_t)m * N + n) = o;
            }
    }
}

static int check_linear(int32_t M, int32_t N, int32_t K, int32_t act, int32_t dtype) {
    if (M < 1 || N < 1 || K < 1) return MASSV_EINVAL;
    if (dtype != MASSV_F32 && dtype != MASSV_BF16) return MASSV_EINVAL;
    if (act < MASSV_LIN_NONE || act > MASSV_LIN_GELU_ERF) return MASSV_EINVAL;
    if (dtype != MASSV_BF16) return MASSV_EUNSUPPORTED;
    if (K % 64 || N % 16) return MASSV_EUNSUPPORTED;
    if ((size_t)((M + kLinTile - 1) / kLinTile) * ((N + kLinTile - 1) / kLinTile) > 0x7fffffffu) return MASSV_EUNSUPPORTED;
    return MASSV_OK;
}

}  // namespace massv

using namespace massv;

extern "C" size_t massv_linear_workspace(int32_t M, int32_t N, int32_t K, int32_t dtype) {
    if (check_linear(M, N, K, MASSV_LIN_NONE, dtype) != MASSV_OK) return 0;
    return align_up(packed_elems(M, K) * sizeof(bf16_t), 256);
}

extern "C" int massv_linear(const void* x, const void* w, const void* bias, void* y, int32_t M, int32_t N, int32_t K,
                            int32_t act, int32_t dtype, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_linear(M, N, K, act, dtype);
    if (rc != MASSV_OK) return rc;
    if (!x || !w || !y) return MASSV_EINVAL;
    if (!workspace || workspace_bytes < massv_linear_workspace(M, N, K, dtype)) return MASSV_EWORKSPACE;
    // the tile kernel needs more LDS than a kernel gets by default: raise its limit once per device
    static std::atomic<bool> lds_ready[64];       // zero-initialised; calls may come from several threads
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MASSV_ELAUNCH;
    if (!lds_ready[dev].load(std::memory_order_acquire)) {
        const void* kernels[4] = {(const void*)linear_tile_kernel<MASSV_LIN_NONE>, (const void*)linear_tile_kernel<MASSV_LIN_SILU>,
                                  (const void*)linear_tile_kernel<MASSV_LIN_GELU_TANH>, (const void*)linear_tile_kernel<MASSV_LIN_GELU_ERF>};
        for (const void* k : kernels)
            if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLinLds) != hipSuccess) return MASSV_ELAUNCH;
        lds_ready[dev].store(true, std::memory_order_release);
    }
    hipStream_t st = (hipStream_t)stream;
    const size_t chunks = packed_elems(M, K) / 8;
    hipLaunchKernelGGL(linear_pack_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, (const bf16_t*)x,
                       (bf16_t*)workspace, chunks, M, K);
    const int tiles_m = (M + kLinTile - 1) / kLinTile, tiles_n = (N + kLinTile - 1) / kLinTile;
    const dim3 grid(tiles_m * tiles_n), block(256);
    const bf16_t* xp = (const bf16_t*)workspace;
    switch (act) {
        case MASSV_LIN_SILU:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_SILU>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
            break;
        case MASSV_LIN_GELU_TANH:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_GELU_TANH>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
            break;
        case MASSV_LIN_GELU_ERF:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_GELU_ERF>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
            break;
        default:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_NONE>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
    }
    return launch_status();
}
