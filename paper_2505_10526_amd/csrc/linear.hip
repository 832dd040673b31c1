// massv_linear: Y = act(X W^T + bias) for prefill-sized inputs (hundreds to thousands of rows), the compute-bound
// counterpart of the verify projections: the multimodal projector that maps the vision encoder's features into
// the language model's embedding space (paper Section 3.1) and the projections of an image-token prefill.
//
// One workgroup of eight waves owns a 256-feature x 256-row tile of Y; each wave a 64 x 128 piece held as 2 x 4
// accumulators of v_mfma_f32_32x32x16_bf16 (128 accumulation registers), two waves per SIMD so that one wave's
// matrix instructions issue while the other waits for its fragments.  (A single wave per SIMD with a 128 x 128
// piece reads less from LDS but gets a matrix instruction out only every 40 cycles instead of 32.)
// Both operands arrive in operand order (W: the streaming layout of massv_weight_pack; X: re-laid out by
// linear_pack_kernel), so every global load and every LDS access is a contiguous 1 KB per wave.
// Pipeline: a ring of four 32-wide k-stages in LDS (4 x 32 KB).  Stages travel from global memory straight into
// LDS (global_load_lds, 16 bytes per lane, no staging registers and no LDS store instructions), three stages ahead
// of the one being multiplied; one barrier per stage; the LDS reads of the next 16-wide quarter-step's fragments sit
// one behind each of the current quarter-step's first matrix instructions.
// The matrix instruction is issued through inline assembly with the accumulator tied as input and output: with
// the builtin the register allocator separates the two whenever an accumulator is updated twice in one loop body
// and then has to shuffle the accumulator registers every iteration.
#include "kernels.h"

#include <atomic>

namespace massv {

constexpr int kLinTile = 256;            // rows / features per workgroup
constexpr int kLinGroupM = 8;            // row tiles per scheduling group
constexpr size_t kLinLds = 4 * 2 * 16 * 64 * sizeof(bf16x8);          // [stage][W|X][tile16 * 64 + lane] = 128 KB
constexpr int kLinWaves = 8;             // waves per workgroup (the kernel also builds with 4: 128 x 128 per wave)

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

// Tile kernel.  WAVES = 4: each wave a 128 x 128 quarter (4 x 4 accumulators, one wave per SIMD); WAVES = 8: each wave
// 64 features x 128 rows (2 x 4 accumulators, two waves per SIMD).
template <int ACT, int WAVES>
__global__ __launch_bounds__(WAVES * 64)
void linear_tile_kernel(const bf16_t* __restrict__ xpk, const bf16_t* __restrict__ wpk, const bf16_t* __restrict__ bias,
                        const bf16_t* __restrict__ mul, const bf16_t* add, bf16_t* y,
                        int M, int N, int K, int tiles_m, int tiles_n) {
    constexpr int FI = WAVES == 4 ? 4 : 2;        // 32-feature fragments per wave
    constexpr int FJ = 4;                         // 32-row fragments per wave
    constexpr int NMF = FI * FJ, NF = FI + FJ;    // matrix instructions and fragment loads per 16-wide quarter-step
    constexpr int U = 32 / WAVES;                 // 1 KB pieces of a stage each wave brings in
    extern __shared__ bf16x8 lds_raw[];
    bf16x8 (*lds)[2][16 * 64] = reinterpret_cast<bf16x8 (*)[2][16 * 64]>(lds_raw);          // [stage][W|X][tile16 * 64 + lane]
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
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

    const int KS = K / 32;
    const int n16 = N / 16, m16 = (M + 15) / 16;
    // Piece u of a stage (u < 16: feature tile u of W, else row tile u - 16 of X) is brought in by wave u / U, straight
    // from global memory into LDS: lane l's 16 bytes land at the piece's base + 16 l, which is the layout the pieces
    // have in memory.  Out-of-range tiles read a valid one instead (their results are never stored).
    const bf16x8* src[U];
#pragma unroll
    for (int t = 0; t < U; ++t) {
        const int u = wave * U + t;
        if (u < 16) {
            int T = tn * 16 + u; T = T < n16 ? T : n16 - 1;
            src[t] = reinterpret_cast<const bf16x8*>(wpk + ((size_t)T * KS) * 512) + lane;
        } else {
            int R = tm * 16 + (u - 16); R = R < m16 ? R : m16 - 1;
            src[t] = reinterpret_cast<const bf16x8*>(xpk + ((size_t)R * KS) * 512) + lane;
        }
    }
    auto issue = [&](int ks, int slot) {
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const int u = wave * U + t;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[t] + (size_t)ks * 64),
                                             (__attribute__((address_space(3))) void*)&lds[slot][u / 16][(u % 16) * 64], 16, 0, 0);
        }
    };

    floatx16 acc[FI][FJ];
#pragma unroll
    for (int i = 0; i < FI; ++i)
#pragma unroll
        for (int j = 0; j < FJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand fragment (32 rows x 16 k) out of the 16-row x 32-k tiles in LDS: lane l takes row l % 32 and k chunk
    // l / 32 of half h, i.e. unit (tile16 = 2 i + (l % 32) / 16, lane' = l % 16 + 16 (2 h + l / 32))
    const int frag_off = ((lane % 32) / 16) * 64 + (lane % 16) + 16 * (lane / 32);
    bf16x8 wf[2][FI], xf[2][FJ];
    // fragment f of half h of a stage: f < FI a feature fragment, else a row fragment
    auto load_frag = [&](int slot, int h, int f, bf16x8 (&w)[FI], bf16x8 (&x4)[FJ]) {
        if (f < FI) w[f] = lds[slot][0][(2 * FI * wy + 2 * f) * 64 + frag_off + 32 * h];
        else x4[f - FI] = lds[slot][1][(8 * wx + 2 * (f - FI)) * 64 + frag_off + 32 * h];
    };
    // Issued as assembly (see the file header), so the compiler's hazard tracking does not know it is a matrix
    // instruction.  What it still sees is the data flow: the operands come out of LDS reads it waits for, successive
    // updates of one accumulator are ordered by the in/out operand (the hardware interlocks dependent matrix
    // instructions), and the one place where something else reads the accumulators -- the epilogue -- is behind the
    // wait written out after the loop.
    auto mfma = [&](floatx16& c, bf16x8 a, bf16x8 b) {
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    };
    // The compiler does not know that the loads above write LDS, so the waits are written here: the loads of a wave
    // complete in order, and the counter operand is how many of the most recent ones may still be in flight.
    auto wait_loads = [&](bool keep_one_stage) {
        if (keep_one_stage) {
            if constexpr (U == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        } else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };

    // Ring of four stages (32 k each).  Stage s + 3 is requested while stage s is multiplied; the barrier in the
    // middle of stage s tells every wave that stage s + 1 has landed for all of them and that nobody reads stage
    // s - 1 any more (its last fragments were fetched during the first half of stage s - 1), whose slot the new
    // request overwrites.
    issue(0, 0);
    if (1 < KS) issue(1, 1);
    if (2 < KS) issue(2, 2);
    if (2 < KS) { if constexpr (U == 8) asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); }
    else wait_loads(1 < KS);
    __syncthreads();
#pragma unroll
    for (int f = 0; f < NF; ++f) load_frag(0, 0, f, wf[0], xf[0]);

    for (int s = 0; s < KS; ++s) {
        const int slot = s & 3;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int idx = 0; idx < NMF; ++idx) {
                __builtin_amdgcn_sched_barrier(0);
                const int j = idx / FI, i = idx % FI;
                mfma(acc[i][j], wf[h][i], xf[h][j]);
                __builtin_amdgcn_sched_barrier(0);
                // the next quarter-step's fragments, one behind each of this one's first matrix instructions (past the
                // last stage they read a slot that holds nothing new; what they bring is never multiplied)
                if (idx < NF) {
                    if (h == 0) load_frag(slot, 1, idx, wf[1], xf[1]);
                    else load_frag((s + 1) & 3, 0, idx, wf[0], xf[0]);
                }
                if (h == 0 && idx == 1) {
                    wait_loads(s + 2 < KS);
                    __syncthreads();
                    if (s + 3 < KS) issue(s + 3, (s + 3) & 3);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // The matrix instructions above are assembly the compiler cannot see into: it does not know that their results
    // arrive up to 16 passes (64 cycles) after issue, so it inserts no wait before the epilogue reads the
    // accumulators.  The wait is written here -- 4 x 16 idle cycles -- and tied to the data: the statements take
    // every accumulator as an in/out operand, so neither a matrix instruction nor an accumulator read can be
    // scheduled across them (several statements because one takes at most 30 operands; volatile keeps their order).
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15"
                 : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]),
                   "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
    if constexpr (FI == 4)
        asm volatile("" : "+a"(acc[FI - 2][0]), "+a"(acc[FI - 2][1]), "+a"(acc[FI - 2][2]), "+a"(acc[FI - 2][3]),
                          "+a"(acc[FI - 1][0]), "+a"(acc[FI - 1][1]), "+a"(acc[FI - 1][2]), "+a"(acc[FI - 1][3]));

    // epilogue: lane holds features 32 i + 8 g + 4 (lane / 32) + r (g, r = 0..3) of row 32 j + lane % 32
#pragma unroll
    for (int j = 0; j < FJ; ++j) {
        const int m = tm * kLinTile + 128 * wx + 32 * j + lane % 32;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < FI; ++i)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int n = tn * kLinTile + 32 * FI * wy + 32 * i + 8 * g4 + 4 * (lane / 32);
                if (n >= N) continue;
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = acc[i][j][4 * g4 + r];
                if (bias) {
                    const bf16x4 bv = *reinterpret_cast<const bf16x4*>(bias + n);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] += (float)bv[r];
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = linear_act<ACT>(v[r]);
                if (mul) {                               // e.g. the up projection's rows: act(gate) * up
                    const bf16x4 mv = *reinterpret_cast<const bf16x4*>(mul + (size_t)m * N + n);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] *= (float)mv[r];
                }
                if (add) {                               // e.g. the residual stream (may be y itself: read before written)
                    const bf16x4 av = *reinterpret_cast<const bf16x4*>(add + (size_t)m * N + n);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] += (float)av[r];
                }
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (bf16_t)v[r];
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

extern "C" int massv_linear_ex(const void* x, const void* w, const void* bias, const void* mul, const void* add, void* y,
                               int32_t M, int32_t N, int32_t K, int32_t act, int32_t dtype, void* workspace,
                               size_t workspace_bytes, void* stream) {
    const int rc = check_linear(M, N, K, act, dtype);
    if (rc != MASSV_OK) return rc;
    if (!x || !w || !y) return MASSV_EINVAL;
    if (!workspace || workspace_bytes < massv_linear_workspace(M, N, K, dtype)) return MASSV_EWORKSPACE;
    // the tile kernel needs more LDS than a kernel gets by default: raise its limit once per device
    static std::atomic<bool> lds_ready[64];       // zero-initialised; calls may come from several threads
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MASSV_ELAUNCH;
    if (!lds_ready[dev].load(std::memory_order_acquire)) {
        const void* kernels[4] = {(const void*)linear_tile_kernel<MASSV_LIN_NONE, kLinWaves>, (const void*)linear_tile_kernel<MASSV_LIN_SILU, kLinWaves>,
                                  (const void*)linear_tile_kernel<MASSV_LIN_GELU_TANH, kLinWaves>, (const void*)linear_tile_kernel<MASSV_LIN_GELU_ERF, kLinWaves>};
        for (const void* k : kernels)
            if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLinLds) != hipSuccess) return MASSV_ELAUNCH;
        lds_ready[dev].store(true, std::memory_order_release);
    }
    hipStream_t st = (hipStream_t)stream;
    const size_t chunks = packed_elems(M, K) / 8;
    hipLaunchKernelGGL(linear_pack_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, (const bf16_t*)x,
                       (bf16_t*)workspace, chunks, M, K);
    const int tiles_m = (M + kLinTile - 1) / kLinTile, tiles_n = (N + kLinTile - 1) / kLinTile;
    const dim3 grid(tiles_m * tiles_n), block(kLinWaves * kWave);
    const bf16_t* xp = (const bf16_t*)workspace;
    switch (act) {
        case MASSV_LIN_SILU:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_SILU, kLinWaves>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (const bf16_t*)mul, (const bf16_t*)add, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
            break;
        case MASSV_LIN_GELU_TANH:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_GELU_TANH, kLinWaves>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (const bf16_t*)mul, (const bf16_t*)add, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
            break;
        case MASSV_LIN_GELU_ERF:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_GELU_ERF, kLinWaves>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (const bf16_t*)mul, (const bf16_t*)add, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
            break;
        default:
            launch_traced(MASSV_K_LINEAR, linear_tile_kernel<MASSV_LIN_NONE, kLinWaves>, grid, block, kLinLds, st, xp, (const bf16_t*)w,
                          (const bf16_t*)bias, (const bf16_t*)mul, (const bf16_t*)add, (bf16_t*)y, M, N, K, tiles_m, tiles_n);
    }
    return launch_status();
}

extern "C" int massv_linear(const void* x, const void* w, const void* bias, void* y, int32_t M, int32_t N, int32_t K,
                            int32_t act, int32_t dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return massv_linear_ex(x, w, bias, nullptr, nullptr, y, M, N, K, act, dtype, workspace, workspace_bytes, stream);
}
