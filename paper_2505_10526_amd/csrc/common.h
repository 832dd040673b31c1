// Internal helpers shared by the gfx950 kernels of libmassv_verify.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

#include "massv_verify.h"

namespace massv {

constexpr int kWave = 64;          // CDNA wavefront width

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Status of the launch that was just enqueued.
static inline int launch_status() {
    return hipGetLastError() == hipSuccess ? MASSV_OK : MASSV_ELAUNCH;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

template <typename T> struct ElemOf;
template <> struct ElemOf<float> {
    __device__ static inline float load(const float* p) { return *p; }
    __device__ static inline void store(float* p, float v) { *p = v; }
};
template <> struct ElemOf<bf16_t> {
    __device__ static inline float load(const bf16_t* p) { return (float)*p; }
    __device__ static inline void store(bf16_t* p, float v) { *p = (bf16_t)v; }
};

template <typename T> __device__ inline float ldf(const T* p) { return ElemOf<T>::load(p); }
template <typename T> __device__ inline void stf(T* p, float v) { ElemOf<T>::store(p, v); }

// ---- streaming loads ----
// Data that is read once in whole 128-byte lines per instruction (logits, the
// blocked value cache) is loaded with the non-temporal hint: on MI355X a plain
// streaming read measured about 6.0 TB/s and the same read with the hint about
// 6.4 TB/s.  Loads that use half a line per instruction (rows of W or K in
// matrix-operand order) stay cached: the second half is a hit.
__device__ inline bf16x8 ldg_stream(const bf16x8* p) { return __builtin_nontemporal_load(p); }
__device__ inline float4 ldg_stream(const float4* p) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}

// ---- operand-order ("packed") activations ----
// The bf16 projections read their activation matrix X[M][K] as the B operand
// of v_mfma_f32_16x16x32_bf16: lane l of a wave needs the 8 values
// X[16*mt + l%16][32*ks + 8*(l/16) .. +8].  Producers store X in exactly that
// order, [K/32][MT][64 lanes][8], MT = ceil(M/16), so that a wave's operand
// load is one contiguous 1 KB read (8 full cache lines instead of 16 half
// lines).  Rows M .. 16*MT-1 are padding and are never read back into results.
__host__ __device__ inline size_t packed_index(int m, int k, int mt_count) {
    return (((size_t)(k >> 5) * mt_count + (m >> 4)) * 64 + ((m & 15) + 16 * ((k & 31) >> 3))) * 8 + (k & 7);
}
__host__ __device__ inline size_t packed_elems(int M, int K) { return (size_t)((M + 15) / 16) * 16 * K; }

// ---- wavefront reductions (all 64 lanes take part, all receive the result) ----
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

}  // namespace massv
