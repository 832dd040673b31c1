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
// blocked key and value caches, weights in the streaming layout) is loaded with
// the non-temporal hint: on MI355X a plain streaming read measured about
// 6.0 TB/s and the same read with the hint up to 7.0 TB/s.  A load that uses
// half a line per instruction (16 rows x 64 bytes of a row-major matrix) must
// stay cached, because the other half is fetched by a later instruction; the
// layouts above exist so that no hot load has that shape.
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

// ---- bf16 key cache ----
// Element (row j, feature c) of (sequence, KV head) pair bg.  Rows live in blocks of 32, a block in two halves
// of 16 rows; a half is stored by 8-feature chunks, the 16 rows of a chunk back to back: lane (slot, chunk % 4)
// of a wave reads its 16-row x 32-feature operand of the score product as one contiguous 1 KB.
__host__ __device__ inline size_t k_cache_index(size_t bg, int l_max, int d, int j, int c) {
    const int jj = j & 31;
    const int half = (jj >> 2) & 1, slot = ((jj >> 3) << 2) | (jj & 3);
    return (bg * (size_t)l_max + (size_t)(j & ~31)) * d + ((size_t)(half * (d >> 3) + (c >> 3)) * 16 + slot) * 8 + (c & 7);
}

// ---- wavefront scans and reductions (all 64 lanes take part, all receive the result) ----
// Built from data-parallel-primitive moves: four shifts inside each row of 16 lanes, then the last lane of
// row 0 / row 2 combined into row 1 / row 3 and the last lane of row 1 into rows 2 and 3; lane 63 then holds the
// combination of all lanes.  A shuffle through the LDS crossbar costs a round trip of about 100 cycles per
// step, and the six steps depend on each other; these moves are ordinary vector-ALU operands.
constexpr int kDppShr1 = 0x111, kDppShr2 = 0x112, kDppShr4 = 0x114, kDppShr8 = 0x118;
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;      // written rows: 0xa (1 and 3), 0xc (2 and 3)

// The source lane's value; `fill` in lanes that have no source lane or lie in a row that is not written.
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_move(int v, int fill) { return __builtin_amdgcn_update_dpp(fill, v, CTRL, ROW_MASK, 0xf, false); }
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_move(float v, float fill) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ inline double dpp_move(double v, double fill) {
    const int lo = __builtin_amdgcn_update_dpp(__double2loint(fill), __double2loint(v), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(__double2hiint(fill), __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
    return __hiloint2double(hi, lo);
}
__device__ inline float lane_value(float v, int src_lane) {  // src_lane uniform over the wave
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}
__device__ inline double lane_value(double v, int src_lane) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), src_lane),
                            __builtin_amdgcn_readlane(__double2loint(v), src_lane));
}
// Inclusive prefix sum in lane order.
template <typename T>
__device__ inline T wave_scan_incl(T v) {
    v += dpp_move<kDppShr1, 0xf>(v, (T)0);
    v += dpp_move<kDppShr2, 0xf>(v, (T)0);
    v += dpp_move<kDppShr4, 0xf>(v, (T)0);
    v += dpp_move<kDppShr8, 0xf>(v, (T)0);
    v += dpp_move<kDppBcast15, 0xa>(v, (T)0);
    v += dpp_move<kDppBcast31, 0xc>(v, (T)0);
    return v;
}
__device__ inline float wave_sum(float v) { return lane_value(wave_scan_incl(v), kWave - 1); }
__device__ inline double wave_sum(double v) { return lane_value(wave_scan_incl(v), kWave - 1); }
__device__ inline float wave_max(float v) {                   // a lane without a source combines with itself
    v = fmaxf(v, dpp_move<kDppShr1, 0xf>(v, v));
    v = fmaxf(v, dpp_move<kDppShr2, 0xf>(v, v));
    v = fmaxf(v, dpp_move<kDppShr4, 0xf>(v, v));
    v = fmaxf(v, dpp_move<kDppShr8, 0xf>(v, v));
    v = fmaxf(v, dpp_move<kDppBcast15, 0xa>(v, v));
    v = fmaxf(v, dpp_move<kDppBcast31, 0xc>(v, v));
    return lane_value(v, kWave - 1);
}

}  // namespace massv
