// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace areal {

// Matrix-core operands (weights, activations, K/V) are IEEE half precision; all
// accumulation, the residual stream, softmax statistics and logits are float32.
typedef _Float16 f16;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16_in;   // only as an input format of parameter sets
typedef float  f32x4 __attribute__((ext_vector_type(4)));
typedef float  f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kBlockTokens = 16;   // tokens per KV block

__device__ __forceinline__ float h2f(f16 x) { return (float)x; }
__device__ __forceinline__ f16 f2h(float x) { return (f16)x; }   // round to nearest even
// Activations and K/V on their way to the matrix cores: magnitudes beyond the half range
// saturate to +-65504 instead of turning into infinities (NaN stays NaN).
__device__ __forceinline__ f16 f2h_sat(float x) {
  return (f16)__builtin_amdgcn_fmed3f(x, -65504.0f, 65504.0f);
}

// 16-byte global load of 8 halves
__device__ __forceinline__ f16x8 ld8(const f16* p) { return *reinterpret_cast<const f16x8*>(p); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

// 16 bytes per lane, HBM -> LDS: lane i of the wave writes dst_wave_base + i*16.
__device__ __forceinline__ void dma16(const void* src, void* dst_wave_base) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)src,
      (__attribute__((address_space(3))) void*)dst_wave_base, 16, 0, 0);
}

__device__ __forceinline__ void wait_vmcnt(int n) {
  // s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt = [15:14]:[3:0]); the counter
  // has 6 bits, so a larger bound is tightened to 63
  switch (n < 63 ? n : 63) {
#define AREAL_W(N) case N: __builtin_amdgcn_s_waitcnt(((N) & 15) | (((N) >> 4) << 14) | 0x0F70); break;
#define AREAL_W8(B) AREAL_W(B) AREAL_W(B + 1) AREAL_W(B + 2) AREAL_W(B + 3) AREAL_W(B + 4) AREAL_W(B + 5) \
                    AREAL_W(B + 6) AREAL_W(B + 7)
    AREAL_W8(0) AREAL_W8(8) AREAL_W8(16) AREAL_W8(24) AREAL_W8(32) AREAL_W8(40) AREAL_W8(48) AREAL_W8(56)
#undef AREAL_W8
#undef AREAL_W
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
  }
}

// ---- paged KV arena addressing --------------------------------------------
// arena = [layer][block][kv_head][K tile | V tile], tiles of 16*d halves.
//   K tile: [c 0..d/32-1][g 0..3][token 0..15][e 0..7] holding K[token][dim 32c+8g+e]:
//           the 16 bytes at (c, lane = g*16 + token) are lane's A-operand
//           registers of MFMA c of the 16x16x32 score product.
//   V tile: [c 0..d/32-1][lane 0..63][e 0..7] with lane = g*16 + j and
//           e = 4*(n&1) + t holding V[token 4g+t][dim 16n+j], n = 2c + (e>>2):
//           the 16 bytes at (c, lane) are lane's B-operand registers of the
//           16x16x16 MFMAs n = 2c, 2c+1 that multiply probabilities by values,
//           and one load instruction of a wave (fixed c) reads 1 KiB in a row.
struct KvGeom {
  int n_kv_heads, head_dim;
  int64_t layer_stride;   // elements between layers = n_blocks * block_stride
  int block_stride;       // elements per block of one layer = n_kv_heads * 2 * 16 * d
};
__device__ __forceinline__ int64_t kv_tile_off(const KvGeom& g, int block, int kvh, int is_v) {
  return (int64_t)block * g.block_stride + (int64_t)(kvh * 2 + is_v) * (kBlockTokens * g.head_dim);
}
__device__ __forceinline__ int k_tile_index(int token, int dim) {
  return (((dim >> 5) * 64 + ((dim >> 3) & 3) * 16 + token) * 8) + (dim & 7);
}
__device__ __forceinline__ int v_tile_index(int head_dim, int token, int dim) {
  (void)head_dim;
  int g = token >> 2, t = token & 3, n = dim >> 4, j = dim & 15;
  return (((n >> 1) * 64 + g * 16 + j) * 8) + (n & 1) * 4 + t;
}

}  // namespace areal
