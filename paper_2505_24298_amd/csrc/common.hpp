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
  // s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt = [15:14]:[3:0])
  switch (n) {
#define AREAL_W(N) case N: __builtin_amdgcn_s_waitcnt(((N) & 15) | (((N) >> 4) << 14) | 0x0F70); break;
    AREAL_W(0) AREAL_W(1) AREAL_W(2) AREAL_W(3) AREAL_W(4) AREAL_W(5) AREAL_W(6) AREAL_W(7) AREAL_W(8)
    AREAL_W(9) AREAL_W(10) AREAL_W(11) AREAL_W(12) AREAL_W(13) AREAL_W(14) AREAL_W(15) AREAL_W(16)
    AREAL_W(18) AREAL_W(20) AREAL_W(21) AREAL_W(24) AREAL_W(27) AREAL_W(28) AREAL_W(30) AREAL_W(32)
    AREAL_W(36) AREAL_W(40) AREAL_W(48)
#undef AREAL_W
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
  }
}

// ---- paged KV arena addressing --------------------------------------------
// arena = [layer][block][kv_head][K tile | V tile], tiles of 16*d halves.
//   K tile: [token 0..15][d]                       (row-major)
//   V tile: [lane 0..63][n 0..d/16-1][t 0..3] with lane = g*16 + j holding
//           V[token 4g+t][dim 16n+j]: exactly the B operand of the 16x16x16
//           MFMA that multiplies probabilities by values, 64 B per lane.
struct KvGeom {
  int n_kv_heads, head_dim;
  int64_t layer_stride;   // elements between layers = n_blocks * block_stride
  int block_stride;       // elements per block of one layer = n_kv_heads * 2 * 16 * d
};
__device__ __forceinline__ int64_t kv_tile_off(const KvGeom& g, int block, int kvh, int is_v) {
  return (int64_t)block * g.block_stride + (int64_t)(kvh * 2 + is_v) * (kBlockTokens * g.head_dim);
}
__device__ __forceinline__ int v_tile_index(int head_dim, int token, int dim) {
  int g = token >> 2, t = token & 3, n = dim >> 4, j = dim & 15;
  return (((g * 16 + j) * (head_dim >> 4)) + n) * 4 + t;
}

}  // namespace areal
