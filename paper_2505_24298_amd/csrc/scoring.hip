// Log-probability of one given token per row of float32 logits:
//   out = z[tok] - max z - log sum_i exp(z_i - max z),   z = logits * (1/T).
// One work-group per row, one pass over the row: every thread keeps a running
// (max, sum of exponentials) pair over its elements, the pairs are combined
// across the wave with shuffles and across waves through LDS.
#include <algorithm>

#include "kernels.hpp"

namespace areal {
namespace {

constexpr int LP_THREADS = 1024;

__device__ __forceinline__ void lse_combine(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  const float mu = mn == -INFINITY ? 0.f : mn;
  s = s * __expf(m - mu) + s2 * __expf(m2 - mu);
  m = mn;
}

__global__ __launch_bounds__(LP_THREADS) void token_logprob_kernel(
    const float* __restrict__ logits, int vocab, float inv_t, const int32_t* __restrict__ target,
    const int32_t* __restrict__ pos, float* __restrict__ out) {
  __shared__ float sm[LP_THREADS / 64], ss[LP_THREADS / 64];
  const int row = blockIdx.x;
  const int tok = target[row];
  if (pos[row] == 0 && threadIdx.x == 0) out[row] = 0.f;      // nothing predicts a first token
  if (tok < 0) return;                                        // last token of its sequence
  const float* z = logits + (int64_t)row * vocab;
  float m = -INFINITY, s = 0.f;
  const int n4 = (vocab & 3) ? 0 : vocab >> 2;             // rows are 16-byte aligned only then
  for (int i = threadIdx.x; i < n4; i += LP_THREADS) {
    const float4 v = reinterpret_cast<const float4*>(z)[i];
    const float a = v.x * inv_t, b = v.y * inv_t, c = v.z * inv_t, d = v.w * inv_t;
    const float mn = fmaxf(fmaxf(fmaxf(a, b), fmaxf(c, d)), m);
    s = s * __expf(m - mn) + __expf(a - mn) + __expf(b - mn) + __expf(c - mn) + __expf(d - mn);
    m = mn;
  }
  for (int i = (n4 << 2) + threadIdx.x; i < vocab; i += LP_THREADS) lse_combine(m, s, z[i] * inv_t, 1.f);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) lse_combine(m, s, __shfl_xor(m, o), __shfl_xor(s, o));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { sm[wave] = m; ss[wave] = s; }
  __syncthreads();
  if (wave == 0) {
    m = lane < LP_THREADS / 64 ? sm[lane] : -INFINITY;
    s = lane < LP_THREADS / 64 ? ss[lane] : 0.f;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) lse_combine(m, s, __shfl_xor(m, o), __shfl_xor(s, o));
    if (lane == 0) out[row + 1] = z[tok] * inv_t - m - __logf(s);
  }
}

// Second half of the fused scoring path: the per-tile (max, sum) pairs of a row, written by the
// output projection's epilogue as float2 [n_tiles][ld_rows], are folded and the row's log-prob
// comes out as target_z - max - log sum.  One thread per row: for a fixed tile the rows of a
// work-group are neighbours in memory.
__global__ __launch_bounds__(256) void lse_finish_kernel(const float2* __restrict__ part, int ld_rows, int n_tiles,
                                                         const float* __restrict__ target_z,
                                                         const int32_t* __restrict__ target,
                                                         const int32_t* __restrict__ pos, int n,
                                                         float* __restrict__ out) {
  const int row = blockIdx.x * 256 + threadIdx.x;
  if (row >= n) return;
  if (pos[row] == 0) out[row] = 0.f;                            // nothing predicts a first token
  const int tok = target[row];
  if (tok < 0) return;                                          // last token of its sequence
  float m = -INFINITY, s = 0.f;
  for (int t = 0; t < n_tiles; ++t) {
    const float2 p = part[(int64_t)t * ld_rows + row];
    lse_combine(m, s, p.x, p.y);
  }
  out[row + 1] = target_z[row] - m - __logf(s);
}

// Decoupled PPO objective, forward value: per token
//   u = exp(lt - lp), w = exp(lp - lb), obj = w * min(u A, clip(u, 1-eps, 1+eps) A),
// optional mask; sums[0] += sum obj, sums[1] += number of tokens whose clipped term is the
// smaller one, sums[2] += tokens counted.  Float64 accumulation (one atomic per work-group).
__global__ __launch_bounds__(256) void ppo_objective_kernel(
    int n, const float* __restrict__ lt, const float* __restrict__ lp, const float* __restrict__ lb,
    const float* __restrict__ adv, const uint8_t* __restrict__ mask, float eps,
    float* __restrict__ obj_out, double* __restrict__ sums) {
  __shared__ double part[3][4];
  double s_obj = 0.0, s_clip = 0.0, s_cnt = 0.0;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
    const bool on = !mask || mask[i];
    const float u = expf(lt[i] - lp[i]), w = expf(lp[i] - lb[i]), a = adv[i];
    const float unclipped = u * a, clipped = fminf(fmaxf(u, 1.f - eps), 1.f + eps) * a;
    const float o = on ? w * fminf(unclipped, clipped) : 0.f;
    if (obj_out) obj_out[i] = o;
    s_obj += (double)o;
    s_clip += (on && clipped < unclipped) ? 1.0 : 0.0;
    s_cnt += on ? 1.0 : 0.0;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    s_obj += __shfl_xor(s_obj, o);
    s_clip += __shfl_xor(s_clip, o);
    s_cnt += __shfl_xor(s_cnt, o);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { part[0][wave] = s_obj; part[1][wave] = s_clip; part[2][wave] = s_cnt; }
  __syncthreads();
  if (threadIdx.x < 3) {
    const double v = part[threadIdx.x][0] + part[threadIdx.x][1] + part[threadIdx.x][2] + part[threadIdx.x][3];
    atomicAdd(&sums[threadIdx.x], v);
  }
}

}  // namespace

hipError_t launch_ppo_objective(hipStream_t s, int n, const float* lt, const float* lp, const float* lb,
                                const float* adv, const uint8_t* mask, float eps, float* obj_out,
                                double* sums) {
  if (n < 0 || !lt || !lp || !lb || !adv || !sums) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  const int grid = std::min((n + 255) / 256, 1024);
  ppo_objective_kernel<<<grid, 256, 0, s>>>(n, lt, lp, lb, adv, mask, eps, obj_out, sums);
  return hipGetLastError();
}

hipError_t launch_lse_finish(hipStream_t s, const void* part, int ld_rows, int n_tiles, const float* target_z,
                             const int32_t* target, const int32_t* pos, int n, float* out) {
  if (n <= 0 || n_tiles <= 0 || ld_rows < n || !part || !target_z || !target || !pos || !out ||
      ((uintptr_t)part & 7))
    return hipErrorInvalidValue;
  lse_finish_kernel<<<(n + 255) / 256, 256, 0, s>>>(reinterpret_cast<const float2*>(part), ld_rows, n_tiles,
                                                    target_z, target, pos, n, out);
  return hipGetLastError();
}

hipError_t launch_token_logprob(hipStream_t s, const float* logits, int n, int vocab, float inv_t,
                                const int32_t* target, const int32_t* pos, float* out) {
  if (n <= 0 || vocab <= 0 || !logits || !target || !pos || !out || !(inv_t > 0.f) ||
      ((uintptr_t)logits & 15))
    return hipErrorInvalidValue;
  token_logprob_kernel<<<n, LP_THREADS, 0, s>>>(logits, vocab, inv_t, target, pos, out);
  return hipGetLastError();
}

}  // namespace areal
