// Fused vocabulary-wide sampler: temperature, fixed-point softmax mass,
// top-p nucleus, Philox draw, behaviour and full log-probabilities.
//
// One work-group of 16 wavefronts per row of logits.  The row is cut into
// segments of 256 consecutive token ids (one wavefront pass, 4 ids per lane,
// 16-byte loads); all order-sensitive steps work on per-segment integer sums
// in LDS, so the result does not depend on how the row was split.
//
// With few rows (fewer than half the compute units) and the whole vocabulary
// kept (top-p = 1) a row is spread over up to 64 work-groups instead: partial
// maxima, then per-segment masses, go through a scratch buffer in device
// memory, and a third launch scans the masses and picks the token.  The masses
// are integers and the maximum is exact, so the token is the same either way.
//
// Determinism contract (include/areal.h, areal_sample_logprob): the token id
// is a pure function of the float32 logits.  Every floating-point step that
// feeds an integer decision is a single IEEE float32 operation; contraction
// into fused multiply-add is switched off for this whole file.
#include <algorithm>
#include <mutex>
#include <string>

#include "../../include/areal.h"
#include "kernels.hpp"

#pragma clang fp contract(off)

namespace areal {

constexpr int SEG = 256, MAX_SEG = 1024;       // ids per segment, segments per row at most
constexpr int SAMPLER_MAX_PARTS = 64;          // work-groups one row can be spread over
constexpr int SAMPLER_SPLIT_MAX_ROWS = AREAL_SAMPLE_STATIC_MAX_ROWS;   // rows the scratch buffer holds
static_assert(AREAL_SAMPLE_STATIC_MAX_VOCAB == SEG * MAX_SEG, "header limit = segments x ids per segment");

namespace {

constexpr int TPB = 1024, NWAVES = 16;
constexpr int NBINS = 257;   // masses are 33-bit (0 .. 2^32); top level bins = c >> 24


typedef unsigned long long u64;

// ---- specified exponential -----------------------------------------------
__device__ __forceinline__ float sexp(float x) {
  const float xs = fmaxf(x, -25.0f);
  const float n = __builtin_rintf(xs * 1.44269502162933349609375f);          // 0x3FB8AA3B
  float r = xs - n * 0.693359375f;                                          // exact product
  r = r - n * -2.12194442749023437500e-4f;                                  // 0xB95E8083
  float p = 1.98412701138295233249664306640625e-4f;                         // 1/7!
  p = p * r; p = p + 1.388888922519981861114501953125e-3f;                   // 1/6!
  p = p * r; p = p + 8.333333767950534820556640625e-3f;                      // 1/5!
  p = p * r; p = p + 4.16666679084300994873046875e-2f;                       // 1/4!
  p = p * r; p = p + 0.1666666716337203979492187500f;                        // 1/3!
  p = p * r; p = p + 0.5f;
  p = p * r; p = p + 1.0f;
  p = p * r; p = p + 1.0f;
  float w = ldexpf(p, (int)n);
  w = fminf(w, 1.0f);
  return x < -25.0f ? 0.0f : w;
}
__device__ __forceinline__ u64 mass_of(float z, float m) {
  // floor(w * 2^32) for w in [0, 1]: the product is exact (power-of-two scale); below 2^32 it
  // fits the 32-bit truncating conversion, and only w = 1 gives 2^32 itself
  const float w = sexp(z - m);
  return w >= 1.0f ? (1ull << 32) : (u64)__float2uint_rz(w * 4294967296.0f);
}

// ---- Philox4x32-10 (Salmon et al., SC'11) ----------------------------------
__device__ __forceinline__ u64 philox_draw(u64 seed, uint32_t seq_id, uint32_t position) {
  uint32_t c0 = position, c1 = seq_id, c2 = 0, c3 = 0;
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return ((u64)c1 << 32) | c0;
}

// ---- wave / block primitives on 64-bit integers -----------------------------
__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int o) {
  uint32_t lo = __shfl_xor((uint32_t)v, o), hi = __shfl_xor((uint32_t)(v >> 32), o);
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_up_u64(u64 v, int o) {
  uint32_t lo = __shfl_up((uint32_t)v, o), hi = __shfl_up((uint32_t)(v >> 32), o);
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_u64(u64 v, int src) {
  uint32_t lo = __shfl((uint32_t)v, src), hi = __shfl((uint32_t)(v >> 32), src);
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += shfl_xor_u64(v, o);
  return v;
}
__device__ __forceinline__ u64 wave_incl_scan_u64(u64 v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const u64 t = shfl_up_u64(v, o);
    if (lane >= o) v += t;
  }
  return v;
}
// Inclusive scan over the 1024 threads of the block; `total` = sum of all.
__device__ __forceinline__ u64 block_incl_scan_u64(u64 v, u64* wave_tot, u64& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_incl_scan_u64(v, lane);
  __syncthreads();                       // wave_tot may still be read from a previous use
  if (lane == 63) wave_tot[wave] = v;
  __syncthreads();
  u64 before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NWAVES; ++w) {
    const u64 t = wave_tot[w];
    if (w < wave) before += t;
    all += t;
  }
  total = all;
  return v + before;
}

struct Row {
  const float* lp;
  int V;
  bool vec;            // rows are 16-byte aligned and V % 4 == 0
  float inv_t;
};
// z of ids id0 .. id0+3 (-inf beyond the vocabulary)
__device__ __forceinline__ void load_z4(const Row& r, int id0, float (&z)[4]) {
  if (r.vec) {
    if (id0 < r.V) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(r.lp + id0);
#pragma unroll
      for (int k = 0; k < 4; ++k) z[k] = v[k] * r.inv_t;
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) z[k] = -INFINITY;
    }
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) z[k] = id0 + k < r.V ? r.lp[id0 + k] * r.inv_t : -INFINITY;
  }
}

// Highest bin b with  sum_{b' >= b} hist[b'] >= need ; returns b and the mass
// strictly above it.  Executed by wave 0 (all 64 lanes), result in every lane.
__device__ __forceinline__ int find_bin(const u64* hist, u64 need, int lane, u64& above_out) {
  constexpr int PER = 5;                 // 64 * 5 >= 257
  u64 chunk = 0;
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    const int b = lane * PER + k;
    if (b < NBINS) chunk += hist[b];
  }
  // suffix[lane] = sum of chunks of lanes >= lane
  u64 suf = chunk;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const u64 t = shfl_u64(suf, min(lane + o, 63));
    if (lane + o < 64) suf += t;
  }
  const u64 ok = __ballot(suf >= need);
  const int L = 63 - __builtin_clzll(ok);        // ok != 0: total mass >= need
  int bsel = 0;
  u64 above = 0;
  if (lane == L) {
    above = suf - chunk;
    for (int k = PER - 1; k >= 0; --k) {
      const int b = lane * PER + k;
      if (b >= NBINS) continue;
      const u64 h = hist[b];
      if (above + h >= need) { bsel = b; break; }
      above += h;
    }
  }
  bsel = __shfl(bsel, L);
  above_out = shfl_u64(above, L);
  return bsel;
}

// The last step of both variants.  segmass[s] = kept mass of segment s (LDS), segtie[s] = ties
// at the threshold before segment s (top-p < 1 only); draws (or takes the forced token), walks
// the chosen segment in id order and writes the outputs of `row`.
__device__ __forceinline__ void choose_token(const Row& R, int row, int nseg, float m, u64 S_total, u64 S_nuc,
                                             bool all_in, u64 tau, u64 n_take, const u64* segmass,
                                             const uint32_t* segtie, u64* wave_tot, u64* sh_u64, int* sh_int,
                                             u64 seed, const int32_t* __restrict__ seq_ids,
                                             const int32_t* __restrict__ positions,
                                             const int32_t* __restrict__ forced,
                                             int32_t* __restrict__ tokens_out, float* __restrict__ logp_behav,
                                             float* __restrict__ logp_full) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, V = R.V;
  int tok;
  u64 base = 0;          // kept mass before the chosen segment (draw path)
  u64 r = 0;
  if (forced) {
    tok = forced[row];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    if (tid == 0) sh_int[2] = tok / SEG;
  } else {
    const u64 Rbits = philox_draw(seed, (uint32_t)seq_ids[row], (uint32_t)positions[row]);
    r = __umul64hi(Rbits, S_nuc);
    u64 tot;
    const u64 mine = tid < nseg ? segmass[tid] : 0;
    const u64 incl = block_incl_scan_u64(mine, wave_tot, tot);
    if (tid < nseg && incl > r && incl - mine <= r) { sh_int[2] = tid; sh_u64[1] = incl - mine; }
    tok = -1;
  }
  __syncthreads();
  const int sseg = sh_int[2];
  base = sh_u64[1];

  // wave 0 walks the chosen segment in id order
  if (wave == 0) {
    float z[4];
    load_z4(R, sseg * SEG + lane * 4, z);
    u64 c[4], kept[4];
    uint32_t tie_lane = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      c[k] = mass_of(z[k], m);
      if (!all_in && sseg * SEG + lane * 4 + k < V && c[k] == tau) tie_lane += 1;
    }
    // ties before this lane's first id
    uint32_t tie_before = 0;
    if (!all_in) {
      const u64 incl = wave_incl_scan_u64(tie_lane, lane);
      tie_before = segtie[sseg] + (uint32_t)(incl - tie_lane);
    }
    u64 lane_sum = 0;
    bool member[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool in = sseg * SEG + lane * 4 + k < V;
      if (all_in) {
        member[k] = in;
      } else if (c[k] > tau) {
        member[k] = in;
      } else if (c[k] == tau && in) {
        member[k] = tie_before < n_take;
        tie_before += 1;
      } else {
        member[k] = false;
      }
      kept[k] = member[k] ? c[k] : 0;
      lane_sum += kept[k];
    }
    int k_sel = -1;
    if (forced) {
      if ((tok % SEG) / 4 == lane) k_sel = tok & 3;
    } else {
      const u64 incl = wave_incl_scan_u64(lane_sum, lane);
      u64 run = base + incl - lane_sum;
      if (run <= r && r < run + lane_sum) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if (k_sel < 0) {
            run += kept[k];
            if (run > r) k_sel = k;
          }
        }
      }
    }
    if (k_sel >= 0) {
      const int t = sseg * SEG + lane * 4 + k_sel;
      u64 ct = 0;
      float zt = 0.f;
      bool mem = false;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (k == k_sel) { ct = c[k]; zt = z[k]; mem = member[k]; }
      tokens_out[row] = t;
      logp_behav[row] = (mem && ct > 0) ? (float)(log((double)ct) - log((double)S_nuc)) : -INFINITY;
      if (logp_full)
        logp_full[row] = (float)((double)(zt - m) - (log((double)S_total) - 32.0 * 0.69314718055994530942));
    }
  }
}

__global__ __launch_bounds__(TPB) void sampler_kernel(
    int V, const float* __restrict__ logits, const int32_t* __restrict__ seq_ids,
    const int32_t* __restrict__ positions, float inv_t, float top_p, u64 seed,
    const int32_t* __restrict__ forced, int32_t* __restrict__ tokens_out,
    float* __restrict__ logp_behav, float* __restrict__ logp_full) {
  __shared__ u64 segmass[MAX_SEG];
  __shared__ uint32_t segtie[MAX_SEG];       // ties per segment, then exclusive prefix
  __shared__ u64 hist_mass[NBINS];
  __shared__ uint32_t hist_cnt[NBINS];
  __shared__ u64 wave_tot[NWAVES];
  __shared__ float wave_max_s[NWAVES];
  __shared__ u64 sh_u64[4];                  // broadcast slots
  __shared__ int sh_int[4];

  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  Row R;
  R.lp = logits + (int64_t)row * V;
  R.V = V;
  R.vec = (V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
  R.inv_t = inv_t;
  const int nseg = (V + SEG - 1) / SEG;
  const bool all_in = top_p >= 1.0f;

  // ---- pass A: m = max z ----------------------------------------------------
  float mx = -INFINITY;
  for (int s = wave; s < nseg; s += NWAVES) {
    float z[4];
    load_z4(R, s * SEG + lane * 4, z);
    mx = fmaxf(fmaxf(mx, fmaxf(z[0], z[1])), fmaxf(z[2], z[3]));
  }
  mx = wave_max(mx);
  if (lane == 0) wave_max_s[wave] = mx;
  __syncthreads();
  float m = wave_max_s[0];
#pragma unroll
  for (int w = 1; w < NWAVES; ++w) m = fmaxf(m, wave_max_s[w]);

  // ---- pass B: per-segment mass, S = total mass --------------------------------
  for (int s = wave; s < nseg; s += NWAVES) {
    float z[4];
    load_z4(R, s * SEG + lane * 4, z);
    u64 c = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) c += mass_of(z[k], m);
    c = wave_sum_u64(c);
    if (lane == 0) segmass[s] = c;
  }
  __syncthreads();
  u64 S_total;
  block_incl_scan_u64(tid < nseg ? segmass[tid] : 0, wave_tot, S_total);

  // ---- nucleus threshold (top_p < 1): radix select on the 33-bit masses ---------
  u64 tau = 0, n_take = 0, S_nuc = S_total;
  if (!all_in) {
    u64 target = (u64)ceil((double)top_p * (double)S_total);
    if (target < 1) target = 1;
    if (target > S_total) target = S_total;
    u64 mass_above = 0, prefix = 0;
    uint32_t cnt_tau = 0;
    for (int level = 0; level < 4; ++level) {
      const int shift = 24 - 8 * level;
      for (int b = tid; b < NBINS; b += TPB) { hist_mass[b] = 0; hist_cnt[b] = 0; }
      __syncthreads();
      for (int s = wave; s < nseg; s += NWAVES) {
        float z[4];
        load_z4(R, s * SEG + lane * 4, z);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const u64 c = mass_of(z[k], m);
          const bool in = (s * SEG + lane * 4 + k < V) && (level == 0 || (c >> (shift + 8)) == prefix);
          const int bin = level == 0 ? (int)(c >> 24) : (int)((c >> shift) & 255);
          // near-flat logits put most ids into one bin: add once per wave then
          const int bin0 = __builtin_amdgcn_readfirstlane(bin);
          if (__all(in && bin == bin0)) {
            const u64 tot = wave_sum_u64(c);
            if (lane == 0) {
              atomicAdd(&hist_mass[bin0], tot);
              atomicAdd(&hist_cnt[bin0], 64u);
            }
          } else if (in) {
            atomicAdd(&hist_mass[bin], c);
            atomicAdd(&hist_cnt[bin], 1u);
          }
        }
      }
      __syncthreads();
      if (wave == 0) {
        u64 above;
        const int b = find_bin(hist_mass, target - mass_above, lane, above);
        if (lane == 0) {
          sh_int[0] = b;
          sh_u64[0] = mass_above + above;
          sh_int[1] = (int)hist_cnt[b];
        }
      }
      __syncthreads();
      const int bsel = sh_int[0];
      mass_above = sh_u64[0];
      cnt_tau = (uint32_t)sh_int[1];
      __syncthreads();
      if (level == 0) {
        prefix = (u64)bsel;
        if (bsel == 256) { prefix = 1ull << 32; break; }   // only c = 2^32 lives in this bin
      } else {
        prefix = (prefix << 8) | (u64)bsel;
      }
    }
    tau = prefix;
    n_take = (target - mass_above + tau - 1) / tau;
    if (n_take > cnt_tau) n_take = cnt_tau;                 // cannot happen; keeps indices sane
    S_nuc = mass_above + n_take * tau;

    // per-segment mass above tau and tie counts; then fold the taken ties in
    for (int s = wave; s < nseg; s += NWAVES) {
      float z[4];
      load_z4(R, s * SEG + lane * 4, z);
      u64 gt = 0;
      uint32_t tie = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const u64 c = mass_of(z[k], m);
        const bool in = s * SEG + lane * 4 + k < V;
        if (in && c > tau) gt += c;
        if (in && c == tau) tie += 1;
      }
      gt = wave_sum_u64(gt);
      tie = (uint32_t)wave_sum_u64(tie);
      if (lane == 0) { segmass[s] = gt; segtie[s] = tie; }
    }
    __syncthreads();
    {
      u64 tot;
      const u64 mine = tid < nseg ? segtie[tid] : 0;
      const u64 incl = block_incl_scan_u64(mine, wave_tot, tot);
      const u64 excl = incl - mine;
      __syncthreads();
      if (tid < nseg) {
        const u64 takes = excl >= n_take ? 0 : (n_take - excl < mine ? n_take - excl : mine);
        segmass[tid] += takes * tau;
        segtie[tid] = (uint32_t)excl;                       // now: ties before this segment
      }
      __syncthreads();
    }
  }

  choose_token(R, row, nseg, m, S_total, S_nuc, all_in, tau, n_take, segmass, segtie, wave_tot, sh_u64, sh_int,
               seed, seq_ids, positions, forced, tokens_out, logp_behav, logp_full);
}

// ---- a row spread over several work-groups (top-p = 1, few rows) -------------------
// Work-group (part, row) of 4 waves takes segments part*4 + wave, then every parts*4-th.
constexpr int SPLIT_TPB = 256, SPLIT_WAVES = 4;

__global__ __launch_bounds__(SPLIT_TPB) void sampler_split_max_kernel(int V, const float* __restrict__ logits,
                                                                      float inv_t, int parts,
                                                                      float* __restrict__ pmax) {
  __shared__ float wmax[SPLIT_WAVES];
  const int row = blockIdx.y, part = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Row R;
  R.lp = logits + (int64_t)row * V;
  R.V = V;
  R.vec = (V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
  R.inv_t = inv_t;
  const int nseg = (V + SEG - 1) / SEG;
  float mx = -INFINITY;
  for (int sg = part * SPLIT_WAVES + wave; sg < nseg; sg += parts * SPLIT_WAVES) {
    float z[4];
    load_z4(R, sg * SEG + lane * 4, z);
    mx = fmaxf(fmaxf(mx, fmaxf(z[0], z[1])), fmaxf(z[2], z[3]));
  }
  mx = wave_max(mx);
  if (lane == 0) wmax[wave] = mx;
  __syncthreads();
  if (threadIdx.x == 0)
    pmax[row * SAMPLER_MAX_PARTS + part] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
}

__device__ __forceinline__ float row_max_of_parts(const float* __restrict__ pmax, int row, int parts) {
  float m = pmax[row * SAMPLER_MAX_PARTS];
  for (int p = 1; p < parts; ++p) m = fmaxf(m, pmax[row * SAMPLER_MAX_PARTS + p]);
  return m;
}

__global__ __launch_bounds__(SPLIT_TPB) void sampler_split_mass_kernel(int V, const float* __restrict__ logits,
                                                                       float inv_t, int parts,
                                                                       const float* __restrict__ pmax,
                                                                       u64* __restrict__ segmass_g) {
  const int row = blockIdx.y, part = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Row R;
  R.lp = logits + (int64_t)row * V;
  R.V = V;
  R.vec = (V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
  R.inv_t = inv_t;
  const int nseg = (V + SEG - 1) / SEG;
  const float m = row_max_of_parts(pmax, row, parts);
  for (int sg = part * SPLIT_WAVES + wave; sg < nseg; sg += parts * SPLIT_WAVES) {
    float z[4];
    load_z4(R, sg * SEG + lane * 4, z);
    u64 c = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) c += mass_of(z[k], m);
    c = wave_sum_u64(c);
    if (lane == 0) segmass_g[(int64_t)row * MAX_SEG + sg] = c;
  }
}

__global__ __launch_bounds__(TPB) void sampler_split_pick_kernel(
    int V, const float* __restrict__ logits, const int32_t* __restrict__ seq_ids,
    const int32_t* __restrict__ positions, float inv_t, u64 seed, const int32_t* __restrict__ forced, int parts,
    const float* __restrict__ pmax, const u64* __restrict__ segmass_g, int32_t* __restrict__ tokens_out,
    float* __restrict__ logp_behav, float* __restrict__ logp_full) {
  __shared__ u64 segmass[MAX_SEG];
  __shared__ u64 wave_tot[NWAVES];
  __shared__ u64 sh_u64[4];
  __shared__ int sh_int[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  Row R;
  R.lp = logits + (int64_t)row * V;
  R.V = V;
  R.vec = (V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
  R.inv_t = inv_t;
  const int nseg = (V + SEG - 1) / SEG;
  const float m = row_max_of_parts(pmax, row, parts);
  const u64 mine = tid < nseg ? segmass_g[(int64_t)row * MAX_SEG + tid] : 0;
  segmass[tid] = mine;
  u64 S_total;
  block_incl_scan_u64(mine, wave_tot, S_total);        // its barriers also publish segmass
  choose_token(R, row, nseg, m, S_total, S_total, true, 0, 0, segmass, nullptr, wave_tot, sh_u64, sh_int, seed,
               seq_ids, positions, forced, tokens_out, logp_behav, logp_full);
}

}  // namespace

size_t sampler_scratch_bytes() { return SAMPLER_SPLIT_MAX_ROWS * (SAMPLER_MAX_PARTS * 4 + (size_t)MAX_SEG * 8); }

hipError_t launch_sampler(hipStream_t s, int n, int vocab, const float* logits, const int32_t* seq_ids,
                          const int32_t* positions, float inv_temperature, float top_p, uint64_t seed,
                          const int32_t* forced, int32_t* tokens_out, float* logp_behav,
                          float* logp_full, void* scratch) {
  if (n <= 0 || vocab <= 0 || (vocab + SEG - 1) / SEG > MAX_SEG || !logits || !tokens_out ||
      !logp_behav || !(inv_temperature > 0.f) || !(top_p > 0.f))
    return hipErrorInvalidValue;
  if (!forced && (!seq_ids || !positions)) return hipErrorInvalidValue;
  // few rows, whole vocabulary kept: 2 .. 64 work-groups of four waves per row, about four per
  // compute unit (the specified exponential is arithmetic-bound: it wants every SIMD's wave slots)
  const int nseg = (vocab + SEG - 1) / SEG;
  int parts = std::min(SAMPLER_MAX_PARTS, 1024 / n);
  parts = std::min(parts, (nseg + SPLIT_WAVES - 1) / SPLIT_WAVES);
  if (scratch && top_p >= 1.0f && n <= SAMPLER_SPLIT_MAX_ROWS && parts >= 2) {
    if ((uintptr_t)scratch & 15) return hipErrorInvalidValue;
    u64* segmass_g = reinterpret_cast<u64*>(scratch);
    float* pmax = reinterpret_cast<float*>(segmass_g + (size_t)SAMPLER_SPLIT_MAX_ROWS * MAX_SEG);
    const dim3 grid(parts, n);
    sampler_split_max_kernel<<<grid, SPLIT_TPB, 0, s>>>(vocab, logits, inv_temperature, parts, pmax);
    sampler_split_mass_kernel<<<grid, SPLIT_TPB, 0, s>>>(vocab, logits, inv_temperature, parts, pmax, segmass_g);
    sampler_split_pick_kernel<<<n, TPB, 0, s>>>(vocab, logits, seq_ids, positions, inv_temperature, (u64)seed,
                                                forced, parts, pmax, segmass_g, tokens_out, logp_behav, logp_full);
    return hipGetLastError();
  }
  sampler_kernel<<<n, TPB, 0, s>>>(vocab, logits, seq_ids, positions, inv_temperature, top_p,
                                   (u64)seed, forced, tokens_out, logp_behav, logp_full);
  return hipGetLastError();
}

}  // namespace areal

// ---- the entry point that allocates nothing -----------------------------------------
// Same sampler, for callers that cannot allocate or hand over a workspace: the scratch
// buffer of the spread variant is a file-scope device array.  Each GPU the library runs on
// holds its own copy (about 1 MiB) at its own address until the process ends; the address is
// looked up once per device, with that device current, and only that pointer (never the
// array's name, which in host code is a stand-in, not a device address) is handed to kernels.
namespace {

static __device__ __align__(256) unsigned char g_sampler_scratch[areal::SAMPLER_SPLIT_MAX_ROWS *
                                                                (areal::SAMPLER_MAX_PARTS * 4 +
                                                                 (size_t)areal::MAX_SEG * 8)];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of the array (null + message on failure).
void* static_scratch(std::string* why) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *why = std::string("hipGetDevice: ") + (e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_sampler_scratch));
    if (e != hipSuccess || !p) {
      *why = std::string("hipGetSymbolAddress(sampler scratch): ") + hipGetErrorString(e);
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int areal_sample_logprob_static(void* hip_stream, int32_t n, int32_t vocab, const float* logits,
                                           const int32_t* seq_ids, const int32_t* positions, float temperature,
                                           float top_p, uint64_t seed, const int32_t* forced,
                                           int32_t* tokens_out, float* logp_behav, float* logp_full) {
  if (n == 0) return AREAL_OK;
  if (n < 0 || vocab <= 0 || !logits || !tokens_out || !logp_behav || (!forced && (!seq_ids || !positions))) {
    areal::set_global_error("areal_sample_logprob_static: NULL argument, negative count or no vocabulary");
    return AREAL_E_INVAL;
  }
  if (n > AREAL_SAMPLE_STATIC_MAX_ROWS || vocab > AREAL_SAMPLE_STATIC_MAX_VOCAB) {
    areal::set_global_error("areal_sample_logprob_static: at most " +
                            std::to_string(AREAL_SAMPLE_STATIC_MAX_ROWS) + " rows of at most " +
                            std::to_string(AREAL_SAMPLE_STATIC_MAX_VOCAB) +
                            " logits fit the static scratch buffer: split the batch, or use areal_sample_logprob");
    return AREAL_E_NOMEM;
  }
  if (!(temperature > 0.f) || !(top_p > 0.f)) {
    areal::set_global_error("areal_sample_logprob_static: temperature and top_p must be > 0");
    return AREAL_E_INVAL;
  }
  std::string why;
  void* scratch = static_scratch(&why);
  if (!scratch) {
    areal::set_global_error(why);
    return AREAL_E_HIP;
  }
  const hipError_t e = areal::launch_sampler((hipStream_t)hip_stream, n, vocab, logits, seq_ids, positions,
                                             1.0f / temperature, top_p, seed, forced, tokens_out, logp_behav,
                                             logp_full, scratch);
  if (e != hipSuccess) {
    areal::set_global_error(std::string("areal_sample_logprob_static: ") + hipGetErrorString(e));
    return e == hipErrorInvalidValue ? AREAL_E_INVAL : AREAL_E_HIP;
  }
  return AREAL_OK;
}
