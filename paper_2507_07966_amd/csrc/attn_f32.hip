// fp32 attention pass (prefix or causal suffix) for fp32 inputs: plain FMA arithmetic, one
// wavefront per stacked query row, online softmax over chunks of 64 keys.  This path exists
// for small fp32 problems where exactness matters and speed does not; the bf16 MFMA
// kernels are the performance path.
//
// Same contract as the bf16 pass: for each stacked row it writes a normalised partial output
// and the natural-log LSE over the keys the pass covers (all P prefix keys, or the rollout's
// own keys 0..i).
#include <hip/hip_runtime.h>

#include "common.h"

namespace pa {
namespace {

__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <int D>
__global__ __launch_bounds__(256) void pass_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                       const float* __restrict__ v, float* __restrict__ o_part,
                                                       float* __restrict__ lse_part, const WorkItem* __restrict__ items,
                                                       const int32_t* __restrict__ cu, int Hq, int Hkv, int group,
                                                       float scale, bool causal) {
  __shared__ float qs[4][D];
  const WorkItem it = items[blockIdx.x];
  if (it.g < 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int off_g = cu[it.g];
  const int S_g = cu[it.g + 1] - off_g;
  const int nrows = S_g * group;
  const int64_t kv_row0 = causal ? off_g : 0;
  constexpr int ROWS_PER_WAVE = ROWS_PER_ITEM / 4;
  for (int rr = 0; rr < ROWS_PER_WAVE; ++rr) {
    const int m = it.row0 + wave * ROWS_PER_WAVE + rr;
    if (m >= nrows) break;  // wave-uniform
    const int i = m / group, hh = m - i * group;
    const int64_t row = (int64_t)(off_g + i) * Hq + it.c * group + hh;
    for (int d = lane; d < D; d += 64) qs[wave][d] = q[row * D + d];
    __builtin_amdgcn_wave_barrier();
    const int nk = causal ? i + 1 : it.nkeys;
    float mrun = -INFINITY, lrun = 0.f, o0 = 0.f, o1 = 0.f;
    for (int base = 0; base < nk; base += 64) {
      const int j = base + lane;
      float s = -INFINITY;
      if (j < nk) {
        const float* kr = k + ((kv_row0 + j) * Hkv + it.c) * D;
        float acc = 0.f;
        for (int d = 0; d < D; ++d) acc = fmaf(qs[wave][d], kr[d], acc);
        s = scale * acc;
      }
      const float m_new = fmaxf(mrun, wave_max(s));
      const float p = (j < nk) ? expf(s - m_new) : 0.f;
      const float alpha = expf(mrun - m_new);  // first chunk: exp(-inf) = 0
      lrun = lrun * alpha + wave_sum(p);
      o0 *= alpha;
      o1 *= alpha;
      const int cnt = (nk - base < 64) ? nk - base : 64;
      for (int jj = 0; jj < cnt; ++jj) {
        const float pj = __shfl(p, jj);
        const float* vr = v + ((kv_row0 + base + jj) * Hkv + it.c) * D;
        o0 = fmaf(pj, vr[lane], o0);
        if (D > 64) o1 = fmaf(pj, vr[lane + 64], o1);
      }
      mrun = m_new;
    }
    const float inv = 1.0f / lrun;
    o_part[row * D + lane] = o0 * inv;
    if (D > 64) o_part[row * D + lane + 64] = o1 * inv;
    if (lane == 0) lse_part[row] = mrun + logf(lrun);
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace

int launch_pass_f32(const PassArgs& a, void* stream) {
  if (a.num_items == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float* q = static_cast<const float*>(a.q);
  const float* k = static_cast<const float*>(a.k);
  const float* v = static_cast<const float*>(a.v);
  if (a.D == 64)
    pass_f32_kernel<64><<<(unsigned)a.num_items, 256, 0, s>>>(q, k, v, a.o_part, a.lse_part, a.items, a.cu, a.Hq,
                                                                 a.Hkv, a.group, a.scale, a.causal);
  else
    pass_f32_kernel<128><<<(unsigned)a.num_items, 256, 0, s>>>(q, k, v, a.o_part, a.lse_part, a.items, a.cu, a.Hq,
                                                                  a.Hkv, a.group, a.scale, a.causal);
  return (int)hipGetLastError();
}

}  // namespace pa
