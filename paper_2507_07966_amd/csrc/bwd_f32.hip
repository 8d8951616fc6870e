// Backward in fp32 (small problems, tight checks): plain kernels, one wavefront per query
// row for dQ and one wavefront per (key, kv head) for dK/dV.  Lanes split the head dimension;
// every dot product is a wavefront reduction.  Same arithmetic as the bf16 path:
//   W_j = exp(scale <q, k_j> - LSE),  dS_j = W_j (<dO, v_j> - delta),
//   dQ = scale sum_j dS_j k_j,  dK_j = scale sum_rows dS_j q,  dV_j = sum_rows W_j dO,
// a prefix key summing over the rows of all rollouts (paper Sec. 5.1: shared video prefix).
#include <hip/hip_runtime.h>

#include "bwd.h"

namespace pa {
namespace {

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) x += __shfl_xor(x, s, 64);
  return x;
}

// E = D / 64 channels per lane: lane l holds channels l + 64 e
template <int E>
__device__ inline void load_row(const float* p, int lane, float (&x)[E]) {
#pragma unroll
  for (int e = 0; e < E; ++e) x[e] = p[lane + 64 * e];
}
template <int E>
__device__ inline float dot_row(const float (&a)[E], const float (&b)[E]) {
  float acc = 0.f;
#pragma unroll
  for (int e = 0; e < E; ++e) acc += a[e] * b[e];
  return wave_sum(acc);
}

template <int E>
__global__ __launch_bounds__(256) void bwd_dq_f32_kernel(const float* __restrict__ q, const float* __restrict__ d_out,
                                                         const float* __restrict__ k_prefix,
                                                         const float* __restrict__ v_prefix,
                                                         const float* __restrict__ k_suffix,
                                                         const float* __restrict__ v_suffix,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         float* __restrict__ dq, const int32_t* __restrict__ cu, int G,
                                                         int64_t T, int64_t P, int Hq, int Hkv, int group,
                                                         float scale) {
  constexpr int D = 64 * E;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (token, head) row
  if (row >= T * Hq) return;
  const int t = (int)(row / Hq), h = (int)(row - (int64_t)t * Hq), c = h / group;
  int g = 0;
  while (g + 1 < G && cu[g + 1] <= t) ++g;
  const int off_g = cu[g];
  float qv[E], dov[E], acc[E];
  load_row<E>(q + row * D, lane, qv);
  load_row<E>(d_out + row * D, lane, dov);
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  const float l = lse[row], dl = delta[row];
  const int64_t nk = P + (t - off_g) + 1;
  for (int64_t j = 0; j < nk; ++j) {
    const int64_t kr = (j < P ? j : (int64_t)off_g + (j - P)) * Hkv + c;
    const float* kp = (j < P ? k_prefix : k_suffix) + kr * D;
    const float* vp = (j < P ? v_prefix : v_suffix) + kr * D;
    float kv[E], vv[E];
    load_row<E>(kp, lane, kv);
    load_row<E>(vp, lane, vv);
    const float w = expf(scale * dot_row<E>(qv, kv) - l);
    const float ds = w * (dot_row<E>(dov, vv) - dl);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += ds * kv[e];
  }
#pragma unroll
  for (int e = 0; e < E; ++e) dq[row * D + lane + 64 * e] = scale * acc[e];
}

template <int E>
__global__ __launch_bounds__(256) void bwd_dkv_f32_kernel(const float* __restrict__ q, const float* __restrict__ d_out,
                                                          const float* __restrict__ k_prefix,
                                                          const float* __restrict__ v_prefix,
                                                          const float* __restrict__ k_suffix,
                                                          const float* __restrict__ v_suffix,
                                                          const float* __restrict__ lse, const float* __restrict__ delta,
                                                          float* __restrict__ dk_prefix, float* __restrict__ dv_prefix,
                                                          float* __restrict__ dk_suffix, float* __restrict__ dv_suffix,
                                                          const int32_t* __restrict__ cu, int G, int64_t T, int64_t P,
                                                          int Hq, int Hkv, int group, float scale) {
  constexpr int D = 64 * E;
  const int lane = threadIdx.x & 63;
  const int64_t kc = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (key, kv head), prefix keys first
  if (kc >= (P + T) * Hkv) return;
  const int64_t jj = kc / Hkv;
  const int c = (int)(kc - jj * Hkv);
  const bool pre = jj < P;
  const int64_t kr = (pre ? jj : jj - P) * Hkv + c;
  float kv[E], vv[E], ak[E], av[E];
  load_row<E>((pre ? k_prefix : k_suffix) + kr * D, lane, kv);
  load_row<E>((pre ? v_prefix : v_suffix) + kr * D, lane, vv);
#pragma unroll
  for (int e = 0; e < E; ++e) {
    ak[e] = 0.f;
    av[e] = 0.f;
  }
  // rows that see the key: all packed tokens for a prefix key, else its own rollout from the key on
  int64_t t0 = 0, t1 = T;
  if (!pre) {
    const int tj = (int)(jj - P);
    int g = 0;
    while (g + 1 < G && cu[g + 1] <= tj) ++g;
    t0 = tj;
    t1 = cu[g + 1];
  }
  for (int64_t t = t0; t < t1; ++t)
    for (int h = c * group; h < (c + 1) * group; ++h) {
      const int64_t row = t * Hq + h;
      float qv[E], dov[E];
      load_row<E>(q + row * D, lane, qv);
      load_row<E>(d_out + row * D, lane, dov);
      const float w = expf(scale * dot_row<E>(qv, kv) - lse[row]);
      const float ds = w * (dot_row<E>(dov, vv) - delta[row]);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        ak[e] += ds * qv[e];
        av[e] += w * dov[e];
      }
    }
  float* dk = (pre ? dk_prefix : dk_suffix) + kr * D;
  float* dv = (pre ? dv_prefix : dv_suffix) + kr * D;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    dk[lane + 64 * e] = scale * ak[e];
    dv[lane + 64 * e] = av[e];
  }
}

const float* f(const void* p) { return static_cast<const float*>(p); }
float* fw(void* p) { return static_cast<float*>(p); }

}  // namespace

int launch_bwd_dq_f32(const BwdF32Args& a, void* stream) {
  const int64_t rows = a.T * a.Hq;
  if (rows == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = (unsigned)((rows + 3) / 4);
#define PA_LAUNCH(E)                                                                                          \
  bwd_dq_f32_kernel<E><<<grid, 256, 0, s>>>(f(a.q), f(a.d_out), f(a.k_prefix), f(a.v_prefix), f(a.k_suffix), \
                                            f(a.v_suffix), a.lse, a.delta, fw(a.dq), a.cu, a.G, a.T, a.P,    \
                                            a.Hq, a.Hkv, a.group, a.scale)
  if (a.D == 128) PA_LAUNCH(2); else PA_LAUNCH(1);
#undef PA_LAUNCH
  return (int)hipGetLastError();
}

int launch_bwd_dkv_f32(const BwdF32Args& a, void* stream) {
  const int64_t n = (a.P + a.T) * a.Hkv;
  if (n == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned grid = (unsigned)((n + 3) / 4);
#define PA_LAUNCH(E)                                                                                           \
  bwd_dkv_f32_kernel<E><<<grid, 256, 0, s>>>(f(a.q), f(a.d_out), f(a.k_prefix), f(a.v_prefix), f(a.k_suffix), \
                                             f(a.v_suffix), a.lse, a.delta, fw(a.dk_prefix), fw(a.dv_prefix), \
                                             fw(a.dk_suffix), fw(a.dv_suffix), a.cu, a.G, a.T, a.P, a.Hq,     \
                                             a.Hkv, a.group, a.scale)
  if (a.D == 128) PA_LAUNCH(2); else PA_LAUNCH(1);
#undef PA_LAUNCH
  return (int)hipGetLastError();
}

}  // namespace pa
