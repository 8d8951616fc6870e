// Log-sum-exp merge of the prefix partial and the suffix partial, and the LSE export.
//
// Two attention results over disjoint key sets A and B of the same query combine as
//   LSE = ln(e^{LSE_A} + e^{LSE_B}),  O = e^{LSE_A - LSE} O_A + e^{LSE_B - LSE} O_B,
// which is exactly the softmax over A u B.  Here A = the shared video prefix (Sec. 5.1 of
// the paper: computed once, reused by all rollouts) and B = the rollout's own tokens.
// Pure streaming work: 2 fp32 partial rows in, one output row out; HBM-bound.
#include <hip/hip_runtime.h>

#include "common.h"

namespace pa {
namespace {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// One thread handles 4 consecutive channels of one row; rows are walked grid-stride.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void merge_kernel(const float* __restrict__ o1, const float* __restrict__ lse1,
                                                    const float* __restrict__ o2, const float* __restrict__ lse2,
                                                    void* __restrict__ out, float* __restrict__ lse, int64_t rows,
                                                    int D, bool has_prefix) {
  const int per_row = D / 4;
  const int64_t total = rows * per_row;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    const int64_t row = idx / per_row;
    const int ch = (int)(idx - row * per_row);
    const float l2 = lse2[row];
    float a1 = 0.f, a2 = 1.f, l = l2;
    if (has_prefix) {
      const float l1 = lse1[row];
      const float m = fmaxf(l1, l2);  // finite: every row sees at least its own key
      const float w1 = expf(l1 - m), w2 = expf(l2 - m);
      const float tot = w1 + w2;
      const float inv = 1.0f / tot;
      a1 = w1 * inv;
      a2 = w2 * inv;
      l = m + logf(tot);
    }
    f32x4 r = a2 * *reinterpret_cast<const f32x4*>(o2 + idx * 4);
    if (has_prefix) r += a1 * *reinterpret_cast<const f32x4*>(o1 + idx * 4);
    if (OUT_BF16) {
      bf16x4 b = __builtin_convertvector(r, bf16x4);
      *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(out) + idx * 4) = b;
    } else {
      *reinterpret_cast<f32x4*>(static_cast<float*>(out) + idx * 4) = r;
    }
    if (ch == 0) lse[row] = l;
  }
}

// n-way merge: one thread handles 4 consecutive channels of one (token, head) row.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void merge_n_kernel(MergeNArgs a) {
  const int per_row = a.D / 4;
  const int64_t rows = a.T * a.Hq;
  const int64_t total = rows * per_row;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    const int64_t row = idx / per_row;
    const int ch = (int)(idx - row * per_row);
    float m = -INFINITY;
    for (int i = 0; i < a.n; ++i) m = fmaxf(m, a.lse[i][row]);
    float tot = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < a.n; ++i) {
      const float w = expf(a.lse[i][row] - m);  // a partial over no keys has LSE = -inf and weight 0
      tot += w;
      acc += w * *reinterpret_cast<const f32x4*>(a.o[i] + idx * 4);
    }
    const f32x4 r = acc * (1.0f / tot);
    if (OUT_BF16) {
      *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(a.out) + idx * 4) = __builtin_convertvector(r, bf16x4);
    } else {
      *reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + idx * 4) = r;
    }
    if (ch == 0) {
      const float l = m + logf(tot);
      if (a.lse_out) {
        const int64_t t = row / a.Hq, h = row - t * a.Hq;
        a.lse_out[h * a.T + t] = l;
      }
      if (a.lse_th_out) a.lse_th_out[row] = l;
    }
  }
}

// [T, Hq] -> [Hq, T]
__global__ __launch_bounds__(256) void lse_export_kernel(const float* __restrict__ in, float* __restrict__ out,
                                                         int64_t T, int Hq) {
  const int64_t total = T * Hq;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    const int64_t h = idx / T, t = idx - h * T;
    out[idx] = in[t * Hq + h];
  }
}

}  // namespace

int launch_merge(const MergeArgs& a, void* stream) {
  if (a.rows == 0) return 0;
  const int64_t total = a.rows * (a.D / 4);
  const int64_t want = (total + 255) / 256;
  const int blocks = (int)(want < 256 * 32 ? want : 256 * 32);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (a.dtype == PA_BF16)
    merge_kernel<true><<<blocks, 256, 0, s>>>(a.o1, a.lse1, a.o2, a.lse2, a.out, a.lse, a.rows, a.D, a.has_prefix);
  else
    merge_kernel<false><<<blocks, 256, 0, s>>>(a.o1, a.lse1, a.o2, a.lse2, a.out, a.lse, a.rows, a.D, a.has_prefix);
  return (int)hipGetLastError();
}

int launch_merge_n(const MergeNArgs& a, void* stream) {
  const int64_t total = a.T * a.Hq * (a.D / 4);
  if (total == 0) return 0;
  const int64_t want = (total + 255) / 256;
  const int blocks = (int)(want < 256 * 32 ? want : 256 * 32);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (a.dtype == PA_BF16)
    merge_n_kernel<true><<<blocks, 256, 0, s>>>(a);
  else
    merge_n_kernel<false><<<blocks, 256, 0, s>>>(a);
  return (int)hipGetLastError();
}

int launch_lse_export(const float* lse_th, float* lse_ht, int64_t T, int32_t Hq, void* stream) {
  const int64_t total = T * Hq;
  if (total == 0) return 0;
  const int64_t want = (total + 255) / 256;
  const int blocks = (int)(want < 256 * 16 ? want : 256 * 16);
  lse_export_kernel<<<blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(lse_th, lse_ht, T, Hq);
  return (int)hipGetLastError();
}

}  // namespace pa
