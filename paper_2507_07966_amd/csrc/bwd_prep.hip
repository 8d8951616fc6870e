// Backward pre-pass: delta = <dO, O> per query row, and (bf16 path) the layouts the two
// backward passes read.
//
// The dK/dV pass walks, per kv head c, the stacked query rows M = t * group + j (t = packed
// token, j = q head inside the GQA group) in tiles of 64.  For each such tile this kernel writes
//   - the rows of Q and dO gathered into one contiguous row-major block [64][D],
//   - per row: LSE * log2(e), -delta and the packed token index.
// Rows past the last stacked row are zero, with a huge LSE (their weights become exactly 0)
// and token index INT32_MAX.  Cost: Q, dO and O are read once and Q, dO written once.
#include <hip/hip_runtime.h>

#include <climits>

#include "bwd.h"

namespace pa {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LSE_PAST_END = 1.0e30f;

__device__ inline float bf16_bits_to_float(unsigned short b) { return __uint_as_float((unsigned)b << 16); }

__device__ inline float dot8(u32x4 a, u32x4 b) {
  float acc = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    acc += bf16_bits_to_float((unsigned short)(a[w] & 0xffffu)) * bf16_bits_to_float((unsigned short)(b[w] & 0xffffu));
    acc += bf16_bits_to_float((unsigned short)(a[w] >> 16)) * bf16_bits_to_float((unsigned short)(b[w] >> 16));
  }
  return acc;
}

template <int D>
__global__ __launch_bounds__(256) void bwd_prep_bf16_kernel(
    const unsigned short* __restrict__ q, const unsigned short* __restrict__ out,
    const unsigned short* __restrict__ d_out, const float* __restrict__ lse, unsigned short* __restrict__ qs, unsigned short* __restrict__ dos,
    float* __restrict__ lse2s, float* __restrict__ deltas,
    int32_t* __restrict__ toks, int64_t T, int64_t Mpad, int Hq, int group) {
  constexpr int CPR = D / 8;  // 16-byte chunks per row
  const int64_t tiles_per_head = Mpad / ROWS_PER_ROW_TILE;
  const int c = (int)(blockIdx.x / tiles_per_head);
  const int64_t tile = blockIdx.x - c * tiles_per_head;
  const int64_t nrows = T * group;
  for (int n = threadIdx.x; n < ROWS_PER_ROW_TILE * CPR; n += 256) {
    const int row = n / CPR, ch = n - row * CPR;
    const int64_t m = tile * ROWS_PER_ROW_TILE + row;
    const bool valid = m < nrows;
    u32x4 wq = {0, 0, 0, 0}, wd = {0, 0, 0, 0}, wo = {0, 0, 0, 0};
    int64_t th = 0;
    int t = INT_MAX, h = 0;
    if (valid) {
      t = (int)(m / group);
      h = c * group + (int)(m - (int64_t)t * group);
      th = (int64_t)t * Hq + h;
      wq = *reinterpret_cast<const u32x4*>(q + th * D + ch * 8);
      wd = *reinterpret_cast<const u32x4*>(d_out + th * D + ch * 8);
      wo = *reinterpret_cast<const u32x4*>(out + th * D + ch * 8);
    }
    const int64_t srow = (int64_t)c * Mpad + m;
    *reinterpret_cast<u32x4*>(qs + srow * D + ch * 8) = wq;
    *reinterpret_cast<u32x4*>(dos + srow * D + ch * 8) = wd;
    // delta: the CPR consecutive lanes of a row add their partial dot products
    float part = dot8(wd, wo);
#pragma unroll
    for (int s = CPR / 2; s >= 1; s >>= 1) part += __shfl_xor(part, s, CPR);
    if (ch == 0) {
      deltas[srow] = -part;  // negated: the dK/dV pass starts its dW accumulators from it
      lse2s[srow] = valid ? lse[(int64_t)h * T + t] * LOG2E : LSE_PAST_END;
      toks[srow] = t;
    }
  }
}

// fp32 path: delta and the LSE in [T, Hq] order, one thread per (token, head) row.
__global__ __launch_bounds__(256) void bwd_delta_f32_kernel(const float* __restrict__ out,
                                                            const float* __restrict__ d_out,
                                                            const float* __restrict__ lse, float* __restrict__ delta,
                                                            float* __restrict__ lse_th, int64_t T, int Hq, int D) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= T * Hq) return;
  float acc = 0.f;
  for (int d = 0; d < D; ++d) acc += out[r * D + d] * d_out[r * D + d];
  delta[r] = acc;
  const int64_t t = r / Hq, h = r - t * Hq;
  lse_th[r] = lse[h * T + t];
}

}  // namespace

int launch_bwd_prep(const BwdPrepArgs& a, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (a.dtype != PA_BF16) {
    const int64_t rows = a.T * a.Hq;
    bwd_delta_f32_kernel<<<(unsigned)((rows + 255) / 256), 256, 0, s>>>(
        static_cast<const float*>(a.out), static_cast<const float*>(a.d_out), a.lse, a.delta, a.lse_th, a.T, a.Hq,
        a.D);
    return (int)hipGetLastError();
  }
  const int64_t blocks = (int64_t)a.Hkv * (a.Mpad / ROWS_PER_ROW_TILE);
  auto u = [](const void* p) { return static_cast<const unsigned short*>(p); };
  auto w = [](void* p) { return static_cast<unsigned short*>(p); };
  if (a.D == 128)
    bwd_prep_bf16_kernel<128><<<(unsigned)blocks, 256, 0, s>>>(u(a.q), u(a.out), u(a.d_out), a.lse, w(a.qs),
                                                                w(a.dos), a.lse2s, a.deltas,
                                                                a.toks, a.T, a.Mpad, a.Hq, a.group);
  else
    bwd_prep_bf16_kernel<64><<<(unsigned)blocks, 256, 0, s>>>(u(a.q), u(a.out), u(a.d_out), a.lse, w(a.qs),
                                                               w(a.dos), a.lse2s, a.deltas,
                                                               a.toks, a.T, a.Mpad, a.Hq, a.group);
  return (int)hipGetLastError();
}

}  // namespace pa
