// Stand-alone measurement program (not part of the library): what the MI355X sustains on its bf16 MFMA pipe under
// the board's power limit, and what LDS operand reads take away from it.  Every workgroup of 8 wavefronts (two
// per SIMD, one workgroup per CU) runs a loop of v_mfma_f32_32x32x16_bf16 on four accumulators; per group of four
// MFMAs (131,072 FLOP per wavefront), R of the A operands are re-read from LDS (16 bytes per lane, 1 KiB per read,
// distinct addresses per lane), as the main loop of a GEMM or attention kernel does.  Operands are random bf16 values of magnitude
// around one ("random": high toggle rate) or all 1.0 ("constant").  The same is measured with eight
// v_mfma_f32_16x16x32_bf16 (the same FLOP) per group.
//
//   hipcc --offload-arch=gfx950 -O3 power_probe.hip -o power_probe && ./power_probe
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                 \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      std::exit(1);                                                           \
    }                                                                         \
  } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int WORDS = 4096;  // 16-byte words of operand data (64 KiB)

// R LDS operand reads per four 32x32x16 MFMAs (R = 0 ... 4); SHAPE16: eight 16x16x32 MFMAs (the same FLOP) instead.
template <int R, bool SHAPE16>
__global__ __launch_bounds__(512) void probe_kernel(float* out, const u32x4* data, int iters) {
  __shared__ u32x4 lds[WORDS];
  const int l = threadIdx.x;
  for (int i = l; i < WORDS; i += 512) lds[i] = data[i];
  __syncthreads();
  bf16x8 a[8], b[8];
  for (int j = 0; j < 8; ++j) {
    a[j] = __builtin_bit_cast(bf16x8, data[(l * 16 + j) & (WORDS - 1)]);
    b[j] = __builtin_bit_cast(bf16x8, data[(l * 16 + 8 + j + blockIdx.x) & (WORDS - 1)]);
  }
  float s = 0.f;
  if (SHAPE16) {
    f32x4 c[8] = {{0}, {0}, {0}, {0}, {0}, {0}, {0}, {0}};
    const int idx = l & 63;
    for (int i = 0; i < iters; ++i) {  // 8 x 16,384 FLOP per lane group = the FLOP of four 32x32x16
      bf16x8 na[4];
#pragma unroll
      for (int r = 0; r < R; ++r) na[r] = __builtin_bit_cast(bf16x8, lds[(idx + 64 * r + 256 * (i & 15)) & (WORDS - 1)]);
#pragma unroll
      for (int j = 0; j < 8; ++j) c[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j], b[j], c[j], 0, 0, 0);
#pragma unroll
      for (int r = 0; r < R; ++r) a[2 * r] = na[r];
    }
    for (int k = 0; k < 8; ++k)
      for (int i = 0; i < 4; ++i) s += c[k][i];
  } else {
    f32x16 c[4] = {{0}, {0}, {0}, {0}};
    const int idx = l & 63;
    for (int i = 0; i < iters; ++i) {
      bf16x8 na[4];
#pragma unroll
      for (int r = 0; r < R; ++r) na[r] = __builtin_bit_cast(bf16x8, lds[(idx + 64 * r + 256 * (i & 15)) & (WORDS - 1)]);
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], c[j], 0, 0, 0);
#pragma unroll
      for (int r = 0; r < R; ++r) a[r] = na[r];
    }
    for (int k = 0; k < 4; ++k)
      for (int i = 0; i < 16; ++i) s += c[k][i];
  }
  out[blockIdx.x * 512 + l] = s;
}

template <int R, bool SHAPE16>
double run(float* out, const u32x4* data, int cus) {
  const int iters = 40000;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  probe_kernel<R, SHAPE16><<<cus, 512>>>(out, data, iters);  // untimed: brings the chip to its sustained state
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  probe_kernel<R, SHAPE16><<<cus, 512>>>(out, data, iters);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  float ms = 0.f;
  CK(hipEventElapsedTime(&ms, e0, e1));
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
  const double flop = (double)cus * 8 * iters * 4.0 * 32768;  // 8 wavefronts x 4 MFMAs (or their equivalent) x 32,768 FLOP
  return flop / ms * 1e-9;
}

int main() {
  int cus = 0;
  CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  std::vector<unsigned> rnd(WORDS * 4), one(WORDS * 4, 0x3f803f80u);
  std::srand(3);
  for (auto& x : rnd) {  // two bf16 per word: random sign and mantissa, exponent 120 ... 127 (|v| in [2^-7, 2))
    const unsigned lo = (std::rand() & 0x807f) | ((120 + std::rand() % 8) << 7);
    const unsigned hi = (std::rand() & 0x807f) | ((120 + std::rand() % 8) << 7);
    x = lo | (hi << 16);
  }
  u32x4 *d_rnd, *d_one;
  float* out;
  CK(hipMalloc(&d_rnd, rnd.size() * 4));
  CK(hipMalloc(&d_one, one.size() * 4));
  CK(hipMalloc(&out, (size_t)cus * 512 * 4));
  CK(hipMemcpy(d_rnd, rnd.data(), rnd.size() * 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_one, one.data(), one.size() * 4, hipMemcpyHostToDevice));
  std::printf("%d compute units, one workgroup of 8 wavefronts each, 40,000 x 4 MFMAs per wavefront and launch\n", cus);
  std::printf("TFLOP/s; three passes with random operands (the first also warms the chip up), then constant operands\n");
  for (int pass = 0; pass < 3; ++pass) {
    const double r0 = run<0, false>(out, d_rnd, cus), r2 = run<2, false>(out, d_rnd, cus);
    const double r3 = run<3, false>(out, d_rnd, cus), r4 = run<4, false>(out, d_rnd, cus);
    const double s0 = run<0, true>(out, d_rnd, cus), s2 = run<2, true>(out, d_rnd, cus), s4 = run<4, true>(out, d_rnd, cus);
    std::printf("pass %d: 32x32x16: no LDS reads %.0f | 2 reads per 131,072 FLOP %.0f | 3 reads %.0f | 4 reads %.0f || 16x16x32: none %.0f | 2 reads %.0f | 4 reads %.0f\n",
                pass, r0, r2, r3, r4, s0, s2, s4);
    std::fflush(stdout);
  }
  std::printf("constant operands: 32x32x16: no LDS reads %.0f | 4 reads per 131,072 FLOP %.0f || 16x16x32: none %.0f | 4 reads %.0f\n",
              run<0, false>(out, d_one, cus), run<4, false>(out, d_one, cus), run<0, true>(out, d_one, cus),
              run<4, true>(out, d_one, cus));
  CK(hipFree(d_rnd));
  CK(hipFree(d_one));
  CK(hipFree(out));
  return 0;
}
