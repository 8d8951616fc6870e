// Layout pre-pass of the bf16 path: rewrites V ([key][d], as a QKV projection emits it) into
// transposed tile images, one per (kv head, tile of 64 keys).  An image is exactly the byte
// layout the attention passes want in LDS, so they copy it global -> LDS linearly with
// direct-to-LDS loads and read MFMA A-operands of V^T with conflict-free 16-byte LDS reads.
//
// Image layout (D rows of 128 bytes; row d holds the 64 keys of the tile for channel d):
//   - forward passes (v_mfma_f32_16x16x32_bf16): inside every group of 32 keys, slot 8*g + e (g = 0..3,
//     e = 0..7) holds key 4*g + e (e < 4) or 16 + 4*g + (e - 4): keys 0-3, 16-19, 4-7, 20-23, 8-11, 24-27,
//     12-15, 28-31.  That is the order in which two 16 x 16 score accumulator blocks of S^T = K Q^T hand the
//     probabilities of one query to the four lanes that share it (lane group g contracts over slots
//     8*g .. 8*g + 7).
//   - the backward's dQ pass (v_mfma_f32_32x32x16_bf16, images of K): key k of the tile sits in slot
//     16*(k/16) + swap_bits_2_3(k%16), i.e. inside every group of 16 keys the order is 0-3, 8-11, 4-7, 12-15, the
//     order in which a 32 x 32 accumulator block hands its values to the two lane halves.
//   - the 16-byte chunk j = s/8 of row d is stored at chunk position j ^ ((d >> 1) & 7), which
//     spreads the rows a wavefront reads together over all LDS banks.
//   - keys past the end of the sequence are zero.
//
// The prefix images are shared by all rollouts: the video values are computed once per layer
// and reused (paper Sec. 5.1); the suffix images are per rollout.  Cost: one read and one
// write of V, about 1 % of the attention time.
#include <hip/hip_runtime.h>

#include "common.h"

namespace pa {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

template <int D, bool ORDER32>
__global__ __launch_bounds__(256) void vt_image_kernel(const unsigned short* __restrict__ v_prefix,
                                                       const unsigned short* __restrict__ v_suffix,
                                                       unsigned short* __restrict__ vt_prefix,
                                                       unsigned short* __restrict__ vt_suffix,
                                                       const int32_t* __restrict__ cu,
                                                       const int32_t* __restrict__ vt_off, int64_t P, int tiles_prefix,
                                                       int tiles_suffix, int G, int Hkv) {
  constexpr int LD = D + 2;  // padded row of the staging tile: odd dword stride
  __shared__ unsigned short t[KEYS_PER_TILE * LD];
  const int tiles_per_head = tiles_prefix + tiles_suffix;
  const int c = blockIdx.x / tiles_per_head;
  int tile = blockIdx.x - c * tiles_per_head;
  const unsigned short* src;
  unsigned short* dst;
  int64_t key0;   // first key row of the tile in src
  int nvalid;     // keys of the tile that exist
  if (tile < tiles_prefix) {
    src = v_prefix;
    key0 = (int64_t)tile * KEYS_PER_TILE;
    const int64_t left = P - key0;
    nvalid = left < KEYS_PER_TILE ? (int)left : KEYS_PER_TILE;
    dst = vt_prefix + ((int64_t)c * tiles_prefix + tile) * (D * KEYS_PER_TILE);
  } else {
    tile -= tiles_prefix;
    int g = 0;
    while (g + 1 < G && vt_off[g + 1] <= tile) ++g;  // rollout that owns this tile
    const int j = tile - vt_off[g];
    const int S_g = cu[g + 1] - cu[g];
    src = v_suffix;
    key0 = (int64_t)cu[g] + (int64_t)j * KEYS_PER_TILE;
    const int left = S_g - j * KEYS_PER_TILE;
    nvalid = left < KEYS_PER_TILE ? left : KEYS_PER_TILE;
    dst = vt_suffix + ((int64_t)c * tiles_suffix + tile) * (D * KEYS_PER_TILE);
  }
  // stage [key][d], zero rows for missing keys
  constexpr int CPR = D / 8;  // 16-byte chunks per source row
  for (int n = threadIdx.x; n < KEYS_PER_TILE * CPR; n += 256) {
    const int key = n / CPR, ch = n - key * CPR;
    u32x4 w = {0, 0, 0, 0};
    if (key < nvalid) w = *reinterpret_cast<const u32x4*>(src + ((key0 + key) * Hkv + c) * D + ch * 8);
    unsigned* row = reinterpret_cast<unsigned*>(t + key * LD + ch * 8);
    row[0] = w[0]; row[1] = w[1]; row[2] = w[2]; row[3] = w[3];
  }
  __syncthreads();
  // emit the image, 16 bytes per thread per step
  for (int n = threadIdx.x; n < D * 8; n += 256) {
    const int d = n >> 3, pos = n & 7;
    const int j = pos ^ ((d >> 1) & 7);  // logical chunk stored at this position
    u16x8 w;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int s = j * 8 + e;                    // slot
      int key;
      if (ORDER32) {
        const int lo = s & 15;
        key = (s & ~15) + ((lo & 3) | ((lo & 4) << 1) | ((lo & 8) >> 1));  // swap bits 2 and 3
      } else {
        const int g = (s >> 3) & 3;               // lane group inside the 32-key chunk
        key = (s & ~31) + (e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4));
      }
      w[e] = t[key * LD + d];
    }
    *reinterpret_cast<u16x8*>(dst + (int64_t)n * 8) = w;
  }
}

}  // namespace

int launch_vt_images(const VtArgs& a, void* stream) {
  const int64_t blocks = (int64_t)a.Hkv * (a.tiles_prefix + a.tiles_suffix);
  if (blocks == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto vp = static_cast<const unsigned short*>(a.v_prefix);
  auto vs = static_cast<const unsigned short*>(a.v_suffix);
  auto tp = static_cast<unsigned short*>(a.vt_prefix);
  auto ts = static_cast<unsigned short*>(a.vt_suffix);
#define PA_VT(DD, OO)                                                                                            \
  vt_image_kernel<DD, OO><<<(unsigned)blocks, 256, 0, s>>>(vp, vs, tp, ts, a.cu, a.vt_off, a.P, a.tiles_prefix, \
                                                            a.tiles_suffix, a.G, a.Hkv)
  if (a.D == 128) {
    if (a.order_32x32) PA_VT(128, true); else PA_VT(128, false);
  } else {
    if (a.order_32x32) PA_VT(64, true); else PA_VT(64, false);
  }
#undef PA_VT
  return (int)hipGetLastError();
}

}  // namespace pa
