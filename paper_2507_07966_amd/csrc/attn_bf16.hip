// bf16 MFMA attention pass for gfx950: the prefix pass (no mask, shared video K/V) and the
// causal suffix pass (a rollout's own prompt+response K/V) are two instantiations of one
// kernel.  Each produces, per stacked query row, a normalised fp32 partial output and the
// natural-log LSE over the keys it covers; the merge kernel combines the two.
//
// Why the prefix K/V can be shared at all: the video embeddings are gathered once per step
// and reused by every rollout (paper Sec. 5.1), so all G rollouts of a question attend to
// the same prefix keys/values; only the prompt+response part differs (Sec. 4.2, Sec. 5.2).
//
// Mapping onto the hardware
//   - A workgroup (4 wavefronts) owns ROWS_PER_ITEM = 256 stacked rows m = i * group + (h % group) of one
//     (kv head, rollout): all q heads of a GQA group and consecutive positions are stacked,
//     so every K/V tile staged in LDS is used by 256 rows.  Each wavefront owns 64 rows.
//   - Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: the
//     accumulator then holds, per lane, 16 keys of ONE query column, so the row maximum and
//     row sum are in-register plus one exchange between lane l and lane l+32, and the
//     probabilities are already laid out as the B operand of O^T += V^T P^T.
//   - V is staged row-major ([key][d]) and read with the LDS transpose load
//     (ds_read_b64_tr_b16), which hands each lane 4 consecutive keys of one channel d.
//   - Online softmax with a lazily updated reference maximum: the accumulators are rescaled
//     only when some row's maximum exceeds the reference by more than 2^8, which keeps every
//     probability below 2^8 (exact in fp32/bf16 range) and removes almost all rescaling work.
#include <hip/hip_runtime.h>

#include "common.h"

namespace pa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int BN = KEYS_PER_TILE;   // keys per LDS tile
constexpr int NTHREADS = 256;
constexpr float RESCALE_LOG2 = 8.0f;  // lazy-rescale threshold in log2 units

template <int D>
struct Lds {
  // Row strides in bytes.  K rows are read 16 B per lane by 32 different keys at the same
  // channel offset: stride = 16 (mod 256) spreads 16 keys over all 64 banks.  V rows are read
  // 8 B per lane by 4 keys x 64 contiguous bytes per half-wave: stride = 64 (mod 256).
  static constexpr int KSTRIDE = D * 2 + 16;
  static constexpr int VSTRIDE = D * 2 + 64;
  static constexpr int KBYTES = BN * KSTRIDE;
  static constexpr int VBYTES = BN * VSTRIDE;
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int TOTAL = 2 * STAGE;
};

// One K or V tile in flight from global memory to LDS: each thread carries PASSES x 16 bytes.
template <int D>
struct TileRegs {
  static constexpr int LANES_PER_ROW = D / 8;                // 16-byte pieces per row
  static constexpr int ROWS_PER_PASS = NTHREADS / LANES_PER_ROW;
  static constexpr int PASSES = BN / ROWS_PER_PASS;
  u32x4 k[PASSES], v[PASSES];
};

template <int D>
__device__ inline void load_tile(TileRegs<D>& t, const __bf16* __restrict__ kbase, const __bf16* __restrict__ vbase,
                                 int64_t row_stride, int key0, int nkeys, int tid) {
  constexpr int LPR = TileRegs<D>::LANES_PER_ROW;
  const int r0 = tid / LPR, col = (tid % LPR) * 8;
#pragma unroll
  for (int p = 0; p < TileRegs<D>::PASSES; ++p) {
    const int key = key0 + r0 + p * TileRegs<D>::ROWS_PER_PASS;
    if (key < nkeys) {
      t.k[p] = *reinterpret_cast<const u32x4*>(kbase + key * row_stride + col);
      t.v[p] = *reinterpret_cast<const u32x4*>(vbase + key * row_stride + col);
    } else {  // rows past the end are zero so that masked probabilities meet finite values
      t.k[p] = u32x4{0, 0, 0, 0};
      t.v[p] = u32x4{0, 0, 0, 0};
    }
  }
}

template <int D>
__device__ inline void store_tile(const TileRegs<D>& t, unsigned char* stage, int tid) {
  constexpr int LPR = TileRegs<D>::LANES_PER_ROW;
  const int r0 = tid / LPR, colb = (tid % LPR) * 16;
#pragma unroll
  for (int p = 0; p < TileRegs<D>::PASSES; ++p) {
    const int row = r0 + p * TileRegs<D>::ROWS_PER_PASS;
    *reinterpret_cast<u32x4*>(stage + row * Lds<D>::KSTRIDE + colb) = t.k[p];
    *reinterpret_cast<u32x4*>(stage + Lds<D>::KBYTES + row * Lds<D>::VSTRIDE + colb) = t.v[p];
  }
}

// Exchange between lane l and lane l^32 with v_permlane32_swap.  The two results are read
// through named unsigned temporaries: bit-casting the builtin's vector elements directly was
// observed to make the compiler use the first result twice.
__device__ inline void pair_exchange(float x, float& lo, float& hi) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const unsigned r0 = r[0], r1 = r[1];
  lo = __uint_as_float(r0);
  hi = __uint_as_float(r1);
}
__device__ inline float pair_max(float x) {
  float a, b;
  pair_exchange(x, a, b);
  return fmaxf(a, b);
}
__device__ inline float pair_sum(float x) {
  float a, b;
  pair_exchange(x, a, b);
  return a + b;
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(NTHREADS) void pass_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                                                             const __bf16* __restrict__ v, float* __restrict__ o_part,
                                                             float* __restrict__ lse_part,
                                                             const WorkItem* __restrict__ items,
                                                             const int32_t* __restrict__ cu, int Hq, int Hkv, int group,
                                                             float scale) {
  constexpr int KK = D / 16;  // contraction steps of QK^T
  constexpr int DB = D / 32;  // 32-channel blocks of the output
  __shared__ __attribute__((aligned(16))) unsigned char smem[Lds<D>::TOTAL];

  const WorkItem it = items[blockIdx.x];
  if (it.g < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int off_g = cu[it.g];
  const int S_g = cu[it.g + 1] - off_g;
  const int nrows = S_g * group;
  const int nkeys = it.nkeys;
  const int64_t row_stride = (int64_t)Hkv * D;
  const __bf16* kbase = k + ((int64_t)(CAUSAL ? off_g : 0) * Hkv + it.c) * D;
  const __bf16* vbase = v + ((int64_t)(CAUSAL ? off_g : 0) * Hkv + it.c) * D;

  // ---- this lane's two query columns (one per 32-row block of the wavefront)
  bf16x8 Q[2][KK];
  int pos[2];        // suffix position of the query (causal bound)
  int64_t orow[2];   // packed (token, head) row of the query, -1 when past the end
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int m = it.row0 + wave * 64 + qb * 32 + l32;
    if (m < nrows) {
      const int i = m / group, hh = m - i * group;
      pos[qb] = i;
      orow[qb] = (int64_t)(off_g + i) * Hq + it.c * group + hh;
      const __bf16* qp = q + orow[qb] * D + 8 * hf;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) Q[qb][kk] = *reinterpret_cast<const bf16x8*>(qp + 16 * kk);
    } else {
      pos[qb] = 0x7fffffff;
      orow[qb] = -1;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) Q[qb][kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }
  // first suffix position among the wavefront's rows: tiles reaching past it need the mask
  const int wave_first_pos = (it.row0 + wave * 64) / group;

  f32x16 O[DB][2];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) O[db][qb][i] = 0.f;
  float mref[2] = {-INFINITY, -INFINITY};  // reference maximum (raw dot-product units)
  float lsum[2] = {0.f, 0.f};              // this lane's share of the row sum
  const float c_log2 = scale * 1.4426950408889634f;
  const float rescale_raw = RESCALE_LOG2 / c_log2;

  const int ntiles = (nkeys + BN - 1) / BN;
  TileRegs<D> regs;
  load_tile<D>(regs, kbase, vbase, row_stride, 0, nkeys, tid);
  store_tile<D>(regs, smem, tid);
  __syncthreads();

  for (int tile = 0; tile < ntiles; ++tile) {
    unsigned char* stage = smem + (tile & 1) * Lds<D>::STAGE;
    const bool has_next = tile + 1 < ntiles;
    if (has_next) load_tile<D>(regs, kbase, vbase, row_stride, (tile + 1) * BN, nkeys, tid);

    // ---- S^T = K Q^T : [64 keys][64 queries] as 2x2 blocks of 32x32
    f32x16 S[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) S[kb][qb][i] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const unsigned char* krow = stage + (kb * 32 + l32) * Lds<D>::KSTRIDE + hf * 16;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(krow + kk * 32);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) S[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Q[qb][kk], S[kb][qb], 0, 0, 0);
      }
    }

    // ---- mask: register i of block kb holds key tile*64 + kb*32 + 8*(i/4) + 4*hf + i%4
    const int key_tile0 = tile * BN;
    const bool need_mask = CAUSAL ? (key_tile0 + BN - 1 > wave_first_pos) : (key_tile0 + BN > nkeys);
    if (need_mask) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int limit = CAUSAL ? pos[qb] : nkeys - 1;  // last visible key
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = key_tile0 + kb * 32 + 8 * (i / 4) + 4 * hf + (i % 4);
            if (key > limit) S[kb][qb][i] = -INFINITY;
          }
      }
    }

    // ---- online softmax with lazy reference maximum
    float mx[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float t = S[0][qb][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) t = fmaxf(t, S[0][qb][i]);
#pragma unroll
      for (int i = 0; i < 16; ++i) t = fmaxf(t, S[1][qb][i]);
      mx[qb] = pair_max(t);
    }
    const bool grow = (mx[0] - mref[0] > rescale_raw) || (mx[1] - mref[1] > rescale_raw);
    if (__any(grow)) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const float mnew = fmaxf(mref[qb], mx[qb]);
        const float alpha = __builtin_amdgcn_exp2f((mref[qb] - mnew) * c_log2);  // first tile: exp2(-inf) = 0
        lsum[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) O[db][qb][i] *= alpha;
        mref[qb] = mnew;
      }
    }
    bf16x8 Pb[2][4];  // [qb][16-key chunk]: B operand of the PV product
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float mc = mref[qb] * c_log2;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        float pr[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          pr[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][qb][i], c_log2, -mc));
          lsum[qb] += pr[i];
        }
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          bf16x8 b;
#pragma unroll
          for (int e = 0; e < 8; ++e) b[e] = (__bf16)pr[8 * h2 + e];
          Pb[qb][kb * 2 + h2] = b;
        }
      }
    }

    // ---- O^T += V^T P^T.  Chunk ch covers keys 16*ch .. 16*ch+15 of the tile; slot e of lane
    //      half hf is key 16*ch + 4*hf + e (e < 4) or 16*ch + 8 + 4*hf + (e - 4), the order in
    //      which the score accumulator delivered the probabilities.
    const unsigned char* vst = stage + Lds<D>::KBYTES;
    const int vkey = 4 * hf + ((lane & 15) >> 2);
    const int vcol = (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const unsigned char* p0 = vst + (16 * ch + vkey) * Lds<D>::VSTRIDE + db * 64 + vcol;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))p0);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p0 + 8 * Lds<D>::VSTRIDE));
        const s16x8 a16 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 a = __builtin_bit_cast(bf16x8, a16);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Pb[qb][ch], O[db][qb], 0, 0, 0);
      }
    }

    if (has_next) store_tile<D>(regs, smem + ((tile + 1) & 1) * Lds<D>::STAGE, tid);
    __syncthreads();
  }

  // ---- epilogue: normalise and write the partial.  Register i of block db is channel
  //      db*32 + 8*(i/4) + 4*hf + i%4 of this lane's query.
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l = pair_sum(lsum[qb]);
    if (orow[qb] < 0) continue;
    const float inv = 1.0f / l;
    float* op = o_part + orow[qb] * D + 4 * hf;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        f32x4 w = {O[db][qb][4 * a] * inv, O[db][qb][4 * a + 1] * inv, O[db][qb][4 * a + 2] * inv, O[db][qb][4 * a + 3] * inv};
        *reinterpret_cast<f32x4*>(op + db * 32 + 8 * a) = w;
      }
    if (hf == 0) lse_part[orow[qb]] = mref[qb] * scale + __logf(l);
  }
}

}  // namespace

int launch_pass_bf16(const PassArgs& a, void* stream) {
  if (a.num_items == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const __bf16* q = static_cast<const __bf16*>(a.q);
  const __bf16* k = static_cast<const __bf16*>(a.k);
  const __bf16* v = static_cast<const __bf16*>(a.v);
  const unsigned grid = (unsigned)a.num_items;
#define PA_LAUNCH(DD, CC) \
  pass_bf16_kernel<DD, CC><<<grid, NTHREADS, 0, s>>>(q, k, v, a.o_part, a.lse_part, a.items, a.cu, a.Hq, a.Hkv, a.group, a.scale)
  if (a.D == 128) {
    if (a.causal) PA_LAUNCH(128, true); else PA_LAUNCH(128, false);
  } else {
    if (a.causal) PA_LAUNCH(64, true); else PA_LAUNCH(64, false);
  }
#undef PA_LAUNCH
  return (int)hipGetLastError();
}

}  // namespace pa
