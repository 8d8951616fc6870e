// Backward, query-stationary pass (bf16 MFMA, gfx950): dQ of every suffix token.
//
// A workgroup owns the same 256 stacked rows (8 wavefronts x 32 rows of one rollout and kv
// head) as in the forward passes and sweeps first the shared prefix keys (paper Sec. 5.1: one
// cached video prefix for all rollouts) and then the rollout's own keys up to the diagonal.
// Because the softmax statistics are saved (LSE) no online rescaling is needed, so prefix and
// suffix keys accumulate into one dQ and nothing has to be merged.  Per 32-key block:
//   S^T  = K Q^T                 (A = K tile rows from LDS,      B = Q in registers)
//   dW^T = V dO^T                (A = V tile rows from LDS,      B = dO in registers)
//   dS^T = W^T * (dW^T - delta),  W = exp2(c S - LSE log2 e)      (VALU, per lane = per query)
//   dQ^T += K^T dS^T             (A = transposed K image in LDS, B = dS^T packed to bf16)
// K, V tiles and the K^T image go global -> LDS with direct-to-LDS loads, double buffered, one
// barrier per 64-key tile.
#include <hip/hip_runtime.h>

#include "bwd.h"
#include "mfma_tiles.h"

namespace pa {
namespace {

using namespace mt;

constexpr int DQ_WAVES = ROWS_PER_ITEM / 32;
constexpr int DQ_THREADS = DQ_WAVES * 64;

// PARTIAL (calls with few rows): the item sweeps only the prefix keys [key0, key0 + pkeys) (split 0:
// also the own keys) and leaves an unscaled fp32 partial dQ in slot `split`; a reduction adds the slots.
template <int D, bool PARTIAL>
__global__ __launch_bounds__(DQ_THREADS, 512 / DQ_THREADS) void bwd_dq_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ d_out, const __bf16* __restrict__ k_prefix,
    const __bf16* __restrict__ v_prefix, const __bf16* __restrict__ k_suffix, const __bf16* __restrict__ v_suffix,
    const __bf16* __restrict__ kt_prefix, const __bf16* __restrict__ kt_suffix, const float* __restrict__ lse2s,
    const float* __restrict__ deltas, int64_t Mpad, __bf16* __restrict__ dq, float* __restrict__ dq_partial,
    int64_t part_rows, const WorkItem* __restrict__ items, const int32_t* __restrict__ cu,
    const int32_t* __restrict__ vt_off, int tiles_prefix, int tiles_suffix, int Hq, int Hkv, int group, float scale) {
  using G = Geo<D>;
  constexpr int KK = G::KK, DB = G::DB;
  constexpr int STAGE = 2 * G::ROW_TILE_BYTES + G::IMAGE_BYTES;  // K tile, V tile, K^T image
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * STAGE];

  const WorkItem it = items[blockIdx.x];
  if (it.g < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int off_g = cu[it.g];
  const int S_g = cu[it.g + 1] - off_g;
  const int nrows = S_g * group;
  const int nkeys = it.nkeys;  // causal extent of the item's last row (0: this split sweeps prefix keys only)
  const int P = it.pkeys;      // prefix keys this item sweeps, starting at it.key0 (a multiple of the tile)
  const int64_t row_stride = (int64_t)Hkv * D;

  // ---- this lane's query: Q and dO columns, LSE and delta
  bf16x8 Q[KK], dOb[KK];
  int pos;        // suffix position of the query (causal bound)
  int64_t orow;   // packed (token, head) row, -1 past the end
  float lse2 = 0.f, dl = 0.f;
  {
    const int m = it.row0 + wave * 32 + l32;
    if (m < nrows) {
      const int i = m / group, hh = m - i * group;
      pos = i;
      orow = (int64_t)(off_g + i) * Hq + it.c * group + hh;
      const __bf16* qp = q + orow * D + 8 * hf;
      const __bf16* dp = d_out + orow * D + 8 * hf;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        Q[kk] = *reinterpret_cast<const bf16x8*>(qp + 16 * kk);
        dOb[kk] = *reinterpret_cast<const bf16x8*>(dp + 16 * kk);
      }
      const int64_t srow = (int64_t)it.c * Mpad + (int64_t)off_g * group + m;  // stacked row over all packed tokens
      lse2 = lse2s[srow];
      dl = -deltas[srow];  // the array holds -delta
    } else {
      pos = -1;  // sees nothing: every weight is masked to zero
      orow = -1;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        Q[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        dOb[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
  }
  const float c_log2 = scale * 1.4426950408889634f;

  int koff[KK], ioff[4];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) koff[kk] = row_operand_offset<D>(l32, hf, kk);
#pragma unroll
  for (int ch = 0; ch < 4; ++ch) ioff[ch] = image_operand_offset(l32, hf, ch);

  // tiles 0 .. tp-1 cover the prefix, tp .. tp+ts-1 the rollout's own keys
  const int tp = (P + TILE - 1) / TILE;
  const int ts = (nkeys + TILE - 1) / TILE;
  const int first_pos = it.row0 / group;  // smallest causal bound among the item's rows
  const int ntiles = tp + ts;
  const __bf16* kpb = k_prefix + ((int64_t)it.key0 * Hkv + it.c) * D;
  const __bf16* vpb = v_prefix + ((int64_t)it.key0 * Hkv + it.c) * D;
  const __bf16* ksb = k_suffix + ((int64_t)off_g * Hkv + it.c) * D;
  const __bf16* vsb = v_suffix + ((int64_t)off_g * Hkv + it.c) * D;
  const __bf16* ktpb = kt_prefix + ((int64_t)it.c * tiles_prefix + it.key0 / TILE) * (D * TILE);
  const __bf16* ktsb = kt_suffix + ((int64_t)it.c * tiles_suffix + vt_off[it.g]) * (D * TILE);

  // The loads of a tile are issued in three pieces so they can be spread over the MFMA stream.
  RowTileOffsets<D, DQ_WAVES> lane_off;
  lane_off.init(row_stride, wave, lane);
  auto issue_piece = [&](int u, int buf, int piece) {
    unsigned char* dst = smem + buf * STAGE;
    const bool pre = u < tp;
    const int j = pre ? u : u - tp;                 // tile index inside its key set
    const int left = (pre ? P : nkeys) - j * TILE;  // keys of the tile that exist (>= 1)
    if (piece < 2) {
      const __bf16* first = (piece == 0 ? (pre ? kpb : ksb) : (pre ? vpb : vsb)) + (int64_t)j * TILE * row_stride;
      unsigned char* d2 = dst + piece * G::ROW_TILE_BYTES;
      if (left >= TILE)
        issue_full_row_tile<D, DQ_WAVES>(d2, first, lane_off, wave);
      else
        issue_row_tile<D, DQ_WAVES>(d2, first, row_stride, left, wave, lane);
    } else
      issue_linear<G::IMAGE_BYTES, DQ_WAVES>(dst + 2 * G::ROW_TILE_BYTES,
                                              (pre ? ktpb : ktsb) + (int64_t)j * (D * TILE), wave, lane);
  };

  f32x16 dQ[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dQ[db][i] = 0.f;

  // One 32-key block = a stream of KK + DB steps of two MFMAs each, operands read from LDS PF
  // steps ahead:  steps [0, KK): S += K Q^T, dW += V dO^T;  steps [KK, KK + DB): dQ += K^T dS,
  // two channel blocks per step.  The two wavefronts of a SIMD overlap each other's VALU part.
  constexpr int NB = KK + DB, PF = 2;

#pragma unroll
  for (int piece = 0; piece < 3; ++piece) issue_piece(0, 0, piece);
  // The tile body exists once per LDS buffer: LDS addresses are then lane constants plus immediates.
  auto tile_body = [&](int u, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's share of tile u has landed
    __syncthreads();                      // everyone's share has; buffer buf^1 is no longer read
    // the tile after the last one is the last one again: a harmless reload into the idle buffer
    const int next = u + 1 < ntiles ? u + 1 : u;
    const unsigned char* kt = smem + buf * STAGE;
    const unsigned char* vt = kt + G::ROW_TILE_BYTES;
    const unsigned char* im = kt + 2 * G::ROW_TILE_BYTES;
    const bool pre = u < tp;
    const int key_tile0 = (pre ? u : u - tp) * TILE;
    // last visible key index inside this tile's key set, for this lane's query
    const int limit = pre ? P - 1 : pos;
    // no masking where every key of the tile exists and is visible to every row of the item: a full prefix
    // tile, or a tile of own keys that ends at or before the item's first position (rows past the rollout's
    // end carry zero Q and dO, so their dS is zero either way)
    const bool no_mask = pre ? (key_tile0 + TILE <= P) : (key_tile0 + TILE - 1 <= first_pos);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 S, W;
      bf16x8 dSb[2];
      bf16x8 op0[NB], op1[NB];  // operand pair of each step (PF + 1 of them live at a time)
      auto fetch = [&](int s) {
        if (s < KK) {
          op0[s] = lds_operand(kt + kb * 32 * G::ROWB + koff[s]);
          op1[s] = lds_operand(vt + kb * 32 * G::ROWB + koff[s]);
        } else {
          const int v = s - KK, c2 = v / (DB / 2), db = 2 * (v % (DB / 2));
          op0[s] = lds_operand(im + db * 32 * 128 + ioff[2 * kb + c2]);
          op1[s] = lds_operand(im + (db + 1) * 32 * 128 + ioff[2 * kb + c2]);
        }
      };
#pragma unroll
      for (int s = 0; s < PF; ++s) fetch(s);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < NB; ++s) {
        if (s + PF < NB) fetch(s + PF);
        if (s == 0) {
          const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op0[s], Q[s], zero, 0, 0, 0);
          W = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op1[s], dOb[s], zero, 0, 0, 0);
        } else if (s < KK) {
          S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op0[s], Q[s], S, 0, 0, 0);
          W = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op1[s], dOb[s], W, 0, 0, 0);
        } else {
          const int v = s - KK, c2 = v / (DB / 2), db = 2 * (v % (DB / 2));
          dQ[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op0[s], dSb[c2], dQ[db], 0, 0, 0);
          dQ[db + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op1[s], dSb[c2], dQ[db + 1], 0, 0, 0);
        }
        // next tile's loads, one piece after each of the first odd steps of the first block
        if (kb == 0 && (s & 1) && s < 6) issue_piece(next, buf ^ 1, s >> 1);
        __builtin_amdgcn_sched_barrier(0);
        if (s == KK - 1) {
          // register i: key key_tile0 + kb*32 + 8*(i/4) + 4*hf + i%4
          if (no_mask) {
#pragma unroll
            for (int a = 0; a < 4; ++a) {
              float ds[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const int i = 4 * a + e;
                ds[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[i], c_log2, -lse2)) * (W[i] - dl);
              }
              pack4(ds, 4 * a, dSb);
            }
          } else {
#pragma unroll
            for (int a = 0; a < 4; ++a) {
              float ds[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const int i = 4 * a + e;
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(S[i], c_log2, -lse2));
                if (key_tile0 + kb * 32 + 8 * a + 4 * hf + e > limit) p = 0.f;
                ds[e] = p * (W[i] - dl);
              }
              pack4(ds, 4 * a, dSb);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  {
    int u = 0;
    for (; u + 1 < ntiles; u += 2) {
      tile_body(u, std::integral_constant<int, 0>{});
      tile_body(u + 1, std::integral_constant<int, 1>{});
    }
    if (u < ntiles) tile_body(u, std::integral_constant<int, 0>{});
  }

  // ---- epilogue: register i of block db is channel db*32 + 8*(i/4) + 4*hf + i%4 of this lane's query
  if (PARTIAL) {
    if (orow >= 0) {
      float* op = dq_partial + ((int64_t)it.split * part_rows + orow) * D + 4 * hf;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const f32x4 w = {dQ[db][4 * a], dQ[db][4 * a + 1], dQ[db][4 * a + 2], dQ[db][4 * a + 3]};
          *reinterpret_cast<f32x4*>(op + db * 32 + 8 * a) = w;
        }
    }
  } else if (orow >= 0) {
    __bf16* op = dq + orow * D + 4 * hf;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const f32x4 w = {dQ[db][4 * a] * scale, dQ[db][4 * a + 1] * scale, dQ[db][4 * a + 2] * scale,
                         dQ[db][4 * a + 3] * scale};
        *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * a) = __builtin_convertvector(w, bf16x4);
      }
  }
}

// dq = scale * (sum of the key splits' fp32 partials), 4 channels per thread, fixed order.
__global__ __launch_bounds__(256) void bwd_dq_reduce_kernel(const float* __restrict__ partial, __bf16* __restrict__ dq,
                                                            int64_t n4, int splits, float scale) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) acc += *reinterpret_cast<const f32x4*>(partial + ((int64_t)s * n4 + i) * 4);
    acc *= scale;
    *reinterpret_cast<bf16x4*>(dq + i * 4) = __builtin_convertvector(acc, bf16x4);
  }
}

}  // namespace

int launch_bwd_dq_bf16(const BwdDqArgs& a, void* stream) {
  if (a.num_items == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto b = [](const void* p) { return static_cast<const __bf16*>(p); };
  const unsigned grid = (unsigned)a.num_items;
  const bool part = a.key_splits > 1;
  const int64_t part_rows = a.T * a.Hq;
#define PA_LAUNCH(DD, PP)                                                                                          \
  bwd_dq_kernel<DD, PP><<<grid, DQ_THREADS, 0, s>>>(                                                               \
      b(a.q), b(a.d_out), b(a.k_prefix), b(a.v_prefix), b(a.k_suffix), b(a.v_suffix), b(a.kt_prefix), b(a.kt_suffix), \
      a.lse2s, a.deltas, a.Mpad, static_cast<__bf16*>(a.dq), a.dq_partial, part_rows, a.items, a.cu, a.vt_off,     \
      a.tiles_prefix, a.tiles_suffix, a.Hq, a.Hkv, a.group, a.scale)
  if (a.D == 128) {
    if (part) PA_LAUNCH(128, true); else PA_LAUNCH(128, false);
  } else {
    if (part) PA_LAUNCH(64, true); else PA_LAUNCH(64, false);
  }
#undef PA_LAUNCH
  if (hipGetLastError() != hipSuccess) return 1;
  if (part) {
    const int64_t n4 = part_rows * a.D / 4;
    const int64_t want = (n4 + 255) / 256;
    bwd_dq_reduce_kernel<<<(unsigned)(want < 8192 ? want : 8192), 256, 0, s>>>(
        a.dq_partial, static_cast<__bf16*>(a.dq), n4, a.key_splits, a.scale);
  }
  return (int)hipGetLastError();
}

}  // namespace pa
