// Backward, key-stationary pass (bf16 MFMA, gfx950): dK and dV.
//
// A workgroup owns 128 keys of one kv head (4 wavefronts x 32 keys; K and V columns stay in
// registers) and streams the stacked query rows that see those keys past them, 64 rows per
// tile.  For the shared video prefix these are the rows of ALL rollouts (paper Sec. 5.1: one
// cached prefix for every rollout), so the sum over rollouts happens in the accumulators and
// each prefix key is written exactly once, with no atomics.  For a rollout's own keys the rows
// are the rollout's later positions (causal).  Per 32-row block:
//   S  = Q K^T                   (A = Q rows from LDS,  B = K in registers)
//   dW = dO V^T                  (A = dO rows from LDS, B = V in registers)
//   W  = exp2(c S - LSE log2 e),  dS = W * (dW - delta)   (VALU; the dW accumulator starts from
//                                                          -delta, read from LDS in register order)
//   dV^T += dO^T W               (A = dO tile read TRANSPOSED from LDS, B = W packed to bf16)
//   dK^T += Q^T dS               (A = Q tile read transposed,           B = dS packed to bf16)
// Q and dO rows of a kv head, gathered into contiguous stacked order by the pre-pass, go
// global -> LDS with buffer loads (2 x 16 KiB + statistics per tile; directly for a rollout's own
// keys, through registers for prefix keys), double buffered, one barrier per tile.  The same two row-major tiles serve both kinds of product: read
// along the rows with 16-byte LDS reads for S and dW, and transposed with ds_read_b64_tr_b16 for
// dV and dK (two 8-byte transposed reads build one operand); the tile's XOR swizzle is chosen so
// that both access patterns are bank-conflict free (mfma_tiles.h).  One wavefront per SIMD (the
// accumulators, 128 registers, and the K/V columns, 64, need more than half of the register
// file), so MFMA and VALU work is arranged inside the wavefront: see the step stream in the
// kernel.  Built with the MFMA results in ordinary vector registers (-amdgpu-mfma-vgpr-form): the
// compiler then keeps the K/V columns in the accumulation registers, which the MFMA reads as B
// operands directly, and the softmax VALU code needs no register-file copies.
#include <hip/hip_runtime.h>

#include "bwd.h"
#include "mfma_tiles.h"

namespace pa {
namespace {

using namespace mt;

constexpr int KV_THREADS = KEY_WAVES * 64;
constexpr float LOG2E = 1.4426950408889634f;

// PARTIAL: the item leaves unscaled fp32 partial gradients in slot `it.split` of `partial`
// ([2][splits][P][Hkv][D], P = number of keys of the array k / v) and a reduction kernel adds the slots.  Used for
// the prefix keys of a short prefix (each item streams one range of row tiles) and for a rollout's own keys
// when their pass is split: the CAUSAL instantiation then streams only the tiles that need the mask (the
// block's diagonal, and the rollout's last tile if rows of the next rollout share it), the mask-free
// instantiation the tiles between, with the keys indexed over all packed tokens (P = T).
template <int D, bool CAUSAL, bool PARTIAL>
__global__ __launch_bounds__(KV_THREADS, 1) void bwd_dkv_kernel(
    const __bf16* __restrict__ k, const __bf16* __restrict__ v, const __bf16* __restrict__ qs,
    const __bf16* __restrict__ dos,
    const float* __restrict__ lse2s, const float* __restrict__ deltas, const int32_t* __restrict__ toks,
    __bf16* __restrict__ dk,
    __bf16* __restrict__ dv, float* __restrict__ partial, int64_t P, int splits,
    const KeyItem* __restrict__ items, const int32_t* __restrict__ cu, int64_t T, int64_t Mpad, int Hkv, int group,
    float scale) {
  using G = Geo<D>;
  constexpr int KK = G::KK, DB = G::DB;
  constexpr int STATS = 1024;  // per row: LSE*log2e, delta, packed token index (3 x 64 words)
  constexpr int STAGE = 2 * G::ROW_TILE_BYTES + STATS;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * STAGE];

  const KeyItem it = items[blockIdx.x];
  if (it.c < 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int off_g = CAUSAL ? cu[it.g] : 0;
  const int end_g = CAUSAL ? cu[it.g + 1] : 0;

  // ---- this lane's key column: K and V in registers (zeros past the end of the block)
  const int kloc = wave * 32 + l32;        // key inside the block
  const int key = it.key0 + kloc;          // prefix index, or position inside the rollout
  const bool key_ok = kloc < it.nkeys;
  const int64_t krow = (int64_t)(off_g + key) * Hkv + it.c;  // row of k / v / dk / dv
  bf16x8 Kb[KK], Vb[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    if (key_ok) {
      Kb[kk] = *reinterpret_cast<const bf16x8*>(k + krow * D + 16 * kk + 8 * hf);
      Vb[kk] = *reinterpret_cast<const bf16x8*>(v + krow * D + 16 * kk + 8 * hf);
    } else {
      Kb[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      Vb[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }
  const float c_log2 = scale * LOG2E;

  int roff[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) roff[kk] = row_operand_offset_tr<D>(l32, hf, kk);
  // transposed operands: byte offsets for chunk 0 of every (half, channel block); chunk ch adds 16 rows
  // (the swizzle term repeats every 16 rows)
  int troff[2][DB];
#pragma unroll
  for (int half = 0; half < 2; ++half)
#pragma unroll
    for (int db = 0; db < DB; ++db) troff[half][db] = tr_operand_offset<D>(lane, db, 0, half);

  // ---- row tiles: stacked rows M = t * group + j of kv head c, 64 per tile, numbered over all packed tokens
  // the plan names the row tiles: [tile0, tile1) and, for a masked item, possibly one more tile after them
  const int tile0 = it.tile0, tile1 = it.tile1;
  // A mask-free item of a rollout's own keys (g == -2) walks its tiles from the rollout's end backwards: all key
  // blocks of a rollout share that end, so the blocks running at the same time stream the same tiles and share
  // them in L2 (walking forwards from its own diagonal, every block would be somewhere else).
  const int extra = CAUSAL ? it.extra_tile : -1;
  const bool backwards = !CAUSAL && it.g == -2;
  const int ntile = tile1 - tile0 + (extra >= 0 ? 1 : 0);
  auto tile_at = [&](int n) { return backwards ? tile1 - 1 - n : (n < tile1 - tile0 ? tile0 + n : extra); };
  const int64_t head_rows = (int64_t)it.c * Mpad;
  const __bf16* qs_c = qs + head_rows * D;
  const __bf16* dos_c = dos + head_rows * D;
  const float* lse_c = lse2s + head_rows;
  const float* del_c = deltas + head_rows;

  const int* tok_c = toks + head_rows;
  // rows visible to this lane's key in the causal pass: packed tokens tkey .. end_g - 1
  const unsigned tkey = (unsigned)(off_g + key);
  const unsigned tspan = (unsigned)(end_g - (off_g + key));

  // The loads of a tile are issued in four pieces so they can be spread over the MFMA stream.
  RowTileOffsets<D, KEY_WAVES> lane_off;
  lane_off.init(D, wave, lane, true);
  const rsrc_t r_qs = make_rsrc(qs_c), r_dos = make_rsrc(dos_c);
  const rsrc_t r_lse = make_rsrc(lse_c), r_del = make_rsrc(del_c), r_tok = make_rsrc(tok_c);
  // Prefix key blocks: the Q and dO tiles travel global -> registers -> LDS instead of directly into the LDS.  A
  // wavefront that runs alone on its SIMD has the 32 registers to spare, and a plain 16-byte load plus a 16-byte
  // LDS write cost its instruction stream less than a direct-to-LDS load (-4.3 % on the pass; the causal
  // instantiation, with its mask registers, got 4 % slower and keeps the direct loads, as do the kernels that
  // run two wavefronts per SIMD: the log-probability GEMM lost 9 % with staged loads).
  constexpr bool STAGED = !CAUSAL;
  constexpr int NBLK = RowTileOffsets<D, KEY_WAVES>::BLOCKS_PER_WAVE;
  i32x4 stage_q[NBLK], stage_do[NBLK];
  auto stage_to_lds = [&](int buf) {
    unsigned char* dst = smem + buf * STAGE;
#pragma unroll
    for (int n = 0; n < NBLK; ++n) {
      *reinterpret_cast<i32x4*>(dst + (wave * NBLK + n) * 1024 + lane * 16) = stage_q[n];
      *reinterpret_cast<i32x4*>(dst + G::ROW_TILE_BYTES + (wave * NBLK + n) * 1024 + lane * 16) = stage_do[n];
    }
  };
  auto issue_piece = [&](int tile, int buf, int piece) {
    unsigned char* dst = smem + buf * STAGE;
    const unsigned b0 = (unsigned)tile * (TILE * D * 2);  // byte offset of the tile in each of the four arrays
    if (piece == 0) {
      if (wave == 0) {  // per-row statistics: 64 dwords each, lane l's word lands at word l
        unsigned char* st = dst + 2 * G::ROW_TILE_BYTES;
        const unsigned m4 = (unsigned)tile * (TILE * 4);
        load_dword_to_lds(r_lse, st, lane * 4, m4);
        load_dword_to_lds(r_del, st + TILE * 4, lane * 4, m4);
        if (CAUSAL) load_dword_to_lds(r_tok, st + 2 * TILE * 4, lane * 4, m4);
      }
      if (STAGED) {
#pragma unroll
        for (int n = 0; n < NBLK; ++n) stage_q[n] = load_chunk(r_qs, lane_off.off[n], b0);
      } else {
        issue_full_row_tile<D, KEY_WAVES>(dst, r_qs, b0, lane_off, wave);
      }
    } else if (piece == 1) {
      if (STAGED) {
#pragma unroll
        for (int n = 0; n < NBLK; ++n) stage_do[n] = load_chunk(r_dos, lane_off.off[n], b0);
      } else {
        issue_full_row_tile<D, KEY_WAVES>(dst + G::ROW_TILE_BYTES, r_dos, b0, lane_off, wave);
      }
    }
  };

  f32x16 dK[DB], dV[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      dK[db][i] = 0.f;
      dV[db][i] = 0.f;
    }

  // One tile = a stream of NS steps of two MFMAs each, operands read from LDS PF steps ahead:
  //   steps [0, 2KK):       S[rb] += Q_rb K^T,  dW[rb] += dO_rb V^T        (rb = step / KK)
  //   steps [2KK, 2KK+4DB): dV += dO^T W,  dK += Q^T dS, 16-row chunk by chunk (block, chunk, channel block)
  // The VALU work that turns (S, dW) of a 32-row block into the bf16 operands (W, dS) is cut into
  // four slices per block and interleaved with the MFMAs of later steps, so both pipes stay busy
  // although only one wavefront runs per SIMD.
  constexpr int NSW = 2 * KK, NDK = 4 * DB, NS = NSW + NDK, PF = 2;

  if (ntile > 0) {
#pragma unroll
    for (int piece = 0; piece < 2; ++piece) issue_piece(tile_at(0), 0, piece);
  }
  // The tile body exists once per LDS buffer, so that every LDS address in it is the lane's constant offset
  // plus an immediate (no address arithmetic in the step stream).
  auto tile_body = [&](int n, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's loads of the tile have landed (LDS or registers)
    if (STAGED) stage_to_lds(buf);        // staged tile -> LDS; buffer `buf` was last read two tiles ago
    __syncthreads();                      // all shares of the tile (and wavefront 0's statistics) are visible
    // the tile after the last one is the last one again: a harmless reload into the idle buffer,
    // which keeps the step stream free of branches
    const int next_tile = tile_at(n + 1 < ntile ? n + 1 : n);
    const unsigned char* qt = smem + buf * STAGE;
    const unsigned char* dt = qt + G::ROW_TILE_BYTES;
    const float* st = reinterpret_cast<const float*>(qt + 2 * G::ROW_TILE_BYTES);

    f32x16 S[2], W[2];
    bf16x8 Pb[2][2], dSb[2][2];
    f32x4 l4[2][4];           // LSE * log2(e) of a slice's four rows, loaded one slot before its use
    i32x4 p4[2][4];
    bf16x8 op0[NS], op1[NS];  // operand pair of each step (only PF+1 of them are live at a time)

    // steps [0, NSW): block rb = s % 2, contraction step kk = s / 2, i.e. four independent
    // accumulation chains (S and dW of both blocks): one wavefront alone cannot issue dependent
    // MFMAs back to back at full rate
    auto fetch = [&](int s) {
      if (s < NSW) {
        const int rb = s % 2, kk = s / 2;
        op0[s] = lds_operand(qt + rb * 32 * G::ROWB + roff[kk]);
        op1[s] = lds_operand(dt + rb * 32 * G::ROWB + roff[kk]);
      } else {
        const int u = s - NSW, blk = u / (2 * DB), c2 = (u / DB) % 2, db = u % DB;
        const int chunk_rows = (2 * blk + c2) * 16 * G::ROWB;
        op0[s] = lds_operand_tr(dt + chunk_rows + troff[0][db], dt + chunk_rows + troff[1][db]);   // dO^T: channels x rows
        op1[s] = lds_operand_tr(qt + chunk_rows + troff[0][db], qt + chunk_rows + troff[1][db]);   // Q^T
      }
    };
    auto load_stats = [&](int rb, int a) {
      const int r0 = rb * 32 + 8 * a + 4 * hf;
      l4[rb][a] = *reinterpret_cast<const f32x4*>(st + r0);
      if (CAUSAL) p4[rb][a] = *reinterpret_cast<const i32x4*>(st + 2 * TILE + r0);
    };
    // slice a of block rb: registers [4a, 4a+4) = rows rb*32 + 8a + 4hf + (0..3) of the tile, this
    // lane's key.  W already holds dW - delta (its accumulator started from -delta).
    auto slice = [&](int rb, int a) {
      float p[4], ds[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = 4 * a + e;
        p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[rb][i], c_log2, -l4[rb][a][e]));
        if (CAUSAL && (unsigned)p4[rb][a][e] - tkey >= tspan) p[e] = 0.f;
        ds[e] = p[e] * W[rb][i];
      }
      pack4(p, 4 * a, Pb[rb]);
      pack4(ds, 4 * a, dSb[rb]);
    };

    // dW accumulators start from -delta of their rows: register i is row rb*32 + 8*(i/4) + 4*hf + i%4,
    // so four 16-byte reads of the (negated) delta array fill a block's 16 registers
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const f32x4 nd = *reinterpret_cast<const f32x4*>(st + TILE + rb * 32 + 8 * a + 4 * hf);
#pragma unroll
        for (int e = 0; e < 4; ++e) W[rb][4 * a + e] = nd[e];
      }
#pragma unroll
    for (int s = 0; s < PF; ++s) fetch(s);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (s + PF < NS) fetch(s + PF);
      if (s < NSW) {
        const int rb = s % 2, kk = s / 2;
        if (kk == 0) {
          const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          S[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op0[s], Kb[kk], zero, 0, 0, 0);
        } else {
          S[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op0[s], Kb[kk], S[rb], 0, 0, 0);
        }
        W[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op1[s], Vb[kk], W[rb], 0, 0, 0);
      } else {
        const int u = s - NSW, blk = u / (2 * DB), c2 = (u / DB) % 2, db = u % DB;
        dV[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op0[s], Pb[blk][c2], dV[db], 0, 0, 0);
        dK[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op1[s], dSb[blk][c2], dK[db], 0, 0, 0);
      }
      // next tile's loads, one piece after each of the first odd steps
      if ((s & 1) && s < 4) issue_piece(next_tile, buf ^ 1, s >> 1);
      __builtin_amdgcn_sched_barrier(0);
      // softmax slices: block 0 once both blocks' S and dW are complete, block 1 during the first
      // dV/dK steps of block 0; a slice's LSE values are read one slot earlier
      if (s == NSW - 2) load_stats(0, 0);
      if (s == NSW - 1) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          if (a + 1 < 4) load_stats(0, a + 1); else load_stats(1, 0);
          slice(0, a);
        }
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
        if (s == NSW + a) {
          if (a + 1 < 4) load_stats(1, a + 1);
          slice(1, a);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  {
    int n = 0;
    for (; n + 1 < ntile; n += 2) {
      tile_body(n, std::integral_constant<int, 0>{});
      tile_body(n + 1, std::integral_constant<int, 1>{});
    }
    if (n < ntile) tile_body(n, std::integral_constant<int, 0>{});
  }

  // ---- epilogue: register i of block db is channel db*32 + 8*(i/4) + 4*hf + i%4 of this lane's key
  if (PARTIAL) {
    if (key_ok) {
      float* pk = partial + (((int64_t)it.split * P + off_g + key) * Hkv + it.c) * D + 4 * hf;
      float* pv = pk + (int64_t)splits * P * Hkv * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const f32x4 wk = {dK[db][4 * a], dK[db][4 * a + 1], dK[db][4 * a + 2], dK[db][4 * a + 3]};
          const f32x4 wv = {dV[db][4 * a], dV[db][4 * a + 1], dV[db][4 * a + 2], dV[db][4 * a + 3]};
          *reinterpret_cast<f32x4*>(pk + db * 32 + 8 * a) = wk;
          *reinterpret_cast<f32x4*>(pv + db * 32 + 8 * a) = wv;
        }
    }
  } else if (key_ok) {
    __bf16* kp = dk + krow * D + 4 * hf;
    __bf16* vp = dv + krow * D + 4 * hf;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const f32x4 wk = {dK[db][4 * a] * scale, dK[db][4 * a + 1] * scale, dK[db][4 * a + 2] * scale,
                          dK[db][4 * a + 3] * scale};
        const f32x4 wv = {dV[db][4 * a], dV[db][4 * a + 1], dV[db][4 * a + 2], dV[db][4 * a + 3]};
        *reinterpret_cast<bf16x4*>(kp + db * 32 + 8 * a) = __builtin_convertvector(wk, bf16x4);
        *reinterpret_cast<bf16x4*>(vp + db * 32 + 8 * a) = __builtin_convertvector(wv, bf16x4);
      }
  }
}

// Adds the row splits' fp32 partials of the prefix gradients and converts: 4 channels per thread.
__global__ __launch_bounds__(256) void bwd_dkv_reduce_kernel(const float* __restrict__ partial, __bf16* __restrict__ dk,
                                                             __bf16* __restrict__ dv, int64_t n4, int splits,
                                                             float scale) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) {
      sk += *reinterpret_cast<const f32x4*>(partial + ((int64_t)s * n4 + i) * 4);
      sv += *reinterpret_cast<const f32x4*>(partial + (((int64_t)splits + s) * n4 + i) * 4);
    }
    sk *= scale;
    *reinterpret_cast<bf16x4*>(dk + i * 4) = __builtin_convertvector(sk, bf16x4);
    *reinterpret_cast<bf16x4*>(dv + i * 4) = __builtin_convertvector(sv, bf16x4);
  }
}

}  // namespace

int launch_bwd_dkv_bf16(const BwdDkvArgs& a, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto b = [](const void* p) { return static_cast<const __bf16*>(p); };
  if (a.num_items > 0) {
    const unsigned grid = (unsigned)a.num_items;
#define PA_LAUNCH(DD, CC, PP)                                                                                      \
  bwd_dkv_kernel<DD, CC, PP><<<grid, KV_THREADS, 0, s>>>(                                                          \
      b(a.k), b(a.v), b(a.qs), b(a.dos), a.lse2s, a.deltas, a.toks, static_cast<__bf16*>(a.dk),                    \
      static_cast<__bf16*>(a.dv), a.partial, a.P, a.splits, a.items, a.cu, a.T, a.Mpad, a.Hkv, a.group, a.scale)
#define PA_LAUNCH_D(DD)                                                                                            \
  if (a.causal && a.partials) PA_LAUNCH(DD, true, true);                                                           \
  else if (a.causal) PA_LAUNCH(DD, true, false);                                                                   \
  else if (a.partials) PA_LAUNCH(DD, false, true);                                                                 \
  else PA_LAUNCH(DD, false, false)
    if (a.D == 128) {
      PA_LAUNCH_D(128);
    } else {
      PA_LAUNCH_D(64);
    }
#undef PA_LAUNCH_D
#undef PA_LAUNCH
    if (hipGetLastError() != hipSuccess) return 1;
  }
  if (a.partials && a.reduce) {
    const int64_t n4 = a.P * a.Hkv * a.D / 4;
    const int64_t want = (n4 + 255) / 256;
    bwd_dkv_reduce_kernel<<<(unsigned)(want < 8192 ? want : 8192), 256, 0, s>>>(
        a.partial, static_cast<__bf16*>(a.dk), static_cast<__bf16*>(a.dv), n4, a.splits, a.scale);
  }
  return (int)hipGetLastError();
}

}  // namespace pa
