// bf16 MFMA attention pass for gfx950: the prefix pass (no mask, shared video K/V) and the
// causal suffix pass (a rollout's own prompt+response K/V) are two instantiations of one
// kernel.  Each produces, per stacked query row, a normalised fp32 partial output and the
// natural-log LSE over the keys it covers.  The two partials are combined by log-sum-exp either
// by the merge kernel or, for whole calls, in the suffix pass's own epilogue (it reads the prefix
// partial of its rows and writes the final output).  A third mode of the suffix pass sweeps the
// prefix keys and then the own keys in one online softmax (prefixes up to 65,536 keys: one launch, no
// partials); the part of that sweep that lies inside the prefix runs the prefix pass's instruction stream.
//
// Why the prefix K/V can be shared at all: the video embeddings are gathered once per step
// and reused by every rollout (paper Sec. 5.1), so all G rollouts of a question attend to
// the same prefix keys/values; only the prompt+response part differs (Sec. 4.2, Sec. 5.2).
//
// Mapping onto the hardware
//   - A workgroup (8 wavefronts) owns ROWS_PER_ITEM = 256 stacked rows
//     m = i * group + (h % group) of one (kv head, rollout): the q heads of a GQA group and
//     consecutive positions are stacked, so every K/V tile staged in LDS serves 256 rows.
//     Each wavefront owns 32 rows (two blocks of 16 query columns); two wavefronts share a SIMD (<= 256
//     registers each), so one wavefront's softmax VALU work also overlaps the other's MFMA work.
//   - K tiles and the pre-transposed V tile images go global -> LDS with direct-to-LDS
//     16-byte loads (no staging registers), double buffered, one barrier per tile.  Whole tiles
//     use buffer addressing (tile offset in a scalar register + a constant per-lane offset), so
//     the loads need no per-lane address arithmetic.  The LDS layouts are XOR-swizzled so every
//     16-byte operand read is bank-conflict free.
//   - Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16 (two 16-query blocks per
//     wavefront share every K operand read): the accumulator then holds, per lane, 4 keys of ONE query column,
//     four lanes (l, l+16, l+32, l+48) share a column, and the probabilities are already laid out as the
//     B operand of O^T += V^T P^T.  The 16 x 16 x 32 shape does the same work with half the accumulator
//     traffic of 32 x 32 x 16; under the board's power limit that is worth 10 % of MFMA rate on data that
//     toggles (power_probe.hip), which the kernel takes as a higher clock.
//   - Software pipeline inside a wavefront: the MFMAs that compute the scores of tile t+1 are
//     interleaved with the VALU softmax of tile t, so both pipes work at once.
//   - Online softmax with a lazily updated reference maximum: the reference of a query column is the maximum of
//     its first tile, and a later tile's probabilities are taken against it with no maximum search as long as
//     they stay in a safe range, which is detected from the tile's row sum.  The row sum is accumulated in fp32
//     from the unrounded probabilities, which keeps the LSE error at fp32 level even for rows that see only a few
//     keys.
//   - Two kernels per pass.  The COMMON kernel has no code for a moving reference: a wavefront that finds a tile
//     outside the safe range only records that in a word of its own (flags) and writes nothing.  The CAREFUL
//     kernel, launched right after it over the same work list, leaves at once unless a wavefront of its item
//     said so, and otherwise redoes the item with the full online softmax (new maximum, rescaled accumulators,
//     recomputed probabilities).  With N(0,1)-like scores no item needs it: a score would have to exceed its
//     column's first-tile maximum by 16 / (scale log2 e), 125 at D = 128.  Splitting the two is what keeps the
//     common kernel inside 256 registers without spills (the rescue code joins renamed copies of all 64
//     accumulators into the main loop); an empty second launch costs a few microseconds.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "common.h"
#include "mfma_tiles.h"

namespace pa {
namespace {

using namespace mt;  // vector types, swizzle_term

#define LDS_PTR(T) PA_LDS_PTR(T)
#define GLB_PTR(T) PA_GLB_PTR(T)

constexpr int BN = KEYS_PER_TILE;  // keys per LDS tile
constexpr int NQ = 2;                       // 16-query MFMA blocks per wavefront
constexpr int ROWS_PER_WAVE = 16 * NQ;
constexpr int NWAVES = WAVES_PER_ITEM;      // two wavefronts per SIMD, at most 256 registers each
constexpr int NTHREADS = NWAVES * 64;
static_assert(NWAVES * ROWS_PER_WAVE == ROWS_PER_ITEM, "the wavefronts of a workgroup cover the item's rows");
// A tile's probabilities are accepted without a maximum search while each lane's partial row
// sum of the tile stays below SAFE_SUM; every probability is then below 2^16, far inside the
// fp32/bf16 range, and the running sums cannot overflow (2^16 * 2^30 keys < 2^127).
constexpr float SAFE_SUM = 65536.0f;
// LDS operand reads run this many operands (two MFMAs each) ahead of the MFMAs that use them (6 is no faster)
constexpr int RING = 4;

// LDS buffers: K tile [64 keys][D] (rows of D*2 bytes) and V^T image [D][64 slots] (rows of
// 128 bytes), two of each.  16-byte chunk j of a row r is stored at chunk position
//   j ^ (r & 15)          for 256-byte rows,
//   j ^ ((r >> 1) & 7)    for 128-byte rows,
// so that 16 consecutive rows read at the same logical chunk cover all 64 banks.
template <int D>
struct Tile {
  static constexpr int ROWB = D * 2;
  static constexpr int KBYTES = BN * ROWB;
  static constexpr int VBYTES = D * 128;
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int KBLOCKS_PER_WAVE = KBYTES / 1024 / NWAVES;  // 1 KiB per wavefront-wide load
  static constexpr int VBLOCKS_PER_WAVE = VBYTES / 1024 / NWAVES;
  static_assert(KBLOCKS_PER_WAVE >= 1 && VBLOCKS_PER_WAVE >= 1, "every wavefront copies at least one block");
};

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
// The four lanes l, l^16, l^32, l^48 hold the same query column: reductions over them (seldom used: first tile,
// a moving reference maximum, the end of an item).
__device__ inline float quad_max(float x) { return pair_max(fmaxf(x, __shfl_xor(x, 16))); }
__device__ inline float quad_sum(float x) { return pair_sum(x + __shfl_xor(x, 16)); }

// EPI (suffix pass only): 0 = leave an fp32 partial; 1 = the partial is the result (no prefix): write it
// in bf16 with its LSE; 2 = combine with the prefix partial (o1, lse1) by log-sum-exp and write the result.
// SWEEP (suffix pass with EPI 0 or 1): the item first sweeps the prefix keys [0, it.pkeys) (no mask) and then
// the rollout's own keys, all in one online softmax, so its result is the result of the call (EPI 1) or the
// fp32 partial over a prefix shard and the own keys together (EPI 0).
template <int D, bool CAUSAL, int EPI, bool SWEEP, bool CAREFUL>
__global__ __launch_bounds__(NTHREADS, 512 / NTHREADS) void pass_bf16_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ vt,
    float* __restrict__ o_part, float* __restrict__ lse_part, const float* __restrict__ o1,
    const float* __restrict__ lse1, __bf16* __restrict__ out_final, float* __restrict__ lse_final,
    const WorkItem* __restrict__ items,
    const int32_t* __restrict__ cu, const int32_t* __restrict__ vt_off, int64_t vt_tiles_per_head,
    const __bf16* __restrict__ k_pre, const __bf16* __restrict__ vt_pre, int64_t vt_pre_tiles_per_head,
    int64_t part_rows, int Hq, int Hkv, int group, float scale, int32_t* __restrict__ flags) {
  static_assert(EPI == 0 || CAUSAL, "only the suffix pass can finish the call");
  static_assert(!SWEEP || (CAUSAL && EPI != 2), "a sweep over prefix and own keys has nothing to combine with");
  using TL = Tile<D>;
  constexpr int KK = D / 16;  // 16-channel halves of the contraction steps (granularity of the load placement)
  constexpr int KS = D / 32;  // contraction steps of QK^T (32 channels per MFMA)
  constexpr int CB = D / 16;  // 16-channel blocks of the output
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * TL::STAGE];

  const WorkItem it = items[blockIdx.x];
  if (it.g < 0) return;
  int32_t* const item_flags = flags + (int64_t)blockIdx.x * NWAVES;
  if (CAREFUL) {  // only the items on which a wavefront of the common kernel gave up
    int any = 0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) any |= item_flags[w];
    if (any == 0) return;
  }
  bool bad = false;  // common kernel: a tile's probabilities left the safe range (the whole wavefront agrees)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;
  const int off_g = cu[it.g];
  const int S_g = cu[it.g + 1] - off_g;
  const int nrows = S_g * group;
  const int nkeys = it.nkeys;
  const int64_t row_stride = (int64_t)Hkv * D;
  // prefix pass: the item sweeps prefix keys [key0, key0 + nkeys), key0 a multiple of the tile
  const __bf16* kown = k + ((int64_t)(CAUSAL ? off_g : it.key0) * Hkv + it.c) * D;
  const __bf16* vtbase = vt + ((int64_t)it.c * vt_tiles_per_head + (CAUSAL ? vt_off[it.g] : it.key0 / BN)) * (D * BN);

  // ---- this lane's two query columns: query block nq (16 rows) of the wavefront's 32 rows, column l16; the
  //      lane holds channels 32*ks + 8*g4 .. +7 of each contraction step ks
  bf16x8 Q[NQ][KS];
  int pos[NQ];  // suffix position of the query (causal bound); rows past the rollout's end see everything of Q = 0
  // packed (token, head) row of query column nq, -1 when past the end (recomputed where needed: two 64-bit values
  // less to carry through the main loop)
  auto out_row = [&](int nq) -> int64_t {
    const int m = it.row0 + wave * ROWS_PER_WAVE + nq * 16 + l16;
    if (m >= nrows) return -1;
    const int i = m / group, hh = m - i * group;
    return (int64_t)(off_g + i) * Hq + it.c * group + hh;
  };
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int64_t row = out_row(nq);
    if (row >= 0) {
      pos[nq] = (it.row0 + wave * ROWS_PER_WAVE + nq * 16 + l16) / group;
      const __bf16* qp = q + row * D + 8 * g4;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) Q[nq][ks] = *reinterpret_cast<const bf16x8*>(qp + 32 * ks);
    } else {
      pos[nq] = 0x7fffffff;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) Q[nq][ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }
  // first suffix position among the wavefront's rows: tiles reaching past it need the mask
  const int wave_first_pos = (it.row0 + wave * ROWS_PER_WAVE) / group;

  // ---- LDS: two K buffers then two V^T buffers.  Per-lane byte offsets of the operand reads
  //      inside a buffer (the buffer base is an immediate).
  constexpr int KBUF0 = 0, VBUF0 = 2 * TL::KBYTES;
  int koff[KS];  // K operand (key = kb*16 + l16, channels 32ks + 8g4 ..): chunk 4ks + g4
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    koff[ks] = l16 * TL::ROWB + (((4 * ks + g4) ^ swizzle_term(l16, TL::ROWB)) << 4);
  int voff[2];   // V^T operand (channel = cb*16 + l16, 32-key chunk c32, this lane's 8 keys of it): chunk 4c32 + g4
#pragma unroll
  for (int c32 = 0; c32 < 2; ++c32) voff[c32] = l16 * 128 + (((4 * c32 + g4) ^ swizzle_term(l16, 128)) << 4);

  // ---- per-lane source of the direct-to-LDS K loads: lane writes LDS chunk `lane` of its block.
  //      Address = uniform tile base (scalar registers) + a per-lane 32-bit byte offset.
  constexpr int LANES_PER_ROW = TL::ROWB / 16, ROWS_PER_BLOCK = 1024 / TL::ROWB;
  unsigned koffs[TL::KBLOCKS_PER_WAVE];  // byte offset of this lane's 16 bytes inside a K tile in global memory
#pragma unroll
  for (int n = 0; n < TL::KBLOCKS_PER_WAVE; ++n) {
    const int row = (wave * TL::KBLOCKS_PER_WAVE + n) * ROWS_PER_BLOCK + lane / LANES_PER_ROW;
    const int col = ((lane % LANES_PER_ROW) ^ swizzle_term(row, TL::ROWB)) * 8;  // logical chunk -> element offset
    koffs[n] = (unsigned)((row * row_stride + col) * 2);
  }
  const int64_t ktile_bytes = (int64_t)BN * row_stride * 2;  // bytes per tile of K in global memory
  // SWEEP: tiles [0, tp) are prefix tiles, tiles [tp, ntiles) the rollout's own
  const int P = SWEEP ? it.pkeys : 0;
  const int tp = SWEEP ? (P + BN - 1) / BN : 0;
  const int ntiles = tp + (nkeys + BN - 1) / BN;
  const __bf16* kpre = SWEEP ? k_pre + (int64_t)it.c * D : nullptr;
  const __bf16* vtpre = SWEEP ? vt_pre + (int64_t)it.c * vt_pre_tiles_per_head * (D * BN) : nullptr;
  // Whole tiles are fetched with buffer loads: uniform tile offset in a scalar register plus the lane's
  // constant 32-bit offset.  Every such access lies inside the arrays (a ragged last K tile takes the
  // clamped path below), so the descriptors' range (2 GiB) never comes into play.
  const rsrc_t krs_own = make_rsrc(kown), vrs_own = make_rsrc(vtbase);
  const rsrc_t krs_pre = make_rsrc(SWEEP ? kpre : kown), vrs_pre = make_rsrc(SWEEP ? vtpre : vtbase);

  // LEAN (a compile-time flag of the sweep's prefix loop): the tile is a whole prefix tile, so neither the
  // choice between the two key sets nor the ragged-tile path is in the instruction stream.
  auto issue_k = [&](int gtile, auto buf_c, auto lean_c) {  // K tile -> K buffer buf
    unsigned char* dst = smem + KBUF0 + decltype(buf_c)::value * TL::KBYTES;
    constexpr bool LEAN = decltype(lean_c)::value;
    const bool pre = LEAN || (SWEEP && gtile < tp);
    const int tile = pre ? gtile : gtile - tp;       // tile index inside its key set
    const int set_keys = pre ? P : nkeys;            // keys of that set
    const __bf16* kbase = pre ? kpre : kown;
    if (LEAN || tile < set_keys / BN) {              // all 64 keys exist
      const unsigned soff = (unsigned)(tile * ktile_bytes);
#pragma unroll
      for (int n = 0; n < TL::KBLOCKS_PER_WAVE; ++n) {
        unsigned char* d = dst + (wave * TL::KBLOCKS_PER_WAVE + n) * 1024;
        if (pre) load_chunk_to_lds(krs_pre, d, koffs[n], soff); else load_chunk_to_lds(krs_own, d, koffs[n], soff);
      }
    } else {  // last, partial tile: rows past the end repeat the last key; their scores are masked
#pragma unroll
      for (int n = 0; n < TL::KBLOCKS_PER_WAVE; ++n) {
        const int row = (wave * TL::KBLOCKS_PER_WAVE + n) * ROWS_PER_BLOCK + lane / LANES_PER_ROW;
        const int col = ((lane % LANES_PER_ROW) ^ swizzle_term(row, TL::ROWB)) * 8;
        int key = tile * BN + row;
        key = key < set_keys ? key : set_keys - 1;
        __builtin_amdgcn_global_load_lds((GLB_PTR(const void))(kbase + key * row_stride + col),
                                         (LDS_PTR(void))(dst + (wave * TL::KBLOCKS_PER_WAVE + n) * 1024), 16, 0, 0);
      }
    }
  };
  const unsigned voffs = (unsigned)(((wave * TL::VBLOCKS_PER_WAVE) * 512 + lane * 8) * 2);
  auto issue_v = [&](int gtile, auto buf_c, auto lean_c) {  // V^T image -> V buffer buf (a linear copy)
    unsigned char* dst = smem + VBUF0 + decltype(buf_c)::value * TL::VBYTES;
    const bool pre = decltype(lean_c)::value || (SWEEP && gtile < tp);
    const unsigned soff = (unsigned)((pre ? gtile : gtile - tp) * (D * BN * 2));
#pragma unroll
    for (int n = 0; n < TL::VBLOCKS_PER_WAVE; ++n) {
      unsigned char* d = dst + (wave * TL::VBLOCKS_PER_WAVE + n) * 1024;
      if (pre) load_chunk_to_lds(vrs_pre, d, voffs + n * 1024, soff); else load_chunk_to_lds(vrs_own, d, voffs + n * 1024, soff);
    }
  };

  f32x4 O[CB][NQ];  // O^T: channel block cb (16 channels), query block nq; register i is channel 16cb + 4g4 + i
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) O[cb][nq] = f32x4{0.f, 0.f, 0.f, 0.f};
  float mref[NQ];  // reference maximum of each query column (raw dot-product units)
  float lsum[NQ];  // this lane's share of each row sum
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) lsum[nq] = 0.f;
  const float c_log2 = scale * 1.4426950408889634f;

  auto zero = [](f32x4 (&S)[4][NQ]) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) S[kb][nq] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  auto k_operand = [&](const unsigned char* kbuf, int kb, int ks) {
    return *reinterpret_cast<const bf16x8*>(kbuf + kb * 16 * TL::ROWB + koff[ks]);
  };
  // register i of block (kb, nq) holds key tile*64 + kb*16 + 4*g4 + i of query column nq
  auto mask_scores = [&](f32x4 (&S)[4][NQ], int gtile) {
    const bool pre = SWEEP && gtile < tp;
    const bool causal = CAUSAL && !pre;
    const int key_tile0 = (pre ? gtile : gtile - tp) * BN;
    const int set_keys = pre ? P : nkeys;
    const bool need_mask = causal ? (key_tile0 + BN - 1 > wave_first_pos) : (key_tile0 + BN > set_keys);
    if (need_mask) {
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        const int limit = causal ? pos[nq] : set_keys - 1;  // last visible key
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int key = key_tile0 + kb * 16 + 4 * g4 + i;
            if (key > limit) S[kb][nq][i] = -INFINITY;
          }
      }
    }
  };
  auto row_max = [&](const f32x4 (&S)[4][NQ], int nq) {
    float t = fmaxf(fmaxf(S[0][nq][0], S[0][nq][1]), fmaxf(S[0][nq][2], S[0][nq][3]));
#pragma unroll
    for (int kb = 1; kb < 4; ++kb)
      t = fmaxf(t, fmaxf(fmaxf(S[kb][nq][0], S[kb][nq][1]), fmaxf(S[kb][nq][2], S[kb][nq][3])));
    return quad_max(t);
  };
  // probabilities of score block j = NQ*kb + nq (4 of the scores this lane holds): p = exp2(c*s - c*mref).
  // They land in the B operand of the PV product: 32-key chunk kb/2, slots 4*(kb%2) .. +3 (the V^T image stores
  // its keys in the same order).
  auto prob_slice = [&](const f32x4 (&S)[4][NQ], int j, const float (&mc)[NQ], bf16x8 (&Pb)[2][NQ], float (&lacc)[NQ]) {
    const int kb = j / NQ, nq = j % NQ;
#pragma unroll
    for (int e = 0; e < 4; e += 2) {
      const f32x2 pr = {__builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][nq][e], c_log2, -mc[nq])),
                        __builtin_amdgcn_exp2f(__builtin_fmaf(S[kb][nq][e + 1], c_log2, -mc[nq]))};
      const bf16x2 pk = __builtin_convertvector(pr, bf16x2);
      lacc[nq] += pr[0] + pr[1];
      Pb[kb >> 1][nq][(kb & 1) * 4 + e] = pk[0];
      Pb[kb >> 1][nq][(kb & 1) * 4 + e + 1] = pk[1];
    }
  };

  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;

  f32x4 S[4][NQ];     // scores of the tile being soft-maxed: [16-key block][query block]
  bf16x8 Pb[2][NQ];   // probabilities of the previous tile, [32-key chunk][query block]: B operand of the PV product
  // S^T = K Q^T with v_mfma_f32_16x16x32_bf16, operand reads four operands ahead of the MFMAs; every K
  // operand feeds the MFMAs of both query blocks.  mid(kk) runs after each half of a contraction step (kk counts
  // 16 channels): the steady state uses it to issue the next tile's loads inside the MFMA stream instead of as
  // one burst.
  auto scores = [&](const unsigned char* kbuf, auto&& mid) {
    zero(S);
    constexpr int NOP = 4 * KS;  // K operands of the tile: [contraction step][16-key block]
    bf16x8 ka[RING];             // refilled RING operands ahead, right after the MFMAs that read it
#pragma unroll
    for (int t = 0; t < RING; ++t) ka[t] = k_operand(kbuf, t % 4, t / 4);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);  // see pv()
#pragma unroll
    for (int t = 0; t < NOP; ++t) {
      const int ks = t / 4, kb = t % 4;
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq)
        S[kb][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t % RING], Q[nq][ks], S[kb][nq], 0, 0, 0);
      if (t + RING < NOP) ka[t % RING] = k_operand(kbuf, (t + RING) % 4, (t + RING) / 4);
      if (kb & 1) mid(2 * ks + (kb >> 1));
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // Online softmax against a lazily updated reference maximum: p = exp2(c*s - c*mref) is taken
  // with no maximum search; the tile's row sum (needed anyway) tells whether any p left the
  // safe range, and only then the maximum is searched, the reference moved, the accumulators
  // rescaled and the probabilities recomputed.
  auto finish_softmax = [&](bf16x8 (&Pn)[2][NQ], float (&lacc)[NQ]) {
    // each p <= this lane's partial sum of its column; !(x <= bound) is also true for NaN
    bool unsafe = false;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) unsafe = unsafe || !(lacc[nq] <= SAFE_SUM);
    if (!CAREFUL) {
      bad = bad || __any(unsafe);
    } else if (__any(unsafe)) {
      float mc2[NQ];
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        const float mnew = fmaxf(mref[nq], row_max(S, nq));
        const float alpha = __builtin_amdgcn_exp2f((mref[nq] - mnew) * c_log2);
        lsum[nq] *= alpha;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int i = 0; i < 4; ++i) O[cb][nq][i] *= alpha;
        mref[nq] = mnew;
        lacc[nq] = 0.f;
        mc2[nq] = mnew * c_log2;
      }
#pragma unroll
      for (int j = 0; j < 4 * NQ; ++j) prob_slice(S, j, mc2, Pn, lacc);
    }
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      lsum[nq] += lacc[nq];
#pragma unroll
      for (int c32 = 0; c32 < 2; ++c32) Pb[c32][nq] = Pn[c32][nq];
    }
  };
  // O^T += V^T P^T for the tile whose probabilities are in Pb.  Chunk c32 covers keys 32*c32 .. +31 of the
  // tile; slot e of lane group g4 is key 32*c32 + 4*g4 + e (e < 4) or 32*c32 + 16 + 4*g4 + (e - 4), the order in
  // which two score accumulator blocks delivered the probabilities (and the V^T image stores).  Every V^T
  // operand feeds the MFMAs of both query blocks.  With OVERLAP the softmax of the next tile (scores in S) is
  // interleaved, one 4-score block per two operands, so the VALU works while the MFMA pipe does; each V^T
  // operand register is refilled, four operands ahead, right after the MFMAs that read it.
  // Both MFMA phases of a step run at wave priority 1, the bookkeeping after them, the wait for the step's
  // loads and the barrier at priority 0: of the two wavefronts sharing a SIMD, the one that is still
  // computing is served before the one that is about to wait anyway, which shortens the skew at the
  // barrier (+0.4 ... 0.9 % on every workload; giving the two phases different levels, or priority to the
  // MFMAs only, was no better or worse).
  auto pv = [&](const unsigned char* vbuf, auto overlap_c, bf16x8 (&Pn)[2][NQ], float (&lacc)[NQ]) {
    constexpr bool OVERLAP = decltype(overlap_c)::value;
    constexpr int NOP = 2 * CB;  // operands of the tile: [32-key chunk][channel block]
    float mc[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) mc[nq] = mref[nq] * c_log2;
    auto v_operand = [&](int t) {
      return *reinterpret_cast<const bf16x8*>(vbuf + (t % CB) * 16 * 128 + voff[t / CB]);
    };
    bf16x8 va[RING];
#pragma unroll
    for (int t = 0; t < RING; ++t) va[t] = v_operand(t);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int t = 0; t < NOP; ++t) {
      const int c32 = t / CB, cb = t % CB;
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq)
        O[cb][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t % RING], Pb[c32][nq], O[cb][nq], 0, 0, 0);
      if (t + RING < NOP) va[t % RING] = v_operand(t + RING);
      // the 4 NQ score blocks of the next tile are soft-maxed during this phase, spread evenly over it
      if (OVERLAP) {
#pragma unroll
        for (int j = t * (4 * NQ) / NOP; j < (t + 1) * (4 * NQ) / NOP; ++j) prob_slice(S, j, mc, Pn, lacc);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep this MFMA / VALU interleave
    }
    __builtin_amdgcn_s_setprio(0);
  };

  using GENERAL = std::false_type;
  // ---- prologue: tiles 0 (and K of tile 1) in flight; scores and softmax of tile 0
  issue_k(0, B0{}, GENERAL{});
  issue_v(0, B0{}, GENERAL{});
  if (ntiles > 1) issue_k(1, B1{}, GENERAL{});
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __syncthreads();
  scores(smem + KBUF0, [](int) {});
  mask_scores(S, 0);
  {
    bf16x8 Pn[2][NQ];
    float lacc[NQ], mc[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      mref[nq] = row_max(S, nq);  // finite: key 0 is visible to every row
      mc[nq] = mref[nq] * c_log2;
      lacc[nq] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < 4 * NQ; ++j) prob_slice(S, j, mc, Pn, lacc);
    finish_softmax(Pn, lacc);
  }
  __syncthreads();  // every wavefront is done with K buffer 0 before tile 2 overwrites it

  // ---- steady state, step t >= 1 (BUF = t & 1): scores of tile t, then PV of tile t-1 on the
  //      MFMA pipe interleaved with the softmax of tile t on the VALU.
  //      LEAN steps (sweep only) are those whose tiles t and t + 1 are both whole prefix tiles: no mask, no
  //      choice of key set, no bounds on t.
  auto step = [&](int t, auto buf_c, auto lean_c) {
    constexpr int BUF = decltype(buf_c)::value;
    constexpr bool LEAN = decltype(lean_c)::value;
    scores(smem + KBUF0 + BUF * TL::KBYTES, [&](int kk) {
      if (kk == KK / 8 && (LEAN || t + 1 < ntiles)) issue_k(t + 1, std::integral_constant<int, BUF ^ 1>{}, lean_c);
      if (kk == KK / 2 + KK / 8) issue_v(t, std::integral_constant<int, BUF>{}, lean_c);
    });
    if (!LEAN) mask_scores(S, t);
    bf16x8 Pn[2][NQ];
    float lacc[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) lacc[nq] = 0.f;
    pv(smem + VBUF0 + (BUF ^ 1) * TL::VBYTES, std::true_type{}, Pn, lacc);
    finish_softmax(Pn, lacc);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // the loads issued in this step have landed
    __syncthreads();
  };
  {
    int t = 1;
    if constexpr (SWEEP) {  // pairs of steps inside the prefix, away from its last tile (which may be ragged)
      const int lean_end = P / BN - 1;  // steps t <= lean_end - 1 have tiles t and t + 1 whole and in the prefix
      for (; t + 1 < lean_end; t += 2) {
        step(t, B1{}, std::true_type{});
        step(t + 1, B0{}, std::true_type{});
      }
    }
    for (; t + 1 < ntiles; t += 2) {
      step(t, B1{}, GENERAL{});
      step(t + 1, B0{}, GENERAL{});
    }
    if (t < ntiles) step(t, B1{}, GENERAL{});
  }
  // ---- drain: PV of the last tile
  {
    bf16x8 Pn[2][NQ];
    float lacc[NQ];
    pv(smem + VBUF0 + ((ntiles - 1) & 1) * TL::VBYTES, std::false_type{}, Pn, lacc);
  }

  if (!CAREFUL) {  // tell the careful kernel whether it has to redo this item (every wavefront owns a word)
    if (lane == 0) item_flags[wave] = bad ? 1 : 0;
    if (bad) return;
  }
  // ---- epilogue: normalise and write.  Register i of block (cb, nq) is channel 16*cb + 4*g4 + i of query
  //      column nq of this lane.
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const float l = quad_sum(lsum[nq]);
    const int64_t row = out_row(nq);
    if (EPI != 0) {
      if (row >= 0) {
        float lse_f = mref[nq] * scale + __logf(l);
        float a1 = 0.f, a2 = 1.0f / l;
        if (EPI == 2) {  // weights of the two partials, as in the merge kernel
          const float l1 = lse1[row];
          const float m = fmaxf(l1, lse_f);  // finite: every row sees at least its own key
          const float w1 = expf(l1 - m), w2 = expf(lse_f - m);
          const float tot = w1 + w2;
          const float inv = 1.0f / tot;
          a1 = w1 * inv;
          a2 *= w2 * inv;
          lse_f = m + logf(tot);
        }
        __bf16* op = out_final + row * D + 4 * g4;
        const float* p1 = o1 + row * D + 4 * g4;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          f32x4 w = O[cb][nq] * a2;
          if (EPI == 2) w += a1 * *reinterpret_cast<const f32x4*>(p1 + cb * 16);
          *reinterpret_cast<bf16x4*>(op + cb * 16) = __builtin_convertvector(w, bf16x4);
        }
        if (g4 == 0) lse_final[row] = lse_f;
      }
    } else if (row >= 0) {
      const float inv = 1.0f / l;
      const int64_t prow = (CAUSAL ? 0 : (int64_t)it.split * part_rows) + row;  // key split s fills partial s
      float* op = o_part + prow * D + 4 * g4;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) *reinterpret_cast<f32x4*>(op + cb * 16) = O[cb][nq] * inv;
      if (g4 == 0) lse_part[prow] = mref[nq] * scale + __logf(l);
    }
  }
}

}  // namespace

int launch_pass_bf16(const PassArgs& a, void* stream) {
  if (a.num_items == 0) return 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const __bf16* q = static_cast<const __bf16*>(a.q);
  const __bf16* k = static_cast<const __bf16*>(a.k);
  const __bf16* vt = static_cast<const __bf16*>(a.vt);
  const unsigned grid = (unsigned)a.num_items;
  __bf16* outf = static_cast<__bf16*>(a.out_final);
  const __bf16* kpre = static_cast<const __bf16*>(a.k_pre);
  const __bf16* vtpre = static_cast<const __bf16*>(a.vt_pre);
// Every pass is two launches over the same work list: the common kernel, whose step has no code for a moving
// reference maximum, and the careful kernel, which redoes the items the first one gave up on (none, normally).
#define PA_LAUNCH(DD, CC, EE, SS)                                                                                  \
  do {                                                                                                             \
    pass_bf16_kernel<DD, CC, EE, SS, false><<<grid, NTHREADS, 0, s>>>(                                             \
        q, k, vt, a.o_part, a.lse_part, a.o1, a.lse1, outf, a.lse_final, a.items, a.cu, a.vt_off,                  \
        a.vt_tiles_per_head, kpre, vtpre, a.vt_pre_tiles_per_head, a.part_rows, a.Hq, a.Hkv, a.group, a.scale,     \
        a.flags);                                                                                                  \
    pass_bf16_kernel<DD, CC, EE, SS, true><<<grid, NTHREADS, 0, s>>>(                                              \
        q, k, vt, a.o_part, a.lse_part, a.o1, a.lse1, outf, a.lse_final, a.items, a.cu, a.vt_off,                  \
        a.vt_tiles_per_head, kpre, vtpre, a.vt_pre_tiles_per_head, a.part_rows, a.Hq, a.Hkv, a.group, a.scale,     \
        a.flags);                                                                                                  \
  } while (0)
#define PA_LAUNCH_D(DD)                                                                                            \
  if (!a.causal) PA_LAUNCH(DD, false, 0, false);                                                                   \
  else if (a.epilogue == 0 && a.sweep_prefix) PA_LAUNCH(DD, true, 0, true);                                        \
  else if (a.epilogue == 0) PA_LAUNCH(DD, true, 0, false);                                                         \
  else if (a.epilogue == 1 && a.sweep_prefix) PA_LAUNCH(DD, true, 1, true);                                        \
  else if (a.epilogue == 1) PA_LAUNCH(DD, true, 1, false);                                                         \
  else PA_LAUNCH(DD, true, 2, false)
  if (!a.flags) return 1;
  if (a.epilogue < 0 || a.epilogue > 2 || (!a.causal && a.epilogue != 0)) return 1;
  if (a.sweep_prefix && (!a.causal || a.epilogue == 2 || !a.k_pre || !a.vt_pre)) return 1;
  if (a.D == 128) {
    PA_LAUNCH_D(128);
  } else {
    PA_LAUNCH_D(64);
  }
#undef PA_LAUNCH_D
#undef PA_LAUNCH
  return (int)hipGetLastError();
}

}  // namespace pa
