// Response-token log-probabilities: logp_n = z_{y_n} - ln sum_v exp(z_v), z = logit_scale * W h_n,
// without ever materialising the [tokens, vocabulary] logits.
//
// The GRPO objective (paper Eq. 1) needs the probabilities the policy, the old policy and the
// reference model give to the sampled response tokens; after the prefill each device computes the
// logits of its token slice (Sec. 5.2).  With a 7B-class model that is a [N, 3584] x [3584, 152064]
// product per model, 1.8e13 FLOP for 16K response tokens, and the logits (10 GB in fp32) are only
// ever reduced to two numbers per token.
//
// Kernel 1 (bf16 MFMA GEMM with a reducing epilogue).  A workgroup (8 wavefronts) computes one
// 256-vocabulary x 256-token tile of Z^T = W H^T: wavefront (wv, wt) owns 64 vocabulary rows x 128
// tokens (4 x 8 accumulator blocks of v_mfma_f32_16x16x32_bf16, 128 registers; that shape moves half
// the accumulator data per FLOP of the 32 x 32 x 16 one and sustains about 10 % more under the board's
// power limit).  W and H panels of
// 64 channels go global -> LDS through range-checked buffer loads (rows past the end of either
// matrix read as zero), double buffered, one barrier per 64 channels; 12 LDS operand reads feed 32
// MFMAs.  In the epilogue every lane holds 16 logits of each of 8 tokens: it reduces them to a
// maximum and a sum of exponentials, combines with the three lanes holding the token's other rows and, through
// LDS, with the other three row blocks, so the tile writes one (m, l) pair per token; the lane that
// holds the target's logit writes it out.  Workgroups are numbered so that the 32 tiles running together on one XCD form an
// 8-token-tile x 4-vocabulary-tile block: 12 distinct panels per step share that XCD's L2
// instead of 64.
// Kernel 2 combines the (m, l) pairs of a token over all vocabulary blocks: LSE = m + ln l,
// logp = z_target - LSE.
#include <hip/hip_runtime.h>

#include "logprob.h"
#include "mfma_tiles.h"

namespace pa {
namespace {

using namespace mt;

constexpr int LP_WAVES = 8, LP_THREADS = LP_WAVES * 64;
constexpr int BK = 64;                      // channels per stage
constexpr int PANEL_BYTES = LP_TILE * BK * 2;  // one 256-row x 64-channel panel
constexpr int LP_STAGE = 2 * PANEL_BYTES;      // W panel, H panel
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// v_mfma_f32_16x16x32_bf16 (l16 = lane % 16, g4 = lane / 16): A: lane holds row l16, contraction indices
// 8*g4 .. 8*g4+7; B: column l16, the same indices; C: register i holds row 4*g4 + i, column l16.
// The four lanes l16, l16 + 16, l16 + 32, l16 + 48 hold the 16 rows of a column: maximum / sum over them.
__device__ inline void pair_values(float x, float& a, float& b) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const unsigned r0 = r[0], r1 = r[1];   // read through named temporaries, see attn_bf16.hip
  a = __uint_as_float(r0);
  b = __uint_as_float(r1);
}
__device__ inline float column_max(float x) {
  x = fmaxf(x, __shfl_xor(x, 16));
  float u, w;
  pair_values(x, u, w);
  return fmaxf(u, w);
}
__device__ inline float column_sum(float x) {
  x += __shfl_xor(x, 16);
  float u, w;
  pair_values(x, u, w);
  return u + w;
}

__global__ __launch_bounds__(LP_THREADS, 1) void logprob_tile_kernel(
    const __bf16* __restrict__ hidden, const __bf16* __restrict__ lm_head, const int32_t* __restrict__ targets,
    float2* __restrict__ partials, float* __restrict__ target_logit, int64_t N, int d, int V, int TM, int TV,
    int by_tm, float logit_scale) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * LP_STAGE];

  // ---- which tile: XCD x = blockIdx % 8 owns a slice of the token tiles (or, with fewer than 8
  //      token tiles, of the vocabulary tiles) and walks it in 8 x 4 blocks of tiles
  int tm, tv;
  {
    const int n = blockIdx.x, x = n & 7, j = n >> 3;
    if (by_tm) {
      const int mine = (TM - x + 7) / 8;          // token tiles tm = x + 8 k, k < mine
      const int ngm = ((TM + 7) / 8 + 7) / 8;     // groups of 8 owned token tiles (same for every XCD)
      const int g = j / 32, i = j % 32;
      const int k = (g % ngm) * 8 + (i & 7);
      tv = (g / ngm) * 4 + (i >> 3);
      tm = x + 8 * k;
      if (k >= mine || tv >= TV) return;
    } else {
      tm = j % TM;
      tv = x + 8 * (j / TM);
      if (tv >= TV) return;
    }
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;
  const int wv = wave & 3, wt = wave >> 2;
  const int64_t v0 = (int64_t)tv * LP_TILE, t0 = (int64_t)tm * LP_TILE;

  // ---- loads: a panel is 256 rows x 128 bytes = 32 blocks of 1 KiB (8 rows each), 4 per wavefront
  const int64_t rowb = (int64_t)d * 2;
  const int64_t w_rows = V - v0 < LP_TILE ? V - v0 : LP_TILE, h_rows = N - t0 < LP_TILE ? N - t0 : LP_TILE;
  const rsrc_t r_w = make_rsrc(lm_head + v0 * d, w_rows * rowb);
  const rsrc_t r_h = make_rsrc(hidden + t0 * d, h_rows * rowb);
  unsigned loff[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    const int row = (wave * 4 + n) * 8 + lane / 8;
    const int chunk = (lane % 8) ^ swizzle_term(row, 128);  // logical chunk stored at this position
    loff[n] = (unsigned)(row * rowb + chunk * 16);
  }
  auto issue = [&](int stage, int buf) {
    unsigned char* dst = smem + buf * LP_STAGE;
    const unsigned k_off = (unsigned)stage * (BK * 2);
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_w, (PA_LDS_PTR(void))(dst + (wave * 4 + n) * 1024), 16, loff[n], k_off, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_h, (PA_LDS_PTR(void))(dst + PANEL_BYTES + (wave * 4 + n) * 1024), 16,
                                               loff[n], k_off, 0, 0);
    }
  };

  constexpr int NA = 4, NB = 8;   // 16-row blocks of the wavefront's 64 vocabulary rows / 128 tokens
  f32x4 C[NA][NB];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b) C[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Per-lane LDS addresses of the operand reads, one set per buffer (the second buffer lies 64 KiB on,
  // beyond the reach of a read's immediate offset), so the main loop itself holds no address arithmetic.
  // (Row blocks of 16 share the swizzle of rows 0..15.)
  const unsigned char* wop[2][BK / 32];
  const unsigned char* hop[2][BK / 32];
#pragma unroll
  for (int bufi = 0; bufi < 2; ++bufi)
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      const int off = l16 * 128 + (((4 * ks + g4) ^ swizzle_term(l16, 128)) << 4);
      wop[bufi][ks] = smem + bufi * LP_STAGE + (wv * 64) * 128 + off;
      hop[bufi][ks] = smem + bufi * LP_STAGE + PANEL_BYTES + (wt * 128) * 128 + off;
    }

  const int nstages = (d + BK - 1) / BK;  // channels past d read as zero (range-checked loads)
  auto stage = [&](int s, auto buf_c) {
    constexpr int BUF = decltype(buf_c)::value;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's share of stage s has landed
    __syncthreads();                      // everyone's share has; the other buffer is no longer read
    if (s + 1 < nstages) issue(s + 1, BUF ^ 1);
    // The MFMA part of a stage runs at wave priority 1, the wait, the barrier and the issue of the next stage's
    // loads at priority 0: of the two wavefronts sharing a SIMD, the one already in its MFMAs is served before
    // the one still issuing loads (+1.5 %; priority for the loads instead: -0.4 %).
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      bf16x8 wa[NA], hb[NB];
#pragma unroll
      for (int a = 0; a < NA; ++a) wa[a] = lds_operand(wop[BUF][ks] + a * 16 * 128);
#pragma unroll
      for (int b = 0; b < NB; ++b) hb[b] = lds_operand(hop[BUF][ks] + b * 16 * 128);
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int a = 0; a < NA; ++a) C[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[a], hb[b], C[a][b], 0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  issue(0, 0);
  {
    int s = 0;
    for (; s + 1 < nstages; s += 2) {
      stage(s, std::integral_constant<int, 0>{});
      stage(s + 1, std::integral_constant<int, 1>{});
    }
    if (s < nstages) stage(s, std::integral_constant<int, 0>{});
  }

  // ---- epilogue.  Register i of C[a][b]: vocabulary row v0 + wv*64 + a*16 + 4*g4 + i,
  //      token t0 + wt*128 + b*16 + l16.
  const float c2 = logit_scale * LOG2E;  // work in base 2
  __syncthreads();                        // every wavefront is done with the panels: reuse the LDS
  float2* stage_ml = reinterpret_cast<float2*>(smem);  // [4 row blocks][256 tokens] (m in base-2 units, l)
  const int64_t vlane = v0 + wv * 64 + 4 * g4;         // this lane's first vocabulary row
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int64_t tok = t0 + wt * 128 + b * 16 + l16;
    float m = -INFINITY;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (vlane + a * 16 + i < V) m = fmaxf(m, C[a][b][i]);
    m = column_max(m) * c2;  // -inf only when none of the block's 64 rows exists
    float l = 0.f;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (vlane + a * 16 + i < V) l += __builtin_amdgcn_exp2f(__builtin_fmaf(C[a][b][i], c2, -m));
    l = column_sum(l);
    if (g4 == 0) stage_ml[wv * LP_TILE + wt * 128 + b * 16 + l16] = float2{m, l};  // m = -inf, l = 0 for a block past V
    if (tok < N) {
      // the target's logit, if it lies in this wavefront's 64 rows and this lane's four of every 16
      const int64_t rel = (int64_t)targets[tok] - (v0 + wv * 64);
      if (rel >= 0 && rel < 64) {
        const int r = (int)rel & 15, a_t = (int)rel >> 4;
        if ((r >> 2) == g4) {
          const int i_t = r & 3;
          float z = 0.f;
#pragma unroll
          for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (a == a_t && i == i_t) z = C[a][b][i];
          target_logit[tok] = z * logit_scale;
        }
      }
    }
  }
  // one (m, l) pair per token for the tile's 256 vocabulary rows (block 0 always exists)
  __syncthreads();
  if (tid < LP_TILE && t0 + tid < N) {
    float m = stage_ml[tid].x;
#pragma unroll
    for (int k = 1; k < 4; ++k) m = fmaxf(m, stage_ml[k * LP_TILE + tid].x);
    float l = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2 v = stage_ml[k * LP_TILE + tid];
      l += v.y * __builtin_amdgcn_exp2f(v.x - m);
    }
    partials[(int64_t)tv * N + t0 + tid] = float2{m * LN2, l};
  }
}

// (m, l) pairs of a token over all vocabulary tiles -> LSE and log-probability.  A block handles
// 64 tokens; its 4 thread groups each walk every fourth tile with an online combine, then merge.
__global__ __launch_bounds__(256) void logprob_finalize_kernel(const float2* __restrict__ partials,
                                                               const float* __restrict__ target_logit,
                                                               const int32_t* __restrict__ targets,
                                                               float* __restrict__ logprob, float* __restrict__ lse_out,
                                                               int64_t N, int nparts, int V) {
  __shared__ float2 sm[4][64];
  const int tl = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int64_t tok = (int64_t)blockIdx.x * 64 + tl;
  float m = -INFINITY, l = 0.f;
  if (tok < N)
    for (int p = grp; p < nparts; p += 4) {
      const float2 v = partials[(int64_t)p * N + tok];
      const float mn = fmaxf(m, v.x);
      l = l * expf(m - mn) + v.y * expf(v.x - mn);  // first term: 0 * exp(-inf) = 0
      m = mn;
    }
  sm[grp][tl] = float2{m, l};
  __syncthreads();
  if (grp == 0 && tok < N) {
    float mm = m;
#pragma unroll
    for (int k = 1; k < 4; ++k) mm = fmaxf(mm, sm[k][tl].x);
    float ll = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2 v = sm[k][tl];
      ll += v.y > 0.f ? v.y * expf(v.x - mm) : 0.f;  // a group that saw no tile holds (-inf, 0)
    }
    const float lse = mm + logf(ll);
    // no tile holds the logit of an id outside [0, V) (an ignore index, say): its slot was never written
    const int32_t y = targets[tok];
    logprob[tok] = (y >= 0 && y < V) ? target_logit[tok] - lse : __builtin_nanf("");
    if (lse_out) lse_out[tok] = lse;
  }
}

// Eq. 2: A_i = (r_i - mean) / std over one group of G rewards (population std; equal rewards -> 0).
__global__ __launch_bounds__(64) void group_advantages_kernel(const float* __restrict__ rewards,
                                                              float* __restrict__ adv, int G, int num_groups) {
  const int g = blockIdx.x * 64 + threadIdx.x;
  if (g >= num_groups) return;
  const float* r = rewards + (int64_t)g * G;
  float mean = 0.f;
  for (int i = 0; i < G; ++i) mean += r[i];
  mean /= (float)G;
  float var = 0.f;
  for (int i = 0; i < G; ++i) var += (r[i] - mean) * (r[i] - mean);
  const float sd = sqrtf(var / (float)G);
  for (int i = 0; i < G; ++i) adv[(int64_t)g * G + i] = sd > 0.f ? (r[i] - mean) / sd : 0.f;
}

}  // namespace

int launch_logprob(const LogprobArgs& a, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int TM = (int)((a.N + LP_TILE - 1) / LP_TILE), TV = (a.V + LP_TILE - 1) / LP_TILE;
  const int by_tm = TM >= 8;
  int64_t grid;
  if (by_tm) {
    const int ngm = ((TM + 7) / 8 + 7) / 8;
    grid = (int64_t)8 * 32 * ngm * ((TV + 3) / 4);
  } else {
    grid = (int64_t)8 * TM * ((TV + 7) / 8);
  }
  logprob_tile_kernel<<<(unsigned)grid, LP_THREADS, 0, s>>>(
      static_cast<const __bf16*>(a.hidden), static_cast<const __bf16*>(a.lm_head), a.targets,
      reinterpret_cast<float2*>(a.partials), a.target_logit, a.N, a.d, a.V, TM, TV, by_tm, a.logit_scale);
  if (hipGetLastError() != hipSuccess) return 1;
  logprob_finalize_kernel<<<(unsigned)((a.N + 63) / 64), 256, 0, s>>>(
      reinterpret_cast<const float2*>(a.partials), a.target_logit, a.targets, a.logprob, a.lse, a.N, TV, a.V);
  return (int)hipGetLastError();
}

int launch_group_advantages(const float* rewards, float* adv, int G, int num_groups, void* stream) {
  if (num_groups == 0) return 0;
  group_advantages_kernel<<<(unsigned)((num_groups + 63) / 64), 64, 0, static_cast<hipStream_t>(stream)>>>(
      rewards, adv, G, num_groups);
  return (int)hipGetLastError();
}

}  // namespace pa
