// Building blocks shared by the bf16 MFMA kernels (gfx950): vector types, the two LDS tile
// layouts with their bank-conflict-free XOR swizzles, direct-to-LDS tile loads and the lane
// exchange.  Device code only.
//
// v_mfma_f32_32x32x16_bf16 operand layout (64 lanes, l32 = lane % 32, hf = lane / 32):
//   A: lane holds row l32 of the 32-row block, contraction indices 8*hf .. 8*hf+7
//   B: lane holds column l32,                  contraction indices 8*hf .. 8*hf+7
//   C: register i holds row 8*(i/4) + 4*hf + i%4, column l32
// An accumulator of a first product is turned into the B operand of a second product by
// packing registers 0..7 and 8..15 into two 8-element operands; contraction slot e of half hf
// then is accumulator row 4*hf + e (e < 4) or 8 + 4*hf + (e - 4) of the 16-row chunk, i.e. the
// rows of a chunk appear in the order 0-3, 8-11, 4-7, 12-15.  The transposed tile images store
// their 64 columns in exactly this order, so the second product's A operand matches.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace pa {
namespace mt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

#define PA_LDS_PTR(T) __attribute__((address_space(3))) T*
#define PA_GLB_PTR(T) __attribute__((address_space(1))) T*

constexpr int TILE = 64;  // rows of a row-major tile = columns of a transposed image

// Row-major tile: 64 rows of D bf16 (rows of 2*D bytes).  Transposed image: D rows of 64 bf16
// (rows of 128 bytes).  The 16-byte chunk j of row r is stored at chunk position
//   j ^ (r & 15)         for 256-byte rows,
//   j ^ ((r >> 1) & 7)   for 128-byte rows,
// so 16 consecutive rows read at one logical chunk cover all 64 banks.
__device__ inline int swizzle_term(int row, int rowb) { return rowb == 256 ? (row & 15) : ((row >> 1) & 7); }

// A second swizzle for row-major tiles that are read both as MFMA operands along the row (16-byte
// reads, 16 consecutive rows at one logical chunk) and transposed with ds_read_b64_tr_b16 (per
// 16 lanes: 4 consecutive rows x two 16-byte chunks).  Both patterns are conflict free with
//   256-byte rows: chunk ^ (((r & 3) << 2) | ((r >> 2) & 3))
//   128-byte rows: chunk ^ (((L & 1) << 2) | ((L >> 1) & 3)),  L = (r >> 1) & 7.
__device__ inline int swizzle_term_tr(int row, int rowb) {
  if (rowb == 256) return ((row & 3) << 2) | ((row >> 2) & 3);
  const int L = (row >> 1) & 7;
  return ((L & 1) << 2) | ((L >> 1) & 3);
}

template <int D>
struct Geo {
  static constexpr int ROWB = D * 2;            // bytes per row of a row-major tile
  static constexpr int ROW_TILE_BYTES = TILE * ROWB;
  static constexpr int IMAGE_BYTES = D * 128;
  static constexpr int KK = D / 16;             // contraction steps over the head dimension
  static constexpr int DB = D / 32;             // 32-channel blocks
};

// Byte offset, inside a row-major tile, of the A/B operand of row (blk*32 + l32) and channels
// 16*kk + 8*hf .. +7.  (Rows blk*32.. share the swizzle of rows 0..31 because 32 % 16 == 0.)
template <int D>
__device__ inline int row_operand_offset(int l32, int hf, int kk) {
  return l32 * Geo<D>::ROWB + (((2 * kk + hf) ^ swizzle_term(l32, Geo<D>::ROWB)) << 4);
}
// Byte offset, inside a transposed image, of the A operand of channel (db*32 + l32) and the
// 16-column chunk ch (contraction slots 8*hf .. 8*hf+7 of that chunk).
__device__ inline int image_operand_offset(int l32, int hf, int ch) {
  return l32 * 128 + (((2 * ch + hf) ^ swizzle_term(l32, 128)) << 4);
}

__device__ inline bf16x8 lds_operand(const unsigned char* p) { return *reinterpret_cast<const bf16x8*>(p); }

// The same operand offset for a tile stored with swizzle_term_tr.
template <int D>
__device__ inline int row_operand_offset_tr(int l32, int hf, int kk) {
  return l32 * Geo<D>::ROWB + (((2 * kk + hf) ^ swizzle_term_tr(l32, Geo<D>::ROWB)) << 4);
}
// Transposed operand from a row-major tile [64 rows][D] stored with swizzle_term_tr: the A operand
// of a product that contracts over the tile's ROWS.  Lane (l32, hf) receives channel db*32 + l32 and
// contraction slots e = 0..7 = rows 16*ch + 4*hf + e (e < 4), 16*ch + 8 + 4*hf + (e - 4): the order in
// which a packed accumulator delivers its rows.  ds_read_b64_tr_b16 hands lane i of a 16-lane group
// element (i % 4) of the 8 bytes addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12; so lane s of the
// group addresses row R0 + s/4, channels Cb + 4*(s % 4) .. +3, and lane i receives channel Cb + i of
// rows R0 .. R0 + 3.  `lane_byte` is this lane's byte offset for (db = 0, ch = 0, first half).
template <int D>
__device__ inline int tr_lane_row(int lane) { return 4 * (lane >> 5) + ((lane & 15) >> 2); }
template <int D>
__device__ inline int tr_operand_offset(int lane, int db, int ch, int half) {
  constexpr int ROWB = Geo<D>::ROWB;
  const int r = 16 * ch + 8 * half + tr_lane_row<D>(lane);
  const int c = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  return r * ROWB + (((c >> 3) ^ swizzle_term_tr(r, ROWB)) << 4) + (c & 7) * 2;
}
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
__device__ inline bf16x8 lds_operand_tr(const unsigned char* lo, const unsigned char* hi) {
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((PA_LDS_PTR(s16x4))lo);
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((PA_LDS_PTR(s16x4))hi);
  const s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Direct-to-LDS copy of 1 KiB per wavefront-wide instruction: lane l's 16 bytes land at dst + 16*l.
__device__ inline void load16_to_lds(const void* src, unsigned char* dst) {
  __builtin_amdgcn_global_load_lds((PA_GLB_PTR(const void))src, (PA_LDS_PTR(void))dst, 16, 0, 0);
}

// Row-major tile -> LDS, NW wavefronts cooperating.  `first` points at channel 0 of the tile's
// first row, rows are row_stride elements apart, rows at or past `rows_left` repeat the last
// existing row (callers mask what those rows produce).  rows_left >= 1.
template <int D, int NW>
__device__ inline void issue_row_tile(unsigned char* dst, const __bf16* first, int64_t row_stride, int rows_left,
                                      int wave, int lane, bool tr_swizzle = false) {
  constexpr int ROWB = Geo<D>::ROWB;
  constexpr int BLOCKS_PER_WAVE = Geo<D>::ROW_TILE_BYTES / 1024 / NW;
  constexpr int LANES_PER_ROW = ROWB / 16, ROWS_PER_BLOCK = 1024 / ROWB;
  static_assert(BLOCKS_PER_WAVE >= 1, "every wavefront copies at least one block");
#pragma unroll
  for (int n = 0; n < BLOCKS_PER_WAVE; ++n) {
    const int blk = wave * BLOCKS_PER_WAVE + n;
    int row = blk * ROWS_PER_BLOCK + lane / LANES_PER_ROW;
    const int swz = tr_swizzle ? swizzle_term_tr(row, ROWB) : swizzle_term(row, ROWB);
    const int col = ((lane % LANES_PER_ROW) ^ swz) * 8;  // logical chunk stored at this position
    row = row < rows_left ? row : rows_left - 1;
    load16_to_lds(first + row * row_stride + col, dst + blk * 1024);
  }
}

// The same for a tile whose 64 rows all exist, with the per-lane byte offsets computed once:
// the address is a uniform tile base plus a 32-bit lane offset.
template <int D, int NW>
struct RowTileOffsets {
  static constexpr int BLOCKS_PER_WAVE = Geo<D>::ROW_TILE_BYTES / 1024 / NW;
  unsigned off[BLOCKS_PER_WAVE];
  __device__ inline void init(int64_t row_stride, int wave, int lane, bool tr_swizzle = false) {
    constexpr int ROWB = Geo<D>::ROWB, LANES_PER_ROW = ROWB / 16, ROWS_PER_BLOCK = 1024 / ROWB;
#pragma unroll
    for (int n = 0; n < BLOCKS_PER_WAVE; ++n) {
      const int row = (wave * BLOCKS_PER_WAVE + n) * ROWS_PER_BLOCK + lane / LANES_PER_ROW;
      const int swz = tr_swizzle ? swizzle_term_tr(row, ROWB) : swizzle_term(row, ROWB);
      const int col = ((lane % LANES_PER_ROW) ^ swz) * 8;
      off[n] = (unsigned)((row * row_stride + col) * 2);
    }
  }
};
template <int D, int NW>
__device__ inline void issue_full_row_tile(unsigned char* dst, const __bf16* first, const RowTileOffsets<D, NW>& o,
                                           int wave) {
  const char* base = reinterpret_cast<const char*>(first);
#pragma unroll
  for (int n = 0; n < RowTileOffsets<D, NW>::BLOCKS_PER_WAVE; ++n)
    load16_to_lds(base + o.off[n], dst + (wave * RowTileOffsets<D, NW>::BLOCKS_PER_WAVE + n) * 1024);
}

// Linear copy of `bytes` (a multiple of 1024 * NW) global -> LDS.
template <int BYTES, int NW>
__device__ inline void issue_linear(unsigned char* dst, const void* src, int wave, int lane) {
  constexpr int BLOCKS_PER_WAVE = BYTES / 1024 / NW;
  static_assert(BLOCKS_PER_WAVE >= 1 && BYTES % (1024 * NW) == 0, "whole blocks per wavefront");
  const char* s = static_cast<const char*>(src) + (wave * BLOCKS_PER_WAVE) * 1024 + lane * 16;
#pragma unroll
  for (int n = 0; n < BLOCKS_PER_WAVE; ++n) load16_to_lds(s + n * 1024, dst + (wave * BLOCKS_PER_WAVE + n) * 1024);
}

// ---- the same copies through buffer instructions: a 128-bit resource descriptor in scalar
// registers (base address, no stride, 2 GiB range, raw dword format), a uniform byte offset in
// a scalar register, a 32-bit lane offset and an immediate.  No vector address arithmetic at
// all, and offsets past the range read as zero instead of faulting (a range shorter than the
// tile replaces explicit clamping of a ragged last tile).
#if defined(__HIP_DEVICE_COMPILE__)
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ inline rsrc_t make_rsrc(const void* base, int64_t bytes = 0x7fffffff) {
  const int n = bytes < 0 ? 0 : (bytes > 0x7fffffff ? 0x7fffffff : (int)bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}
template <int D, int NW>
__device__ inline void issue_full_row_tile(unsigned char* dst, rsrc_t r, unsigned tile_byte_offset,
                                           const RowTileOffsets<D, NW>& o, int wave) {
#pragma unroll
  for (int n = 0; n < RowTileOffsets<D, NW>::BLOCKS_PER_WAVE; ++n)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        r, (PA_LDS_PTR(void))(dst + (wave * RowTileOffsets<D, NW>::BLOCKS_PER_WAVE + n) * 1024), 16, o.off[n],
        tile_byte_offset, 0, 0);
}
template <int BYTES, int NW>
__device__ inline void issue_linear(unsigned char* dst, rsrc_t r, unsigned byte_offset, int wave, int lane) {
  constexpr int BLOCKS_PER_WAVE = BYTES / 1024 / NW;
  static_assert(BLOCKS_PER_WAVE >= 1 && BLOCKS_PER_WAVE <= 4 && BYTES % (1024 * NW) == 0, "whole blocks, small immediates");
  const unsigned soff = byte_offset + (unsigned)(wave * BLOCKS_PER_WAVE) * 1024u;
  unsigned char* d0 = dst + (wave * BLOCKS_PER_WAVE) * 1024;
  const unsigned voff = (unsigned)lane * 16u;
  // The instruction's immediate offset is added to the memory address AND to the LDS address, so
  // all blocks name the same LDS base.  It must be a literal, hence no loop.
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (PA_LDS_PTR(void))d0, 16, voff, soff, 0, 0);
  if constexpr (BLOCKS_PER_WAVE > 1)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (PA_LDS_PTR(void))d0, 16, voff, soff, 1024, 0);
  if constexpr (BLOCKS_PER_WAVE > 2)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (PA_LDS_PTR(void))d0, 16, voff, soff, 2048, 0);
  if constexpr (BLOCKS_PER_WAVE > 3)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (PA_LDS_PTR(void))d0, 16, voff, soff, 3072, 0);
}
// one dword per lane: lane l's word lands at dst + 4*l
__device__ inline void load_dword_to_lds(rsrc_t r, unsigned char* dst, unsigned lane_byte_offset, unsigned byte_offset) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (PA_LDS_PTR(void))dst, 4, lane_byte_offset, byte_offset, 0, 0);
}
// 16 bytes per lane: lane l's chunk lands at dst + 16*l; the source is base + lane_byte_offset + byte_offset
// (byte_offset uniform: it travels in a scalar register, so no per-lane address arithmetic is needed)
__device__ inline void load_chunk_to_lds(rsrc_t r, unsigned char* dst, unsigned lane_byte_offset, unsigned byte_offset) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (PA_LDS_PTR(void))dst, 16, lane_byte_offset, byte_offset, 0, 0);
}
// 16 bytes per lane into registers (same addressing)
__device__ inline i32x4 load_chunk(rsrc_t r, unsigned lane_byte_offset, unsigned byte_offset) {
  return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_byte_offset, byte_offset, 0));
}
#else
// The host pass of hipcc still parses kernel bodies but has no buffer-resource type: empty stand-ins.
struct rsrc_t {};
__device__ inline rsrc_t make_rsrc(const void*, int64_t = 0) { return {}; }
template <int D, int NW>
__device__ inline void issue_full_row_tile(unsigned char*, rsrc_t, unsigned, const RowTileOffsets<D, NW>&, int) {}
template <int BYTES, int NW>
__device__ inline void issue_linear(unsigned char*, rsrc_t, unsigned, int, int) {}
__device__ inline void load_dword_to_lds(rsrc_t, unsigned char*, unsigned, unsigned) {}
__device__ inline void load_chunk_to_lds(rsrc_t, unsigned char*, unsigned, unsigned) {}
__device__ inline i32x4 load_chunk(rsrc_t, unsigned, unsigned) { return i32x4{0, 0, 0, 0}; }
#endif

// Pack four fp32 accumulator registers [r0, r0+4) of a 16-register block into the B operand
// pair Pb[2]: register r goes to operand r >> 3, slot r & 7.
__device__ inline void pack4(const float (&x)[4], int r0, bf16x8 (&Pb)[2]) {
  const f32x2 a = {x[0], x[1]}, b = {x[2], x[3]};
  const bf16x2 pa = __builtin_convertvector(a, bf16x2), pb = __builtin_convertvector(b, bf16x2);
  Pb[r0 >> 3][(r0 & 7) + 0] = pa[0];
  Pb[r0 >> 3][(r0 & 7) + 1] = pa[1];
  Pb[r0 >> 3][(r0 & 7) + 2] = pb[0];
  Pb[r0 >> 3][(r0 & 7) + 3] = pb[1];
}

}  // namespace mt
}  // namespace pa
