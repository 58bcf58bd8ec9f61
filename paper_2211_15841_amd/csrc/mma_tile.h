// LDS staging and MFMA operand fetch shared by the block-sparse products and the router-backward products.
//
// A 128 x BK operand slab is staged in LDS one of two ways round:
//   KC  [row][k], k contiguous (the operand's K index is the contiguous one in memory): read with ds_read_b128;
//   NC  [k][row], row contiguous (K is the strided index in memory): kept as it lies in memory and read with the
//       transposing ds_read_b64_tr_b16, so nothing is ever transposed in HBM or in registers.
// Both are XOR-swizzled instead of padded, which keeps every slab a power of two and lets a direct global->LDS
// load (which writes 1 KB contiguously per wave) produce the swizzled image by permuting what each lane fetches.
#pragma once
#include "common.h"

namespace dmoe {

enum Layout { KC = 0, NC = 1 };

// ---- LDS addressing -------------------------------------------------------------------------------------------
// KC slab: 128 rows x 128 bytes.  16-byte chunk c of row r sits at chunk c ^ ((r >> 1) & 7): the 16 lanes that a
// ds_read_b128 serves per clock (16 consecutive rows, same logical chunk) then cover all 64 banks once.
// (BK = 32: rows are 64 bytes, four rows share a 256-byte bank line, and the swizzle is c ^ ((r >> 2) & 3).)
template <int BK>
__device__ __forceinline__ int kc_offset(int row, int chunk) {
  static_assert(BK == 32 || BK == 64, "unsupported K tile");
  if constexpr (BK == 64) return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
  else                    return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4);
}
// NC slab: 64 k-rows x 256 bytes.  32-byte unit u of k-row k sits at unit u ^ (2 * (k & 3)): the 32 lanes that a
// ds_read_b64_tr_b16 serves per clock (4 k-rows x two adjacent units) then cover all 64 banks once.

typedef __attribute__((address_space(3))) s16x4_v* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* glb_void_ptr;

// A direct global->LDS load writes, for the whole wave, 1 KB at a wave-uniform LDS address: lane l's 16 bytes land
// at +16 l.  To obtain the swizzled slabs the permutation is therefore applied on the global side: this returns
// the element offset (relative to the slab's base pointer) that lane `lane` must fetch for 1 KB chunk `ch`.
template <int L, int BK>
__device__ __forceinline__ uint32_t dma_lane_offset(int ch, int lane, uint32_t ld) {
  static_assert(BK == 32 || BK == 64, "unsupported K tile");
  if constexpr (L == KC && BK == 64) {         // chunk = 8 rows x 128 B
    const int row = 8 * ch + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    return (uint32_t)row * ld + c * 8;
  } else if constexpr (L == KC) {              // chunk = 16 rows x 64 B
    const int row = 16 * ch + (lane >> 2);
    const int c = (lane & 3) ^ ((row >> 2) & 3);
    return (uint32_t)row * ld + c * 8;
  } else {                                     // chunk = 4 k-rows x 256 B
    const int krow = 4 * ch + (lane >> 4);
    const int pc = lane & 15;
    const int u = (pc >> 1) ^ ((krow & 3) << 1);
    return (uint32_t)krow * ld + (2 * u + (pc & 1)) * 8;
  }
}

// MFMA operand for the 32 rows starting at `row0` of the slab and K step ks (16 k): lane l gets row row0 + l%32
// and the 8 consecutive k = 16 ks + 8 (l / 32) + 0..7, whichever way round the slab is staged.
template <int L, int BK>
__device__ __forceinline__ bf16x8_v load_frag(const char* lds, int row0, int ks, int lane) {
  if constexpr (L == KC) {
    const int row = row0 + (lane & 31);
    return *reinterpret_cast<const bf16x8_v*>(lds + kc_offset<BK>(row, 2 * ks + (lane >> 5)));
  } else {
    // ds_read_b64_tr_b16 works on groups of 16 lanes: lane i of a group receives element i of each of the four
    // 16-element rows whose addresses are supplied by lanes 4j..4j+3 (j = 0..3) of the group.
    const int l16 = lane & 15;
    const int kq = l16 >> 2;                                   // k-row (mod 4) this lane supplies the address of
    const int unit = (row0 >> 4) + ((lane >> 4) & 1);
    const int k0 = 16 * ks + 8 * (lane >> 5) + kq;
    const int off0 = k0 * 256 + ((unit ^ (kq << 1)) << 5) + ((l16 & 3) << 3);
    const int off1 = off0 + 4 * 256;                           // k0 + 4 has the same k & 3
    const s16x4_v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + off0));
    const s16x4_v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + off1));
    union { struct { s16x4_v a, b; } s; bf16x8_v v; } u;
    u.s.a = lo;
    u.s.b = hi;
    return u.v;
  }
}


// Byte offset of 16-byte chunk `chunk16` (8 values) of k-row `krow` inside an NC slab (256-byte rows).
__device__ __forceinline__ int nc_offset(int krow, int chunk16) {
  return krow * 256 + ((((chunk16 >> 1) ^ ((krow & 3) << 1)) << 5) | ((chunk16 & 1) << 4));
}

}  // namespace dmoe
