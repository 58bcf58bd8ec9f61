// Block-sparse matrix products of the two-layer expert FFN on bf16 MFMA with fp32 accumulation (Section 5.1):
//
//   SDD    H  = Xp  W1          sampled on the nonzero blocks, epilogue A = gelu(H)       (forward, layer 1)
//   DSD    Yp = A   W2          sparse lhs iterated through blocked CSR                   (forward, layer 2)
//   SDD^T  dA = dYp W2^T        sampled on the nonzero blocks, epilogue dH = dA gelu'(H)  (layer-2 data gradient)
//   DS^TD  dW2 = A^T dYp        sparse lhs iterated through the transpose indices         (layer-2 weight gradient)
//   DSD^T  dXp = dH W1^T                                                                  (layer-1 data gradient)
//   DD^TS  dW1 = Xp^T dH        sparse rhs iterated through the transpose indices         (layer-1 weight gradient)
//
// Block size 128x128 (Section 5.1.2); values of block b (primary, row-wise order) are a contiguous row-major
// 128x128 bf16 tile at offset b*16384.  SDD-type kernels find their block through row_indices/column_indices
// (the COO half of the hybrid encoding, Section 5.1.3); DSD-type kernels walk row_offsets/column_indices;
// the weight-gradient kernels walk column_offsets_t/row_indices_t/block_offsets_t (Section 5.1.4).
//
// One workgroup = 4 waves = one 128x128 output tile, K advanced 64 at a time through double-buffered LDS.
// Each wave owns a 64x64 quadrant as 2x2 v_mfma_f32_32x32x16_bf16 tiles.  An operand whose K index is
// contiguous in memory is staged as [row][64 k] and read with ds_read_b128; an operand whose K index is the
// strided one is staged as it lies in memory, [k][128], and read with the transposing ds_read_b64_tr_b16, so
// no operand is ever transposed in HBM or in registers.  Both stagings are XOR-swizzled instead of padded.
#include "common.h"

namespace dmoe {

constexpr int kBK = 64;                       // K per pipeline stage
constexpr int kTileBytes = 16384;             // 128 x 64 bf16 either way round
constexpr int kBlockElems = kBlock * kBlock;  // 16384 values per sparse block

enum Layout { KC = 0, NC = 1 };               // KC: [row][k] k-contiguous;  NC: [k][row] row-contiguous

struct BsParams {
  const bf16_t* dense_a;
  const bf16_t* dense_b;
  const bf16_t* sparse_in;
  bf16_t* out0;
  bf16_t* out1;
  const int32_t* row_offsets;
  const int32_t* column_indices;
  const int32_t* row_indices;
  const int32_t* column_offsets_t;
  const int32_t* row_indices_t;
  const int32_t* block_offsets_t;
  const int32_t* counts;
  const int32_t* expert_order;
  int d, h, E, hb, db;
};

template <int OP> struct OpLayouts;
template <> struct OpLayouts<OP_SDD>  { static constexpr int A = KC, B = NC; };
template <> struct OpLayouts<OP_DSD>  { static constexpr int A = KC, B = NC; };
template <> struct OpLayouts<OP_SDDT> { static constexpr int A = KC, B = KC; };
template <> struct OpLayouts<OP_DSTD> { static constexpr int A = NC, B = NC; };
template <> struct OpLayouts<OP_DSDT> { static constexpr int A = KC, B = KC; };
template <> struct OpLayouts<OP_DDTS> { static constexpr int A = NC, B = NC; };

// ---- LDS addressing -------------------------------------------------------------------------------------------
// KC tile: 128 rows x 128 bytes.  16-byte chunk c of row r sits at chunk c ^ ((r >> 1) & 7): the 16 lanes that a
// ds_read_b128 serves per clock (16 consecutive rows, same logical chunk) then cover all 64 banks once.
__device__ __forceinline__ int kc_offset(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }
// NC tile: 64 k-rows x 256 bytes.  32-byte unit u of k-row k sits at unit u ^ (2 * (k & 3)): the 32 lanes that a
// ds_read_b64_tr_b16 serves per clock (4 k-rows x two adjacent units) then cover all 64 banks once.
__device__ __forceinline__ int nc_offset(int krow, int chunk16) {
  return krow * 256 + ((((chunk16 >> 1) ^ ((krow & 3) << 1)) << 5) | ((chunk16 & 1) << 4));
}

template <int L>
__device__ __forceinline__ void global_to_regs(uint4 (&regs)[4], const bf16_t* __restrict__ base, size_t ld, int tid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = tid + 256 * i;
    const int row = L == KC ? (q >> 3) : (q >> 4);
    const int c = L == KC ? (q & 7) : (q & 15);
    regs[i] = *reinterpret_cast<const uint4*>(base + (size_t)row * ld + c * 8);
  }
}
template <int L>
__device__ __forceinline__ void regs_to_lds(const uint4 (&regs)[4], char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = tid + 256 * i;
    const int off = L == KC ? kc_offset(q >> 3, q & 7) : nc_offset(q >> 4, q & 15);
    *reinterpret_cast<uint4*>(lds + off) = regs[i];
  }
}

typedef __attribute__((address_space(3))) s16x4_v* lds_s16x4_ptr;

// MFMA operand for the 32 rows starting at `row0` of the tile and K step ks (16 k): lane l gets row row0 + l%32
// and the 8 consecutive k = 16 ks + 8 (l / 32) + 0..7, whichever way round the tile is staged.
template <int L>
__device__ __forceinline__ bf16x8_v load_frag(const char* lds, int row0, int ks, int lane) {
  if constexpr (L == KC) {
    const int row = row0 + (lane & 31);
    return *reinterpret_cast<const bf16x8_v*>(lds + kc_offset(row, 2 * ks + (lane >> 5)));
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

// Workgroup index -> tile index.  Workgroups are handed to the 8 XCDs round-robin; this gives each XCD a
// contiguous run of tiles so that tiles sharing operands meet in the same L2.
__device__ __forceinline__ int xcd_remap(int wg, int total) {
  const int per = total >> 3;
  if (wg >= (per << 3)) return wg;                 // ragged tail (and workgroups beyond `total`) keep their index
  return (wg & 7) * per + (wg >> 3);
}

template <int OP>
__global__ void __launch_bounds__(256, 2) bsmm_kernel(const BsParams p) {
  constexpr int LA = OpLayouts<OP>::A, LB = OpLayouts<OP>::B;
  __shared__ __attribute__((aligned(16))) char lds[2][2][kTileBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int d = p.d, hb = p.hb, db = p.db;
  const size_t ldw = (size_t)p.E * p.h;            // leading dimension of W1 / dW1

  // ---- which tile ----------------------------------------------------------------------------------------
  int nk = 0, first = 0, r = 0, c = 0, j = 0;
  if constexpr (OP == OP_SDD || OP == OP_SDDT) {
    const int nnz = p.counts[2];
    if ((int)blockIdx.x >= nnz) return;
    const int b = xcd_remap(blockIdx.x, nnz);
    first = b;
    r = p.row_indices[b];
    c = p.column_indices[b];
    nk = d / kBK;
  } else if constexpr (OP == OP_DSD || OP == OP_DSDT) {
    const int tiles = p.counts[1] * db;
    if ((int)blockIdx.x >= tiles) return;
    const int wg = xcd_remap(blockIdx.x, tiles);
    r = wg / db;
    j = wg % db;
    first = p.row_offsets[r];
    nk = 2 * (p.row_offsets[r + 1] - first);
  } else {
    const int wg = blockIdx.x;
    const int cs = wg / db;
    j = wg % db;
    const int e = p.expert_order[cs / hb];         // heaviest experts first
    c = e * hb + cs % hb;
    first = p.column_offsets_t[c];
    nk = 2 * (p.column_offsets_t[c + 1] - first);
  }

  const bf16_t* a_ptr;
  const bf16_t* b_ptr;
  size_t lda, ldb;
  auto tile_ptrs = [&](int kt) {
    if constexpr (OP == OP_SDD) {
      a_ptr = p.dense_a + (size_t)r * kBlock * d + kt * kBK;  lda = d;
      b_ptr = p.dense_b + (size_t)kt * kBK * ldw + (size_t)c * kBlock;  ldb = ldw;
    } else if constexpr (OP == OP_SDDT) {
      a_ptr = p.dense_a + (size_t)r * kBlock * d + kt * kBK;  lda = d;
      b_ptr = p.dense_b + (size_t)c * kBlock * d + kt * kBK;  ldb = d;
    } else if constexpr (OP == OP_DSD) {
      const int blk = first + (kt >> 1), half = kt & 1;
      const int col = p.column_indices[blk];
      a_ptr = p.sparse_in + (size_t)blk * kBlockElems + half * kBK;  lda = kBlock;
      b_ptr = p.dense_b + ((size_t)col * kBlock + half * kBK) * d + j * kBlock;  ldb = d;
    } else if constexpr (OP == OP_DSDT) {
      const int blk = first + (kt >> 1), half = kt & 1;
      const int col = p.column_indices[blk];
      a_ptr = p.sparse_in + (size_t)blk * kBlockElems + half * kBK;  lda = kBlock;
      b_ptr = p.dense_b + (size_t)j * kBlock * ldw + (size_t)col * kBlock + half * kBK;  ldb = ldw;
    } else if constexpr (OP == OP_DSTD) {
      const int i = first + (kt >> 1), half = kt & 1;
      const int blk = p.block_offsets_t[i], row = p.row_indices_t[i];
      a_ptr = p.sparse_in + (size_t)blk * kBlockElems + half * kBK * kBlock;  lda = kBlock;
      b_ptr = p.dense_a + ((size_t)row * kBlock + half * kBK) * d + j * kBlock;  ldb = d;
    } else {  // OP_DDTS
      const int i = first + (kt >> 1), half = kt & 1;
      const int blk = p.block_offsets_t[i], row = p.row_indices_t[i];
      a_ptr = p.dense_a + ((size_t)row * kBlock + half * kBK) * d + j * kBlock;  lda = d;
      b_ptr = p.sparse_in + (size_t)blk * kBlockElems + half * kBK * kBlock;  ldb = kBlock;
    }
  };

  f32x16_v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][jj][q] = 0.0f;

  uint4 ra[4], rb[4];
  if (nk > 0) {
    tile_ptrs(0);
    global_to_regs<LA>(ra, a_ptr, lda, tid);
    global_to_regs<LB>(rb, b_ptr, ldb, tid);
    regs_to_lds<LA>(ra, lds[0][0], tid);
    regs_to_lds<LB>(rb, lds[0][1], tid);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) {
      tile_ptrs(kt + 1);
      global_to_regs<LA>(ra, a_ptr, lda, tid);
      global_to_regs<LB>(rb, b_ptr, ldb, tid);
    }
    const char* sa = lds[cur][0];
    const char* sb = lds[cur][1];
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8_v af[2], bf[2];
      af[0] = load_frag<LA>(sa, wm * 64, ks, lane);
      af[1] = load_frag<LA>(sa, wm * 64 + 32, ks, lane);
      bf[0] = load_frag<LB>(sb, wn * 64, ks, lane);
      bf[1] = load_frag<LB>(sb, wn * 64 + 32, ks, lane);
      // Operands swapped on purpose: the MFMA "row" index runs over n and the "column" index over m, so each lane
      // ends up with four consecutive n of one output row and can store them as one 8-byte word.
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[jj], af[i], acc[i][jj], 0, 0, 0);
    }
    if (more) {
      regs_to_lds<LA>(ra, lds[cur ^ 1][0], tid);
      regs_to_lds<LB>(rb, lds[cur ^ 1][1], tid);
    }
    __syncthreads();
  }

  // ---- epilogue: lane l, accumulator register 4q+u of tile (i, jj) is
  //      C[wm*64 + 32 i + l%32][wn*64 + 32 jj + 8 q + 4 (l/32) + u]
  bf16_t* out;
  size_t ldo;
  if constexpr (OP == OP_SDD || OP == OP_SDDT) {
    out = p.out0 + (size_t)first * kBlockElems;  ldo = kBlock;
  } else if constexpr (OP == OP_DSD || OP == OP_DSDT) {
    out = p.out0 + (size_t)r * kBlock * d + j * kBlock;  ldo = d;
  } else if constexpr (OP == OP_DSTD) {
    out = p.out0 + (size_t)c * kBlock * d + j * kBlock;  ldo = d;
  } else {
    out = p.out0 + (size_t)j * kBlock * ldw + (size_t)c * kBlock;  ldo = ldw;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = wm * 64 + 32 * i + (lane & 31);
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn * 64 + 32 * jj + 8 * q + 4 * (lane >> 5);
        const float v0 = acc[i][jj][4 * q + 0], v1 = acc[i][jj][4 * q + 1];
        const float v2 = acc[i][jj][4 * q + 2], v3 = acc[i][jj][4 * q + 3];
        const size_t o = (size_t)m * ldo + n;
        if constexpr (OP == OP_SDD) {
          uint2 hv, av;
          hv.x = pack_bf16(v0, v1);  hv.y = pack_bf16(v2, v3);
          av.x = pack_bf16(gelu_fwd(v0), gelu_fwd(v1));  av.y = pack_bf16(gelu_fwd(v2), gelu_fwd(v3));
          *reinterpret_cast<uint2*>(out + o) = hv;
          *reinterpret_cast<uint2*>(p.out1 + (size_t)first * kBlockElems + o) = av;
        } else if constexpr (OP == OP_SDDT) {
          const uint2 hv = *reinterpret_cast<const uint2*>(p.sparse_in + (size_t)first * kBlockElems + o);
          uint2 gv;
          gv.x = pack_bf16(v0 * gelu_bwd(bf16_lo(hv.x)), v1 * gelu_bwd(bf16_hi(hv.x)));
          gv.y = pack_bf16(v2 * gelu_bwd(bf16_lo(hv.y)), v3 * gelu_bwd(bf16_hi(hv.y)));
          *reinterpret_cast<uint2*>(out + o) = gv;
        } else {
          uint2 ov;
          ov.x = pack_bf16(v0, v1);  ov.y = pack_bf16(v2, v3);
          *reinterpret_cast<uint2*>(out + o) = ov;
        }
      }
    }
  }
}

void launch_bsmm(BsOp op, const BsArgs& a, hipStream_t s) {
  BsParams p;
  p.dense_a = a.dense_a;  p.dense_b = a.dense_b;  p.sparse_in = a.sparse_in;
  p.out0 = a.out0;  p.out1 = a.out1;
  const dmoe_topology_t& t = *a.topo;
  p.row_offsets = t.row_offsets;  p.column_indices = t.column_indices;  p.row_indices = t.row_indices;
  p.column_offsets_t = t.column_offsets_t;  p.row_indices_t = t.row_indices_t;  p.block_offsets_t = t.block_offsets_t;
  p.counts = t.counts;  p.expert_order = t.expert_order;
  p.d = a.d;  p.h = a.h;  p.E = a.E;  p.hb = a.h / kBlock;  p.db = a.d / kBlock;
  switch (op) {
    case OP_SDD:  hipLaunchKernelGGL(bsmm_kernel<OP_SDD>,  dim3(a.nnz_max), dim3(256), 0, s, p); break;
    case OP_SDDT: hipLaunchKernelGGL(bsmm_kernel<OP_SDDT>, dim3(a.nnz_max), dim3(256), 0, s, p); break;
    case OP_DSD:  hipLaunchKernelGGL(bsmm_kernel<OP_DSD>,  dim3(a.r_max * p.db), dim3(256), 0, s, p); break;
    case OP_DSDT: hipLaunchKernelGGL(bsmm_kernel<OP_DSDT>, dim3(a.r_max * p.db), dim3(256), 0, s, p); break;
    case OP_DSTD: hipLaunchKernelGGL(bsmm_kernel<OP_DSTD>, dim3(a.E * p.hb * p.db), dim3(256), 0, s, p); break;
    case OP_DDTS: hipLaunchKernelGGL(bsmm_kernel<OP_DDTS>, dim3(a.E * p.hb * p.db), dim3(256), 0, s, p); break;
  }
}

}  // namespace dmoe
