// Block-sparse matrix products of the two-layer expert FFN on bf16 MFMA with fp32 accumulation (Section 5.1):
//
//   SDD    H  = Xp  W1          sampled on the nonzero blocks, epilogue A = gelu(H), G = gelu'(H)   (forward, layer 1)
//   DSD    Yp = A   W2          sparse lhs iterated through blocked CSR                   (forward, layer 2)
//   SDD^T  dA = dYp W2^T        sampled on the nonzero blocks, epilogue dH = dA * G       (layer-2 data gradient)
//   DS^TD  dW2 = A^T dYp        sparse lhs iterated through the transpose indices         (layer-2 weight gradient)
//   DSD^T  dXp = dH W1^T                                                                  (layer-1 data gradient)
//   DD^TS  dW1 = Xp^T dH        sparse rhs iterated through the transpose indices         (layer-1 weight gradient)
//
// Block size 128x128 (Section 5.1.2); values of block b (primary, row-wise order) are a contiguous row-major
// 128x128 bf16 tile at offset b*16384.  SDD-type kernels find their blocks through row_offsets/column_indices,
// DSD-type kernels walk row_offsets/column_indices along K, the weight-gradient kernels walk
// column_offsets_t/row_indices_t/block_offsets_t (Section 5.1.4) along K.
//
// Tiling.  A 128x128 tile moves one operand byte per 64 flops, which on this chip saturates the L2->CU path
// long before the MFMA pipes.  One workgroup (8 waves) therefore owns a 256x256 MACRO tile = 2x2 sparse
// blocks: two "A panels" of 128 rows and two "B panels" of 128 columns, each panel an independent
// 128x64 (K-contiguous) or 64x128 (K-strided) slab with its own base pointer, so that a macro tile can be
// two block-rows of one expert times two block-columns, whichever operand is the sparse one.  A missing
// panel (odd number of block-rows in an expert, odd h/128 or d/128) is simply skipped by the waves that own it.
// K advances 64 at a time through two LDS stages filled by direct global->LDS loads (global_load_lds_dwordx4),
// so operands never pass through registers on their way in.  Each wave computes 128x64 of the macro tile as
// 4x2 v_mfma_f32_32x32x16_bf16 tiles.  K-contiguous slabs are read with ds_read_b128, K-strided slabs as they
// lie in memory with the transposing ds_read_b64_tr_b16; both are XOR-swizzled instead of padded.
#include "common.h"
#include "mma_tile.h"
#include <mutex>

namespace dmoe {

// K per pipeline stage (BK) and number of LDS stages (NS) are template parameters of the kernel:
// a slab is 128 x BK bf16 = 256*BK bytes either way round, a stage is four slabs (A0 A1 B0 B1).
constexpr int kBlockElems = kBlock * kBlock;  // 16384 values per sparse block
constexpr int kPatch = 32;                    // macro tiles that should run together on one XCD (one per CU)
constexpr int kMaxGradGrid = 8192;            // cap on the grid of a weight-gradient launch (multiple of 8 * kPatch)
constexpr int kPersistGrid = 256;             // workgroups of a persistent launch: one per CU (a multiple of 8 * kPatch)
constexpr int kPatchSlack = 5;                // tolerated XCD imbalance, in 64ths, when the patch size is chosen

struct BsParams {
  const bf16_t* dense_a;
  const bf16_t* dense_b;
  const bf16_t* sparse_in;
  bf16_t* out0;
  bf16_t* out1;
  const int32_t* row_offsets;
  const int32_t* column_indices;
  const int32_t* row_indices;         // block-row of every nonzero block (the COO half of the encoding, Section 5.1.3)
  const int32_t* column_offsets_t;
  const int32_t* row_indices_t;
  const int32_t* block_offsets_t;
  const int32_t* group_offsets;
  const int32_t* row_group;
  const int32_t* expert_order;
  const int32_t* counts;
  const int32_t* sched;
  const int32_t* tokens_per_expert;   // dMoE topologies only (NULL for a general mask): lets the weight gradients skip padding
  const int32_t* token_of;            // dMoE topologies only: tells a block row whose second half is all padding (a fringe)
  int d, h, E, hb, db;
  int force_tile;          // 0: device-side choice for the weight gradients, 1: 128x128, 2: 256x256, 3: 256x256 on two stages
  int patch;               // > 0: tiles per XCD patch (see patch_item); <= 0: balanced_patch with slack -patch
  int items;               // work items of this launch (weight gradients: may exceed the grid)
  int plain;               // 1: SDD / SDD^T without their fused epilogues (general block-sparse products)
  int accum;               // 1: weight gradients are added, in fp32, to the fp32 matrix that out0 then points to
  int ka;                  // DDS: leading dimension of dense_a
  int coo;                 // 1: SDD / SDD^T take one nonzero block per workgroup, found through row_indices
  int dual;                // 1: DSD / DSD^T were launched in both tile shapes; sched[2] says which one works
  long long* trace;        // optional (NULL = off): per work item, four 100 MHz time stamps and the K tile count
  int trace_cap;           // work items the trace buffer has room for
};

template <int OP> struct OpLayouts;
template <> struct OpLayouts<OP_SDD>  { static constexpr int A = KC, B = NC; };
template <> struct OpLayouts<OP_DSD>  { static constexpr int A = KC, B = NC; };
template <> struct OpLayouts<OP_SDDT> { static constexpr int A = KC, B = KC; };
template <> struct OpLayouts<OP_DSTD> { static constexpr int A = NC, B = NC; };
template <> struct OpLayouts<OP_DSDT> { static constexpr int A = KC, B = KC; };
template <> struct OpLayouts<OP_DDTS> { static constexpr int A = NC, B = NC; };
template <> struct OpLayouts<OP_DDS>  { static constexpr int A = KC, B = NC; };
template <> struct OpLayouts<OP_SDTD>  { static constexpr int A = NC, B = NC; };   // S = X^T W    (X given as [D, M])
template <> struct OpLayouts<OP_SDTDT> { static constexpr int A = NC, B = KC; };   // S = X^T W^T
template <> struct OpLayouts<OP_DSTDT> { static constexpr int A = NC, B = KC; };   // Y = S^T X^T  (X given as [D, M])
template <> struct OpLayouts<OP_DDST>  { static constexpr int A = KC, B = KC; };   // Y = X S^T    (S walked by rows)
template <> struct OpLayouts<OP_DDTST> { static constexpr int A = NC, B = KC; };   // Y = X^T S^T  (X given as [N, D])

// Workgroups are handed to the 8 XCDs round-robin (workgroup w runs on XCD w % 8).  Work items are cut into
// patches of P consecutive items that share operands; patch p goes to XCD p % 8, so the items of a patch run
// side by side on the CUs behind one L2 (P = 32: one per CU).  P = 1 deals the items out one by one.
__device__ __forceinline__ int patch_item(int wg, int P) {
  const int xcd = wg & 7, slot = wg >> 3;
  return ((slot / P) * 8 + xcd) * P + slot % P;
}

// Patch size for `items` equally expensive tiles: the assignment of patches to XCDs is static, so with few patches
// some XCDs get a whole patch more than others.  Take the largest power of two up to 32 whose most loaded XCD
// carries at most `slack`/64 more than the best of them.
__device__ __forceinline__ int balanced_patch(int items, int slack) {
  int load[6], best = 0x7fffffff;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    const int P = 32 >> i;
    load[i] = (((items + P - 1) / P + 7) / 8) * P;
    best = load[i] < best ? load[i] : best;
  }
  int P = 1;
#pragma unroll
  for (int i = 5; i >= 0; --i)
    if (64 * load[i] <= (64 + slack) * best) P = 32 >> i;
  return P;
}

// PA, PB = number of 128-row A panels and 128-column B panels of the tile:
//   2,2 -> the 256x256 macro tile (each of 8 waves 128x64; or 16 waves of 64x64), two LDS stages;
//   2,1 -> 256x128 (each wave 64x64), three LDS stages;
//   1,1 -> a single 128x128 block shared by eight waves (32x64 each), two or more workgroups per CU: half the
//          arithmetic intensity but four times as many work items, for under-filled launches.
// One work item of a launch: which blocks of the macro tile exist, where their operands start, how long K is.
struct TileState {
  bool a_ok1, b_ok1;               // the second A panel / B panel of the tile exists (the first always does)
  int nk;                          // K tiles
  int r0, r1, first0, first1, c0, c1, jd0;
  int ix0, ix1, ix2;               // lane-distributed topology indices of the K loop (see refill)
  int live;                        // 128, or 64 when rows 64..127 of the tile's block row are padding (one-block-row tiles)
};

template <int OP, int PA, int PB, int NS, int NW, int BK = 64, int ACT = 0>
__global__ void __launch_bounds__(NW * 64, (8 * PA * PB / NW) >= 4 ? 2 : 4) bsmm_kernel(const BsParams p) {
  constexpr int LA = OpLayouts<OP>::A, LB = OpLayouts<OP>::B;
  constexpr int kSub = kBlock / BK;                 // K tiles per 128-wide sparse block
  constexpr int kPanelBytes = 256 * BK;             // one 128 x 64 bf16 slab, either way round
  constexpr int kStageBytes = (PA + PB) * kPanelBytes;
  constexpr int kCpw = (BK / 4) / NW;               // 1 KB DMA chunks per wave per slab (a slab has BK / 4)
  static_assert(kCpw >= 1, "a slab must have at least one chunk per wave");
  constexpr int kDmaPerTile = (PA + PB) * kCpw;     // DMA instructions per wave per K tile
  // 32-row MFMA tiles per wave (a wave is always 64 columns wide): 8 waves on 2x2 blocks -> 128x64 per wave,
  // 16 waves on 2x2 blocks -> 64x64 per wave (four waves per SIMD), 8 waves on one block -> 32x64 per wave.
  constexpr int WB = NW / (PA * PB);                // waves per 128x128 block of the tile
  constexpr int MI = 8 / WB;
  static_assert(WB == 2 || WB == 4 || WB == 8, "unsupported tile / workgroup shape");
  constexpr bool kSparseOut = OP == OP_SDD || OP == OP_SDDT || OP == OP_SDTD || OP == OP_SDTDT;
  constexpr bool kRowsInB = OP == OP_DDST || OP == OP_DDTST;   // dense x sparse^T: the block rows of S are the B panel
  constexpr bool kRowMajor = kSparseOut || OP == OP_DSD || OP == OP_DSDT || kRowsInB;   // items enumerate block rows
  static_assert(OP < OP_SDTD || PA * PB == 1, "the products beyond the layer's run one 128x128 block per workgroup");
  // The 256x256 tiles of the token-row products run as a persistent, software-pipelined loop over the items of a
  // workgroup (see the end of the kernel); everything else takes one item at a time.
  constexpr bool kPipe = kRowMajor && PA == 2 && PB == 2 && NS == 2 && NW == 8;
  // The same loop over a slab ring: three stages for the A slabs, two for the B slabs (160 KB, all of LDS).  The A
  // slabs of a K tile are requested two tiles ahead and the B slabs one, so 96 KB instead of 64 KB are in flight.
  constexpr bool kRing = kRowMajor && PA == 2 && PB == 2 && NS == 3 && NW == 8;
  // tiles of one block row of the token-row products of the layer skip the padding half of a fringe block row
  constexpr bool kFringe = kRowMajor && PA == 1 && NS == 2 && NW == 8 && BK == 64 && OP <= OP_DDTS;
  constexpr int kEpRows = MI >= 2 ? 64 : 32;        // rows of the wave's tile that pass through its staging tile at a time
  constexpr int kEpBytes = kEpRows * 128;           // per wave: 8 KB (4 KB for the 32-row waves)
  extern __shared__ __attribute__((aligned(1024))) char lds[];   // [NS stages][A slabs, B slabs]

  const int tid = threadIdx.x;
  // the wave number is the same for all lanes: saying so keeps everything derived from it in scalar registers
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wq = wave / WB;                         // which 128x128 block of the tile: A panel pm, B panel pn
  const int pm = wq / PB, pn = wq % PB;
  const int arow0 = ((wave % WB) >> 1) * (32 * MI);  // first row of the wave inside its A panel
  const int hn = wave & 1;                          // which 64-column half of the B panel
  const int d = p.d, hb = p.hb, db = p.db;
  const size_t ldw = (size_t)p.E * p.h;             // leading dimension of W1 / dW1
  // Which dimension the A panels and the B panels span: rows x block-columns (SDD, SDD^T), rows x d-blocks (DSD,
  // DSD^T), block-columns x d-blocks (DS^TD), d-blocks x block-columns (DD^TS).
  constexpr bool kColsInB = OP == OP_DDTS || OP == OP_DDS;      // dense x sparse: the block-columns are the B panels
  constexpr int UC = (kSparseOut || kColsInB) ? PB : PA;        // block-columns per unit (where columns matter)
  constexpr int UD = kColsInB ? PA : PB;                        // d-blocks per unit
  const int ncu = (hb + UC - 1) / UC, nju = (db + UD - 1) / UD;

  // ---- which tile ------------------------------------------------------------------------------------------
  // Items are numbered so that 4 consecutive "major" indices (row units, or column units for the weight
  // gradients) times all "minor" indices form a run: id = (major / 4 * nminor + minor) * 4 + major % 4.
  // Returns false when the item does not exist for this routing (grids are sized for upper bounds).
  const bool coo_launch = kSparseOut && PA * PB == 1 && p.coo;
  const int nminor = coo_launch ? 1 : kSparseOut ? ncu : nju;
  int majors_live = 0, patch = 1;
  if constexpr (kRowMajor) {
    majors_live = coo_launch ? p.counts[2] : PA == 2 ? p.group_offsets[p.E] : p.counts[1];
    patch = p.patch > 0 ? p.patch : balanced_patch((majors_live + 3) / 4 * 4 * nminor, -p.patch);
  } else {
    patch = p.sched[1];                             // 1 or 16, chosen with the routing in hand (offsets_kernel)
  }
  auto decode = [&](const int wgi, TileState& t) -> bool {
    const int item = patch_item(wgi, patch);
    const int run = item / (4 * nminor), rem = item % (4 * nminor);
    const int major = run * 4 + (rem & 3), minor = rem >> 2;
    t.a_ok1 = false;  t.b_ok1 = false;
    t.nk = 0;  t.r0 = t.r1 = t.first0 = t.first1 = t.c0 = t.c1 = t.jd0 = 0;
    t.ix0 = t.ix1 = t.ix2 = 0;
    t.live = kBlock;
    if constexpr (kRowMajor) {
      if (major >= majors_live) return false;
      if (coo_launch) {
        // A general mask may have any number of blocks in a row; the per-block row index of the hybrid encoding lets
        // SDD give every nonzero block its own workgroup without searching the row offsets (Section 5.1.3).
        t.first0 = t.first1 = major;
        t.r0 = t.r1 = p.row_indices[major];
        t.c0 = t.c1 = p.column_indices[major];
        t.nk = d / BK;
        return true;
      }
      if constexpr (PA == 2) {
        const int rg = p.row_group[major];            // first block-row * 2 + (group has a second row)
        t.r0 = rg >> 1;
        t.a_ok1 = rg & 1;
      } else {
        t.r0 = major;
        // Partial fringe blocks (Section 5.2 pads every expert to whole blocks; Section 6.2 notes the cost at small
        // batches): when the last block row of an expert holds at most 64 tokens, rows 64..127 are padding.  Nothing
        // downstream reads them -- the gathers go through row_of, and the weight gradients skip K tiles of 64 rows
        // that lie wholly in padding -- so a tile of one block row neither loads, multiplies nor writes that half.
        if constexpr (kFringe) {
          if (p.token_of && p.token_of[(size_t)major * kBlock + 64] < 0) t.live = 64;
        }
      }
      t.r1 = t.a_ok1 ? t.r0 + 1 : t.r0;
      t.first0 = p.row_offsets[t.r0];
      t.first1 = p.row_offsets[t.r1];
      const int nblk = p.row_offsets[t.r0 + 1] - t.first0;
      if constexpr (kSparseOut) {
        if (PB * minor >= nblk) return false;
        t.b_ok1 = PB == 2 && 2 * minor + 1 < nblk;
        t.first0 += PB * minor;                       // block (r0, c0); (r0, c1) is the next one
        t.first1 += PB * minor;
        t.c0 = p.column_indices[t.first0];
        t.c1 = t.b_ok1 ? p.column_indices[t.first0 + 1] : t.c0;
        t.nk = d / BK;
      } else {
        t.jd0 = PB * minor;
        t.b_ok1 = PB == 2 && t.jd0 + 1 < db;
        t.nk = kSub * nblk;
      }
      return true;
    } else {
      if (major >= p.E * ncu) return false;
      // heaviest experts first; with patches, consecutive experts go to consecutive XCDs, so every second group of
      // eight is taken in reverse (the XCD that got the heaviest of one group gets the lightest of the next)
      int rank = major / ncu;
      if (patch > 1 && (rank & 8) && (rank | 7) < p.E) rank = (rank & ~7) | (7 - (rank & 7));
      const int e = p.expert_order[rank];
      const int cu = major % ncu;
      t.jd0 = UD * minor;
      t.c0 = e * hb + UC * cu;
      const bool second_col = UC == 2 && 2 * cu + 1 < hb;
      const bool second_d = UD == 2 && t.jd0 + 1 < db;
      t.c1 = second_col ? t.c0 + 1 : t.c0;
      t.first0 = p.column_offsets_t[t.c0];
      t.first1 = p.column_offsets_t[t.c1];
      t.nk = kSub * (p.column_offsets_t[t.c0 + 1] - t.first0);
      // The rows of an expert beyond its token count are padding (Section 5.2): zero in both operands of a weight
      // gradient, so K tiles that lie entirely in the padding of the last block are skipped.
      if (p.tokens_per_expert) t.nk = min(t.nk, (p.tokens_per_expert[e] + BK - 1) / BK);
      if constexpr (OP == OP_DSTD || OP == OP_DSTDT) { t.a_ok1 = second_col;  t.b_ok1 = second_d; }
      else                         { t.a_ok1 = second_d;    t.b_ok1 = second_col; }
      return true;
    }
  };

  // ---- per-K-tile slab base pointers (wave-uniform) --------------------------------------------------------
  const bf16_t *a0, *a1, *b0, *b1;
  uint32_t lda, ldb;
  if constexpr (OP == OP_SDD)       { lda = d;      ldb = (uint32_t)ldw; }
  else if constexpr (OP == OP_SDDT) { lda = d;      ldb = d; }
  else if constexpr (OP == OP_DSD)  { lda = kBlock; ldb = d; }
  else if constexpr (OP == OP_DSDT) { lda = kBlock; ldb = (uint32_t)ldw; }
  else if constexpr (OP == OP_DSTD) { lda = kBlock; ldb = d; }
  else if constexpr (OP == OP_DDS)  { lda = (uint32_t)p.ka;  ldb = kBlock; }
  else if constexpr (OP == OP_SDTD)  { lda = (uint32_t)p.ka;  ldb = (uint32_t)ldw; }
  else if constexpr (OP == OP_SDTDT) { lda = (uint32_t)p.ka;  ldb = d; }
  else if constexpr (OP == OP_DSTDT) { lda = kBlock;  ldb = (uint32_t)p.ka; }
  else if constexpr (OP == OP_DDST)  { lda = (uint32_t)ldw;  ldb = kBlock; }
  else if constexpr (OP == OP_DDTST) { lda = d;  ldb = kBlock; }
  else                              { lda = d;      ldb = kBlock; }

  // The K loop of the products that walk the topology needs one to three index values per sparse block.  They are
  // kept lane-distributed in registers, 64 blocks at a time (lane i holds the values of block 64 c + i), and picked
  // out with v_readlane: an index load inside the loop would put its latency between the barrier and the loads
  // that the barrier releases, with every wave waiting.
  auto refill = [&](TileState& t, int kb0) {
    const int n = (t.nk + kSub - 1) / kSub - kb0;   // blocks left from kb0 on (the last one may be cut short)
    if (lane < n) {
      if constexpr (OP == OP_DSD || OP == OP_DSDT || kRowsInB) {
        t.ix0 = p.column_indices[t.first0 + kb0 + lane];
      } else if constexpr (OP == OP_DSTD || OP == OP_DDTS || OP == OP_DDS || OP == OP_DSTDT) {
        t.ix0 = p.block_offsets_t[t.first0 + kb0 + lane];
        t.ix1 = p.block_offsets_t[t.first1 + kb0 + lane];
        t.ix2 = p.row_indices_t[t.first0 + kb0 + lane];
      }
    }
    // consume the values here, so that the wait for these loads is placed inside this rarely taken branch and not
    // in front of the v_readlane of every iteration
    asm volatile("" : "+v"(t.ix0), "+v"(t.ix1), "+v"(t.ix2));
  };
  bool refill_ok = true;             // cleared around a second visit to a K tile whose indices are already in registers
  auto slab_ptrs = [&](TileState& t, int kt) {
    if constexpr (OP == OP_SDD) {
      a0 = p.dense_a + (size_t)t.r0 * kBlock * d + kt * BK;
      a1 = p.dense_a + (size_t)t.r1 * kBlock * d + kt * BK;
      b0 = p.dense_b + (size_t)kt * BK * ldw + (size_t)t.c0 * kBlock;
      b1 = p.dense_b + (size_t)kt * BK * ldw + (size_t)t.c1 * kBlock;
    } else if constexpr (OP == OP_SDDT) {
      a0 = p.dense_a + (size_t)t.r0 * kBlock * d + kt * BK;
      a1 = p.dense_a + (size_t)t.r1 * kBlock * d + kt * BK;
      b0 = p.dense_b + (size_t)t.c0 * kBlock * d + kt * BK;
      b1 = p.dense_b + (size_t)t.c1 * kBlock * d + kt * BK;
    } else if constexpr (OP == OP_SDTD || OP == OP_SDTDT) {
      // the left input is given transposed, [D, M]: its K index is the strided one
      a0 = p.dense_a + (size_t)kt * BK * lda + (size_t)t.r0 * kBlock;
      a1 = p.dense_a + (size_t)kt * BK * lda + (size_t)t.r1 * kBlock;
      if constexpr (OP == OP_SDTD) {
        b0 = p.dense_b + (size_t)kt * BK * ldw + (size_t)t.c0 * kBlock;
        b1 = p.dense_b + (size_t)kt * BK * ldw + (size_t)t.c1 * kBlock;
      } else {
        b0 = p.dense_b + (size_t)t.c0 * kBlock * d + kt * BK;
        b1 = p.dense_b + (size_t)t.c1 * kBlock * d + kt * BK;
      }
    } else if constexpr (kRowsInB) {
      // Y = X S^T (or X^T S^T): output block-column r is block-row r of S; its blocks (r, col), walked in the primary
      // order, are the B operand as they lie in memory ([n][k], k contiguous); X supplies the block-column col
      const int kb = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, kb);
      const int col = __builtin_amdgcn_readlane(t.ix0, kb & 63);
      if constexpr (OP == OP_DDST) a0 = p.dense_a + (size_t)t.jd0 * kBlock * lda + (size_t)col * kBlock + half * BK;
      else                         a0 = p.dense_a + ((size_t)col * kBlock + half * BK) * lda + (size_t)t.jd0 * kBlock;
      a1 = a0;
      b0 = p.sparse_in + (size_t)(t.first0 + kb) * kBlockElems + half * BK;
      b1 = b0;
    } else if constexpr (OP == OP_DSTDT) {
      // Y = S^T X^T with X given as [D, M]: as DS^TD, but the dense operand has its K index contiguous
      const int i = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, i);
      const int blk0 = __builtin_amdgcn_readlane(t.ix0, i & 63), blk1 = __builtin_amdgcn_readlane(t.ix1, i & 63);
      const int row = __builtin_amdgcn_readlane(t.ix2, i & 63);
      a0 = p.sparse_in + (size_t)blk0 * kBlockElems + half * BK * kBlock;
      a1 = p.sparse_in + (size_t)blk1 * kBlockElems + half * BK * kBlock;
      b0 = p.dense_a + (size_t)t.jd0 * kBlock * ldb + (size_t)row * kBlock + half * BK;
      b1 = b0;
    } else if constexpr (OP == OP_DSD) {
      const int kb = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, kb);
      const int col = __builtin_amdgcn_readlane(t.ix0, kb & 63);
      a0 = p.sparse_in + (size_t)(t.first0 + kb) * kBlockElems + half * BK;
      a1 = p.sparse_in + (size_t)(t.first1 + kb) * kBlockElems + half * BK;
      b0 = p.dense_b + ((size_t)col * kBlock + half * BK) * d + (size_t)t.jd0 * kBlock;
      b1 = b0 + (t.b_ok1 ? kBlock : 0);
    } else if constexpr (OP == OP_DSDT) {
      const int kb = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, kb);
      const int col = __builtin_amdgcn_readlane(t.ix0, kb & 63);
      a0 = p.sparse_in + (size_t)(t.first0 + kb) * kBlockElems + half * BK;
      a1 = p.sparse_in + (size_t)(t.first1 + kb) * kBlockElems + half * BK;
      b0 = p.dense_b + (size_t)t.jd0 * kBlock * ldw + (size_t)col * kBlock + half * BK;
      b1 = b0 + (t.b_ok1 ? (size_t)kBlock * ldw : 0);
    } else if constexpr (OP == OP_DSTD) {
      const int i = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, i);
      const int blk0 = __builtin_amdgcn_readlane(t.ix0, i & 63), blk1 = __builtin_amdgcn_readlane(t.ix1, i & 63);
      const int row = __builtin_amdgcn_readlane(t.ix2, i & 63);
      a0 = p.sparse_in + (size_t)blk0 * kBlockElems + half * BK * kBlock;
      a1 = p.sparse_in + (size_t)blk1 * kBlockElems + half * BK * kBlock;
      b0 = p.dense_a + ((size_t)row * kBlock + half * BK) * d + (size_t)t.jd0 * kBlock;
      b1 = b0 + (t.b_ok1 ? kBlock : 0);
    } else if constexpr (OP == OP_DDS) {
      // Y = X S: for the blocks (row, c) of column c, in the order of the transposed lists, X[:, row] times the block
      const int i = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, i);
      const int blk0 = __builtin_amdgcn_readlane(t.ix0, i & 63), blk1 = __builtin_amdgcn_readlane(t.ix1, i & 63);
      const int row = __builtin_amdgcn_readlane(t.ix2, i & 63);
      a0 = p.dense_a + (size_t)t.jd0 * kBlock * p.ka + (size_t)row * kBlock + half * BK;
      a1 = a0 + (t.a_ok1 ? (size_t)kBlock * p.ka : 0);
      b0 = p.sparse_in + (size_t)blk0 * kBlockElems + half * BK * kBlock;
      b1 = p.sparse_in + (size_t)blk1 * kBlockElems + half * BK * kBlock;
    } else {  // OP_DDTS
      const int i = kt / kSub, half = kt % kSub;
      if ((kt & (64 * kSub - 1)) == 0 && refill_ok) refill(t, i);
      const int blk0 = __builtin_amdgcn_readlane(t.ix0, i & 63), blk1 = __builtin_amdgcn_readlane(t.ix1, i & 63);
      const int row = __builtin_amdgcn_readlane(t.ix2, i & 63);
      a0 = p.dense_a + ((size_t)row * kBlock + half * BK) * d + (size_t)t.jd0 * kBlock;
      a1 = a0 + (t.a_ok1 ? kBlock : 0);
      b0 = p.sparse_in + (size_t)blk0 * kBlockElems + half * BK * kBlock;
      b1 = p.sparse_in + (size_t)blk1 * kBlockElems + half * BK * kBlock;
    }
  };

  // Each wave moves 1 KB chunk `wave` (and `wave + 8` when there are eight waves) of every slab.  All slabs are always loaded (a missing panel
  // re-reads its sibling): the number of loads per K tile must be a constant for the counted waits below.
  // A load takes the slab's base pointer from scalar registers (it is the same for the whole wave) and a per-lane
  // 32-bit byte offset from one vector register: against a 64-bit address per lane this halves the vector-register
  // reads of every load and removes the 64-bit vector additions that built the addresses inside the MFMA stream
  // (-11 % cycles per K tile in a dense probe of this loop).  Offsets stay below 2^32 bytes (127 rows of fewer than
  // 2^24 elements).
  uint32_t oa[kCpw], ob[kCpw];
#pragma unroll
  for (int i = 0; i < kCpw; ++i) {
    oa[i] = 2u * dma_lane_offset<LA, BK>(wave + NW * i, lane, lda);
    ob[i] = 2u * dma_lane_offset<LB, BK>(wave + NW * i, lane, ldb);
  }
  // The loads are written as inline assembly on purpose: the compiler's own wait-count insertion treats a
  // direct-to-LDS load as aliasing every later LDS read and would wait for it before the first ds_read of the
  // stage being computed, which serialises load latency and MFMA work.  Here the waits are explicit.
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)lds;
  auto dma16 = [](const bf16_t* base, uint32_t byte_off, uint32_t lds_addr) {
    // the base is the same for every lane; say so to the compiler where it cannot prove it (a no-op where it can)
    const uint64_t b64 = reinterpret_cast<uint64_t>(base);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32));
    base = reinterpret_cast<const bf16_t*>((static_cast<uint64_t>(hi) << 32) | lo);
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 : : "v"(byte_off), "s"(base), "s"(lds_addr) : "memory", "m0");
  };
  // part 0 = the A slabs, part 1 = the B slabs (issued at different points of the MFMA loop, see below)
  int live_rows = kBlock;            // rows of the (single) A panel that are loaded: 64 for a fringe block row
  auto issue_loads = [&](int stage, int part) {
    const uint32_t s = __builtin_amdgcn_readfirstlane(lds_base + stage * kStageBytes + wave * 1024);
#pragma unroll
    for (int i = 0; i < kCpw; ++i) {
      if (part == 0) {
        if (kFringe && i * NW * 8 >= 64 && live_rows <= 64) continue;      // chunk i holds rows 8 (wave + NW i) ...
        dma16(a0, oa[i], s + NW * 1024 * i);
        if (PA == 2) dma16(a1, oa[i], s + kPanelBytes + NW * 1024 * i);
      } else {
        dma16(b0, ob[i], s + PA * kPanelBytes + NW * 1024 * i);
        if (PB == 2) dma16(b1, ob[i], s + (PA + 1) * kPanelBytes + NW * 1024 * i);
      }
    }
  };

  f32x16_v acc[MI][2];
  auto clear_acc = [&]() {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][jj][q] = 0.0f;
  };

  struct Frags { bf16x8_v a[MI], b[2]; };
  auto read_frags = [&](Frags& f, const char* sa, const char* sb, int ks) {
#pragma unroll
    for (int i = 0; i < MI; ++i) f.a[i] = load_frag<LA, BK>(sa, arow0 + 32 * i, ks, lane);
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) f.b[jj] = load_frag<LB, BK>(sb, hn * 64 + 32 * jj, ks, lane);
  };
  // Operands swapped on purpose: the MFMA "row" index runs over n and the "column" index over m, so each
  // lane ends up with four consecutive n of one output row and can store them as one 8-byte word.
  auto mfma_frags = [&](const Frags& f) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
        acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[jj], f.a[i], acc[i][jj], 0, 0, 0);
  };
  auto multiply = [&](const char* sa, const char* sb, int ks) {
    Frags f;
    read_frags(f, sa, sb, ks);
    mfma_frags(f);
  };

  // ---- epilogue.  Lane l, accumulator register 4q+u of tile (i, jj) is
  //      C[arow0 + 32 i + l%32][hn*64 + 32 jj + 8 q + 4 (l/32) + u]  of this wave's 128x128 block (pm, pn).
  // Written straight from there, every store instruction would touch 32 rows with 16 bytes each; instead the
  // wave's tile is rounded to bf16 into a wave-private LDS staging tile (128-byte rows, chunk-swizzled like a
  // KC slab), kEpRows rows at a time, and written out as whole 128-byte row segments, 1 KB per store instruction.
  // `ep`: this wave's staging tile (kEpBytes; the accumulating form of the weight gradients uses 4 KB per 32 rows).
  const int lane_of_thread = lane;
  auto epilogue = [&](const TileState& t, char* ep) {
    // In a loop over items the per-lane addresses below would be computed once, ahead of the loop, spilled (the K loop
    // needs every register) and reloaded one by one between the stores, each reload waiting for every load and store
    // issued before it.  A lane number counted afresh (and opaque to the compiler) keeps them inside the epilogue.
    int lane = lane_of_thread;
    if constexpr (kRing) {
      lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
      asm volatile("" : "+v"(lane));
    }
    bf16_t* out;
    size_t ldo;
    size_t blk = 0;
    if constexpr (kSparseOut) {
      blk = (size_t)((pm ? t.first1 : t.first0) + pn) * kBlockElems + (size_t)arow0 * kBlock + hn * 64;
      out = p.out0 + blk;  ldo = kBlock;
    } else if constexpr (OP == OP_DSD || OP == OP_DSDT) {
      out = p.out0 + ((size_t)(pm ? t.r1 : t.r0) * kBlock + arow0) * d + (size_t)(t.jd0 + pn) * kBlock + hn * 64;  ldo = d;
    } else if constexpr (kRowsInB) {
      out = p.out0 + ((size_t)t.jd0 * kBlock + arow0) * p.ka + (size_t)t.r0 * kBlock + hn * 64;  ldo = p.ka;
    } else if constexpr (OP == OP_DSTD || OP == OP_DSTDT) {
      out = p.out0 + ((size_t)(pm ? t.c1 : t.c0) * kBlock + arow0) * d + (size_t)(t.jd0 + pn) * kBlock + hn * 64;  ldo = d;
    } else {
      out = p.out0 + ((size_t)(t.jd0 + pm) * kBlock + arow0) * ldw + (size_t)(pn ? t.c1 : t.c0) * kBlock + hn * 64;  ldo = ldw;
    }
    if constexpr (!kRowMajor) {
      if (p.accum) {
        // fp32 accumulation: out0 is an fp32 matrix of the same shape.  The staging tile holds 32 columns at a time
        // (128-byte rows again), so every load and store below covers whole 128-byte row segments.  The tile belongs
        // to this workgroup alone, so a plain read-modify-write is enough.
        float* outf = reinterpret_cast<float*>(p.out0) + (out - p.out0);
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              float4 v;
              v.x = acc[i][jj][4 * q + 0];  v.y = acc[i][jj][4 * q + 1];
              v.z = acc[i][jj][4 * q + 2];  v.w = acc[i][jj][4 * q + 3];
              *reinterpret_cast<float4*>(ep + kc_offset<64>(32 * i + (lane & 31), 2 * q + (lane >> 5))) = v;
            }
#pragma unroll 2                               // not fully: the hoisted addresses would cost registers in every variant
          for (int it = 0; it < 4 * MI; ++it) {
            const int row = 8 * it + (lane >> 3), chunk = lane & 7;
            const float4 v = *reinterpret_cast<const float4*>(ep + kc_offset<64>(row, chunk));
            float4* g = reinterpret_cast<float4*>(outf + (size_t)row * ldo + 32 * jj + chunk * 4);
            float4 o = *g;
            o.x += v.x;  o.y += v.y;  o.z += v.z;  o.w += v.w;
            *g = o;
          }
        }
        return;
      }
    }
    if constexpr (OP == OP_SDDT) {
      if (!p.plain) {
        // dH = dA * G with G = gelu'(H) kept by the forward pass.  G comes in by direct-to-LDS loads, 32 rows at a time
        // and two steps ahead of its use, straight into the wave's staging tile in the tile's own swizzled layout; the
        // product is formed in place and written out as whole 128-byte row segments.  No vector register carries G,
        // and the counted waits below let the stores of earlier steps stay in flight (loads and stores retire in
        // order): [G(i+1)] or [stores(i-1), G(i+1)] may be outstanding when G(i) is needed.
        constexpr int NH = kEpRows / 32;                         // 4 KB halves of the staging tile
        static_assert((MI == 4 && NH == 2) || (MI == 1 && NH == 1), "wait counts below are written for these shapes");
        const bf16_t* gsrc = p.sparse_in + blk;
        const uint32_t ep_lds = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_ptr)ep);
        const uint32_t off_even = 2u * dma_lane_offset<KC, 64>(0, lane, kBlock);
        const uint32_t off_odd = 2u * (dma_lane_offset<KC, 64>(1, lane, kBlock) - 8 * kBlock);
        auto fetch_g = [&](int i) {
#pragma unroll
          for (int ch = 0; ch < 4; ++ch)
            dma16(gsrc + (32 * i + 8 * ch) * kBlock, (ch & 1) ? off_odd : off_even, ep_lds + (i % NH) * 4096 + 1024 * ch);
        };
        fetch_g(0);
        if constexpr (MI > 1) fetch_g(1);
#pragma unroll
        for (int i = 0; i < MI; ++i) {
          const int il = i % NH;
          if constexpr (MI == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          else if (i == 0 || i == MI - 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
          else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              uint2* sl = reinterpret_cast<uint2*>(ep + kc_offset<64>(32 * il + (lane & 31), 4 * jj + q) + 8 * (lane >> 5));
              const uint2 gv = *sl;
              uint2 ov;
              ov.x = pack_bf16(acc[i][jj][4 * q + 0] * bf16_lo(gv.x), acc[i][jj][4 * q + 1] * bf16_hi(gv.x));
              ov.y = pack_bf16(acc[i][jj][4 * q + 2] * bf16_lo(gv.y), acc[i][jj][4 * q + 3] * bf16_hi(gv.y));
              *sl = ov;
            }
          bf16_t* dst = out + (size_t)(32 * i) * ldo;
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const int row = 8 * it + (lane >> 3), chunk = lane & 7;
            const uint4 v = *reinterpret_cast<const uint4*>(ep + kc_offset<64>(32 * il + row, chunk));
            *reinterpret_cast<uint4*>(dst + (size_t)row * ldo + chunk * 8) = v;
          }
          if (i + NH < MI) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");    // the reads of this half are done before it is refilled
            fetch_g(i + NH);
          }
        }
        return;
      }
    }
    constexpr int CH = kEpRows / 32;                             // 32-row MFMA tiles per pass through the staging tile
    auto slot = [&](int il, int jj, int q) -> uint2* {          // this lane's 4 values of tile (il, jj) of the pass, quad q
      return reinterpret_cast<uint2*>(ep + kc_offset<64>(32 * il + (lane & 31), 4 * jj + q) + 8 * (lane >> 5));
    };
    auto flush = [&](bf16_t* dst) {                             // staging tile -> global, row-contiguous
#pragma unroll
      for (int it = 0; it < 4 * CH; ++it) {
        const int row = 8 * it + (lane >> 3), chunk = lane & 7;
        const uint4 v = *reinterpret_cast<const uint4*>(ep + kc_offset<64>(row, chunk));
        *reinterpret_cast<uint4*>(dst + (size_t)row * ldo + chunk * 8) = v;
      }
    };
    // SDD writes two tensors from the same fp32 values: out1 <- A = gelu(H) = H Phi(H) for the second layer, and
    // out0 <- G = gelu'(H) = Phi(H) + H phi(H), which is all the backward pass needs of H (one evaluation of Phi and
    // phi serves both, and SDD^T then only multiplies).
    // (The form of the activation, ACT, is a template parameter: a run-time choice inside this loop made the compiler
    // evaluate both forms for every element, and one copy of the loop per form cost the 256x256 tile its registers.)
#pragma unroll
    for (int c = 0; c < MI / CH; ++c) {
      const size_t row_off = (size_t)(32 * CH * c) * ldo;
      if (OP == OP_SDDT && !p.plain) {                          // global -> staging tile: G = gelu'(H)
        const bf16_t* src = p.sparse_in + blk + row_off;
#pragma unroll
        for (int it = 0; it < 4 * CH; ++it) {
          const int row = 8 * it + (lane >> 3), chunk = lane & 7;
          *reinterpret_cast<uint4*>(ep + kc_offset<64>(row, chunk)) =
              *reinterpret_cast<const uint4*>(src + (size_t)row * ldo + chunk * 8);
        }
      }
#pragma unroll
      for (int il = 0; il < CH; ++il) {
        const int i = CH * c + il;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float v[4] = {acc[i][jj][4 * q + 0], acc[i][jj][4 * q + 1], acc[i][jj][4 * q + 2], acc[i][jj][4 * q + 3]};
            uint2 ov;
            if (OP == OP_SDDT && !p.plain) {
              const uint2 gv = *slot(il, jj, q);
              ov.x = pack_bf16(v[0] * bf16_lo(gv.x), v[1] * bf16_hi(gv.x));
              ov.y = pack_bf16(v[2] * bf16_lo(gv.y), v[3] * bf16_hi(gv.y));
            } else if (OP == OP_SDD && !p.plain) {
              float g[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                float cdf, pdf;
                if constexpr (ACT == 1) tanh_gelu_cdf_pdf(v[u], cdf, pdf);
                else                    normal_cdf_pdf(v[u], cdf, pdf);
                g[u] = fmaf(v[u], pdf, cdf);
                v[u] *= cdf;
                acc[i][jj][4 * q + u] = v[u];          // keep A for the second pass through the staging tile
              }
              ov.x = pack_bf16(g[0], g[1]);  ov.y = pack_bf16(g[2], g[3]);
            } else {
              ov.x = pack_bf16(v[0], v[1]);  ov.y = pack_bf16(v[2], v[3]);
            }
            *slot(il, jj, q) = ov;
          }
      }
      flush(out + row_off);
      if (OP == OP_SDD && !p.plain) {
#pragma unroll
        for (int il = 0; il < CH; ++il) {
          const int i = CH * c + il;
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              uint2 av;
              av.x = pack_bf16(acc[i][jj][4 * q + 0], acc[i][jj][4 * q + 1]);
              av.y = pack_bf16(acc[i][jj][4 * q + 2], acc[i][jj][4 * q + 3]);
              *slot(il, jj, q) = av;
            }
        }
        flush(p.out1 + blk + row_off);
      }
    }
  };

  // Optional trace (measurement aid): wave 0 of the workgroup stamps the 100 MHz wall counter at four points of an item.
  auto stamp = [&](int wgi, int k, int nk) {
    if (p.trace && tid == 0 && wgi < p.trace_cap) {
      p.trace[(size_t)wgi * 5 + k] = wall_clock64();
      if (k == 0) p.trace[(size_t)wgi * 5 + 4] = nk;
    }
  };
  if constexpr (kRowMajor && !kSparseOut) {
    // launched in both tile shapes: the device-side flag says whether the single blocks (1) or the macro tiles (0) work
    if (p.dual && p.sched[2] != (PA * PB == 1 ? 1 : 0)) return;
  }
  if constexpr (kRing) {
    // "far" operand: three stages, requested two K tiles ahead; "near" operand: two stages, one tile ahead.  The
    // weights (B, rows hundreds of KB apart) are the far operand, except in DSD^T, which measured better with the
    // blocks of dH far (-3 % on that product; the other three gain 0-2 % from the weights being far).
    constexpr bool kFarB = OP != OP_DSDT;
    static_assert(PA == PB, "the two rings hold slabs of one size");
    constexpr int kStage = PA * kPanelBytes, kNearBase = 3 * kStage;
    constexpr int kDmaFar = PA * kCpw;                             // loads per wave for the far slabs of one K tile
    auto issue_ab = [&](bool b_slabs, uint32_t base) {
      const uint32_t s = __builtin_amdgcn_readfirstlane(lds_base + base + wave * 1024);
#pragma unroll
      for (int i = 0; i < kCpw; ++i) {
        dma16(b_slabs ? b0 : a0, b_slabs ? ob[i] : oa[i], s + NW * 1024 * i);
        dma16(b_slabs ? b1 : a1, b_slabs ? ob[i] : oa[i], s + kPanelBytes + NW * 1024 * i);
      }
    };
    auto issue_far = [&](int st) { issue_ab(kFarB, st * kStage); };
    auto issue_near = [&](int st) { issue_ab(!kFarB, kNearBase + st * kStage); };
    const int items = ((majors_live + 3) / 4 * 4 * nminor + 8 * kPatch - 1) / (8 * kPatch) * (8 * kPatch);
    TileState cur, nxt;
    int wgi = blockIdx.x;
    bool have = false;
    for (; wgi < items; wgi += gridDim.x)
      if (decode(wgi, cur)) { have = true; break; }
    int gf = 0, gn = 0;                 // stages of the K tile being multiplied: far ring of three, near ring of two
    bool far_ahead = false;             // the far slabs of the next K tile were requested after the near slabs of this one
    if (have) {                         // every item has at least two K tiles
      slab_ptrs(cur, 0);
      issue_far(0);
      issue_near(0);
      slab_ptrs(cur, 1);
      issue_far(1);
      far_ahead = true;
    }
    while (have) {
      bool have_next = false;
      int nwgi = wgi + gridDim.x;
      for (; nwgi < items; nwgi += gridDim.x)
        if (decode(nwgi, nxt)) { have_next = true; break; }
      const int nk = cur.nk;
      const bool mine = (pm == 0 || cur.a_ok1) && (pn == 0 || cur.b_ok1);
      clear_acc();
      Frags f0, f1;
      stamp(wgi, 0, nk);
      for (int kt = 0; kt < nk; ++kt) {
        // K tile kt needs its far slabs (requested two tiles ago) and its near slabs (one tile ago); the far slabs of the
        // next K tile, requested after those, may stay in flight (loads retire in order)
        if (far_ahead) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kDmaFar) : "memory");
        else           asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();            // K tile kt visible; every wave is done with the tile before it (and its staging tile)
        if (kt == 0) stamp(wgi, 1, nk);
        const char* sfar = lds + gf * kStage;
        const char* snear = lds + kNearBase + gn * kStage;
        const char* sa = (kFarB ? snear : sfar) + pm * kPanelBytes;
        const char* sb = (kFarB ? sfar : snear) + pn * kPanelBytes;
        if (mine) read_frags(f0, sa, sb, 0);
        // the near slabs of the next K tile go where those of the previous one were, the far slabs of the one after
        // next where the previous far slabs were; near the end of an item both belong to the next item
        const bool one = kt + 1 < nk || have_next;
        const bool two = kt + 2 < nk || have_next;
        if (one) {
          if (kt + 1 < nk) {
            slab_ptrs(cur, kt + 1);
          } else {                  // the far slabs of this K tile were requested an iteration ago: its indices are there
            refill_ok = false;
            slab_ptrs(nxt, 0);
            refill_ok = true;
          }
          issue_near(gn ^ 1);
        }
        if (mine) {
          if (kt > 0) mfma_frags(f1);                            // K step 3 of the previous K tile
          read_frags(f1, sa, sb, 1);
        }
        if (two) {
          if (kt + 2 < nk) slab_ptrs(cur, kt + 2);
          else             slab_ptrs(nxt, kt + 2 - nk);
          issue_far(gf == 0 ? 2 : gf - 1);                        // (gf + 2) % 3
        }
        far_ahead = two;
        if (mine) {
          mfma_frags(f0);
          read_frags(f0, sa, sb, 2);
          mfma_frags(f1);
          read_frags(f1, sa, sb, 3);
          mfma_frags(f0);
        }
        if (kt + 1 < nk) {
          gf = gf == 2 ? 0 : gf + 1;
          gn ^= 1;
        }
      }
      if (mine) mfma_frags(f1);
      stamp(wgi, 2, nk);
      __syncthreads();              // every wave has read the last K tile: its slabs are free for the staging tiles
      // waves 0-3 stage in the far slabs of the last K tile, waves 4-7 in its near slabs (32 KB each)
      if (mine) epilogue(cur, lds + (wave < 4 ? gf * kStage + wave * kEpBytes : kNearBase + gn * kStage + (wave - 4) * kEpBytes));
      stamp(wgi, 3, nk);
      gf = gf == 2 ? 0 : gf + 1;
      gn ^= 1;
      cur = nxt;
      wgi = nwgi;
      have = have_next;
    }
  } else
  if constexpr (kPipe) {
    // ---- persistent, software-pipelined loop over this workgroup's items (256x256 tiles of the token-row products)
    // One workgroup per CU walks the items blockIdx, blockIdx + grid, ...  Two things are overlapped that a
    // tile-per-workgroup launch leaves exposed (together about a fifth of a tile's time when K is 16-24 K tiles):
    //  * the next item's set-up (a chain of dependent index loads) and the loads of its first K tile are issued during
    //    the last K tile of the current item and land while its epilogue runs.  The two LDS stages alternate across
    //    items: the first K tile of the next item goes to the stage that the last K tile of this one does not use,
    //    and the epilogue's staging tiles live in the stage that it does use;
    //  * inside an item, the MFMA operands of K step s+1 are read from LDS before the MFMAs of step s are issued
    //    (two fragment sets), and the last K step of a K tile is multiplied after the barrier of the next K tile, behind
    //    the LDS reads of its first step, so the matrix pipe has work across the barrier.
    // live items (the grid's upper bound may be larger), rounded up to whole patches on every XCD: workgroup -> item
    // is a permutation inside blocks of 8 * patch indices (patch is a power of two <= 32), so whole blocks are walked
    const int items = ((majors_live + 3) / 4 * 4 * nminor + 8 * kPatch - 1) / (8 * kPatch) * (8 * kPatch);
    TileState cur, nxt;
    int wgi = blockIdx.x;
    bool have = false;
    for (; wgi < items; wgi += gridDim.x)
      if (decode(wgi, cur)) { have = true; break; }
    int s0 = 0;                                                  // LDS stage of the current item's first K tile
    if (have) {
      slab_ptrs(cur, 0);
      issue_loads(s0, 0);
      issue_loads(s0, 1);
    }
    while (have) {
      bool have_next = false;
      int nwgi = wgi + gridDim.x;
      for (; nwgi < items; nwgi += gridDim.x)
        if (decode(nwgi, nxt)) { have_next = true; break; }
      const int nk = cur.nk;
      const bool mine = (pm == 0 || cur.a_ok1) && (pn == 0 || cur.b_ok1);   // this wave's part of the tile exists
      clear_acc();
      Frags f0, f1;
      stamp(wgi, 0, nk);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();              // K tile 0 visible; every wave is done with the previous item's staging tiles
      stamp(wgi, 1, nk);
      {
        const char* st = lds + s0 * kStageBytes;
        if (mine) read_frags(f0, st + pm * kPanelBytes, st + (PA + pn) * kPanelBytes, 0);
      }
      for (int kt = 0; kt < nk; ++kt) {
        const int stage = (s0 + kt) & 1;
        const char* sa = lds + stage * kStageBytes + pm * kPanelBytes;
        const char* sb = lds + stage * kStageBytes + (PA + pn) * kPanelBytes;
        // what the other stage receives while this K tile is multiplied: the next K tile, or the next item's first
        const bool more = kt + 1 < nk;
        const bool feed = more || have_next;
        if (more) slab_ptrs(cur, kt + 1);
        else if (have_next) slab_ptrs(nxt, 0);
        if (feed) issue_loads(stage ^ 1, 0);
        if (mine) {
          if (kt > 0) mfma_frags(f1);                            // K step 3 of the previous K tile
          read_frags(f1, sa, sb, 1);
        }
        if (feed) issue_loads(stage ^ 1, 1);
        if (mine) {
          mfma_frags(f0);
          read_frags(f0, sa, sb, 2);
          mfma_frags(f1);
          read_frags(f1, sa, sb, 3);
          mfma_frags(f0);
        }
        if (more) {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();          // K tile kt+1 visible; everyone has read all of K tile kt
          if (mine) {
            const char* st = lds + (stage ^ 1) * kStageBytes;
            read_frags(f0, st + pm * kPanelBytes, st + (PA + pn) * kPanelBytes, 0);
          }
        }
      }
      if (mine) mfma_frags(f1);
      const int last_stage = (s0 + nk - 1) & 1;
      stamp(wgi, 2, nk);
      __syncthreads();              // every wave has read the last K tile: its stage is free for the staging tiles
      if (mine) epilogue(cur, lds + last_stage * kStageBytes + wave * kEpBytes);
      stamp(wgi, 3, nk);
      s0 = last_stage ^ 1;
      cur = nxt;
      wgi = nwgi;
      have = have_next;
    }
  } else {
  auto tile = [&](const int wgi) {
  TileState t;
  if (!decode(wgi, t)) return;
  const int nk = t.nk;
  clear_acc();
  stamp(wgi, 0, nk);
  stamp(wgi, 1, nk);
  live_rows = t.live;
  const bool fringe = kFringe && t.live <= 64;
  // this wave's part of the tile exists (and is not the padding half of a fringe block row)
  const bool mine = (pm == 0 || t.a_ok1) && (pn == 0 || t.b_ok1) && arow0 < t.live;
  // Software pipeline over NS LDS stages: K tile t lives in stage t % NS; tiles t+1 .. t+NS-2 are in flight while
  // tile t is multiplied.  Loads return in order, so "at most (NS-2) tiles' worth of loads outstanding" means tile
  // t has landed; near the end of K, when fewer tiles are in flight, the wait is for everything.
  // The 128x128 tile spends about 130 cycles of an iteration on MFMAs and the rest waiting for memory, so hiding
  // the loads behind the arithmetic of the same iteration buys nothing there.  Its two stages are used the other
  // way round: a stage is refilled (with tile kt + 2) as soon as every wave has multiplied it, one barrier later,
  // which keeps two tiles in flight instead of one (-9 % on the weight gradients under skewed routing, -1...4 % on a step).
  if constexpr (PA * PB <= 2 && NS == 2) {
    for (int kt = 0; kt < 2; ++kt) {
      if (kt < nk) {
        slab_ptrs(t, kt);
        issue_loads(kt, 0);
        issue_loads(kt, 1);
      }
    }
    for (int kt = 0; kt < nk; ++kt) {
      // a fringe tile issues one load fewer per K tile (the chunk of rows 64..127 of the A slab)
      static_assert(!kFringe || kCpw == 2, "a fringe tile skips exactly one A chunk per wave");
      if (kt + 1 >= nk) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      else if (fringe)  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kDmaPerTile - 1) : "memory");
      else              asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kDmaPerTile) : "memory");
      __syncthreads();                             // tile kt visible to all
      const char* sa = lds + (kt & 1) * kStageBytes + pm * kPanelBytes;
      const char* sb = lds + (kt & 1) * kStageBytes + (PA + pn) * kPanelBytes;
      if (mine) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) multiply(sa, sb, ks);
      }
      if (kt + 2 < nk) {
        __syncthreads();                           // everyone is done reading this stage
        slab_ptrs(t, kt + 2);
        issue_loads(kt & 1, 0);
        issue_loads(kt & 1, 1);
      }
    }
  } else {
#pragma unroll
  for (int kt = 0; kt < NS - 1; ++kt) {
    if (kt < nk) {
      slab_ptrs(t, kt);
      issue_loads(kt, 0);
      issue_loads(kt, 1);
    }
  }
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + NS - 2 < nk) asm volatile("s_waitcnt vmcnt(%0)" : : "n"((NS - 2) * kDmaPerTile) : "memory");
    else                  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                               // tile kt visible to all; everyone is done with tile kt-1
    const bool more = kt + NS - 1 < nk;
    const int next_stage = (kt + NS - 1) % NS;
    if (more) slab_ptrs(t, kt + NS - 1);
    const char* sa = lds + (kt % NS) * kStageBytes + pm * kPanelBytes;
    const char* sb = lds + (kt % NS) * kStageBytes + (PA + pn) * kPanelBytes;
    // The loads of the next tile are spread over the first two K steps instead of being issued in one burst: a
    // wave cannot start its MFMAs before its own loads have been issued.
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (more && ks < 2) issue_loads(next_stage, ks);
      if (mine) multiply(sa, sb, ks);
    }
  }
  }
  stamp(wgi, 2, nk);
  __syncthreads();                                 // every wave is done with the operand stages: LDS is free
  if (tid == 0 && !mine) stamp(wgi, 3, nk);
  if (!mine) return;
  // the accumulating form of the weight gradients stages 32 columns of fp32 per 32 rows: 4 KB per 32-row tile
  epilogue(t, lds + wave * (MI * 4096));
  stamp(wgi, 3, nk);
  };   // tile

  if constexpr (kRowMajor) {
    tile(blockIdx.x);
  } else {
    // Both tile shapes are launched for the weight gradients; the routing decides on the device which one works.
    const int want_small = p.force_tile ? (p.force_tile == 1) : p.sched[0];
    if (want_small != (PA * PB == 1 ? 1 : 0)) return;
    // The weight-gradient launches are capped at kMaxGradGrid workgroups, each taking the items wgi, wgi + gridDim,
    // ... (heaviest first, so the strided lists cost about the same): the launch that the device-side choice leaves
    // idle then costs a few microseconds instead of one dispatch per tile (40-50 us for the 30 000 small tiles of the
    // larger configurations).  Under skewed routing a workgroup that drew a tile of the hot expert still takes its
    // share of light ones afterwards.
    for (int wgi = blockIdx.x; wgi < p.items; wgi += gridDim.x) {
      tile(wgi);
      __syncthreads();                               // the epilogue's staging tiles are the next item's stages
    }
  }
  }
}

template <int OP, int PA, int PB, int NS, int NW, int BK = 64, int ACT = 0>
static void launch_variant(const BsParams& p, int majors, int nminor, hipStream_t s) {
  constexpr bool ring = PA == 2 && PB == 2 && NS == 3 && NW == 8;       // three A stages and two B stages
  constexpr int kLds = ring ? (3 * PA + 2 * PB) * 256 * BK : NS * (PA + PB) * 256 * BK;
  // raise the dynamic-LDS limit of this instantiation once per process (thread-safe; a failure is reported by every
  // later launch of the variant instead of surfacing as an unexplained launch error)
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [] {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&bsmm_kernel<OP, PA, PB, NS, NW, BK, ACT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  });
  if (attr_rc != hipSuccess) {
    fail_pending(DMOE_ELAUNCH, "bsmm<op %d, %dx%d panels>: cannot reserve %d bytes of LDS: %s", OP, PA, PB, kLds,
         hipGetErrorString(attr_rc));
    return;
  }
  const int items = ((majors + 3) / 4) * 4 * nminor;          // majors are consumed in runs of 4
  int grid = ((items + 8 * kPatch - 1) / (8 * kPatch)) * (8 * kPatch);   // whole patches on every XCD
  BsParams q = p;
  q.items = grid;
  constexpr bool grad = OP == OP_DSTD || OP == OP_DDTS || OP == OP_DDS || OP == OP_DSTDT;
  if (grad && grid > kMaxGradGrid) grid = kMaxGradGrid;
  // the 256x256 tiles of the token-row products run as a persistent loop: one workgroup per CU (128 KB of LDS each)
  constexpr bool pipe = !grad && PA == 2 && PB == 2 && (NS == 2 || NS == 3) && NW == 8;
  if (pipe && grid > kPersistGrid) grid = kPersistGrid;
  hipLaunchKernelGGL((bsmm_kernel<OP, PA, PB, NS, NW, BK, ACT>), dim3(grid), dim3(NW * 64), kLds, s, q);
}

// Other shapes the template covers were measured on MI355X and lost: 16 waves of 64x64 on the 256x256 tile (-2..6 %),
// 256x128 tiles with three LDS stages (-15..20 %), K = 32 per stage with three to five stages (-5..8 %; -20 % on the
// 128x128 tile, where 64-byte row pieces double the number of memory requests), deeper pipelines on the 128x128 tile
// at one workgroup per CU (no faster per K tile, and one workgroup per CU quantises worse), four extra waves that
// only issue the loads (-15 %), staging through registers (global_load + ds_write, -8..12 %), and four waves of
// 128x128 on the 256x256 tile with the accumulators in the accumulation registers (a third less LDS read traffic,
// but one wave per SIMD: K loop -7 %, epilogues -30..60 %; LDS read bandwidth is not what bounds the loop).  A wave can issue
// one direct-to-LDS load per ~120 cycles (a CU one per ~20, i.e. ~50 B/clk), which is why the loads are spread over
// the first two K steps of the MFMA loop.  The products are bound by operand delivery into LDS, not by load latency, so
// intensity wins over pipeline depth.
//
// Tile choice (host side, from the configuration only -- the routing is not known to the host):
//  * 256x256 macro tiles, two LDS stages: when there are enough of them to fill 256 CUs a few times over; they halve
//    the L2->LDS traffic per flop, which is what bounds the MFMA-bound configurations.
//  * single 128x128 blocks, two or more workgroups per CU: when the big tiles would be too few to fill the machine
//    (small T*k).  For the weight gradients the same question depends on the routing (one popular expert owns few
//    big tiles with a very long K), so both shapes are launched and a flag computed on the device picks one.
template <int OP>
static void launch_one(const BsParams& p, const BsArgs& a, hipStream_t s) {
  const int hb = p.hb, db = p.db;
  constexpr bool row_major = OP == OP_SDD || OP == OP_SDDT || OP == OP_DSD || OP == OP_DSDT;
  constexpr bool sparse_out = OP == OP_SDD || OP == OP_SDDT;
  if constexpr (OP >= OP_SDTD) {
    // general masks only, one block per workgroup: sparse outputs enumerate the nonzero blocks, Y = X S^T the block
    // rows of S times the row blocks of X, Y = S^T X^T the block columns times the row blocks of X
    if constexpr (OP == OP_SDTD || OP == OP_SDTDT) launch_variant<OP, 1, 1, 2, 8>(p, a.nnz, 1, s);
    else if constexpr (OP == OP_DSTDT)             launch_variant<OP, 1, 1, 2, 8>(p, a.E * hb, db, s);
    else                                           launch_variant<OP, 1, 1, 2, 8>(p, a.r_max, db, s);
  } else {
  const int big_minor = sparse_out ? (hb + 1) / 2 : (db + 1) / 2;
  if constexpr (row_major) {
    const long long big_items = (long long)a.groups_est * big_minor;
    // SDD / SDD^T: macro tiles once there is one for every CU.  DSD / DSD^T (long K, few tiles): single blocks while
    // they are sure to fit one round of 512 workgroup slots whatever the routing (r_max bounds the block rows); beyond
    // that the device decides (below) -- one block row too many doubles the rounds, and the time, of the single blocks.
    bool small = sparse_out ? big_items <= 256 : (long long)a.r_max * db <= 512;
    // DSD / DSD^T have a long K (= ffn_hidden) and few tiles; with fewer than about two and a half rounds of macro
    // tiles the last, partly filled round can cost up to half the launch (312 tiles on 256 CUs: 62 % of the CUs busy
    // on average), and how many tiles there are depends on the routing, which the host does not know.  The single
    // blocks come in rounds of 512 (two workgroups per CU) that take about 1.0 us per K tile against the 1.6 us of a
    // macro tile's, four blocks large: they win when their rounds are fewer than 1.6 x the macro tiles' -- DSD^T
    // 286 -> 211 us for 16 384 tokens over 64 experts under Zipf routing (312 macro tiles) -- and lose otherwise (192
    // macro tiles: 194 us against 160; 512: +15 %; 8 192 tokens over 8 experts at d = 1 024, where 68 block rows make
    // 544 single blocks: 139 us against 104).  So in that range both shapes are launched and a flag computed on the
    // device with the routing in hand (sched[2], offsets_kernel) picks one; the other exits at once.
    bool few_rounds = !sparse_out && !small && !a.plain && big_items < 640;
    if (a.force_tile == 1) small = true;
    if (a.force_tile >= 2) small = false;
    const bool two_stage = a.force_tile == 3;       // macro tiles on two LDS stages instead of the slab ring
    if (a.force_tile) few_rounds = false;
    if constexpr (OP == OP_SDD) {
      if (a.act == 1 && !a.plain) {               // the tanh form of the activation is its own instantiation
        if (small)          launch_variant<OP, 1, 1, 2, 8, 64, 1>(p, a.r_max, hb, s);
        else if (two_stage) launch_variant<OP, 2, 2, 2, 8, 64, 1>(p, a.g_max, big_minor, s);
        else                launch_variant<OP, 2, 2, 3, 8, 64, 1>(p, a.g_max, big_minor, s);
        return;
      }
    }
    if constexpr (OP == OP_DSD) {
      // 128x256 tiles for DSD when the rows are few but the output is wide enough for every other CU to get one: the
      // block of A is then read once per two output blocks and W2 in 512-byte row pieces (-12 % on this product for
      // 8 192 tokens over 64 experts at d = 512; the other three token-row products did not gain)
      // (one workgroup per CU: only while its tiles are sure to fit one round)
      if (small && !a.plain && 2LL * a.groups_est * big_minor >= 128 && db >= 2 && (long long)a.r_max * big_minor <= 256) {
        launch_variant<OP, 1, 2, 2, 8>(p, a.r_max, big_minor, s);
        return;
      }
    }
    if constexpr (sparse_out) {
      if (small && a.coo) {                       // general masks: one workgroup per nonzero block
        launch_variant<OP, 1, 1, 2, 8>(p, a.nnz, 1, s);
        return;
      }
    }
    if (few_rounds) {
      BsParams q = p;
      q.dual = 1;
      launch_variant<OP, 2, 2, 3, 8>(q, a.g_max, big_minor, s);
      launch_variant<OP, 1, 1, 2, 8>(q, a.r_max, db, s);
    } else if (small) {
      launch_variant<OP, 1, 1, 2, 8>(p, a.r_max, sparse_out ? hb : db, s);
    } else {
      if (two_stage) launch_variant<OP, 2, 2, 2, 8>(p, a.g_max, big_minor, s);
      else           launch_variant<OP, 2, 2, 3, 8>(p, a.g_max, big_minor, s);
    }
  } else {
    // the device-side flag sched[0] selects which of the two launches does the work (the other exits at once)
    launch_variant<OP, 2, 2, 2, 8>(p, a.E * ((hb + 1) / 2), big_minor, s);
    launch_variant<OP, 1, 1, 2, 8>(p, a.E * hb, db, s);
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
  p.group_offsets = t.group_offsets;  p.row_group = t.row_group;  p.expert_order = t.expert_order;
  p.counts = t.counts;  p.sched = t.sched;
  p.tokens_per_expert = a.plain ? nullptr : t.tokens_per_expert;
  p.token_of = a.plain ? nullptr : t.token_of;
  p.d = a.d;  p.h = a.h;  p.E = a.E;  p.hb = a.h / kBlock;  p.db = a.d / kBlock;  p.force_tile = a.force_tile;
  p.plain = a.plain;
  p.accum = a.accum;
  p.ka = a.ka;
  p.coo = a.coo;
  p.dual = 0;
  p.trace = a.trace;  p.trace_cap = a.trace_cap;
  // Patches of 32 tiles per XCD pay off when all tiles cost the same (the products with the token dimension as
  // rows).  The weight-gradient tiles differ in K by orders of magnitude and are ordered heaviest first; the
  // workgroup -> XCD assignment is static, so they are dealt out one by one to keep the eight XCDs level, unless
  // the routing is even enough for patches (sched[1], decided on the device).
  p.patch = (op == OP_DSTD || op == OP_DDTS || op == OP_DDS || op == OP_DSTDT) ? 1 : -kPatchSlack;
  switch (op) {
    case OP_SDD:  launch_one<OP_SDD>(p, a, s); break;
    case OP_SDDT: launch_one<OP_SDDT>(p, a, s); break;
    case OP_DSD:  launch_one<OP_DSD>(p, a, s); break;
    case OP_DSDT: launch_one<OP_DSDT>(p, a, s); break;
    case OP_DSTD: launch_one<OP_DSTD>(p, a, s); break;
    case OP_DDTS: launch_one<OP_DDTS>(p, a, s); break;
    case OP_DDS:  launch_one<OP_DDS>(p, a, s); break;
    case OP_SDTD:  launch_one<OP_SDTD>(p, a, s); break;
    case OP_SDTDT: launch_one<OP_SDTDT>(p, a, s); break;
    case OP_DSTDT: launch_one<OP_DSTDT>(p, a, s); break;
    case OP_DDST:  launch_one<OP_DDST>(p, a, s); break;
    case OP_DDTST: launch_one<OP_DDTST>(p, a, s); break;
  }
}

}  // namespace dmoe
