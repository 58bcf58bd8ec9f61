// C ABI of the general block-sparse products (declared in include/dmoe.h): the same six kernels that the dMoE layer
// uses, on a caller-supplied 128x128 block mask of any shape (Sections 4.2 and 5.1: the products are general
// primitives; the block-diagonal dMoE topology is one instance).  The topology of a mask is encoded on the host
// (hybrid blocked-CSR-COO plus transpose indices, Sections 5.1.3-5.1.4) and uploaded; this is a set-up call, not
// part of any hot path.  The products run one 128x128 block per workgroup and without the fused dMoE epilogues.
#include "common.h"
#include <vector>

namespace dmoe {

struct MaskLayout { size_t off[8]; size_t total; };
static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static MaskLayout mask_layout(int R, int C, int nnz) {
  const size_t n[8] = {
      (size_t)(R + 1) * 4,   // row_offsets
      (size_t)nnz * 4,       // column_indices
      (size_t)nnz * 4,       // row_indices
      (size_t)(C + 1) * 4,   // column_offsets_t
      (size_t)nnz * 4,       // row_indices_t
      (size_t)nnz * 4,       // block_offsets_t
      64,                    // counts[4] | sched[4] | expert_order[1] | group_offsets[2] | zero
      256,                   // zeros: the arrays of dmoe_topology_t that a mask does not have
  };
  MaskLayout l;
  size_t at = 0;
  for (int i = 0; i < 8; ++i) { l.off[i] = at; at += align256(n[i] ? n[i] : 4); }
  l.total = at;
  return l;
}

static int check_mask_dims(int R, int C, int nnz) {
  if (R < 1 || C < 1) return fail(DMOE_EINVAL, "block_rows and block_cols must be >= 1 (got %d, %d)", R, C);
  if ((long long)R * kBlock >= (1ll << 24) || (long long)C * kBlock >= (1ll << 24))
    return fail(DMOE_EINVAL, "matrix dimensions must stay below 2^24");
  if (nnz < 0 || (long long)nnz > (long long)R * C || nnz >= (1 << 27))
    return fail(DMOE_EINVAL, "nnz out of range (got %d)", nnz);
  return DMOE_OK;
}

// Register-only MFMA loop: every wave keeps eight independent 32x32 accumulators busy with the instruction the
// block-sparse products use; nothing touches memory until the one store that keeps the results alive.
__global__ void __launch_bounds__(256) mfma_peak_kernel(float* sink, int iters) {
  bf16x8_v a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)((threadIdx.x + i) & 3);  b[i] = (__bf16)0.5f; }
  f32x16_v acc[8];
  for (int j = 0; j < 8; ++j)
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.0f;
  for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][15];
  if (s == -1.0f) sink[0] = s;                        // never true: the products are non-negative
}

// The same loop shaped like a wave of the 256x256 tile (4 A fragments x 2 B fragments, eight accumulators, two waves
// per SIMD), fed with pseudo-random operands whose mantissa bits change every iteration, and run long enough for the
// power management to settle: the matrix-pipe rate the device SUSTAINS on data that toggles like real data.  Lane 0
// of workgroup 0 brackets the loop with the shader-clock counter and the 100 MHz wall counter.
__global__ void __launch_bounds__(512) mfma_sustained_kernel(float* sink, int iters, long long* clocks) {
  uint32_t seed = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
  auto next = [&]() { seed = seed * 1664525u + 1013904223u; return seed; };
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 ar[4], br[2];
  // bf16 pairs with exponent 126..127 (magnitude 0.5..2), random sign and mantissa
  auto rnd_pair = [&]() { const uint32_t r = next(); return (r & 0x80ff80ffu) | 0x3f003f00u | ((r >> 9) & 0x00800080u); };
  for (int i = 0; i < 4; ++i) for (int q = 0; q < 4; ++q) ar[i][q] = rnd_pair();
  for (int j = 0; j < 2; ++j) for (int q = 0; q < 4; ++q) br[j][q] = rnd_pair();
  f32x16_v acc[4][2];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 2; ++j) for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;
  long long c0 = 0, w0 = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0) { c0 = clock64(); w0 = wall_clock64(); }
  for (int it = 0; it < iters; ++it) {
    const uint32_t flip = (next() >> 8) & 0x007f007fu;          // new mantissa bits, exponents and signs stay
    ar[it & 3][it & 3 ^ 1] ^= flip;
    br[it & 1][(it >> 1) & 3] ^= flip;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        union { u32x4 u; bf16x8_v v; } a, b;
        a.u = ar[i];  b.u = br[j];
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b.v, a.v, acc[i][j], 0, 0, 0);
      }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = clock64() - c0; clocks[1] = wall_clock64() - w0; }
  float sum = 0.0f;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 2; ++j) sum += acc[i][j][0] + acc[i][j][15];
  if (sum == 1.2345e-30f) sink[0] = sum;              // practically never: keeps the accumulators alive
}

}  // namespace dmoe

using namespace dmoe;

extern "C" {

int dmoe_bsmm_sizes(int block_rows, int block_cols, int nnz, size_t* topology_bytes) {
  if (int rc = check_mask_dims(block_rows, block_cols, nnz)) return rc;
  if (topology_bytes) *topology_bytes = mask_layout(block_rows, block_cols, nnz).total;
  return DMOE_OK;
}

int dmoe_bsmm_topology(const uint8_t* mask, int block_rows, int block_cols, void* topology_mem, size_t bytes,
                       dmoe_topology_t* out, int32_t* nnz_out) {
  const int R = block_rows, C = block_cols;
  if (!mask) return fail(DMOE_EINVAL, "mask is NULL");
  if (!out) return fail(DMOE_EINVAL, "out is NULL");
  if (int rc = check_mask_dims(R, C, 0)) return rc;
  if (int rc = check_ptr(topology_mem, "topology_mem")) return rc;
  long long count = 0;
  for (long long i = 0; i < (long long)R * C; ++i) count += mask[i] != 0;
  if (int rc = check_mask_dims(R, C, (int)count)) return rc;
  const int nnz = (int)count;
  const MaskLayout l = mask_layout(R, C, nnz);
  if (bytes < l.total) return fail(DMOE_ENOMEM, "topology buffer has %zu bytes, needs %zu", bytes, l.total);

  // primary encoding: blocks numbered row by row, ascending column inside a row
  std::vector<char> host(l.total, 0);
  int32_t* row_offsets = reinterpret_cast<int32_t*>(host.data() + l.off[0]);
  int32_t* column_indices = reinterpret_cast<int32_t*>(host.data() + l.off[1]);
  int32_t* row_indices = reinterpret_cast<int32_t*>(host.data() + l.off[2]);
  int32_t* column_offsets_t = reinterpret_cast<int32_t*>(host.data() + l.off[3]);
  int32_t* row_indices_t = reinterpret_cast<int32_t*>(host.data() + l.off[4]);
  int32_t* block_offsets_t = reinterpret_cast<int32_t*>(host.data() + l.off[5]);
  int32_t* small = reinterpret_cast<int32_t*>(host.data() + l.off[6]);
  int b = 0;
  for (int r = 0; r < R; ++r) {
    row_offsets[r] = b;
    for (int c = 0; c < C; ++c)
      if (mask[(size_t)r * C + c]) { column_indices[b] = c; row_indices[b] = r; ++b; }
  }
  row_offsets[R] = b;
  // transpose indices: the blocks of each column in ascending row order, each with its offset in the primary order
  std::vector<int32_t> fill(C + 1, 0);
  for (int i = 0; i < nnz; ++i) ++fill[column_indices[i] + 1];
  for (int c = 0; c < C; ++c) fill[c + 1] += fill[c];
  for (int c = 0; c <= C; ++c) column_offsets_t[c] = fill[c];
  for (int i = 0; i < nnz; ++i) {                    // primary order is ascending in the row index already
    const int at = fill[column_indices[i]]++;
    row_indices_t[at] = row_indices[i];
    block_offsets_t[at] = i;
  }
  small[0] = R * kBlock;  small[1] = R;  small[2] = nnz;  small[3] = 0;      // counts
  small[4] = 1;  small[5] = 1;  small[6] = 0;  small[7] = 0;                  // sched: one block per workgroup, no patches
  small[8] = 0;                                                               // expert_order[0]
  small[9] = 0;  small[10] = 0;                                               // group_offsets (no row groups)

  if (hipMemcpy(topology_mem, host.data(), l.total, hipMemcpyHostToDevice) != hipSuccess)
    return fail(DMOE_ELAUNCH, "copying the topology to the device failed: %s", hipGetErrorString(hipGetLastError()));

  char* d = static_cast<char*>(topology_mem);
  int32_t* zi = reinterpret_cast<int32_t*>(d + l.off[7]);
  int32_t* sm = reinterpret_cast<int32_t*>(d + l.off[6]);
  out->expert_idx = zi;  out->weights = reinterpret_cast<float*>(zi);  out->logits = reinterpret_cast<float*>(zi);
  out->tokens_per_expert = zi;  out->padded_offsets = zi;  out->row_of = zi;  out->token_of = zi;
  out->row_offsets = reinterpret_cast<int32_t*>(d + l.off[0]);
  out->column_indices = reinterpret_cast<int32_t*>(d + l.off[1]);
  out->row_indices = reinterpret_cast<int32_t*>(d + l.off[2]);
  out->column_offsets_t = reinterpret_cast<int32_t*>(d + l.off[3]);
  out->row_indices_t = reinterpret_cast<int32_t*>(d + l.off[4]);
  out->block_offsets_t = reinterpret_cast<int32_t*>(d + l.off[5]);
  out->counts = sm;  out->sched = sm + 4;  out->expert_order = sm + 8;  out->group_offsets = sm + 9;
  out->row_group = zi;
  if (nnz_out) *nnz_out = nnz;
  return DMOE_OK;
}

int dmoe_bsmm(int op, const dmoe_topology_t* topo, int block_rows, int block_cols, int nnz, int dense, const void* a,
              const void* b, void* out, void* stream) {
  if (op < DMOE_OP_SDD || op > DMOE_OP_DDTST) return fail(DMOE_EINVAL, "unknown product %d", op);
  if (!topo || !topo->row_offsets || !topo->counts) return fail(DMOE_EINVAL, "topology is NULL or not built");
  if (int rc = check_mask_dims(block_rows, block_cols, nnz)) return rc;
  if (dense < kBlock || dense % kBlock) return fail(DMOE_EINVAL, "dense must be a positive multiple of 128 (got %d)", dense);
  if (dense >= (1 << 24)) return fail(DMOE_EINVAL, "dense must stay below 2^24 (got %d)", dense);   // 32-bit byte offsets in a slab
  if ((long long)block_cols * kBlock * dense >= (1ll << 40) || (long long)block_cols * kBlock * kBlock >= (1ll << 32) ||
      (long long)block_rows * kBlock * kBlock >= (1ll << 32))
    return fail(DMOE_EINVAL, "operands too large");
  const bool sparse_out = op == DMOE_OP_SDD || op == DMOE_OP_SDDT || op == DMOE_OP_SDTD || op == DMOE_OP_SDTDT;
  if (sparse_out && nnz == 0) return DMOE_OK;      // no block to write
  if (int rc = check_ptr(a, "a")) return rc;
  if (int rc = check_ptr(b, "b")) return rc;
  if (int rc = check_ptr(out, "out")) return rc;
  BsArgs g{};
  g.topo = topo;  g.d = dense;  g.h = block_cols * kBlock;  g.E = 1;
  g.r_max = block_rows;  g.g_max = 0;  g.groups_est = 0;  g.force_tile = 1;  g.plain = 1;  g.coo = 1;  g.nnz = nnz;
  const bf16_t* pa = static_cast<const bf16_t*>(a);
  const bf16_t* pb = static_cast<const bf16_t*>(b);
  g.out0 = static_cast<bf16_t*>(out);
  switch (op) {
    case DMOE_OP_SDD:  g.dense_a = pa;  g.dense_b = pb;  break;      // S = X W
    case DMOE_OP_DSD:  g.sparse_in = pa;  g.dense_b = pb;  break;    // Y = S W
    case DMOE_OP_SDDT: g.dense_a = pa;  g.dense_b = pb;  break;      // S = X W^T
    case DMOE_OP_DSTD: g.sparse_in = pa;  g.dense_a = pb;  break;    // Y = S^T X
    case DMOE_OP_DSDT: g.sparse_in = pa;  g.dense_b = pb;  break;    // Y = S W^T
    case DMOE_OP_DDTS: g.dense_a = pa;  g.sparse_in = pb;  break;    // Y = X^T S
    case DMOE_OP_DDS:  g.dense_a = pa;  g.sparse_in = pb;  g.ka = block_rows * kBlock;  break;   // Y = X S
    case DMOE_OP_SDTD:  g.dense_a = pa;  g.dense_b = pb;  g.ka = block_rows * kBlock;  break;    // S = X^T W
    case DMOE_OP_SDTDT: g.dense_a = pa;  g.dense_b = pb;  g.ka = block_rows * kBlock;  break;    // S = X^T W^T
    case DMOE_OP_DSTDT: g.sparse_in = pa;  g.dense_a = pb;  g.ka = block_rows * kBlock;  break;  // Y = S^T X^T
    case DMOE_OP_DDST:  g.dense_a = pa;  g.sparse_in = pb;  g.ka = block_rows * kBlock;  break;  // Y = X S^T
    case DMOE_OP_DDTST: g.dense_a = pa;  g.sparse_in = pb;  g.ka = block_rows * kBlock;  break;  // Y = X^T S^T
  }
  (void)hipGetLastError();
  launch_bsmm(static_cast<BsOp>(op), g, static_cast<hipStream_t>(stream));
  return launch_status();
}

int dmoe_probe_mfma_tflops(float* tflops, void* scratch4, void* stream) {
  if (!tflops) return fail(DMOE_EINVAL, "tflops is NULL");
  if (int rc = check_ptr(scratch4, "scratch4")) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return fail(DMOE_ELAUNCH, "hipEventCreate failed");
  const int grid = 256 * 4, iters = 4096;             // four workgroups of four waves per CU: four waves per SIMD
  (void)hipGetLastError();
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(grid), dim3(256), 0, s, static_cast<float*>(scratch4), 64);   // warm-up
  (void)hipEventRecord(e0, s);
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(grid), dim3(256), 0, s, static_cast<float*>(scratch4), iters);
  (void)hipEventRecord(e1, s);
  float ms = 0.0f;
  hipError_t err = hipEventSynchronize(e1);
  if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess || ms <= 0.0f) return fail(DMOE_ELAUNCH, "timing the probe failed: %s", hipGetErrorString(err));
  const double flops = (double)grid * 4 /* waves */ * iters * 8 /* MFMAs */ * (2.0 * 32 * 32 * 16);
  *tflops = (float)(flops / (ms * 1e-3) / 1e12);
  return launch_status();
}

int dmoe_probe_mfma_sustained(float* tflops, float* shader_ghz, float seconds, void* scratch64, void* stream) {
  if (!tflops || !shader_ghz) return fail(DMOE_EINVAL, "tflops or shader_ghz is NULL");
  if (!(seconds > 0.0f) || seconds > 5.0f) return fail(DMOE_EINVAL, "seconds must be in (0, 5]");
  if (int rc = check_ptr(scratch64, "scratch64")) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return fail(DMOE_ELAUNCH, "hipEventCreate failed");
  float* sink = static_cast<float*>(scratch64);
  long long* clocks = reinterpret_cast<long long*>(static_cast<char*>(scratch64) + 16);
  const int grid = 256, iters = 1 << 16;              // one workgroup of eight waves per CU; about 10 ms per launch
  const double flops_per_launch = (double)grid * 8 * iters * 8 * (2.0 * 32 * 32 * 16);
  (void)hipGetLastError();
  // launches back to back until `seconds` have passed on the host clock; the last five are the ones timed
  float ms = 0.0f;
  hipError_t err = hipSuccess;
  int launches = 0;
  const int max_launches = (int)(seconds * 1000.0f / 5.0f) + 8;
  double elapsed_ms = 0.0;
  while (err == hipSuccess && launches < max_launches && elapsed_ms < seconds * 1000.0) {
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < 5; ++i)
      hipLaunchKernelGGL(mfma_sustained_kernel, dim3(grid), dim3(512), 0, s, sink, iters, clocks);
    (void)hipEventRecord(e1, s);
    err = hipEventSynchronize(e1);
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    elapsed_ms += ms;
    launches += 5;
  }
  long long host_clocks[2] = {0, 0};
  if (err == hipSuccess) err = hipMemcpy(host_clocks, clocks, sizeof(host_clocks), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess || ms <= 0.0f || host_clocks[1] <= 0)
    return fail(DMOE_ELAUNCH, "timing the sustained probe failed: %s", hipGetErrorString(err));
  *tflops = (float)(5.0 * flops_per_launch / (ms * 1e-3) / 1e12);
  *shader_ghz = (float)((double)host_clocks[0] / ((double)host_clocks[1] / 0.1) );   // wall counter: 100 MHz
  return launch_status();
}

}  // extern "C"
