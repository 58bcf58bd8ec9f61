// Shared device/host helpers of the gfx950 dMoE library (internal; the public boundary is include/dmoe.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dmoe.h"

namespace dmoe {

typedef unsigned short bf16_t;                                        // raw bfloat16 bits in memory
typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_v __attribute__((ext_vector_type(8)));
typedef float f32x2_v __attribute__((ext_vector_type(2)));
typedef float f32x4_v __attribute__((ext_vector_type(4)));
typedef float f32x16_v __attribute__((ext_vector_type(16)));
typedef short s16x4_v __attribute__((ext_vector_type(4)));

constexpr int kBlock = DMOE_BLOCK;   // 128x128 sparse blocks (Section 5.1.2)
constexpr int kMaxTopK = 8;
constexpr int kMaxExperts = 256;
constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Two fp32 -> packed bf16 pair (round to nearest even; one v_cvt_pk_bf16_f32 on gfx950). `lo` lands in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2_v v = {lo, hi};
  bf16x2_v b = __builtin_convertvector(v, bf16x2_v);
  return *reinterpret_cast<uint32_t*>(&b);
}

// Standard normal CDF Phi(v) and density phi(v), fp32.  erfc through the five-term rational-exponential
// approximation of Abramowitz & Stegun 7.1.26 (absolute error < 1.5e-7), arranged so that the small tail is
// computed directly rather than as 1 - (almost 1).
// The SDD epilogue is bound by the vector ALU, so the constants are folded (the 1/sqrt(2) into the rational argument,
// the 1/2 into the polynomial, the -1/2 and log2(e) into one factor in front of the hardware's base-2 exponential)
// and the two branches of the CDF are joined with a sign copy: Phi(v) = 1/2 + sign(v) (1/2 - Phi(-|v|)).
__device__ __forceinline__ void normal_cdf_pdf(float v, float& cdf, float& pdf) {
  const float t = __builtin_amdgcn_rcpf(fmaf(fabsf(v), 0.3275911f * 0.70710678118654752f, 1.0f));
  float poly = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
  poly = fmaf(poly, t, 0.5f * 1.421413741f);
  poly = fmaf(poly, t, 0.5f * -0.284496736f);
  poly = fmaf(poly, t, 0.5f * 0.254829592f);
  poly *= t;
  const float ex = __builtin_amdgcn_exp2f(v * v * (-0.5f * 1.4426950408889634f));   // exp(-v^2 / 2)
  const float half_minus_tail = fmaf(-poly, ex, 0.5f);                                // 1/2 - Phi(-|v|), in [0, 1/2]
  cdf = 0.5f + __builtin_copysignf(half_minus_tail, v);
  pdf = ex * 0.39894228040143268f;
}
// The tanh form of GELU, 0.5 v (1 + tanh(u)) with u = sqrt(2/pi) (v + 0.044715 v^3), written the same way: `cdf` is
// the factor that multiplies v (0.5 (1 + tanh u) = 1 / (1 + exp(-2u))) and `pdf` the factor of v in the derivative,
// d/dv = cdf + v * pdf with pdf = 0.5 (1 - tanh^2 u) u' = 2 cdf (1 - cdf) u'.
__device__ __forceinline__ void tanh_gelu_cdf_pdf(float v, float& cdf, float& pdf) {
  const float v2 = v * v;
  const float u = 0.79788456080286536f * v * fmaf(0.044715f, v2, 1.0f);
  cdf = __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u));           // exp overflow -> rcp(inf) = 0, as it should be
  pdf = 2.0f * cdf * (1.0f - cdf) * 0.79788456080286536f * fmaf(0.134145f, v2, 1.0f);
}
struct StageEvents {            // optional per-stage timing events (see dmoe_set_stage_events)
  hipEvent_t* ev;
  hipStream_t stream;
  __host__ void begin(int stage) const { if (ev && ev[2 * stage]) (void)hipEventRecord(ev[2 * stage], stream); }
  __host__ void end(int stage) const { if (ev && ev[2 * stage + 1]) (void)hipEventRecord(ev[2 * stage + 1], stream); }
};

// ---- launchers implemented in the .hip files (all enqueue on `s`, none synchronises) -------------------------
struct Scratch;  // forward

void launch_router(const dmoe_config& c, const bf16_t* x, const bf16_t* wr, const float* bias,
                   const dmoe_topology_t& t, hipStream_t s);
void launch_sort(const dmoe_config& c, const dmoe_topology_t& t, int32_t* chunk_counts, int p_max, hipStream_t s);
void launch_make_topology(const dmoe_config& c, const dmoe_topology_t& t, int p_max, int nnz_max, hipStream_t s);

void launch_padded_gather(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* x, bf16_t* xp, int p_max,
                          hipStream_t s);
void launch_weighted_scatter(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* yp, bf16_t* y,
                             hipStream_t s);
void launch_bwd_gather(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* dy, const bf16_t* yp,
                       bf16_t* dyp, float* dweights, int p_max, hipStream_t s);
void launch_router_bwd(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* x, const bf16_t* wr,
                       const float* dweights, const bf16_t* dxp, float* dlogits, float* partials, int num_partials,
                       bf16_t* dx, float* dw_router, bool accumulate, hipStream_t s);
int router_bwd_num_partials(const dmoe_config& c);

// The products the layer uses (0-5), DDS, and the remaining combinations of transposed inputs (Section 5.1.1), which
// exist for general masks only (one 128x128 block per workgroup): a superscript T in the paper's notation is a `T`
// after the operand's letter here (SDTD = S D^T D: the left dense input is given transposed).
enum BsOp { OP_SDD = 0, OP_DSD = 1, OP_SDDT = 2, OP_DSTD = 3, OP_DSDT = 4, OP_DDTS = 5, OP_DDS = 6,
            OP_SDTD = 7, OP_SDTDT = 8, OP_DSTDT = 9, OP_DDST = 10, OP_DDTST = 11 };
struct BsArgs {
  const dmoe_topology_t* topo;
  int d, h, E;
  int g_max, r_max;        // upper bounds on the number of row groups / block rows
  int groups_est;          // T*k/256: row groups if the routing were perfectly packed (tile-size heuristic)
  int force_tile;          // 0: heuristic, 1: 128x128 tiles, 2: 256x256 macro tiles, 3: the same on two LDS stages (tests)
  int plain;               // 1: no fused epilogue (SDD writes the product to out0, SDD^T does not multiply by sparse_in)
  int accum;               // 1: DS^TD / DD^TS add their result, in fp32, to the fp32 matrix at out0
  int ka;                  // DDS and the products of Section 5.1.1 beyond the layer's: 128 * block rows of S
  int act;                 // SDD's fused activation: 0 exact (erf) GELU, 1 tanh form
  int coo;                 // 1 (general masks): SDD / SDD^T enumerate the nonzero blocks through row_indices
  int nnz;                 // ... and this many of them
  long long* trace;        // optional per-item time stamps of this launch (NULL = off), room for trace_cap items
  int trace_cap;
  const bf16_t* dense_a;   // Xp / dYp           (SDD, SDDT: lhs;  DSTD, DDTS: the dense operand)
  const bf16_t* dense_b;   // W1 / W2            (SDD, DSD, SDDT, DSDT: rhs)
  const bf16_t* sparse_in; // block values read  (DSD, DSTD, DSDT, DDTS: sparse operand; SDDT: G = gelu'(H))
  bf16_t* out0;            // SDD: G = gelu'(H) blocks; SDDT: dH blocks; others: dense output
  bf16_t* out1;            // SDD: A = gelu(H) blocks
};
void launch_bsmm(BsOp op, const BsArgs& a, hipStream_t s);

// ---- host-side helpers shared by the C-ABI source files ----------------------------------------------------------
int fail(int code, const char* fmt, ...);           // records the message for dmoe_last_error, returns `code`
void fail_pending(int code, const char* fmt, ...);  // for launchers (void): the next launch_status() returns `code`
int check_ptr(const void* p, const char* name);     // non-NULL and 256-byte aligned
int launch_status();                                // DMOE_OK, or DMOE_ELAUNCH with the pending HIP error

}  // namespace dmoe
