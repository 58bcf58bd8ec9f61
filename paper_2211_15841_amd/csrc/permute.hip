// Bandwidth-bound kernels around the block-sparse products: padded gather (Figure 6 step 3, Section 5.2),
// weighted un-permute (step 5, Section 2.4), their backward counterparts, and the router's backward pass.
#include "common.h"

namespace dmoe {

// One wave per padded row: Xp[r] = x[token_of[r] / k], zeros on padding rows.  16 bytes per lane per step.
__global__ void __launch_bounds__(256) padded_gather_kernel(const bf16_t* __restrict__ x, const int32_t* __restrict__ token_of,
                                                            const int32_t* __restrict__ counts, bf16_t* __restrict__ xp,
                                                            int d, int k) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= counts[0]) return;
  const int lane = threadIdx.x & 63;
  const int f = token_of[r];
  uint4* dst = reinterpret_cast<uint4*>(xp + (size_t)r * d);
  if (f < 0) {
    for (int c = lane; c < d / 8; c += 64) dst[c] = make_uint4(0, 0, 0, 0);
  } else {
    const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)(f / k) * d);
    for (int c = lane; c < d / 8; c += 64) dst[c] = src[c];
  }
}

// One wave per token: y[t] = sum_s weights[t,s] * Yp[row_of[t,s]], accumulated in fp32 in slot order.
__global__ void __launch_bounds__(256) weighted_scatter_kernel(const bf16_t* __restrict__ yp, const int32_t* __restrict__ row_of,
                                                               const float* __restrict__ weights, bf16_t* __restrict__ y,
                                                               int T, int d, int k) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const int lane = threadIdx.x & 63;
  for (int c = lane; c < d / 8; c += 64) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int s = 0; s < k; ++s) {
      const int row = row_of[t * k + s];
      const float w = weights[t * k + s];
      const uint4 v = reinterpret_cast<const uint4*>(yp + (size_t)row * d)[c];
      acc[0] = fmaf(w, bf16_lo(v.x), acc[0]); acc[1] = fmaf(w, bf16_hi(v.x), acc[1]);
      acc[2] = fmaf(w, bf16_lo(v.y), acc[2]); acc[3] = fmaf(w, bf16_hi(v.y), acc[3]);
      acc[4] = fmaf(w, bf16_lo(v.z), acc[4]); acc[5] = fmaf(w, bf16_hi(v.z), acc[5]);
      acc[6] = fmaf(w, bf16_lo(v.w), acc[6]); acc[7] = fmaf(w, bf16_hi(v.w), acc[7]);
    }
    uint4 o;
    o.x = pack_bf16(acc[0], acc[1]); o.y = pack_bf16(acc[2], acc[3]);
    o.z = pack_bf16(acc[4], acc[5]); o.w = pack_bf16(acc[6], acc[7]);
    reinterpret_cast<uint4*>(y + (size_t)t * d)[c] = o;
  }
}

// Backward of the un-permute.  One wave per padded row r holding assignment f of token t:
//   dYp[r] = weights[f] * dY[t]   (zeros on padding rows),    dweights[f] = <dY[t], Yp[r]>.
__global__ void __launch_bounds__(256) bwd_gather_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ yp,
                                                         const int32_t* __restrict__ token_of, const float* __restrict__ weights,
                                                         const int32_t* __restrict__ counts, bf16_t* __restrict__ dyp,
                                                         float* __restrict__ dweights, int d, int k) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= counts[0]) return;
  const int lane = threadIdx.x & 63;
  const int f = token_of[r];
  uint4* dst = reinterpret_cast<uint4*>(dyp + (size_t)r * d);
  if (f < 0) {
    for (int c = lane; c < d / 8; c += 64) dst[c] = make_uint4(0, 0, 0, 0);
    return;
  }
  const float w = weights[f];
  const uint4* g = reinterpret_cast<const uint4*>(dy + (size_t)(f / k) * d);
  const uint4* o = reinterpret_cast<const uint4*>(yp + (size_t)r * d);
  float dot = 0.0f;
  for (int c = lane; c < d / 8; c += 64) {
    const uint4 gv = g[c], ov = o[c];
    const float g0 = bf16_lo(gv.x), g1 = bf16_hi(gv.x), g2 = bf16_lo(gv.y), g3 = bf16_hi(gv.y);
    const float g4 = bf16_lo(gv.z), g5 = bf16_hi(gv.z), g6 = bf16_lo(gv.w), g7 = bf16_hi(gv.w);
    dot = fmaf(g0, bf16_lo(ov.x), dot); dot = fmaf(g1, bf16_hi(ov.x), dot);
    dot = fmaf(g2, bf16_lo(ov.y), dot); dot = fmaf(g3, bf16_hi(ov.y), dot);
    dot = fmaf(g4, bf16_lo(ov.z), dot); dot = fmaf(g5, bf16_hi(ov.z), dot);
    dot = fmaf(g6, bf16_lo(ov.w), dot); dot = fmaf(g7, bf16_hi(ov.w), dot);
    uint4 q;
    q.x = pack_bf16(w * g0, w * g1); q.y = pack_bf16(w * g2, w * g3);
    q.z = pack_bf16(w * g4, w * g5); q.w = pack_bf16(w * g6, w * g7);
    dst[c] = q;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
  if (lane == 0) dweights[f] = dot;
}

// ------------------------------------------------------------------------------------------------ router backward
// Chain rule through  weights = softmax(scores)[chosen]  (optionally renormalised over the k slots), with the
// chosen experts held constant.  G lanes per token.
//   dsel_s = dweights_s                                   (raw probabilities)
//   dsel_s = (dweights_s - sum_j dweights_j w_j) / Z      (renormalised; Z = sum of the chosen probabilities)
//   dscores = p * (dp - <dp, p>),  dp = dsel scattered to the chosen experts.
template <int G>
__global__ void __launch_bounds__(256) dlogits_kernel(const float* __restrict__ logits, const int32_t* __restrict__ expert_idx,
                                                      const float* __restrict__ weights, const float* __restrict__ dweights,
                                                      float* __restrict__ dlogits, int T, int E, int k, int normalize) {
  const int tid = threadIdx.x;
  const int sub = tid % G;
  const int t = blockIdx.x * (256 / G) + tid / G;
  const bool live = t < T;
  const size_t tt = live ? t : 0;
  const float* lg = logits + tt * E;
  float m = -INFINITY;
  for (int e = sub; e < E; e += G) m = fmaxf(m, lg[e]);
#pragma unroll
  for (int off = G / 2; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, G));
  float sum = 0.0f;
  for (int e = sub; e < E; e += G) sum += __expf(lg[e] - m);
#pragma unroll
  for (int off = G / 2; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, G);
  const float inv = 1.0f / sum;

  int sel[kMaxTopK];
  float dsel[kMaxTopK];
  float dot_dw_w = 0.0f, Z = 0.0f;
#pragma unroll
  for (int s = 0; s < kMaxTopK; ++s) {
    sel[s] = -1; dsel[s] = 0.0f;
    if (s < k) {
      sel[s] = expert_idx[tt * k + s];
      dsel[s] = dweights[tt * k + s];
      dot_dw_w = fmaf(dsel[s], weights[tt * k + s], dot_dw_w);
      Z += __expf(lg[sel[s]] - m) * inv;
    }
  }
  if (normalize) {
    const float iz = 1.0f / Z;
#pragma unroll
    for (int s = 0; s < kMaxTopK; ++s) dsel[s] = (dsel[s] - dot_dw_w) * iz;
  }
  float dpp = 0.0f;                         // <dp, p>: only the chosen experts contribute
#pragma unroll
  for (int s = 0; s < kMaxTopK; ++s)
    if (s < k) dpp = fmaf(dsel[s], __expf(lg[sel[s]] - m) * inv, dpp);
  if (!live) return;
  for (int e = sub; e < E; e += G) {
    const float p = __expf(lg[e] - m) * inv;
    float dp = 0.0f;
#pragma unroll
    for (int s = 0; s < kMaxTopK; ++s) dp = (s < k && sel[s] == e) ? dsel[s] : dp;
    dlogits[tt * E + e] = p * (dp - dpp);
  }
}

// dx[t, i] = sum_s dXp[row_of[t,s], i] + sum_e dscores[t, e] * Wr[i, e].   Thread = hidden index i, workgroup =
// 32 tokens x 256 hidden indices; dscores rows are broadcast from LDS.
constexpr int kDxTok = 32;
__global__ void __launch_bounds__(256) dx_kernel(const bf16_t* __restrict__ dxp, const int32_t* __restrict__ row_of,
                                                 const float* __restrict__ dlogits, const bf16_t* __restrict__ wr,
                                                 bf16_t* __restrict__ dx, int T, int d, int E, int k) {
  extern __shared__ float dl_s[];           // [kDxTok][E]
  const int t0 = blockIdx.x * kDxTok;
  const int i = blockIdx.y * 256 + threadIdx.x;
  const int nt = min(kDxTok, T - t0);
  for (int q = threadIdx.x; q < nt * E; q += 256) dl_s[q] = dlogits[(size_t)t0 * E + q];
  __syncthreads();
  if (i >= d) return;
  float acc[kDxTok];
#pragma unroll
  for (int j = 0; j < kDxTok; ++j) acc[j] = 0.0f;
  const bf16_t* wrow = wr + (size_t)i * E;
  for (int e = 0; e < E; ++e) {
    const float w = bf16_to_f32(wrow[e]);
#pragma unroll
    for (int j = 0; j < kDxTok; ++j)
      if (j < nt) acc[j] = fmaf(dl_s[j * E + e], w, acc[j]);
  }
#pragma unroll
  for (int j = 0; j < kDxTok; ++j) {
    if (j < nt) {
      const int t = t0 + j;
      float v = acc[j];
      for (int s = 0; s < k; ++s) v += bf16_to_f32(dxp[(size_t)row_of[t * k + s] * d + i]);
      dx[(size_t)t * d + i] = (bf16_t)(pack_bf16(v, 0.0f) & 0xffffu);
    }
  }
}

// dWr[i, e] = sum_t x[t, i] * dscores[t, e]: per chunk of tokens into partials[chunk][i][e], then summed over
// chunks in ascending order (deterministic).  Thread = (hidden index i, 16 experts).
constexpr int kDwrTok = 64;
constexpr int kDwrE = 16;
__global__ void __launch_bounds__(256) dwr_partial_kernel(const bf16_t* __restrict__ x, const float* __restrict__ dlogits,
                                                          float* __restrict__ partials, int T, int d, int E) {
  extern __shared__ float dl_s[];           // [kDwrTok][E]
  const int chunk = blockIdx.x;
  const int t0 = chunk * kDwrTok;
  const int nt = min(kDwrTok, T - t0);
  for (int q = threadIdx.x; q < nt * E; q += 256) dl_s[q] = dlogits[(size_t)t0 * E + q];
  __syncthreads();
  const int i = blockIdx.y * 256 + threadIdx.x;
  if (i >= d) return;
  for (int e0 = 0; e0 < E; e0 += kDwrE) {
    float acc[kDwrE];
#pragma unroll
    for (int j = 0; j < kDwrE; ++j) acc[j] = 0.0f;
    for (int t = 0; t < nt; ++t) {
      const float xv = bf16_to_f32(x[(size_t)(t0 + t) * d + i]);
#pragma unroll
      for (int j = 0; j < kDwrE; ++j)
        if (e0 + j < E) acc[j] = fmaf(xv, dl_s[t * E + e0 + j], acc[j]);
    }
#pragma unroll
    for (int j = 0; j < kDwrE; ++j)
      if (e0 + j < E) partials[((size_t)chunk * d + i) * E + e0 + j] = acc[j];
  }
}
__global__ void __launch_bounds__(256) dwr_reduce_kernel(const float* __restrict__ partials, int nchunks, int n,
                                                         float* __restrict__ dwr) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  float s = 0.0f;
  for (int c = 0; c < nchunks; ++c) s += partials[(size_t)c * n + idx];
  dwr[idx] = s;
}

// ------------------------------------------------------------------------------------------------ launchers
void launch_padded_gather(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* x, bf16_t* xp, int p_max,
                          hipStream_t s) {
  hipLaunchKernelGGL(padded_gather_kernel, dim3((p_max + 3) / 4), dim3(256), 0, s, x, t.token_of, t.counts, xp,
                     c.d_model, c.top_k);
}

void launch_weighted_scatter(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* yp, bf16_t* y,
                             hipStream_t s) {
  hipLaunchKernelGGL(weighted_scatter_kernel, dim3((c.num_tokens + 3) / 4), dim3(256), 0, s, yp, t.row_of, t.weights,
                     y, c.num_tokens, c.d_model, c.top_k);
}

void launch_bwd_gather(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* dy, const bf16_t* yp,
                       bf16_t* dyp, float* dweights, int p_max, hipStream_t s) {
  hipLaunchKernelGGL(bwd_gather_kernel, dim3((p_max + 3) / 4), dim3(256), 0, s, dy, yp, t.token_of, t.weights,
                     t.counts, dyp, dweights, c.d_model, c.top_k);
}

int router_bwd_num_partials(const dmoe_config& c) { return (c.num_tokens + kDwrTok - 1) / kDwrTok; }

void launch_router_bwd(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* x, const bf16_t* wr,
                       const float* dweights, const bf16_t* dxp, float* dlogits, float* partials, int num_partials,
                       bf16_t* dx, float* dw_router, hipStream_t s) {
  const int T = c.num_tokens, d = c.d_model, E = c.num_experts, k = c.top_k;
  int g = 1;
  while (g < E && g < 64) g <<= 1;
#define DMOE_DL_CASE(G)                                                                                        \
  case G:                                                                                                      \
    hipLaunchKernelGGL(dlogits_kernel<G>, dim3((T + 256 / G - 1) / (256 / G)), dim3(256), 0, s, t.logits,      \
                       t.expert_idx, t.weights, dweights, dlogits, T, E, k, c.normalize_topk);                 \
    break;
  switch (g) {
    DMOE_DL_CASE(1)
    DMOE_DL_CASE(2)
    DMOE_DL_CASE(4)
    DMOE_DL_CASE(8)
    DMOE_DL_CASE(16)
    DMOE_DL_CASE(32)
    DMOE_DL_CASE(64)
  }
#undef DMOE_DL_CASE
  hipLaunchKernelGGL(dx_kernel, dim3((T + kDxTok - 1) / kDxTok, (d + 255) / 256), dim3(256),
                     (size_t)kDxTok * E * sizeof(float), s, dxp, t.row_of, dlogits, wr, dx, T, d, E, k);
  hipLaunchKernelGGL(dwr_partial_kernel, dim3(num_partials, (d + 255) / 256), dim3(256),
                     (size_t)kDwrTok * E * sizeof(float), s, x, dlogits, partials, T, d, E);
  hipLaunchKernelGGL(dwr_reduce_kernel, dim3((d * E + 255) / 256), dim3(256), 0, s, partials, num_partials, d * E,
                     dw_router);
}

}  // namespace dmoe
