// Bandwidth-bound kernels around the block-sparse products: padded gather (Figure 6 step 3, Section 5.2),
// weighted un-permute (step 5, Section 2.4), their backward counterparts, and the router's backward pass.
#include "common.h"
#include "mma_tile.h"

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
      if (row < 0) continue;                       // a dropped assignment contributes nothing (Section 2.2)
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
                                                      const int32_t* __restrict__ row_of,
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
      dsel[s] = row_of[tt * k + s] < 0 ? 0.0f : dweights[tt * k + s];   // a dropped assignment has no gradient
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

// Split an fp32 value into two bf16 values hi + lo (hi = nearest bf16, lo = nearest bf16 of the remainder), so that
// a pair of bf16 MFMAs reproduces an fp32 operand to about 16 bits.
__device__ __forceinline__ void split8(const float (&v)[8], bf16x8_v& hi, bf16x8_v& lo) {
  union { uint32_t u[4]; bf16x8_v v; } h, l;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h.u[i] = pack_bf16(v[2 * i], v[2 * i + 1]);
    l.u[i] = pack_bf16(v[2 * i] - bf16_lo(h.u[i]), v[2 * i + 1] - bf16_hi(h.u[i]));
  }
  hi = h.v;
  lo = l.v;
}

// dx[t, i] = sum_s dXp[row_of[t,s], i] + sum_e dscores[t, e] * Wr[i, e].
// A 128-token x 128-hidden tile per workgroup on MFMA with K = E; both operands have K contiguous in memory
// (dscores [T,E], Wr [d,E]), so every lane loads its operand straight from global memory: no LDS.  The fp32
// dscores are fed as a bf16 hi/lo pair.  The epilogue adds the un-permuted expert gradient rows and rounds to bf16.
template <bool VEC>
__global__ void __launch_bounds__(256) dx_mfma_kernel(const bf16_t* __restrict__ dxp, const int32_t* __restrict__ row_of,
                                                      const float* __restrict__ dlogits, const bf16_t* __restrict__ wr,
                                                      bf16_t* __restrict__ dx, int T, int d, int E, int k) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // column tiles of one token block are neighbours in launch order: together they read and write whole rows
  const int t0 = blockIdx.y * 128 + (wave >> 1) * 64;
  const int i0 = blockIdx.x * 128 + (wave & 1) * 64;
  f32x16_v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  for (int e0 = 0; e0 < E; e0 += 16) {
    const int e = e0 + 8 * (lane >> 5);
    bf16x8_v ah[2], al[2], bf[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int t = t0 + 32 * i + (lane & 31);
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = 0.0f;
      if (t < T) {
        const float* src = dlogits + (size_t)t * E + e;
        if (VEC) {
          if (e < E) {
            const float4 p0 = *reinterpret_cast<const float4*>(src), p1 = *reinterpret_cast<const float4*>(src + 4);
            v[0] = p0.x; v[1] = p0.y; v[2] = p0.z; v[3] = p0.w; v[4] = p1.x; v[5] = p1.y; v[6] = p1.z; v[7] = p1.w;
          }
        } else {
#pragma unroll
          for (int u = 0; u < 8; ++u) if (e + u < E) v[u] = src[u];
        }
      }
      split8(v, ah[i], al[i]);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const bf16_t* src = wr + (size_t)(i0 + 32 * j + (lane & 31)) * E + e;
      union { uint4 q; bf16_t s[8]; bf16x8_v v; } w;
      w.q = make_uint4(0, 0, 0, 0);
      if (VEC) { if (e < E) w.q = *reinterpret_cast<const uint4*>(src); }
      else {
#pragma unroll
        for (int u = 0; u < 8; ++u) if (e + u < E) w.s[u] = src[u];
      }
      bf[j] = w.v;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], ah[i], acc[i][j], 0, 0, 0);
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], al[i], acc[i][j], 0, 0, 0);
      }
  }
  // operands were swapped: lane l, register 4q+u of tile (i, j) is C[t0 + 32i + l%32][i0 + 32j + 8q + 4(l/32) + u].
  // Straight from there every load of a dXp row and every store of dx would touch 32 rows with 8 bytes each; the
  // wave's 64x64 fp32 tile goes through a wave-private LDS tile instead, and rows are then handled 128 bytes at a
  // time (8 lanes per row, 16 bytes per lane).
  __shared__ __attribute__((aligned(16))) float stg[4][64 * 68];
  float* st = stg[wave];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&st[(32 * i + (lane & 31)) * 68 + 32 * j + 8 * q + 4 * (lane >> 5)]) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
  // (same wave writes and reads: no barrier needed, the compiler orders the LDS accesses of one wave)
  // The gathers of the first two slots of all eight row groups are issued before any of them is used: a chain of
  // row_of -> dXp row -> store per group would expose two memory latencies eight times over.
  const int c8 = (lane & 7) * 8;
  int rows[8][2];
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int t = min(t0 + 8 * it + (lane >> 3), T - 1);
#pragma unroll
    for (int s = 0; s < 2; ++s) rows[it][s] = s < k ? row_of[(size_t)t * k + s] : 0;
  }
  uint4 g[8][2];
#pragma unroll
  for (int it = 0; it < 8; ++it)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      g[it][s] = make_uint4(0, 0, 0, 0);
      if (s < k && rows[it][s] >= 0) g[it][s] = *reinterpret_cast<const uint4*>(dxp + (size_t)rows[it][s] * d + i0 + c8);
    }
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = 8 * it + (lane >> 3);
    const int t = t0 + r;
    const float4 v0 = *reinterpret_cast<const float4*>(&st[r * 68 + c8]);
    const float4 v1 = *reinterpret_cast<const float4*>(&st[r * 68 + c8 + 4]);
    float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    auto add = [&](const uint4 q) {
      v[0] += bf16_lo(q.x); v[1] += bf16_hi(q.x); v[2] += bf16_lo(q.y); v[3] += bf16_hi(q.y);
      v[4] += bf16_lo(q.z); v[5] += bf16_hi(q.z); v[6] += bf16_lo(q.w); v[7] += bf16_hi(q.w);
    };
    add(g[it][0]);                                   // slot order, as the sum is defined (zeros when k < 2)
    add(g[it][1]);
    if (t < T) {
      for (int s = 2; s < k; ++s) {
        const int row = row_of[(size_t)t * k + s];
        if (row >= 0) add(*reinterpret_cast<const uint4*>(dxp + (size_t)row * d + i0 + c8));
      }
      uint4 o;
      o.x = pack_bf16(v[0], v[1]);  o.y = pack_bf16(v[2], v[3]);
      o.z = pack_bf16(v[4], v[5]);  o.w = pack_bf16(v[6], v[7]);
      *reinterpret_cast<uint4*>(dx + (size_t)t * d + i0 + c8) = o;
    }
  }
}

// dWr[i, e] = sum_t x[t, i] * dscores[t, e].  Both operands have the reduction index t as their slow index, so both
// are staged as [t][.] slabs and read with transposing LDS loads.  One workgroup = 128 hidden indices x up to 128
// experts x a chunk of tokens, written as an fp32 partial; the partials are then summed over chunks in ascending
// order (deterministic).  dscores are fed as a bf16 hi/lo pair.  The chunk is 256 tokens when that still gives
// every CU a workgroup, else 128 or 64: the kernel is a chain of load -> LDS -> MFMA steps of 64 tokens, and with
// few workgroups their latencies are all exposed.
static int dwr_chunk_tokens(const dmoe_config& c) {
  const int col_tiles = c.d_model / 128;
  for (int tok = 256; tok > 64; tok >>= 1)
    if (((c.num_tokens + tok - 1) / tok) * col_tiles >= 256) return tok;
  return 64;
}
__global__ void __launch_bounds__(256, 3) dwr_mfma_kernel(const bf16_t* __restrict__ x, const float* __restrict__ dlogits,
                                                       float* __restrict__ partials, int T, int d, int E, int kDwrTok) {
  __shared__ __attribute__((aligned(16))) char xs[16384];
  __shared__ __attribute__((aligned(16))) char hs[16384];
  __shared__ __attribute__((aligned(16))) char ls[16384];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, i0 = blockIdx.y * 128, t0 = chunk * kDwrTok;

  for (int eb = 0; eb < E; eb += 128) {
    const int nsub = min(4, (E - eb + 31) / 32);
    f32x16_v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;

    for (int kt = 0; kt < kDwrTok / 64; ++kt) {
      const int tb = t0 + kt * 64;
      if (tb >= T) break;
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int q = tid + 256 * r;
        const int krow = q >> 4, c16 = q & 15;
        const int t = tb + krow;
        uint4 xv = make_uint4(0, 0, 0, 0);
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = 0.0f;
        if (t < T) {
          xv = *reinterpret_cast<const uint4*>(x + (size_t)t * d + i0 + c16 * 8);
          const int e = eb + c16 * 8;
          const float* src = dlogits + (size_t)t * E + e;
          if ((E & 7) == 0) {                     // rows of dscores are 32-byte aligned: two 16-byte loads
            if (e < E) {
              const float4 p0 = *reinterpret_cast<const float4*>(src), p1 = *reinterpret_cast<const float4*>(src + 4);
              v[0] = p0.x; v[1] = p0.y; v[2] = p0.z; v[3] = p0.w; v[4] = p1.x; v[5] = p1.y; v[6] = p1.z; v[7] = p1.w;
            }
          } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) if (e + u < E) v[u] = src[u];
          }
        }
        bf16x8_v hi, lo;
        split8(v, hi, lo);
        const int off = nc_offset(krow, c16);
        *reinterpret_cast<uint4*>(xs + off) = xv;
        *reinterpret_cast<bf16x8_v*>(hs + off) = hi;
        *reinterpret_cast<bf16x8_v*>(ls + off) = lo;
      }
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8_v af = load_frag<NC, 64>(xs, 32 * wave, ks, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (j < nsub) {
            const bf16x8_v bh = load_frag<NC, 64>(hs, 32 * j, ks, lane);
            const bf16x8_v bl = load_frag<NC, 64>(ls, 32 * j, ks, lane);
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bh, acc[j], 0, 0, 0);
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bl, acc[j], 0, 0, 0);
          }
        }
      }
    }
    // lane l, register r of tile j is C[i0 + 32 wave + 8 (r/4) + 4 (l/32) + r%4][eb + 32 j + l%32]
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = eb + 32 * j + (lane & 31);
      if (j < nsub && e < E) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = i0 + 32 * wave + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          partials[((size_t)chunk * d + row) * E + e] = acc[j][r];
        }
      }
    }
  }
}
__global__ void __launch_bounds__(256) dwr_reduce_kernel(const float* __restrict__ partials, int nchunks, int n,
                                                         float* __restrict__ dwr, int accumulate) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  float s = 0.0f;
  int c = 0;
  for (; c + 8 <= nchunks; c += 8) {               // eight loads in flight; the additions stay in ascending order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partials[(size_t)(c + u) * n + idx];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; c < nchunks; ++c) s += partials[(size_t)c * n + idx];
  dwr[idx] = accumulate ? dwr[idx] + s : s;
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

int router_bwd_num_partials(const dmoe_config& c) {
  const int tok = dwr_chunk_tokens(c);
  return (c.num_tokens + tok - 1) / tok;
}

void launch_router_bwd(const dmoe_config& c, const dmoe_topology_t& t, const bf16_t* x, const bf16_t* wr,
                       const float* dweights, const bf16_t* dxp, float* dlogits, float* partials, int num_partials,
                       bf16_t* dx, float* dw_router, bool accumulate, hipStream_t s) {
  const int T = c.num_tokens, d = c.d_model, E = c.num_experts, k = c.top_k;
  int g = 1;
  while (g < E && g < 64) g <<= 1;
#define DMOE_DL_CASE(G)                                                                                        \
  case G:                                                                                                      \
    hipLaunchKernelGGL(dlogits_kernel<G>, dim3((T + 256 / G - 1) / (256 / G)), dim3(256), 0, s, t.logits,      \
                       t.expert_idx, t.weights, dweights, t.row_of, dlogits, T, E, k, c.normalize_topk);       \
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
  if (E % 8 == 0)
    hipLaunchKernelGGL(dx_mfma_kernel<true>, dim3(d / 128, (T + 127) / 128), dim3(256), 0, s, dxp, t.row_of, dlogits,
                       wr, dx, T, d, E, k);
  else
    hipLaunchKernelGGL(dx_mfma_kernel<false>, dim3(d / 128, (T + 127) / 128), dim3(256), 0, s, dxp, t.row_of, dlogits,
                       wr, dx, T, d, E, k);
  hipLaunchKernelGGL(dwr_mfma_kernel, dim3(num_partials, d / 128), dim3(256), 0, s, x, dlogits, partials, T, d, E,
                     dwr_chunk_tokens(c));
  hipLaunchKernelGGL(dwr_reduce_kernel, dim3((d * E + 255) / 256), dim3(256), 0, s, partials, num_partials, d * E,
                     dw_router, accumulate ? 1 : 0);
}

}  // namespace dmoe
