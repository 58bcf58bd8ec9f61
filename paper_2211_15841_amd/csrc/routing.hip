// Router, stable grouping by expert, and block-sparse topology construction (steps (1)-(2) of Figure 6).
//
//   router_logits_kernel  scores = x Wr (+ bias), fp32, accumulated in ascending hidden index  (Section 2.1)
//   topk_kernel           greedy top-k on the scores, softmax confidences                      (Section 2.1)
//   chunk_hist_kernel     per-chunk expert histogram (wave ballots)                            (Section 5.2)
//   offsets_kernel        scan over chunks and experts: n_e, padded offsets, counts, expert order
//   rank_kernel           stable destination row of every assignment, and its inverse
//   topology_kernel       blocked CSR + per-block row indices + transpose indices              (Sections 5.1.3-5.1.4)
#include "common.h"

namespace dmoe {

// ------------------------------------------------------------------------------------------------ scores
// One lane owns one expert (of a chunk of EPAD experts) for TPT tokens; a wave holds 64/EPAD token groups.
// The x tile is staged in LDS as fp32 and read as broadcasts, the Wr tile as fp32 rows.  Every (token, expert)
// accumulator sees its products in ascending hidden index, one fused multiply-add each: a bf16 x bf16 product
// is exact in fp32, so the sum is reproducible bit for bit by any implementation that keeps the order.
// The multiply-adds run on the matrix pipes all the same: v_mfma_f32_4x4x1_16b_f32 is sixteen independent 4x4 outer
// products with K = 1, so every output element receives exactly one product per instruction, c + a*b rounded once.
// Block b = lanes 4b..4b+3 holds four consecutive experts (B operand: one expert per lane, as before) and four
// tokens (A operand: lane l supplies token l%4 of its group); accumulator register r of a lane is the score of
// token r of the group for the lane's expert.  Issued once per hidden index in ascending order this is the same
// chain, at a quarter of the issue slots and half the LDS reads.
constexpr int kRouterKT = 64;

template <int EPAD, int kRouterTPT>
__global__ void __launch_bounds__(256) router_logits_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wr,
                                                            const float* __restrict__ bias, float* __restrict__ logits,
                                                            int T, int d, int E) {
  constexpr int GW = 64 / EPAD;                 // token groups per wave
  constexpr int TT = 4 * GW * kRouterTPT;       // tokens per workgroup
  constexpr int XP = kRouterKT + 4;             // padded row of the x tile (floats)
  __shared__ __attribute__((aligned(16))) float xs[TT * XP];
  __shared__ __attribute__((aligned(16))) float ws[kRouterKT * EPAD];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int el = lane % EPAD;
  const int group = wave * GW + lane / EPAD;
  const int tile0 = blockIdx.x * TT;
  const int tok_local = group * kRouterTPT;
  const bool vec_w = (E % 8) == 0;              // rows of Wr are 16-byte aligned

  for (int e0 = 0; e0 < E; e0 += EPAD) {
    static_assert(kRouterTPT % 4 == 0, "tokens per lane come in groups of four (one 4x4 block each)");
    f32x4_v acc4[kRouterTPT / 4];
    constexpr int NX = (TT * (kRouterKT / 8) + 255) / 256;                        // 16-byte loads of x per thread and K tile
    constexpr int NWV = EPAD >= 8 ? (kRouterKT * (EPAD / 8) + 255) / 256 : 1;     // ... of Wr (vector path)
    uint4 xr[NX], wv[NWV];
#pragma unroll
    for (int g = 0; g < kRouterTPT / 4; ++g) acc4[g] = f32x4_v{0.0f, 0.0f, 0.0f, 0.0f};

    // The raw bf16 of the next K tile is fetched into registers while the current one is multiplied: without that,
    // every K tile exposes one global-load latency between two barriers.
    auto fetch = [&](int i0) {
#pragma unroll
      for (int u = 0; u < NX; ++u) {
        const int q = tid + 256 * u;
        xr[u] = make_uint4(0, 0, 0, 0);
        if (q < TT * (kRouterKT / 8)) {
          const int tl = q / (kRouterKT / 8), c = q % (kRouterKT / 8);
          const int t = tile0 + tl;
          if (t < T) xr[u] = *reinterpret_cast<const uint4*>(x + (size_t)t * d + i0 + c * 8);
        }
      }
      if constexpr (EPAD >= 8) {
        if (vec_w) {
#pragma unroll
          for (int u = 0; u < NWV; ++u) {
            const int q = tid + 256 * u;
            wv[u] = make_uint4(0, 0, 0, 0);
            if (q < kRouterKT * (EPAD / 8)) {
              const int i = q / (EPAD / 8), c = q % (EPAD / 8);
              const int e = e0 + c * 8;
              if (e < E) wv[u] = *reinterpret_cast<const uint4*>(wr + (size_t)(i0 + i) * E + e);
            }
          }
        }
      }
    };
    auto widen_store = [](float* dst, uint4 raw) {
      *reinterpret_cast<float4*>(dst) = make_float4(bf16_lo(raw.x), bf16_hi(raw.x), bf16_lo(raw.y), bf16_hi(raw.y));
      *reinterpret_cast<float4*>(dst + 4) = make_float4(bf16_lo(raw.z), bf16_hi(raw.z), bf16_lo(raw.w), bf16_hi(raw.w));
    };
    fetch(0);
    for (int i0 = 0; i0 < d; i0 += kRouterKT) {
      __syncthreads();
#pragma unroll
      for (int u = 0; u < NX; ++u) {
        const int q = tid + 256 * u;
        if (q < TT * (kRouterKT / 8)) widen_store(&xs[(q / (kRouterKT / 8)) * XP + (q % (kRouterKT / 8)) * 8], xr[u]);
      }
      bool staged = false;
      if constexpr (EPAD >= 8) {
        if (vec_w) {
#pragma unroll
          for (int u = 0; u < NWV; ++u) {
            const int q = tid + 256 * u;
            if (q < kRouterKT * (EPAD / 8)) widen_store(&ws[(q / (EPAD / 8)) * EPAD + (q % (EPAD / 8)) * 8], wv[u]);
          }
          staged = true;
        }
      }
      if (!staged) {
        for (int q = tid; q < kRouterKT * EPAD; q += 256) {
          const int i = q / EPAD, e = e0 + q % EPAD;
          ws[q] = e < E ? bf16_to_f32(wr[(size_t)(i0 + i) * E + e]) : 0.0f;
        }
      }
      __syncthreads();
      if (i0 + kRouterKT < d) fetch(i0 + kRouterKT);
#pragma unroll 4
      for (int i = 0; i < kRouterKT; i += 4) {
        const float w0 = ws[(i + 0) * EPAD + el], w1 = ws[(i + 1) * EPAD + el];
        const float w2 = ws[(i + 2) * EPAD + el], w3 = ws[(i + 3) * EPAD + el];
#pragma unroll
        for (int g = 0; g < kRouterTPT / 4; ++g) {
          const float4 xv = *reinterpret_cast<const float4*>(&xs[(tok_local + 4 * g + (lane & 3)) * XP + i]);
          acc4[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv.x, w0, acc4[g], 0, 0, 0);
          acc4[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv.y, w1, acc4[g], 0, 0, 0);
          acc4[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv.z, w2, acc4[g], 0, 0, 0);
          acc4[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv.w, w3, acc4[g], 0, 0, 0);
        }
      }
    }
    const int e = e0 + el;
    if (e < E) {
      const float b = bias ? bias[e] : 0.0f;
#pragma unroll
      for (int j = 0; j < kRouterTPT; ++j) {
        const int t = tile0 + tok_local + j;
        const float v = acc4[j / 4][j % 4];
        if (t < T) logits[(size_t)t * E + e] = bias ? v + b : v;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ top-k
// G lanes cooperate on one token.  Slot s takes the best score not taken yet (ties -> lower expert index);
// confidences are softmax probabilities of the chosen experts (max-subtracted, fp32).
template <int G>
__global__ void __launch_bounds__(256) topk_kernel(const float* __restrict__ logits, int32_t* __restrict__ expert_idx,
                                                   float* __restrict__ weights, int T, int E, int k, int normalize) {
  const int tid = threadIdx.x;
  const int sub = tid % G;
  const int t = blockIdx.x * (256 / G) + tid / G;
  const bool live = t < T;
  const float* lg = logits + (size_t)(live ? t : 0) * E;

  int sel[kMaxTopK];
  float selv[kMaxTopK];
#pragma unroll
  for (int s = 0; s < kMaxTopK; ++s) { sel[s] = -1; selv[s] = 0.0f; }

#pragma unroll
  for (int s = 0; s < kMaxTopK; ++s) {
    if (s < k) {
      float bv = -INFINITY;
      int bi = 0x7fffffff;
      for (int e = sub; e < E; e += G) {
        const float v = lg[e];
        bool taken = false;
#pragma unroll
        for (int u = 0; u < kMaxTopK; ++u) taken |= (u < s) && (sel[u] == e);
        if (!taken && (bi == 0x7fffffff || v > bv)) { bv = v; bi = e; }   // always lands on a valid expert
      }
#pragma unroll
      for (int off = G / 2; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, G);
        const int oi = __shfl_xor(bi, off, G);
        if (oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi))) { bv = ov; bi = oi; }
      }
      sel[s] = bi;
      selv[s] = bv;
    }
  }
  const float m = selv[0];
  float sum = 0.0f;
  for (int e = sub; e < E; e += G) sum += __expf(lg[e] - m);
#pragma unroll
  for (int off = G / 2; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, G);
  const float inv = 1.0f / sum;
  float w[kMaxTopK];
  float z = 0.0f;
#pragma unroll
  for (int s = 0; s < kMaxTopK; ++s) {
    w[s] = (s < k) ? __expf(selv[s] - m) * inv : 0.0f;
    z += w[s];
  }
  if (normalize) {
    const float iz = 1.0f / z;
#pragma unroll
    for (int s = 0; s < kMaxTopK; ++s) w[s] *= iz;
  }
  if (live && sub == 0) {
#pragma unroll
    for (int s = 0; s < kMaxTopK; ++s) {
      if (s < k) {
        expert_idx[(size_t)t * k + s] = sel[s];
        weights[(size_t)t * k + s] = w[s];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ stable grouping
// A chunk is 256 consecutive flat assignments f, handled by one wave in four steps of 64.  Lanes holding the
// same expert find each other with one ballot per bit of the expert index; the running per-expert count of
// the chunk lives in a wave-private LDS array.  No order-dependent atomics anywhere: ranks are deterministic.
constexpr int kChunk = 256;

template <class Emit>
__device__ __forceinline__ void chunk_ranks(const int32_t* __restrict__ expert_idx, int F, int chunk, int E, int nbits,
                                            int* cnt, Emit&& emit) {
  const int lane = threadIdx.x & 63;
  for (int e = lane; e < E; e += 64) cnt[e] = 0;
  __builtin_amdgcn_wave_barrier();
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int step = 0; step < kChunk / 64; ++step) {
    const int f = chunk * kChunk + step * 64 + lane;
    const bool valid = f < F;
    const int e = valid ? expert_idx[f] : 0;
    unsigned long long mask = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
      const bool bit = (e >> b) & 1;
      const unsigned long long bal = __ballot(valid && bit);
      mask &= bit ? bal : ~bal;
    }
    const int rank = __popcll(mask & below);
    const int size = __popcll(mask);
    const int base = valid ? cnt[e] : 0;
    __builtin_amdgcn_wave_barrier();
    if (valid && rank == 0) cnt[e] = base + size;
    __builtin_amdgcn_wave_barrier();
    if (valid) emit(f, e, base + rank);
  }
}

__global__ void __launch_bounds__(256) chunk_hist_kernel(const int32_t* __restrict__ expert_idx, int F, int E, int nbits,
                                                         int nchunks, int32_t* __restrict__ chunk_counts) {
  __shared__ int cnt_all[4 * kMaxExperts];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int* cnt = cnt_all + wave * kMaxExperts;
  const int chunk = blockIdx.x * 4 + wave;
  if (chunk >= nchunks) return;
  chunk_ranks(expert_idx, F, chunk, E, nbits, cnt, [](int, int, int) {});
  __builtin_amdgcn_wave_barrier();
  for (int e = lane; e < E; e += 64) chunk_counts[(size_t)chunk * E + e] = cnt[e];
}

// Single workgroup.  Turns chunk_counts into exclusive per-expert bases (in place), and writes
// tokens_per_expert, padded_offsets (rows per expert = ceil(n_e/128)*128, Section 5.2), counts and expert_order.
constexpr int kOffsetsThreads = 1024;          // threads of the one workgroup: up to 1024 / E lanes per expert
__global__ void __launch_bounds__(kOffsetsThreads) offsets_kernel(int32_t* __restrict__ chunk_counts, int nchunks, int E, int hb,
                                                              int db, int capacity, int pad_to_capacity,
                                                              int32_t* __restrict__ sched,
                                                       int32_t* __restrict__ tokens_per_expert,
                                                       int32_t* __restrict__ padded_offsets, int32_t* __restrict__ counts,
                                                       int32_t* __restrict__ expert_order,
                                                       int32_t* __restrict__ group_offsets) {
  __shared__ int n_s[kMaxExperts];
  __shared__ int scan_s[kMaxExperts];
  __shared__ int gscan_s[kMaxExperts];
  __shared__ int part_s[kOffsetsThreads];
  const int tid = threadIdx.x;
  // L threads share one expert's column of chunk_counts: each sums a contiguous range of chunks, the ranges are
  // scanned through LDS, then each thread rewrites its range as exclusive bases.
  int epow = 1;
  while (epow < E) epow <<= 1;
  const int L = kOffsetsThreads / epow;
  const int ex = tid % epow, part = tid / epow;
  const int per = (nchunks + L - 1) / L;
  const int cb = min(nchunks, part * per), ce = min(nchunks, cb + per);
  int mine = 0;
  if (ex < E)
    for (int c = cb; c < ce; ++c) mine += chunk_counts[(size_t)c * E + ex];
  part_s[tid] = mine;
  __syncthreads();
  int before = 0, n = 0;
  for (int l = 0; l < L; ++l) {
    const int v = part_s[l * epow + ex];
    before += l < part ? v : 0;
    n += v;
  }
  if (ex < E) {
    int run = before;
    for (int c = cb; c < ce; ++c) {
      const int v = chunk_counts[(size_t)c * E + ex];
      chunk_counts[(size_t)c * E + ex] = run;
      run += v;
    }
  }
  __syncthreads();
  if (tid >= E) n = 0;                      // threads 0..E-1 (part 0, ex == tid) own expert tid from here on
  // Token dropping (Section 2.2): an expert keeps at most `capacity` assignments (the first ones in flat order, see
  // rank_kernel); with pad_to_capacity every expert owns the capacity's worth of rows whatever its load.
  if (capacity > 0) n = min(n, capacity);
  if (tid < E) tokens_per_expert[tid] = n;
  const int padded = ((((pad_to_capacity && tid < E) ? capacity : n) + kBlock - 1) / kBlock) * kBlock;
  const bool slot = tid < kMaxExperts;      // the per-expert arrays have kMaxExperts entries
  if (slot) {
    n_s[tid] = n;
    scan_s[tid] = tid < E ? padded : 0;
    gscan_s[tid] = tid < E ? (padded / kBlock + 1) / 2 : 0;   // row groups: block-rows taken two at a time
  }
  __syncthreads();
  for (int off = 1; off < kMaxExperts; off <<= 1) {       // inclusive Hillis-Steele scans over experts
    const int add = (slot && tid >= off) ? scan_s[tid - off] : 0;
    const int gadd = (slot && tid >= off) ? gscan_s[tid - off] : 0;
    __syncthreads();
    if (slot) {
      scan_s[tid] += add;
      gscan_s[tid] += gadd;
    }
    __syncthreads();
  }
  if (tid < E) { padded_offsets[tid + 1] = scan_s[tid];  group_offsets[tid + 1] = gscan_s[tid]; }
  if (tid == 0) {
    group_offsets[0] = 0;
    padded_offsets[0] = 0;
    const int P = scan_s[E - 1];
    counts[0] = P;
    counts[1] = P / kBlock;
    counts[2] = (P / kBlock) * hb;
    counts[3] = 0;
    // Weight-gradient schedule.  With 256x256 macro tiles an expert owns ceil(hb/2)*ceil(db/2) tiles whose K is its
    // row count; a balanced schedule gives each of the 256 CUs R * tiles / 256 block-steps.  When the most loaded
    // expert's own tiles are much longer than that, the machine would idle behind them: use 128x128 tiles then.
    int max_rows = 0;
    for (int e = 0; e < E; ++e) max_rows = max(max_rows, (n_s[e] + kBlock - 1) / kBlock);
    const long long tiles = (long long)((hb + 1) / 2) * ((db + 1) / 2);
    const long long share = (long long)(P / kBlock) * tiles / 256;
    const bool heavy = 2LL * max_rows > 3 * share;
    sched[0] = (heavy && tiles < 256) ? 1 : 0;
    // Patch size for the weight-gradient tiles (tiles of one XCD patch share operand slabs in that XCD's L2).  The
    // patch -> XCD assignment is static, so patches are only used when they cannot unbalance the XCDs: no expert is
    // large against an XCD's share of the rows (a hot expert's patches all cost its row count, and nine of them over
    // eight XCDs cost 20 % on the skewed 64-expert configuration).  Otherwise the tiles are dealt out one by one,
    // heaviest expert first.
    sched[1] = (!heavy && 16LL * max_rows <= P / kBlock) ? 16 : 1;
    // DSD / DSD^T when the host launched them in both tile shapes: the macro tiles (row groups x pairs of d-blocks) run
    // in rounds of 256 at about 1.6 us per K tile, the single blocks (four per macro tile) in rounds of 512 at about
    // 1.0 us; take whichever needs less time
    const long long big_items = (long long)gscan_s[E - 1] * ((db + 1) / 2);
    const long long rounds_macro = (big_items + 255) / 256, rounds_single = ((long long)(P / kBlock) * db + 511) / 512;
    sched[2] = 10 * rounds_single < 16 * rounds_macro ? 1 : 0;
    sched[3] = 0;
  }
  if (tid < E) {                                           // position of expert `tid` in descending-load order
    int pos = 0;
    for (int o = 0; o < E; ++o) {
      const int no = n_s[o];
      pos += (no > n) || (no == n && o < tid);
    }
    expert_order[pos] = tid;
  }
}

__global__ void __launch_bounds__(256) rank_kernel(const int32_t* __restrict__ expert_idx, int F, int E, int nbits,
                                                   int nchunks, const int32_t* __restrict__ chunk_base,
                                                   const int32_t* __restrict__ padded_offsets, int capacity,
                                                   int32_t* __restrict__ row_of, int32_t* __restrict__ token_of) {
  __shared__ int cnt_all[4 * kMaxExperts];
  const int wave = threadIdx.x >> 6;
  int* cnt = cnt_all + wave * kMaxExperts;
  const int chunk = blockIdx.x * 4 + wave;
  if (chunk >= nchunks) return;
  const int32_t* base = chunk_base + (size_t)chunk * E;
  chunk_ranks(expert_idx, F, chunk, E, nbits, cnt, [&](int f, int e, int r) {
    const int rank = base[e] + r;                          // position of f among the assignments of expert e
    if (capacity > 0 && rank >= capacity) {                // over capacity: dropped (Section 2.2)
      row_of[f] = -1;
      return;
    }
    const int row = padded_offsets[e] + rank;
    row_of[f] = row;
    token_of[row] = f;
  });
}

// ------------------------------------------------------------------------------------------------ topology
// Expert owning block-row r: the last e with first_row[e] <= r (empty experts own nothing).
__device__ __forceinline__ int owner_of_block_row(const int* first_row, int E, int r) {
  int lo = 0, hi = E;                    // invariant: first_row[lo] <= r < first_row[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (first_row[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

// One thread per index.  Primary order numbers the nonzero blocks row by row (valid both as blocked CSR and
// as blocked COO); the transposed order lists, column by column, the block-row of each block and the number
// that block has in the primary order, so the values never have to be moved (Section 5.1.4).
__global__ void __launch_bounds__(256) topology_kernel(const int32_t* __restrict__ padded_offsets,
                                                       const int32_t* __restrict__ tokens_per_expert, int E, int hb,
                                                       int32_t* __restrict__ row_offsets, int32_t* __restrict__ column_indices,
                                                       int32_t* __restrict__ row_indices, int32_t* __restrict__ column_offsets_t,
                                                       int32_t* __restrict__ row_indices_t, int32_t* __restrict__ block_offsets_t,
                                                       int32_t* __restrict__ token_of, const int32_t* __restrict__ group_offsets,
                                                       int32_t* __restrict__ row_group) {
  __shared__ int first_row[kMaxExperts + 1];
  for (int e = threadIdx.x; e <= E; e += 256) first_row[e] = padded_offsets[e] / kBlock;
  __syncthreads();
  const int R = first_row[E];
  const int nnz = R * hb;
  const int P = R * kBlock;
  const int idx = blockIdx.x * 256 + threadIdx.x;

  if (idx < nnz) {
    const int r = idx / hb;
    const int e = owner_of_block_row(first_row, E, r);
    column_indices[idx] = e * hb + idx % hb;
    row_indices[idx] = r;
    const int rows_e = first_row[e + 1] - first_row[e];
    const int local = idx - hb * first_row[e];
    const int j = local / rows_e, jj = local % rows_e;
    row_indices_t[idx] = first_row[e] + jj;
    block_offsets_t[idx] = (first_row[e] + jj) * hb + j;
  }
  if (idx <= R) row_offsets[idx] = idx * hb;
  if (idx < R) {                           // row groups: rows 2i and 2i+1 of an expert share their column list
    const int e = owner_of_block_row(first_row, E, idx);
    const int local = idx - first_row[e];
    if ((local & 1) == 0) row_group[group_offsets[e] + (local >> 1)] = idx * 2 + (idx + 1 < first_row[e + 1]);
  }
  if (idx <= E * hb) {
    const int e = idx / hb, j = idx % hb;
    const int rows_e = e < E ? first_row[e + 1] - first_row[e] : 0;
    column_offsets_t[idx] = hb * first_row[e] + j * rows_e;
  }
  if (idx < P) {
    const int e = owner_of_block_row(first_row, E, idx / kBlock);
    if (idx - first_row[e] * kBlock >= tokens_per_expert[e]) token_of[idx] = -1;
  }
}

// ------------------------------------------------------------------------------------------------ launchers
static int pow2_at_least(int v, int cap) {
  int p = 1;
  while (p < v && p < cap) p <<= 1;
  return p;
}

void launch_router(const dmoe_config& c, const bf16_t* x, const bf16_t* wr, const float* bias,
                   const dmoe_topology_t& t, hipStream_t s) {
  const int T = c.num_tokens, d = c.d_model, E = c.num_experts;
  const int epad = pow2_at_least(E < 4 ? 4 : E, 64);
  // eight tokens per lane amortise the staging of Wr best, four give twice as many workgroups: use eight only when
  // that still leaves at least two workgroups per CU
#define DMOE_ROUTER_CASE(EP)                                                                                   \
  case EP: {                                                                                                   \
    constexpr int TT8 = 4 * (64 / EP) * 8, TT4 = 4 * (64 / EP) * 4;                                            \
    if ((T + TT8 - 1) / TT8 >= 512)                                                                            \
      hipLaunchKernelGGL((router_logits_kernel<EP, 8>), dim3((T + TT8 - 1) / TT8), dim3(256), 0, s, x, wr,     \
                         bias, t.logits, T, d, E);                                                             \
    else                                                                                                       \
      hipLaunchKernelGGL((router_logits_kernel<EP, 4>), dim3((T + TT4 - 1) / TT4), dim3(256), 0, s, x, wr,     \
                         bias, t.logits, T, d, E);                                                             \
  } break;
  switch (epad) {
    DMOE_ROUTER_CASE(4)
    DMOE_ROUTER_CASE(8)
    DMOE_ROUTER_CASE(16)
    DMOE_ROUTER_CASE(32)
    DMOE_ROUTER_CASE(64)
  }
#undef DMOE_ROUTER_CASE
  const int g = pow2_at_least(E, 64);
#define DMOE_TOPK_CASE(G)                                                                                      \
  case G:                                                                                                      \
    hipLaunchKernelGGL(topk_kernel<G>, dim3((T + 256 / G - 1) / (256 / G)), dim3(256), 0, s, t.logits,         \
                       t.expert_idx, t.weights, T, E, c.top_k, c.normalize_topk);                              \
    break;
  switch (g) {
    DMOE_TOPK_CASE(1)
    DMOE_TOPK_CASE(2)
    DMOE_TOPK_CASE(4)
    DMOE_TOPK_CASE(8)
    DMOE_TOPK_CASE(16)
    DMOE_TOPK_CASE(32)
    DMOE_TOPK_CASE(64)
  }
#undef DMOE_TOPK_CASE
}

void launch_sort(const dmoe_config& c, const dmoe_topology_t& t, int32_t* chunk_counts, int p_max, hipStream_t s) {
  (void)p_max;
  const int F = c.num_tokens * c.top_k, E = c.num_experts;
  const int nchunks = (F + kChunk - 1) / kChunk;
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  const int hb = c.ffn_hidden / kBlock;
  hipLaunchKernelGGL(chunk_hist_kernel, dim3((nchunks + 3) / 4), dim3(256), 0, s, t.expert_idx, F, E, nbits, nchunks,
                     chunk_counts);
  hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(kOffsetsThreads), 0, s, chunk_counts, nchunks, E, hb,
                     c.d_model / kBlock, c.expert_capacity, c.pad_to_capacity, t.sched, t.tokens_per_expert,
                     t.padded_offsets, t.counts, t.expert_order, t.group_offsets);
  hipLaunchKernelGGL(rank_kernel, dim3((nchunks + 3) / 4), dim3(256), 0, s, t.expert_idx, F, E, nbits, nchunks,
                     chunk_counts, t.padded_offsets, c.expert_capacity, t.row_of, t.token_of);
}

void launch_make_topology(const dmoe_config& c, const dmoe_topology_t& t, int p_max, int nnz_max, hipStream_t s) {
  const int hb = c.ffn_hidden / kBlock;
  int n = nnz_max > p_max ? nnz_max : p_max;
  if (c.num_experts * hb + 1 > n) n = c.num_experts * hb + 1;
  if (p_max / kBlock + 1 > n) n = p_max / kBlock + 1;
  hipLaunchKernelGGL(topology_kernel, dim3((n + 255) / 256), dim3(256), 0, s, t.padded_offsets, t.tokens_per_expert,
                     c.num_experts, hb, t.row_offsets, t.column_indices, t.row_indices, t.column_offsets_t,
                     t.row_indices_t, t.block_offsets_t, t.token_of, t.group_offsets, t.row_group);
}

}  // namespace dmoe
