// Vendor yardstick for the kernel-level comparison of Figure 9 / Section 6.3: the paper sets its block-sparse
// products, under a uniform assignment of tokens to experts, against the vendor library's dense BATCHED matrix
// multiplication on the same shapes.  This program times rocBLAS' strided-batched bf16 GEMM (fp32 accumulation) for
// the six products of the per-GPU problems of dMoE-XS / -Small / -Medium (8 local experts; Table 1 hidden sizes;
// micro-batch x 1024 tokens) and prints one JSON line.  It runs in a process of its own, on buffers of its own: it
// shares nothing with the dMoE library (bench_uniform_vs_bmm.py measures that side and reads this program's output).
//
// Operand layouts are the vendor's best case, one contiguous matrix per expert (the library's own layout interleaves
// the experts' weight columns, which a batched GEMM would need a stride for):
//   forward  layer 1   [n, d] x [d, h]        backward data    layer 2   [n, d] x [h, d]^T
//   forward  layer 2   [n, h] x [h, d]        backward weights layer 2   [n, h]^T x [n, d]
//                                             backward data    layer 1   [n, h] x [d, h]^T
//                                             backward weights layer 1   [n, d]^T x [n, h]
// with n = tokens / experts rows per expert.  Row-major products are handed to the column-major library as the
// transposed product (C^T = B^T A^T).
//
//   hipcc --offload-arch=gfx950 -O2 bench_vendor_bmm.cpp -lrocblas -o bench_vendor_bmm
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include <algorithm>

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 1; } } while (0)
#define CHECK_BLAS(x) do { rocblas_status s_ = (x); if (s_ != rocblas_status_success) { fprintf(stderr, "rocBLAS error %d at %s:%d\n", (int)s_, __FILE__, __LINE__); return 1; } } while (0)

struct Model { const char* name; int tokens, d, h, experts; };
struct Problem { const char* product; int m, n, k; int a_trans, b_trans; };   // row-major C[m,n] = op(A) op(B)

static unsigned short bf16_of(float f) {
  unsigned u;
  memcpy(&u, &f, 4);
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

int main(int argc, char** argv) {
  int iters = 30, warmup = 5;
  for (int i = 1; i + 1 < argc; ++i) {
    if (!strcmp(argv[i], "--iters")) iters = atoi(argv[i + 1]);
    if (!strcmp(argv[i], "--warmup")) warmup = atoi(argv[i + 1]);
  }
  // the three per-GPU problems of Section 6.3, and (with --large) the shape of this build's largest configuration
  // (8 experts of 4096 x 14336 with 8192 rows each), which the paper does not have
  bool large = false;
  for (int i = 1; i < argc; ++i) if (!strcmp(argv[i], "--large")) large = true;
  const Model all_models[4] = {{"xs", 64 * 1024, 512, 2048, 8}, {"small", 32 * 1024, 1024, 4096, 8}, {"medium", 8 * 1024, 1536, 6144, 8},
                               {"large", 64 * 1024, 4096, 14336, 8}};
  std::vector<Model> models(all_models, all_models + (large ? 4 : 3));
  rocblas_handle handle;
  CHECK_BLAS(rocblas_create_handle(&handle));
  hipStream_t stream;
  CHECK_HIP(hipStreamCreate(&stream));
  CHECK_BLAS(rocblas_set_stream(handle, stream));
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  printf("{\"metric\": \"rocBLAS strided-batched bf16 GEMM on the Figure 9 problems\", \"unit\": \"TFLOP/s\", \"iters\": %d, \"problems\": [", iters);
  bool first = true;
  for (const Model& md : models) {
    const int E = md.experts, n = md.tokens / E, d = md.d, h = md.h;
    const Problem problems[6] = {
        {"sdd", n, h, d, 0, 0},    // [n,d] x [d,h]
        {"dsd", n, d, h, 0, 0},    // [n,h] x [h,d]
        {"sddt", n, h, d, 0, 1},   // [n,d] x [h,d]^T
        {"dstd", h, d, n, 1, 0},   // [n,h]^T x [n,d]
        {"dsdt", n, d, h, 0, 1},   // [n,h] x [d,h]^T
        {"ddts", d, h, n, 1, 0},   // [n,d]^T x [n,h]
    };
    // every operand of every problem fits in three buffers of the largest matrix: n*h, d*h or n*d elements per expert
    const size_t per = std::max({(size_t)n * h, (size_t)d * h, (size_t)n * d});
    const size_t elems = per * E;
    unsigned short *A = nullptr, *B = nullptr, *C = nullptr;
    CHECK_HIP(hipMalloc(&A, elems * 2));
    CHECK_HIP(hipMalloc(&B, elems * 2));
    CHECK_HIP(hipMalloc(&C, elems * 2));
    {
      std::vector<unsigned short> host(elems);
      unsigned seed = 12345u;
      for (size_t i = 0; i < elems; ++i) {
        seed = seed * 1664525u + 1013904223u;
        host[i] = bf16_of(((int)(seed >> 9) % 2001 - 1000) * 1e-3f);        // uniform in [-1, 1]
      }
      CHECK_HIP(hipMemcpy(A, host.data(), elems * 2, hipMemcpyHostToDevice));
      for (size_t i = 0; i < elems; ++i) host[i] = bf16_of(0.02f * (float)((int)(host[i] >> 3) % 201 - 100) * 1e-2f);
      CHECK_HIP(hipMemcpy(B, host.data(), elems * 2, hipMemcpyHostToDevice));
      CHECK_HIP(hipMemset(C, 0, elems * 2));
    }
    for (const Problem& p : problems) {
      // row-major C[m,n] = op(A) op(B)  ==  column-major C^T[n,m] = op(B)^T op(A)^T: operands swapped; a row-major
      // matrix read as column-major is its transpose, so a row-major "not transposed" operand needs no flag
      const int m = p.m, nn = p.n, k = p.k;
      const rocblas_operation op_first = p.b_trans ? rocblas_operation_transpose : rocblas_operation_none;    // B
      const rocblas_operation op_second = p.a_trans ? rocblas_operation_transpose : rocblas_operation_none;   // A
      const int ld_b = p.b_trans ? k : nn;          // row-major B is [k,n] (ld n) or, transposed, [n,k] (ld k)
      const int ld_a = p.a_trans ? m : k;           // row-major A is [m,k] (ld k) or, transposed, [k,m] (ld m)
      const long long stride_a = (long long)m * k, stride_b = (long long)k * nn, stride_c = (long long)m * nn;
      if ((size_t)stride_a > per || (size_t)stride_b > per || (size_t)stride_c > per) { fprintf(stderr, "buffer too small\n"); return 1; }
      const float alpha = 1.0f, beta = 0.0f;
      auto run = [&]() {
        return rocblas_gemm_strided_batched_ex(handle, op_first, op_second, nn, m, k, &alpha, B, rocblas_datatype_bf16_r, ld_b,
                                               stride_b, A, rocblas_datatype_bf16_r, ld_a, stride_a, &beta, C,
                                               rocblas_datatype_bf16_r, nn, stride_c, C, rocblas_datatype_bf16_r, nn, stride_c, E,
                                               rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
      };
      for (int i = 0; i < warmup; ++i) CHECK_BLAS(run());
      CHECK_HIP(hipStreamSynchronize(stream));
      CHECK_HIP(hipEventRecord(e0, stream));
      for (int i = 0; i < iters; ++i) CHECK_BLAS(run());
      CHECK_HIP(hipEventRecord(e1, stream));
      CHECK_HIP(hipEventSynchronize(e1));
      float ms = 0.0f;
      CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
      ms /= iters;
      const double tflops = 2.0 * md.tokens * (double)d * h / (ms * 1e-3) / 1e12;
      printf("%s{\"model\": \"%s\", \"product\": \"%s\", \"m\": %d, \"n\": %d, \"k\": %d, \"batch\": %d, \"ms\": %.4f, \"tflops\": %.1f}",
             first ? "" : ", ", md.name, p.product, m, nn, k, E, ms, tflops);
      first = false;
      fprintf(stderr, "[vendor] %-6s %-5s m=%d n=%d k=%d x%d: %.3f ms, %.0f TFLOP/s\n", md.name, p.product, m, nn, k, E, ms, tflops);
      fflush(stderr);
    }
    CHECK_HIP(hipFree(A));
    CHECK_HIP(hipFree(B));
    CHECK_HIP(hipFree(C));
  }
  printf("]}\n");
  rocblas_destroy_handle(handle);
  return 0;
}
