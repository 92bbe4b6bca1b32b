// Kernel argument block of the GEMM kernels (shared by the host API and the kernel families).
#pragma once
#include <stdint.h>

namespace chn {
namespace gemm {

struct GemmArgs {
  const void *A, *B;
  void *C;
  int M, N, K;
  int64_t lda, ldb, ldc;  // elements; for a K-contiguous operand the stride between rows (m or n),
                          // otherwise the stride between consecutive k
  float alpha, beta;
  int epi;
  int c_bf16;             // C / aux / preact dtype: 0 fp32, 1 bf16
  const float *bias;
  const void *aux;
  int64_t ldaux;
  void *pre;
  int64_t ldpre;
  int piece;              // bytes per global load piece (16, 8 or the item size), common to A and B
  int piece_a, piece_b;   // what A and B would allow each (the 64x64 tile takes them apart when one is element-wise and the other whole)
  int piece_exact;        // the same when no piece may hang over the end of a row (direct-copy kernels)
  int tiles_m, tiles_n;
  int tile;               // macro tile: 2 = 256x256, 1 = 128x128, 0 = 64x64
  int splits;             // number of K splits (1 = none)
  float *partial;         // split-K: [splits][M][ldp] fp32 partial sums in the caller's workspace
  int64_t ldp;
  int epi_vec;            // C, aux, preact and bias allow aligned 4-element vector accesses
  int dma;                // big tile: K-contiguous operands go to LDS by direct global-to-LDS loads
  int w8;                 // ... by the kernel that works with eight waves (bf16)
  float *colsum;          // activation-gradient epilogues, 256x256 tile only: [M / 128][N] column sums of C over
                          // blocks of 128 rows (values as stored), or NULL
  int64_t ldcs;
};

}  // namespace gemm
}  // namespace chn
