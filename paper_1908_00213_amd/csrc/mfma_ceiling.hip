// Measurement aid (stand-alone program, not part of libchn.so): what the matrix cores of this GPU
// sustain on bf16 MFMAs, so that the GEMM kernel's fraction of the published peak can be read against
// what the silicon delivers at the clock it actually holds.
//
// One workgroup of four waves per compute unit; every wave keeps a 128x128 fp32 accumulator tile in
// registers, like the GEMM kernel, and issues 32x32x16 bf16 MFMAs back to back: no memory traffic at
// all in the first two legs.  Each leg reports the rate, the shader clock (cycle counter against the
// 100 MHz wall counter) and the cycles per 16 MFMAs (512 = the pipeline never idles).
//   leg 1  all operands 1.0                 (few bits toggle: the highest clock)
//   leg 2  pseudo-random operands           (what training data looks like to the multipliers)
//   leg 3  random operands, fragments re-read from LDS every 16 MFMAs and one barrier per 32, in the
//          software-pipelined order of the GEMM kernel's inner loop
// Build: hipcc --offload-arch=gfx950 -O3 mfma_ceiling.hip -o mfma_ceiling      Run: ./mfma_ceiling
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } } while (0)

__device__ __forceinline__ uint32_t two_bf16(uint32_t &h, bool random) {
  if (!random) return 0x3f803f80u;
  h ^= h << 13; h ^= h >> 17; h ^= h << 5;
  return (h & 0x807f807fu) | 0x3f003f00u | ((h >> 3) & 0x00800080u);   // sign, exponent 126/127, random mantissa
}

__device__ __forceinline__ void mma16(floatx16 (&acc)[16], const u32x4 (&a)[4], const u32x4 (&b)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]), acc[i * 4 + j], 0, 0, 0);
}

template <bool RANDOM, bool LDS>
__global__ __launch_bounds__(256) void ceiling_kernel(int iters, uint64_t *out, float *sink) {
  __shared__ __attribute__((aligned(16))) u32x4 buf[4096];   // 64 KB, as much as two operand tiles of a tile step
  uint32_t h = (threadIdx.x + 1) * 2654435761u + blockIdx.x * 40503u;
  for (int i = threadIdx.x; i < 4096; i += 256) buf[i] = u32x4{two_bf16(h, RANDOM), two_bf16(h, RANDOM), two_bf16(h, RANDOM), two_bf16(h, RANDOM)};
  __syncthreads();
  floatx16 acc[16];
  for (int i = 0; i < 16; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  u32x4 a0[4], b0[4], a1[4], b1[4];
  int off = threadIdx.x;
  auto read = [&](u32x4 (&a)[4], u32x4 (&b)[4]) {   // every index stays inside buf: masked with 4095
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = buf[(off + i * 257) & 4095]; b[i] = buf[(off + 1024 + i * 257) & 4095]; }
    off += 64;
  };
  read(a0, b0);
  const uint64_t c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; it += 2) {
    if (LDS) {
      read(a1, b1);
      mma16(acc, a0, b0);
#pragma unroll
      for (int g = 0; g < 8; ++g) { __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); }
      __syncthreads();
      read(a0, b0);
      mma16(acc, a1, b1);
#pragma unroll
      for (int g = 0; g < 8; ++g) { __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); __builtin_amdgcn_sched_group_barrier(0x008, 2, 0); }
    } else {
      mma16(acc, a0, b0);
      mma16(acc, a0, b0);
    }
  }
  const uint64_t c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
  for (int i = 0; i < 16; ++i) for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 12345.678f) sink[0] = s;   // keeps the accumulators alive
  if (threadIdx.x == 0) { out[blockIdx.x * 2] = c1 - c0; out[blockIdx.x * 2 + 1] = w1 - w0; }
}

template <bool RANDOM, bool LDS>
static void leg(int blocks, int iters, uint64_t *d_out, float *d_sink, const char *name) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  hipLaunchKernelGGL((ceiling_kernel<RANDOM, LDS>), dim3(blocks), dim3(256), 0, 0, iters / 8, d_out, d_sink);   // warm-up
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  hipLaunchKernelGGL((ceiling_kernel<RANDOM, LDS>), dim3(blocks), dim3(256), 0, 0, iters, d_out, d_sink);
  CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  uint64_t *h = (uint64_t *)malloc((size_t)blocks * 16);
  CHECK(hipMemcpy(h, d_out, (size_t)blocks * 16, hipMemcpyDeviceToHost));
  double cyc = 0, wall = 0;
  for (int i = 0; i < blocks; ++i) { cyc += (double)h[2 * i]; wall += (double)h[2 * i + 1]; }
  const double flop = (double)blocks * 4 * iters * 16 * 32768.0;
  printf("%-44s %8.1f us  %6.0f TFLOP/s  shader clock %4.0f MHz  %6.1f cycles per 16 MFMAs\n", name, ms * 1e3,
         flop / (ms * 1e-3) / 1e12, cyc / wall * 100.0, cyc / blocks / iters);
  free(h);
}

int main() {
  hipDeviceProp_t p;
  CHECK(hipGetDeviceProperties(&p, 0));
  const int blocks = p.multiProcessorCount;
  printf("%s, %d compute units; bf16 32x32x16 MFMA, 4 waves per compute unit\n", p.name, blocks);
  uint64_t *d_out; float *d_sink;
  CHECK(hipMalloc(&d_out, (size_t)blocks * 16)); CHECK(hipMalloc(&d_sink, 4));
  for (int rep = 0; rep < 2; ++rep) {
    leg<false, false>(blocks, 32000, d_out, d_sink, "MFMA only, operands all 1.0");
    leg<true, false>(blocks, 32000, d_out, d_sink, "MFMA only, random operands");
    leg<true, true>(blocks, 32000, d_out, d_sink, "random operands, LDS fragment reads + barrier");
  }
  return 0;
}
