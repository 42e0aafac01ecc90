// Random initial code book (paper: option -c; without an initial code book the map starts from random values).
// Element e of the code book gets a uniform [0,1) value from a counter-based generator:
// a 64-bit mix (splitmix64 finaliser) of seed + e * golden-ratio increment, top 24 bits.
#include "som_internal.hpp"

namespace som {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void k_fill_uniform(float *__restrict__ W, int64_t count, uint64_t seed) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; e < count; e += stride) {
    const uint64_t r = mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(e + 1));
    W[e] = (float)(r >> 40) * (1.0f / 16777216.0f);
  }
}

hipError_t launch_fill_uniform(som_ctx *c, float *W, int64_t count, uint64_t seed) {
  int64_t blocks = (count + 255) / 256;
  if (blocks > (int64_t)c->n_cu * 32) blocks = (int64_t)c->n_cu * 32;
  hipLaunchKernelGGL(k_fill_uniform, dim3((unsigned)blocks), dim3(256), 0, c->stream, W, count, seed);
  return hipGetLastError();
}

// Which XCD (accelerator complex, each with an L2 of its own) every workgroup of a one-dimensional launch
// runs on.  The dense filter and the sparse sweep place the workgroups that share data 8 apart on the
// assumption that the dispatcher deals consecutive workgroups round-robin to the eight XCDs; that is a
// property of the hardware scheduler, not of the programming model, so a test reads it back.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__global__ __launch_bounds__(64) void k_probe_xcc(int32_t *__restrict__ out) {
  unsigned id;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
  if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)(id & 0xf);
}
#pragma clang diagnostic pop

hipError_t launch_probe_xcc(hipStream_t stream, int32_t *out, int n_blocks) {
  hipLaunchKernelGGL(k_probe_xcc, dim3((unsigned)n_blocks), dim3(64), 0, stream, out);
  return hipGetLastError();
}

}  // namespace som
