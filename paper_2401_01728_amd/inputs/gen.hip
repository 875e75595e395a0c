// Device twin of inputs/gen.py: fills device buffers with the same counter-based
// pseudo-random values, bit for bit (integer hash, integer Irwin-Hall sum, then two
// separately rounded fp32 operations).  Draws numbers only; none of the method's
// arithmetic lives here.  Built as its own shared library (librvgen.so).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__host__ __device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
  return x;
}
__host__ __device__ inline uint32_t make_key(uint32_t seed, uint32_t stream) {
  return mix32(mix32(seed + 0x9E3779B9u) ^ stream);
}
__device__ inline uint32_t word(uint32_t key, uint64_t index, uint32_t w) {
  uint64_t ctr = index * 4ull + w;
  uint32_t h = mix32((uint32_t)ctr + key);
  return mix32(h ^ (uint32_t)(ctr >> 32) ^ 0x68E31DA4u);
}
__global__ void fill_normal_kernel(void* out, uint64_t n, uint32_t key, float mean, float std_,
                                   uint64_t offset, float scale, int as_bf16) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int32_t acc = 0;
#pragma unroll
    for (uint32_t w = 0; w < 4; ++w) {
      uint32_t h = word(key, i + offset, w);
      acc += (int32_t)(h & 0xFFFFu) + (int32_t)(h >> 16);
    }
    float z = __fmul_rn((float)(acc - 262140), scale);
    float v = __fadd_rn(__fmul_rn(z, std_), mean);
    if (as_bf16) {
      uint32_t b = __float_as_uint(v);
      b += 0x7FFFu + ((b >> 16) & 1u);
      ((uint16_t*)out)[i] = (uint16_t)(b >> 16);
    } else {
      ((float*)out)[i] = v;
    }
  }
}

__global__ void fill_uniform_kernel(float* out, uint64_t n, uint32_t key, float lo, float hi,
                                    uint64_t offset) {
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  const float span = __fsub_rn(hi, lo);
  for (; i < n; i += stride) {
    uint32_t h = word(key, i + offset, 0);
    float u = __fmul_rn((float)(h >> 8), 5.9604644775390625e-08f);
    out[i] = __fadd_rn(__fmul_rn(u, span), lo);
  }
}

unsigned grid_for(uint64_t n) {
  uint64_t b = (n + 255) / 256;
  return (unsigned)(b > 65536 ? 65536 : (b ? b : 1));
}

}  // namespace

// scale: the fp32 unit-variance constant, passed from Python so both sides use one value.
extern "C" int rvgen_fill_normal(void* out, uint64_t n, uint32_t seed, uint32_t stream, float mean,
                                 float std_, uint64_t offset, float scale, int as_bf16, void* hip_stream) {
  if (!out) return -1;
  if (n == 0) return 0;
  hipLaunchKernelGGL(fill_normal_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)hip_stream, out,
                     n, make_key(seed, stream), mean, std_, offset, scale, as_bf16);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

extern "C" int rvgen_fill_uniform(float* out, uint64_t n, uint32_t seed, uint32_t stream, float lo,
                                  float hi, uint64_t offset, void* hip_stream) {
  if (!out) return -1;
  if (n == 0) return 0;
  hipLaunchKernelGGL(fill_uniform_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)hip_stream, out,
                     n, make_key(seed, stream), lo, hi, offset);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
