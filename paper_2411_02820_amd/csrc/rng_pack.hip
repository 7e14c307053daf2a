// Counter-based synthetic-data generator and weight (re)packing kernels.
//
// Generator: element idx of stream `stream_id` under `seed`:
//   key = mix64(seed*G + stream_id*H + C);  a = mix64(key + 2*idx*G);  b = mix64(key + (2*idx+1)*G)
//   z   = (sum of the eight 16-bit lanes of a and b) - 262140
//   val = fl32(fl32(z)*scale) [+ offset, one more fp32 rounding, when offset != 0]
// mix64 is the SplitMix64 output function.  Integer operations plus explicitly rounded fp32
// multiply/add only, so a host implementation reproduces every bit.
#include <math.h>

#include "dsk_internal.h"

namespace {

constexpr uint64_t kG = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kH = 0xD1342543DE82EF95ull;
constexpr uint64_t kC = 0x632BE59BD9B4E019ull;

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

inline uint64_t stream_key(uint64_t seed, uint64_t stream_id) { return mix64(seed * kG + stream_id * kH + kC); }

inline float scale_for_std(float std) {
  const double lane_sum_std = sqrt(8.0 * (4294967296.0 - 1.0) / 12.0);
  return (float)((double)std / lane_sum_std);
}

__device__ __forceinline__ uint32_t lane_sum(uint64_t a) {
  return (uint32_t)(a & 0xFFFF) + (uint32_t)((a >> 16) & 0xFFFF) + (uint32_t)((a >> 32) & 0xFFFF) + (uint32_t)(a >> 48);
}

__device__ __forceinline__ float ih8(uint64_t key, uint64_t idx, float scale, float offset) {
#pragma clang fp contract(off)  // the multiply and the add round separately, as the definition says
  uint64_t c = key + (2 * idx) * kG;
  uint32_t s = lane_sum(mix64(c)) + lane_sum(mix64(c + kG));
  float v = (float)((int)s - 262140) * scale;
  if (offset != 0.0f) v = v + offset;
  return v;
}

__host__ __device__ inline int64_t packed_row(int map, int gu_block, int64_t row_off, int64_t r) {
  if (map == 0) return row_off + r;
  int64_t blk = r / gu_block, w = r % gu_block;
  return blk * 2 * gu_block + (map == 2 ? gu_block : 0) + w;
}

template <typename T>
__global__ void fill_normal_kernel(T* dst, int64_t n, uint64_t key, float scale, float offset, int64_t idx0) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = from_f32<T>(ih8(key, (uint64_t)(idx0 + i), scale, offset));
}

template <typename T>
__global__ void fill_weight_kernel(T* packed, int64_t rows, int64_t cols, int map, int gu_block, int64_t row_off,
                                   uint64_t key, float scale, float offset) {
  int64_t n = rows * cols;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int64_t r = i / cols, c = i - r * cols;
    packed[packed_row(map, gu_block, row_off, r) * cols + c] = from_f32<T>(ih8(key, (uint64_t)i, scale, offset));
  }
}

template <typename T>
__global__ void pack_rows_kernel(T* packed, T* logical, int64_t rows, int64_t cols, int map, int gu_block,
                                 int64_t row_off, int to_packed) {
  int64_t n = rows * cols;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int64_t r = i / cols, c = i - r * cols;
    int64_t p = packed_row(map, gu_block, row_off, r) * cols + c;
    if (to_packed) packed[p] = logical[i];
    else logical[i] = packed[p];
  }
}

inline int grid_for(int64_t n) {
  int64_t b = (n + 255) / 256;
  if (b > 256 * 64) b = 256 * 64;
  if (b < 1) b = 1;
  return (int)b;
}

}  // namespace

hipError_t launch_fill_normal(void* dst, int64_t n, uint64_t seed, uint64_t stream_id, float std, float offset,
                              int64_t idx0, int dtype, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  uint64_t key = stream_key(seed, stream_id);
  float scale = scale_for_std(std);
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(fill_normal_kernel<float>, dim3(grid_for(n)), dim3(256), 0, s, (float*)dst, n, key, scale, offset, idx0);
  else
    hipLaunchKernelGGL(fill_normal_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, s, (bf16_t*)dst, n, key, scale, offset, idx0);
  return hipGetLastError();
}

hipError_t launch_fill_weight(int dtype, void* packed, int64_t rows, int64_t cols, int map, int gu_block, int64_t row_off,
                              uint64_t seed, uint64_t stream_id, float std, float offset, hipStream_t s) {
  int64_t n = rows * cols;
  if (n <= 0) return hipSuccess;
  uint64_t key = stream_key(seed, stream_id);
  float scale = scale_for_std(std);
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(fill_weight_kernel<float>, dim3(grid_for(n)), dim3(256), 0, s, (float*)packed, rows, cols, map,
                       gu_block, row_off, key, scale, offset);
  else
    hipLaunchKernelGGL(fill_weight_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, s, (bf16_t*)packed, rows, cols, map,
                       gu_block, row_off, key, scale, offset);
  return hipGetLastError();
}

hipError_t launch_pack_rows(int dtype, void* packed, const void* logical, int64_t rows, int64_t cols, int map,
                            int gu_block, int64_t row_off, int to_packed, hipStream_t s) {
  int64_t n = rows * cols;
  if (n <= 0) return hipSuccess;
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(pack_rows_kernel<float>, dim3(grid_for(n)), dim3(256), 0, s, (float*)packed, (float*)logical, rows,
                       cols, map, gu_block, row_off, to_packed);
  else
    hipLaunchKernelGGL(pack_rows_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, s, (bf16_t*)packed, (bf16_t*)logical,
                       rows, cols, map, gu_block, row_off, to_packed);
  return hipGetLastError();
}
