// Memory-bound pieces of the decoder layer: RMSNorm, rotary table, RoPE + KV-cache write, SwiGLU.
// All arithmetic in fp32 (the rotary angle in fp64); storage type T is float or bf16.
#include "dsk_internal.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// y = x * rsqrt(mean(x^2) + eps) * g, one 256-thread block per token row (any d; scalar accesses).
template <typename TX, typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const TX* __restrict__ x, const T* __restrict__ g, T* __restrict__ y,
                                                      int d, float eps) {
  __shared__ float part[4];
  const TX* xr = x + (int64_t)blockIdx.x * d;
  T* yr = y + (int64_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float v = to_f32(xr[i]);
    ss += v * v;
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = part[0] + part[1] + part[2] + part[3];
  float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) yr[i] = from_f32<T>(to_f32(xr[i]) * r * to_f32(g[i]));
}

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
__device__ __forceinline__ f32x4_t load4(const float* p) { return *(const f32x4_t*)p; }
__device__ __forceinline__ f32x4_t load4(const bf16_t* p) {
  bf16x4_t v = *(const bf16x4_t*)p;
  f32x4_t r = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
  return r;
}

// Same for bf16 output with d a multiple of 4 and d <= 4*256*NCH: the row is read once (16- or 8-byte
// vectors), kept in registers across the reduction, and written as 8-byte vectors.
template <typename TX, int NCH>
__global__ void __launch_bounds__(256) rmsnorm_vec_kernel(const TX* __restrict__ x, const bf16_t* __restrict__ g,
                                                          bf16_t* __restrict__ y, int d, float eps) {
  __shared__ float part[4];
  const TX* xr = x + (int64_t)blockIdx.x * d;
  bf16_t* yr = y + (int64_t)blockIdx.x * d;
  f32x4_t v[NCH];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = (threadIdx.x + c * 256) * 4;
    if (i < d) {
      v[c] = load4(xr + i);
      ss += v[c][0] * v[c][0] + v[c][1] * v[c][1] + v[c][2] * v[c][2] + v[c][3] * v[c][3];
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = part[0] + part[1] + part[2] + part[3];
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = (threadIdx.x + c * 256) * 4;
    if (i < d) {
      f32x4_t gg = load4(g + i);
      bf16x4_t o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(v[c][e] * r * gg[e]);
      *(bf16x4_t*)(yr + i) = o;
    }
  }
}

// cos/sin of position * theta_i, angle and sincos in fp64, stored as fp32.
__global__ void rope_table_kernel(const int32_t* __restrict__ pos, const double* __restrict__ theta,
                                  float2* __restrict__ cs, int T, int half) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)T * half) return;
  int t = (int)(i / half), j = (int)(i - (int64_t)t * half);
  double s, c;
  sincos((double)pos[t] * theta[j], &s, &c);
  cs[i] = make_float2((float)c, (float)s);
}

// One block per token.  q and k heads: pair (i, i+dh/2) rotated; rotated k and v go to the cache rows.
template <typename T>
__global__ void __launch_bounds__(256) rope_kv_write_kernel(T* __restrict__ qkv, const float2* __restrict__ cs,
                                                            T* __restrict__ k_rows, T* __restrict__ v_rows, int Hq,
                                                            int Hkv, int dh) {
  const int t = blockIdx.x;
  const int half = dh >> 1;
  const int n_qkv = (Hq + 2 * Hkv) * dh;
  T* row = qkv + (int64_t)t * n_qkv;
  const float2* csr = cs + (int64_t)t * half;
  T* kr = k_rows + (int64_t)t * Hkv * dh;
  T* vr = v_rows + (int64_t)t * Hkv * dh;
  const int n_pairs = (Hq + Hkv) * half;
  for (int p = threadIdx.x; p < n_pairs; p += 256) {
    int head = p / half, i = p - head * half;
    float2 c = csr[i];
    T* hp = row + head * dh;
    float x1 = to_f32(hp[i]), x2 = to_f32(hp[i + half]);
    T y1 = from_f32<T>(x1 * c.x - x2 * c.y);
    T y2 = from_f32<T>(x2 * c.x + x1 * c.y);
    if (head < Hq) {
      hp[i] = y1;
      hp[i + half] = y2;
    } else {
      T* kp = kr + (head - Hq) * dh;
      kp[i] = y1;
      kp[i + half] = y2;
    }
  }
  const T* vsrc = row + (Hq + Hkv) * dh;
  for (int e = threadIdx.x; e < Hkv * dh; e += 256) vr[e] = vsrc[e];
}

// bf16, head_dim a multiple of 16: a lane handles eight neighbouring pairs (i, i + dh/2) of one head (two
// 16-byte loads, two 16-byte stores, 64 bytes of the cos/sin row) or copies 16 bytes of v; the work items of all
// tokens form one flat index space so that every lane of every workgroup has one.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
__global__ void __launch_bounds__(256) rope_kv_write_vec_kernel(bf16_t* __restrict__ qkv, const float2* __restrict__ cs,
                                                                bf16_t* __restrict__ k_rows, bf16_t* __restrict__ v_rows,
                                                                int T, int Hq, int Hkv, int dh) {
  const int half = dh >> 1, cph = half >> 3;  // 8-pair chunks per head
  const int n_rope = (Hq + Hkv) * cph, n_v = Hkv * dh / 8, per_tok = n_rope + n_v;
  const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (w >= (int64_t)T * per_tok) return;
  const int t = (int)(w / per_tok), c = (int)(w - (int64_t)t * per_tok);
  bf16_t* row = qkv + (int64_t)t * (Hq + 2 * Hkv) * dh;
  if (c >= n_rope) {
    const int e = (c - n_rope) * 8;
    *(bf16x8_t*)(v_rows + (int64_t)t * Hkv * dh + e) = *(const bf16x8_t*)(row + (Hq + Hkv) * dh + e);
    return;
  }
  const int head = c / cph, i0 = (c - head * cph) * 8;
  const float2* csr = cs + (int64_t)t * half + i0;
  bf16_t* hp = row + head * dh + i0;
  const bf16x8_t x1 = *(const bf16x8_t*)hp, x2 = *(const bf16x8_t*)(hp + half);
  bf16x8_t y1, y2;
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const f32x4_t c2 = *(const f32x4_t*)(csr + e);  // (cos, sin) of pairs e and e+1
    const float a0 = (float)x1[e], b0 = (float)x2[e], a1 = (float)x1[e + 1], b1 = (float)x2[e + 1];
    y1[e] = (bf16_t)(a0 * c2[0] - b0 * c2[1]);
    y2[e] = (bf16_t)(b0 * c2[0] + a0 * c2[1]);
    y1[e + 1] = (bf16_t)(a1 * c2[2] - b1 * c2[3]);
    y2[e + 1] = (bf16_t)(b1 * c2[2] + a1 * c2[3]);
  }
  bf16_t* dst = head < Hq ? hp : k_rows + (int64_t)t * Hkv * dh + (head - Hq) * dh + i0;
  *(bf16x8_t*)dst = y1;
  *(bf16x8_t*)(dst + half) = y2;
}

template <typename T>
__global__ void swiglu_kernel(const T* __restrict__ gu, T* __restrict__ act, int64_t n, int F, int gu_block) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int64_t t = i / F;
    int f = (int)(i - t * F);
    int pg = (f / gu_block) * 2 * gu_block + (f % gu_block);
    const T* r = gu + t * 2 * F;
    float g = to_f32(r[pg]), u = to_f32(r[pg + gu_block]);
    act[i] = from_f32<T>(g / (1.0f + __expf(-g)) * u);
  }
}

// Link emulation for the loading-strategy experiments: the load stream notes when a call's loads begin and,
// after each chunk, idles until the moment that chunk would have arrived over a link of the chosen rate.
// Time is the constant-rate (100 MHz) counter; the wait ends at its deadline, or after kPaceCap ticks at
// the latest, so the wave always retires.
constexpr unsigned long long kPaceCap = 500000000ull;  // 5 s
__global__ void pace_start_kernel(unsigned long long* t0) { *t0 = __builtin_amdgcn_s_memrealtime(); }
__global__ void pace_wait_kernel(const unsigned long long* t0, unsigned long long ticks) {
  const unsigned long long start = *t0;
  if (ticks > kPaceCap) ticks = kPaceCap;
  while (__builtin_amdgcn_s_memrealtime() - start < ticks) __builtin_amdgcn_s_sleep(32);
}

}  // namespace

static __global__ void set_int4_kernel(int32_t* dst, int a, int b, int c, int d) {
  if (threadIdx.x == 0) { dst[0] = a; dst[1] = b; dst[2] = c; dst[3] = d; }
}

hipError_t launch_set_int4(int32_t* dst, int a, int b, int c, int d, hipStream_t s) {
  hipLaunchKernelGGL(set_int4_kernel, dim3(1), dim3(64), 0, s, dst, a, b, c, d);
  return hipGetLastError();
}

hipError_t launch_pace_start(unsigned long long* t0, hipStream_t s) {
  hipLaunchKernelGGL(pace_start_kernel, dim3(1), dim3(1), 0, s, t0);
  return hipGetLastError();
}

hipError_t launch_pace_wait(const unsigned long long* t0, unsigned long long ticks, hipStream_t s) {
  hipLaunchKernelGGL(pace_wait_kernel, dim3(1), dim3(1), 0, s, t0, ticks);
  return hipGetLastError();
}

hipError_t launch_rmsnorm(int dtype, const void* x, int x_f32, const void* g, void* y, int T, int d, float eps, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  if (dtype == DSK_F32)
    hipLaunchKernelGGL((rmsnorm_kernel<float, float>), dim3(T), dim3(256), 0, s, (const float*)x, (const float*)g, (float*)y, d, eps);
  else if (d % 4 == 0 && d <= 4096) {
    if (x_f32)
      hipLaunchKernelGGL((rmsnorm_vec_kernel<float, 4>), dim3(T), dim3(256), 0, s, (const float*)x, (const bf16_t*)g, (bf16_t*)y, d, eps);
    else
      hipLaunchKernelGGL((rmsnorm_vec_kernel<bf16_t, 4>), dim3(T), dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)g, (bf16_t*)y, d, eps);
  } else if (d % 4 == 0 && d <= 8192) {
    if (x_f32)
      hipLaunchKernelGGL((rmsnorm_vec_kernel<float, 8>), dim3(T), dim3(256), 0, s, (const float*)x, (const bf16_t*)g, (bf16_t*)y, d, eps);
    else
      hipLaunchKernelGGL((rmsnorm_vec_kernel<bf16_t, 8>), dim3(T), dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)g, (bf16_t*)y, d, eps);
  } else if (x_f32)
    hipLaunchKernelGGL((rmsnorm_kernel<float, bf16_t>), dim3(T), dim3(256), 0, s, (const float*)x, (const bf16_t*)g, (bf16_t*)y, d, eps);
  else
    hipLaunchKernelGGL((rmsnorm_kernel<bf16_t, bf16_t>), dim3(T), dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)g, (bf16_t*)y, d, eps);
  return hipGetLastError();
}

hipError_t launch_rope_table(const int32_t* pos, const double* theta, float2* cs, int T, int half, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  int64_t n = (int64_t)T * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, pos, theta, cs, T, half);
  return hipGetLastError();
}

hipError_t launch_rope_kv_write(int dtype, void* qkv, const float2* cs, void* k_rows, void* v_rows, int T, int Hq,
                                int Hkv, int dh, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(rope_kv_write_kernel<float>, dim3(T), dim3(256), 0, s, (float*)qkv, cs, (float*)k_rows, (float*)v_rows, Hq, Hkv, dh);
  else if (dh % 16 == 0 && ((uintptr_t)qkv & 15) == 0 && ((uintptr_t)k_rows & 15) == 0 && ((uintptr_t)v_rows & 15) == 0) {
    const int64_t items = (int64_t)T * ((Hq + Hkv) * (dh / 16) + Hkv * dh / 8);
    hipLaunchKernelGGL(rope_kv_write_vec_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, (bf16_t*)qkv, cs,
                       (bf16_t*)k_rows, (bf16_t*)v_rows, T, Hq, Hkv, dh);
  } else
    hipLaunchKernelGGL(rope_kv_write_kernel<bf16_t>, dim3(T), dim3(256), 0, s, (bf16_t*)qkv, cs, (bf16_t*)k_rows, (bf16_t*)v_rows, Hq, Hkv, dh);
  return hipGetLastError();
}

hipError_t launch_swiglu(int dtype, const void* gu, void* act, int T, int F, int gu_block, hipStream_t s) {
  int64_t n = (int64_t)T * F;
  if (n <= 0) return hipSuccess;
  int64_t b = (n + 255) / 256;
  if (b > 256 * 32) b = 256 * 32;
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(swiglu_kernel<float>, dim3((unsigned)b), dim3(256), 0, s, (const float*)gu, (float*)act, n, F, gu_block);
  else
    hipLaunchKernelGGL(swiglu_kernel<bf16_t>, dim3((unsigned)b), dim3(256), 0, s, (const bf16_t*)gu, (bf16_t*)act, n, F, gu_block);
  return hipGetLastError();
}
