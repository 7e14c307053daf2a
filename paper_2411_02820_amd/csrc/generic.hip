// Plain-ALU kernels for any shape and both dtypes: an LDS-tiled GEMM and a one-wave-per-query
// attention.  They carry the fp32 model (where bf16 MFMA does not apply) and shapes the MFMA
// kernels do not take; arithmetic is fp32 with fp32 accumulation.
#include "dsk_internal.h"

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

// C[M,N] = A[M,K] * W[N,K]^T (+R).  256 threads, each a 4x4 micro-tile; tiles are zero-padded at the edges.
template <typename T>
__global__ void __launch_bounds__(256) gemm_generic_kernel(const T* __restrict__ A, int64_t lda, const T* __restrict__ W,
                                                           int64_t ldw, void* __restrict__ Cv, int64_t ldc,
                                                           const void* __restrict__ Rv, int64_t ldr, int M, int N, int K,
                                                           int epi) {
  __shared__ float sa[TK][TM + 4];
  __shared__ float sw[TK][TN + 4];
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;  // tx: 4 columns, ty: 4 rows
  const int lr = threadIdx.x >> 2, lk = (threadIdx.x & 3) * 4;  // loader: row lr, k offset lk..lk+3
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int k = k0 + lk + j;
      int m = m0 + lr, n = n0 + lr;
      sa[lk + j][lr] = (m < M && k < K) ? to_f32(A[(int64_t)m * lda + k]) : 0.f;
      sw[lk + j][lr] = (n < N && k < K) ? to_f32(W[(int64_t)n * ldw + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sa[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = sw[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (epi & EPI_RESIDUAL)
        v += (epi & EPI_R_F32) ? ((const float*)Rv)[(int64_t)m * ldr + n] : to_f32(((const T*)Rv)[(int64_t)m * ldr + n]);
      if (epi & EPI_C_F32) ((float*)Cv)[(int64_t)m * ldc + n] = v;
      else ((T*)Cv)[(int64_t)m * ldc + n] = from_f32<T>(v);
    }
  }
}

// One wave per (query token, q head).  Keys are taken 64 at a time: lane j scores key j, the chunk
// maximum and sum are wave reductions, then every lane accumulates its output dims over the chunk.
template <typename T>
__global__ void __launch_bounds__(64) attn_generic_kernel(const T* __restrict__ q, int64_t ldq, const T* __restrict__ k_rows,
                                                          const T* __restrict__ v_rows, T* __restrict__ out,
                                                          const int32_t* __restrict__ q_cu, const int32_t* __restrict__ p_cu,
                                                          int n_seqs, int64_t own_row0, int Hq, int Hkv, int dh) {
  __shared__ float sq[256];
  const int i = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
  const int kvh = head / (Hq / Hkv);
  const int64_t ldkv = (int64_t)Hkv * dh;
  // sequence of this query (n_seqs is small; linear scan)
  int b = 0;
  while (b + 1 < n_seqs && q_cu[b + 1] <= i) ++b;
  const int64_t pre0 = p_cu ? p_cu[b] : 0;
  const int n_pre = p_cu ? (p_cu[b + 1] - p_cu[b]) : 0;
  const int64_t own0 = own_row0 + q_cu[b];
  const int n_own = i - q_cu[b] + 1;
  const int n_keys = n_pre + n_own;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int e = lane; e < dh; e += 64) sq[e] = to_f32(q[(int64_t)i * ldq + head * dh + e]) * scale;
  __syncthreads();
  float m = -INFINITY, l = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};  // output dims lane, lane+64, lane+128, lane+192
  for (int c0 = 0; c0 < n_keys; c0 += 64) {
    int j = c0 + lane;
    float s = -INFINITY;
    int64_t row = 0;
    if (j < n_keys) {
      row = j < n_pre ? pre0 + j : own0 + (j - n_pre);
      const T* kp = k_rows + row * ldkv + kvh * dh;
      float dot = 0.f;
      for (int e = 0; e < dh; ++e) dot += sq[e] * to_f32(kp[e]);
      s = dot;
    }
    float cm = s;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cm = fmaxf(cm, __shfl_xor(cm, o, 64));
    float m_new = fmaxf(m, cm);
    float corr = expf(m - m_new);  // m = -inf on the first chunk: corr = 0
    float p = (j < n_keys) ? expf(s - m_new) : 0.f;
    float ps = p;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o, 64);
    l = l * corr + ps;
#pragma unroll
    for (int a = 0; a < 4; ++a) acc[a] *= corr;
    int nj = min(64, n_keys - c0);
    for (int jj = 0; jj < nj; ++jj) {
      float pj = __shfl(p, jj, 64);
      int64_t r = __shfl((int)row, jj, 64);  // rows fit in 32 bits (checked by the caller)
      const T* vp = v_rows + r * ldkv + kvh * dh;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        int e = lane + 64 * a;
        if (e < dh) acc[a] += pj * to_f32(vp[e]);
      }
    }
    m = m_new;
  }
  float inv = 1.0f / l;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    int e = lane + 64 * a;
    if (e < dh) out[(int64_t)i * Hq * dh + head * dh + e] = from_f32<T>(acc[a] * inv);
  }
}

}  // namespace

hipError_t launch_gemm_generic(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                               const void* R, int64_t ldr, int M, int N, int K, int epi, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((N + TN - 1) / TN, (M + TM - 1) / TM);
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(256), 0, s, (const float*)A, lda, (const float*)W, ldw, C,
                       ldc, R, ldr, M, N, K, epi);
  else
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)A, lda, (const bf16_t*)W, ldw,
                       C, ldc, R, ldr, M, N, K, epi);
  return hipGetLastError();
}

hipError_t launch_attn_generic(int dtype, const AttnArgs& a, hipStream_t s) {
  if (a.n_q <= 0) return hipSuccess;
  dim3 grid(a.n_q, a.Hq);
  if (dtype == DSK_F32)
    hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(64), 0, s, (const float*)a.q, a.ldq, (const float*)a.k_rows,
                       (const float*)a.v_rows, (float*)a.out, a.q_cu, a.p_cu, a.n_seqs, a.own_row0, a.Hq, a.Hkv, a.dh);
  else
    hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(64), 0, s, (const bf16_t*)a.q, a.ldq, (const bf16_t*)a.k_rows,
                       (const bf16_t*)a.v_rows, (bf16_t*)a.out, a.q_cu, a.p_cu, a.n_seqs, a.own_row0, a.Hq, a.Hkv, a.dh);
  return hipGetLastError();
}
