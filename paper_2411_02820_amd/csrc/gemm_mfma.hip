// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T  (+ R), fp32 accumulation, bf16 output.
//
// Both operands are K-contiguous, so both feed v_mfma_f32_32x32x16_bf16 with 16-byte vectors and no
// transposition.  A workgroup owns a BM x BN tile of C and walks K in steps of 64:
//   global -> registers (next step, in flight during the MFMAs) -> LDS (double buffered) -> MFMA.
// LDS rows are 64 bf16 = eight 16-byte chunks; chunk c of row r is stored at chunk position c ^ (r & 7),
// which makes both the row-wise stores and the 32-rows-at-one-k fragment reads bank-conflict free.
// W rows play the MFMA "A" role and activation rows the "B" role: a lane then holds four consecutive
// output columns of one row in four consecutive accumulator registers and stores them as 8 bytes.
// Workgroup ids are remapped so that each XCD (own L2) works on a compact patch of the tile grid.
#include "dsk_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int BK = 64;          // k extent of one LDS stage
constexpr int CHUNKS = BK / 8;  // 16-byte chunks per LDS row
constexpr int N_XCD = 8;
constexpr int GROUP_M = 4;      // M-tiles per scheduling group

__device__ __forceinline__ int swz(int row, int chunk) { return (row * CHUNKS + (chunk ^ (row & 7))) * 8; }

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ void __launch_bounds__(WAVES_M* WAVES_N * 64)
    gemm_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ W, int64_t ldw,
                     bf16_t* __restrict__ C, int64_t ldc, const bf16_t* __restrict__ R, int64_t ldr, int M, int N, int K,
                     int epi, int tiles_m, int tiles_n) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;            // 32x32 MFMA tiles per wave
  constexpr int A_LOADS = BM * CHUNKS / NT, W_LOADS = BN * CHUNKS / NT;
  static_assert(BM * CHUNKS % NT == 0 && BN * CHUNKS % NT == 0, "tile/thread mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = (bf16_t*)smem_raw;              // [2][BM][64]
  bf16_t* sW = sA + 2 * BM * BK;               // [2][BN][64]

  // ---- workgroup -> tile, XCD-aware ----
  const int nb = gridDim.x;
  int pid = blockIdx.x;
  {
    const int q = nb / N_XCD, rem = nb % N_XCD;
    const int xcd = pid % N_XCD, loc = pid / N_XCD;
    pid = (xcd < rem) ? xcd * (q + 1) + loc : rem * (q + 1) + (xcd - rem) * q + loc;
  }
  const int per_group = GROUP_M * tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GROUP_M;
  const int gsz = min(GROUP_M, tiles_m - first_m);
  const int in_group = pid - group * per_group;
  const int tm = first_m + in_group % gsz;
  const int tn = in_group / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  // ---- global load assignment: chunk id = tid + i*NT -> (row, chunk) ----
  const bf16_t* a_ptr[A_LOADS];
  const bf16_t* w_ptr[W_LOADS];
  int a_lds[A_LOADS], w_lds[W_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    int id = tid + i * NT, row = id / CHUNKS, ch = id % CHUNKS;
    int gr = min(m0 + row, M - 1);
    a_ptr[i] = A + (int64_t)gr * lda + ch * 8;
    a_lds[i] = swz(row, ch);
  }
#pragma unroll
  for (int i = 0; i < W_LOADS; ++i) {
    int id = tid + i * NT, row = id / CHUNKS, ch = id % CHUNKS;
    int gr = min(n0 + row, N - 1);
    w_ptr[i] = W + (int64_t)gr * ldw + ch * 8;
    w_lds[i] = swz(row, ch);
  }

  u32x4 a_reg[A_LOADS], w_reg[W_LOADS];
  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) a_reg[i] = *(const u32x4*)(a_ptr[i] + k0);
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) w_reg[i] = *(const u32x4*)(w_ptr[i] + k0);
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) *(u32x4*)(sA + buf * BM * BK + a_lds[i]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) *(u32x4*)(sW + buf * BN * BK + w_lds[i]) = w_reg[i];
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  const int frag_row = lane & 31, frag_hi = lane >> 5;
  auto compute = [&](int buf) {
    const bf16_t* a_s = sA + buf * BM * BK;
    const bf16_t* w_s = sW + buf * BN * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int ch = ks * 2 + frag_hi;
      bf16x8 xf[TM], wf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) xf[i] = *(const bf16x8*)(a_s + swz(wm * WTM + i * 32 + frag_row, ch));
#pragma unroll
      for (int j = 0; j < TN; ++j) wf[j] = *(const bf16x8*)(w_s + swz(wn * WTN + j * 32 + frag_row, ch));
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
          acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], xf[i], acc[j][i], 0, 0, 0);
    }
  };

  const int KT = K / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const bool more = kt + 1 < KT;
    if (more) load_global((kt + 1) * BK);
    compute(kt & 1);
    if (more) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: accumulator register 4q+e of tile (j,i) is C[m][n + e],
  //      m = tile row base + lane%32, n = tile col base + 8q + 4*(lane/32) ----
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * WTM + i * 32 + frag_row;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WTN + j * 32 + 8 * q + 4 * frag_hi;
        if (n >= N) continue;  // N is a multiple of 4
        float v0 = acc[j][i][4 * q], v1 = acc[j][i][4 * q + 1], v2 = acc[j][i][4 * q + 2], v3 = acc[j][i][4 * q + 3];
        if (epi == EPI_RESIDUAL) {
          bf16x4 r = *(const bf16x4*)(R + (int64_t)m * ldr + n);
          v0 += (float)r[0]; v1 += (float)r[1]; v2 += (float)r[2]; v3 += (float)r[3];
        }
        bf16x4 o;
        o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
        *(bf16x4*)(C + (int64_t)m * ldc + n) = o;
      }
    }
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc, const void* R, int64_t ldr,
                  int M, int N, int K, int epi, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N>;
  constexpr int lds = 2 * (BM + BN) * BK * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WAVES_M * WAVES_N * 64), lds, s, (const bf16_t*)A, lda,
                     (const bf16_t*)W, ldw, (bf16_t*)C, ldc, (const bf16_t*)R, ldr, M, N, K, epi, tiles_m, tiles_n);
  return hipGetLastError();
}

int g_variant = 0;

}  // namespace

void gemm_mfma_set_variant(int v) { g_variant = v; }

hipError_t launch_gemm_mfma_bf16(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                                 const void* R, int64_t ldr, int M, int N, int K, int epi, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K < BK || K % BK || N % 4 || (lda & 7) || (ldw & 7) || (ldc & 3) || (epi == EPI_RESIDUAL && (ldr & 3)))
    return hipErrorNotSupported;
  switch (g_variant) {
    case 1: return launch<256, 256, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 2: return launch<256, 128, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 3: return launch<128, 128, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 4: return launch<128, 256, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    default: return launch<256, 256, 2, 4>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
  }
}
