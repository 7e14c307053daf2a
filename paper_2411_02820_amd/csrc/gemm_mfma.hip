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

template <int BM, int BN, int WAVES_M, int WAVES_N, int DBG = 0>
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
  // fragments of k-step ks+1 are fetched from LDS before the MFMAs of k-step ks are issued
  auto load_frags = [&](const bf16_t* a_s, const bf16_t* w_s, int ks, bf16x8* xf, bf16x8* wf) {
    const int ch = ks * 2 + frag_hi;
#pragma unroll
    for (int i = 0; i < TM; ++i) xf[i] = *(const bf16x8*)(a_s + swz(wm * WTM + i * 32 + frag_row, ch));
#pragma unroll
    for (int j = 0; j < TN; ++j) wf[j] = *(const bf16x8*)(w_s + swz(wn * WTN + j * 32 + frag_row, ch));
  };
  // One k-tile of MFMAs.  Interleaved with them: first the LDS stores of the NEXT tile (already in
  // registers, loaded during the previous iteration), then the global loads of the tile after that into
  // the same registers, so that neither sits between the MFMAs and the barrier.
  auto compute = [&](int buf, bool do_store, int store_buf, bool do_load, int load_k0) {
    const bf16_t* a_s = sA + buf * BM * BK;
    const bf16_t* w_s = sW + buf * BN * BK;
    bf16x8 xf[2][TM], wf[2][TN];
    load_frags(a_s, w_s, 0, xf[0], wf[0]);
    if (DBG == 2) load_frags(a_s, w_s, 1, xf[1], wf[1]);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int cur = ks & 1;
      if (DBG != 2 && ks + 1 < BK / 16) load_frags(a_s, w_s, ks + 1, xf[cur ^ 1], wf[cur ^ 1]);
      if (ks == 0 && do_store) store_lds(store_buf);
      if (ks == 1 && do_load) load_global(load_k0);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
          acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][j], xf[cur][i], acc[j][i], 0, 0, 0);
    }
  };

  const int KT = K / BK;
  load_global(0);
  store_lds(0);
  if (KT > 1) load_global(BK);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const bool st = kt + 1 < KT && (DBG == 0 || DBG == 3 || DBG == 4);
    const bool ld = kt + 2 < KT && (DBG == 0 || DBG == 3 || DBG == 5);
    compute(kt & 1, st, (kt + 1) & 1, ld, (kt + 2) * BK);
    __syncthreads();
  }
  if (DBG == 5) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) asm volatile("" ::"v"(a_reg[i]));
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) asm volatile("" ::"v"(w_reg[i]));
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

// Variant with direct global->LDS loads (global_load_lds_dwordx4): no staging registers and no ds_write.
// LDS rows hold BKT bf16 = CH 16-byte slots; a wave instruction fills 64 consecutive slots = 64/CH rows.
// The swizzle is applied on the global side: the lane that fills slot p of row r fetches chunk
// p ^ ((r >> SH) & (CH-1)).  NSTAGE LDS stages form a ring; the loads of k-tile kt+NSTAGE-1 are issued
// right after the barrier that ends k-tile kt-1 (its stage is free from then on), so up to NSTAGE-1 tiles
// are in flight while the MFMAs of tile kt run.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BKT, int NSTAGE>
__global__ void __launch_bounds__(WAVES_M* WAVES_N * 64)
    gemm_bf16_dlds_kernel(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ W, int64_t ldw,
                          bf16_t* __restrict__ C, int64_t ldc, const bf16_t* __restrict__ R, int64_t ldr, int M, int N,
                          int K, int epi, int tiles_m, int tiles_n) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int CH = BKT / 8;              // 16-byte slots per LDS row
  constexpr int SH = CH == 8 ? 1 : 2;      // swizzle uses row bits [SH, SH+log2(CH))
  constexpr int RPI = 64 / CH;             // rows per wave instruction
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_INST = BM / RPI / NW, W_INST = BN / RPI / NW;
  constexpr int NKS = BKT / 16;
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile/wave mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = (bf16_t*)smem_raw;       // [NSTAGE][BM][BKT]
  bf16_t* sW = sA + NSTAGE * BM * BKT;  // [NSTAGE][BN][BKT]

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

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  const int lr = lane / CH, lp = lane % CH;
  const bf16_t* a_src[A_INST];
  const bf16_t* w_src[W_INST];
#pragma unroll
  for (int i = 0; i < A_INST; ++i) {
    int row = RPI * (wave * A_INST + i) + lr;
    a_src[i] = A + (int64_t)min(m0 + row, M - 1) * lda + (lp ^ ((row >> SH) & (CH - 1))) * 8;
  }
#pragma unroll
  for (int i = 0; i < W_INST; ++i) {
    int row = RPI * (wave * W_INST + i) + lr;
    w_src[i] = W + (int64_t)min(n0 + row, N - 1) * ldw + (lp ^ ((row >> SH) & (CH - 1))) * 8;
  }
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void glb_void;
  auto issue_loads = [&](int stage, int k0) {
#pragma unroll
    for (int i = 0; i < A_INST; ++i)
      __builtin_amdgcn_global_load_lds((glb_void*)(a_src[i] + k0),
                                       (lds_void*)(sA + stage * BM * BKT + RPI * (wave * A_INST + i) * BKT), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < W_INST; ++i)
      __builtin_amdgcn_global_load_lds((glb_void*)(w_src[i] + k0),
                                       (lds_void*)(sW + stage * BN * BKT + RPI * (wave * W_INST + i) * BKT), 16, 0, 0);
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  const int frag_row = lane & 31, frag_hi = lane >> 5;
  auto slot = [&](int row, int chunk) { return (row * CH + (chunk ^ ((row >> SH) & (CH - 1)))) * 8; };
  auto load_frags = [&](const bf16_t* a_s, const bf16_t* w_s, int ks, bf16x8* xf, bf16x8* wf) {
    const int ch = ks * 2 + frag_hi;
#pragma unroll
    for (int i = 0; i < TM; ++i) xf[i] = *(const bf16x8*)(a_s + slot(wm * WTM + i * 32 + frag_row, ch));
#pragma unroll
    for (int j = 0; j < TN; ++j) wf[j] = *(const bf16x8*)(w_s + slot(wn * WTN + j * 32 + frag_row, ch));
  };

  const int KT = K / BKT;
  constexpr int PER_TILE = A_INST + W_INST;  // load instructions per wave per k-tile
#pragma unroll
  for (int p = 0; p < NSTAGE - 1; ++p)
    if (p < KT) issue_loads(p, p * BKT);
  // wait for tile 0 (at most the younger NSTAGE-2 tiles may still be in flight)
  if (NSTAGE == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if (KT >= NSTAGE - 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * PER_TILE) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int stage = kt % NSTAGE;
    const int kn = kt + NSTAGE - 1;
    if (kn < KT) issue_loads(kn % NSTAGE, kn * BKT);
    const bf16_t* a_s = sA + stage * BM * BKT;
    const bf16_t* w_s = sW + stage * BN * BKT;
    bf16x8 xf[2][TM], wf[2][TN];
    load_frags(a_s, w_s, 0, xf[0], wf[0]);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int cur = ks & 1;
      if (ks + 1 < NKS) load_frags(a_s, w_s, ks + 1, xf[cur ^ 1], wf[cur ^ 1]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
          acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][j], xf[cur][i], acc[j][i], 0, 0, 0);
    }
    // tile kt+1 must have landed before the barrier; tiles kt+2.. may stay in flight
    if (NSTAGE == 2 || kn >= KT) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * PER_TILE) : "memory");
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * WTM + i * 32 + frag_row;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WTN + j * 32 + 8 * q + 4 * frag_hi;
        if (n >= N) continue;
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

template <int BM, int BN, int WAVES_M, int WAVES_N, int BKT, int NSTAGE>
hipError_t launch_dlds(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc, const void* R,
                       int64_t ldr, int M, int N, int K, int epi, hipStream_t s) {
  auto kern = gemm_bf16_dlds_kernel<BM, BN, WAVES_M, WAVES_N, BKT, NSTAGE>;
  constexpr int lds = NSTAGE * (BM + BN) * BKT * 2;
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

template <int BM, int BN, int WAVES_M, int WAVES_N, int DBG = 0>
hipError_t launch(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc, const void* R, int64_t ldr,
                  int M, int N, int K, int epi, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, DBG>;
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
    case 20: return launch_dlds<256, 256, 2, 4, 64, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 22: return launch_dlds<256, 256, 2, 4, 32, 4>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 23: return launch_dlds<256, 256, 2, 4, 32, 3>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 11: return launch<256, 256, 2, 4, 1>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 12: return launch<256, 256, 2, 4, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 13: return launch<256, 256, 2, 4, 3>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 14: return launch<256, 256, 2, 4, 4>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 15: return launch<256, 256, 2, 4, 5>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 1: return launch<256, 256, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 2: return launch<256, 128, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 3: return launch<128, 128, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    case 4: return launch<128, 256, 2, 2>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    default: return launch<256, 256, 2, 4>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
  }
}
