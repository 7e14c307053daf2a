// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T  (+ R), fp32 accumulation, bf16 output.
//
// Both operands are K-contiguous, so both feed the MFMA with 16-byte vectors and no transposition.  Two
// kernels: gemm16_bf16_kernel on v_mfma_f32_16x16x32_bf16 for the large prefill problems (256 x 256 tile; the chip
// is power-limited there and that instruction takes less energy per flop), gemm_bf16_kernel on
// v_mfma_f32_32x32x16_bf16 for everything else (128 x 128 tile, K-split tiles for few rows).  A workgroup owns a BM x BN tile of C and walks K in steps of 64 through a two-stage
// LDS ring filled by direct global->LDS loads (global_load_lds_dwordx4: no staging registers, no
// ds_write).  The loads of k-tile kt+2 go out, between MFMAs, as soon as a barrier shows that every wave
// has read k-tile kt out of the stage they overwrite; fragments are read from LDS one or two k-steps ahead
// of the MFMAs that use them.  Two schedules (SCHED): 0 frees the stage before the last k-step (one
// barrier per k-tile; any tile shape), 1 frees it before k-step 2 of 4 and spreads the loads over two
// k-steps (two barriers; the 256 x 256 and 128 x 128 tiles, where it is 5-8 % and up to 25 % faster).
//
// LDS rows hold 64 bf16 = eight 16-byte slots.  A wave load instruction fills 64 consecutive slots
// (8 rows); the swizzle is applied on the global side: the lane that fills slot p of row r fetches chunk
// p ^ ((r >> 1) & 7).  With that, the 16 lanes that one LDS cycle serves (rows r..r+15 at one k chunk)
// touch 16 different 16-byte bank groups of the 256-byte LDS line.
//
// W rows play the MFMA "A" role and activation rows the "B" role: a lane then holds four consecutive
// output columns of one row in four consecutive accumulator registers (the epilogue regroups them through LDS so
// that stores cover whole rows of the tile).
// Workgroup ids are remapped so that each XCD (own L2) works on a compact patch of the tile grid.
//
// Small M (the suffix pass: tens of rows) is a weight-streaming problem: a 64 x 64 tile, K split over
// blockIdx.y so that enough workgroups stream W to fill HBM; each split writes an fp32 partial tile and a
// second kernel adds the partials in a fixed order (deterministic), applies the residual and rounds.
#include <type_traits>

#include "dsk_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BK = 64;        // k extent of one LDS stage
constexpr int CH = BK / 8;    // 16-byte slots per LDS row
constexpr int RPI = 64 / CH;  // rows filled by one wave load instruction
constexpr int NSTAGE = 2;
constexpr int N_XCD = 8;
constexpr int GROUP_M = 4;    // M-tiles per scheduling group

__device__ __forceinline__ int slot(int row, int chunk) { return (row * CH + (chunk ^ ((row >> 1) & (CH - 1)))) * 8; }

// C[m][n..n+3] = v (+ R[m][n..n+3]); R and C are bf16 or fp32 as the epilogue flags say.
__device__ __forceinline__ void store_quad(void* C, int64_t ldc, const void* R, int64_t ldr, int m, int n, f32x4 v, int epi) {
  if (epi & EPI_RESIDUAL) {
    if (epi & EPI_R_F32) {
      f32x4 r = *(const f32x4*)((const float*)R + (int64_t)m * ldr + n);
      v += r;
    } else {
      bf16x4 r = *(const bf16x4*)((const bf16_t*)R + (int64_t)m * ldr + n);
      v[0] += (float)r[0]; v[1] += (float)r[1]; v[2] += (float)r[2]; v[3] += (float)r[3];
    }
  }
  if (epi & EPI_C_F32) {
    *(f32x4*)((float*)C + (int64_t)m * ldc + n) = v;
  } else {
    bf16x4 o;
    o[0] = (bf16_t)v[0]; o[1] = (bf16_t)v[1]; o[2] = (bf16_t)v[2]; o[3] = (bf16_t)v[3];
    *(bf16x4*)((bf16_t*)C + (int64_t)m * ldc + n) = o;
  }
}

// PARTIAL: write the fp32 accumulators of this K split to P[split][M][N] instead of the bf16 result.
// EPI_SWIGLU (run-time flag; wave tiles with an even number of 32-column MFMA tiles): W holds gate and up
// rows interleaved in blocks of 32 (packed rows 64b..64b+31 = gate rows 32b.., the next 32 = the same up
// rows), so MFMA tiles j (even) and j+1 of a wave are gate and up of the same 32 FFN indices at the same
// lane/register; the epilogue writes silu(gate)*up to C[M, N/2].
// SCHED: software-pipeline schedule of the k loop, see the top of the file.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool PARTIAL, int SCHED = 0>
__global__ void __launch_bounds__(WAVES_M* WAVES_N * 64)
    gemm_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ W, int64_t ldw,
                     void* __restrict__ C, int64_t ldc, const void* __restrict__ R, int64_t ldr,
                     float* __restrict__ P, int M, int N, int K, int epi, int tiles_m, int tiles_n, int kt_per_split) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;            // 32x32 MFMA tiles per wave
  constexpr int A_INST = BM / RPI / NW, W_INST = BN / RPI / NW;
  constexpr int NKS = BK / 16;
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile/wave mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = (bf16_t*)smem_raw;      // [NSTAGE][BM][BK]
  bf16_t* sW = sA + NSTAGE * BM * BK;  // [NSTAGE][BN][BK]

  // ---- workgroup -> tile, XCD-aware: consecutive ids go to different XCDs, so give each XCD a
  //      contiguous range of the (grouped) tile order ----
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

  // ---- per-lane global source of each wave load instruction: a 32-bit byte offset from the (uniform) matrix
  //      base, so that the loads use the scalar-base + vector-offset address form and the walk along K only
  //      moves the scalar base ----
  const int lr = lane / CH, lp = lane % CH;
  uint32_t a_off[A_INST], w_off[W_INST];
#pragma unroll
  for (int i = 0; i < A_INST; ++i) {
    int row = RPI * (wave * A_INST + i) + lr;
    a_off[i] = (uint32_t)(((int64_t)min(m0 + row, M - 1) * lda + (lp ^ ((row >> 1) & (CH - 1))) * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < W_INST; ++i) {
    int row = RPI * (wave * W_INST + i) + lr;
    w_off[i] = (uint32_t)(((int64_t)min(n0 + row, N - 1) * ldw + (lp ^ ((row >> 1) & (CH - 1))) * 8) * 2);
  }
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void glb_void;
  constexpr int PER_TILE = A_INST + W_INST;  // load instructions per wave per k-tile
  // global_load_lds_dwordx4 in its scalar-base + 32-bit vector-offset form; M0 carries the LDS byte address
  // of the 1 KB the wave fills (lane i lands at M0 + 16*i)
  const uint32_t sA_lds = (uint32_t)(uintptr_t)sA, sW_lds = (uint32_t)(uintptr_t)sW;
  auto issue_load = [&](int stage, int k0, int idx) {
    const bool is_a = idx < A_INST;
    const int li = is_a ? idx : idx - A_INST;
    const char* base = (is_a ? (const char*)A : (const char*)W) + (int64_t)k0 * 2;
    const uint32_t voff = is_a ? a_off[li] : w_off[li];
    const uint32_t dst = is_a ? sA_lds + (uint32_t)(stage * BM * BK + RPI * (wave * A_INST + li) * BK) * 2
                              : sW_lds + (uint32_t)(stage * BN * BK + RPI * (wave * W_INST + li) * BK) * 2;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(dst), "v"(voff), "s"(base)
                 : "memory", "m0");
  };
  auto issue_loads = [&](int stage, int k0) {
#pragma unroll
    for (int i = 0; i < PER_TILE; ++i) issue_load(stage, k0, i);
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  const int frag_row = lane & 31, frag_hi = lane >> 5;
  auto load_frags = [&](const bf16_t* a_s, const bf16_t* w_s, int ks, bf16x8* xf, bf16x8* wf) {
    const int ch = ks * 2 + frag_hi;
#pragma unroll
    for (int i = 0; i < TM; ++i) xf[i] = *(const bf16x8*)(a_s + slot(wm * WTM + i * 32 + frag_row, ch));
#pragma unroll
    for (int j = 0; j < TN; ++j) wf[j] = *(const bf16x8*)(w_s + slot(wn * WTN + j * 32 + frag_row, ch));
  };

  // ---- K range of this workgroup ----
  const int KT_all = K / BK;
  const int kt_begin = PARTIAL ? (int)blockIdx.y * kt_per_split : 0;
  const int kt_end = PARTIAL ? min(KT_all, kt_begin + kt_per_split) : KT_all;

  // Software pipeline over k-tiles with ONE barrier per tile, placed between the MFMAs of k-step NKS-2 and
  // NKS-1: by then every LDS read of the current tile has been issued and waited for, so the barrier both
  // publishes tile kt+1 (each wave has waited for its own loads) and frees the current stage for the loads of
  // tile kt+2.  After the barrier a wave still owns the MFMAs of the last k-step (fragments already in
  // registers) and issues the first fragment reads of tile kt+1 under them, so the restart after a barrier
  // never waits on LDS.
  const int n_kt = kt_end - kt_begin;
  issue_loads(0, kt_begin * BK);
  if (n_kt > 1) {
    issue_loads(1, (kt_begin + 1) * BK);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER_TILE) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  if constexpr (SCHED == 1) {
    // Early-freed stage, for k-tiles of four k-steps.  Fragments are read two k-steps ahead (sets 1 and 2 during
    // k-step 0, set 3 during k-step 1), so every LDS read of the tile has returned before k-step 2: the barrier
    // there frees the stage, and the loads of tile t+2 go out one per two MFMAs over k-steps 2 and 3 instead of
    // all in the last one.  A second barrier before k-step 3 publishes tile t+1: its loads were issued a whole
    // tile earlier, and only the LD loads issued since the first barrier may still be in flight.
    static_assert(NKS == 4 && PER_TILE % 2 == 0, "schedule written for four k-steps");
    constexpr int NM = TN * TM;
    constexpr int LD = PER_TILE / 2;  // loads per wave in each of the last two k-steps
    bf16x8 xs[NKS][TM], ws[NKS][TN];
    load_frags(sA, sW, 0, xs[0], ws[0]);
    auto tile_step = [&](int t, auto has_next, auto has_next2) {
      const int stage = t & 1;
      const bf16_t* a_s = sA + stage * BM * BK;
      const bf16_t* w_s = sW + stage * BN * BK;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        if (ks == 2) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        if (ks == 3) {
          if (has_next2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LD) : "memory");
          else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int m = j * TM + i;
            if (m == (NM >= 8 ? 2 : 1)) {
              __builtin_amdgcn_sched_barrier(0);
              if (ks == 0) { load_frags(a_s, w_s, 1, xs[1], ws[1]); load_frags(a_s, w_s, 2, xs[2], ws[2]); }
              if (ks == 1) load_frags(a_s, w_s, 3, xs[3], ws[3]);
              if (ks == 3 && has_next) load_frags(sA + (stage ^ 1) * BM * BK, sW + (stage ^ 1) * BN * BK, 0, xs[0], ws[0]);
              __builtin_amdgcn_sched_barrier(0);
            }
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ws[ks][j], xs[ks][i], acc[j][i], 0, 0, 0);
            if (ks >= 2 && has_next2) {
              __builtin_amdgcn_sched_barrier(0);
#pragma unroll
              for (int q = m * LD / NM; q < (m + 1) * LD / NM; ++q)
                issue_load(stage, (kt_begin + t + 2) * BK, (ks - 2) * LD + q);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    int t = 0;
    for (; t + 2 < n_kt; ++t) tile_step(t, std::true_type{}, std::true_type{});
    if (t + 1 < n_kt) { tile_step(t, std::true_type{}, std::false_type{}); ++t; }
    if (t < n_kt) tile_step(t, std::false_type{}, std::false_type{});
  } else {
    bf16x8 xf[2][TM], wf[2][TN];
    load_frags(sA, sW, 0, xf[0], wf[0]);
    // one k-tile; the two flags are compile-time so that the steady-state loop body is a single basic block
    // (precise s_waitcnt counts) and the tail tiles are peeled
    auto tile_step = [&](int t, auto has_next, auto has_next2) {
      const int stage = t & 1;
      const bf16_t* a_s = sA + stage * BM * BK;
      const bf16_t* w_s = sW + stage * BN * BK;
  #pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const int cur = ks & 1;
        constexpr int NM = TN * TM;
        constexpr int LEAD = NM >= 8 ? 2 : 1;  // MFMAs issued before the next fragment reads
        if (ks + 1 == NKS) {
          // all reads of this tile are done; tile t+1 has landed (only its loads are outstanding)
          asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
          __syncthreads();
          if (has_next)
            load_frags(sA + (stage ^ 1) * BM * BK, sW + (stage ^ 1) * BN * BK, 0, xf[cur ^ 1], wf[cur ^ 1]);
        }
        __builtin_amdgcn_sched_barrier(0);
  #pragma unroll
        for (int j = 0; j < TN; ++j)
  #pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int m = j * TM + i;
            if (ks + 1 < NKS && m == LEAD) {
              // Fragment reads of the next k-step go out after the first MFMAs of this one: the s_waitcnt the
              // compiler puts in front of this k-step then only covers reads issued a whole k-step earlier, and
              // the new reads have the remaining MFMAs to land.
              __builtin_amdgcn_sched_barrier(0);
              load_frags(a_s, w_s, ks + 1, xf[cur ^ 1], wf[cur ^ 1]);
              __builtin_amdgcn_sched_barrier(0);
            }
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][j], xf[cur][i], acc[j][i], 0, 0, 0);
            if (ks + 1 == NKS && has_next2) {
              // the loads of tile t+2 (its stage was freed by the barrier) go out one by one between the MFMAs of
              // the last k-step: a wave that queues several vector-memory instructions back to back cannot issue
              // its MFMAs until the address unit has taken them
              __builtin_amdgcn_sched_barrier(0);
  #pragma unroll
              for (int q = m * PER_TILE / NM; q < (m + 1) * PER_TILE / NM; ++q)
                issue_load(stage, (kt_begin + t + 2) * BK, q);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    int t = 0;
    for (; t + 2 < n_kt; ++t) tile_step(t, std::true_type{}, std::true_type{});
    if (t + 1 < n_kt) { tile_step(t, std::true_type{}, std::false_type{}); ++t; }
    if (t < n_kt) tile_step(t, std::false_type{}, std::false_type{});

  }

  // ---- epilogue: accumulator register 4q+e of tile (j,i) is C[m][n + e],
  //      m = tile row base + lane%32, n = tile col base + 8q + 4*(lane/32) ----
  // Wave tiles of 64 columns go through LDS (free by now: every wave has read its last fragments before the last
  // barrier, and no load is in flight): stored straight from the accumulators, a store instruction would touch
  // 32 rows with 8 or 16 bytes each; staged, a wave writes 32 x 64 fp32 values to a padded region of its own and
  // reads them back row by row, so that 16 lanes cover one output row (128 contiguous bytes of bf16, 256 of fp32)
  // and the residual is read the same way.  Only the wave itself touches its region: no barrier.
  if constexpr (!PARTIAL && TN == 2) {
    constexpr int ROW_F = 64 + 4;  // floats per staged row: 16-byte pad, conflict-free for 16 lanes at a time
    float* stage = (float*)smem_raw + wave * (32 * ROW_F);
    static_assert(NW * 32 * ROW_F * 4 <= NSTAGE * (BM + BN) * BK * 2, "staging region fits the tile ring");
    const bool swiglu = (epi & EPI_SWIGLU) != 0;
    // the lane's indices are derived here from an opaque copy of the lane id: computed before the k loop (where the
    // compiler would otherwise hoist them) they would take the kernel from 248 to 252 registers, i.e. to all 512
    // of a SIMD for its two waves, and no other kernel's wave (a copy, a pacing kernel) could share the CU
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int frag_row = lane_e & 31, frag_hi = lane_e >> 5;
    const int rr = lane_e >> 4, c4 = (lane_e & 15) * 4;  // read-back: 4 rows per instruction, 4 columns per lane
    const int rr_s = lane_e >> 3, c4_s = (lane_e & 7) * 4;  // SwiGLU: 32 result columns per row, 8 rows per instruction
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if (swiglu) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = acc[0][i][4 * q + e], u = acc[1][i][4 * q + e];
            const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
            o[e] = g * sig * u;
          }
          *(f32x4*)(stage + frag_row * ROW_F + 8 * q + 4 * frag_hi) = o;
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f32x4 o = {acc[j][i][4 * q], acc[j][i][4 * q + 1], acc[j][i][4 * q + 2], acc[j][i][4 * q + 3]};
            *(f32x4*)(stage + frag_row * ROW_F + j * 32 + 8 * q + 4 * frag_hi) = o;
          }
      }
      __builtin_amdgcn_wave_barrier();
      const int mb = m0 + wm * WTM + i * 32;
      if (swiglu) {
        const int fb = (n0 + wn * WTN) / 2;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int r = it * 8 + rr_s, m = mb + r, f = fb + c4_s;
          const f32x4 v = *(const f32x4*)(stage + r * ROW_F + c4_s);
          if (m < M && f < N / 2) {
            bf16x4 o;
            o[0] = (bf16_t)v[0]; o[1] = (bf16_t)v[1]; o[2] = (bf16_t)v[2]; o[3] = (bf16_t)v[3];
            *(bf16x4*)((bf16_t*)C + (int64_t)m * ldc + f) = o;
          }
        }
      } else {
        const int n = n0 + wn * WTN + c4;
        // the eight residual quads of this 32-row block are requested together, then added and stored: one
        // memory round trip per block instead of one per store
        f32x4 res[8];
        if (epi & EPI_RESIDUAL) {
#pragma unroll
          for (int it = 0; it < 8; ++it) {
            const int m = min(mb + it * 4 + rr, M - 1), nn = min(n, N - 4);  // clamped: masked below
            if (epi & EPI_R_F32) {
              res[it] = *(const f32x4*)((const float*)R + (int64_t)m * ldr + nn);
            } else {
              const bf16x4 rb = *(const bf16x4*)((const bf16_t*)R + (int64_t)m * ldr + nn);
              res[it][0] = (float)rb[0]; res[it][1] = (float)rb[1]; res[it][2] = (float)rb[2]; res[it][3] = (float)rb[3];
            }
          }
        }
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int r = it * 4 + rr, m = mb + r;
          f32x4 v = *(const f32x4*)(stage + r * ROW_F + c4);
          if (epi & EPI_RESIDUAL) v += res[it];
          if (m < M && n < N) store_quad(C, ldc, nullptr, 0, m, n, v, epi & ~(EPI_RESIDUAL | EPI_R_F32));  // N % 4 == 0
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
    return;
  }
  if constexpr (TN % 2 == 0 && !PARTIAL) if (epi & EPI_SWIGLU) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * WTM + i * 32 + frag_row;
      if (m >= M) continue;
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = (n0 + wn * WTN + j * 32) / 2 + 8 * q + 4 * frag_hi;
          if (f >= N / 2) continue;
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = acc[j][i][4 * q + e], u = acc[j + 1][i][4 * q + e];
            const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
            o[e] = (bf16_t)(g * sig * u);
          }
          *(bf16x4*)((bf16_t*)C + (int64_t)m * ldc + f) = o;
        }
      }
    }
    return;
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
        if (n >= N) continue;  // N is a multiple of 4
        float v0 = acc[j][i][4 * q], v1 = acc[j][i][4 * q + 1], v2 = acc[j][i][4 * q + 2], v3 = acc[j][i][4 * q + 3];
        if (PARTIAL) {
          f32x4 o = {v0, v1, v2, v3};
          *(f32x4*)(P + ((int64_t)blockIdx.y * M + m) * N + n) = o;
        } else {
          f32x4 v = {v0, v1, v2, v3};
          store_quad(C, ldc, R, ldr, m, n, v, epi);
        }
      }
    }
  }
}

// The same GEMM on v_mfma_f32_16x16x32_bf16 (wave tiles of 64 columns, no K split).  Under a bf16 GEMM on random
// data the chip sits at its power limit, and a register-only loop of this instruction sustains about 10 % more
// flops there than the 32x32x16 one (the 16x16 accumulator tile is read and written half as often per flop).
// W rows are the MFMA "A" operand again: lane l holds row l%16 and the eight k values 8*(l/16)..+7 of a 32-wide
// k-step; accumulator register r of tile (j,i) is C[m][n + r], m = 16i + l%16, n = 16j + 4*(l/16).
// Schedule per k-tile (two k-steps of 32 MFMAs): the fragments of k-step 1 are read during k-step 0; a barrier
// between the k-steps frees the stage; the loads of tile t+2 go out one per four MFMAs of k-step 1; a barrier in
// the middle of k-step 1 publishes tile t+1, whose first fragments are read during the rest of it.
// GROUPED (the expert projections of a mixture-of-experts layer): the token rows are sorted by expert, and row tile
// tm of the grid is described by tile_tab[tm] = {expert, first row, end of the expert's rows, -} (built on the
// device; tile_tab[tiles_m].x = number of tiles that exist; expert < 0: no such tile, the workgroup leaves); the
// expert's matrix is W + expert * w_group_stride.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool GROUPED = false>
__global__ void __launch_bounds__(WAVES_M* WAVES_N * 64)
    gemm16_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ W_all, int64_t ldw,
                       void* __restrict__ C, int64_t ldc, const void* __restrict__ R, int64_t ldr, int M_all, int N, int K,
                       int epi, int tiles_m, int tiles_n, const int4* __restrict__ tile_tab, int64_t w_group_stride) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 16, TN = WTN / 16;  // 16x16 MFMA tiles per wave
  constexpr int A_INST = BM / RPI / NW, W_INST = BN / RPI / NW;
  constexpr int PER_TILE = A_INST + W_INST;
  constexpr int NM = TM * TN;                  // MFMAs per k-step
  constexpr int NF = TM + TN;                  // fragment reads per k-step
  static_assert(WTN == 64 && BK == 64 && PER_TILE % 2 == 0 && NM % 4 == 0, "written for 64-column wave tiles, two k-steps");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = (bf16_t*)smem_raw;
  bf16_t* sW = sA + NSTAGE * BM * BK;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  int pid = blockIdx.x;
  int nb = gridDim.x, n_tiles_m = tiles_m;
  if constexpr (GROUPED) {
    // the grid is sized for the worst case; the tiles that exist are the first tile_tab[tiles_m].x of the table, and
    // only their workgroups are spread over the dies (the rest, the highest block ids, leave at once)
    n_tiles_m = min(tile_tab[tiles_m].x, tiles_m);
    nb = n_tiles_m * tiles_n;
    if (pid >= nb) return;
  }
  {
    const int q = nb / N_XCD, rem = nb % N_XCD;
    const int xcd = pid % N_XCD, loc = pid / N_XCD;
    pid = (xcd < rem) ? xcd * (q + 1) + loc : rem * (q + 1) + (xcd - rem) * q + loc;
  }
  const int per_group = GROUP_M * tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GROUP_M;
  const int gsz = min(GROUP_M, n_tiles_m - first_m);
  const int in_group = pid - group * per_group;
  int m0 = (first_m + in_group % gsz) * BM, M = M_all;
  const int n0 = (in_group / gsz) * BN;
  const bf16_t* W = W_all;
  if constexpr (GROUPED) {
    const int4 te = tile_tab[first_m + in_group % gsz];
    if (te.x < 0) return;  // uniform over the workgroup, before any barrier
    m0 = te.y;
    M = te.z;
    W = W_all + (int64_t)te.x * w_group_stride;
  }

  const int lr = lane / CH, lp = lane % CH;
  uint32_t a_off[A_INST], w_off[W_INST];
#pragma unroll
  for (int i = 0; i < A_INST; ++i) {
    int row = RPI * (wave * A_INST + i) + lr;
    a_off[i] = (uint32_t)(((int64_t)min(m0 + row, M - 1) * lda + (lp ^ ((row >> 1) & (CH - 1))) * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < W_INST; ++i) {
    int row = RPI * (wave * W_INST + i) + lr;
    w_off[i] = (uint32_t)(((int64_t)min(n0 + row, N - 1) * ldw + (lp ^ ((row >> 1) & (CH - 1))) * 8) * 2);
  }
  const uint32_t sA_lds = (uint32_t)(uintptr_t)sA, sW_lds = (uint32_t)(uintptr_t)sW;
  auto issue_load = [&](int stage, int k0, int idx) {
    const bool is_a = idx < A_INST;
    const int li = is_a ? idx : idx - A_INST;
    const char* base = (is_a ? (const char*)A : (const char*)W) + (int64_t)k0 * 2;
    const uint32_t voff = is_a ? a_off[li] : w_off[li];
    const uint32_t dst = is_a ? sA_lds + (uint32_t)(stage * BM * BK + RPI * (wave * A_INST + li) * BK) * 2
                              : sW_lds + (uint32_t)(stage * BN * BK + RPI * (wave * W_INST + li) * BK) * 2;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(dst), "v"(voff), "s"(base)
                 : "memory", "m0");
  };

  f32x4 acc[TN][TM];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[j][i][r] = 0.f;

  // fragment f of a k-step, in the order the MFMAs (j outer, i inner) first need them: W 0, X 0..TM-1, W 1..TN-1
  const int frow = lane & 15, fq = lane >> 4;
  bf16x8 xs[2][TM], ws[2][TN];
  auto read_frag = [&](const bf16_t* a_s, const bf16_t* w_s, int ks, int f) {
    const int ch = ks * 4 + fq;
    if (f == 0) ws[ks][0] = *(const bf16x8*)(w_s + slot(wn * WTN + frow, ch));
    else if (f <= TM) xs[ks][f - 1] = *(const bf16x8*)(a_s + slot(wm * WTM + (f - 1) * 16 + frow, ch));
    else ws[ks][f - TM] = *(const bf16x8*)(w_s + slot(wn * WTN + (f - TM) * 16 + frow, ch));
  };

  const int n_kt = K / BK;
#pragma unroll
  for (int i = 0; i < PER_TILE; ++i) issue_load(0, 0, i);
  if (n_kt > 1) {
#pragma unroll
    for (int i = 0; i < PER_TILE; ++i) issue_load(1, BK, i);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER_TILE) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
#pragma unroll
  for (int f = 0; f < NF; ++f) read_frag(sA, sW, 0, f);

  constexpr int LD = PER_TILE / 2;  // loads per wave in each half of k-step 1
  auto tile_step = [&](int t, auto has_next, auto has_next2) {
    const int stage = t & 1;
    const bf16_t* a_s = sA + stage * BM * BK;
    const bf16_t* w_s = sW + stage * BN * BK;
    const bf16_t* a_n = sA + (stage ^ 1) * BM * BK;
    const bf16_t* w_n = sW + (stage ^ 1) * BN * BK;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      if (ks == 1) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int m = j * TM + i;
          if (ks == 1 && m == NM / 2) {
            if (has_next2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LD) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
          }
          // fragment reads between the MFMAs: k-step 1's during k-step 0 (done a quarter before its end), the
          // next tile's first ones during the second half of k-step 1
          if (ks == 0 && m >= 1) {
            constexpr int D = NM * 3 / 4 - 1;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = min(NF, (m - 1) * NF / D); f < min(NF, m * NF / D); ++f) read_frag(a_s, w_s, 1, f);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (ks == 1 && has_next && m > NM / 2) {
            constexpr int D = NM / 2 - 2;
            const int mm = m - NM / 2;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = min(NF, (mm - 1) * NF / D); f < min(NF, mm * NF / D); ++f) read_frag(a_n, w_n, 0, f);
            __builtin_amdgcn_sched_barrier(0);
          }
          acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ws[ks][j], xs[ks][i], acc[j][i], 0, 0, 0);
          if (ks == 1 && has_next2) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = m * PER_TILE / NM; q < (m + 1) * PER_TILE / NM; ++q) issue_load(stage, (t + 2) * BK, q);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  int t = 0;
  for (; t + 2 < n_kt; ++t) tile_step(t, std::true_type{}, std::true_type{});
  if (t + 1 < n_kt) { tile_step(t, std::true_type{}, std::false_type{}); ++t; }
  if (t < n_kt) tile_step(t, std::false_type{}, std::false_type{});

  // ---- epilogue through the wave's own LDS region, 32 rows at a time (as in the 32x32 kernel) ----
  constexpr int ROW_F = 64 + 4;
  float* stage_f = (float*)smem_raw + wave * (32 * ROW_F);
  static_assert(NW * 32 * ROW_F * 4 <= NSTAGE * (BM + BN) * BK * 2, "staging region fits the tile ring");
  const bool swiglu = (epi & EPI_SWIGLU) != 0;
  int lane_e = lane;
  asm volatile("" : "+v"(lane_e));  // indices derived after the k loop: not kept in registers across it
  const int er = lane_e & 15, eq = lane_e >> 4;
  const int rr = lane_e >> 4, c4 = (lane_e & 15) * 4;
  const int rr_s = lane_e >> 3, c4_s = (lane_e & 7) * 4;
#pragma unroll
  for (int ib = 0; ib < TM / 2; ++ib) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int i = 2 * ib + h;
      float* rowp = stage_f + (16 * h + er) * ROW_F + 4 * eq;
      if (swiglu) {
        // gate rows are the first 32 W rows of the wave's 64, up rows the next 32: tiles j and j + TN/2
#pragma unroll
        for (int j = 0; j < TN / 2; ++j) {
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = acc[j][i][e], u = acc[j + TN / 2][i][e];
            const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
            o[e] = g * sig * u;
          }
          *(f32x4*)(rowp + 16 * j) = o;
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) *(f32x4*)(rowp + 16 * j) = acc[j][i];
      }
    }
    __builtin_amdgcn_wave_barrier();
    const int mb = m0 + wm * WTM + ib * 32;
    if (swiglu) {
      const int fb = (n0 + wn * WTN) / 2;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int r = it * 8 + rr_s, m = mb + r, f = fb + c4_s;
        const f32x4 v = *(const f32x4*)(stage_f + r * ROW_F + c4_s);
        if (m < M && f < N / 2) {
          bf16x4 o;
          o[0] = (bf16_t)v[0]; o[1] = (bf16_t)v[1]; o[2] = (bf16_t)v[2]; o[3] = (bf16_t)v[3];
          *(bf16x4*)((bf16_t*)C + (int64_t)m * ldc + f) = o;
        }
      }
    } else {
      const int n = n0 + wn * WTN + c4;
      f32x4 res[8];
      if (epi & EPI_RESIDUAL) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int m = min(mb + it * 4 + rr, M - 1), nn = min(n, N - 4);
          if (epi & EPI_R_F32) {
            res[it] = *(const f32x4*)((const float*)R + (int64_t)m * ldr + nn);
          } else {
            const bf16x4 rb = *(const bf16x4*)((const bf16_t*)R + (int64_t)m * ldr + nn);
            res[it][0] = (float)rb[0]; res[it][1] = (float)rb[1]; res[it][2] = (float)rb[2]; res[it][3] = (float)rb[3];
          }
        }
      }
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int r = it * 4 + rr, m = mb + r;
        f32x4 v = *(const f32x4*)(stage_f + r * ROW_F + c4);
        if (epi & EPI_RESIDUAL) v += res[it];
        if (m < M && n < N) store_quad(C, ldc, nullptr, 0, m, n, v, epi & ~(EPI_RESIDUAL | EPI_R_F32));
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// Sum over the K splits of the quads at P + k * stride, k = 0 .. splits-1, added in split order.  The reductions are
// short chains of dependent steps on little data: what they take is round trips to memory, so the loads of four
// splits (of two columns at once in the second form) are requested together.
__device__ __forceinline__ f32x4 sum_splits(const float* __restrict__ p, int64_t stride, int splits) {
  f32x4 a = *(const f32x4*)p;
  int k = 1;
  for (; k + 3 < splits; k += 4) {
    f32x4 b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) b[u] = *(const f32x4*)(p + (k + u) * stride);
#pragma unroll
    for (int u = 0; u < 4; ++u) a += b[u];
  }
  {  // the last one to three splits, requested together as well
    f32x4 b[3];
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (k + u < splits) b[u] = *(const f32x4*)(p + (k + u) * stride);
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (k + u < splits) a += b[u];
  }
  return a;
}
__device__ __forceinline__ void sum_splits2(const float* __restrict__ p, const float* __restrict__ q, int64_t stride,
                                            int splits, f32x4* a_out, f32x4* c_out) {
  f32x4 a = *(const f32x4*)p, c = *(const f32x4*)q;
  int k = 1;
  for (; k + 3 < splits; k += 4) {
    f32x4 b[4], d[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      b[u] = *(const f32x4*)(p + (k + u) * stride);
      d[u] = *(const f32x4*)(q + (k + u) * stride);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      a += b[u];
      c += d[u];
    }
  }
  {
    f32x4 b[3], d[3];
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (k + u < splits) {
        b[u] = *(const f32x4*)(p + (k + u) * stride);
        d[u] = *(const f32x4*)(q + (k + u) * stride);
      }
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (k + u < splits) {
        a += b[u];
        c += d[u];
      }
  }
  *a_out = a;
  *c_out = c;
}

// C[m][n] = bf16( sum_s P[s][m][n] (+ R[m][n]) ), the partials added in split order.
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float* __restrict__ P, void* __restrict__ C, int64_t ldc,
                                                            const void* __restrict__ R, int64_t ldr, int M, int N,
                                                            int splits, int epi) {
  const int64_t quads = (int64_t)M * (N / 4);
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= quads) return;
  const int m = (int)(i / (N / 4)), n = (int)(i - (int64_t)m * (N / 4)) * 4;
  const f32x4 s = sum_splits(P + (int64_t)m * N + n, (int64_t)M * N, splits);
  store_quad(C, ldc, R, ldr, m, n, s, epi);
}

// The same for the gate/up projection, with SwiGLU applied to the sums: act[m][f] = silu(gate) * up, where gate
// column f sits at packed column (f/32)*64 + f%32 of P and its up column 32 further (rows of W interleaved in
// blocks of 32).  N = 2F columns in P, F columns in act.
// ssq != nullptr: the projection's input rows were x*g without the RMSNorm factor; the sums of row m are multiplied
// by rsqrt(mean(x^2) + eps) here, from the row's n_parts partial sums of squares (row_scale below).
__device__ __forceinline__ float row_scale(const float* __restrict__ ssq, int m, int n_parts, float inv_d, float eps) {
  float ss = 0.f;
  for (int c = 0; c < n_parts; ++c) ss += ssq[m * n_parts + c];
  return rsqrtf(ss * inv_d + eps);
}

__global__ void __launch_bounds__(256) splitk_reduce_swiglu_kernel(const float* __restrict__ P, bf16_t* __restrict__ act,
                                                                   int64_t ldc, int M, int N, int splits,
                                                                   const float* __restrict__ ssq, int n_parts, float inv_d,
                                                                   float eps) {
  const int F = N / 2;
  const int64_t quads = (int64_t)M * (F / 4);
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= quads) return;
  const int m = (int)(i / (F / 4)), f = (int)(i - (int64_t)m * (F / 4)) * 4;
  const int pg = (f / 32) * 64 + f % 32;
  f32x4 g, u;
  sum_splits2(P + (int64_t)m * N + pg, P + (int64_t)m * N + pg + 32, (int64_t)M * N, splits, &g, &u);
  if (ssq) {
    const float rs = row_scale(ssq, m, n_parts, inv_d, eps);
    g *= rs;
    u *= rs;
  }
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g[e]));
    o[e] = (bf16_t)(g[e] * sig * u[e]);
  }
  *(bf16x4*)(act + (int64_t)m * ldc + f) = o;
}

// The same for the fused QKV projection of few token rows, followed by what rope_kv_write_kernel does: q and k
// heads rotated with the (cos, sin) table of the tokens (pairs (i, i + dh/2)), q written to the qkv buffer, rotated
// k and v written to the rows of the cache.  One thread per 4 rotary pairs, or per 4 values of v.
__global__ void __launch_bounds__(256) splitk_reduce_rope_kernel(const float* __restrict__ P, bf16_t* __restrict__ qkv,
                                                                 int64_t ldq, const float2* __restrict__ cs,
                                                                 bf16_t* __restrict__ k_rows, bf16_t* __restrict__ v_rows,
                                                                 int M, int N, int splits, int Hq, int Hkv, int dh,
                                                                 const float* __restrict__ ssq, int n_parts, float inv_d,
                                                                 float eps) {
  const int half = dh / 2;
  const int rot_units = (Hq + Hkv) * (half / 4), v_units = Hkv * dh / 4;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)M * (rot_units + v_units)) return;
  const int m = (int)(i / (rot_units + v_units)), u = (int)(i - (int64_t)m * (rot_units + v_units));
  const int kvw = Hkv * dh;
  const float rs = ssq ? row_scale(ssq, m, n_parts, inv_d, eps) : 1.0f;
  const float* row = P + (int64_t)m * N;
  const int64_t stride = (int64_t)M * N;
  auto to_bf16 = [](f32x4 v) {
    bf16x4 o;
    o[0] = (bf16_t)v[0]; o[1] = (bf16_t)v[1]; o[2] = (bf16_t)v[2]; o[3] = (bf16_t)v[3];
    return o;
  };
  if (u < rot_units) {
    const int head = u / (half / 4), i0 = (u % (half / 4)) * 4;
    f32x4 x1, x2;
    sum_splits2(row + head * dh + i0, row + head * dh + i0 + half, stride, splits, &x1, &x2);
    x1 *= rs;  // 1 when the input rows carried their RMSNorm factor already
    x2 *= rs;
    f32x4 y1, y2;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float2 c = cs[(int64_t)m * half + i0 + e];
      y1[e] = x1[e] * c.x - x2[e] * c.y;
      y2[e] = x2[e] * c.x + x1[e] * c.y;
    }
    bf16_t* dst = head < Hq ? qkv + (int64_t)m * ldq + head * dh + i0 : k_rows + (int64_t)m * kvw + (head - Hq) * dh + i0;
    *(bf16x4*)dst = to_bf16(y1);
    *(bf16x4*)(dst + half) = to_bf16(y2);
  } else {
    const int j = (u - rot_units) * 4;
    *(bf16x4*)(v_rows + (int64_t)m * kvw + j) = to_bf16(sum_splits(row + (Hq + Hkv) * dh + j, stride, splits) * rs);
  }
}

// The same for a projection with residual whose result feeds an RMSNorm (the O projection before the MLP): one
// workgroup per token row adds the partial sums and the residual, writes the fp32 residual stream h and the
// normalised row xn = h * rsqrt(mean(h^2) + eps) * g in bf16.  d <= 1024 * NCH.
template <int NCH>
__global__ void __launch_bounds__(256) splitk_reduce_rmsnorm_kernel(const float* __restrict__ P, float* __restrict__ h,
                                                                    const void* __restrict__ R, int r_f32,
                                                                    const bf16_t* __restrict__ g, bf16_t* __restrict__ xn,
                                                                    int M, int d, int splits, float eps) {
  __shared__ float part[4];
  const int m = blockIdx.x;
  f32x4 v[NCH];
  float ss = 0.f;
  // partial sums in split order; the loads of four splits are issued together (one workgroup per row: it is
  // the loads in flight per lane that decide how fast the row arrives)
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int n = (threadIdx.x + c * 256) * 4;
    if (n < d) v[c] = *(const f32x4*)(P + (int64_t)m * d + n);
  }
  int k = 1;
  for (; k + 3 < splits; k += 4) {
    f32x4 b[4][NCH];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int n = (threadIdx.x + c * 256) * 4;
        if (n < d) b[u][c] = *(const f32x4*)(P + ((int64_t)(k + u) * M + m) * d + n);
      }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int n = (threadIdx.x + c * 256) * 4;
        if (n < d) v[c] += b[u][c];
      }
  }
  for (; k < splits; ++k) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int n = (threadIdx.x + c * 256) * 4;
      if (n < d) v[c] += *(const f32x4*)(P + ((int64_t)k * M + m) * d + n);
    }
  }
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int n = (threadIdx.x + c * 256) * 4;
    if (n < d) {
      f32x4 a = v[c];
      if (r_f32) {
        a += *(const f32x4*)((const float*)R + (int64_t)m * d + n);
      } else {
        const bf16x4 r = *(const bf16x4*)((const bf16_t*)R + (int64_t)m * d + n);
        a[0] += (float)r[0]; a[1] += (float)r[1]; a[2] += (float)r[2]; a[3] += (float)r[3];
      }
      *(f32x4*)(h + (int64_t)m * d + n) = a;
      v[c] = a;
      ss += a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3];
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float r = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int n = (threadIdx.x + c * 256) * 4;
    if (n < d) {
      const bf16x4 gg = *(const bf16x4*)(g + n);
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(v[c][e] * r * (float)gg[e]);
      *(bf16x4*)(xn + (int64_t)m * d + n) = o;
    }
  }
}

// A projection with residual whose result feeds an RMSNorm, with the norm's row factor left to the next projection's
// reduction: h = sum of the partials + R (fp32 residual stream), a = bf16(h * g) (what that projection reads), and
// ssq[m][c] = sum of h^2 over columns 1024c .. 1024c+1023 (one workgroup per row and 1024 columns; the partial sums
// of a row are added in index order by row_scale).  N a multiple of 1024.
__global__ void __launch_bounds__(256) splitk_reduce_prescale_kernel(const float* __restrict__ P, float* __restrict__ h,
                                                                     const void* __restrict__ R, int r_f32,
                                                                     const bf16_t* __restrict__ g, bf16_t* __restrict__ a,
                                                                     float* __restrict__ ssq, int M, int N, int splits) {
  __shared__ float part[4];
  const int n_parts = N / 1024;
  const int m = blockIdx.x / n_parts, c = blockIdx.x % n_parts;
  const int n = c * 1024 + threadIdx.x * 4;
  f32x4 v = sum_splits(P + (int64_t)m * N + n, (int64_t)M * N, splits);
  if (r_f32) {
    v += *(const f32x4*)((const float*)R + (int64_t)m * N + n);
  } else {
    const bf16x4 rb = *(const bf16x4*)((const bf16_t*)R + (int64_t)m * N + n);
    v[0] += (float)rb[0]; v[1] += (float)rb[1]; v[2] += (float)rb[2]; v[3] += (float)rb[3];
  }
  *(f32x4*)(h + (int64_t)m * N + n) = v;
  const bf16x4 gg = *(const bf16x4*)(g + n);
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(v[e] * (float)gg[e]);
  *(bf16x4*)(a + (int64_t)m * N + n) = o;
  float ss = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssq[m * n_parts + c] = (part[0] + part[1]) + (part[2] + part[3]);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool PARTIAL, int SCHED = 0>
hipError_t launch(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc, const void* R, int64_t ldr,
                  float* P, int M, int N, int K, int epi, int splits, int kt_per_split, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, PARTIAL, SCHED>;
  constexpr int lds = NSTAGE * (BM + BN) * BK * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  DSK_LAUNCH_TIMED(kern, dim3(tiles_m * tiles_n, splits), dim3(WAVES_M * WAVES_N * 64), lds, s, (const bf16_t*)A, lda,
                   (const bf16_t*)W, ldw, C, ldc, R, ldr, P, M, N, K, epi, tiles_m, tiles_n, kt_per_split);
  return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch16(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc, const void* R, int64_t ldr,
                    int M, int N, int K, int epi, hipStream_t s) {
  auto kern = gemm16_bf16_kernel<BM, BN, WAVES_M, WAVES_N>;
  constexpr int lds = NSTAGE * (BM + BN) * BK * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  DSK_LAUNCH_TIMED(kern, dim3(tiles_m * tiles_n), dim3(WAVES_M * WAVES_N * 64), lds, s, (const bf16_t*)A, lda,
                   (const bf16_t*)W, ldw, C, ldc, R, ldr, M, N, K, epi, tiles_m, tiles_n, (const int4*)nullptr, (int64_t)0);
  return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch16_grouped(const void* A, int64_t lda, const void* W, int64_t ldw, int64_t w_group_stride, void* C,
                            int64_t ldc, int N, int K, int epi, const int4* tile_tab, int tile_rows, hipStream_t s) {
  auto kern = gemm16_bf16_kernel<BM, BN, WAVES_M, WAVES_N, true>;
  constexpr int lds = NSTAGE * (BM + BN) * BK * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles_n = (N + BN - 1) / BN;
  DSK_LAUNCH_TIMED(kern, dim3(tile_rows * tiles_n), dim3(WAVES_M * WAVES_N * 64), lds, s, (const bf16_t*)A, lda,
                   (const bf16_t*)W, ldw, C, ldc, (const void*)nullptr, (int64_t)0, 0, N, K, epi, tile_rows, tiles_n,
                   tile_tab, w_group_stride);
  return hipGetLastError();
}

int g_variant = 0;

}  // namespace

void gemm_mfma_set_variant(int v) { g_variant = v; }

// How a projection over few token rows (M <= 64) is split: 64x64 tiles and about 768 workgroups; a very wide N
// (the gate/up projection) has enough 64x128 tiles to fill the chip with few splits, which halves the share of the
// token rows in the tile loads (measured on M = 64, N = 28672, K = 4096: 54 us against 64 us; narrower shapes are
// best left as they are).  Returns whether the K-split path can run (more than one split, partials fit in ws).
static bool small_m_plan(int M, int N, int K, int64_t ws_bytes, bool* wide, int* splits, int* per) {
  const int KT = K / BK;
  *wide = (N + 127) / 128 >= 192;
  const int tiles = ((M + 63) / 64) * (*wide ? (N + 127) / 128 : (N + 63) / 64);
  int sp = ((*wide ? 512 : 768) + tiles - 1) / tiles;
  sp = max(1, min(sp, KT / 2));
  *per = (KT + sp - 1) / sp;
  *splits = (KT + *per - 1) / *per;
  return *splits > 1 && (int64_t)*splits * M * N * 4 <= ws_bytes;
}

// The fused gate/up epilogue needs whole 64-column gate/up blocks; over few token rows it is applied by the
// split-K reduction, so there it needs the K-split path.
bool gemm_mfma_swiglu_supported(int M, int N, int K, int64_t ws_bytes) {
  if (N % 64 != 0 || K < BK || K % BK != 0) return false;
  if (M > 64) return true;
  bool wide;
  int splits, per;
  return small_m_plan(M, N, K, ws_bytes, &wide, &splits, &per);
}

// 64 token rows x (splits x N) floats: about 768 tiles of 64 columns (+ one more split's worth) for the 64x64
// tiling, up to 4 splits of a wide N for the 64x128 tiling
int64_t gemm_mfma_workspace_bytes(int max_n) { return (int64_t)64 * 4 * ((int64_t)768 * 64 + (int64_t)4 * max_n); }

// Whether a projection of this size runs on the 256 x 256 prefill tiling (the kernel the roofline figure is about).
bool gemm_mfma_uses_prefill_tile(int M, int N) {
  return M > 64 && (int64_t)((M + 255) / 256) * ((N + 255) / 256) >= 192;
}

hipError_t launch_gemm_mfma_bf16(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                                 const void* R, int64_t ldr, int M, int N, int K, int epi, void* ws, int64_t ws_bytes,
                                 hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K < BK || K % BK || N % 4 || (lda & 7) || (ldw & 7) || (ldc & 3) || ((epi & EPI_RESIDUAL) && (ldr & 3)))
    return hipErrorNotSupported;
  // rows are addressed by 32-bit byte offsets from the matrix base
  if ((int64_t)M * lda * 2 >= ((int64_t)1 << 32) || (int64_t)N * ldw * 2 >= ((int64_t)1 << 32)) return hipErrorNotSupported;
  const int KT = K / BK;
  int variant = g_variant;
  if (epi & EPI_SWIGLU) {
    if (!gemm_mfma_swiglu_supported(M, N, K, ws ? ws_bytes : 0)) return hipErrorNotSupported;
    if (M <= 64) {
      bool wide;
      int splits, per;
      small_m_plan(M, N, K, ws_bytes, &wide, &splits, &per);
      hipError_t e = wide ? launch<64, 128, 1, 4, true>(A, lda, W, ldw, C, ldc, R, ldr, (float*)ws, M, N, K, 0, splits, per, s)
                          : launch<64, 64, 1, 2, true>(A, lda, W, ldw, C, ldc, R, ldr, (float*)ws, M, N, K, 0, splits, per, s);
      if (e != hipSuccess) return e;
      const int64_t quads = (int64_t)M * (N / 8);
      hipLaunchKernelGGL(splitk_reduce_swiglu_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s,
                         (const float*)ws, (bf16_t*)C, ldc, M, N, splits, (const float*)nullptr, 0, 0.f, 0.f);
      return hipGetLastError();
    }
    if ((int64_t)((M + 255) / 256) * ((N + 255) / 256) >= 192 || variant == 1)
      return launch16<256, 256, 2, 4>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
    return launch<128, 128, 2, 2, false, 1>(A, lda, W, ldw, C, ldc, R, ldr, nullptr, M, N, K, epi, 1, KT, s);
  }
  // A few hundred token rows: too few 128 x 128 tiles to fill the chip, so K is split over workgroups as on the
  // few-row path (fp32 partial planes, fixed-order reduce); every split gets at least two k-tiles.
  if (variant == 0 && M > 64 && ws) {
    const int64_t tiles = (int64_t)((M + 127) / 128) * ((N + 127) / 128);
    if (tiles <= 256) {
      int sp = (int)((512 + tiles - 1) / tiles);
      sp = max(1, min(sp, KT / 2));
      while (sp > 1 && (int64_t)sp * M * N * 4 > ws_bytes) --sp;
      const int per = (KT + sp - 1) / sp;
      const int splits = (KT + per - 1) / per;
      if (splits > 1) {
        hipError_t e = launch<128, 128, 2, 2, true, 1>(A, lda, W, ldw, C, ldc, R, ldr, (float*)ws, M, N, K, epi, splits, per, s);
        if (e != hipSuccess) return e;
        const int64_t quads = (int64_t)M * (N / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, (const float*)ws,
                           C, ldc, R, ldr, M, N, splits, epi);
        return hipGetLastError();
      }
    }
  }
  if (variant == 0) {
    if (M <= 64) variant = 3;
    else if ((int64_t)((M + 255) / 256) * ((N + 255) / 256) >= 192) variant = 1;
    else variant = 2;
  }
  switch (variant) {
    case 3: {  // weight streaming: K split over workgroups, fp32 partial planes, fixed-order reduce
      bool wide;
      int splits, per;
      if (ws && small_m_plan(M, N, K, ws_bytes, &wide, &splits, &per)) {
        hipError_t e = wide ? launch<64, 128, 1, 4, true>(A, lda, W, ldw, C, ldc, R, ldr, (float*)ws, M, N, K, epi, splits, per, s)
                            : launch<64, 64, 1, 2, true>(A, lda, W, ldw, C, ldc, R, ldr, (float*)ws, M, N, K, epi, splits, per, s);
        if (e != hipSuccess) return e;
        const int64_t quads = (int64_t)M * (N / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, (const float*)ws,
                           C, ldc, R, ldr, M, N, splits, epi);
        return hipGetLastError();
      }
      return launch<64, 64, 1, 2, false>(A, lda, W, ldw, C, ldc, R, ldr, nullptr, M, N, K, epi, 1, KT, s);
    }
    // the two prefill tilings: the 256x256 tile on the 16x16x32 MFMA (1; large problems are power-limited, and that
    // instruction is the thriftier one) and the 128x128 tile on the 32x32x16 MFMA (2; medium sizes are issue- and
    // latency-bound, where it is 15-30 % faster)
    case 2: return launch<128, 128, 2, 2, false, 1>(A, lda, W, ldw, C, ldc, R, ldr, nullptr, M, N, K, epi, 1, KT, s);
    default: return launch16<256, 256, 2, 4>(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
  }
}

// Projections of a mixture-of-experts layer over token rows sorted by expert: one launch over all experts, on the
// 256-row prefill tiling.  tile_tab[0..tile_rows) describes the row tiles and tile_tab[tile_rows] holds their number
// (see the kernel); rows of A and C are the sorted slots.  epi: EPI_SWIGLU (C bf16 [slots, N/2]) or EPI_C_F32 / EPI_STORE (C [slots, N]); no residual.
hipError_t launch_gemm_mfma_grouped(const void* A, int64_t lda, int64_t a_rows, const void* W, int64_t ldw,
                                    int64_t w_group_stride, void* C, int64_t ldc, int N, int K, int epi,
                                    const void* tile_tab, int tile_rows, hipStream_t s) {
  if (tile_rows <= 0) return hipSuccess;
  if (K < BK || K % BK || N % 64 || (lda & 7) || (ldw & 7) || (ldc & 3) || (epi & EPI_RESIDUAL)) return hipErrorNotSupported;
  if (a_rows * lda * 2 >= ((int64_t)1 << 32) || (int64_t)N * ldw * 2 >= ((int64_t)1 << 32)) return hipErrorNotSupported;
  return launch16_grouped<256, 256, 2, 4>(A, lda, W, ldw, w_group_stride, C, ldc, N, K, epi, (const int4*)tile_tab,
                                          tile_rows, s);
}

// ---- few token rows (M <= 64): projection + the step that follows it, in the split-K reduction ----

bool gemm_small_m_fused_supported(int M, int N, int K, int64_t lda, int64_t ldw, int64_t ws_bytes) {
  if (M < 1 || M > 64 || K < BK || K % BK || N % 4 || (lda & 7) || (ldw & 7)) return false;
  if ((int64_t)M * lda * 2 >= ((int64_t)1 << 32) || (int64_t)N * ldw * 2 >= ((int64_t)1 << 32)) return false;
  bool wide;
  int splits, per;
  return small_m_plan(M, N, K, ws_bytes, &wide, &splits, &per);
}

static hipError_t small_m_partials(const void* A, int64_t lda, const void* W, int64_t ldw, int M, int N, int K, void* ws,
                                   int64_t ws_bytes, int* splits, hipStream_t s) {
  if (!ws || !gemm_small_m_fused_supported(M, N, K, lda, ldw, ws_bytes)) return hipErrorNotSupported;
  bool wide;
  int per;
  small_m_plan(M, N, K, ws_bytes, &wide, splits, &per);
  return wide ? launch<64, 128, 1, 4, true>(A, lda, W, ldw, nullptr, N, nullptr, 0, (float*)ws, M, N, K, 0, *splits, per, s)
              : launch<64, 64, 1, 2, true>(A, lda, W, ldw, nullptr, N, nullptr, 0, (float*)ws, M, N, K, 0, *splits, per, s);
}

// The two fused launchers below refuse exactly what these predicates refuse; the layer asks them first and takes
// the unfused steps (projection, then RoPE / RMSNorm kernel) otherwise.
bool gemm_small_m_rope_supported(int M, int K, int Hq, int Hkv, int dh, int64_t lda, int64_t ldw, int64_t ldq,
                                 int64_t ws_bytes) {
  return dh % 8 == 0 && (ldq & 3) == 0 && gemm_small_m_fused_supported(M, (Hq + 2 * Hkv) * dh, K, lda, ldw, ws_bytes);
}

bool gemm_small_m_rmsnorm_supported(int M, int d, int K, int64_t lda, int64_t ldw, int64_t ws_bytes) {
  return d % 4 == 0 && d <= 8192 && gemm_small_m_fused_supported(M, d, K, lda, ldw, ws_bytes);
}

// qkv projection + RoPE + KV-cache write: N = (Hq + 2 Hkv) dh
// ssq (optional): the rows of A are x*g of an RMSNorm over K columns without its row factor, ssq [M, K/1024] holds
// the partial sums of x^2 (splitk_reduce_prescale_kernel), and the factor is applied to the sums here
hipError_t launch_gemm_small_m_rope(const void* A, int64_t lda, const void* W, int64_t ldw, void* qkv, int64_t ldq,
                                    const float2* cs, void* k_rows, void* v_rows, int M, int K, int Hq, int Hkv, int dh,
                                    void* ws, int64_t ws_bytes, const float* ssq, float eps, hipStream_t s) {
  const int N = (Hq + 2 * Hkv) * dh;
  if (!ws || !gemm_small_m_rope_supported(M, K, Hq, Hkv, dh, lda, ldw, ldq, ws_bytes)) return hipErrorNotSupported;
  if (ssq && K % 1024) return hipErrorNotSupported;
  int splits = 0;
  hipError_t e = small_m_partials(A, lda, W, ldw, M, N, K, ws, ws_bytes, &splits, s);
  if (e != hipSuccess) return e;
  const int64_t units = (int64_t)M * ((Hq + Hkv) * (dh / 8) + Hkv * dh / 4);
  hipLaunchKernelGGL(splitk_reduce_rope_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s, (const float*)ws,
                     (bf16_t*)qkv, ldq, cs, (bf16_t*)k_rows, (bf16_t*)v_rows, M, N, splits, Hq, Hkv, dh, ssq, K / 1024,
                     1.0f / (float)K, eps);
  return hipGetLastError();
}

// gate/up projection + SwiGLU over few rows whose input lacks the RMSNorm row factor (see above): act [M, N/2]
hipError_t launch_gemm_small_m_swiglu_scaled(const void* A, int64_t lda, const void* W, int64_t ldw, void* act, int64_t ldc,
                                             int M, int N, int K, void* ws, int64_t ws_bytes, const float* ssq, float eps,
                                             hipStream_t s) {
  if (!ws || !ssq || K % 1024 || N % 64 || !gemm_small_m_fused_supported(M, N, K, lda, ldw, ws_bytes)) return hipErrorNotSupported;
  int splits = 0;
  hipError_t e = small_m_partials(A, lda, W, ldw, M, N, K, ws, ws_bytes, &splits, s);
  if (e != hipSuccess) return e;
  const int64_t quads = (int64_t)M * (N / 8);
  hipLaunchKernelGGL(splitk_reduce_swiglu_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, (const float*)ws,
                     (bf16_t*)act, ldc, M, N, splits, ssq, K / 1024, 1.0f / (float)K, eps);
  return hipGetLastError();
}

// projection + residual, result prepared for an RMSNorm whose row factor the next projection applies:
// h [M, d] fp32 = x W^T + R, a [M, d] bf16 = h * g, ssq [M, d/1024] partial sums of h^2; d a multiple of 1024
bool gemm_small_m_prescale_supported(int M, int d, int K, int64_t lda, int64_t ldw, int64_t ws_bytes) {
  return d % 1024 == 0 && d / 1024 <= DSK_MAX_SSQ_PARTS && gemm_small_m_fused_supported(M, d, K, lda, ldw, ws_bytes);
}

hipError_t launch_gemm_small_m_prescale(const void* A, int64_t lda, const void* W, int64_t ldw, float* h, const void* R,
                                        int r_f32, const void* g, void* a, float* ssq, int M, int d, int K, void* ws,
                                        int64_t ws_bytes, hipStream_t s) {
  if (!ws || !gemm_small_m_prescale_supported(M, d, K, lda, ldw, ws_bytes)) return hipErrorNotSupported;
  int splits = 0;
  hipError_t e = small_m_partials(A, lda, W, ldw, M, d, K, ws, ws_bytes, &splits, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(splitk_reduce_prescale_kernel, dim3((unsigned)(M * (d / 1024))), dim3(256), 0, s, (const float*)ws, h, R,
                     r_f32, (const bf16_t*)g, (bf16_t*)a, ssq, M, d, splits);
  return hipGetLastError();
}

// projection + residual + RMSNorm: h[M, d] (fp32) = x W^T + R, xn[M, d] (bf16) = rmsnorm(h) * g; dense rows
hipError_t launch_gemm_small_m_rmsnorm(const void* A, int64_t lda, const void* W, int64_t ldw, float* h, const void* R,
                                       int r_f32, const void* g, void* xn, float eps, int M, int d, int K, void* ws,
                                       int64_t ws_bytes, hipStream_t s) {
  if (!ws || !gemm_small_m_rmsnorm_supported(M, d, K, lda, ldw, ws_bytes)) return hipErrorNotSupported;
  int splits = 0;
  hipError_t e = small_m_partials(A, lda, W, ldw, M, d, K, ws, ws_bytes, &splits, s);
  if (e != hipSuccess) return e;
  if (d <= 4096)
    hipLaunchKernelGGL(splitk_reduce_rmsnorm_kernel<4>, dim3(M), dim3(256), 0, s, (const float*)ws, h, R, r_f32,
                       (const bf16_t*)g, (bf16_t*)xn, M, d, splits, eps);
  else
    hipLaunchKernelGGL(splitk_reduce_rmsnorm_kernel<8>, dim3(M), dim3(256), 0, s, (const float*)ws, h, R, r_f32,
                       (const bf16_t*)g, (bf16_t*)xn, M, d, splits, eps);
  return hipGetLastError();
}
