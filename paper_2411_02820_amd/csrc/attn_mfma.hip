// bf16 MFMA flash attention for gfx950: causal grouped-query attention over packed sequences,
// keys taken from up to two row ranges of a cache layer (a fully visible prefix range and the
// queries' own causal range), online softmax in fp32.
//
// A workgroup (4 waves) owns 128 query rows of one (sequence, q head); each wave 32 of them.
// Keys are walked in tiles of 64 cache rows (aligned to multiples of 64), staged in two-stage LDS rings
// by direct global->LDS loads (global_load_lds_dwordx4):
//   K tile  [64 keys][dh]   - rows permuted (bits 2 and 3 of the key offset swapped), see below
//   Vt tile [dh][64 keys]   - from a transposed copy of V kept in the model's workspace
// Both the row permutation and the 16-byte slot swizzle are applied on the global side (which address a
// lane fetches), since the LDS destination of such a load is fixed by the lane id.
// Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16 (K rows as the MFMA A
// operand, Q rows as B): a lane then owns ONE query (column lane%32) and 16 keys per 32-key tile in its
// accumulator registers, so the softmax row maximum/sum are in-lane reductions plus a single exchange
// with lane^32.  With the K-row permutation the 8 registers [8t, 8t+8) of a lane are 8 consecutive keys
// (16t + 8*(lane/32) + 0..7), i.e. exactly the B-operand layout of P^T for O^T += Vt P^T, and the
// matching Vt fragment is one 16-byte LDS read.  The output accumulator O^T[d][q] keeps the query in the
// lane as well, so rescaling by the running maximum is a per-lane scalar multiply.
//
// Few queries against many keys (the suffix pass) would leave most CUs idle, so the key tiles of a
// workgroup can be split over blockIdx.z; each split writes its unnormalised fp32 output with its running
// maximum and sum, and a second kernel merges the splits in a fixed order.
#include "dsk_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BQ = 128;  // query rows per workgroup
constexpr int BKV = 64;  // keys per tile

struct AttnParams {
  const bf16_t* q; int64_t ldq;
  const bf16_t* k; const bf16_t* vt; int64_t ldvt;
  bf16_t* out;
  float* part_o; float* part_ml;  // split mode: [n_q][Hq][splits][dh] and [n_q][Hq][splits][2]
  const int32_t* q_cu; const int32_t* p_cu;
  int n_seqs; int own_row0; int Hq, Hkv; int total_tiles; int splits;
  float c;         // softmax scale * log2(e)
  int k_row_max;   // last cache row that may be read
};

// MFMA row of key offset u inside a 64-key tile: bits 2 and 3 swapped (an involution)
__device__ __forceinline__ int perm_key(int u) { return (u & ~0xC) | ((u & 4) << 1) | ((u & 8) >> 1); }

template <int DH, bool SPLIT>
__global__ void __launch_bounds__(256, 2) attn_bf16_kernel(AttnParams p) {
  constexpr int KCH = DH / 8;             // 16-byte slots per K row
  constexpr int K_RPI = 64 / KCH;         // K rows per wave load instruction
  constexpr int K_INST = BKV / K_RPI / 4; // per wave
  constexpr int V_INST = DH / 8 / 4;      // Vt rows are 64 keys = 8 slots -> 8 rows per instruction
  constexpr int NKS = DH / 16, NDT = DH / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sK = (bf16_t*)smem_raw;        // [2][BKV * DH]  K ring
  bf16_t* sV = sK + 2 * BKV * DH;        // [2][DH * BKV]  Vt ring

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, hh = lane >> 5;
  // ---- which (head, sequence, query tile).  Workgroups are handed out in blockIdx.x order, round-robin over
  //      the 8 XCDs (each with its own L2).  Late query tiles carry the most key tiles, so they come first for
  //      every head (a heavy workgroup started late would run on alone at the end), and with a head count
  //      that is a multiple of 8 each XCD serves a fixed eighth of the heads, so the q heads of one kv group
  //      read their K and Vt through the same L2. ----
  int h, rank;
  {
    const int L = blockIdx.x;
    if ((p.Hq & 7) == 0) {
      const int hpx = p.Hq >> 3, j = L >> 3;
      h = (L & 7) * hpx + j % hpx;
      rank = j / hpx;
    } else {
      h = L % p.Hq;
      rank = L / p.Hq;
    }
  }
  const int kvh = h / (p.Hq / p.Hkv);
  int tile = p.total_tiles - 1 - rank;
  int b = 0, seq_begin = 0, seq_end = 0;
  for (;; ++b) {
    seq_begin = p.q_cu[b];
    seq_end = p.q_cu[b + 1];
    int nt = (seq_end - seq_begin + BQ - 1) / BQ;
    if (tile < nt || b + 1 >= p.n_seqs) break;
    tile -= nt;
  }
  const int q0 = seq_begin + tile * BQ;  // first query row (packed index) of this workgroup
  if (q0 >= seq_end) return;              // cannot happen for a well-formed grid
  const int qw0 = q0 + 32 * wave;         // first query row of this wave
  const bool wave_active = qw0 < seq_end;
  const int qi = min(qw0 + lq, seq_end - 1);  // this lane's query (clamped for the padding rows)

  const int own_begin = p.own_row0 + seq_begin;
  const int lim = p.own_row0 + qi;                                   // last own row this lane's query sees
  const int wave_lim_min = p.own_row0 + min(qw0, seq_end - 1);       // smallest limit in the wave
  const int wave_lim_max = p.own_row0 + min(qw0 + 31, seq_end - 1);  // largest limit in the wave
  const int blk_lim = p.own_row0 + min(q0 + BQ, seq_end) - 1;
  const int pre_begin = p.p_cu ? p.p_cu[b] : 0, pre_end = p.p_cu ? p.p_cu[b + 1] : 0;
  const int ta0 = pre_begin / BKV, nA = pre_end > pre_begin ? (pre_end - 1) / BKV - ta0 + 1 : 0;
  const int tb0 = own_begin / BKV, nB = blk_lim / BKV - tb0 + 1;
  const int n_tiles = nA + nB;
  // key-tile range of this split
  int it_begin = 0, it_end = n_tiles;
  if (SPLIT) {
    const int per = (n_tiles + p.splits - 1) / p.splits;
    it_begin = min(n_tiles, (int)blockIdx.z * per);
    it_end = min(n_tiles, it_begin + per);
  }

  // ---- Q fragments (B operand): query = lane%32, d = 16*ks + 8*(lane/32) .. +7 ----
  bf16x8 qf[NKS];
  {
    const bf16_t* qp = p.q + (int64_t)qi * p.ldq + h * DH + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const bf16x8*)(qp + 16 * ks);
  }

  // ---- tile loads, direct to LDS.  K: LDS row rho (MFMA row) holds key offset perm_key(rho); slot s of a
  //      row holds chunk s ^ kswz(rho).  Vt: LDS row d, slot s holds key chunk s ^ vswz(d).  A 16-byte
  //      fragment read is served 16 lanes (consecutive rows, one slot index) per cycle over 64 banks, so the
  //      16 lanes must land in 16 different 16-byte bank groups: a 256-byte row covers all banks and needs 16
  //      different slots (xor with row % 16); 128-byte rows come two per bank sweep and need 8 different
  //      slots per row pair (xor with (row / 2) % 8). ----
  auto kswz = [](int row) { return DH * 2 == 256 ? (row & 15) : ((row >> 1) & 7); };
  auto vswz = [](int d) { return (d >> 1) & 7; };
  const int64_t ldkv = (int64_t)p.Hkv * DH;
  const bf16_t* k_base = p.k + kvh * DH;
  int k_u[K_INST], k_coff[K_INST];
  const bf16_t* v_src[V_INST];
#pragma unroll
  for (int i = 0; i < K_INST; ++i) {
    const int rho = K_RPI * (wave * K_INST + i) + lane / KCH, s = lane % KCH;
    k_u[i] = perm_key(rho);
    k_coff[i] = (s ^ kswz(rho)) * 8;
  }
#pragma unroll
  for (int i = 0; i < V_INST; ++i) {
    const int d = 8 * (wave * V_INST + i) + (lane >> 3), s = lane & 7;
    v_src[i] = p.vt + ((int64_t)kvh * DH + d) * p.ldvt + (s ^ vswz(d)) * 8;
  }
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void glb_void;
  auto tile_row0 = [&](int it) { return (it < nA ? ta0 + it : tb0 + (it - nA)) * BKV; };
  auto issue_k = [&](int it) {
    const int r0 = tile_row0(it), stage = (it - it_begin) & 1;
#pragma unroll
    for (int i = 0; i < K_INST; ++i) {
      const int row = min(r0 + k_u[i], p.k_row_max);
      __builtin_amdgcn_global_load_lds((glb_void*)(k_base + (int64_t)row * ldkv + k_coff[i]),
                                       (lds_void*)(sK + stage * BKV * DH + K_RPI * (wave * K_INST + i) * DH), 16, 0, 0);
    }
  };
  auto issue_v = [&](int it) {
    const int r0 = tile_row0(it), stage = (it - it_begin) & 1;
#pragma unroll
    for (int i = 0; i < V_INST; ++i)
      __builtin_amdgcn_global_load_lds((glb_void*)(v_src[i] + r0),
                                       (lds_void*)(sV + stage * DH * BKV + 8 * (wave * V_INST + i) * BKV), 16, 0, 0);
  };
  // a wave skips a tile that lies wholly beyond the causal limit of all its queries
  auto tile_skipped = [&](int it) { return !wave_active || (it >= nA && tile_row0(it) > wave_lim_max); };
  // S^T = K Q^T for the two 32-key halves of tile `it`
  auto scores = [&](int it, f32x16* s) {
    const bf16_t* kt_s = sK + ((it - it_begin) & 1) * BKV * DH;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
      const int row = 32 * kt + lq;
      const bf16_t* kr = kt_s + row * DH;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        bf16x8 kf = *(const bf16x8*)(kr + (((2 * ks + hh) ^ kswz(row)) * 8));
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kt], 0, 0, 0);
      }
    }
  };

  f32x16 o[NDT];
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  // Software pipeline over key tiles, one barrier per tile:
  //   [wait K(i+1), Vt(i); barrier]  issue loads K(i+2), Vt(i+1)  |  S(i+1) = K(i+1) Q^T (MFMA)
  //   softmax of S(i) (VALU, runs while the MFMAs of S(i+1) drain)  |  O^T += Vt(i) P(i)^T (MFMA)
  // so a wave always has matrix work in flight during its softmax.  Two-stage rings suffice: K(i+2) overwrites
  // K(i), whose last reader S(i) ran one iteration earlier (before this iteration's barrier); Vt(i+1)
  // overwrites Vt(i-1), last read by the previous iteration's O update.
  f32x16 s_cur[2], s_nxt[2];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) s_cur[kt][r] = s_nxt[kt][r] = 0.f;
  if (it_begin < it_end) {
    issue_k(it_begin);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (it_begin + 1 < it_end) issue_k(it_begin + 1);
    issue_v(it_begin);
    if (!tile_skipped(it_begin)) scores(it_begin, s_cur);
  }
  for (int it = it_begin; it < it_end; ++it) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // K(it+1) and Vt(it): this wave's part
    __syncthreads();
    if (it + 2 < it_end) issue_k(it + 2);
    if (it + 1 < it_end) issue_v(it + 1);
    const bool skip_next = it + 1 >= it_end || tile_skipped(it + 1);
    if (!skip_next) scores(it + 1, s_nxt);
    const int r0 = tile_row0(it);
    const bool segA = it < nA;
    // visible key rows for this lane in this segment: [lo, hi]
    const int lo = segA ? pre_begin : own_begin;
    const int hi = segA ? pre_end - 1 : lim;
    if (!tile_skipped(it)) {
      f32x16* s = s_cur;
      // mask: register r of half kt is key r0 + 32*kt + 16*(r/8) + 8*(lane/32) + r%8
      const bool full = r0 >= lo && r0 + BKV - 1 <= (segA ? pre_end - 1 : wave_lim_min);
      if (!full) {
        const int kb = r0 + 8 * hh;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kb + 32 * kt + 16 * (r >> 3) + (r & 7);
            s[kt][r] = (key >= lo && key <= hi) ? s[kt][r] : -INFINITY;
          }
      }
      // online softmax; the query's 64 scores sit in this lane and in lane^32
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f((m - m_safe) * p.c);
      const float mc = m_safe * p.c;
      float psum = 0.f;
      bf16x8 pf[2][2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float e = __builtin_amdgcn_exp2f(s[kt][r] * p.c - mc);
          psum += e;
          pf[kt][r >> 3][r & 7] = (bf16_t)e;
        }
      l = l * alpha + psum;
      m = m_new;
      // rescale the output accumulators only if some query of the wave saw a new maximum (after the first
      // few tiles of a row that is rare)
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
      }
      // O^T += Vt P^T
      const bf16_t* vt_s = sV + ((it - it_begin) & 1) * DH * BKV;
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt) {
        const int d = 32 * dt + lq;
        const bf16_t* vr = vt_s + d * BKV;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            bf16x8 vf = *(const bf16x8*)(vr + (((4 * kt + 2 * t + hh) ^ vswz(d)) * 8));
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kt][t], o[dt], 0, 0, 0);
          }
      }
    }
    s_cur[0] = s_nxt[0];
    s_cur[1] = s_nxt[1];
  }

  // ---- store: register 4g+e of d-tile dt is out[q][32dt + 8g + 4*(lane/32) + e] ----
  const float l_tot = l + __shfl_xor(l, 32, 64);
  if (wave_active && qw0 + lq < seq_end) {
    const int64_t qrow = qw0 + lq;
    if (SPLIT) {
      float* po = p.part_o + ((qrow * p.Hq + h) * p.splits + blockIdx.z) * DH;
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 v = {o[dt][4 * g], o[dt][4 * g + 1], o[dt][4 * g + 2], o[dt][4 * g + 3]};
          *(f32x4*)(po + 32 * dt + 8 * g + 4 * hh) = v;
        }
      if (hh == 0) {
        float* pm = p.part_ml + ((qrow * p.Hq + h) * p.splits + blockIdx.z) * 2;
        pm[0] = m;
        pm[1] = l_tot;
      }
    } else {
      const float inv = 1.0f / l_tot;
      bf16_t* op = p.out + qrow * p.Hq * DH + h * DH;
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(o[dt][4 * g + e] * inv);
          *(bf16x4*)(op + 32 * dt + 8 * g + 4 * hh) = v;
        }
    }
  }
}

// out[q][h][:] = sum_s o_s * 2^((m_s - M) c) / sum_s l_s * 2^((m_s - M) c), M = max_s m_s; one wave per (q, h).
template <int DH>
__global__ void __launch_bounds__(64) attn_combine_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                          bf16_t* __restrict__ out, int Hq, int splits, float c) {
  const int64_t qh = (int64_t)blockIdx.x * Hq + blockIdx.y;
  const float* ml = part_ml + qh * splits * 2;
  float M = -INFINITY;
  for (int s = 0; s < splits; ++s) M = fmaxf(M, ml[2 * s]);
  float den = 0.f, acc[DH / 64] = {};
  for (int s = 0; s < splits; ++s) {
    const float ms = ml[2 * s];
    if (ms == -INFINITY) continue;  // this split saw no visible key
    const float w = __builtin_amdgcn_exp2f((ms - M) * c);
    den += ml[2 * s + 1] * w;
#pragma unroll
    for (int a = 0; a < DH / 64; ++a) acc[a] += part_o[(qh * splits + s) * DH + threadIdx.x + 64 * a] * w;
  }
  const float inv = 1.0f / den;
#pragma unroll
  for (int a = 0; a < DH / 64; ++a) out[qh * DH + threadIdx.x + 64 * a] = (bf16_t)(acc[a] * inv);
}

// Vt[(kvh*dh + d)*ldvt + row] = V[row][kvh*dh + d] for the valid rows, 0 for the others, over whole
// 64-row tiles.  valid(row) = row < n_pre || own_row0 <= row < own_row0 + n_own.
__global__ void __launch_bounds__(256) transpose_v_kernel(const bf16_t* __restrict__ v_rows, bf16_t* __restrict__ vt,
                                                          int64_t ldvt, int width, int64_t n_pre, int64_t own_row0,
                                                          int64_t n_own) {
  __shared__ bf16_t tile[64][66];
  const int64_t r0 = (int64_t)blockIdx.x * 64;
  const int c0 = blockIdx.y * 64;
  const int tid = threadIdx.x;
  {
    const int r = tid >> 3, ch = tid & 7;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int rr = r + 32 * half;
      const int64_t row = r0 + rr;
      const bool valid = row < n_pre || (row >= own_row0 && row < own_row0 + n_own);
      bf16x8 x;
      if (valid) x = *(const bf16x8*)(v_rows + row * width + c0 + ch * 8);
      else
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (bf16_t)0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) tile[rr][ch * 8 + e] = x[e];
    }
  }
  __syncthreads();
  {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int id = tid + 256 * half, d = id >> 3, rc = id & 7;
      bf16x8 x;
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = tile[rc * 8 + e][d];
      *(bf16x8*)(vt + (int64_t)(c0 + d) * ldvt + r0 + rc * 8) = x;
    }
  }
}

int g_variant = 0;

}  // namespace

void attn_mfma_set_variant(int v) { g_variant = v; }

// fp32 scratch for the split mode: n_q * splits <= kMaxSplitRows partial rows of (dh + 2) floats per q head
constexpr int64_t kMaxSplitRows = 4096;
int64_t attn_mfma_workspace_bytes(int Hq, int dh) { return kMaxSplitRows * Hq * (dh + 2) * 4; }

hipError_t launch_transpose_v(const void* v_rows, void* vt, int64_t ldvt, int width, int64_t n_pre, int64_t own_row0,
                              int64_t n_own, hipStream_t s) {
  const int64_t end = own_row0 + n_own;
  if (end <= 0) return hipSuccess;
  dim3 grid((unsigned)((end + 63) / 64), width / 64);
  hipLaunchKernelGGL(transpose_v_kernel, grid, dim3(256), 0, s, (const bf16_t*)v_rows, (bf16_t*)vt, ldvt, width, n_pre,
                     own_row0, n_own);
  return hipGetLastError();
}

template <int DH, bool SPLIT>
hipError_t launch_attn(const AttnParams& p, dim3 grid, hipStream_t s) {
  auto kern = attn_bf16_kernel<DH, SPLIT>;
  constexpr int lds = (2 * BKV * DH + 2 * DH * BKV) * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_attn_mfma_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_q <= 0) return hipSuccess;
  if ((a.dh != 128 && a.dh != 64) || !a.vt || (a.ldq & 7) || a.own_row0 + a.n_q >= ((int64_t)1 << 31))
    return hipErrorNotSupported;
  AttnParams p;
  p.q = (const bf16_t*)a.q; p.ldq = a.ldq; p.k = (const bf16_t*)a.k_rows; p.vt = (const bf16_t*)a.vt; p.ldvt = a.ldvt;
  p.out = (bf16_t*)a.out; p.q_cu = a.q_cu; p.p_cu = a.p_cu; p.n_seqs = a.n_seqs; p.own_row0 = (int)a.own_row0;
  p.Hq = a.Hq; p.Hkv = a.Hkv;
  int total = 0;
  int64_t max_keys = 0;
  for (int b = 0; b < a.n_seqs; ++b) {
    const int len = a.q_cu_host[b + 1] - a.q_cu_host[b];
    total += (len + BQ - 1) / BQ;
    int64_t keys = len + (a.p_cu_host ? a.p_cu_host[b + 1] - a.p_cu_host[b] : 0);
    if (keys > max_keys) max_keys = keys;
  }
  p.total_tiles = total;
  p.c = (float)(1.4426950408889634 / sqrt((double)a.dh));
  p.k_row_max = (int)(a.own_row0 + a.n_q - 1);
  // split the key tiles when the grid alone cannot fill the chip
  int splits = 1;
  const int64_t blocks = (int64_t)total * a.Hq;
  const int key_tiles = (int)((max_keys + BKV - 1) / BKV) + 1;
  if (a.ws && blocks < 512 && key_tiles >= 8) {
    splits = (int)((1024 + blocks - 1) / blocks);
    if (splits > key_tiles / 4) splits = key_tiles / 4;
    while (splits > 1 && ((int64_t)a.n_q * splits > kMaxSplitRows ||
                          (int64_t)a.n_q * splits * a.Hq * (a.dh + 2) * 4 > a.ws_bytes))
      --splits;
  }
  if (g_variant == 1) splits = 1;
  p.splits = splits;
  p.part_o = nullptr;
  p.part_ml = nullptr;
  if (splits > 1) {
    p.part_o = (float*)a.ws;
    p.part_ml = p.part_o + (int64_t)a.n_q * a.Hq * splits * a.dh;
    dim3 grid((unsigned)total * a.Hq, 1, splits);
    hipError_t e = a.dh == 128 ? launch_attn<128, true>(p, grid, s) : launch_attn<64, true>(p, grid, s);
    if (e != hipSuccess) return e;
    dim3 cgrid(a.n_q, a.Hq);
    if (a.dh == 128)
      hipLaunchKernelGGL(attn_combine_kernel<128>, cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    else
      hipLaunchKernelGGL(attn_combine_kernel<64>, cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    return hipGetLastError();
  }
  dim3 grid((unsigned)total * a.Hq);
  return a.dh == 128 ? launch_attn<128, false>(p, grid, s) : launch_attn<64, false>(p, grid, s);
}
