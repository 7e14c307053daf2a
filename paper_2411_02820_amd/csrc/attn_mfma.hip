// bf16 MFMA flash attention for gfx950: causal grouped-query attention over packed sequences,
// keys taken from up to two row ranges of a cache layer (a fully visible prefix range and the
// queries' own causal range), online softmax in fp32.
//
// A workgroup of NW waves (4 are used) owns 32*NW query rows of one (sequence, q head); each wave 32 of them.
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
#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

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

// PACK (few queries per sequence, several q heads per kv head): the NW waves of a workgroup take the same 32
// query rows of NW different q heads of one kv group instead of 32*NW rows of one head, so that no wave idles on
// rows past the end of a short sequence and the K / Vt tiles of the group are loaded once for NW heads.
template <int DH, bool SPLIT, int NW, bool PACK = false>
__global__ void __launch_bounds__(64 * NW, 8 / NW) attn_bf16_kernel(AttnParams p) {
  constexpr int BQ = PACK ? 32 : 32 * NW;  // query rows per workgroup: 32 per wave
  constexpr int KCH = DH / 8;             // 16-byte slots per K row
  constexpr int K_RPI = 64 / KCH;         // K rows per wave load instruction
  constexpr int K_INST = BKV / K_RPI / NW; // per wave
  constexpr int V_INST = DH / 8 / NW;     // Vt rows are 64 keys = 8 slots -> 8 rows per instruction
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
  if (PACK) {
    const int quads = p.Hq / NW;  // groups of NW q heads, all within one kv group (the host checks (Hq/Hkv) % NW == 0)
    const int L = blockIdx.x;
    h = (L % quads) * NW + wave;
    rank = L / quads;
  } else {
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
  // Tiles are handed out from the end of the packed batch.  A strict heaviest-first order over all sequences (tiles
  // by their index inside the sequence, from host-built tables) was measured on a batch of eight ragged prefixes:
  // no change (1.895 ms per launch either way), so the plain order stays.
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
  const int qw0 = PACK ? q0 : q0 + 32 * wave;  // first query row of this wave
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
  // A load instruction takes a scalar base (tile origin) plus a 32-bit per-lane byte offset that is the same
  // for every tile; only a tile that reaches past the last readable cache row needs per-lane clamping.
  const int ldkv = p.Hkv * DH;
  const bf16_t* k_base = p.k + kvh * DH;
  const bf16_t* vt_base = p.vt + (int64_t)kvh * DH * p.ldvt;
  const uint32_t sK_lds = (uint32_t)(uintptr_t)sK, sV_lds = (uint32_t)(uintptr_t)sV;
  uint32_t k_off[K_INST], v_off[V_INST];
#pragma unroll
  for (int i = 0; i < K_INST; ++i) {
    const int rho = K_RPI * (wave * K_INST + i) + lane / KCH, s = lane % KCH;
    k_off[i] = (uint32_t)(perm_key(rho) * ldkv + (s ^ kswz(rho)) * 8) * 2u + 4096u - 1024u * i;
  }
#pragma unroll
  for (int i = 0; i < V_INST; ++i) {
    const int d = 8 * (wave * V_INST + i) + (lane >> 3), s = lane & 7;
    v_off[i] = (uint32_t)(d * (int)p.ldvt + (s ^ vswz(d)) * 8) * 2u + 4096u - 1024u * i;
  }
  // LDS destination of a direct load = M0 + instruction offset + 16 * lane, and the instruction offset also
  // adds to the global address.  The load instructions of a tile write LDS pieces 1024 bytes apart, so they
  // share one M0 value and differ in the instruction offset (the lane offsets k_off / v_off compensate it on
  // the global side, biased by 4096 so that they stay non-negative).  M0 is written once per group of
  // loads: a write to M0 has to wait until earlier direct loads have consumed the old value.
  auto set_m0 = [](uint32_t dst) { asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(dst) : "memory", "m0"); };
  auto lds_load = [](uint32_t voff, const void* base, int i) {
    switch (i) {
      case 0: asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base) : "memory"); break;
      case 1: asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" : : "v"(voff), "s"(base) : "memory"); break;
      case 2: asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" : : "v"(voff), "s"(base) : "memory"); break;
      default: asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" : : "v"(voff), "s"(base) : "memory"); break;
    }
  };
  auto tile_row0 = [&](int it) { return (it < nA ? ta0 + it : tb0 + (it - nA)) * BKV; };
  // i-th load instruction of a K tile / a Vt tile; the first one of a tile sets M0
  static_assert(K_INST <= 4 && V_INST <= 4 && K_RPI * DH * 2 == 1024, "instruction offsets assume 1024-byte pieces");
  auto issue_k1 = [&](int it, int i) {
    const int r0 = tile_row0(it), stage = (it - it_begin) & 1;
    const char* base = (const char*)(k_base + (int64_t)r0 * ldkv) - 4096;
    uint32_t off = k_off[i];
    if (r0 + BKV - 1 > p.k_row_max) {
      const int rho = K_RPI * (wave * K_INST + i) + lane / KCH, s = lane % KCH;
      off = (uint32_t)(min(perm_key(rho), p.k_row_max - r0) * ldkv + (s ^ kswz(rho)) * 8) * 2u + 4096u - 1024u * i;
    }
    if (i == 0) set_m0(sK_lds + (uint32_t)(stage * BKV * DH + K_RPI * wave * K_INST * DH) * 2u);
    lds_load(off, base, i);
  };
  auto issue_v1 = [&](int it, int i) {
    const int r0 = tile_row0(it), stage = (it - it_begin) & 1;
    if (i == 0) set_m0(sV_lds + (uint32_t)(stage * DH * BKV + 8 * wave * V_INST * BKV) * 2u);
    lds_load(v_off[i], (const char*)(vt_base + r0) - 4096, i);
  };
  auto issue_k = [&](int it) {
#pragma unroll
    for (int i = 0; i < K_INST; ++i) issue_k1(it, i);
  };
  auto issue_v = [&](int it) {
#pragma unroll
    for (int i = 0; i < V_INST; ++i) issue_v1(it, i);
  };
  // A wave has nothing to do in tiles that lie wholly beyond the causal limit of all its queries; those are
  // the last tiles of the range, so the wave's active tiles are [it_begin, act_end).
  int act_end = it_begin;
  if (wave_active) act_end = max(it_begin, min(it_end, nA + wave_lim_max / BKV - tb0 + 1));

  f32x16 o[NDT];
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  // running state: m = row maximum over the tiles scored so far, mc = m * c (0 while no key was visible),
  // alpha = factor that brings sums and outputs accumulated under the previous maximum to m
  float m = -INFINITY, mc = 0.f, alpha = 1.f, l = 0.f;

  constexpr int NQK = 2 * NKS;   // MFMAs of one score tile
  constexpr int NPV = 4 * NDT;   // MFMAs of one output update
  // MFMA j of a score tile works on key half j % 2 and head-dim step j / 2, MFMA j of an output update on
  // d-tile j % NDT and key chunk j / NDT: consecutive MFMAs go to different accumulators
  auto k_frag = [&](const bf16_t* kt_s, int j) {
    const int kt = j % 2, ks = j / 2, row = 32 * kt + lq;
    return *(const bf16x8*)(kt_s + row * DH + (((2 * ks + hh) ^ kswz(row)) * 8));
  };
  auto v_frag = [&](const bf16_t* vt_s, int j) {
    const int dt = j % NDT, kt = j / NDT / 2, t = (j / NDT) % 2, d = 32 * dt + lq;
    return *(const bf16x8*)(vt_s + d * BKV + (((4 * kt + 2 * t + hh) ^ vswz(d)) * 8));
  };
  // masks the scores of tile `it` where a key is outside this lane's visible range;
  // register r of half kt is key r0 + 32*kt + 16*(r/8) + 8*(lane/32) + r%8
  auto mask = [&](int it, f32x16* s) {
    const int r0 = tile_row0(it);
    const bool segA = it < nA;
    const int lo = segA ? pre_begin : own_begin;
    const int hi = segA ? pre_end - 1 : lim;
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
  };
  // the lane's query has its 64 scores of a tile in this lane and in lane^32
  // The exponentials are taken relative to a reference maximum m that follows the true running maximum
  // lazily: it moves only when the true maximum exceeds it by more than 2^8 in the exponent, so that
  // probabilities stay below 2^8 and the accumulated sums and outputs rarely need rescaling.  The
  // normalised result does not depend on the reference.
  auto new_max = [&](float mx) {
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_true = fmaxf(m, mx);
    const bool keep = (m_true - m) * p.c <= 8.0f;  // false for m = -inf (first visible key)
    const float m_new = keep ? m : m_true;
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    alpha = keep ? 1.0f : __builtin_amdgcn_exp2f((m - m_safe) * p.c);
    mc = m_safe * p.c;
    m = m_new;
  };

  // One key tile.  The matrix pipe and the vector ALU of a SIMD run side by side only when their
  // instructions alternate in the instruction stream, so the two matrix phases of a tile are interleaved,
  // MFMA by MFMA, with the vector work of the neighbouring tile:
  //   phase 1:  S(it+1) = K(it+1) Q^T      with   P(it) = exp2(S(it) c - m c), row sums, bf16 packing
  //   phase 2:  O^T += Vt(it) P(it)^T       with   row maximum of S(it+1)
  // s_i holds the masked scores of tile `it` (m, mc, alpha already include it), s_n receives tile it+1.
  // Fragments are read from LDS two MFMAs ahead.
  auto tile_step = [&](auto has_next_c, int it, f32x16* s_i, f32x16* s_n) {
    constexpr bool HN = decltype(has_next_c)::value;
    // outputs and sums accumulated so far move to the current maximum (rare after the first tiles of a row)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
    float psum = 0.f;
    u32x4 pf[2][2];
    {
      const bf16_t* kt_s = sK + ((it + 1 - it_begin) & 1) * BKV * DH;
      constexpr int EPM = 32 / NQK;
      bf16x8 kf[NQK];
      if (HN) {
        kf[0] = k_frag(kt_s, 0);
        kf[1] = k_frag(kt_s, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NQK; ++j) {
        if (HN) {
          if (j + 2 < NQK) kf[j + 2] = k_frag(kt_s, j + 2);
          const int kt = j % 2, ks = j / 2;
          if (ks == 0) {
            const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s_n[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[ks], z, 0, 0, 0);
          } else {
            s_n[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[ks], s_n[kt], 0, 0, 0);
          }
        }
#pragma unroll
        for (int e = 0; e < EPM; e += 2) {
          const int idx = j * EPM + e, kt = idx / 16, r = idx % 16;
          const float e0 = __builtin_amdgcn_exp2f(s_i[kt][r] * p.c - mc);
          const float e1 = __builtin_amdgcn_exp2f(s_i[kt][r + 1] * p.c - mc);
          psum += e0;
          psum += e1;
          bf16x2 pk = {(bf16_t)e0, (bf16_t)e1};
          uint32_t pku = __builtin_bit_cast(uint32_t, pk);
          // keeps this arithmetic between the neighbouring MFMAs (its results are first used in phase 2, and
          // the optimiser would otherwise move it there)
          asm volatile("" : "+v"(pku), "+v"(psum));
          pf[kt][r >> 3][(r & 7) >> 1] = pku;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    l = l * alpha + psum;
    if (HN) mask(it + 1, s_n);
    {
      const bf16_t* vt_s = sV + ((it - it_begin) & 1) * DH * BKV;
      constexpr int EPM = 32 / NPV;
      bf16x8 vf[NPV];
      vf[0] = v_frag(vt_s, 0);
      vf[1] = v_frag(vt_s, 1);
      float mx = -INFINITY;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NPV; ++j) {
        if (j + 2 < NPV) vf[j + 2] = v_frag(vt_s, j + 2);
        const int dt = j % NDT, kt = j / NDT / 2, t = (j / NDT) % 2;
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j], __builtin_bit_cast(bf16x8, pf[kt][t]), o[dt], 0, 0, 0);
        if (HN) {
#pragma unroll
          for (int e = 0; e < EPM; ++e) {
            const int idx = j * EPM + e;
            mx = fmaxf(mx, s_n[idx / 16][idx % 16]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (HN) new_max(mx);
    }
  };

  // Per tile and workgroup one barrier: after it K(it+1) and Vt(it) are complete in LDS and every wave is
  // done with K(it) and Vt(it-1), whose ring stages the loads issued next overwrite.
  // The loads the barrier released go out right behind it, in one burst (about 55 cycles each): spread between
  // the MFMAs of phase 1 they cost the wave more than that (measured with per-phase timestamps).
  auto tile_sync = [&](int it) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): as a builtin the compiler accounts for it
    __syncthreads();
    if (it + 2 < it_end) issue_k(it + 2);
    if (it + 1 < it_end) issue_v(it + 1);
  };

  f32x16 s_a[2], s_b[2];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) s_a[kt][r] = s_b[kt][r] = 0.f;
  if (it_begin < it_end) {
    // (A four-stage ring for the packed few-query launch, where a workgroup has a compute unit to itself and next to
    // no arithmetic per tile, was measured: 23.8 us per launch against 21.2 us with two stages; not kept.)
    // the first two K tiles and the first Vt tile are requested together, behind the Q fragments, and waited for
    // once: one round trip to memory at the start of a workgroup instead of two (the wait is for everything: the
    // compiler's own count for the Q fragments cannot see the direct-to-LDS loads, so a partial wait would be turned
    // into a full one in front of the first use of Q anyway)
    issue_k(it_begin);
    if (it_begin + 1 < it_end) issue_k(it_begin + 1);
    issue_v(it_begin);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): as a builtin the compiler accounts for it
    __syncthreads();
    if (it_begin < act_end) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
          s_a[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(sK, 2 * ks + kt), qf[ks], s_a[kt], 0, 0, 0);
      mask(it_begin, s_a);
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_a[kt][r]);
      new_max(mx);
      alpha = 1.f;  // nothing accumulated yet
    }
  }
  {
    // steady state in pairs so that the two score buffers swap roles without copies; then the wave's last
    // active tile (no successor to score); then the tiles this wave only helps to load
    int it = it_begin;
    for (; it + 2 < act_end; it += 2) {
      tile_sync(it);
      tile_step(std::true_type{}, it, s_a, s_b);
      tile_sync(it + 1);
      tile_step(std::true_type{}, it + 1, s_b, s_a);
    }
    if (it + 1 < act_end) {
      tile_sync(it);
      tile_step(std::true_type{}, it, s_a, s_b);
      tile_sync(it + 1);
      tile_step(std::false_type{}, it + 1, s_b, s_a);
      it += 2;
    } else if (it < act_end) {
      tile_sync(it);
      tile_step(std::false_type{}, it, s_a, s_b);
      it += 1;
    }
    for (; it < it_end; ++it) tile_sync(it);
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

// The same for at most MAXS splits, with every partial result requested before the first is used: the merge is a
// chain of small dependent steps, and what it takes is the round trips to memory, not the arithmetic.  Same sums in
// the same order as above.
template <int DH, int MAXS>
__global__ void __launch_bounds__(64) attn_combine_batched_kernel(const float* __restrict__ part_o,
                                                                  const float* __restrict__ part_ml, bf16_t* __restrict__ out,
                                                                  int Hq, int splits, float c) {
  const int64_t qh = (int64_t)blockIdx.x * Hq + blockIdx.y;
  const float* ml = part_ml + qh * splits * 2;
  float ms[MAXS], ls[MAXS], po[MAXS][DH / 64];
#pragma unroll
  for (int s = 0; s < MAXS; ++s) {
    const bool on = s < splits;
    ms[s] = on ? ml[2 * s] : -INFINITY;
    ls[s] = on ? ml[2 * s + 1] : 0.f;
#pragma unroll
    for (int a = 0; a < DH / 64; ++a) po[s][a] = on ? part_o[(qh * splits + s) * DH + threadIdx.x + 64 * a] : 0.f;
  }
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < MAXS; ++s) M = fmaxf(M, ms[s]);
  float den = 0.f, acc[DH / 64] = {};
#pragma unroll
  for (int s = 0; s < MAXS; ++s) {
    if (ms[s] == -INFINITY) continue;  // not a split, or one that saw no visible key
    const float w = __builtin_amdgcn_exp2f((ms[s] - M) * c);
    den += ls[s] * w;
#pragma unroll
    for (int a = 0; a < DH / 64; ++a) acc[a] += po[s][a] * w;
  }
  const float inv = 1.0f / den;
#pragma unroll
  for (int a = 0; a < DH / 64; ++a) out[qh * DH + threadIdx.x + 64 * a] = (bf16_t)(acc[a] * inv);
}

// Vt[(kvh*dh + d)*ldvt + row] = V[row][kvh*dh + d] for the valid rows, 0 for the others, over whole
// 64-row tiles.  valid(row) = row < n_pre || own_row0 <= row < own_row0 + n_own.
__global__ void __launch_bounds__(256) transpose_v_kernel(const bf16_t* __restrict__ v_rows, bf16_t* __restrict__ vt,
                                                          int64_t ldvt, int width, int64_t n_pre, int64_t own_row0,
                                                          int64_t n_own, int64_t tile0) {
  __shared__ bf16_t tile[64][66];
  const int64_t r0 = ((int64_t)blockIdx.x + tile0) * 64;
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

}  // namespace

// how many launches took the key-split path, and how many of those with four q heads packed per workgroup
static int64_t g_split_launches = 0, g_packed_launches = 0;
void attn_mfma_counts(int64_t* split, int64_t* packed, int reset) {
  if (split) *split = g_split_launches;
  if (packed) *packed = g_packed_launches;
  if (reset) g_split_launches = g_packed_launches = 0;
}

// fp32 scratch for the split mode: n_q * splits <= kMaxSplitRows partial rows of (dh + 2) floats per q head
constexpr int64_t kMaxSplitRows = 4096;
int64_t attn_mfma_workspace_bytes(int Hq, int dh) { return kMaxSplitRows * Hq * (dh + 2) * 4; }

hipError_t launch_transpose_v(const void* v_rows, void* vt, int64_t ldvt, int width, int64_t n_pre, int64_t own_row0,
                              int64_t n_own, int64_t first_row, hipStream_t s) {
  const int64_t end = own_row0 + n_own, tile0 = first_row / 64;
  if (end <= tile0 * 64) return hipSuccess;
  dim3 grid((unsigned)((end + 63) / 64 - tile0), width / 64);
  hipLaunchKernelGGL(transpose_v_kernel, grid, dim3(256), 0, s, (const bf16_t*)v_rows, (bf16_t*)vt, ldvt, width, n_pre,
                     own_row0, n_own, tile0);
  return hipGetLastError();
}

template <int DH, bool SPLIT, int NW, bool PACK = false>
hipError_t launch_attn(const AttnParams& p, dim3 grid, hipStream_t s) {
  auto kern = attn_bf16_kernel<DH, SPLIT, NW, PACK>;
  constexpr int lds = (2 * BKV * DH + 2 * DH * BKV) * 2;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  DSK_LAUNCH_TIMED(kern, grid, dim3(64 * NW), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_attn_mfma_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_q <= 0) return hipSuccess;
  if ((a.dh != 128 && a.dh != 64) || !a.vt || (a.ldq & 7) || a.own_row0 + a.n_q >= ((int64_t)1 << 31))
    return hipErrorNotSupported;
  // per-lane tile offsets are 32-bit byte offsets
  if ((int64_t)a.dh * a.ldvt * 2 >= ((int64_t)1 << 32) || (int64_t)BKV * a.Hkv * a.dh * 2 >= ((int64_t)1 << 32))
    return hipErrorNotSupported;
  AttnParams p;
  p.q = (const bf16_t*)a.q; p.ldq = a.ldq; p.k = (const bf16_t*)a.k_rows; p.vt = (const bf16_t*)a.vt; p.ldvt = a.ldvt;
  p.out = (bf16_t*)a.out; p.q_cu = a.q_cu; p.p_cu = a.p_cu; p.n_seqs = a.n_seqs; p.own_row0 = (int)a.own_row0;
  p.Hq = a.Hq; p.Hkv = a.Hkv;
  // 4-wave workgroups (128 queries).  8-wave workgroups halve the tile loads a wave issues per key tile and are
  // faster when the kernel is timed alone (+14 % at 8k tokens) but slower inside the layer, behind the projections
  // (25.05 -> 25.26 ms for eight 8B layers at 8k tokens, 58.3 -> 59.5 ms at 16k), so only this shape is built.
  auto count_tiles = [&](int bq) {
    int64_t t = 0;
    for (int b = 0; b < a.n_seqs; ++b) t += (a.q_cu_host[b + 1] - a.q_cu_host[b] + bq - 1) / bq;
    return t;
  };
  constexpr int nw = 4;
  int64_t max_keys = 0;
  int max_len = 0;
  for (int b = 0; b < a.n_seqs; ++b) {
    const int len = a.q_cu_host[b + 1] - a.q_cu_host[b];
    int64_t keys = len + (a.p_cu_host ? a.p_cu_host[b + 1] - a.p_cu_host[b] : 0);
    if (keys > max_keys) max_keys = keys;
    if (len > max_len) max_len = len;
  }
  // sequences of at most 64 queries would leave half of a 128-row workgroup idle: there the four waves take four
  // q heads of a kv group and 32 rows each (the key-split path only; needs four heads per kv group)
  // (Eight waves per packed workgroup, two 32-row tiles of the four heads sharing the K / Vt tiles, with twice the
  // splits to keep 256 workgroups: 5.53 against 5.33 ms for the 8B suffix pass of 64 tokens; not kept.)
  bool pack = a.ws && a.dh == 128 && max_len <= 64 && (a.Hq / a.Hkv) % nw == 0;
  p.c = (float)(1.4426950408889634 / sqrt((double)a.dh));
  p.k_row_max = (int)(a.own_row0 + a.n_q - 1);
  const int key_tiles = (int)((max_keys + BKV - 1) / BKV) + 1;
  int total = 0, splits = 1;
  int64_t blocks = 0;
  for (;;) {
    total = (int)count_tiles(pack ? 32 : 32 * nw);
    blocks = pack ? (int64_t)total * (a.Hq / nw) : (int64_t)total * a.Hq;
    // split the key tiles when the grid alone cannot fill the chip
    splits = 1;
    if (a.ws && blocks < 512 && key_tiles >= 8) {
      // about two workgroups per CU; measured on 64 queries against 8k and 16k keys: 16 splits beat 8 and 32
      // (more splits pay more for partial outputs and the per-workgroup start-up than they gain in parallelism)
      splits = (int)(((pack ? 256 : 512) + blocks - 1) / blocks);
      if (splits > key_tiles / 4) splits = key_tiles / 4;
      while (splits > 1 && ((int64_t)a.n_q * splits > kMaxSplitRows ||
                            (int64_t)a.n_q * splits * a.Hq * (a.dh + 2) * 4 > a.ws_bytes))
        --splits;
    }
    if (pack && splits <= 1) { pack = false; continue; }  // the packed mapping exists for the key-split kernel only
    break;
  }
  p.total_tiles = total;
  p.splits = splits;
  p.part_o = nullptr;
  p.part_ml = nullptr;
  if (splits > 1) {
    p.part_o = (float*)a.ws;
    p.part_ml = p.part_o + (int64_t)a.n_q * a.Hq * splits * a.dh;
    dim3 grid((unsigned)blocks, 1, splits);
    ++g_split_launches;
    if (pack) ++g_packed_launches;
    hipError_t e = pack ? launch_attn<128, true, 4, true>(p, grid, s)
                        : a.dh == 128 ? launch_attn<128, true, 4>(p, grid, s) : launch_attn<64, true, 4>(p, grid, s);
    if (e != hipSuccess) return e;
    dim3 cgrid(a.n_q, a.Hq);
    if (a.dh == 128 && splits <= 16)
      hipLaunchKernelGGL((attn_combine_batched_kernel<128, 16>), cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    else if (a.dh == 128 && splits <= 32)
      hipLaunchKernelGGL((attn_combine_batched_kernel<128, 32>), cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    else if (a.dh == 128)
      hipLaunchKernelGGL(attn_combine_kernel<128>, cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    else if (splits <= 32)
      hipLaunchKernelGGL((attn_combine_batched_kernel<64, 32>), cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    else
      hipLaunchKernelGGL(attn_combine_kernel<64>, cgrid, dim3(64), 0, s, p.part_o, p.part_ml, p.out, a.Hq, splits, p.c);
    return hipGetLastError();
  }
  dim3 grid((unsigned)total * a.Hq);
  return a.dh == 128 ? launch_attn<128, false, 4>(p, grid, s) : launch_attn<64, false, 4>(p, grid, s);
}
