// C-ABI entry points and the host-side scheduler (streams, per-layer load events) of libdsk.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <new>

#include "dsk_internal.h"

// Split-K partial sums of dsk_linear_static, the entry point for callers that cannot allocate: a fixed array in the
// code object, one copy per GPU, held until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels and copies get the per-device address that call returns.
static __device__ __align__(256) unsigned char scratch[DSK_STATIC_SCRATCH_BYTES];

thread_local hipEvent_t g_launch_ev_start = nullptr, g_launch_ev_stop = nullptr;
thread_local int g_last_hip_error = 0;  // shared with the cache store

namespace {

// A launcher that answers hipErrorNotSupported has refused the shape before enqueuing anything: that is the
// caller's DSK_ESHAPE, not a failed HIP call.
#define HIP_TRY(expr)                                                   \
  do {                                                                  \
    hipError_t e_ = (expr);                                             \
    if (e_ != hipSuccess) {                                             \
      g_last_hip_error = (int)e_;                                       \
      return e_ == hipErrorNotSupported ? DSK_ESHAPE : DSK_EHIP;        \
    }                                                                   \
  } while (0)

inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

int alloc_dev(void** p, int64_t bytes, int64_t* total) {
  if (bytes <= 0) bytes = 16;
  hipError_t e = hipMalloc(p, (size_t)bytes);
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    *p = nullptr;
    return e == hipErrorOutOfMemory ? DSK_ENOMEM : DSK_EHIP;
  }
  *total += bytes;
  return DSK_OK;
}

void free_model(dsk_model* m) {
  if (!m) return;
  if (m->layers) {
    for (int l = 0; l < m->cfg.n_layers; ++l) {
      LayerWeights& w = m->layers[l];
      (void)hipFree(w.g1); (void)hipFree(w.wqkv); (void)hipFree(w.wo);
      (void)hipFree(w.g2); (void)hipFree(w.wgu); (void)hipFree(w.wd); (void)hipFree(w.wr);
    }
    free(m->layers);
  }
  (void)hipFree(m->xn); (void)hipFree(m->qkv); (void)hipFree(m->attn); (void)hipFree(m->gu);
  (void)hipFree(m->act); (void)hipFree(m->h); (void)hipFree(m->e_stage); (void)hipFree(m->pace_t0); (void)hipFree(m->rope_cs); (void)hipFree(m->theta); (void)hipFree(m->vt); (void)hipFree(m->gemm_ws); (void)hipFree(m->attn_ws); (void)hipFree(m->ssq);
  if (m->ev_kv) {
    for (int l = 0; l < m->cfg.n_layers; ++l)
      if (m->ev_kv[l]) (void)hipEventDestroy(m->ev_kv[l]);
    free(m->ev_kv);
  }
  if (m->ev_entry) (void)hipEventDestroy(m->ev_entry);
  if (m->ev_e) (void)hipEventDestroy(m->ev_e);
  if (m->ev_stage_free) (void)hipEventDestroy(m->ev_stage_free);
  if (m->ev_all) (void)hipEventDestroy(m->ev_all);
  for (int i = 0; i < DSK_MAX_E_CHUNKS; ++i)
    if (m->ev_e_chunk[i]) (void)hipEventDestroy(m->ev_e_chunk[i]);
  (void)hipFree(m->chunk_cu);
  (void)hipFree(m->moe_experts); (void)hipFree(m->moe_gates); (void)hipFree(m->moe_slot); (void)hipFree(m->moe_src);
  (void)hipFree(m->moe_tab); (void)hipFree(m->moe_xg); (void)hipFree(m->moe_y);
  if (m->load_stream) (void)hipStreamDestroy(m->load_stream);
  free(m->pending);
  free(m);
}

int check_batch(const dsk_batch_t* b, bool need_positions) {
  if (!b || !b->cu_seqlens_host || !b->cu_seqlens_dev) return DSK_EINVAL;
  if (need_positions && !b->positions_dev) return DSK_EINVAL;
  if (b->n_seqs < 1 || b->n_tokens < 1) return DSK_EINVAL;
  if (b->cu_seqlens_host[0] != 0) return DSK_EINVAL;
  for (int i = 0; i < b->n_seqs; ++i)
    if (b->cu_seqlens_host[i + 1] <= b->cu_seqlens_host[i]) return DSK_EINVAL;
  if (b->cu_seqlens_host[b->n_seqs] != b->n_tokens) return DSK_EINVAL;
  return DSK_OK;
}

int check_kv(const dsk_model* m, const dsk_kv_t* kv, int64_t rows_needed, bool must_be_device) {
  if (!kv || !kv->base || !aligned16(kv->base)) return DSK_EINVAL;
  if (kv->mem != DSK_MEM_DEVICE && kv->mem != DSK_MEM_HOST_PINNED) return DSK_EINVAL;
  if (must_be_device && kv->mem != DSK_MEM_DEVICE) return DSK_EINVAL;
  const int64_t row_bytes = (int64_t)m->cfg.n_kv_heads * m->cfg.head_dim * m->elem;
  if (kv->n_rows < rows_needed || kv->n_rows >= (int64_t)1 << 31) return DSK_EINVAL;
  if (kv->v_offset < kv->n_rows * row_bytes || (kv->v_offset & 15)) return DSK_EINVAL;
  if (kv->layer_stride < kv->v_offset + kv->n_rows * row_bytes || (kv->layer_stride & 15)) return DSK_EINVAL;
  return DSK_OK;
}

inline char* kv_k(const dsk_kv_t* kv, int l) { return (char*)kv->base + (int64_t)l * kv->layer_stride; }
inline char* kv_v(const dsk_kv_t* kv, int l) { return kv_k(kv, l) + kv->v_offset; }

int g_force_generic = 0;
int g_time_gemm = 0;
int g_e_chunk_rows = 0;  // test hook: 0 = chunk a host-resident E cache by the rule below, -1 = never, > 0 = this many rows

// Launch counters (atomic: models on different host threads share them) and the event pairs recorded under
// "time_gemm" (a benchmark hook; the timed lists are guarded by their mutex): one list for the prefill GEMM
// launches, one for the attention launches over the prefix (at least 1024 query rows)
struct TimedList {
  static constexpr int kMax = 8192;
  hipEvent_t* ev = nullptr;  // 2*kMax events, created on first use
  int n = 0;
  double flops = 0.0;
  // hands the event pair of the next launch to the launcher (which attaches them to the kernel's dispatch); false
  // when the list is full
  // creates the events (when the hook is switched on: creating thousands of events takes milliseconds, which must not
  // fall into a timed region)
  hipError_t prepare() {
    if (ev) return hipSuccess;
    hipEvent_t* fresh = (hipEvent_t*)calloc(2 * kMax, sizeof(hipEvent_t));
    if (!fresh) return hipErrorOutOfMemory;
    for (int i = 0; i < 2 * kMax; ++i) {
      hipError_t e = hipEventCreate(&fresh[i]);
      if (e != hipSuccess) {
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(fresh[j]);
        free(fresh);
        return e;
      }
    }
    ev = fresh;
    return hipSuccess;
  }
  hipError_t begin(hipStream_t, bool* on) {
    *on = false;
    if (n >= kMax) return hipSuccess;
    if (!ev) {
      hipError_t e = prepare();
      if (e != hipSuccess) return e;
    }
    *on = true;
    g_launch_ev_start = ev[2 * n];
    g_launch_ev_stop = ev[2 * n + 1];
    return hipSuccess;
  }
  // the launch failed before any kernel was enqueued: the pair goes back
  void abandon() { g_launch_ev_start = g_launch_ev_stop = nullptr; }
  hipError_t end(hipStream_t, double launch_flops) {
    if (g_launch_ev_start) {  // no launcher took the pair (a kernel other than the timed ones ran): not counted
      g_launch_ev_start = g_launch_ev_stop = nullptr;
      return hipSuccess;
    }
    flops += launch_flops;
    ++n;
    return hipSuccess;
  }
  int total_ms(double* ms_out) {
    double total = 0.0;
    for (int i = 0; i < n; ++i) {
      HIP_TRY(hipEventSynchronize(ev[2 * i + 1]));
      float ms = 0.f;
      HIP_TRY(hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]));
      total += ms;
    }
    *ms_out = total;
    return DSK_OK;
  }
};

struct Stats {
  std::atomic<int64_t> gemm_mfma{0}, gemm_generic{0}, attn_mfma{0}, attn_generic{0};
  std::atomic<int64_t> e_chunks{0};  // row chunks of host-resident E caches that the first recomputed layer followed
  std::mutex timed_mu;
  TimedList gemm, attn;
} g_stats;

hipError_t gemm_any(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                    const void* R, int64_t ldr, int M, int N, int K, int epi, void* ws, int64_t ws_bytes, hipStream_t s) {
  if (dtype == DSK_BF16 && !g_force_generic) {
    std::unique_lock<std::mutex> timed_lock(g_stats.timed_mu, std::defer_lock);
    bool timed = false;
    if (g_time_gemm && gemm_mfma_uses_prefill_tile(M, N)) {
      timed_lock.lock();
      hipError_t ee = g_stats.gemm.begin(s, &timed);
      if (ee != hipSuccess) return ee;
    }
    // a shape the tensor-core kernels refuse comes back as hipErrorNotSupported (the caller's DSK_ESHAPE): a bf16
    // problem never drops to the plain-ALU kernel behind the caller's back, that kernel is a hundred times slower
    hipError_t e = launch_gemm_mfma_bf16(A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, ws, ws_bytes, s);
    if (e == hipSuccess) {
      ++g_stats.gemm_mfma;
      if (timed) e = g_stats.gemm.end(s, 2.0 * M * N * K);
    } else if (timed) {
      g_stats.gemm.abandon();
    }
    return e;
  }
  ++g_stats.gemm_generic;
  return launch_gemm_generic(dtype, A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, s);
}

hipError_t gemm(const dsk_model* m, const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                const void* R, int64_t ldr, int M, int N, int K, int epi, hipStream_t s) {
  return gemm_any(m->cfg.dtype, A, lda, W, ldw, C, ldc, R, ldr, M, N, K, epi, m->gemm_ws, m->gemm_ws_bytes, s);
}

hipError_t attention_any(int dtype, const AttnArgs& a, hipStream_t s) {
  if (dtype == DSK_BF16 && !g_force_generic && a.vt) {  // no transposed V: the caller chose the plain kernel
    std::unique_lock<std::mutex> timed_lock(g_stats.timed_mu, std::defer_lock);
    bool timed = false;
    if (g_time_gemm && a.n_q >= 1024 && !a.p_cu) {  // the prefix pass: causal self-attention, no earlier rows
      timed_lock.lock();
      hipError_t ee = g_stats.attn.begin(s, &timed);
      if (ee != hipSuccess) return ee;
    }
    hipError_t e = launch_attn_mfma_bf16(a, s);
    if (e == hipSuccess) {
      ++g_stats.attn_mfma;
      if (timed) {
        // algorithmic flops: every query row against the keys it may see (causal), 4*Hq*dh per (query, key) pair
        double pairs = 0.0;
        for (int b = 0; b < a.n_seqs; ++b) {
          const double len = a.q_cu_host[b + 1] - a.q_cu_host[b];
          const double pre = a.p_cu_host ? a.p_cu_host[b + 1] - a.p_cu_host[b] : 0.0;
          pairs += len * (len + 1.0) / 2.0 + len * pre;
        }
        e = g_stats.attn.end(s, 4.0 * a.Hq * a.dh * pairs);
      }
    } else if (timed) {
      g_stats.attn.abandon();
    }
    return e;
  }
  ++g_stats.attn_generic;
  return launch_attn_generic(dtype, a, s);
}

hipError_t attention(const dsk_model* m, const AttnArgs& a, hipStream_t s) { return attention_any(m->cfg.dtype, a, s); }

// The MLP of a mixture-of-experts layer (Sec. 5.4; routing as in Mixtral) over the n normalised rows in m->xn:
// h_out = h_mid + sum over the token's top_k experts of gate * SwiGLU-MLP_e(xn).  On the tensor-core path with more
// than 64 rows the (token, expert) pairs are grouped by expert and the two projections run once over all experts;
// otherwise (few rows: every expert's weights are streamed anyway; fp32 models) every expert runs over all rows and
// the sum picks the chosen ones.
int run_moe_mlp(dsk_model* m, const LayerWeights& w, int n, const float* h_mid, void* h_out, int out_f32, hipStream_t s) {
  const dsk_config_t& c = m->cfg;
  const int d = c.hidden, F = c.ffn, E = c.n_experts, k = c.top_k;
  const int64_t wgu_stride = 2 * (int64_t)F * d, wd_stride = (int64_t)d * F;  // elements per expert
  HIP_TRY(launch_moe_route(c.dtype, m->xn, w.wr, m->moe_experts, m->moe_gates, n, d, E, k, s));
  const bool tensor_cores = c.dtype == DSK_BF16 && !g_force_generic;
  if (tensor_cores && n > 64) {
    if (m->gu_block != 32) return DSK_ESHAPE;
    int tile_rows = moe_tile_table_rows((int64_t)n * k, E);
    if (tile_rows > m->moe_tile_rows) tile_rows = m->moe_tile_rows;
    HIP_TRY(launch_moe_place(m->moe_experts, m->moe_slot, m->moe_src, m->moe_tab, n, k, E, 256, tile_rows, s));
    HIP_TRY(launch_moe_gather(c.dtype, m->xn, m->moe_src, m->moe_xg, n * k, n, d, s));
    // under "time_gemm" the two grouped launches are bracketed like the other prefill projections (n*k rows each)
    auto grouped = [&](const void* A, int64_t lda, const void* W, int64_t ldw, int64_t w_stride, void* C, int64_t ldc, int N,
                       int K, int epi) -> int {
      std::unique_lock<std::mutex> timed_lock(g_stats.timed_mu, std::defer_lock);
      bool timed = false;
      if (g_time_gemm && gemm_mfma_uses_prefill_tile(n * k, N)) {
        timed_lock.lock();
        HIP_TRY(g_stats.gemm.begin(s, &timed));
      }
      const hipError_t e = launch_gemm_mfma_grouped(A, lda, (int64_t)n * k, W, ldw, w_stride, C, ldc, N, K, epi, m->moe_tab,
                                                    tile_rows, s);
      if (e != hipSuccess && timed) g_stats.gemm.abandon();
      HIP_TRY(e);
      ++g_stats.gemm_mfma;
      if (timed) HIP_TRY(g_stats.gemm.end(s, 2.0 * n * k * N * K));
      return DSK_OK;
    };
    int rc = grouped(m->moe_xg, d, w.wgu, d, wgu_stride, m->act, F, 2 * F, d, EPI_SWIGLU);
    if (rc == DSK_OK) rc = grouped(m->act, F, w.wd, F, wd_stride, m->moe_y, d, d, F, EPI_C_F32);
    if (rc) return rc;
    HIP_TRY(launch_moe_combine(m->moe_y, h_mid, m->moe_gates, m->moe_experts, m->moe_slot, h_out, out_f32, n, d, k,
                               (int64_t)n * k, s));
    return DSK_OK;
  }
  if ((int64_t)E * n > m->moe_y_rows) return DSK_EINVAL;
  const bool fused_swiglu = tensor_cores && m->gu_block == 32 &&
                            gemm_mfma_swiglu_supported(n, 2 * F, d, m->gemm_ws ? m->gemm_ws_bytes : 0);
  for (int e = 0; e < E; ++e) {
    const char* wgu = (const char*)w.wgu + e * wgu_stride * m->elem;
    const char* wd = (const char*)w.wd + e * wd_stride * m->elem;
    if (fused_swiglu) {
      HIP_TRY(gemm(m, m->xn, d, wgu, d, m->act, F, nullptr, 0, n, 2 * F, d, EPI_SWIGLU, s));
    } else {
      HIP_TRY(gemm(m, m->xn, d, wgu, d, m->gu, 2 * (int64_t)F, nullptr, 0, n, 2 * F, d, EPI_STORE, s));
      HIP_TRY(launch_swiglu(c.dtype, m->gu, m->act, n, F, m->gu_block, s));
    }
    HIP_TRY(gemm(m, m->act, F, wd, F, m->moe_y + (int64_t)e * n * d, d, nullptr, 0, n, d, F, EPI_C_F32, s));
  }
  HIP_TRY(launch_moe_combine(m->moe_y, h_mid, m->moe_gates, m->moe_experts, nullptr, h_out, out_f32, n, d, k,
                             (int64_t)E * n, s));
  return DSK_OK;
}

// One decoder layer over n token rows.  h_in: residual stream entering the layer; h_out: where the
// state leaving the layer is written (may equal h_in).  K/V of the tokens go to rows own_row0.. of the
// cache layer (k_rows, v_rows); attention additionally sees the prefix rows delimited by p_cu.
// h_in is the model dtype unless h_in_f32; h_out likewise unless h_out_f32 (the workspace stream m->h is fp32).
// h_mid: fp32 rows that receive the state after the attention block (h_out may be the same rows); cs: rotary table
// of the n tokens.  vt_first_row: rows of the layer's V before it are already in the transposed copy m->vt.
int run_layer(dsk_model* m, int l, const void* h_in, int h_in_f32, void* h_out, int h_out_f32, char* k_layer,
              char* v_layer, int64_t own_row0,
              const int32_t* q_cu, const int32_t* q_cu_host, const int32_t* p_cu, const int32_t* p_cu_host,
              int64_t n_pre_rows, int n_seqs, int n, hipStream_t s, float* h_mid = nullptr, const float2* cs = nullptr,
              int64_t vt_first_row = 0, bool xn_prescaled = false, const void* g_next = nullptr,
              bool* next_prescaled = nullptr) {
  if (!h_mid) h_mid = m->h;
  if (!cs) cs = m->rope_cs;
  if (next_prescaled) *next_prescaled = false;
  const dsk_config_t& c = m->cfg;
  const LayerWeights& w = m->layers[l];
  const int d = c.hidden, F = c.ffn, nq = c.n_q_heads * c.head_dim;
  const int64_t row_bytes = (int64_t)c.n_kv_heads * c.head_dim * m->elem;
  char* k_own = k_layer + own_row0 * row_bytes;
  char* v_own = v_layer + own_row0 * row_bytes;
  const int all_f32 = c.dtype == DSK_F32;  // an fp32 model: every buffer is fp32 anyway
  // few token rows (the suffix pass) on the tensor-core path: RoPE + KV write, and below the post-attention
  // RMSNorm, are done by the split-K reduction of the projection in front of them
  const bool few_rows = c.dtype == DSK_BF16 && !g_force_generic && n <= 64 && m->gemm_ws;
  // ... and with a hidden width in whole 1024-column blocks each RMSNorm is split in two: the reduction in front of it
  // leaves h * g and the row's sums of squares, the reduction behind the next projection applies the row factor
  // (xn_prescaled: the layer before has done so for this layer's input norm).  Dense MLP only: the router of an
  // expert layer reads the normalised rows themselves.
  const bool split_norm = few_rows && c.n_experts == 0 && m->ssq && m->gu_block == 32 &&
                          gemm_small_m_prescale_supported(n, d, nq, nq, nq, m->gemm_ws_bytes) &&
                          gemm_small_m_prescale_supported(n, d, F, F, F, m->gemm_ws_bytes) &&
                          gemm_small_m_fused_supported(n, 2 * F, d, d, d, m->gemm_ws_bytes);
  if (xn_prescaled && !split_norm) return DSK_EINVAL;  // the caller decides both from the same conditions
  if (!xn_prescaled) HIP_TRY(launch_rmsnorm(c.dtype, h_in, h_in_f32 || all_f32, w.g1, m->xn, n, d, (float)c.rms_eps, s));
  if (few_rows && gemm_small_m_rope_supported(n, d, c.n_q_heads, c.n_kv_heads, c.head_dim, d, d, m->n_qkv, m->gemm_ws_bytes)) {
    HIP_TRY(launch_gemm_small_m_rope(m->xn, d, w.wqkv, d, m->qkv, m->n_qkv, cs, k_own, v_own, n, d, c.n_q_heads,
                                     c.n_kv_heads, c.head_dim, m->gemm_ws, m->gemm_ws_bytes,
                                     xn_prescaled ? m->ssq : nullptr, (float)c.rms_eps, s));
    ++g_stats.gemm_mfma;
  } else {
    if (xn_prescaled) return DSK_EINVAL;
    HIP_TRY(gemm(m, m->xn, d, w.wqkv, d, m->qkv, m->n_qkv, nullptr, 0, n, m->n_qkv, d, EPI_STORE, s));
    HIP_TRY(launch_rope_kv_write(c.dtype, m->qkv, cs, k_own, v_own, n, c.n_q_heads, c.n_kv_heads, c.head_dim, s));
  }
  AttnArgs a;
  a.q = m->qkv; a.ldq = m->n_qkv; a.k_rows = k_layer; a.v_rows = v_layer; a.out = m->attn;
  a.q_cu = q_cu; a.p_cu = p_cu; a.q_cu_host = q_cu_host; a.p_cu_host = p_cu_host; a.n_seqs = n_seqs;
  a.own_row0 = own_row0; a.n_q = n; a.ws = m->attn_ws; a.ws_bytes = m->attn_ws_bytes;
  a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads; a.dh = c.head_dim;
  a.vt = nullptr; a.ldvt = 0;
  if (m->vt && !g_force_generic) {
    HIP_TRY(launch_transpose_v(v_layer, m->vt, m->ldvt, c.n_kv_heads * c.head_dim, n_pre_rows, own_row0, n, vt_first_row, s));
    a.vt = m->vt; a.ldvt = m->ldvt;
  }
  HIP_TRY(attention(m, a, s));
  if (split_norm) {
    HIP_TRY(launch_gemm_small_m_prescale(m->attn, nq, w.wo, nq, h_mid, h_in, h_in_f32 ? 1 : 0, w.g2, m->xn, m->ssq, n, d, nq,
                                         m->gemm_ws, m->gemm_ws_bytes, s));
    HIP_TRY(launch_gemm_small_m_swiglu_scaled(m->xn, d, w.wgu, d, m->act, F, n, 2 * F, d, m->gemm_ws, m->gemm_ws_bytes, m->ssq,
                                              (float)c.rms_eps, s));
    g_stats.gemm_mfma += 2;
    if (g_next && h_out_f32) {
      // the down projection prepares the next layer's input norm the same way
      HIP_TRY(launch_gemm_small_m_prescale(m->act, F, w.wd, F, (float*)h_out, h_mid, 1, g_next, m->xn, m->ssq, n, d, F,
                                           m->gemm_ws, m->gemm_ws_bytes, s));
      ++g_stats.gemm_mfma;
      if (next_prescaled) *next_prescaled = true;
      return DSK_OK;
    }
    HIP_TRY(gemm(m, m->act, F, w.wd, F, h_out, d, h_mid, d, n, d, F, EPI_RESIDUAL | EPI_R_F32 | (h_out_f32 ? EPI_C_F32 : 0), s));
    return DSK_OK;
  }
  if (few_rows && gemm_small_m_rmsnorm_supported(n, d, nq, nq, nq, m->gemm_ws_bytes)) {
    HIP_TRY(launch_gemm_small_m_rmsnorm(m->attn, nq, w.wo, nq, h_mid, h_in, h_in_f32 ? 1 : 0, w.g2, m->xn, (float)c.rms_eps, n,
                                        d, nq, m->gemm_ws, m->gemm_ws_bytes, s));
    ++g_stats.gemm_mfma;
  } else {
    HIP_TRY(gemm(m, m->attn, nq, w.wo, nq, h_mid, d, h_in, d, n, d, nq,
                 EPI_RESIDUAL | EPI_C_F32 | ((h_in_f32 || all_f32) ? EPI_R_F32 : 0), s));
    HIP_TRY(launch_rmsnorm(c.dtype, h_mid, 1, w.g2, m->xn, n, d, (float)c.rms_eps, s));
  }
  if (c.n_experts > 0) return run_moe_mlp(m, w, n, h_mid, h_out, h_out_f32 || all_f32, s);
  if (c.dtype == DSK_BF16 && !g_force_generic && m->gu_block == 32 && gemm_mfma_swiglu_supported(n, 2 * F, d, m->gemm_ws ? m->gemm_ws_bytes : 0)) {
    HIP_TRY(gemm(m, m->xn, d, w.wgu, d, m->act, F, nullptr, 0, n, 2 * F, d, EPI_SWIGLU, s));  // SwiGLU in the epilogue
  } else {
    HIP_TRY(gemm(m, m->xn, d, w.wgu, d, m->gu, 2 * (int64_t)F, nullptr, 0, n, 2 * F, d, EPI_STORE, s));
    HIP_TRY(launch_swiglu(c.dtype, m->gu, m->act, n, F, m->gu_block, s));
  }
  HIP_TRY(gemm(m, m->act, F, w.wd, F, h_out, d, h_mid, d, n, d, F,
               EPI_RESIDUAL | EPI_R_F32 | ((h_out_f32 || all_f32) ? EPI_C_F32 : 0), s));
  return DSK_OK;
}

// A host-resident E cache arrives over the link in row chunks, and the first recomputed layer runs chunk by chunk
// behind it (each chunk attends to the rows before it through the cache rows already written), so that all but the
// first chunk's transfer hides under compute (Sec. 4.3, Fig. 13(c): recomputation starts when the E cache is there).
// Returns the number of chunks (0 or 1: not chunked) and their row boundaries in bounds[0..n].
// By itself the library chunks only where every row's result keeps its bits: one sequence, a bf16 model, chunks of
// 4096 rows (a multiple of every tile) that each still fill the chip, i.e. run the same GEMM tiling and the same
// unsplit attention as the whole prefix would.
int plan_e_chunks(const dsk_model* m, int T, int n_seqs, int* bounds) {
  const dsk_config_t& c = m->cfg;
  if (g_e_chunk_rows < 0 || n_seqs != 1 || c.dtype != DSK_BF16 || g_force_generic || !m->vt) return 0;
  int rows = g_e_chunk_rows;
  if (rows == 0) {
    rows = 4096;
    const int widths[4] = {m->n_qkv, c.hidden, 2 * c.ffn, c.hidden};
    for (int i = 0; i < 4; ++i)
      if (!gemm_mfma_uses_prefill_tile(rows, widths[i])) return 0;
    if ((int64_t)(rows / 128) * c.n_q_heads < 512) return 0;
  }
  if (rows % 256 || T < 2 * rows) return 0;
  int n = T / rows;
  if (n > DSK_MAX_E_CHUNKS) {
    rows = ((T + DSK_MAX_E_CHUNKS - 1) / DSK_MAX_E_CHUNKS + 255) / 256 * 256;
    n = T / rows;
  }
  for (int i = 0; i < n; ++i) bounds[i] = i * rows;
  bounds[n] = T;  // the last chunk takes the remainder
  return n;
}

struct TensorPlace { void* base; int64_t rows, cols; int map; int64_t row_off; };

int place_tensor(const dsk_model* m, int layer, int tensor, TensorPlace* p) {
  if (layer < 0 || layer >= m->cfg.n_layers) return DSK_EINVAL;
  const dsk_config_t& c = m->cfg;
  const LayerWeights& w = m->layers[layer];
  const int64_t d = c.hidden, nq = (int64_t)c.n_q_heads * c.head_dim, nkv = (int64_t)c.n_kv_heads * c.head_dim, F = c.ffn;
  if (c.n_experts > 0) {
    // a mixture-of-experts layer: router, and WG/WU/WD per expert under DSK_EXPERT(e, t)
    if (tensor == DSK_WG || tensor == DSK_WU || tensor == DSK_WD) return DSK_EINVAL;
    if (tensor == DSK_WR) { *p = {w.wr, c.n_experts, d, 0, 0}; return DSK_OK; }
    if (tensor >= 16) {
      const int e = (tensor - 16) / 16, t = (tensor - 16) % 16;
      if (e >= c.n_experts) return DSK_EINVAL;
      char* gu = (char*)w.wgu + (int64_t)e * 2 * F * d * m->elem;
      char* dn = (char*)w.wd + (int64_t)e * d * F * m->elem;
      switch (t) {
        case DSK_WG: *p = {gu, F, d, 1, 0}; return DSK_OK;
        case DSK_WU: *p = {gu, F, d, 2, 0}; return DSK_OK;
        case DSK_WD: *p = {dn, d, F, 0, 0}; return DSK_OK;
        default: return DSK_EINVAL;
      }
    }
  } else if (tensor == DSK_WR || tensor >= 16) {
    return DSK_EINVAL;
  }
  switch (tensor) {
    case DSK_G1: *p = {w.g1, 1, d, 0, 0}; break;
    case DSK_G2: *p = {w.g2, 1, d, 0, 0}; break;
    case DSK_WQ: *p = {w.wqkv, nq, d, 0, 0}; break;
    case DSK_WK: *p = {w.wqkv, nkv, d, 0, nq}; break;
    case DSK_WV: *p = {w.wqkv, nkv, d, 0, nq + nkv}; break;
    case DSK_WO: *p = {w.wo, d, nq, 0, 0}; break;
    case DSK_WG: *p = {w.wgu, F, d, 1, 0}; break;
    case DSK_WU: *p = {w.wgu, F, d, 2, 0}; break;
    case DSK_WD: *p = {w.wd, d, F, 0, 0}; break;
    default: return DSK_EINVAL;
  }
  return DSK_OK;
}

}  // namespace

extern "C" {

int dsk_model_create(const dsk_config_t* cfg, int64_t max_tokens, int64_t max_kv_rows, dsk_model_t** out) {
  if (!cfg || !out || max_tokens < 1 || max_kv_rows < max_tokens || max_kv_rows >= ((int64_t)1 << 31)) return DSK_EINVAL;
  if (cfg->dtype != DSK_F32 && cfg->dtype != DSK_BF16) return DSK_EDTYPE;
  if (cfg->n_layers < 1 || cfg->hidden < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 || cfg->head_dim < 2 ||
      cfg->ffn < 1)
    return DSK_ESHAPE;
  if (cfg->n_q_heads % cfg->n_kv_heads || (cfg->head_dim & 1) || cfg->head_dim > 256) return DSK_ESHAPE;
  // rows of every matrix must keep 16-byte alignment
  const int elem = cfg->dtype == DSK_F32 ? 4 : 2;
  const int per16 = 16 / elem;
  if (cfg->hidden % per16 || cfg->ffn % per16 || cfg->head_dim % per16) return DSK_ESHAPE;
  if (!(cfg->rope_base > 0.0) || !(cfg->rms_eps >= 0.0)) return DSK_EINVAL;
  if (cfg->n_experts < 0 || cfg->n_experts > DSK_MOE_MAX_EXPERTS) return DSK_ESHAPE;
  if (cfg->n_experts == 0 ? cfg->top_k != 0
                          : (cfg->top_k < 1 || cfg->top_k > cfg->n_experts || cfg->top_k > DSK_MOE_MAX_TOP_K || cfg->hidden % 8))
    return DSK_ESHAPE;
  const int E = cfg->n_experts, top_k = cfg->top_k;
  // A bf16 model runs on the tensor-core kernels or not at all (the plain-ALU kernels serve fp32 models and the
  // "force_generic" test hook): contraction lengths in whole 64-element k-tiles, head_dim 64 or 128, K/V rows in
  // whole 64-element blocks, and token rows addressable by the kernels' 32-bit byte offsets.
  if (cfg->dtype == DSK_BF16 && !g_force_generic) {
    const int64_t nq_ = (int64_t)cfg->n_q_heads * cfg->head_dim, kvw_ = (int64_t)cfg->n_kv_heads * cfg->head_dim;
    if (cfg->hidden % 64 || nq_ % 64 || cfg->ffn % 64 || kvw_ % 64 || (cfg->head_dim != 64 && cfg->head_dim != 128))
      return DSK_ESHAPE;
    const int64_t d_ = cfg->hidden, f_ = cfg->ffn, lim = (int64_t)1 << 32;
    int64_t widest = d_ > f_ ? d_ : f_;  // longest activation row the projections read
    if (nq_ > widest) widest = nq_;
    if (max_tokens * (E > 0 ? top_k : 1) * widest * 2 >= lim) return DSK_ESHAPE;  // expert rows: top_k per token
    if ((nq_ + 2 * kvw_) * d_ * 2 >= lim || d_ * nq_ * 2 >= lim || 2 * f_ * d_ * 2 >= lim) return DSK_ESHAPE;
  }

  dsk_model* m = (dsk_model*)calloc(1, sizeof(dsk_model));
  if (!m) return DSK_ENOMEM;
  m->cfg = *cfg;
  m->elem = elem;
  m->max_tokens = max_tokens;
  m->max_kv_rows = max_kv_rows;
  m->ldvt = (max_kv_rows + 63) / 64 * 64;
  m->n_qkv = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
  m->gu_block = 1;
  for (int g = 32; g >= 1; g >>= 1)
    if (cfg->ffn % g == 0) { m->gu_block = g; break; }
  const int L = cfg->n_layers;
  const int64_t d = cfg->hidden, nq = (int64_t)cfg->n_q_heads * cfg->head_dim, F = cfg->ffn;
  int rc = DSK_OK;
  m->layers = (LayerWeights*)calloc(L, sizeof(LayerWeights));
  m->ev_kv = (hipEvent_t*)calloc(L, sizeof(hipEvent_t));
  m->pending = (unsigned char*)calloc(L, 1);
  if (!m->layers || !m->ev_kv || !m->pending) rc = DSK_ENOMEM;
  for (int l = 0; l < L && rc == DSK_OK; ++l) {
    LayerWeights& w = m->layers[l];
    if ((rc = alloc_dev(&w.g1, d * elem, &m->weight_bytes))) break;
    if ((rc = alloc_dev(&w.g2, d * elem, &m->weight_bytes))) break;
    if ((rc = alloc_dev(&w.wqkv, (int64_t)m->n_qkv * d * elem, &m->weight_bytes))) break;
    if ((rc = alloc_dev(&w.wo, d * nq * elem, &m->weight_bytes))) break;
    const int64_t n_mlp = E > 0 ? E : 1;
    if ((rc = alloc_dev(&w.wgu, n_mlp * 2 * F * d * elem, &m->weight_bytes))) break;
    if ((rc = alloc_dev(&w.wd, n_mlp * d * F * elem, &m->weight_bytes))) break;
    if (E > 0 && (rc = alloc_dev(&w.wr, (int64_t)E * d * elem, &m->weight_bytes))) break;
  }
  const int64_t T = max_tokens;
  const int half = cfg->head_dim / 2;
  if (rc == DSK_OK) rc = alloc_dev(&m->xn, T * d * elem, &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev(&m->qkv, T * m->n_qkv * elem, &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev(&m->attn, T * nq * elem, &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev(&m->gu, T * 2 * F * elem, &m->workspace_bytes);
  // with experts on the tensor-core path the MLP works on top_k rows per token, grouped by expert
  const bool moe_grouped = E > 0 && cfg->dtype == DSK_BF16;
  if (rc == DSK_OK) rc = alloc_dev(&m->act, T * (moe_grouped ? top_k : 1) * F * elem, &m->workspace_bytes);
  if (rc == DSK_OK && E > 0) {
    m->moe_y_rows = (int64_t)E * T;  // every expert over all rows (few rows, fp32, "force_generic"); grouped: T * top_k
    m->moe_tile_rows = moe_tile_table_rows(T * top_k, E);
    rc = alloc_dev((void**)&m->moe_experts, T * top_k * 4, &m->workspace_bytes);
    if (rc == DSK_OK) rc = alloc_dev((void**)&m->moe_gates, T * top_k * 4, &m->workspace_bytes);
    if (rc == DSK_OK) rc = alloc_dev((void**)&m->moe_slot, T * top_k * 4, &m->workspace_bytes);
    if (rc == DSK_OK) rc = alloc_dev((void**)&m->moe_src, T * top_k * 4, &m->workspace_bytes);
    if (rc == DSK_OK) rc = alloc_dev(&m->moe_tab, ((int64_t)m->moe_tile_rows + 1) * 16, &m->workspace_bytes);
    if (rc == DSK_OK && moe_grouped) rc = alloc_dev(&m->moe_xg, T * top_k * d * elem, &m->workspace_bytes);
    if (rc == DSK_OK) rc = alloc_dev((void**)&m->moe_y, m->moe_y_rows * d * 4, &m->workspace_bytes);
  }
  if (rc == DSK_OK) rc = alloc_dev((void**)&m->h, T * d * 4, &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev(&m->e_stage, T * d * elem, &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev((void**)&m->pace_t0, 8, &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev((void**)&m->chunk_cu, DSK_MAX_E_CHUNKS * 4 * (int64_t)sizeof(int32_t), &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev((void**)&m->rope_cs, T * half * (int64_t)sizeof(float2), &m->workspace_bytes);
  if (rc == DSK_OK) rc = alloc_dev((void**)&m->theta, half * (int64_t)sizeof(double), &m->workspace_bytes);
  const int64_t kvw = (int64_t)cfg->n_kv_heads * cfg->head_dim;
  if (rc == DSK_OK && cfg->dtype == DSK_BF16 && kvw % 64 == 0 && (cfg->head_dim == 64 || cfg->head_dim == 128))
    rc = alloc_dev(&m->vt, kvw * m->ldvt * elem, &m->workspace_bytes);
  if (rc == DSK_OK && m->vt) {
    m->attn_ws_bytes = attn_mfma_workspace_bytes(cfg->n_q_heads, cfg->head_dim);
    rc = alloc_dev(&m->attn_ws, m->attn_ws_bytes, &m->workspace_bytes);
  }
  if (rc == DSK_OK && cfg->dtype == DSK_BF16) {
    int max_n = m->n_qkv > 2 * cfg->ffn ? m->n_qkv : 2 * cfg->ffn;
    if (cfg->hidden > max_n) max_n = cfg->hidden;
    m->gemm_ws_bytes = gemm_mfma_workspace_bytes(max_n);
    rc = alloc_dev(&m->gemm_ws, m->gemm_ws_bytes, &m->workspace_bytes);
    if (rc == DSK_OK) rc = alloc_dev((void**)&m->ssq, 64 * DSK_MAX_SSQ_PARTS * (int64_t)sizeof(float), &m->workspace_bytes);
  }
  if (rc == DSK_OK) {
    double* th = (double*)malloc(half * sizeof(double));
    if (!th) rc = DSK_ENOMEM;
    else {
      for (int i = 0; i < half; ++i) th[i] = pow(cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
      hipError_t e = hipMemcpy(m->theta, th, half * sizeof(double), hipMemcpyHostToDevice);
      free(th);
      if (e != hipSuccess) { g_last_hip_error = (int)e; rc = DSK_EHIP; }
    }
  }
  auto hip_ok = [&](hipError_t e) {
    if (e != hipSuccess && rc == DSK_OK) { g_last_hip_error = (int)e; rc = DSK_EHIP; }
  };
  if (rc == DSK_OK) {
    hip_ok(hipStreamCreateWithFlags(&m->load_stream, hipStreamNonBlocking));
    hip_ok(hipEventCreateWithFlags(&m->ev_entry, hipEventDisableTiming));
    hip_ok(hipEventCreateWithFlags(&m->ev_e, hipEventDisableTiming));
    hip_ok(hipEventCreateWithFlags(&m->ev_stage_free, hipEventDisableTiming));
    hip_ok(hipEventCreateWithFlags(&m->ev_all, hipEventDisableTiming));
    for (int l = 0; l < L; ++l) hip_ok(hipEventCreateWithFlags(&m->ev_kv[l], hipEventDisableTiming));
    for (int i = 0; i < DSK_MAX_E_CHUNKS; ++i) hip_ok(hipEventCreateWithFlags(&m->ev_e_chunk[i], hipEventDisableTiming));
  }
  if (rc != DSK_OK) {
    free_model(m);
    return rc;
  }
  *out = m;
  return DSK_OK;
}

int dsk_model_destroy(dsk_model_t* model) {
  if (!model) return DSK_EINVAL;
  (void)hipStreamSynchronize(model->load_stream);
  (void)hipDeviceSynchronize();
  free_model(model);
  return DSK_OK;
}

int dsk_model_set_tensor(dsk_model_t* model, int layer, int tensor, const void* src, int src_mem, void* stream) {
  if (!model || !src) return DSK_EINVAL;
  if (src_mem != DSK_MEM_DEVICE && src_mem != DSK_MEM_HOST_PINNED) return DSK_EINVAL;
  TensorPlace p;
  int rc = place_tensor(model, layer, tensor, &p);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  const int64_t bytes = p.rows * p.cols * model->elem;
  if (src_mem == DSK_MEM_DEVICE) {
    HIP_TRY(launch_pack_rows(model->cfg.dtype, p.base, src, p.rows, p.cols, p.map, model->gu_block, p.row_off, 1, s));
    return DSK_OK;
  }
  // host source: staged through a temporary device buffer; this path waits for the copy to finish
  void* staging = nullptr;
  HIP_TRY(hipMalloc(&staging, (size_t)bytes));
  hipError_t e = hipMemcpy(staging, src, (size_t)bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess)
    e = launch_pack_rows(model->cfg.dtype, p.base, staging, p.rows, p.cols, p.map, model->gu_block, p.row_off, 1, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(staging);
  HIP_TRY(e);
  return DSK_OK;
}

int dsk_model_get_tensor(const dsk_model_t* model, int layer, int tensor, void* dst_device, void* stream) {
  if (!model || !dst_device) return DSK_EINVAL;
  TensorPlace p;
  int rc = place_tensor(model, layer, tensor, &p);
  if (rc) return rc;
  HIP_TRY(launch_pack_rows(model->cfg.dtype, p.base, dst_device, p.rows, p.cols, p.map, model->gu_block, p.row_off, 0,
                           (hipStream_t)stream));
  return DSK_OK;
}

int dsk_model_init_random(dsk_model_t* model, uint64_t seed, float std, void* stream) {
  if (!model || !(std >= 0.f)) return DSK_EINVAL;
  const int E = model->cfg.n_experts;
  auto fill = [&](int l, int tensor, uint64_t stream_id) -> int {
    TensorPlace p;
    int rc = place_tensor(model, l, tensor, &p);
    if (rc) return rc;
    const float offset = (tensor == DSK_G1 || tensor == DSK_G2) ? 1.0f : 0.0f;
    HIP_TRY(launch_fill_weight(model->cfg.dtype, p.base, p.rows, p.cols, p.map, model->gu_block, p.row_off, seed, stream_id,
                               std, offset, (hipStream_t)stream));
    return (int)DSK_OK;
  };
  for (int l = 0; l < model->cfg.n_layers; ++l) {
    for (int t = DSK_G1; t <= (E > 0 ? DSK_G2 : DSK_WD); ++t) {
      int rc = fill(l, t, (uint64_t)l * 16 + (uint64_t)t);
      if (rc) return rc;
    }
    if (E == 0) continue;
    int rc = fill(l, DSK_WR, (uint64_t)l * 16 + DSK_WR);
    if (rc) return rc;
    for (int e = 0; e < E; ++e)
      for (int j = 0; j < 3; ++j)
        if ((rc = fill(l, DSK_EXPERT(e, DSK_WG + j), ((uint64_t)1 << 20) + ((uint64_t)l * 64 + e) * 4 + j))) return rc;
  }
  return DSK_OK;
}

int dsk_fill_normal(void* dst_device, int64_t n, uint64_t seed, uint64_t stream_id, float std, float offset,
                    int64_t idx0, int dtype, void* stream) {
  if (!dst_device || n < 0 || idx0 < 0) return DSK_EINVAL;
  if (dtype != DSK_F32 && dtype != DSK_BF16) return DSK_EDTYPE;
  HIP_TRY(launch_fill_normal(dst_device, n, seed, stream_id, std, offset, idx0, dtype, (hipStream_t)stream));
  return DSK_OK;
}

// One transfer on the load stream.  With a throttle set it goes in chunks, each followed by a wait until the
// time the bytes sent so far would have needed on a link of that rate.
static int load_copy(dsk_model* m, void* dst, const void* src, int64_t bytes, hipMemcpyKind kind) {
  hipStream_t ls = m->load_stream;
  if (m->throttle_gbps <= 0.0) {
    HIP_TRY(hipMemcpyAsync(dst, src, (size_t)bytes, kind, ls));
    return DSK_OK;
  }
  const int64_t chunk = (int64_t)1 << 20;
  for (int64_t off = 0; off < bytes; off += chunk) {
    const int64_t n = bytes - off < chunk ? bytes - off : chunk;
    HIP_TRY(hipMemcpyAsync((char*)dst + off, (const char*)src + off, (size_t)n, kind, ls));
    m->paced_bytes += n;
    const double ticks = (double)m->paced_bytes / (m->throttle_gbps * 1e9) * 1e8;  // 100 MHz clock
    HIP_TRY(launch_pace_wait(m->pace_t0, (unsigned long long)ticks, ls));
  }
  return DSK_OK;
}

int dsk_partial_prefill_groups(dsk_model_t* model, const dsk_group_t* groups, int n_groups,
                               const dsk_kv_t* kv_reused, const dsk_kv_t* kv_out, const dsk_batch_t* batch,
                               uint32_t flags, void* stream) {
  if (!model || !kv_out || !batch || n_groups < 0 || (n_groups > 0 && !groups)) return DSK_EINVAL;
  dsk_model* m = model;
  const dsk_config_t& c = m->cfg;
  const int L = c.n_layers;
  int n_recomputed = 0;
  for (int g = 0, prev_hi = 0; g < n_groups; ++g) {
    const dsk_group_t& G = groups[g];
    if (!(prev_hi <= G.lo && G.lo <= G.hi && G.hi <= L)) return DSK_EINVAL;  // ascending, disjoint
    if (!G.hidden_in) return DSK_EINVAL;
    if (G.hidden_in_mem != DSK_MEM_DEVICE && G.hidden_in_mem != DSK_MEM_HOST_PINNED) return DSK_EINVAL;
    if (!aligned16(G.hidden_in) || !aligned16(G.hidden_out)) return DSK_EINVAL;
    prev_hi = G.hi;
    n_recomputed += G.hi - G.lo;
  }
  if (flags & ~DSK_DEFER_JOIN) return DSK_EINVAL;
  int rc = check_batch(batch, true);
  if (rc) return rc;
  const int T = batch->n_tokens;
  if (T > m->max_tokens || T > m->max_kv_rows) return DSK_EINVAL;
  if ((rc = check_kv(m, kv_out, T, true))) return rc;
  const bool need_reused = n_recomputed < L;
  if (need_reused || kv_reused)
    if ((rc = check_kv(m, kv_reused, T, false))) return rc;

  hipStream_t s = (hipStream_t)stream;
  hipStream_t ls = m->load_stream;
  const int64_t row_bytes = (int64_t)c.n_kv_heads * c.head_dim * m->elem;
  const int64_t hid_bytes = (int64_t)T * c.hidden * m->elem;
  const bool alias = kv_reused && kv_reused->base == kv_out->base && kv_reused->mem == DSK_MEM_DEVICE &&
                     kv_reused->layer_stride == kv_out->layer_stride && kv_reused->v_offset == kv_out->v_offset;
  const hipMemcpyKind kv_kind = (kv_reused && kv_reused->mem == DSK_MEM_HOST_PINNED) ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice;
  const int mode = m->load_mode;
  auto recomputed = [&](int l) {
    for (int g = 0; g < n_groups; ++g)
      if (l >= groups[g].lo && l < groups[g].hi) return true;
    return false;
  };

  // Loads that an earlier call with DSK_DEFER_JOIN left outstanding, and that no suffix pass or dsk_join_loads
  // has waited for, are joined here: the per-layer events and flags are about to be reused for this call.
  if (m->any_pending) HIP_TRY(hipStreamWaitEvent(s, m->ev_all, 0));
  // loads start after everything the caller already enqueued on `stream`
  HIP_TRY(hipEventRecord(m->ev_entry, s));
  HIP_TRY(hipStreamWaitEvent(ls, m->ev_entry, 0));
  if (m->throttle_gbps > 0.0) {
    m->paced_bytes = 0;
    HIP_TRY(launch_pace_start(m->pace_t0, ls));
  }

  // The first group's E cache goes first (Fig. 13(c)): recomputation can start as soon as it has arrived.
  // A host-resident E cache passes through the model's one staging buffer.
  auto stage_e = [&](const dsk_group_t& G) -> int {
    int r = load_copy(m, m->e_stage, G.hidden_in, hid_bytes, hipMemcpyHostToDevice);
    if (r) return r;
    HIP_TRY(hipEventRecord(m->ev_e, ls));
    return DSK_OK;
  };
  int e_bounds[DSK_MAX_E_CHUNKS + 1];
  int n_e_chunks = 0;
  if (n_groups > 0 && groups[0].hidden_in_mem == DSK_MEM_HOST_PINNED) {
    if (groups[0].hi > groups[0].lo && mode == DSK_LOAD_PIPELINED) n_e_chunks = plan_e_chunks(m, T, batch->n_seqs, e_bounds);
    if (n_e_chunks > 1) {
      const int64_t row_b = (int64_t)c.hidden * m->elem;
      for (int ch = 0; ch < n_e_chunks; ++ch) {
        const int64_t off = e_bounds[ch] * row_b;
        if ((rc = load_copy(m, (char*)m->e_stage + off, (const char*)groups[0].hidden_in + off,
                            (e_bounds[ch + 1] - e_bounds[ch]) * row_b, hipMemcpyHostToDevice)))
          return rc;
        HIP_TRY(hipEventRecord(m->ev_e_chunk[ch], ls));
      }
      HIP_TRY(hipEventRecord(m->ev_e, ls));
    } else if ((rc = stage_e(groups[0]))) return rc;
  }

  // reused layers, ascending (the order the suffix prefill consumes them), one event per layer
  memset(m->pending, 0, L);
  m->any_pending = 0;
  for (int l = 0; l < L; ++l) {
    if (recomputed(l) && mode != DSK_LOAD_ALL_FIRST) continue;
    if (!kv_reused || alias) continue;
    const int64_t bytes = (int64_t)T * row_bytes;
    const bool one_piece = kv_reused->v_offset == bytes && kv_out->v_offset == bytes;
    if (one_piece) {
      if ((rc = load_copy(m, kv_k(kv_out, l), kv_k(kv_reused, l), 2 * bytes, kv_kind))) return rc;
    } else {
      if ((rc = load_copy(m, kv_k(kv_out, l), kv_k(kv_reused, l), bytes, kv_kind))) return rc;
      if ((rc = load_copy(m, kv_v(kv_out, l), kv_v(kv_reused, l), bytes, kv_kind))) return rc;
    }
    HIP_TRY(hipEventRecord(m->ev_kv[l], ls));
    m->pending[l] = 1;
    m->any_pending = 1;
  }
  HIP_TRY(hipEventRecord(m->ev_all, ls));
  if (mode != DSK_LOAD_PIPELINED) HIP_TRY(hipStreamWaitEvent(s, m->ev_all, 0));  // strategies (a), (b): load, then compute

  // recompute the groups on the compute stream, each from its own E cache
  bool table_done = false;
  for (int g = 0; g < n_groups; ++g) {
    const dsk_group_t& G = groups[g];
    const void* h_cur = G.hidden_in;
    const bool chunked = g == 0 && n_e_chunks > 1;
    if (G.hidden_in_mem == DSK_MEM_HOST_PINNED) {
      // this group's copy into the staging buffer (recorded above / below); a chunked one is waited for chunk by chunk
      if (!chunked) HIP_TRY(hipStreamWaitEvent(s, m->ev_e, 0));
      h_cur = m->e_stage;
    }
    // the next host-resident E cache may enter the staging buffer once this group's first layer has read
    // it; its copy queues behind the layer loads, which the suffix prefill needs first
    const bool next_host = g + 1 < n_groups && groups[g + 1].hidden_in_mem == DSK_MEM_HOST_PINNED;
    auto hand_over_stage = [&]() -> int {
      HIP_TRY(hipEventRecord(m->ev_stage_free, s));
      HIP_TRY(hipStreamWaitEvent(ls, m->ev_stage_free, 0));
      return stage_e(groups[g + 1]);
    };
    if (G.hi > G.lo) {
      if (!table_done) {
        HIP_TRY(launch_rope_table(batch->positions_dev, m->theta, m->rope_cs, T, c.head_dim / 2, s));
        table_done = true;
      }
      for (int l = G.lo; l < G.hi; ++l) {
        const bool last = l == G.hi - 1 && G.hidden_out;
        void* h_next = last ? G.hidden_out : (void*)m->h;
        if (chunked && l == G.lo) {
          // the first layer, chunk by chunk behind the arriving E cache: rows before the chunk are a fully visible
          // prefix range of the cache layer, the chunk's own rows the causal range
          const int half = c.head_dim / 2;
          for (int ch = 0; ch < n_e_chunks; ++ch) {
            const int r0 = e_bounds[ch], n = e_bounds[ch + 1] - r0;
            const int32_t p_host[2] = {0, r0}, q_host[2] = {0, n};
            int32_t* cu = m->chunk_cu + 4 * ch;
            HIP_TRY(launch_set_int4(cu, 0, r0, 0, n, s));
            HIP_TRY(hipStreamWaitEvent(s, m->ev_e_chunk[ch], 0));
            const char* h_in = (const char*)m->e_stage + (int64_t)r0 * c.hidden * m->elem;
            float* h_mid = m->h + (int64_t)r0 * c.hidden;
            void* h_out = last ? (void*)((char*)G.hidden_out + (int64_t)r0 * c.hidden * m->elem) : (void*)h_mid;
            rc = run_layer(m, l, h_in, 0, h_out, !last, kv_k(kv_out, l), kv_v(kv_out, l), r0, cu + 2, q_host, cu, p_host, r0, 1,
                           n, s, h_mid, m->rope_cs + (int64_t)r0 * half, r0);
            if (rc) return rc;
            ++g_stats.e_chunks;
          }
          h_cur = h_next;
          if (next_host && (rc = hand_over_stage())) return rc;
          continue;
        }
        rc = run_layer(m, l, h_cur, l > G.lo, h_next, !last, kv_k(kv_out, l), kv_v(kv_out, l), 0, batch->cu_seqlens_dev,
                       batch->cu_seqlens_host, nullptr, nullptr, 0, batch->n_seqs, T, s);
        if (rc) return rc;
        h_cur = h_next;
        if (l == G.lo && next_host && (rc = hand_over_stage())) return rc;
      }
    } else {
      if (G.hidden_out && G.hidden_out != h_cur)
        HIP_TRY(hipMemcpyAsync(G.hidden_out, h_cur, (size_t)hid_bytes, hipMemcpyDeviceToDevice, s));
      if (next_host && (rc = hand_over_stage())) return rc;
    }
  }

  if (!(flags & DSK_DEFER_JOIN) || mode != DSK_LOAD_PIPELINED) {
    HIP_TRY(hipStreamWaitEvent(s, m->ev_all, 0));
    memset(m->pending, 0, L);
    m->any_pending = 0;
  }
  return DSK_OK;
}

int dsk_partial_prefill(dsk_model_t* model, const void* hidden_in, int hidden_in_mem, int lo, int hi,
                        const dsk_kv_t* kv_reused, const dsk_kv_t* kv_out, const dsk_batch_t* batch,
                        void* hidden_out, uint32_t flags, void* stream) {
  if (!hidden_in) return DSK_EINVAL;
  dsk_group_t g;
  g.lo = lo; g.hi = hi; g.hidden_in = hidden_in; g.hidden_in_mem = hidden_in_mem; g.hidden_out = hidden_out;
  return dsk_partial_prefill_groups(model, &g, 1, kv_reused, kv_out, batch, flags, stream);
}

int dsk_suffix_prefill(dsk_model_t* model, const void* suffix_hidden_in, const dsk_kv_t* kv,
                       const dsk_batch_t* prefix, const dsk_batch_t* suffix, int64_t suffix_row0,
                       void* hidden_out, void* stream) {
  if (!model || !suffix_hidden_in || !kv || !prefix || !suffix || !hidden_out) return DSK_EINVAL;
  dsk_model* m = model;
  const dsk_config_t& c = m->cfg;
  if (!aligned16(suffix_hidden_in) || !aligned16(hidden_out)) return DSK_EINVAL;
  int rc = check_batch(prefix, false);
  if (rc) return rc;
  if ((rc = check_batch(suffix, true))) return rc;
  if (prefix->n_seqs != suffix->n_seqs) return DSK_EINVAL;
  const int S = suffix->n_tokens;
  if (S > m->max_tokens) return DSK_EINVAL;
  if (suffix_row0 < prefix->n_tokens || suffix_row0 + S > m->max_kv_rows) return DSK_EINVAL;
  if ((rc = check_kv(m, kv, suffix_row0 + S, true))) return rc;

  hipStream_t s = (hipStream_t)stream;
  HIP_TRY(launch_rope_table(suffix->positions_dev, m->theta, m->rope_cs, S, c.head_dim / 2, s));
  const void* h_cur = suffix_hidden_in;
  bool prescaled = false;  // whether the layer before has prepared this layer's input norm (few rows, see run_layer)
  for (int l = 0; l < c.n_layers; ++l) {
    if (m->pending[l]) {
      HIP_TRY(hipStreamWaitEvent(s, m->ev_kv[l], 0));
      m->pending[l] = 0;
    }
    const bool last = l == c.n_layers - 1;
    void* h_next = last ? hidden_out : (void*)m->h;
    bool next_prescaled = false;
    rc = run_layer(m, l, h_cur, l > 0, h_next, !last, kv_k(kv, l), kv_v(kv, l), suffix_row0, suffix->cu_seqlens_dev,
                   suffix->cu_seqlens_host, prefix->cu_seqlens_dev, prefix->cu_seqlens_host, prefix->n_tokens,
                   suffix->n_seqs, S, s, nullptr, nullptr, 0, prescaled, last ? nullptr : m->layers[l + 1].g1, &next_prescaled);
    if (rc) return rc;
    prescaled = next_prescaled;
    h_cur = h_next;
  }
  m->any_pending = 0;
  return DSK_OK;
}

int dsk_join_loads(dsk_model_t* model, void* stream) {
  if (!model) return DSK_EINVAL;
  if (model->any_pending) {
    HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, model->ev_all, 0));
    memset(model->pending, 0, model->cfg.n_layers);
    model->any_pending = 0;
  }
  return DSK_OK;
}

int dsk_set_load_throttle(dsk_model_t* model, double gb_per_s) {
  if (!model || !(gb_per_s >= 0.0)) return DSK_EINVAL;
  model->throttle_gbps = gb_per_s;
  return DSK_OK;
}

int dsk_set_load_mode(dsk_model_t* model, int load_mode) {
  if (!model || load_mode < DSK_LOAD_PIPELINED || load_mode > DSK_LOAD_ALL_FIRST) return DSK_EINVAL;
  model->load_mode = load_mode;
  return DSK_OK;
}

int dsk_linear(int dtype, const void* x, const void* w, void* y, const void* r, int M, int N, int K, void* stream) {
  if (!x || !w || !y || M < 1 || N < 1 || K < 1) return DSK_EINVAL;
  if (dtype != DSK_F32 && dtype != DSK_BF16) return DSK_EDTYPE;
  if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(r)) return DSK_EINVAL;
  const int epi = r ? EPI_RESIDUAL : EPI_STORE;
  // split-K partials of the small-M path: one buffer per process, allocated at the first small-M call and kept
  // (calls that overlap on different streams would share it: this entry point is for tests and micro-benchmarks)
  static void* ws = nullptr;
  static int64_t ws_bytes = 0;
  static std::mutex ws_mu;
  std::lock_guard<std::mutex> ws_lock(ws_mu);  // host threads take turns; the buffer itself is still one per process
  const bool may_split = M <= 4096;  // the K-split paths are for few and for a few hundred token rows
  if (dtype == DSK_BF16 && may_split && gemm_mfma_workspace_bytes(N) > ws_bytes) {
    if (ws) HIP_TRY(hipFree(ws));
    ws = nullptr; ws_bytes = 0;
    HIP_TRY(hipMalloc(&ws, (size_t)gemm_mfma_workspace_bytes(N)));
    ws_bytes = gemm_mfma_workspace_bytes(N);
  }
  HIP_TRY(gemm_any(dtype, x, K, w, K, y, N, r, N, M, N, K, epi, may_split ? ws : nullptr, may_split ? ws_bytes : 0,
                   (hipStream_t)stream));
  return DSK_OK;
}

int dsk_linear_static(int dtype, const void* x, const void* w, void* y, const void* r, int M, int N, int K, void* stream) {
  if (!x || !w || !y || M < 1 || N < 1 || K < 1) return DSK_EINVAL;
  if (dtype != DSK_F32 && dtype != DSK_BF16) return DSK_EDTYPE;
  if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(r)) return DSK_EINVAL;
  if (M > DSK_STATIC_MAX_M || N > DSK_STATIC_MAX_N) return DSK_ELIMIT;
  // the device's own copy of the array: looked up once per device, with that device current
  constexpr int kMaxDevices = 64;
  static void* dev_ptr[kMaxDevices] = {};
  static std::mutex mu;
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DSK_ELIMIT;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!dev_ptr[dev]) HIP_TRY(hipGetSymbolAddress(&dev_ptr[dev], HIP_SYMBOL(scratch)));
    ptr = dev_ptr[dev];
  }
  const int epi = r ? EPI_RESIDUAL : EPI_STORE;
  hipStream_t s = (hipStream_t)stream;
  // no launch timing here (its event pool is allocated on first use); the kernels are those of dsk_linear
  if (dtype == DSK_BF16 && !g_force_generic) {
    HIP_TRY(launch_gemm_mfma_bf16(x, K, w, K, y, N, r, N, M, N, K, epi, ptr, DSK_STATIC_SCRATCH_BYTES, s));
    ++g_stats.gemm_mfma;
  } else {
    HIP_TRY(launch_gemm_generic(dtype, x, K, w, K, y, N, r, N, M, N, K, epi, s));
    ++g_stats.gemm_generic;
  }
  return DSK_OK;
}

int dsk_attention(int dtype, const void* q, const void* k_rows, const void* v_rows, void* out,
                  const dsk_batch_t* queries, const dsk_batch_t* prefix, int64_t own_row0, int n_q_heads,
                  int n_kv_heads, int head_dim, void* scratch, int64_t scratch_bytes, void* stream) {
  if (!q || !k_rows || !v_rows || !out || own_row0 < 0 || !aligned16(scratch)) return DSK_EINVAL;
  if (dtype != DSK_F32 && dtype != DSK_BF16) return DSK_EDTYPE;
  if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || head_dim < 2 || (head_dim & 1) || head_dim > 256)
    return DSK_ESHAPE;
  if (!aligned16(q) || !aligned16(k_rows) || !aligned16(v_rows) || !aligned16(out)) return DSK_EINVAL;
  int rc = check_batch(queries, false);
  if (rc) return rc;
  if (prefix) {
    if ((rc = check_batch(prefix, false))) return rc;
    if (prefix->n_seqs != queries->n_seqs) return DSK_EINVAL;
    if (prefix->n_tokens > own_row0) return DSK_EINVAL;  // the two row ranges must not overlap
  }
  AttnArgs a;
  a.q = q; a.ldq = (int64_t)n_q_heads * head_dim; a.k_rows = k_rows; a.v_rows = v_rows; a.out = out;
  a.q_cu = queries->cu_seqlens_dev; a.q_cu_host = queries->cu_seqlens_host;
  a.p_cu = prefix ? prefix->cu_seqlens_dev : nullptr;
  a.p_cu_host = prefix ? prefix->cu_seqlens_host : nullptr;
  a.ws = nullptr; a.ws_bytes = 0;
  a.n_seqs = queries->n_seqs; a.own_row0 = own_row0; a.n_q = queries->n_tokens;
  a.Hq = n_q_heads; a.Hkv = n_kv_heads; a.dh = head_dim;
  a.vt = nullptr; a.ldvt = 0;
  const int64_t kvw = (int64_t)n_kv_heads * head_dim;
  const int64_t rows64 = (own_row0 + queries->n_tokens + 63) / 64 * 64;
  if (dtype == DSK_BF16 && !g_force_generic && scratch) {
    // the caller asked for the tensor-core kernel: a shape it does not handle is an error, not a slower kernel
    if (kvw % 64 || (head_dim != 64 && head_dim != 128) || scratch_bytes < kvw * rows64 * 2) return DSK_ESHAPE;
    HIP_TRY(launch_transpose_v(v_rows, scratch, rows64, (int)kvw, prefix ? prefix->n_tokens : 0, own_row0,
                               queries->n_tokens, 0, (hipStream_t)stream));
    a.vt = scratch; a.ldvt = rows64;
  }
  HIP_TRY(attention_any(dtype, a, (hipStream_t)stream));
  return DSK_OK;
}

int dsk_moe_route(int dtype, const void* x, const void* wr, int n, int d, int n_experts, int top_k, int32_t* experts_out,
                  float* gates_out, void* stream) {
  if (!x || !wr || !experts_out || !gates_out || n < 0 || d < 1) return DSK_EINVAL;
  if (dtype != DSK_F32 && dtype != DSK_BF16) return DSK_EDTYPE;
  HIP_TRY(launch_moe_route(dtype, x, wr, experts_out, gates_out, n, d, n_experts, top_k, (hipStream_t)stream));
  return DSK_OK;
}

int dsk_set_option(const char* name, int value) {
  if (!name) return DSK_EINVAL;
  if (!strcmp(name, "gemm_tiling")) {
    if (value < 0 || value > 2) return DSK_EINVAL;
    gemm_mfma_set_variant(value);
  } else if (!strcmp(name, "e_chunk_rows")) {
    if (value < -1 || (value > 0 && value % 256)) return DSK_EINVAL;
    g_e_chunk_rows = value;
  } else if (!strcmp(name, "force_generic")) g_force_generic = value;
  else if (!strcmp(name, "time_gemm")) {
    if (value) {
      std::lock_guard<std::mutex> lock(g_stats.timed_mu);
      HIP_TRY(g_stats.gemm.prepare());
      HIP_TRY(g_stats.attn.prepare());
    }
    g_time_gemm = value;
  }
  else if (!strcmp(name, "reset_stats")) {
    g_stats.gemm_mfma = 0; g_stats.gemm_generic = 0; g_stats.attn_mfma = 0; g_stats.attn_generic = 0; g_stats.e_chunks = 0;
    std::lock_guard<std::mutex> timed_lock(g_stats.timed_mu);
    g_stats.gemm.n = g_stats.attn.n = 0;
    g_stats.gemm.flops = g_stats.attn.flops = 0.0;
    attn_mfma_counts(nullptr, nullptr, 1);
  } else return DSK_EINVAL;
  return DSK_OK;
}

int dsk_get_stat(const char* name, double* value) {
  if (!name || !value) return DSK_EINVAL;
  if (!strcmp(name, "gemm_mfma_launches")) *value = (double)g_stats.gemm_mfma.load();
  else if (!strcmp(name, "gemm_generic_launches")) *value = (double)g_stats.gemm_generic.load();
  else if (!strcmp(name, "attn_mfma_launches")) *value = (double)g_stats.attn_mfma.load();
  else if (!strcmp(name, "attn_generic_launches")) *value = (double)g_stats.attn_generic.load();
  else if (!strcmp(name, "e_cache_chunks")) *value = (double)g_stats.e_chunks.load();
  else if (!strcmp(name, "attn_key_split_launches") || !strcmp(name, "attn_packed_head_launches")) {
    int64_t split = 0, packed = 0;
    attn_mfma_counts(&split, &packed, 0);
    *value = (double)(name[5] == 'k' ? split : packed);
  }
  else if (!strncmp(name, "timed_gemm_", 11) || !strncmp(name, "timed_attn_", 11)) {
    std::lock_guard<std::mutex> timed_lock(g_stats.timed_mu);
    TimedList& t = name[6] == 'g' ? g_stats.gemm : g_stats.attn;
    const char* what = name + 11;
    if (!strcmp(what, "launches")) *value = (double)t.n;
    else if (!strcmp(what, "flops")) *value = t.flops;
    else if (!strcmp(what, "ms")) return t.total_ms(value);
    else return DSK_EINVAL;
  } else return DSK_EINVAL;
  return DSK_OK;
}

int64_t dsk_model_weight_bytes(const dsk_model_t* model) { return model ? model->weight_bytes : 0; }
int64_t dsk_model_workspace_bytes(const dsk_model_t* model) { return model ? model->workspace_bytes : 0; }

const char* dsk_strerror(int status) {
  switch (status) {
    case DSK_OK: return "ok";
    case DSK_EINVAL: return "invalid argument";
    case DSK_ESHAPE: return "unsupported model shape";
    case DSK_EDTYPE: return "unsupported dtype";
    case DSK_ENOMEM: return "out of memory";
    case DSK_EHIP: return "HIP call failed";
    case DSK_ENOENT: return "no such entry in the cache store";
    case DSK_ELIMIT: return "size beyond the fixed limit of this entry point";
    default: return "unknown status";
  }
}

int dsk_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
