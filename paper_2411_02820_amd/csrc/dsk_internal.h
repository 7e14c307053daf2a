// Internal declarations shared by the HIP sources of libdsk (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "dsk.h"

typedef __bf16 bf16_t;

// ---- element conversion (fp32 math everywhere; storage is float or bf16) ----
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }  // RNE (v_cvt_pk_bf16_f32)

// ---- packed weight layout ----
// QKV rows are [Wq; Wk; Wv].  Gate and up rows are interleaved in blocks of gu_block rows:
// packed rows [2*gu_block*j, 2*gu_block*j+gu_block) hold gate rows [gu_block*j, ..+gu_block),
// the next gu_block packed rows hold the same up rows, so that a GEMM tile owns gate and up of
// the same FFN index.
struct LayerWeights {
  void* g1;
  void* wqkv;  // [(Hq+2Hkv)*dh, d]
  void* wo;    // [d, Hq*dh]
  void* g2;
  void* wgu;   // [2F, d] interleaved; a mixture-of-experts layer: [E][2F, d]
  void* wd;    // [d, F]; a mixture-of-experts layer: [E][d, F]
  void* wr;    // router [E, d] of a mixture-of-experts layer
};

constexpr int DSK_MAX_E_CHUNKS = 16;

struct dsk_model {
  dsk_config_t cfg;
  int elem;         // bytes per element
  int64_t max_tokens;
  int64_t max_kv_rows;
  int gu_block;
  int n_qkv;        // (Hq+2Hkv)*dh
  LayerWeights* layers;
  int64_t weight_bytes;
  // workspace
  void* xn;         // [maxT, d]      normalised activations
  void* qkv;        // [maxT, n_qkv]
  void* attn;       // [maxT, Hq*dh]
  void* gu;         // [maxT, 2F]
  void* act;        // [maxT, F]
  float* h;         // [maxT, d]      residual stream between the layers of one call, kept in fp32
  void* e_stage;    // [maxT, d]      landing buffer for an E cache that arrives from pinned host memory
  float2* rope_cs;  // [maxT, dh/2]   cos, sin
  double* theta;    // [dh/2]         rope_base^(-2i/dh)
  void* vt;         // [Hkv*dh, ldvt] transposed V of the layer in flight (bf16 MFMA attention)
  int64_t ldvt;     // max_kv_rows rounded up to 64
  float* ssq;       // [64, DSK_MAX_SSQ_PARTS] partial sums of squares of the few-row pass (RMSNorm split in two)
  void* gemm_ws;    // fp32 partial tiles of the K-split small-M GEMM
  int64_t gemm_ws_bytes;
  void* attn_ws;    // fp32 partial outputs of the key-split attention
  int64_t attn_ws_bytes;
  // mixture-of-experts layers (cfg.n_experts > 0)
  int32_t* moe_experts;  // [maxT, top_k] chosen experts
  float* moe_gates;      // [maxT, top_k] their gate weights
  int32_t* moe_slot;     // [maxT, top_k] row of the entry once the rows are grouped by expert
  int32_t* moe_src;      // [maxT*top_k]  token of every grouped row
  void* moe_tab;         // int4 [moe_tile_rows] row tiles of the grouped projections
  int moe_tile_rows;
  void* moe_xg;          // [maxT*top_k, d] normalised activations, grouped by expert
  float* moe_y;          // expert outputs, fp32: [maxT*top_k, d] grouped, or [E][n][d] when every expert runs over all rows
  int64_t moe_y_rows;
  int64_t workspace_bytes;
  // load pipeline
  hipStream_t load_stream;
  hipEvent_t ev_entry, ev_e, ev_all, ev_stage_free;
  hipEvent_t ev_e_chunk[DSK_MAX_E_CHUNKS];  // arrival of the row chunks of a host-resident E cache
  int32_t* chunk_cu;                        // device [DSK_MAX_E_CHUNKS][4]: {0, rows before the chunk, 0, rows of the chunk}
  hipEvent_t* ev_kv;        // [L]
  unsigned char* pending;   // [L] 1 if ev_kv[l] must be waited for by the suffix
  int any_pending;
  int load_mode;
  double throttle_gbps;        // > 0: loads are paced to this rate (emulates a slower link); 0 = off
  unsigned long long* pace_t0; // device: start time of the current call's loads (constant-rate clock ticks)
  int64_t paced_bytes;         // bytes handed to the load stream since pace_t0 was taken
};

// epilogues of the GEMM family
// bit 0: add R; bit 1: R is fp32 (else the model dtype); bit 2: C is fp32 (else the model dtype)
// bit 3 (bf16 MFMA kernel only): W is the interleaved gate/up matrix, C[M, N/2] = silu(gate) * up
enum { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_R_F32 = 2, EPI_C_F32 = 4, EPI_SWIGLU = 8 };

// ---- launchers (each validates nothing: the C-ABI layer has checked shapes) ----
// C[M,N] = A[M,K] * W[N,K]^T (+ R[M,N] when epi has EPI_RESIDUAL); row strides in elements.
hipError_t launch_gemm_generic(int dtype, const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                               const void* R, int64_t ldr, int M, int N, int K, int epi, hipStream_t s);
// bf16 MFMA GEMM; returns hipErrorNotSupported when the shape is outside what it handles.
// ws: optional fp32 scratch for the K-split partial tiles of the small-M path (see gemm_mfma_workspace_bytes).
hipError_t launch_gemm_mfma_bf16(const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                                 const void* R, int64_t ldr, int M, int N, int K, int epi, void* ws, int64_t ws_bytes,
                                 hipStream_t s);
int64_t gemm_mfma_workspace_bytes(int max_n);
bool gemm_mfma_swiglu_supported(int M, int N, int K, int64_t ws_bytes);
// Few token rows (M <= 64, bf16): the projection and the step that follows it in one pass of the split-K reduction.
bool gemm_small_m_fused_supported(int M, int N, int K, int64_t lda, int64_t ldw, int64_t ws_bytes);
bool gemm_small_m_rope_supported(int M, int K, int Hq, int Hkv, int dh, int64_t lda, int64_t ldw, int64_t ldq,
                                 int64_t ws_bytes);
bool gemm_small_m_rmsnorm_supported(int M, int d, int K, int64_t lda, int64_t ldw, int64_t ws_bytes);
// ssq (optional, with eps): the input rows lack the RMSNorm row factor, which is applied to the sums (see prescale)
hipError_t launch_gemm_small_m_rope(const void* A, int64_t lda, const void* W, int64_t ldw, void* qkv, int64_t ldq,
                                    const float2* cs, void* k_rows, void* v_rows, int M, int K, int Hq, int Hkv, int dh,
                                    void* ws, int64_t ws_bytes, const float* ssq, float eps, hipStream_t s);
// Few rows, RMSNorm split in two: a projection with residual writes h, a = bf16(h * g) and per-row partial sums of
// h^2 (ssq [M, d/1024]); the projection that reads a multiplies its sums by rsqrt(mean(h^2) + eps).  One launch less
// per norm than normalising in between, and the reduction stays spread over all compute units.
constexpr int DSK_MAX_SSQ_PARTS = 16;
bool gemm_small_m_prescale_supported(int M, int d, int K, int64_t lda, int64_t ldw, int64_t ws_bytes);
hipError_t launch_gemm_small_m_prescale(const void* A, int64_t lda, const void* W, int64_t ldw, float* h, const void* R,
                                        int r_f32, const void* g, void* a, float* ssq, int M, int d, int K, void* ws,
                                        int64_t ws_bytes, hipStream_t s);
hipError_t launch_gemm_small_m_swiglu_scaled(const void* A, int64_t lda, const void* W, int64_t ldw, void* act, int64_t ldc,
                                             int M, int N, int K, void* ws, int64_t ws_bytes, const float* ssq, float eps,
                                             hipStream_t s);
hipError_t launch_gemm_small_m_rmsnorm(const void* A, int64_t lda, const void* W, int64_t ldw, float* h, const void* R,
                                       int r_f32, const void* g, void* xn, float eps, int M, int d, int K, void* ws,
                                       int64_t ws_bytes, hipStream_t s);

// x is fp32 when x_f32 is set, else the model dtype; g and y are the model dtype
hipError_t launch_rmsnorm(int dtype, const void* x, int x_f32, const void* g, void* y, int T, int d, float eps, hipStream_t s);
extern thread_local int g_last_hip_error;  // hipError_t of the last failed HIP call on this thread
// Timing of single launches (the "time_gemm" hook): when set, the next tensor-core GEMM or attention launch on this
// thread attaches the two events to its own dispatch (they receive the kernel's start and stop times; no extra
// packets go into the stream) and clears the pair.
extern thread_local hipEvent_t g_launch_ev_start, g_launch_ev_stop;
#define DSK_LAUNCH_TIMED(kern, grid, block, lds, stream, ...)                                                        \
  do {                                                                                                               \
    if (g_launch_ev_start) {                                                                                         \
      hipExtLaunchKernelGGL(kern, grid, block, lds, stream, g_launch_ev_start, g_launch_ev_stop, 0, __VA_ARGS__);    \
      g_launch_ev_start = g_launch_ev_stop = nullptr;                                                                \
    } else {                                                                                                         \
      hipLaunchKernelGGL(kern, grid, block, lds, stream, __VA_ARGS__);                                               \
    }                                                                                                                \
  } while (0)

// pacing of the load stream against the 100 MHz constant-rate clock
hipError_t launch_pace_start(unsigned long long* t0, hipStream_t s);
hipError_t launch_pace_wait(const unsigned long long* t0, unsigned long long ticks, hipStream_t s);
hipError_t launch_rope_table(const int32_t* pos, const double* theta, float2* cs, int T, int half, hipStream_t s);
// rotates q (in place) and k of qkv [T, n_qkv]; writes rotated k and v to the cache rows row0..row0+T-1
hipError_t launch_rope_kv_write(int dtype, void* qkv, const float2* cs, void* k_rows, void* v_rows, int T, int Hq,
                                int Hkv, int dh, hipStream_t s);
// act[t,f] = silu(gate) * up from the interleaved gate/up GEMM output gu [T, 2F]
hipError_t launch_swiglu(int dtype, const void* gu, void* act, int T, int F, int gu_block, hipStream_t s);

// Causal grouped-query attention over packed sequences.  Query token i of sequence b (rows q_cu[b]..)
// sees cache rows p_cu[b] .. p_cu[b+1]-1 (all of them; p_cu may be NULL: no such segment) and rows
// own_row0 + q_cu[b] .. own_row0 + i.  q rows have stride ldq elements, out rows Hq*dh.
struct AttnArgs {
  const void* q; int64_t ldq;
  const void* k_rows; const void* v_rows;  // layer base of K and V rows (row stride Hkv*dh)
  void* out;
  const int32_t* q_cu; const int32_t* p_cu; const int32_t* q_cu_host; const int32_t* p_cu_host; int n_seqs;
  int64_t own_row0; int n_q; int Hq, Hkv, dh;
  const void* vt; int64_t ldvt;  // transposed V (see launch_transpose_v); NULL: not available
  void* ws; int64_t ws_bytes;    // fp32 scratch for key-split partial results (attn_mfma_workspace_bytes); optional
};
hipError_t launch_attn_generic(int dtype, const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_mfma_bf16(const AttnArgs& a, hipStream_t s);
int64_t attn_mfma_workspace_bytes(int Hq, int dh);
// vt[(c)*ldvt + row] = v_rows[row][c] for valid rows (row < n_pre or own_row0 <= row < own_row0+n_own), 0 otherwise,
// over the whole 64-row tiles from the one that holds first_row up to own_row0+n_own (earlier tiles of vt are left as
// they are); width = Hkv*dh must be a multiple of 64.
hipError_t launch_transpose_v(const void* v_rows, void* vt, int64_t ldvt, int width, int64_t n_pre, int64_t own_row0,
                              int64_t n_own, int64_t first_row, hipStream_t s);
// cu[0..3] = {a, b, c, d} on the device (sequence boundaries of a row chunk, set in stream order)
hipError_t launch_set_int4(int32_t* dst, int a, int b, int c, int d, hipStream_t s);

hipError_t launch_fill_normal(void* dst, int64_t n, uint64_t seed, uint64_t stream_id, float std, float offset,
                              int64_t idx0, int dtype, hipStream_t s);
// weight (re)packing: logical tensor rows <-> packed rows.  map: 0 identity + row_off, 1 gate rows, 2 up rows.
hipError_t launch_pack_rows(int dtype, void* packed, const void* logical, int64_t rows, int64_t cols, int map,
                            int gu_block, int64_t row_off, int to_packed, hipStream_t s);
hipError_t launch_fill_weight(int dtype, void* packed, int64_t rows, int64_t cols, int map, int gu_block, int64_t row_off,
                              uint64_t seed, uint64_t stream_id, float std, float offset, hipStream_t s);

// mixture-of-experts MLP: router, grouping by expert, grouped projections, gate-weighted sum (moe.hip, gemm_mfma.hip)
hipError_t launch_moe_route(int dtype, const void* xn, const void* wr, int32_t* experts, float* gates, int n, int d, int E,
                            int top_k, hipStream_t s);
// tile_tab: int4 [tile_rows_max + 1] (the last entry receives the number of tiles)
hipError_t launch_moe_place(const int32_t* experts, int32_t* slot_of, int32_t* src_token, void* tile_tab, int n, int top_k,
                            int E, int tile_m, int tile_rows_max, hipStream_t s);
// rows of the grouped projections' tile table for n_rows rows over E experts (every expert may end in a partial tile)
inline int moe_tile_table_rows(int64_t n_rows, int E) { return (int)((n_rows + 255) / 256) + E; }
hipError_t launch_moe_gather(int dtype, const void* xn, const int32_t* src_token, void* xg, int n_slots, int n_tokens, int d,
                             hipStream_t s);
hipError_t launch_moe_combine(const float* y, const float* h_mid, const float* gates, const int32_t* experts,
                              const int32_t* slot_of, void* out, int out_f32, int n, int d, int top_k, int64_t y_rows,
                              hipStream_t s);
hipError_t launch_gemm_mfma_grouped(const void* A, int64_t lda, int64_t a_rows, const void* W, int64_t ldw,
                                    int64_t w_group_stride, void* C, int64_t ldc, int N, int K, int epi,
                                    const void* tile_tab, int tile_rows, hipStream_t s);

// tuning knobs (dsk_set_option)
void gemm_mfma_set_variant(int v);
void attn_mfma_counts(int64_t* split, int64_t* packed, int reset);
bool gemm_mfma_uses_prefill_tile(int M, int N);
