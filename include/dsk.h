/*
 * dsk - selective-layer prefill for cross-model KV-cache reuse on AMD MI355X (gfx950).
 *
 * C ABI of the hot path of DroidSpeak (arxiv 2411.02820).  A receiver LLM takes the KV
 * cache a sender LLM of the same architecture produced for a context, recomputes one
 * contiguous group of decoder layers [lo, hi) from the sender's E cache (the hidden
 * state entering layer lo), keeps the sender's KV for every other layer, and then
 * prefills the new tokens against that mixed cache (Sec. 4.1).  Loading the reused
 * layers runs on a side stream under the recomputation (Sec. 4.3 "Smart KV Cache
 * Loading", Sec. 4.4: transfers on a stream other than the compute stream).
 *
 * Conventions
 *  - Every function returns DSK_OK (0) or a negative dsk_status.  Arguments are checked
 *    before anything is enqueued: a failed call has written nothing.
 *  - "device" pointers are HIP device memory of the current device, "host" pointers are
 *    ordinary host memory, "pinned" means page-locked host memory (hipHostMalloc).
 *  - Streams are hipStream_t passed as void*; NULL is the default stream.  Calls are
 *    asynchronous: they enqueue work and return without waiting for the device.
 *  - Layer indices are 0-based and half open: [lo, hi).  The paper's "recompute layers
 *    4-10 of 10" is lo=3, hi=10.
 *  - Element type is the model's dtype (fp32 or bf16) for hidden states, KV and weights.
 *  - Tokens of several sequences are packed back to back; sequence b owns token rows
 *    cu_seqlens[b] .. cu_seqlens[b+1]-1; causal order inside a sequence is packed order.
 *  - A model must not be used from two host threads at once, and two calls on one model
 *    must be issued on the same stream or be ordered by the caller.
 */
#ifndef DSK_H
#define DSK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define DSK_API __attribute__((visibility("default")))
#else
#define DSK_API
#endif

typedef struct dsk_model dsk_model_t;

typedef enum {
  DSK_OK = 0,
  DSK_EINVAL = -1, /* null pointer, bad layer range, bad batch descriptor, misaligned pointer */
  DSK_ESHAPE = -2, /* shape not supported (Hq % Hkv, odd head_dim, head_dim > 256, a bf16 shape outside what the
                      tensor-core kernels handle, ...) */
  DSK_EDTYPE = -3, /* dtype not DSK_F32 / DSK_BF16 */
  DSK_ENOMEM = -4, /* device or host allocation failed */
  DSK_EHIP = -5,   /* a HIP call failed; see dsk_last_hip_error() */
  DSK_ENOENT = -6, /* the cache store holds no such entry */
  DSK_ELIMIT = -7  /* size beyond the fixed limit of an entry point that works without allocating */
} dsk_status;

typedef enum { DSK_F32 = 0, DSK_BF16 = 1 } dsk_dtype;
typedef enum { DSK_MEM_DEVICE = 0, DSK_MEM_HOST_PINNED = 1 } dsk_mem;

/* Tensors of one decoder layer, each in its logical [out, in] row-major shape:
 * G1,G2 [d]; WQ [Hq*dh, d]; WK,WV [Hkv*dh, d]; WO [d, Hq*dh]; WG,WU [F, d]; WD [d, F]. */
typedef enum {
  DSK_G1 = 0, DSK_WQ = 1, DSK_WK = 2, DSK_WV = 3, DSK_WO = 4,
  DSK_G2 = 5, DSK_WG = 6, DSK_WU = 7, DSK_WD = 8,
  DSK_WR = 9 /* router [E, d] of a mixture-of-experts layer */
} dsk_tensor;
/* Mixture-of-experts models (n_experts > 0) have no layer-wide WG/WU/WD; expert e's are addressed as
 * DSK_EXPERT(e, DSK_WG | DSK_WU | DSK_WD) wherever a tensor id is taken. */
#define DSK_EXPERT(e, t) (16 + (e) * 16 + (t))
#define DSK_MOE_MAX_EXPERTS 64
#define DSK_MOE_MAX_TOP_K 8

/* Llama-style decoder: pre-norm residual blocks, RMSNorm (eps inside the root), rotary
 * embedding on pairs (i, i+dh/2) with theta_i = rope_base^(-2i/dh), grouped-query causal
 * attention (kv head = q head / (Hq/Hkv)), SwiGLU MLP, no biases. */
typedef struct {
  int32_t n_layers;   /* L */
  int32_t hidden;     /* d */
  int32_t n_q_heads;  /* Hq */
  int32_t n_kv_heads; /* Hkv, divides Hq */
  int32_t head_dim;   /* dh, even, <= 256 */
  int32_t ffn;        /* F */
  double rope_base;
  double rms_eps;
  int32_t dtype;      /* dsk_dtype */
  /* Mixture-of-experts receiver (Sec. 5.4, Mixtral): the MLP of every layer is n_experts SwiGLU MLPs of width F
   * behind a router; a token goes through its top_k experts by router logit (equal logits: lower index first) and
   * their outputs are added with the softmax of those top_k logits.  Attention and the KV cache are as in the dense
   * model, so everything the selective prefill does with caches is unchanged.  0 / 0: dense MLP. */
  int32_t n_experts;  /* E <= DSK_MOE_MAX_EXPERTS */
  int32_t top_k;      /* 1 <= top_k <= min(E, DSK_MOE_MAX_TOP_K) */
} dsk_config_t;

/* A per-layer KV cache (Sec. 4.4: the cache is split into layers).  Layer l's keys are
 * rows of Hkv*dh elements starting at base + l*layer_stride, its values start v_offset
 * bytes later; row r is at + r*Hkv*dh*elem_size.  Keys are stored after the rotary
 * embedding, values as projected.  Prefix token t lives in row t (its packed index). */
typedef struct {
  void* base;
  int32_t mem;          /* dsk_mem: where base points */
  int64_t layer_stride; /* bytes between layers */
  int64_t v_offset;     /* bytes from a layer's K rows to its V rows, >= n_rows*Hkv*dh*elem */
  int64_t n_rows;       /* rows allocated per layer for K (and for V) */
} dsk_kv_t;

/* A packed (ragged) batch of token rows. */
typedef struct {
  int32_t n_seqs;                 /* B >= 1 */
  int32_t n_tokens;               /* = cu_seqlens[B] */
  const int32_t* cu_seqlens_host; /* host, [B+1], cu[0]=0, strictly increasing */
  const int32_t* cu_seqlens_dev;  /* device copy of the same array */
  const int32_t* positions_dev;   /* device, [n_tokens], rotary position of every token; may be NULL for
                                     descriptors that only delimit sequences */
} dsk_batch_t;

/* flags of dsk_partial_prefill */
#define DSK_DEFER_JOIN 1u /* do not make `stream` wait for the reused-layer loads at the end of the call;
                             the following dsk_suffix_prefill waits layer by layer, or call dsk_join_loads */
/* How the reused layers are brought in (the three strategies of Sec. 4.3, Fig. 13). */
typedef enum {
  DSK_LOAD_PIPELINED = 0,    /* (c) E cache first, reused layers on the side stream under the recompute */
  DSK_LOAD_REUSED_FIRST = 1, /* (b) load the reused layers, then recompute */
  DSK_LOAD_ALL_FIRST = 2     /* (a) load every layer of the sender's KV, then recompute */
} dsk_load_mode;

/* Creates a model: allocates its weights (library-owned, in the library's own packed
 * layout), a workspace for up to max_tokens token rows per call and for caches whose used rows
 * stay below max_kv_rows (>= max_tokens; prefix rows plus suffix rows), a side stream and
 * per-layer events, on the current device.  Weights start undefined: fill them with
 * dsk_model_set_tensor or dsk_model_init_random.  *out is written only on success. */
DSK_API int dsk_model_create(const dsk_config_t* cfg, int64_t max_tokens, int64_t max_kv_rows, dsk_model_t** out);

/* Waits for the model's outstanding work and frees everything it owns. */
DSK_API int dsk_model_destroy(dsk_model_t* model);

/* Copies one tensor (logical [out,in] row-major, model dtype) into the model.  A device src is
 * read on `stream`, asynchronously.  A host src (pinned or ordinary memory, src_mem =
 * DSK_MEM_HOST_PINNED) is staged through a temporary device buffer and the call returns after
 * the copy has completed. */
DSK_API int dsk_model_set_tensor(dsk_model_t* model, int layer, int tensor, const void* src, int src_mem, void* stream);

/* Writes one tensor back in its logical layout to device memory dst (for checks). */
DSK_API int dsk_model_get_tensor(const dsk_model_t* model, int layer, int tensor, void* dst_device, void* stream);

/* Fills all weights on the device with the counter-based generator of dsk_fill_normal:
 * tensor `t` of layer `l` is stream l*16+t, element index = out*in_dim + in; projection
 * matrices N(0, std), norm gains 1 + N(0, std); WG, WU, WD of expert e are streams
 * 2^20 + (l*64 + e)*4 + {0, 1, 2}.  For synthetic workloads (the 70B shape cannot be staged
 * through host memory). */
DSK_API int dsk_model_init_random(dsk_model_t* model, uint64_t seed, float std, void* stream);

/* dst[i] = offset + std * z(seed, stream_id, idx0 + i), i < n, rounded to dtype; z is an
 * integer-only approximately normal variate (sum of eight 16-bit lanes of two SplitMix64
 * outputs, centred, scaled in fp32), so any implementation reproduces it bit for bit. */
DSK_API int dsk_fill_normal(void* dst_device, int64_t n, uint64_t seed, uint64_t stream_id, float std, float offset,
                    int64_t idx0, int dtype, void* stream);

/* Selective-layer prefill (Sec. 4.1; the partial_prefill interface of Sec. 4.4).
 *   hidden_in   [n_tokens, d]  E cache at the transition layer lo (the token embeddings when lo = 0);
 *               device, or pinned host (then it is transferred first, before any KV: Fig. 13(c); a long single
 *               sequence arrives in row chunks and layer lo starts on the first chunk while the rest is in flight).
 *   kv_reused   the sender's cache, device or pinned host; may be NULL when lo=0 and hi=L.
 *   kv_out      device cache that receives, for lo <= l < hi, K and V recomputed by the receiver
 *               (rows 0..n_tokens-1), and for every other l a byte-exact copy of kv_reused's rows
 *               0..n_tokens-1.  kv_out may alias kv_reused (same base and strides, device): the
 *               splice is then free.  Rows >= n_tokens are left untouched.
 *   batch       the packed prefix tokens with their positions.
 *   hidden_out  optional device [n_tokens, d]: state leaving layer hi-1 (a copy of hidden_in if lo=hi).
 * lo = hi is valid (pure splice).  Compute runs on `stream`, loads on the model's side stream
 * after everything already enqueued on `stream`; on return from the call nothing has been waited
 * for.  Unless DSK_DEFER_JOIN is set, work enqueued on `stream` afterwards sees the whole cache.
 * Host buffers must stay valid until `stream` (and, with DSK_DEFER_JOIN, the loads) have drained. */
DSK_API int dsk_partial_prefill(dsk_model_t* model, const void* hidden_in, int hidden_in_mem, int lo, int hi,
                        const dsk_kv_t* kv_reused, const dsk_kv_t* kv_out, const dsk_batch_t* batch,
                        void* hidden_out, uint32_t flags, void* stream);

/* One recomputed layer group of dsk_partial_prefill_groups. */
typedef struct dsk_group_t {
  int32_t lo, hi;         /* layers lo <= l < hi are recomputed */
  const void* hidden_in;  /* [n_tokens, d] E cache at layer lo, device or pinned host */
  int32_t hidden_in_mem;  /* dsk_mem */
  void* hidden_out;       /* optional device [n_tokens, d]: state leaving layer hi-1 */
} dsk_group_t;

/* Selective-layer prefill with several recomputed groups (Sec. 4.1: the layers worth recomputing form
 * "critical layer groups", not necessarily one run).  groups[0..n_groups) must be ascending and disjoint
 * (groups[g].hi <= groups[g+1].lo), else DSK_EINVAL; every group restarts from its own E cache and what it
 * leaves in the residual stream is only reported through its hidden_out.  Layers outside all groups are
 * spliced from kv_reused as in dsk_partial_prefill, whose other rules (aliasing, streams, flags, lifetime
 * of host buffers) apply unchanged; n_groups = 0 is a pure splice.  Host-resident E caches share one
 * staging buffer: the first is transferred before any KV, a later one after the KV loads and after the
 * preceding group's first layer has consumed the buffer.  dsk_partial_prefill is the one-group case. */
DSK_API int dsk_partial_prefill_groups(dsk_model_t* model, const dsk_group_t* groups, int n_groups,
                               const dsk_kv_t* kv_reused, const dsk_kv_t* kv_out, const dsk_batch_t* batch,
                               uint32_t flags, void* stream);

/* Prefill of the new tokens against the mixed cache through all L layers (Sec. 4.1: a layer whose
 * KV is reused only sees the new tokens).  Suffix token j of sequence b attends to prefix rows
 * prefix.cu[b] .. prefix.cu[b+1]-1 and to suffix tokens suffix.cu[b] .. j; its K/V is written to
 * row suffix_row0 + j of every layer of kv.  Per layer, waits for that layer's load if a preceding
 * dsk_partial_prefill deferred its join.
 *   suffix_hidden_in [suffix.n_tokens, d] device;  hidden_out [suffix.n_tokens, d] device: state
 *   leaving the last layer (before any final norm).  prefix.positions_dev is not used. */
DSK_API int dsk_suffix_prefill(dsk_model_t* model, const void* suffix_hidden_in, const dsk_kv_t* kv,
                       const dsk_batch_t* prefix, const dsk_batch_t* suffix, int64_t suffix_row0,
                       void* hidden_out, void* stream);

/* Makes `stream` wait for all loads a deferred dsk_partial_prefill left outstanding. */
DSK_API int dsk_join_loads(dsk_model_t* model, void* stream);

/* Selects the loading strategy used by later dsk_partial_prefill calls (default pipelined). */
DSK_API int dsk_set_load_mode(dsk_model_t* model, int load_mode);

/* Paces later loads (E caches and reused layers) to at most gb_per_s GB/s by idling the load stream after
 * every 1 MiB chunk until that chunk would have arrived over such a link; 0 switches pacing off.  It
 * emulates a slower link between the cache's home and the GPU for the loading-strategy and bandwidth
 * experiments (Sec. 4.3 Fig. 13; Sec. 5.5 Fig. 20); results are unchanged. */
DSK_API int dsk_set_load_throttle(dsk_model_t* model, double gb_per_s);

/* ---- cache store: the store / fetch interfaces of Sec. 4.4 ----
 * A key-value store of KV and E caches, split by layer, keyed by the hash of the context text and the model that
 * produced them, kept in GPU memory (the paper's choice) with pinned host memory as a second tier.  The store
 * owns the memory; pointers and descriptors it hands out stay valid until the entry is erased or the store
 * destroyed, and what they point to is complete once the stream given to the put call has drained.  Calls are
 * serialised by an internal lock.  partial_prefill (Sec. 4.4) is dsk_partial_prefill[_groups] fed with these
 * descriptors. */
typedef struct dsk_store dsk_store_t;
typedef enum { DSK_TIER_AUTO = 0, DSK_TIER_DEVICE = 1, DSK_TIER_HOST = 2 } dsk_tier; /* AUTO: device while it fits */

/* Key of a context: 64-bit FNV-1a of the bytes of its text (Sec. 4.4 keys the store by a hash of the context
 * text and does not name the function). */
DSK_API uint64_t dsk_hash_context(const void* bytes, int64_t n);

/* Capacities bound what each tier may hold; a put that fits nowhere returns DSK_ENOMEM. */
DSK_API int dsk_store_create(int64_t device_capacity_bytes, int64_t host_capacity_bytes, dsk_store_t** out);
/* Frees every entry (waits for device work on them) and the store. */
DSK_API int dsk_store_destroy(dsk_store_t* store);

/* store(Cache, context, LLM) for a KV cache: copies rows 0..n_rows-1 of all n_layers layers of `kv` (device or
 * pinned host; row_bytes = Hkv*dh*element size) into a compact slab of the chosen tier, on `stream`.  If the
 * (context, model) pair is already present nothing happens (Sec. 4.4) and *inserted (optional) is 0. */
DSK_API int dsk_store_put_kv(dsk_store_t* store, uint64_t context, uint64_t model_id, const dsk_kv_t* kv, int n_layers,
                     int64_t n_rows, int64_t row_bytes, int tier, void* stream, int* inserted);
/* The same for the E cache at transition layer `layer` ([n_tokens, d], `bytes` in all). */
DSK_API int dsk_store_put_e(dsk_store_t* store, uint64_t context, uint64_t model_id, int layer, const void* e_cache,
                    int e_mem, int64_t bytes, int tier, void* stream, int* inserted);

/* fetch(context, LLM, layer_id) -> Cache.  Per layer: K and V row blocks of that layer; or the whole cache as a
 * descriptor that dsk_partial_prefill accepts as kv_reused; or the E cache stored for a transition layer.
 * DSK_ENOENT if nothing was stored under the key. */
DSK_API int dsk_store_fetch_kv_layer(dsk_store_t* store, uint64_t context, uint64_t model_id, int layer,
                             const void** k_rows, const void** v_rows, int* mem, int64_t* bytes_each);
DSK_API int dsk_store_fetch_kv(dsk_store_t* store, uint64_t context, uint64_t model_id, dsk_kv_t* out, int* n_layers);
DSK_API int dsk_store_fetch_e(dsk_store_t* store, uint64_t context, uint64_t model_id, int layer, const void** e_cache,
                      int* mem, int64_t* bytes);

/* Drops everything stored for (context, model); waits for device work that may still use it. */
DSK_API int dsk_store_erase(dsk_store_t* store, uint64_t context, uint64_t model_id);
DSK_API int dsk_store_usage(dsk_store_t* store, int64_t* device_bytes, int64_t* host_bytes, int64_t* n_entries);

/* ---- run-time choice of the re-computation configuration (App. B); host code, no device work ---- */

/* One point of the offline profile's Pareto frontier (Sec. 4.2): recomputing layers [lo, hi) gave `quality`. */
typedef struct dsk_frontier_point_t {
  int32_t lo, hi;
  double quality;
} dsk_frontier_point_t;

/* Profiled prefill-delay model in ms: c0 + R*(c_layer_token*T + c_layer_token2*T^2) + (L-R)*c_reused_token*T
 * for R recomputed of L layers and T tokens (projections and MLP are linear in T, causal attention quadratic,
 * a reused layer costs its KV transfer). */
typedef struct dsk_latency_model_t {
  double c0, c_layer_token, c_layer_token2, c_reused_token;
} dsk_latency_model_t;

DSK_API double dsk_estimate_prefill_ms(const dsk_latency_model_t* lat, int n_layers, int n_recomputed, int64_t n_tokens);

/* App. B: with requests waiting (n_waiting > 0) the point with the fewest recomputed layers whose quality
 * reaches quality_target; otherwise the point with the most recomputed layers whose estimated delay for
 * n_tokens meets slo_ms.  If no point qualifies the one with the fewest layers is taken; equal layer counts go
 * to the better quality, then to the lower index.  *chosen receives the index into frontier.  DSK_EINVAL for
 * null or empty input or a point outside [0, n_layers]. */
DSK_API int dsk_select_recompute(const dsk_frontier_point_t* frontier, int n_points, int n_layers, int64_t n_tokens,
                         const dsk_latency_model_t* lat, double slo_ms, double quality_target, int n_waiting,
                         int* chosen);

/* ---- component entry points: single steps of the layer, for parity tests and micro-benchmarks ---- */

/* y[M,N] = x[M,K] * w[N,K]^T (+ r[M,N] if r != NULL); all device, row-major, dense rows, dtype as given.
 * The projection step of the layer (QKV, O, gate/up, down); y may alias r.  bf16 runs on the tensor-core kernels
 * and needs K a multiple of 64, N a multiple of 4 and M*K, N*K below 2^31 elements, else DSK_ESHAPE. */
DSK_API int dsk_linear(int dtype, const void* x, const void* w, void* y, const void* r, int M, int N, int K, void* stream);

/* dsk_linear for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as dsk_linear for the few-row
 * projections of the suffix pass, M <= DSK_STATIC_MAX_M rows and N <= DSK_STATIC_MAX_N columns (any K the
 * kernels handle); larger M or N return DSK_ELIMIT and nothing is enqueued.  The fp32 partial sums of the K-split
 * go to a fixed array of DSK_STATIC_SCRATCH_BYTES inside the library's code object (every GPU the library runs on
 * holds its copy until the process ends) instead of a buffer allocated on first use: the call allocates and frees
 * nothing, on the host or on the device.  Nothing in the array has to start at zero (a call writes every partial
 * sum before its reduction reads it), so it is never cleared.  All calls on one GPU share the array: calls that
 * overlap in time (different streams, or one stream under concurrent graph launches) race on it and must be
 * ordered by the caller. */
#define DSK_STATIC_MAX_M 64
#define DSK_STATIC_MAX_N 65536
#define DSK_STATIC_SCRATCH_BYTES (32 << 20) /* 64 rows x (at most 131072 split x column pairs) x 4 bytes */
DSK_API int dsk_linear_static(int dtype, const void* x, const void* w, void* y, const void* r, int M, int N, int K,
                              void* stream);

/* Causal grouped-query attention of packed query tokens q [n_q, Hq*dh] (already rotated) against cache
 * rows k_rows/v_rows (row stride Hkv*dh): query i of sequence b sees rows prefix.cu[b]..prefix.cu[b+1]-1
 * (prefix may be NULL) and rows own_row0+queries.cu[b] .. own_row0+i.  out [n_q, Hq*dh].  All device.
 * prefix.n_tokens <= own_row0 (the two row ranges do not overlap), else DSK_EINVAL.
 * scratch: device buffer of scratch_bytes >= Hkv*dh*roundup64(own_row0+n_q)*elem bytes: the bf16 tensor-core
 * kernel keeps a transposed copy of V there.  scratch = NULL selects the plain-ALU kernel (any dtype); a bf16 call
 * with scratch whose shape the tensor-core kernel does not handle (head_dim other than 64 or 128, Hkv*dh not a
 * multiple of 64, scratch too small) returns DSK_ESHAPE. */
DSK_API int dsk_attention(int dtype, const void* q, const void* k_rows, const void* v_rows, void* out,
                          const dsk_batch_t* queries, const dsk_batch_t* prefix, int64_t own_row0, int n_q_heads,
                          int n_kv_heads, int head_dim, void* scratch, int64_t scratch_bytes, void* stream);

/* Router of a mixture-of-experts layer (Sec. 5.4; routing as in Mixtral) on its own: for token rows x [n, d] and
 * router weights wr [E, d] (both `dtype`, device) writes the top_k experts of every token by fp32 router logit,
 * highest first, equal logits to the lower index (experts_out int32 [n, top_k]) and the softmax of those logits
 * (gates_out fp32 [n, top_k]).  d a multiple of 8; limits as in dsk_config_t, else DSK_ESHAPE. */
DSK_API int dsk_moe_route(int dtype, const void* x, const void* wr, int n, int d, int n_experts, int top_k,
                          int32_t* experts_out, float* gates_out, void* stream);

/* ---- hooks for tests and benchmarks (process-wide, not thread-safe; no production caller needs them) ----
 * Unknown names and out-of-range values return DSK_EINVAL.
 *   "force_generic": 1 = bf16 work runs on the plain-ALU kernels that serve fp32 models (about a hundred times
 *                slower).  Without it a bf16 shape the tensor-core kernels do not handle is an error (DSK_ESHAPE
 *                from dsk_model_create, dsk_linear, dsk_attention), never a silent switch of kernels.
 *   "gemm_tiling": force one of the two prefill tilings of the bf16 GEMM on any M > 64 (default 0 = picked by
 *                size): 1 = 256x256 tiles on the 16x16x32 MFMA, 2 = 128x128 tiles on the 32x32x16 MFMA
 *   "e_chunk_rows": how a host-resident E cache is cut into row chunks that the first recomputed layer follows as
 *                they arrive: 0 (default) = 4096-row chunks where that keeps every result bit-identical to the
 *                unchunked run (one sequence, bf16, chunks that still fill the chip), -1 = never, n > 0 (a multiple
 *                of 256) = n-row chunks on any single-sequence bf16 call (results then agree within tolerance only)
 *   "time_gemm": 1 = bracket every tensor-core GEMM launch that runs on the 256 x 256 prefill tiling (at least
 *                192 such tiles), and every tensor-core attention launch of the prefix pass (at least 1024 query rows, no
 *                earlier rows), by a pair of HIP events attached to the kernel's own dispatch (they receive its start and
 *                stop times, nothing else is put into the stream; read back through dsk_get_stat)
 *   "reset_stats": any value; clears all counters and recorded timings */
DSK_API int dsk_set_option(const char* name, int value);

/* Counters since the last reset: "e_cache_chunks" (row chunks of host-resident E caches that a first recomputed
 * layer followed as they arrived), "gemm_mfma_launches", "gemm_generic_launches", "attn_mfma_launches",
 * "attn_generic_launches", "attn_key_split_launches" (tensor-core attention launches that split the keys over
 * workgroups) and, of those, "attn_packed_head_launches" (four q heads of a kv group per workgroup); and for the
 * launches bracketed under "time_gemm": "timed_gemm_launches", "timed_gemm_ms" (sum of their durations; waits for
 * them to finish), "timed_gemm_flops" (sum of 2*M*N*K), and the same three as "timed_attn_..." for the attention
 * launches (flops = 4*Hq*dh per (query, visible key) pair, i.e. causal). */
DSK_API int dsk_get_stat(const char* name, double* value);

/* Sizes, for callers that budget memory. */
DSK_API int64_t dsk_model_weight_bytes(const dsk_model_t* model);
DSK_API int64_t dsk_model_workspace_bytes(const dsk_model_t* model);

DSK_API const char* dsk_strerror(int status);
/* hipError_t (as int) of the last failed HIP call on this host thread, 0 if none. */
DSK_API int dsk_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DSK_H */
