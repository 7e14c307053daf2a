// Mixture-of-experts MLP (the Mixtral receiver of Sec. 5.4): router, grouping of the token rows by expert, and the
// gate-weighted sum of the expert outputs.  The expert projections themselves run on the GEMM kernels.
//
// Routing as in Mixtral: router logits = xn * Wr^T in fp32, the top_k experts of a token by logit (equal logits go to
// the lower expert index), gate weights = softmax over the chosen logits.
#include "dsk_internal.h"

namespace {

constexpr int MAX_K = DSK_MOE_MAX_TOP_K;

template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> { typedef __attribute__((ext_vector_type(8))) __bf16 type; };
template <> struct Vec8<float> { typedef __attribute__((ext_vector_type(8))) float type; };

// One wave per token: the E dot products one after the other (the row of xn stays in the cache), each reduced over
// the wave in a fixed order, then the top_k choice and the softmax on values every lane holds.
template <typename T>
__global__ void __launch_bounds__(256) moe_route_kernel(const T* __restrict__ xn, const T* __restrict__ wr,
                                                        int32_t* __restrict__ experts, float* __restrict__ gates, int n,
                                                        int d, int E, int top_k) {
  typedef typename Vec8<T>::type vec8;
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= n) return;
  float best_v[MAX_K];
  int best_e[MAX_K];
#pragma unroll
  for (int j = 0; j < MAX_K; ++j) { best_v[j] = -INFINITY; best_e[j] = -1; }
  const T* x = xn + (int64_t)t * d;
  // the token's row is read once and kept in registers (widths up to 512 * XCH; wider rows are re-read per expert)
  constexpr int XCH = 8;
  const bool in_regs = d <= 512 * XCH;
  vec8 xr[XCH];
  if (in_regs) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const int c = lane * 8 + 512 * i;
      if (c < d) xr[i] = *(const vec8*)(x + c);
    }
  }
  for (int e = 0; e < E; ++e) {
    const T* w = wr + (int64_t)e * d;
    float acc = 0.f;
    if (in_regs) {
      // same products in the same order as the loop below
      vec8 wv[XCH];
#pragma unroll
      for (int i = 0; i < XCH; ++i) {
        const int c = lane * 8 + 512 * i;
        if (c < d) wv[i] = *(const vec8*)(w + c);
      }
#pragma unroll
      for (int i = 0; i < XCH; ++i) {
        const int c = lane * 8 + 512 * i;
        if (c < d) {
#pragma unroll
          for (int u = 0; u < 8; ++u) acc = fmaf(to_f32(xr[i][u]), to_f32(wv[i][u]), acc);
        }
      }
    } else {
      for (int c = lane * 8; c < d; c += 512) {
        const vec8 a = *(const vec8*)(x + c), b = *(const vec8*)(w + c);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = fmaf(to_f32(a[u]), to_f32(b[u]), acc);
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (!(acc == acc)) acc = -3.0e38f;  // a NaN logit ranks last: every list entry below is then a real expert
    // insert into the descending list; strictly greater only, so that an earlier expert keeps its place on a tie
    float v = acc;
    int id = e;
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
      if (j < top_k && v > best_v[j]) {
        const float tv = best_v[j];
        const int te = best_e[j];
        best_v[j] = v; best_e[j] = id;
        v = tv; id = te;
      }
    }
  }
  if (lane == 0) {
    float p[MAX_K], sum = 0.f;
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
      p[j] = j < top_k ? expf(best_v[j] - best_v[0]) : 0.f;
      sum += p[j];
    }
    const float inv = 1.0f / sum;
#pragma unroll
    for (int j = 0; j < MAX_K; ++j)
      if (j < top_k) {
        experts[(int64_t)t * top_k + j] = best_e[j];
        gates[(int64_t)t * top_k + j] = p[j] * inv;
      }
  }
}

// Groups the n*top_k (token, choice) entries by expert, keeping token order inside an expert (so the result does not
// depend on timing).  One workgroup per expert e: it counts the entries of every expert (LDS histogram), derives the
// first slot of its own rows and the first row tile of its own tiles, then walks the entries in order and gives the
// j-th entry of expert e the slot first + j.  slot_of[entry] = slot, src_token[slot] = token.  tile_tab[r], r <
// tile_rows_max: {expert, first slot of the tile, end of the expert's slots, 0}, the tiles of all experts back to back,
// expert -1 past the last tile; tile_tab[tile_rows_max].x = number of tiles (the GEMM spreads exactly those over the
// chip: a grid sized for the worst case would leave the dies that get its empty end idle).
__global__ void __launch_bounds__(256) moe_place_kernel(const int32_t* __restrict__ experts, int32_t* __restrict__ slot_of,
                                                        int32_t* __restrict__ src_token, int4* __restrict__ tile_tab,
                                                        int n_entries, int top_k, int E, int tile_m, int tile_rows_max) {
  __shared__ int hist[DSK_MOE_MAX_EXPERTS];
  __shared__ int wave_cnt[2][4][4];
  const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < DSK_MOE_MAX_EXPERTS) hist[tid] = 0;
  __syncthreads();
  for (int base = tid; base < n_entries; base += 1024) {
    int x[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) x[q] = base + 256 * q < n_entries ? experts[base + 256 * q] : -1;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if ((unsigned)x[q] < (unsigned)E) atomicAdd(&hist[x[q]], 1);  // the router only writes experts below E
  }
  __syncthreads();
  int first = 0, first_tile = 0;
  for (int x = 0; x < e; ++x) {
    first += hist[x];
    first_tile += (hist[x] + tile_m - 1) / tile_m;
  }
  const int mine = hist[e];
  const int my_tiles = (mine + tile_m - 1) / tile_m;
  for (int r = tid; r < my_tiles; r += 256)
    if (first_tile + r < tile_rows_max) tile_tab[first_tile + r] = make_int4(e, first + r * tile_m, first + mine, 0);
  if (e == E - 1) {
    for (int r = first_tile + my_tiles + tid; r < tile_rows_max; r += 256) tile_tab[r] = make_int4(-1, 0, 0, 0);
    if (tid == 0) tile_tab[tile_rows_max] = make_int4(min(first_tile + my_tiles, tile_rows_max), 0, 0, 0);
  }
  // rounds of 1024 entries, four groups of 256 in entry order; a thread's four entries are requested together (the
  // walk is a chain of short rounds: what it takes is the round trips to memory)
  int running = 0;
  int buf = 0;
  for (int base = 0; base < n_entries; base += 1024, buf ^= 1) {
    int ex[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = base + 256 * q + tid;
      ex[q] = i < n_entries ? experts[i] : -1;
    }
    unsigned long long mask[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      mask[q] = __ballot(ex[q] == e);
      if (lane == 0) wave_cnt[buf][q][wave] = __popcll(mask[q]);
    }
    __syncthreads();  // the other buffer is written in the next round, after every wave has passed this barrier
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int before = __popcll(mask[q] & ((1ull << lane) - 1ull));
      int total = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int c = wave_cnt[buf][q][w];
        if (w < wave) before += c;
        total += c;
      }
      if (ex[q] == e) {
        const int i = base + 256 * q + tid;
        const int slot = first + running + before;
        slot_of[i] = slot;
        src_token[slot] = i / top_k;
      }
      running += total;
    }
  }
}

// xg[slot][:] = xn[src_token[slot]][:], rows of d elements moved 16 bytes at a time
template <typename T>
__global__ void __launch_bounds__(256) moe_gather_kernel(const T* __restrict__ xn, const int32_t* __restrict__ src_token,
                                                         T* __restrict__ xg, int n_slots, int n_tokens, int d) {
  const int per_row = d * (int)sizeof(T) / 16;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)n_slots * per_row) return;
  const int slot = (int)(i / per_row), c = (int)(i - (int64_t)slot * per_row);
  const int tok = min(max(src_token[slot], 0), n_tokens - 1);  // always inside xn, whatever the table holds
  const int4* src = (const int4*)(xn + (int64_t)tok * d);
  ((int4*)(xg + (int64_t)slot * d))[c] = src[c];
}

// out[t][:] = h_mid[t][:] + sum_j gates[t][j] * y[row(t, j)][:], j in the order of the router's list (highest logit
// first).  row(t, j) = slot_of[t*top_k + j] when the rows are grouped by expert, experts[t*top_k + j] * n + t when
// every expert ran over all n rows.  y and h_mid are fp32; out is fp32 or the model dtype.
template <typename TO>
__global__ void __launch_bounds__(256) moe_combine_kernel(const float* __restrict__ y, const float* __restrict__ h_mid,
                                                          const float* __restrict__ gates,
                                                          const int32_t* __restrict__ experts,
                                                          const int32_t* __restrict__ slot_of, TO* __restrict__ out, int n,
                                                          int d, int top_k, int64_t y_rows) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const int quads = d / 4;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)n * quads) return;
  const int t = (int)(i / quads), c = (int)(i - (int64_t)t * quads) * 4;
  f32x4 acc = *(const f32x4*)(h_mid + (int64_t)t * d + c);
  for (int j = 0; j < top_k; ++j) {
    int64_t row = slot_of ? (int64_t)slot_of[(int64_t)t * top_k + j] : (int64_t)experts[(int64_t)t * top_k + j] * n + t;
    row = row < 0 ? 0 : (row >= y_rows ? y_rows - 1 : row);  // always inside y, whatever the tables hold
    const float g = gates[(int64_t)t * top_k + j];
    const f32x4 v = *(const f32x4*)(y + row * d + c);
    acc[0] = fmaf(g, v[0], acc[0]); acc[1] = fmaf(g, v[1], acc[1]);
    acc[2] = fmaf(g, v[2], acc[2]); acc[3] = fmaf(g, v[3], acc[3]);
  }
  TO* o = out + (int64_t)t * d + c;
#pragma unroll
  for (int u = 0; u < 4; ++u) o[u] = from_f32<TO>(acc[u]);
}

}  // namespace

hipError_t launch_moe_route(int dtype, const void* xn, const void* wr, int32_t* experts, float* gates, int n, int d, int E,
                            int top_k, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (E < 1 || E > DSK_MOE_MAX_EXPERTS || top_k < 1 || top_k > MAX_K || top_k > E || d % 8) return hipErrorNotSupported;
  const dim3 grid((unsigned)((n + 3) / 4));
  if (dtype == DSK_BF16)
    hipLaunchKernelGGL(moe_route_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)xn, (const bf16_t*)wr, experts, gates,
                       n, d, E, top_k);
  else
    hipLaunchKernelGGL(moe_route_kernel<float>, grid, dim3(256), 0, s, (const float*)xn, (const float*)wr, experts, gates, n,
                       d, E, top_k);
  return hipGetLastError();
}

hipError_t launch_moe_place(const int32_t* experts, int32_t* slot_of, int32_t* src_token, void* tile_tab, int n, int top_k,
                            int E, int tile_m, int tile_rows_max, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(moe_place_kernel, dim3(E), dim3(256), 0, s, experts, slot_of, src_token, (int4*)tile_tab, n * top_k,
                     top_k, E, tile_m, tile_rows_max);
  return hipGetLastError();
}

hipError_t launch_moe_gather(int dtype, const void* xn, const int32_t* src_token, void* xg, int n_slots, int n_tokens,
                             int d, hipStream_t s) {
  if (n_slots <= 0) return hipSuccess;
  const int elem = dtype == DSK_BF16 ? 2 : 4;
  const int64_t units = (int64_t)n_slots * (d * elem / 16);
  const dim3 grid((unsigned)((units + 255) / 256));
  if (dtype == DSK_BF16)
    hipLaunchKernelGGL(moe_gather_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)xn, src_token, (bf16_t*)xg, n_slots,
                       n_tokens, d);
  else
    hipLaunchKernelGGL(moe_gather_kernel<float>, grid, dim3(256), 0, s, (const float*)xn, src_token, (float*)xg, n_slots,
                       n_tokens, d);
  return hipGetLastError();
}

hipError_t launch_moe_combine(const float* y, const float* h_mid, const float* gates, const int32_t* experts,
                              const int32_t* slot_of, void* out, int out_f32, int n, int d, int top_k, int64_t y_rows,
                              hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int64_t units = (int64_t)n * (d / 4);
  const dim3 grid((unsigned)((units + 255) / 256));
  if (out_f32)
    hipLaunchKernelGGL(moe_combine_kernel<float>, grid, dim3(256), 0, s, y, h_mid, gates, experts, slot_of, (float*)out, n, d,
                       top_k, y_rows);
  else
    hipLaunchKernelGGL(moe_combine_kernel<bf16_t>, grid, dim3(256), 0, s, y, h_mid, gates, experts, slot_of, (bf16_t*)out, n,
                       d, top_k, y_rows);
  return hipGetLastError();
}
