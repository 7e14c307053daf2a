// Per-layer KV / E cache store keyed by (context hash, model id) with a device tier and a pinned-host tier
// (the store / fetch interfaces of Sec. 4.4).  Host-side bookkeeping; the only device work is the copy of a
// stored cache into its slab.
#include "dsk_internal.h"

#include <map>
#include <mutex>
#include <tuple>

struct dsk_store {
  struct Entry {
    void* base = nullptr;
    int mem = DSK_MEM_DEVICE;
    int64_t bytes = 0;
    // KV slabs: compact [n_layers][K rows | V rows]
    int n_layers = 0;
    int64_t n_rows = 0, row_bytes = 0;
  };
  // kind 0 = KV (layer field -1: one slab holds every layer), kind 1 = E cache at transition layer `layer`
  typedef std::tuple<uint64_t, uint64_t, int, int> Key;
  std::map<Key, Entry> entries;
  int64_t cap[2] = {0, 0}, used[2] = {0, 0};  // by dsk_mem
  std::mutex mu;
};

namespace {

int store_alloc(dsk_store* st, int tier, int64_t bytes, dsk_store::Entry* e) {
  // DSK_TIER_AUTO: device memory while it lasts, then pinned host memory
  int order[2], n = 0;
  if (tier == DSK_TIER_DEVICE || tier == DSK_TIER_AUTO) order[n++] = DSK_MEM_DEVICE;
  if (tier == DSK_TIER_HOST || tier == DSK_TIER_AUTO) order[n++] = DSK_MEM_HOST_PINNED;
  for (int i = 0; i < n; ++i) {
    const int mem = order[i];
    if (st->used[mem] + bytes > st->cap[mem]) continue;
    void* p = nullptr;
    hipError_t err = mem == DSK_MEM_DEVICE ? hipMalloc(&p, (size_t)bytes) : hipHostMalloc(&p, (size_t)bytes, hipHostMallocDefault);
    if (err != hipSuccess) {
      (void)hipGetLastError();
      continue;
    }
    st->used[mem] += bytes;
    e->base = p; e->mem = mem; e->bytes = bytes;
    return DSK_OK;
  }
  return DSK_ENOMEM;
}

void store_free(dsk_store* st, dsk_store::Entry& e) {
  if (!e.base) return;
  if (e.mem == DSK_MEM_DEVICE) (void)hipFree(e.base);
  else (void)hipHostFree(e.base);
  st->used[e.mem] -= e.bytes;
  e.base = nullptr;
}

hipMemcpyKind copy_kind(int src_mem, int dst_mem) {
  if (src_mem == DSK_MEM_DEVICE) return dst_mem == DSK_MEM_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
  return dst_mem == DSK_MEM_DEVICE ? hipMemcpyHostToDevice : hipMemcpyHostToHost;
}

}  // namespace

extern "C" {

// FNV-1a, 64 bit (offset basis 0xcbf29ce484222325, prime 0x100000001b3)
uint64_t dsk_hash_context(const void* bytes, int64_t n) {
  uint64_t h = 0xcbf29ce484222325ull;
  const unsigned char* p = (const unsigned char*)bytes;
  for (int64_t i = 0; p && i < n; ++i) {
    h ^= p[i];
    h *= 0x100000001b3ull;
  }
  return h;
}

int dsk_store_create(int64_t device_capacity_bytes, int64_t host_capacity_bytes, dsk_store_t** out) {
  if (!out || device_capacity_bytes < 0 || host_capacity_bytes < 0) return DSK_EINVAL;
  dsk_store* st = new (std::nothrow) dsk_store();
  if (!st) return DSK_ENOMEM;
  st->cap[DSK_MEM_DEVICE] = device_capacity_bytes;
  st->cap[DSK_MEM_HOST_PINNED] = host_capacity_bytes;
  *out = st;
  return DSK_OK;
}

int dsk_store_destroy(dsk_store_t* store) {
  if (!store) return DSK_OK;
  for (auto& kv : store->entries) store_free(store, kv.second);
  delete store;
  return DSK_OK;
}

int dsk_store_put_kv(dsk_store_t* store, uint64_t context, uint64_t model_id, const dsk_kv_t* kv, int n_layers,
                     int64_t n_rows, int64_t row_bytes, int tier, void* stream, int* inserted) {
  if (!store || !kv || !kv->base || n_layers < 1 || n_rows < 1 || row_bytes < 1 || (row_bytes & 15)) return DSK_EINVAL;
  if (tier < DSK_TIER_AUTO || tier > DSK_TIER_HOST) return DSK_EINVAL;
  if (kv->mem != DSK_MEM_DEVICE && kv->mem != DSK_MEM_HOST_PINNED) return DSK_EINVAL;
  if (kv->n_rows < n_rows || kv->v_offset < kv->n_rows * row_bytes || kv->layer_stride < kv->v_offset + kv->n_rows * row_bytes)
    return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  const dsk_store::Key key(context, model_id, 0, -1);
  if (inserted) *inserted = 0;
  if (store->entries.count(key)) return DSK_OK;  // an existing (context, model) entry is kept (Sec. 4.4)
  dsk_store::Entry e;
  const int64_t half = n_rows * row_bytes;
  int rc = store_alloc(store, tier, (int64_t)n_layers * 2 * half, &e);
  if (rc) return rc;
  e.n_layers = n_layers; e.n_rows = n_rows; e.row_bytes = row_bytes;
  const hipMemcpyKind kind = copy_kind(kv->mem, e.mem);
  for (int l = 0; l < n_layers; ++l) {
    const char* src = (const char*)kv->base + (int64_t)l * kv->layer_stride;
    char* dst = (char*)e.base + (int64_t)l * 2 * half;
    hipError_t err = hipMemcpyAsync(dst, src, (size_t)half, kind, (hipStream_t)stream);
    if (err == hipSuccess) err = hipMemcpyAsync(dst + half, src + kv->v_offset, (size_t)half, kind, (hipStream_t)stream);
    if (err != hipSuccess) {
      g_last_hip_error = (int)err;
      store_free(store, e);
      return DSK_EHIP;
    }
  }
  store->entries[key] = e;
  if (inserted) *inserted = 1;
  return DSK_OK;
}

int dsk_store_put_e(dsk_store_t* store, uint64_t context, uint64_t model_id, int layer, const void* e_cache, int e_mem,
                    int64_t bytes, int tier, void* stream, int* inserted) {
  if (!store || !e_cache || layer < 0 || bytes < 1) return DSK_EINVAL;
  if (tier < DSK_TIER_AUTO || tier > DSK_TIER_HOST) return DSK_EINVAL;
  if (e_mem != DSK_MEM_DEVICE && e_mem != DSK_MEM_HOST_PINNED) return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  const dsk_store::Key key(context, model_id, 1, layer);
  if (inserted) *inserted = 0;
  if (store->entries.count(key)) return DSK_OK;
  dsk_store::Entry e;
  int rc = store_alloc(store, tier, bytes, &e);
  if (rc) return rc;
  hipError_t err = hipMemcpyAsync(e.base, e_cache, (size_t)bytes, copy_kind(e_mem, e.mem), (hipStream_t)stream);
  if (err != hipSuccess) {
    g_last_hip_error = (int)err;
    store_free(store, e);
    return DSK_EHIP;
  }
  store->entries[key] = e;
  if (inserted) *inserted = 1;
  return DSK_OK;
}

int dsk_store_fetch_kv(dsk_store_t* store, uint64_t context, uint64_t model_id, dsk_kv_t* out, int* n_layers) {
  if (!store || !out) return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  auto it = store->entries.find(dsk_store::Key(context, model_id, 0, -1));
  if (it == store->entries.end()) return DSK_ENOENT;
  const dsk_store::Entry& e = it->second;
  out->base = e.base; out->mem = e.mem; out->n_rows = e.n_rows;
  out->v_offset = e.n_rows * e.row_bytes;
  out->layer_stride = 2 * out->v_offset;
  if (n_layers) *n_layers = e.n_layers;
  return DSK_OK;
}

int dsk_store_fetch_kv_layer(dsk_store_t* store, uint64_t context, uint64_t model_id, int layer, const void** k_rows,
                             const void** v_rows, int* mem, int64_t* bytes_each) {
  if (!store || !k_rows || !v_rows) return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  auto it = store->entries.find(dsk_store::Key(context, model_id, 0, -1));
  if (it == store->entries.end()) return DSK_ENOENT;
  const dsk_store::Entry& e = it->second;
  if (layer < 0 || layer >= e.n_layers) return DSK_EINVAL;
  const int64_t half = e.n_rows * e.row_bytes;
  *k_rows = (const char*)e.base + (int64_t)layer * 2 * half;
  *v_rows = (const char*)*k_rows + half;
  if (mem) *mem = e.mem;
  if (bytes_each) *bytes_each = half;
  return DSK_OK;
}

int dsk_store_fetch_e(dsk_store_t* store, uint64_t context, uint64_t model_id, int layer, const void** e_cache, int* mem,
                      int64_t* bytes) {
  if (!store || !e_cache) return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  auto it = store->entries.find(dsk_store::Key(context, model_id, 1, layer));
  if (it == store->entries.end()) return DSK_ENOENT;
  *e_cache = it->second.base;
  if (mem) *mem = it->second.mem;
  if (bytes) *bytes = it->second.bytes;
  return DSK_OK;
}

int dsk_store_erase(dsk_store_t* store, uint64_t context, uint64_t model_id) {
  if (!store) return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  int n = 0;
  for (auto it = store->entries.begin(); it != store->entries.end();) {
    if (std::get<0>(it->first) == context && std::get<1>(it->first) == model_id) {
      store_free(store, it->second);
      it = store->entries.erase(it);
      ++n;
    } else {
      ++it;
    }
  }
  return n ? DSK_OK : DSK_ENOENT;
}

int dsk_store_usage(dsk_store_t* store, int64_t* device_bytes, int64_t* host_bytes, int64_t* n_entries) {
  if (!store) return DSK_EINVAL;
  std::lock_guard<std::mutex> lock(store->mu);
  if (device_bytes) *device_bytes = store->used[DSK_MEM_DEVICE];
  if (host_bytes) *host_bytes = store->used[DSK_MEM_HOST_PINNED];
  if (n_entries) *n_entries = (int64_t)store->entries.size();
  return DSK_OK;
}

}  // extern "C"
