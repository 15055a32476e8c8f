// C ABI of the library (see include/attncache.h): argument validation, the
// database handle, and the host-side schedule of the pinned-host map path.
// No kernel lives here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <new>
#include <list>
#include <unordered_map>
#include <vector>

#include "../../include/attncache.h"
#include "launch.hpp"

namespace {

thread_local int32_t g_last_hip_error = 0;

int32_t hip_fail(hipError_t e) {
  g_last_hip_error = (int32_t)e;
  (void)hipGetLastError();   // clear the sticky error so later calls are not blamed for it
  return AC_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// 0 = device, 1 = pinned host, -1 = neither / unknown
int memspace(const void* p) {
  hipPointerAttribute_t attr;
  hipError_t e = hipPointerGetAttributes(&attr, p);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return -1;
  }
  if (attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged) return 0;
  if (attr.type == hipMemoryTypeHost) return 1;
  return -1;   // ordinary (unregistered) host memory and anything else
}

// Per-call pointer checks (attncache_set_pointer_checks): on by default.
std::atomic<int32_t> g_pointer_checks{1};

// Whether the memory-space queries below may run for work that goes to `stream`: not when the
// caller switched them off, and not while the stream is being captured into a graph (a capture
// records launches only; the query is skipped rather than risk invalidating the capture).
bool may_query(hipStream_t stream) {
  if (!g_pointer_checks.load(std::memory_order_relaxed)) return false;
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st == hipStreamCaptureStatusNone;
}

// AC_OK when every non-NULL pointer of the list is device memory.
int32_t all_device(std::initializer_list<const void*> ptrs) {
  for (const void* p : ptrs)
    if (p && memspace(p) != 0) return AC_ERR_MEMSPACE;
  return AC_OK;
}

size_t elt_size(int32_t dtype) { return dtype == AC_F32 ? 4 : 2; }

// Search workspace of attncache_search_static: lives in the code object, one copy per GPU the
// library is loaded on, until the process ends.  In host code the NAME of the array is only a
// stand-in; its device address is looked up once per device with hipGetSymbolAddress and that
// pointer is what kernels and copies are given.
__device__ __align__(256) unsigned char scratch[AC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device (looked up on first use; the same value whichever
// thread gets there first).
int32_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return AC_ERR_SHAPE;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!p) return AC_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return AC_OK;
}

int32_t check_desc(const attncache_db_desc* d) {
  if (!d) return AC_ERR_NULL;
  if (d->n_emb < 1 || d->emb_dim < 1 || d->n_entries < 1 || d->n_layers < 1 || d->n_q_heads < 1 ||
      d->n_kv_heads < 1 || d->head_dim < 1 || d->seq_len < 1)
    return AC_ERR_SHAPE;
  if (d->n_q_heads % d->n_kv_heads != 0) return AC_ERR_SHAPE;
  if (d->metric != AC_IP && d->metric != AC_L2) return AC_ERR_DTYPE;
  if (d->emb_dtype == AC_F16) {
    if (d->emb_dim % 8 != 0) return AC_ERR_SHAPE;   // 16-byte rows
  } else if (d->emb_dtype != AC_F32) {
    return AC_ERR_DTYPE;
  }
  if (d->map_dtype == AC_BF16) {
    if (d->seq_len % 32 != 0) return AC_ERR_SHAPE;
    if (d->head_dim != 64 && d->head_dim != 128) return AC_ERR_SHAPE;
  } else if (d->map_dtype == AC_F32) {
    if (d->head_dim > 256) return AC_ERR_SHAPE;
    if (d->map_layout != AC_LAYOUT_DENSE) return AC_ERR_DTYPE;
  } else {
    return AC_ERR_DTYPE;
  }
  if (d->map_layout != AC_LAYOUT_DENSE && d->map_layout != AC_LAYOUT_PACKED) return AC_ERR_DTYPE;
  return AC_OK;
}

size_t entry_bytes_of(const attncache_db_desc* d) {
  const size_t heads = (size_t)d->n_layers * d->n_q_heads;
  if (d->map_layout == AC_LAYOUT_PACKED)
    return heads * (size_t)ac::packed_blocks(d->seq_len, d->causal) * 512 * elt_size(d->map_dtype);
  return heads * d->seq_len * d->seq_len * elt_size(d->map_dtype);
}

}  // namespace

struct attncache_db {
  attncache_db_desc d;
  const void* emb;
  const int32_t* map_of;
  const void* maps;
  // pinned-host path
  unsigned char* staging;
  size_t entry_bytes;
  int n_slots;
  hipStream_t side;
  std::vector<hipEvent_t> copied;     // per slot: host-to-device copy finished
  std::vector<hipEvent_t> consumed;   // per slot: last product reading the slot finished
  std::vector<char> used;             // per slot: consumed[] has been recorded at least once
  // slot cache: which entry (all layers) a slot holds, least recently used slot at the back
  std::vector<int32_t> slot_entry;    // -1: nothing reusable
  std::unordered_map<int32_t, int> where;
  std::list<int> lru;
  std::vector<std::list<int>::iterator> lru_it;
  uint64_t lookups, copies;
};

extern "C" {

int32_t attncache_version(void) { return 1000; }

int32_t attncache_last_hip_error(void) { return g_last_hip_error; }

int32_t attncache_set_pointer_checks(int32_t on) {
  return g_pointer_checks.exchange(on != 0 ? 1 : 0, std::memory_order_relaxed);
}

const char* attncache_status_string(int32_t s) {
  switch (s) {
    case AC_OK: return "ok";
    case AC_ERR_NULL: return "required pointer is NULL";
    case AC_ERR_SHAPE: return "size is non-positive or unsupported";
    case AC_ERR_DTYPE: return "unsupported element type or metric";
    case AC_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case AC_ERR_K_RANGE: return "k outside 1..min(AC_MAX_K, N)";
    case AC_ERR_WORKSPACE: return "workspace or staging buffer too small";
    case AC_ERR_INDEX: return "hit index outside [-1, M)";
    case AC_ERR_HIP: return "HIP call failed";
    case AC_ERR_MEMSPACE: return "pointer is in the wrong memory space";
    case AC_ERR_NOMEM: return "host memory allocation failed";
    default: return "unknown status";
  }
}

int32_t attncache_workspace_bytes(const attncache_db_desc* desc, int32_t max_batch, int32_t k,
                                  size_t* out) {
  if (!out) return AC_ERR_NULL;
  int32_t rc = check_desc(desc);
  if (rc != AC_OK) return rc;
  if (max_batch < 0) return AC_ERR_SHAPE;
  if (k < 1 || k > AC_MAX_K || k > desc->n_emb) return AC_ERR_K_RANGE;
  *out = ac::search_workspace_bytes(desc->n_emb, desc->emb_dim, max_batch, k,
                                    desc->emb_dtype == AC_F16);
  return AC_OK;
}

int32_t attncache_map_entry_bytes(const attncache_db_desc* desc, size_t* out) {
  if (!out) return AC_ERR_NULL;
  int32_t rc = check_desc(desc);
  if (rc != AC_OK) return rc;
  *out = entry_bytes_of(desc);
  return AC_OK;
}

int32_t attncache_pack_maps(const attncache_db_desc* desc, const void* dense, int32_t n_entries,
                            void* packed, void* stream) {
  if (!desc) return AC_ERR_NULL;
  attncache_db_desc d = *desc;
  d.map_layout = AC_LAYOUT_PACKED;
  int32_t rc = check_desc(&d);
  if (rc != AC_OK) return rc;
  if (d.map_dtype != AC_BF16) return AC_ERR_DTYPE;
  if (n_entries < 0) return AC_ERR_SHAPE;
  if (n_entries == 0) return AC_OK;
  if (!dense || !packed) return AC_ERR_NULL;
  if (!aligned16(dense) || !aligned16(packed)) return AC_ERR_ALIGN;
  const int64_t tiles = (int64_t)n_entries * d.n_layers * d.n_q_heads;
  if (tiles > 0x7fffffffLL) return AC_ERR_SHAPE;
  if (may_query(reinterpret_cast<hipStream_t>(stream))) {
    const int32_t rc = all_device({dense, packed});
    if (rc != AC_OK) return rc;
  }
  hipError_t e = ac::launch_pack_maps(dense, packed, tiles, d.seq_len, d.causal != 0,
                                      reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AC_OK : hip_fail(e);
}

int32_t attncache_build_db(const attncache_db_desc* desc, const void* emb, const int32_t* map_of,
                           const void* maps, void* staging, size_t staging_bytes,
                           void* side_stream, attncache_db** out) {
  if (!out) return AC_ERR_NULL;
  *out = nullptr;
  int32_t rc = check_desc(desc);
  if (rc != AC_OK) return rc;
  if (!emb || !maps) return AC_ERR_NULL;
  if (!map_of && desc->n_emb != desc->n_entries) return AC_ERR_SHAPE;
  if (!aligned16(emb) || !aligned16(maps) || (map_of && !aligned16(map_of))) return AC_ERR_ALIGN;
  if (memspace(emb) != 0) return AC_ERR_MEMSPACE;
  if (map_of && memspace(map_of) != 0) return AC_ERR_MEMSPACE;
  if (memspace(maps) != (desc->maps_on_host ? 1 : 0)) return AC_ERR_MEMSPACE;

  attncache_db* db = new (std::nothrow) attncache_db();
  if (!db) return AC_ERR_NOMEM;
  db->d = *desc;
  db->emb = emb;
  db->map_of = map_of;
  db->maps = maps;
  db->staging = nullptr;
  db->n_slots = 0;
  db->lookups = db->copies = 0;
  db->side = nullptr;
  db->entry_bytes = entry_bytes_of(desc);
  if (desc->maps_on_host) {
    int32_t bad = AC_OK;
    if (!staging) bad = AC_ERR_NULL;
    else if (!aligned16(staging)) bad = AC_ERR_ALIGN;
    else if (memspace(staging) != 0) bad = AC_ERR_MEMSPACE;
    else if (staging_bytes / db->entry_bytes < 2) bad = AC_ERR_WORKSPACE;
    if (bad != AC_OK) { delete db; return bad; }
    db->staging = reinterpret_cast<unsigned char*>(staging);
    db->n_slots = (int)std::min<size_t>(staging_bytes / db->entry_bytes, 1 << 16);
    db->side = reinterpret_cast<hipStream_t>(side_stream);
    hipError_t e = hipSuccess;
    try {   // the containers allocate host memory; nothing may leave an extern "C" function
      db->copied.reserve(db->n_slots);
      db->consumed.reserve(db->n_slots);
      db->used.assign(db->n_slots, 0);
      db->slot_entry.assign(db->n_slots, -1);
      db->where.reserve(db->n_slots);
      db->lru_it.resize(db->n_slots);
      for (int i = 0; i < db->n_slots; ++i) db->lru_it[i] = db->lru.insert(db->lru.end(), i);
      for (int i = 0; i < db->n_slots && e == hipSuccess; ++i) {
        hipEvent_t ev;
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) break;
        db->copied.push_back(ev);
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) break;
        db->consumed.push_back(ev);
      }
    } catch (...) {
      (void)attncache_destroy_db(db);
      return AC_ERR_NOMEM;
    }
    if (e != hipSuccess) {
      (void)attncache_destroy_db(db);   // destroys the events created so far
      return hip_fail(e);
    }
  }
  // set-up is the place to resolve the static search workspace of this device: a first
  // attncache_search_static may then come from a caller that is capturing a graph
  void* unused = nullptr;
  (void)static_scratch(&unused);
  *out = db;
  return AC_OK;
}

int32_t attncache_destroy_db(attncache_db* db) {
  if (!db) return AC_ERR_NULL;
  for (hipEvent_t ev : db->copied) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : db->consumed) (void)hipEventDestroy(ev);
  delete db;
  return AC_OK;
}

int32_t attncache_search(const attncache_db* db, const void* q, int32_t B, int32_t k,
                         float threshold, int32_t* idx, float* score, int32_t* hit, void* ws,
                         size_t ws_bytes, void* stream) {
  if (!db) return AC_ERR_NULL;
  if (B < 0) return AC_ERR_SHAPE;
  if (k < 1 || k > AC_MAX_K || k > db->d.n_emb) return AC_ERR_K_RANGE;
  if (B == 0) return AC_OK;
  if (!q || !idx || !score || !hit || !ws) return AC_ERR_NULL;
  if (!aligned16(q) || !aligned16(ws)) return AC_ERR_ALIGN;
  const size_t need = ac::search_workspace_bytes(db->d.n_emb, db->d.emb_dim, B, k,
                                                 db->d.emb_dtype == AC_F16);
  if (ws_bytes < need) return AC_ERR_WORKSPACE;
  if (may_query(reinterpret_cast<hipStream_t>(stream))) {
    const int32_t rc = all_device({q, idx, score, hit, ws});
    if (rc != AC_OK) return rc;
  }
  ac::SearchLaunch p;
  p.emb = db->emb; p.q = q; p.map_of = db->map_of;
  p.N = db->d.n_emb; p.E = db->d.emb_dim; p.B = B; p.k = k;
  p.is_f16 = db->d.emb_dtype == AC_F16; p.metric = db->d.metric;
  p.threshold = threshold;
  p.idx = idx; p.score = score; p.hit = hit;
  p.ws = ws; p.ws_bytes = ws_bytes;
  hipError_t e = ac::launch_search(p, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AC_OK : hip_fail(e);
}

int32_t attncache_search_static(const attncache_db* db, const void* q, int32_t B, int32_t k,
                                float threshold, int32_t* idx, float* score, int32_t* hit,
                                void* stream) {
  if (!db) return AC_ERR_NULL;
  if (B < 0) return AC_ERR_SHAPE;
  if (k < 1 || k > AC_MAX_K || k > db->d.n_emb) return AC_ERR_K_RANGE;
  if (B == 0) return AC_OK;
  const size_t need = ac::search_workspace_bytes(db->d.n_emb, db->d.emb_dim, B, k,
                                                 db->d.emb_dtype == AC_F16);
  if (need > (size_t)AC_STATIC_SCRATCH_BYTES) return AC_ERR_WORKSPACE;
  void* ws = nullptr;
  int32_t rc = static_scratch(&ws);
  if (rc != AC_OK) return rc;
  return attncache_search(db, q, B, k, threshold, idx, score, hit, ws, AC_STATIC_SCRATCH_BYTES,
                          stream);
}

int32_t attncache_apply(const attncache_db* cdb, const int32_t* hit, const void* V, void* O,
                        int32_t B, int32_t layer_begin, int32_t layer_count, void* stream_) {
  attncache_db* db = const_cast<attncache_db*>(cdb);   // slot bookkeeping of the host path
  if (!db) return AC_ERR_NULL;
  const attncache_db_desc& d = db->d;
  if (B < 0 || layer_begin < 0 || layer_count < 0 || layer_begin + layer_count > d.n_layers)
    return AC_ERR_SHAPE;
  if (B == 0 || layer_count == 0) return AC_OK;
  if (!hit || !V || !O) return AC_ERR_NULL;
  if (!aligned16(V) || !aligned16(O)) return AC_ERR_ALIGN;
  hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);
  const bool query = may_query(stream);
  if (query) {
    const int32_t rc = all_device({V, O});
    if (rc != AC_OK) return rc;
    // hit is read by the kernel (device-resident maps) or by this function (host-resident)
    const int hs = memspace(hit);
    if (d.maps_on_host ? hs == 0 : hs != 0) return AC_ERR_MEMSPACE;
  }

  ac::ApplyLaunch p;
  p.V = V; p.O = O; p.B = B; p.M = d.n_entries; p.L = d.n_layers;
  p.layer_begin = layer_begin; p.Lc = layer_count;
  p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.S = d.seq_len; p.D = d.head_dim;
  p.causal = d.causal; p.is_f32 = d.map_dtype == AC_F32;
  p.packed = d.map_layout == AC_LAYOUT_PACKED;
  p.n_list = 0;

  if (!d.maps_on_host) {
    p.maps = db->maps; p.hit = hit; p.fixed_entry = -1;
    hipError_t e = ac::launch_apply(p, stream);
    return e == hipSuccess ? AC_OK : hip_fail(e);
  }

  // Pinned-host maps: at most one host-to-device copy per distinct entry on the side stream
  // (none when the entry is still in the ring from an earlier batch), the products of all
  // queries sharing that entry on the caller's stream as soon as the copy has landed.  A slot
  // is overwritten only after the products that read it are done.
  for (int32_t b = 0; b < B; ++b)
    if (hit[b] < -1 || hit[b] >= d.n_entries) return AC_ERR_INDEX;
  try {   // the containers below allocate host memory; nothing may leave an extern "C" function
    std::vector<std::pair<int32_t, int32_t>> order;   // (entry, query), grouped by entry
    order.reserve(B);
    for (int32_t b = 0; b < B; ++b)
      if (hit[b] >= 0) order.emplace_back(hit[b], b);
    std::stable_sort(order.begin(), order.end(),
                     [](const auto& x, const auto& y) { return x.first < y.first; });
    const size_t layer_bytes = db->entry_bytes / d.n_layers;
    const size_t copy_bytes = layer_bytes * layer_count;
    // Slot cache: an entry that a previous batch (or an earlier group of this one) left in the
    // ring is used where it lies; otherwise the least recently used slot is overwritten.  Only
    // whole entries (all layers) are remembered.
    const bool whole = layer_begin == 0 && layer_count == d.n_layers;
    // Groups of queries that share an entry.  Entries that are still cached from earlier calls
    // are served first (their products start at once, under the copies of the others, and they
    // are touched before anything is replaced, so a batch never evicts what it is about to
    // use), then the rest; ascending entry inside each class.
    struct Group { int32_t entry; size_t pos, end; };
    std::vector<Group> groups;
    groups.reserve(order.size());
    for (size_t pos = 0; pos < order.size();) {
      size_t end = pos;
      while (end < order.size() && order[end].first == order[pos].first) ++end;
      groups.push_back({order[pos].first, pos, end});
      pos = end;
    }
    if (whole)
      std::stable_partition(groups.begin(), groups.end(), [&](const Group& gr) {
        return db->where.find(gr.entry) != db->where.end();
      });
    for (const Group& gr : groups) {
      const int32_t entry = gr.entry;
      const size_t pos = gr.pos, end = gr.end;
      ++db->lookups;
      int slot = -1;
      if (whole) {
        auto it = db->where.find(entry);
        if (it != db->where.end()) slot = it->second;
      }
      const bool cached = slot >= 0;
      hipError_t e = hipSuccess;
      if (!cached) {
        // The slot's old contents are given up BEFORE the copy is enqueued and the new entry is
        // published only AFTER copy and event are: if a HIP call fails in between, the slot
        // names nothing and no later call can mistake it for a filled one.
        slot = db->lru.back();
        if (db->slot_entry[slot] >= 0) {
          db->where.erase(db->slot_entry[slot]);
          db->slot_entry[slot] = -1;
        }
        ++db->copies;
        const unsigned char* src = reinterpret_cast<const unsigned char*>(db->maps) +
                                   (size_t)entry * db->entry_bytes + (size_t)layer_begin * layer_bytes;
        unsigned char* to = db->staging + (size_t)slot * db->entry_bytes;
        if (db->used[slot]) e = hipStreamWaitEvent(db->side, db->consumed[slot], 0);
        if (e == hipSuccess) e = hipMemcpyAsync(to, src, copy_bytes, hipMemcpyHostToDevice, db->side);
        if (e == hipSuccess) e = hipEventRecord(db->copied[slot], db->side);
        if (e != hipSuccess) return hip_fail(e);
        if (whole) {
          db->where[entry] = slot;
          db->slot_entry[slot] = entry;
        }
      }
      db->lru.splice(db->lru.begin(), db->lru, db->lru_it[slot]);   // most recently used
      unsigned char* dst = db->staging + (size_t)slot * db->entry_bytes;
      e = hipStreamWaitEvent(stream, db->copied[slot], 0);
      // the staged block holds layers [layer_begin, layer_begin + layer_count) only
      p.maps = dst; p.hit = nullptr; p.fixed_entry = 0; p.L = layer_count; p.layer_begin = 0;
      for (size_t q0 = pos; q0 < end && e == hipSuccess; q0 += 32) {
        p.n_list = (int32_t)std::min<size_t>(32, end - q0);
        for (int i = 0; i < p.n_list; ++i) p.q_list[i] = order[q0 + i].second;
        e = ac::launch_apply(p, stream);
      }
      // readers may have been enqueued even when a later launch failed: the slot's next
      // overwrite must wait for them either way
      const hipError_t e2 = hipEventRecord(db->consumed[slot], stream);
      if (e2 == hipSuccess) db->used[slot] = 1;
      if (e != hipSuccess) return hip_fail(e);
      if (e2 != hipSuccess) return hip_fail(e2);
    }
  } catch (...) {
    return AC_ERR_NOMEM;
  }
  return AC_OK;
}

int32_t attncache_cache_stats(const attncache_db* db, uint64_t* lookups, uint64_t* copies) {
  if (!db || !lookups || !copies) return AC_ERR_NULL;
  *lookups = db->lookups;
  *copies = db->copies;
  return AC_OK;
}

int32_t attncache_cache_reset(attncache_db* db) {
  if (!db) return AC_ERR_NULL;
  db->where.clear();
  std::fill(db->slot_entry.begin(), db->slot_entry.end(), -1);
  db->lookups = db->copies = 0;
  return AC_OK;
}

int32_t attention_exact(const void* Q, const void* K, const void* V, void* O,
                        const int32_t* row_sel, const int32_t* key_len, int32_t B, int32_t Hq,
                        int32_t Hkv, int32_t S, int32_t D, int32_t dtype, int32_t causal,
                        float scale, void* stream) {
  if (B < 0 || Hq < 1 || Hkv < 1 || S < 1 || D < 1 || Hq % Hkv != 0) return AC_ERR_SHAPE;
  if (dtype == AC_BF16) {
    if (S % 32 != 0 || (D != 64 && D != 128)) return AC_ERR_SHAPE;
  } else if (dtype == AC_F32) {
    if (D > 256) return AC_ERR_SHAPE;
  } else {
    return AC_ERR_DTYPE;
  }
  if (!(scale >= 0.f)) return AC_ERR_SHAPE;
  if (B == 0) return AC_OK;
  if (!Q || !K || !V || !O) return AC_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return AC_ERR_ALIGN;
  if (may_query(reinterpret_cast<hipStream_t>(stream))) {
    const int32_t rc = all_device({Q, K, V, O, row_sel, key_len});
    if (rc != AC_OK) return rc;
  }
  ac::ExactLaunch p;
  p.Q = Q; p.K = K; p.V = V; p.O = O; p.row_sel = row_sel; p.key_len = key_len;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.S = S; p.D = D;
  p.causal = causal != 0; p.is_f32 = dtype == AC_F32; p.scale = scale;
  hipError_t e = ac::launch_exact(p, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AC_OK : hip_fail(e);
}

int32_t attncache_insert(attncache_db* db, const void* feat, const int32_t* slot,
                         const int32_t* row_sel, const int32_t* key_len, const void* Q,
                         const void* K, const void* V, void* O, int32_t B, int32_t layer_begin,
                         int32_t layer_count, float scale, void* stream) {
  if (!db) return AC_ERR_NULL;
  const attncache_db_desc& d = db->d;
  if (B < 0 || layer_begin < 0 || layer_count < 0 || layer_begin + layer_count > d.n_layers)
    return AC_ERR_SHAPE;
  if (d.map_dtype != AC_BF16) return AC_ERR_DTYPE;
  if (d.maps_on_host) return AC_ERR_MEMSPACE;
  // a slot names a map entry AND a feature row: the two stores must share one index
  if (feat && (db->map_of || d.n_emb != d.n_entries)) return AC_ERR_SHAPE;
  const size_t esz = d.emb_dtype == AC_F16 ? 2 : 4;
  if (feat && (d.emb_dim * esz) % 16 != 0) return AC_ERR_SHAPE;
  if (!(scale >= 0.f)) return AC_ERR_SHAPE;
  if (B == 0 || layer_count == 0) return AC_OK;
  if (!Q || !K || !V || !O) return AC_ERR_NULL;
  if (feat && !slot) return AC_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(feat))
    return AC_ERR_ALIGN;
  if (may_query(reinterpret_cast<hipStream_t>(stream))) {
    const int32_t rc = all_device({Q, K, V, O, feat, slot, row_sel, key_len});
    if (rc != AC_OK) return rc;
  }
  ac::InsertLaunch p;
  p.Q = Q; p.K = K; p.V = V; p.O = O;
  p.maps = const_cast<void*>(db->maps);   // the one entry point that writes the borrowed stores
  p.feat = feat; p.emb = const_cast<void*>(db->emb);
  p.slot = slot; p.row_sel = row_sel; p.key_len = key_len;
  p.B = B; p.M = d.n_entries; p.L = d.n_layers; p.layer_begin = layer_begin; p.Lc = layer_count;
  p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.S = d.seq_len; p.D = d.head_dim;
  p.causal = d.causal != 0; p.packed = d.map_layout == AC_LAYOUT_PACKED;
  p.emb_row_bytes = (int32_t)(d.emb_dim * esz);
  p.scale = scale;
  hipError_t e = ac::launch_insert(p, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AC_OK : hip_fail(e);
}

size_t attncache_project_workspace_bytes(int32_t B, int32_t model_dim, int32_t hidden_dim,
                                         int32_t emb_dim) {
  if (B < 1 || model_dim < 1 || hidden_dim < 1 || emb_dim < 1) return 0;
  return ac::project_workspace_bytes(B, model_dim, hidden_dim, emb_dim);
}

int32_t attncache_project(const void* h, const int32_t* seq_len, const float* W1, const float* b1,
                          const float* W2, const float* b2, void* feat, int32_t B, int32_t S,
                          int32_t model_dim, int32_t hidden_dim, int32_t emb_dim, int32_t h_dtype,
                          int32_t feat_dtype, int32_t normalize, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (B < 0 || B > 65535 || S < 1 || model_dim < 8 || hidden_dim < 8 || emb_dim < 8)
    return AC_ERR_SHAPE;
  if (model_dim % 8 != 0 || hidden_dim % 8 != 0 || emb_dim % 8 != 0 || emb_dim > 2048)
    return AC_ERR_SHAPE;
  if (h_dtype != AC_BF16 && h_dtype != AC_F32) return AC_ERR_DTYPE;
  if (feat_dtype != AC_F16 && feat_dtype != AC_F32) return AC_ERR_DTYPE;
  if (B == 0) return AC_OK;
  if (!h || !W1 || !W2 || !feat || !workspace) return AC_ERR_NULL;
  if (!aligned16(h) || !aligned16(W1) || !aligned16(b1) || !aligned16(W2) || !aligned16(b2) ||
      !aligned16(feat) || !aligned16(workspace))
    return AC_ERR_ALIGN;
  if (workspace_bytes < ac::project_workspace_bytes(B, model_dim, hidden_dim, emb_dim))
    return AC_ERR_WORKSPACE;
  if (may_query(reinterpret_cast<hipStream_t>(stream))) {
    const int32_t rc = all_device({h, seq_len, W1, b1, W2, b2, feat, workspace});
    if (rc != AC_OK) return rc;
  }
  ac::ProjectLaunch p;
  p.h = h; p.seq_len = seq_len; p.W1 = W1; p.b1 = b1; p.W2 = W2; p.b2 = b2;
  p.feat = feat; p.ws = workspace;
  p.B = B; p.S = S; p.dm = model_dim; p.hid = hidden_dim; p.E = emb_dim;
  p.h_is_f32 = h_dtype == AC_F32; p.feat_is_f16 = feat_dtype == AC_F16;
  p.normalize = normalize != 0;
  hipError_t e = ac::launch_project(p, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? AC_OK : hip_fail(e);
}

}  // extern "C"
