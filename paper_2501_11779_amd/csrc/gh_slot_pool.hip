// Context slots backed by HIP virtual memory management: a virtual range per cache, a fixed
// budget of physical pages, pages mapped under a slot as its sequence grows.
// Contract: include/gh_slot_pool.h.
#include "gh_slot_pool.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

namespace {
constexpr int32_t kOk = 0, kNull = -1, kShape = -2, kUnsupported = -3, kCapacity = -5, kHip = -6;
}

struct gh_slot_pool {
  gh_slot_pool_config cfg;
  int32_t capacity = 0;            // rows per slot, whole pages
  int32_t pages_per_slot = 0;
  size_t page_bytes = 0, slot_bytes = 0, range_bytes = 0;
  char* k_va = nullptr;
  char* v_va = nullptr;
  std::vector<hipMemGenericAllocationHandle_t> k_pages, v_pages;   // physical pages
  std::vector<int32_t> free_list;                                  // ids of unmapped pages
  std::vector<std::vector<int32_t>> slot_pages;                    // per slot, in row order
  int64_t mapped = 0;
  int64_t created = 0;             // physical pages created so far (on demand, up to the budget)
  hipMemAllocationProp prop = {};
  // host-only pools (gh_slot_pool_create_host_only): the bookkeeping with no GPU behind it
  bool host_only = false;
  int64_t fail_at = -1, map_calls = 0;
};

namespace {

// Restores the caller's current device when it goes out of scope.
struct DeviceGuard {
  int saved = -1;
  DeviceGuard() { if (hipGetDevice(&saved) != hipSuccess) saved = -1; }
  ~DeviceGuard() { if (saved >= 0) (void)hipSetDevice(saved); }
};

// A physical page for the free list: one already created, or a new one while the budget lasts.
// Returns its id, or -1.
int32_t take_page(gh_slot_pool* p) {
  if (!p->free_list.empty()) {
    const int32_t page = p->free_list.back();
    p->free_list.pop_back();
    return page;
  }
  if (p->created >= p->cfg.physical_pages) return -1;
  if (!p->host_only) {
    hipMemGenericAllocationHandle_t hk, hv;
    if (hipMemCreate(&hk, p->page_bytes, &p->prop, 0) != hipSuccess) return -1;
    if (hipMemCreate(&hv, p->page_bytes, &p->prop, 0) != hipSuccess) {
      (void)hipMemRelease(hk);
      return -1;
    }
    p->k_pages.push_back(hk);
    p->v_pages.push_back(hv);
  }
  return (int32_t)p->created++;
}

bool map_page(gh_slot_pool* p, int32_t slot, int32_t index, int32_t page) {
  if (p->host_only) return p->map_calls++ != p->fail_at;
  const size_t off = (size_t)slot * p->slot_bytes + (size_t)index * p->page_bytes;
  hipMemAccessDesc acc = {};
  acc.location.type = hipMemLocationTypeDevice;
  acc.location.id = p->cfg.device;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  if (hipMemMap(p->k_va + off, p->page_bytes, 0, p->k_pages[page], 0) != hipSuccess) return false;
  if (hipMemMap(p->v_va + off, p->page_bytes, 0, p->v_pages[page], 0) != hipSuccess) {
    (void)hipMemUnmap(p->k_va + off, p->page_bytes);
    return false;
  }
  if (hipMemSetAccess(p->k_va + off, p->page_bytes, &acc, 1) != hipSuccess ||
      hipMemSetAccess(p->v_va + off, p->page_bytes, &acc, 1) != hipSuccess) {
    (void)hipMemUnmap(p->k_va + off, p->page_bytes);
    (void)hipMemUnmap(p->v_va + off, p->page_bytes);
    return false;
  }
  return true;
}

bool unmap_page(gh_slot_pool* p, int32_t slot, int32_t index) {
  if (p->host_only) return true;
  const size_t off = (size_t)slot * p->slot_bytes + (size_t)index * p->page_bytes;
  const bool a = hipMemUnmap(p->k_va + off, p->page_bytes) == hipSuccess;
  const bool b = hipMemUnmap(p->v_va + off, p->page_bytes) == hipSuccess;
  return a && b;
}

}  // namespace

extern "C" {

namespace {
int32_t check_config(const gh_slot_pool_config* cfg, gh_slot_pool** out) {
  if (!cfg || !out) return kNull;
  *out = nullptr;
  if (cfg->n_slots <= 0 || cfg->slot_capacity <= 0 || cfg->n_kv_heads <= 0 || cfg->page_rows <= 0 ||
      cfg->physical_pages <= 0 || cfg->device < 0)
    return kShape;
  if (cfg->head_dim != 128) return kUnsupported;
  if (cfg->layout != GH_POOL_TOKEN_MAJOR && cfg->layout != GH_POOL_HEAD_BLOCKED) return kUnsupported;
  if (cfg->layout == GH_POOL_HEAD_BLOCKED &&
      (cfg->page_rows < 32 || (cfg->page_rows & (cfg->page_rows - 1)) != 0))
    return kUnsupported;
  return kOk;
}
void set_geometry(gh_slot_pool* p, const gh_slot_pool_config* cfg) {
  p->cfg = *cfg;
  p->page_bytes = (size_t)cfg->page_rows * cfg->n_kv_heads * cfg->head_dim * 2;
  p->pages_per_slot = (cfg->slot_capacity + cfg->page_rows - 1) / cfg->page_rows;
  p->capacity = p->pages_per_slot * cfg->page_rows;
  p->slot_bytes = (size_t)p->pages_per_slot * p->page_bytes;
  p->range_bytes = (size_t)cfg->n_slots * p->slot_bytes;
  p->slot_pages.resize(cfg->n_slots);
}
}  // namespace

int32_t gh_slot_pool_create(const gh_slot_pool_config* cfg, gh_slot_pool** out) {
  const int32_t st = check_config(cfg, out);
  if (st != kOk) return st;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || cfg->device >= n_dev) return kHip;
  DeviceGuard keep_callers_device;
  if (hipSetDevice(cfg->device) != hipSuccess) return kHip;
  int vmm = 0;
  if (hipDeviceGetAttribute(&vmm, hipDeviceAttributeVirtualMemoryManagementSupported, cfg->device) !=
          hipSuccess || !vmm)
    return kUnsupported;

  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = cfg->device;
  size_t gran = 0;
  if (hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum) != hipSuccess ||
      gran == 0)
    return kHip;

  gh_slot_pool* p = new (std::nothrow) gh_slot_pool();
  if (!p) return kHip;
  set_geometry(p, cfg);
  p->prop = prop;
  if (p->page_bytes % gran != 0) {
    delete p;
    return kUnsupported;
  }
  void* kv = nullptr;
  void* vv = nullptr;
  if (hipMemAddressReserve(&kv, p->range_bytes, gran, nullptr, 0) != hipSuccess) {
    delete p;
    return kHip;
  }
  if (hipMemAddressReserve(&vv, p->range_bytes, gran, nullptr, 0) != hipSuccess) {
    (void)hipMemAddressFree(kv, p->range_bytes);
    delete p;
    return kHip;
  }
  p->k_va = static_cast<char*>(kv);
  p->v_va = static_cast<char*>(vv);
  // physical pages are created when a reservation first needs them, up to cfg->physical_pages
  *out = p;
  return kOk;
}

int32_t gh_slot_pool_create_host_only(const gh_slot_pool_config* cfg, int64_t fail_at,
                                      gh_slot_pool** out) {
  const int32_t st = check_config(cfg, out);
  if (st != kOk) return st;
  gh_slot_pool* p = new (std::nothrow) gh_slot_pool();
  if (!p) return kHip;
  set_geometry(p, cfg);
  p->host_only = true;
  p->fail_at = fail_at;
  *out = p;
  return kOk;
}

int32_t gh_slot_pool_destroy(gh_slot_pool* p) {
  if (!p) return kNull;
  bool ok = true;
  for (int32_t s = 0; s < (int32_t)p->slot_pages.size(); ++s)
    for (int32_t i = 0; i < (int32_t)p->slot_pages[s].size(); ++i) ok = unmap_page(p, s, i) && ok;
  for (auto h : p->k_pages) ok = hipMemRelease(h) == hipSuccess && ok;
  for (auto h : p->v_pages) ok = hipMemRelease(h) == hipSuccess && ok;
  if (p->k_va) ok = hipMemAddressFree(p->k_va, p->range_bytes) == hipSuccess && ok;
  if (p->v_va) ok = hipMemAddressFree(p->v_va, p->range_bytes) == hipSuccess && ok;
  delete p;
  return ok ? kOk : kHip;
}

void* gh_slot_pool_k(const gh_slot_pool* p) { return p ? p->k_va : nullptr; }
void* gh_slot_pool_v(const gh_slot_pool* p) { return p ? p->v_va : nullptr; }

int32_t gh_slot_pool_strides(const gh_slot_pool* p, int64_t* slot_stride, int64_t* head_stride,
                             int64_t* row_stride) {
  if (!p || !slot_stride || !head_stride || !row_stride) return kNull;
  if (p->cfg.layout == GH_POOL_HEAD_BLOCKED) {
    *row_stride = p->cfg.head_dim;
    *head_stride = (int64_t)p->cfg.page_rows * p->cfg.head_dim;
  } else {
    *row_stride = (int64_t)p->cfg.n_kv_heads * p->cfg.head_dim;
    *head_stride = p->cfg.head_dim;
  }
  *slot_stride = (int64_t)p->capacity * p->cfg.n_kv_heads * p->cfg.head_dim;
  return kOk;
}

int32_t gh_slot_pool_blocks(const gh_slot_pool* p, int32_t* block_rows, int64_t* block_stride) {
  if (!p || !block_rows || !block_stride) return kNull;
  const bool blocked = p->cfg.layout == GH_POOL_HEAD_BLOCKED;
  *block_rows = blocked ? p->cfg.page_rows : 0;
  *block_stride = blocked ? (int64_t)p->cfg.page_rows * p->cfg.n_kv_heads * p->cfg.head_dim : 0;
  return kOk;
}

int32_t gh_slot_pool_reserve(gh_slot_pool* p, const int32_t* slot_id, const int32_t* rows,
                             int32_t count) {
  if (!p || (count > 0 && (!slot_id || !rows))) return kNull;
  if (count < 0) return kShape;
  // First pass: is the whole request satisfiable?  (A slot listed twice counts its larger need.)
  std::vector<int32_t> want(p->slot_pages.size(), 0);
  for (int32_t i = 0; i < count; ++i) {
    if (slot_id[i] < 0 || slot_id[i] >= p->cfg.n_slots || rows[i] < 0) return kShape;
    if (rows[i] > p->capacity) return kCapacity;
    const int32_t need = (rows[i] + p->cfg.page_rows - 1) / p->cfg.page_rows;
    if (need > want[slot_id[i]]) want[slot_id[i]] = need;
  }
  int64_t extra = 0;
  for (size_t s = 0; s < want.size(); ++s) {
    const int32_t have = (int32_t)p->slot_pages[s].size();
    if (want[s] > have) extra += want[s] - have;
  }
  if (extra > (int64_t)p->free_list.size() + (p->cfg.physical_pages - p->created)) return kCapacity;
  // Second pass: map.  If the runtime refuses a page midway, everything this call mapped is taken
  // back, so that the request either holds in full or has changed nothing.
  std::vector<int32_t> touched;                                  // slot of every page mapped here
  bool ok = true;
  for (size_t s = 0; s < want.size() && ok; ++s) {
    while ((int32_t)p->slot_pages[s].size() < want[s]) {
      const int32_t page = take_page(p);
      if (page < 0 || !map_page(p, (int32_t)s, (int32_t)p->slot_pages[s].size(), page)) {
        if (page >= 0) p->free_list.push_back(page);
        ok = false;
        break;
      }
      p->slot_pages[s].push_back(page);
      touched.push_back((int32_t)s);
      ++p->mapped;
    }
  }
  if (ok) return kOk;
  for (size_t i = touched.size(); i-- > 0;) {
    auto& pages = p->slot_pages[touched[i]];
    (void)unmap_page(p, touched[i], (int32_t)pages.size() - 1);
    p->free_list.push_back(pages.back());
    pages.pop_back();
    --p->mapped;
  }
  return kHip;
}

int32_t gh_slot_pool_release(gh_slot_pool* p, const int32_t* slot_id, int32_t count) {
  if (!p || (count > 0 && !slot_id)) return kNull;
  if (count < 0) return kShape;
  for (int32_t i = 0; i < count; ++i)
    if (slot_id[i] < 0 || slot_id[i] >= p->cfg.n_slots) return kShape;
  bool ok = true;
  for (int32_t i = 0; i < count; ++i) {
    auto& pages = p->slot_pages[slot_id[i]];
    while (!pages.empty()) {
      ok = unmap_page(p, slot_id[i], (int32_t)pages.size() - 1) && ok;
      p->free_list.push_back(pages.back());
      pages.pop_back();
      --p->mapped;
    }
  }
  return ok ? kOk : kHip;
}

int32_t gh_slot_pool_mapped_rows(const gh_slot_pool* p, int32_t slot) {
  if (!p || slot < 0 || slot >= p->cfg.n_slots) return 0;
  return (int32_t)p->slot_pages[slot].size() * p->cfg.page_rows;
}

int32_t gh_slot_pool_get_stats(const gh_slot_pool* p, gh_slot_pool_stats* out) {
  if (!p || !out) return kNull;
  out->page_bytes = (int64_t)p->page_bytes;
  out->virtual_bytes = 2 * (int64_t)p->range_bytes;
  out->physical_bytes = 2 * p->cfg.physical_pages * (int64_t)p->page_bytes;
  out->pages_total = p->cfg.physical_pages;
  out->pages_created = p->created;
  out->pages_mapped = p->mapped;
  out->slot_capacity = p->capacity;
  int32_t used = 0;
  for (const auto& s : p->slot_pages) used += s.empty() ? 0 : 1;
  out->slots_in_use = used;
  return kOk;
}

}  // extern "C"
