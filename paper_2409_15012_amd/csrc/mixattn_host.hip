// Host side of libmixattn: descriptor validation, cache/writer resolution, length bookkeeping, launch planning.
// Public interface and argument contracts: include/mixattn.h.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <new>

#include "mixattn_internal.h"

using namespace mixattn;

namespace {

thread_local int g_last_hip = 0;

inline bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  g_last_hip = (int)e;
  return false;
}
#define HIP_TRY(expr)                          \
  do {                                         \
    if (!hip_ok(expr)) return MIXATTN_ERR_HIP; \
  } while (0)

inline int elem_bytes(int dt) { return dt == MIXATTN_F32 ? 4 : 2; }

inline bool use_tiled(int kv_dtype, int D, int G) { return kv_dtype == MIXATTN_BF16 && D == kTiledDim && G <= kMaxGroup; }

// testing aid (MIXATTN_PARAM_TEST_FAIL_ALLOC): > 0 counts device allocations down, the one that reaches 0 fails
thread_local int64_t g_fail_alloc_in = 0;

int dev_alloc(void** p, size_t bytes) {
  *p = nullptr;
  if (bytes == 0) bytes = 16;
  if (g_fail_alloc_in > 0 && --g_fail_alloc_in == 0) return MIXATTN_ERR_ALLOC;
  hipError_t e = hipMalloc(p, bytes);
  if (e == hipErrorOutOfMemory) {
    g_last_hip = (int)e;
    (void)hipGetLastError();
    return MIXATTN_ERR_ALLOC;
  }
  if (!hip_ok(e)) return MIXATTN_ERR_HIP;
  return MIXATTN_OK;
}

int upload(void* dst, const void* src, size_t bytes) {
  HIP_TRY(hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice));
  return MIXATTN_OK;
}

void free_stage(Stage& st) {
  void* ptrs[] = {st.K, st.V, st.d_base, st.d_slots, st.d_done};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  st = Stage();
}

void free_layout(mixattn_layout* L) {
  if (!L) return;
  for (auto& c : L->caches) {
    if (c.K) (void)hipFree(c.K);
    if (c.V) (void)hipFree(c.V);
    if (c.d_base) (void)hipFree(c.d_base);
    if (c.d_slots) (void)hipFree(c.d_slots);
    if (c.d_pages) (void)hipFree(c.d_pages);
    free_stage(c.own_stage);
  }
  void* ptrs[] = {L->d_lens_all, L->d_arrive_all, L->scratch.acc, L->scratch.ml,
                  L->d_stage_lens, L->d_stage_src, L->d_readback, L->d_q_first, L->d_q_len};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  delete L;
}

}  // namespace

extern "C" {

const char* mixattn_version(void) { return "mixattn 0.1 (gfx950)"; }
int mixattn_last_hip_error(void) { return g_last_hip; }

const char* mixattn_strerror(int st) {
  switch (st) {
    case MIXATTN_OK: return "ok";
    case MIXATTN_ERR_NULL: return "required pointer is NULL";
    case MIXATTN_ERR_LAYOUT: return "invalid layout descriptor";
    case MIXATTN_ERR_LAYER: return "index out of range";
    case MIXATTN_ERR_NOT_WRITER: return "layer reads a shared cache and cannot write it";
    case MIXATTN_ERR_CAPACITY: return "full cache capacity exceeded";
    case MIXATTN_ERR_ORDER: return "call not valid in the current cache state";
    case MIXATTN_ERR_ALLOC: return "allocation failed";
    case MIXATTN_ERR_HIP: return "HIP runtime error";
    case MIXATTN_ERR_PARAM: return "bad tuning parameter";
    case MIXATTN_ERR_SCRATCH: return "the call needs more split-K scratch than the static area holds";
    default: return "unknown status";
  }
}

int mixattn_slot_for(int kind, int window, int64_t pos, int64_t* slot) {
  if (!slot) return MIXATTN_ERR_NULL;
  if (pos < 0) return MIXATTN_ERR_LAYER;
  if (kind == MIXATTN_FULL) {
    *slot = pos;
    return MIXATTN_OK;
  }
  if (kind != MIXATTN_SLIDING || window < 1) return MIXATTN_ERR_LAYOUT;
  *slot = pos % window;
  return MIXATTN_OK;
}

int mixattn_validate_config(const mixattn_config* cfg) {
  if (!cfg || !cfg->layers) return MIXATTN_ERR_NULL;
  if (cfg->n_layers < 1 || cfg->batch < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1) return MIXATTN_ERR_LAYOUT;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return MIXATTN_ERR_LAYOUT;
  if (cfg->batch > 65535 || cfg->n_q_heads > 65535) return MIXATTN_ERR_LAYOUT;  // sequences and heads index grid dimensions
  if (cfg->kv_dtype != MIXATTN_F32 && cfg->kv_dtype != MIXATTN_BF16) return MIXATTN_ERR_LAYOUT;
  if (cfg->out_dtype != MIXATTN_F32 && cfg->out_dtype != MIXATTN_BF16) return MIXATTN_ERR_LAYOUT;
  if (cfg->head_dim < 1 || cfg->head_dim > kMaxHeadDim) return MIXATTN_ERR_LAYOUT;
  if (cfg->kv_dtype == MIXATTN_BF16 && (cfg->head_dim % 8) != 0) return MIXATTN_ERR_LAYOUT;
  if (!(cfg->softmax_scale >= 0.f) || isinf(cfg->softmax_scale)) return MIXATTN_ERR_LAYOUT;
  bool any_full = false;
  std::map<int, std::pair<int, int>> seen;  // cache id -> (kind, window)
  for (int i = 0; i < cfg->n_layers; ++i) {
    const mixattn_layer_desc& d = cfg->layers[i];
    if (d.kind != MIXATTN_FULL && d.kind != MIXATTN_SLIDING) return MIXATTN_ERR_LAYOUT;
    if (d.cache_id < 0) return MIXATTN_ERR_LAYOUT;
    if (d.kind == MIXATTN_SLIDING && d.window < 1) return MIXATTN_ERR_LAYOUT;
    const int w = d.kind == MIXATTN_SLIDING ? d.window : 0;
    auto it = seen.find(d.cache_id);
    if (it == seen.end()) {
      seen[d.cache_id] = {d.kind, w};  // the first user is the writer: its kind is the cache's kind
    } else {
      const bool same = it->second == std::make_pair((int)d.kind, w);
      const bool windowed_reader = it->second.first == MIXATTN_FULL && d.kind == MIXATTN_SLIDING;
      if (!same && !windowed_reader) return MIXATTN_ERR_LAYOUT;
    }
    any_full |= d.kind == MIXATTN_FULL;
  }
  if (any_full) {
    if (!cfg->capacity) return MIXATTN_ERR_NULL;
    for (int b = 0; b < cfg->batch; ++b)
      if (cfg->capacity[b] < 1) return MIXATTN_ERR_LAYOUT;
  }
  return MIXATTN_OK;
}

// page_tokens == 0: contiguous caches.  Otherwise the FULL caches are pools of pool_tokens / page_tokens pages.
static int create_layout_impl(const mixattn_config* cfg, int page_tokens, int64_t pool_tokens, mixattn_layout** out) {
  if (!out) return MIXATTN_ERR_NULL;
  int st = mixattn_validate_config(cfg);
  if (st != MIXATTN_OK) return st;
  if (page_tokens != 0) {
    // whole blocks per page, a power of two of them (the kernels split a block index with a shift and a mask)
    if (page_tokens < kBlockKeys || (page_tokens & (page_tokens - 1)) != 0) return MIXATTN_ERR_LAYOUT;
    if (pool_tokens < page_tokens || pool_tokens / page_tokens > INT32_MAX) return MIXATTN_ERR_LAYOUT;
    if (!use_tiled(cfg->kv_dtype, cfg->head_dim, cfg->n_q_heads / cfg->n_kv_heads)) return MIXATTN_ERR_LAYOUT;
  }
  mixattn_layout* L = new (std::nothrow) mixattn_layout();
  if (!L) return MIXATTN_ERR_ALLOC;
  if (!hip_ok(hipGetDevice(&L->device))) {
    delete L;
    return MIXATTN_ERR_HIP;
  }
  L->n_layers = cfg->n_layers;
  L->batch = cfg->batch;
  L->Hq = cfg->n_q_heads;
  L->Hkv = cfg->n_kv_heads;
  L->G = L->Hq / L->Hkv;
  L->D = cfg->head_dim;
  L->kv_dtype = cfg->kv_dtype;
  L->out_dtype = cfg->out_dtype;
  L->elem = elem_bytes(cfg->kv_dtype);
  L->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
  L->tiled = use_tiled(L->kv_dtype, L->D, L->G);
  {
    int cus = 0;
    if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, L->device)) || cus < 1) cus = 256;
    L->n_cus = cus;
  }
  L->layers.assign(cfg->layers, cfg->layers + cfg->n_layers);
  if (cfg->capacity) L->capacity.assign(cfg->capacity, cfg->capacity + cfg->batch);

  // caches in order of first use; the first user is the writer (Section 3, "KV cache reuse")
  std::map<int, int> id2cache;
  L->layer_cache.resize(L->n_layers);
  for (int i = 0; i < L->n_layers; ++i) {
    const auto& d = L->layers[i];
    auto it = id2cache.find(d.cache_id);
    if (it == id2cache.end()) {
      Cache c;
      c.kind = d.kind;
      c.window = d.kind == MIXATTN_SLIDING ? d.window : 0;
      c.writer = i;
      id2cache[d.cache_id] = (int)L->caches.size();
      L->layer_cache[i] = (int)L->caches.size();
      L->caches.push_back(c);
    } else {
      L->layer_cache[i] = it->second;
    }
    L->caches[L->layer_cache[i]].n_users += 1;
  }
  const int B = L->batch;
  const int nc = (int)L->caches.size();
  // the static split-K area of this device (mixattn_decode_noalloc): its address is looked up here, at set-up
  if (!hip_ok(static_scratch_init(L->device))) {
    delete L;
    return MIXATTN_ERR_HIP;
  }
  st = dev_alloc((void**)&L->d_lens_all, sizeof(int32_t) * (size_t)nc * B);
  if (st == MIXATTN_OK && !hip_ok(hipMemset(L->d_lens_all, 0, sizeof(int32_t) * (size_t)nc * B))) st = MIXATTN_ERR_HIP;
  if (st == MIXATTN_OK) st = dev_alloc((void**)&L->d_arrive_all, sizeof(uint32_t) * (size_t)nc);
  if (st == MIXATTN_OK && !hip_ok(hipMemset(L->d_arrive_all, 0, sizeof(uint32_t) * (size_t)nc))) st = MIXATTN_ERR_HIP;
  for (int ci = 0; ci < nc && st == MIXATTN_OK; ++ci) {
    Cache& c = L->caches[ci];
    c.base.resize(B);
    c.slots.resize(B);
    c.len.assign(B, 0);
    c.d_lens = L->d_lens_all + (size_t)ci * B;
    c.d_arrive = L->d_arrive_all + ci;
    int64_t run = 0;  // blocks (tiled) or rows (row-major) before sequence b
    int64_t max_cap = 0;
    for (int b = 0; b < B; ++b) {
      const int64_t want = c.kind == MIXATTN_SLIDING ? c.window : L->capacity[b];
      const int64_t slots = L->tiled ? (want + kBlockKeys - 1) / kBlockKeys * kBlockKeys : want;
      if (slots > INT32_MAX) st = MIXATTN_ERR_LAYOUT;
      c.slots[b] = (int32_t)slots;
      c.base[b] = run;
      run += (int64_t)L->Hkv * (L->tiled ? slots / kBlockKeys : slots);
      max_cap = std::max(max_cap, want);
    }
    if (st != MIXATTN_OK) break;
    c.paged = page_tokens != 0 && c.kind == MIXATTN_FULL;
    if (c.paged) {
      const int page_blocks = page_tokens / kBlockKeys;
      c.page_shift = 0;
      while ((1 << c.page_shift) < page_blocks) ++c.page_shift;
      const int64_t n_pages = pool_tokens / page_tokens;
      c.max_pages = (int)((max_cap + page_tokens - 1) / page_tokens);
      c.free_pages.resize(n_pages);
      for (int64_t i = 0; i < n_pages; ++i) c.free_pages[i] = (int32_t)(n_pages - 1 - i);  // page 0 is handed out first
      c.seq_pages.assign(B, std::vector<int32_t>());
      run = n_pages * L->Hkv * page_blocks;  // blocks in the pool
      if ((st = dev_alloc((void**)&c.d_pages, sizeof(int32_t) * (size_t)B * c.max_pages)) != MIXATTN_OK) break;
      if (!hip_ok(hipMemset(c.d_pages, 0, sizeof(int32_t) * (size_t)B * c.max_pages))) {
        st = MIXATTN_ERR_HIP;
        break;
      }
    }
    c.total_elems = L->tiled ? run * kBlockElems : run * L->D;
    const size_t bytes = (size_t)c.total_elems * L->elem;
    if ((st = dev_alloc(&c.K, bytes)) != MIXATTN_OK) break;
    if ((st = dev_alloc(&c.V, bytes)) != MIXATTN_OK) break;
    if (!hip_ok(hipMemset(c.K, 0, bytes)) || !hip_ok(hipMemset(c.V, 0, bytes))) {
      st = MIXATTN_ERR_HIP;
      break;
    }
    if ((st = dev_alloc((void**)&c.d_base, sizeof(int64_t) * B)) != MIXATTN_OK) break;
    if ((st = dev_alloc((void**)&c.d_slots, sizeof(int32_t) * B)) != MIXATTN_OK) break;
    if ((st = upload(c.d_base, c.base.data(), sizeof(int64_t) * B)) != MIXATTN_OK) break;
    if ((st = upload(c.d_slots, c.slots.data(), sizeof(int32_t) * B)) != MIXATTN_OK) break;
  }
  if (st == MIXATTN_OK && L->tiled) {
    // a group launch serves up to 16 / G layers of one ring at once and keeps partial results for all of them
    int group_layers = 1;
    for (size_t ci = 0; ci < L->caches.size(); ++ci) {
      if (L->caches[ci].kind != MIXATTN_SLIDING) continue;
      int users = 0;
      for (int l = 0; l < L->n_layers; ++l) users += L->layer_cache[l] == (int)ci;
      group_layers = std::max(group_layers, std::min(users, 16 / L->G));
    }
    L->group_layers = group_layers;
    const size_t rows = (size_t)group_layers * B * L->Hq * kMaxChunks;
    st = dev_alloc((void**)&L->scratch.acc, rows * L->D * sizeof(float));
    if (st == MIXATTN_OK) st = dev_alloc((void**)&L->scratch.ml, rows * 2 * sizeof(float));
  }
  if (st == MIXATTN_OK) st = dev_alloc((void**)&L->d_stage_lens, sizeof(int32_t) * B);
  if (st == MIXATTN_OK) st = dev_alloc((void**)&L->d_stage_src, sizeof(int64_t) * B);
  if (st == MIXATTN_OK) st = dev_alloc((void**)&L->d_q_first, sizeof(int64_t) * B);
  if (st == MIXATTN_OK) st = dev_alloc((void**)&L->d_q_len, sizeof(int32_t) * B);
  if (st == MIXATTN_OK) st = dev_alloc(&L->d_readback, 2 * kMaxHeadDim * sizeof(float));
  if (st == MIXATTN_OK && !hip_ok(hipDeviceSynchronize())) st = MIXATTN_ERR_HIP;
  if (st != MIXATTN_OK) {
    free_layout(L);
    return st;
  }
  *out = L;
  return MIXATTN_OK;
}

int mixattn_create_layout(const mixattn_config* cfg, mixattn_layout** out) {
  return create_layout_impl(cfg, 0, 0, out);
}

int mixattn_create_layout_paged(const mixattn_config* cfg, int page_tokens, int64_t pool_tokens,
                                mixattn_layout** out) {
  if (page_tokens < 1) return MIXATTN_ERR_LAYOUT;
  return create_layout_impl(cfg, page_tokens, pool_tokens, out);
}

// Paged caches: make sure sequence b owns pages for want[b] tokens (all sequences or none: a failed call leaves the
// tables as they were).  New table entries reach the device through a small kernel on `s`, ahead of the kernels
// that use them.
static int reserve_pages(mixattn_layout* L, Cache& c, const std::vector<int64_t>& want, hipStream_t s) {
  if (!c.paged) return MIXATTN_OK;
  const int64_t page_tokens = (int64_t)kBlockKeys << c.page_shift;
  int64_t need = 0;
  for (int b = 0; b < L->batch; ++b) {
    const int64_t pages = (want[b] + page_tokens - 1) / page_tokens;
    if (pages > c.max_pages) return MIXATTN_ERR_CAPACITY;
    need += std::max<int64_t>(0, pages - (int64_t)c.seq_pages[b].size());
  }
  if (need == 0) return MIXATTN_OK;
  if (need > (int64_t)c.free_pages.size()) return MIXATTN_ERR_CAPACITY;  // the pool is exhausted
  // plan first, enqueue the table entries, and only then take the pages off the free list
  std::vector<int64_t> index;
  std::vector<int32_t> value;
  std::vector<int> owner;
  size_t top = c.free_pages.size();
  for (int b = 0; b < L->batch; ++b) {
    const int64_t pages = (want[b] + page_tokens - 1) / page_tokens;
    for (int64_t have = (int64_t)c.seq_pages[b].size(); have < pages; ++have) {
      index.push_back((int64_t)b * c.max_pages + have);
      value.push_back(c.free_pages[--top]);
      owner.push_back(b);
    }
  }
  HIP_TRY(launch_scatter_i32(c.d_pages, index.data(), value.data(), (int)index.size(), s));
  for (size_t i = 0; i < value.size(); ++i) c.seq_pages[owner[i]].push_back(value[i]);
  c.free_pages.resize(top);
  return MIXATTN_OK;
}

static void release_pages(Cache& c, int b) {
  if (!c.paged) return;
  for (auto it = c.seq_pages[b].rbegin(); it != c.seq_pages[b].rend(); ++it) c.free_pages.push_back(*it);
  c.seq_pages[b].clear();
}

int mixattn_destroy_layout(mixattn_layout* L) {
  if (!L) return MIXATTN_ERR_NULL;
  (void)hipDeviceSynchronize();
  free_layout(L);
  return MIXATTN_OK;
}

int mixattn_reset(mixattn_layout* L, void* stream) {
  if (!L) return MIXATTN_ERR_NULL;
  HIP_TRY(launch_fill_i32(L->d_lens_all, 0, (int64_t)L->caches.size() * L->batch, (hipStream_t)stream));
  for (auto& c : L->caches) {
    std::fill(c.len.begin(), c.len.end(), 0);
    for (int b = 0; b < L->batch; ++b) release_pages(c, b);
    c.own_stage.cache = -1;
    c.plan_key = -1;
    if (c.own_stage.d_done) HIP_TRY(launch_fill_i32(c.own_stage.d_done, 0, L->batch, (hipStream_t)stream));
  }
  return MIXATTN_OK;
}

int mixattn_release_sequence(mixattn_layout* L, int b, void* stream) {
  if (!L) return MIXATTN_ERR_NULL;
  if (b < 0 || b >= L->batch) return MIXATTN_ERR_LAYER;
  for (auto& c : L->caches) {
    HIP_TRY(launch_fill_i32(c.d_lens + b, kIdle, 1, (hipStream_t)stream));
    if (c.own_stage.d_done) HIP_TRY(launch_fill_i32(c.own_stage.d_done + b, 0, 1, (hipStream_t)stream));
    c.len[b] = kIdle;
    c.plan_key = -1;
    release_pages(c, b);
    c.own_stage.cache = -1;
  }
  return MIXATTN_OK;
}

// Tokens sequence b holds in cache c (an idle sequence holds none).
static inline int64_t held(const Cache& c, int b) { return c.len[b] < 0 ? 0 : c.len[b]; }
static inline bool idle(const Cache& c, int b) { return c.len[b] < 0; }

// A staged prompt chunk describes the cache as its writer's prefill left it: any other change to the cache retires it.
static void retire_stage(mixattn_layout*, Cache& c) { c.own_stage.cache = -1; }

static int check_append(const mixattn_layout* L, const Cache& c, int layer) {
  if (c.writer != layer) return MIXATTN_ERR_NOT_WRITER;
  for (int b = 0; b < L->batch; ++b) {
    if (idle(c, b)) continue;  // takes no token
    if (c.kind == MIXATTN_FULL && c.len[b] + 1 > L->capacity[b]) return MIXATTN_ERR_CAPACITY;
    if (c.len[b] + 1 > INT32_MAX) return MIXATTN_ERR_CAPACITY;
  }
  return MIXATTN_OK;
}

static int reserve_for_append(mixattn_layout* L, Cache& c, hipStream_t s) {
  if (!c.paged) return MIXATTN_OK;
  std::vector<int64_t> want(L->batch);
  for (int b = 0; b < L->batch; ++b) want[b] = idle(c, b) ? 0 : c.len[b] + 1;
  return reserve_pages(L, c, want, s);
}

int mixattn_append_kv(mixattn_layout* L, int layer, const void* k, const void* v, void* stream) {
  if (!L || !k || !v) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  Cache& c = L->caches[L->layer_cache[layer]];
  int st = check_append(L, c, layer);
  if (st != MIXATTN_OK) return st;
  if ((st = reserve_for_append(L, c, (hipStream_t)stream)) != MIXATTN_OK) return st;
  retire_stage(L, c);
  AppendLaunch a;
  a.K = c.K; a.V = c.V; a.d_base = c.d_base; a.d_slots = c.d_slots; a.d_lens = c.lens();
  a.pages = c.page_table();
  a.window = c.window; a.k = k; a.v = v;
  a.batch = L->batch; a.Hkv = L->Hkv; a.D = L->D; a.elem = L->elem;
  HIP_TRY(L->tiled ? launch_append_tiled(a, (hipStream_t)stream) : launch_append_rowmajor(a, (hipStream_t)stream));
  for (int b = 0; b < L->batch; ++b) c.len[b] += idle(c, b) ? 0 : 1;
  return MIXATTN_OK;
}

// tokens a decode streams for a sequence of `len` tokens: all of a full cache, the ring's content, or the window
static inline int64_t tokens_read(const Cache& c, int64_t len, int attn_window) {
  if (c.window > 0) return std::min<int64_t>(len, c.window);
  if (attn_window > 0) return std::min<int64_t>(len, attn_window);
  return len;
}

// A sliding layer that reads a standard layer's (full) cache attends the last `window` positions of it; every other
// layer attends whatever its cache holds.
static inline int layer_attn_window(const mixattn_layout* L, int layer) {
  const Cache& c = L->caches[L->layer_cache[layer]];
  return (c.kind == MIXATTN_FULL && L->layers[layer].kind == MIXATTN_SLIDING) ? L->layers[layer].window : 0;
}

// Split-K plan for the tiled decode kernel: the target chunk length in blocks.  A sequence of nb blocks is cut
// into ceil(nb / target) equal chunks, one workgroup each.  Two effects bound a launch (figures measured on
// MI355X with this kernel): the HBM stream, about 7.0 TB/s once a few hundred workgroups are resident, and the
// rate of one workgroup, whose four wavefronts keep 128 KiB in flight and advance by one 16 KiB block in about
// 0.25 us.  Cutting sequences shortens the second bound but costs a combine launch (about 5 us); with two
// workgroups resident per CU, chunks run in rounds of 2 * CUs.
static int plan_chunk_blocks(const mixattn_layout* L, Cache& c, int max_blocks, int extra, int attn_window) {
  const double slots = 2.0 * L->n_cus;
  const double us_per_block_bw = 2.0 * kBlockElems * 2 / 7.0e6;  // 16 KiB at 7.0 TB/s
  // A wavefront keeps two blocks in flight: a workgroup that is not held back by the memory system takes about
  // 0.25 us per block.  (Workgroups of 8 wavefronts were measured as well: no gain, one CU cannot pull much more.)
  const double us_per_block_wg = 0.25, us_wg_fixed = 1.0, us_combine = 5.0;
  auto blocks_of = [&](int b) {
    if (idle(c, b)) return 0;
    const int64_t n = tokens_read(c, c.len[b] + extra, attn_window);
    return (int)((n + kBlockKeys - 1) / kBlockKeys) + (attn_window > 0 ? 1 : 0);  // a window may straddle a block more
  };
  // the plan only changes when some sequence crosses a block boundary: memoise on the block counts
  int64_t sum_nb = 0;
  int min_nb = INT32_MAX, max_nb = 0;
  for (int b = 0; b < L->batch; ++b) {
    const int nb = blocks_of(b);
    sum_nb += nb;
    min_nb = std::min(min_nb, nb);
    max_nb = std::max(max_nb, nb);
  }
  const int64_t key = ((sum_nb * 1000003 + max_nb) * 1000003 + min_nb) * 131 + attn_window % 131;
  if (c.plan_key == key && c.plan_max_blocks == max_blocks) return c.plan_chunk_blocks;

  const double total_blocks = (double)sum_nb * L->Hkv;
  const double t_bw = total_blocks * us_per_block_bw;
  int best_t = max_blocks;
  double best_cost = 1e300;
  for (int chunks = 1; chunks <= kMaxChunks; ++chunks) {
    const int t = (max_blocks + chunks - 1) / chunks;
    if (chunks > 1 && t < kDecodeMinChunkBlocks) break;
    double wgs = 0;
    int longest = 0;
    if (min_nb == max_nb) {  // uniform batch: closed form
      const int cb = (max_nb + t - 1) / t;
      wgs = (double)cb * L->Hkv * L->batch;
      longest = (max_nb + cb - 1) / cb;
    } else {
      for (int b = 0; b < L->batch; ++b) {
        const int nb = blocks_of(b);
        if (nb == 0) continue;  // idle sequence
        const int cb = (nb + t - 1) / t;
        wgs += (double)cb * L->Hkv;
        longest = std::max(longest, (nb + cb - 1) / cb);
      }
    }
    const double t_long = longest * us_per_block_wg + us_wg_fixed;
    // list-scheduling estimate of the per-workgroup bound over `slots` resident workgroups
    const double t_sched = wgs <= slots ? t_long
                                        : (total_blocks * us_per_block_wg + wgs * us_wg_fixed) / slots + 0.5 * t_long;
    const double cost = std::max(t_bw, std::max(t_long, t_sched)) + (chunks > 1 ? us_combine : 0.0);
    if (cost < best_cost - 1e-9) {
      best_cost = cost;
      best_t = t;
    }
  }
  c.plan_key = key;
  c.plan_max_blocks = max_blocks;
  c.plan_chunk_blocks = std::max(best_t, 1);
  return c.plan_chunk_blocks;
}

// Decode launch shared by mixattn_decode, mixattn_decode_noalloc, mixattn_append_decode and mixattn_decode_group.
// `extra` = 1 when a fused launch appends this step's token itself (lengths on host and device still hold the old
// value while planning).  static_scratch: split-K partials go to the library's static device area; the call is
// refused (SCRATCH) when they do not fit.
static int launch_decode(mixattn_layout* L, Cache& c, int attn_window, const void* q, void* out, const void* k_new,
                         const void* v_new, hipStream_t stream, int n_group = 0, bool static_scratch = false) {
  const int extra = k_new ? 1 : 0;
  int max_blocks = 0;  // most blocks one sequence reads
  for (int b = 0; b < L->batch; ++b) {
    if (idle(c, b)) continue;
    const int64_t len = c.len[b] + extra;
    int64_t blocks;
    if (attn_window > 0 && len > attn_window)
      blocks = (len + kBlockKeys - 1) / kBlockKeys - (len - attn_window) / kBlockKeys;
    else
      blocks = (tokens_read(c, len, attn_window) + kBlockKeys - 1) / kBlockKeys;
    max_blocks = std::max<int>(max_blocks, (int)blocks);
  }
  const bool nothing_to_read = max_blocks == 0;  // every sequence is idle: the launch only writes zero rows
  max_blocks = std::max(max_blocks, 1);
  DecodeLaunch a;
  a.K = c.K; a.V = c.V; a.d_base = c.d_base; a.d_slots = c.d_slots; a.d_lens = c.lens();
  a.pages = c.page_table();
  a.window = c.window; a.attn_window = attn_window; a.q = q; a.out = out;
  a.batch = L->batch; a.Hq = L->Hq; a.Hkv = L->Hkv; a.G = L->G; a.D = L->D;
  a.kv_dtype = L->kv_dtype; a.out_dtype = L->out_dtype; a.scale = L->scale;
  a.scratch = L->scratch;
  a.static_scratch = static_scratch; a.device = L->device;
  a.k_new = k_new; a.v_new = v_new;
  a.d_lens_rw = k_new ? c.lens() : nullptr;
  a.arrive = k_new ? c.d_arrive : nullptr;
  a.n_group = n_group;
  if (!L->tiled) {
    a.max_blocks = a.chunk_blocks = a.n_chunks = 0;
    HIP_TRY(launch_decode_rowmajor(a, stream));
    return MIXATTN_OK;
  }
  int chunk_blocks;
  if (nothing_to_read) {
    chunk_blocks = 1;
  } else if (L->chunk_keys > 0) {
    chunk_blocks = (int)(L->chunk_keys / kBlockKeys);
  } else {
    chunk_blocks = plan_chunk_blocks(L, c, max_blocks, extra, attn_window);
  }
  chunk_blocks = std::max(chunk_blocks, (max_blocks + kMaxChunks - 1) / kMaxChunks);
  a.max_blocks = max_blocks;
  a.chunk_blocks = chunk_blocks;
  a.n_chunks = (max_blocks + chunk_blocks - 1) / chunk_blocks;
  // Full caches: when the sequences differ in length, or have to be cut anyway, the blocks of all (sequence, kv
  // head) streams are cut into equal runs, one per workgroup, instead of cutting every sequence by itself (with one
  // workgroup per sequence and head the long sequences finish alone, at the pace of a few workgroups; per-sequence
  // chunks of one target length come in sizes up to 2:1 and in numbers that do not fill the last round).
  // Measured: ragged batch of 64, 5.68 -> 6.63 TB/s; one sequence of 131072, 4.68 -> 5.23 TB/s; a uniform batch
  // that needs no cut stays on the unsplit launch (6.72 against 6.64 TB/s).  Not with the static scratch area: a
  // balanced launch needs room for the most pieces a stream can fall into, whatever the lengths turn out to be.
  if (c.kind == MIXATTN_FULL && attn_window == 0 && n_group == 0 && L->chunk_keys == 0 && L->balanced != 0 &&
      L->batch <= 1024 && !nothing_to_read && !static_scratch) {
    int64_t sum_nb = 0;
    int max_nb = 0;
    for (int b = 0; b < L->batch; ++b) {
      const int nb = idle(c, b) ? 0 : (int)((c.len[b] + extra + kBlockKeys - 1) / kBlockKeys);
      sum_nb += nb;
      max_nb = std::max(max_nb, nb);
    }
    const bool ragged = (int64_t)max_nb * L->batch * 4 > sum_nb * 5;  // longest sequence > 1.25 x the mean
    const bool uniform = sum_nb == (int64_t)max_nb * L->batch;        // every sequence reads the same number of blocks
    if (uniform && a.n_chunks > 1 && L->balanced != 2) {
      // Equal streams that have to be cut: the plain split-K launch with as many chunks per stream as give two
      // workgroups per CU is the same partition as the balanced one, without its scan and search (config 1's full
      // layer: 42.7 against 45.4 us with the combine launch).
      const int64_t streams = (int64_t)L->batch * L->Hkv;
      int chunks = (int)std::min<int64_t>(kMaxChunks, (2 * (int64_t)L->n_cus + streams - 1) / streams);
      chunks = std::max(1, std::min(chunks, max_blocks / kDecodeMinChunkBlocks));
      a.chunk_blocks = (max_blocks + chunks - 1) / chunks;
      a.n_chunks = (max_blocks + a.chunk_blocks - 1) / a.chunk_blocks;
    } else if (ragged || a.n_chunks > 1 || L->balanced == 2) {
      // the kernels derive the run length from the lengths and the number of runs in the same way
      const int64_t total = sum_nb * L->Hkv;
      const int64_t slots = 2 * (int64_t)L->n_cus;
      int64_t share = (total + slots - 1) / slots;
      share = std::max<int64_t>(share, (max_nb + (kMaxChunks - 2) - 1) / (kMaxChunks - 2));  // pieces per stream <= kMaxChunks
      share = std::max<int64_t>(share, kDecodeMinChunkBlocks);
      const int64_t runs = (total + share - 1) / share;
      if (runs >= 2) a.balanced_runs = (int)runs;
    }
  }
  if (static_scratch && a.n_chunks > 1) {
    const int64_t rows = (int64_t)std::max(n_group, 1) * L->batch * L->Hq;
    if (static_scratch_bytes(rows, a.n_chunks) > (int64_t)kStaticScratchBytes) return MIXATTN_ERR_SCRATCH;
  }
  HIP_TRY(launch_decode_tiled(a, stream));
  return MIXATTN_OK;
}

static int check_decode(const mixattn_layout* L, int layer, const void* q, const void* out) {
  if (!L || !q || !out) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  const Cache& c = L->caches[L->layer_cache[layer]];
  for (int b = 0; b < L->batch; ++b)
    if (c.len[b] == 0) return MIXATTN_ERR_ORDER;  // empty; an idle sequence (negative) is passed over
  return MIXATTN_OK;
}

int mixattn_decode(mixattn_layout* L, int layer, const void* q, void* out, void* stream) {
  const int st = check_decode(L, layer, q, out);
  if (st != MIXATTN_OK) return st;
  Cache& c = L->caches[L->layer_cache[layer]];
  return launch_decode(L, c, layer_attn_window(L, layer), q, out, nullptr, nullptr, (hipStream_t)stream);
}

int mixattn_decode_noalloc(mixattn_layout* L, int layer, const void* q, void* out, void* stream) {
  const int st = check_decode(L, layer, q, out);
  if (st != MIXATTN_OK) return st;
  if (!L->tiled) return MIXATTN_ERR_LAYOUT;  // the scalar path has no scratch to begin with: mixattn_decode
  Cache& c = L->caches[L->layer_cache[layer]];
  return launch_decode(L, c, layer_attn_window(L, layer), q, out, nullptr, nullptr, (hipStream_t)stream, 0, true);
}

int mixattn_append_decode(mixattn_layout* L, int layer, const void* k, const void* v, const void* q, void* out,
                          void* stream) {
  if (!L || !k || !v || !q || !out) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  Cache& c = L->caches[L->layer_cache[layer]];
  int st = check_append(L, c, layer);
  if (st != MIXATTN_OK) return st;
  if (!L->tiled) {  // row-major path: the two launches, one after the other
    st = mixattn_append_kv(L, layer, k, v, stream);
    return st != MIXATTN_OK ? st : mixattn_decode(L, layer, q, out, stream);
  }
  if ((st = reserve_for_append(L, c, (hipStream_t)stream)) != MIXATTN_OK) return st;
  st = launch_decode(L, c, 0, q, out, k, v, (hipStream_t)stream);
  if (st != MIXATTN_OK) return st;
  retire_stage(L, c);
  for (int b = 0; b < L->batch; ++b) c.len[b] += idle(c, b) ? 0 : 1;  // the launch advances the device lengths
  return MIXATTN_OK;
}

int mixattn_decode_group(mixattn_layout* L, const int32_t* layers, int n_layers, const void* k, const void* v,
                         const void* q, void* out, void* stream) {
  if (!L || !layers || !q || !out || (k == nullptr) != (v == nullptr)) return MIXATTN_ERR_NULL;
  if (n_layers < 1) return MIXATTN_ERR_LAYER;
  for (int i = 0; i < n_layers; ++i) {
    if (layers[i] < 0 || layers[i] >= L->n_layers) return MIXATTN_ERR_LAYER;
    for (int j = 0; j < i; ++j)
      if (layers[j] == layers[i]) return MIXATTN_ERR_LAYER;
  }
  const int ci = L->layer_cache[layers[0]];
  Cache& c = L->caches[ci];
  for (int i = 1; i < n_layers; ++i)
    if (L->layer_cache[layers[i]] != ci) return MIXATTN_ERR_LAYOUT;
  if (!L->tiled || c.kind != MIXATTN_SLIDING || n_layers > L->group_layers) return MIXATTN_ERR_LAYOUT;
  if (k) {
    const int st = check_append(L, c, layers[0]);
    if (st != MIXATTN_OK) return st;
  } else {
    for (int b = 0; b < L->batch; ++b)
      if (c.len[b] == 0) return MIXATTN_ERR_ORDER;
  }
  const int st = launch_decode(L, c, 0, q, out, k, v, (hipStream_t)stream, n_layers);
  if (st != MIXATTN_OK) return st;
  if (k) {
    retire_stage(L, c);
    for (int b = 0; b < L->batch; ++b) c.len[b] += idle(c, b) ? 0 : 1;  // the launch advances the device lengths
  }
  return MIXATTN_OK;
}

// ---- captured decode steps (HIP graphs) ---------------------------------------------------------------------
int mixattn_reserve_steps(mixattn_layout* L, int steps, void* stream) {
  if (!L) return MIXATTN_ERR_NULL;
  if (steps < 0) return MIXATTN_ERR_ORDER;
  // every check first, for every cache: a refusal leaves every page table as it was
  for (const Cache& c : L->caches) {
    if (c.kind != MIXATTN_FULL) continue;
    int64_t need = 0;
    const int64_t page_tokens = (int64_t)kBlockKeys << c.page_shift;
    for (int b = 0; b < L->batch; ++b) {
      if (idle(c, b)) continue;
      if (c.len[b] + steps > L->capacity[b]) return MIXATTN_ERR_CAPACITY;
      if (c.paged) need += std::max<int64_t>(0, (c.len[b] + steps + page_tokens - 1) / page_tokens - (int64_t)c.seq_pages[b].size());
    }
    if (c.paged && need > (int64_t)c.free_pages.size()) return MIXATTN_ERR_CAPACITY;
  }
  for (Cache& c : L->caches) {
    if (!c.paged) continue;
    std::vector<int64_t> want(L->batch);
    for (int b = 0; b < L->batch; ++b) want[b] = idle(c, b) ? 0 : c.len[b] + steps;
    const int st = reserve_pages(L, c, want, (hipStream_t)stream);
    if (st != MIXATTN_OK) return st;
  }
  return MIXATTN_OK;
}

int mixattn_account_replays(mixattn_layout* L, int steps) {
  if (!L) return MIXATTN_ERR_NULL;
  if (steps < 0) return MIXATTN_ERR_ORDER;
  for (const Cache& c : L->caches)
    for (int b = 0; b < L->batch; ++b)
      if (!idle(c, b) && c.kind == MIXATTN_FULL && c.len[b] + steps > L->capacity[b]) return MIXATTN_ERR_CAPACITY;
  for (Cache& c : L->caches) {
    for (int b = 0; b < L->batch; ++b) c.len[b] += idle(c, b) ? 0 : steps;
    if (steps > 0) retire_stage(L, c);
  }
  return MIXATTN_OK;
}

// Staging area of cache c for prompt chunks: tile-format copies that the MFMA prefill kernel reads.  A full cache
// stages V only (as fp16, positions 0 .. n-1; K is read from the cache itself), a ring stages K and V of positions
// n_old - (W-1) .. n_new-1.  Growing it synchronises the device and allocates, so callers do it before they change
// any state; mixattn_reserve_prefill sizes every area once, after which no prefill call gets here.
static int grow_stage(mixattn_layout* L, Cache& c, int64_t blocks_per_head) {
  Stage& S = c.own_stage;
  if (S.blocks >= blocks_per_head) return MIXATTN_OK;
  const bool need_k = c.kind == MIXATTN_SLIDING;
  const size_t bytes = (size_t)L->batch * L->Hkv * blocks_per_head * kBlockElems * 2;
  // allocate the new area first: a failure leaves the old one (and whatever it holds) as it was
  void* nK = nullptr;
  void* nV = nullptr;
  int st;
  if (!S.d_base && (st = dev_alloc((void**)&S.d_base, sizeof(int64_t) * L->batch)) != MIXATTN_OK) return st;
  if (!S.d_slots && (st = dev_alloc((void**)&S.d_slots, sizeof(int32_t) * L->batch)) != MIXATTN_OK) return st;
  if (!S.d_done && (st = dev_alloc((void**)&S.d_done, sizeof(int32_t) * L->batch)) != MIXATTN_OK) return st;
  if (need_k && (st = dev_alloc(&nK, bytes)) != MIXATTN_OK) return st;
  if ((st = dev_alloc(&nV, bytes)) != MIXATTN_OK) {
    if (nK) (void)hipFree(nK);
    return st;
  }
  // the old area and its geometry tables may still be in use by work in flight
  if (!hip_ok(hipDeviceSynchronize())) {
    if (nK) (void)hipFree(nK);
    (void)hipFree(nV);
    return MIXATTN_ERR_HIP;
  }
  if (S.K) (void)hipFree(S.K);
  if (S.V) (void)hipFree(S.V);
  S.K = nK;
  S.V = nV;
  S.blocks = 0;
  S.cache = -1;
  std::vector<int64_t> base(L->batch);
  std::vector<int32_t> slots(L->batch, (int32_t)(blocks_per_head * kBlockKeys));
  for (int b = 0; b < L->batch; ++b) base[b] = (int64_t)b * L->Hkv * blocks_per_head;
  if ((st = upload(S.d_base, base.data(), sizeof(int64_t) * L->batch)) != MIXATTN_OK) return st;
  if ((st = upload(S.d_slots, slots.data(), sizeof(int32_t) * L->batch)) != MIXATTN_OK) return st;
  if (!hip_ok(hipMemset(S.d_done, 0, sizeof(int32_t) * L->batch))) return MIXATTN_ERR_HIP;  // the new area holds nothing yet
  S.blocks = blocks_per_head;
  return MIXATTN_OK;
}

// blocks per (sequence, kv head) the staging area of cache c needs for chunks of up to `chunk` tokens
static int64_t stage_blocks_for(const mixattn_layout* L, const Cache& c, int64_t chunk) {
  int64_t tokens;
  if (c.kind == MIXATTN_FULL) {
    tokens = 0;  // a copy of V for everything the cache can hold
    for (int b = 0; b < L->batch; ++b) tokens = std::max<int64_t>(tokens, L->capacity[b]);
  } else {
    tokens = (int64_t)c.window - 1 + chunk;
  }
  return (tokens + kBlockKeys - 1) / kBlockKeys;
}

int mixattn_reserve_prefill(mixattn_layout* L, int max_chunk_tokens) {
  if (!L) return MIXATTN_ERR_NULL;
  if (max_chunk_tokens < 1) return MIXATTN_ERR_ORDER;
  if (!L->tiled) return MIXATTN_OK;  // the scalar path stages nothing
  for (Cache& c : L->caches) {
    const int st = grow_stage(L, c, stage_blocks_for(L, c, max_chunk_tokens));
    if (st != MIXATTN_OK) return st;
  }
  L->reserved_chunk = std::max<int64_t>(L->reserved_chunk, max_chunk_tokens);
  return MIXATTN_OK;
}

int mixattn_release_prefill(mixattn_layout* L) {
  if (!L) return MIXATTN_ERR_NULL;
  // readers of a staged chunk may still be in flight
  if (!hip_ok(hipDeviceSynchronize())) return MIXATTN_ERR_HIP;
  for (Cache& c : L->caches) free_stage(c.own_stage);
  L->reserved_chunk = 0;
  return MIXATTN_OK;
}

int64_t mixattn_staging_bytes(const mixattn_layout* L) {
  if (!L) return MIXATTN_ERR_NULL;
  int64_t t = 0;
  for (const Cache& c : L->caches) {
    const Stage& S = c.own_stage;
    const int64_t area = (int64_t)L->batch * L->Hkv * S.blocks * kBlockElems * 2;
    t += (S.K ? area : 0) + (S.V ? area : 0);
  }
  return t;
}

// Prompt attention for a chunk of lens[b] tokens per sequence (varlen) or seq_len tokens for every sequence
// (lens == nullptr).  In the varlen case seq_len is the longest chunk and q / k / v / out are packed by sequence.
static int prefill_impl(mixattn_layout* L, int layer, const void* q, const void* k, const void* v, void* out,
                        const int32_t* lens, int seq_len, void* stream) {
  const bool varlen = lens != nullptr;
  auto len_of = [&](int b) -> int64_t { return varlen ? lens[b] : seq_len; };
  const int ci = L->layer_cache[layer];
  Cache& c = L->caches[ci];
  const bool writer = c.writer == layer;
  const bool sliding_cache = c.kind == MIXATTN_SLIDING;
  // a reader may pass k = v = NULL to reuse the prompt copy staged by the latest prefill call, if that call was for
  // the same cache and length (tiled path only)
  const bool reuse_stage = !k && !v;
  // every cache stages its chunks in an area of its own, which outlives the calls of other layers
  Stage& S = c.own_stage;
  if (reuse_stage) {
    if (writer || !L->tiled || L->prefill_simple) return MIXATTN_ERR_NULL;
    if (S.cache != ci || (int)S.lens.size() != L->batch) return MIXATTN_ERR_ORDER;
    for (int b = 0; b < L->batch; ++b)
      if (S.lens[b] != len_of(b)) return MIXATTN_ERR_ORDER;
  } else if (!k || !v) {
    return MIXATTN_ERR_NULL;
  }
  // n_old: tokens held before this chunk.  A writer appends the chunk; a reader's cache already holds it.
  bool chunked = false;
  int64_t max_new = 0, max_old = 0;
  for (int b = 0; b < L->batch; ++b) {
    if (len_of(b) == 0) continue;  // sits this call out (and stays idle if it is)
    const int64_t n_old = writer ? held(c, b) : held(c, b) - len_of(b);
    if (n_old < 0) return MIXATTN_ERR_ORDER;  // the writer's prefill of this chunk has not run
    if (c.kind == MIXATTN_FULL && n_old + len_of(b) > L->capacity[b]) return MIXATTN_ERR_CAPACITY;
    if (n_old + len_of(b) > INT32_MAX) return MIXATTN_ERR_CAPACITY;
    chunked |= n_old > 0;
    max_new = std::max(max_new, n_old + len_of(b));
    max_old = std::max(max_old, n_old);
  }
  // Readers of a ring come after their writer's commit, which has overwritten keys the chunk's first rows need:
  // past the first chunk they can only run from the ring's staged copy of that chunk (k = v = NULL).
  if (chunked && sliding_cache && !writer && !reuse_stage) return MIXATTN_ERR_ORDER;
  if (chunked && sliding_cache && !writer && !L->tiled) return MIXATTN_ERR_ORDER;
  const bool simple = !L->tiled || L->prefill_simple != 0;  // scalar kernel on the caller's tensors
  if (simple && L->tiled && chunked) return MIXATTN_ERR_ORDER;  // the cross-check path keeps to whole prompts
  hipStream_t s = (hipStream_t)stream;
  const int attn_window = L->layers[layer].kind == MIXATTN_SLIDING ? L->layers[layer].window : 0;
  // Everything that can fail is done before the first state change: the staging area is grown if mixattn_reserve_prefill
  // has not sized it for this chunk (synchronises and allocates), then a paged cache takes the pages the chunk needs.
  if (L->tiled && !simple && !reuse_stage) {
    const int64_t need = sliding_cache ? (std::min<int64_t>(max_old, c.window - 1) + seq_len + kBlockKeys - 1) / kBlockKeys
                                       : (max_new + kBlockKeys - 1) / kBlockKeys;
    const int e = grow_stage(L, c, need);
    if (e != MIXATTN_OK) return e;
  }
  if (writer && c.paged) {
    std::vector<int64_t> want(L->batch);
    for (int b = 0; b < L->batch; ++b) want[b] = held(c, b) + len_of(b);
    const int e = reserve_pages(L, c, want, s);
    if (e != MIXATTN_OK) return e;
  }
  // per-sequence row tables of a varlen call (every kernel of this call reads them after this point of the stream)
  const int64_t* d_first = nullptr;
  const int32_t* d_len = nullptr;
  if (varlen) {
    std::vector<int64_t> first(L->batch);
    int64_t run = 0;
    for (int b = 0; b < L->batch; ++b) {
      first[b] = run;
      run += lens[b];
    }
    HIP_TRY(launch_set_seq_tables(L->d_q_first, L->d_q_len, first.data(), lens, L->batch, s));
    d_first = L->d_q_first;
    d_len = L->d_q_len;
  }
  // where the chunk's tokens sit in the caller's tensors
  auto set_source = [&](StoreLaunch& st) {
    st.k_src = k; st.v_src = v;
    st.uniform_len = varlen ? 0 : seq_len;
    st.d_src_first = d_first; st.d_src_len = d_len;
  };
  auto remember_stage = [&]() {
    S.cache = ci;
    S.lens.resize(L->batch);
    for (int b = 0; b < L->batch; ++b) S.lens[b] = (int32_t)len_of(b);
  };

  PrefillLaunch p;
  p.q = q; p.out = out; p.k_src = k; p.v_src = v;
  p.window = attn_window;
  p.batch = L->batch; p.S = seq_len; p.Hq = L->Hq; p.Hkv = L->Hkv; p.G = L->G; p.D = L->D;
  p.kv_dtype = L->kv_dtype; p.out_dtype = L->out_dtype; p.scale = L->scale;
  p.waves = (int)L->prefill_waves;
  p.heads = (int)L->prefill_heads;
  p.d_q_first = d_first; p.d_q_len = d_len;

  // commit of the chunk into this layer's cache (writer): the store reads the lengths, a small launch then advances them
  auto commit = [&]() -> int {
    StoreLaunch st;
    st.K = c.K; st.V = c.V; st.d_base = c.d_base; st.d_slots = c.d_slots; st.window = c.window;
    st.pages = c.page_table();
    set_source(st);
    st.d_n_old = c.lens(); st.old_sub = 0;
    if (L->tiled) {
      st.Kold = c.K; st.Vold = c.V; st.old_base = c.d_base; st.old_slots = c.d_slots; st.old_window = c.window;
      st.old_pages = c.page_table();
      st.old_is_dest = 1;
    }
    st.batch = L->batch; st.Hkv = L->Hkv; st.D = L->D; st.elem = L->elem;
    st.max_slots = (int)(c.window > 0 ? std::min<int64_t>(max_new, c.window) : max_new);
    HIP_TRY(L->tiled ? launch_store_tiled(st, s) : launch_store_rowmajor(st, s));
    HIP_TRY(launch_advance_lens(c.lens(), d_len, varlen ? 0 : seq_len, L->batch, s));
    for (int b = 0; b < L->batch; ++b)
      if (len_of(b) > 0) c.len[b] = held(c, b) + len_of(b);  // a chunk also starts an idle sequence
    return MIXATTN_OK;
  };

  if (!L->tiled || (simple && !chunked)) {
    // scalar kernel: the chunk from the caller's tensors, earlier positions from the row-major cache as it was
    // before this chunk (a ring still holds them then, so a sliding writer attends first and commits after)
    if (!L->tiled) {
      p.Kc = c.K; p.Vc = c.V; p.c_base = c.d_base; p.c_slots = c.d_slots; p.ring = c.window;
    }
    if (writer && !sliding_cache) {
      int e = commit();
      if (e != MIXATTN_OK) return e;
    }
    const bool lens_hold_chunk = !(writer && sliding_cache);
    p.d_lens = (!L->tiled && chunked) ? c.lens() : nullptr;
    p.old_sub = lens_hold_chunk ? 1 : 0;
    HIP_TRY(launch_prefill_rowmajor(p, s));
    if (writer && sliding_cache) {
      int e = commit();
      if (e != MIXATTN_OK) return e;
    }
    return MIXATTN_OK;
  }

  // ---- MFMA path
  if (!sliding_cache) {
    // K from the full cache itself (commit first), V from an fp16 copy of positions 0 .. n_new-1 in the staging area
    if (writer) {
      int e = commit();
      if (e != MIXATTN_OK) return e;
    }
    if (!reuse_stage) {
      S.cache = -1;
      StoreLaunch st;
      st.K = nullptr; st.V = S.V; st.v_as_f16 = 1;
      st.d_base = S.d_base; st.d_slots = S.d_slots; st.window = 0;
      set_source(st);
      if (chunked) {
        st.d_n_old = c.lens(); st.old_sub = 1;  // lengths already include the chunk
        st.Vold = c.V; st.old_base = c.d_base; st.old_slots = c.d_slots; st.old_window = 0;
        st.old_pages = c.page_table();
      }
      st.batch = L->batch; st.Hkv = L->Hkv; st.D = L->D; st.elem = L->elem;
      st.max_slots = (int)max_new;
      st.d_done = S.d_done;  // blocks converted by earlier chunks stay as they are
      HIP_TRY(launch_store_tiled(st, s));
      HIP_TRY(launch_mark_done(S.d_done, c.lens(), d_len, varlen ? 0 : seq_len, L->batch, s));
      remember_stage();
    }
    p.Kt = c.K; p.k_base = c.d_base; p.k_slots = c.d_slots;
    p.k_pages = c.page_table();
    p.Vt = S.V; p.v_base = S.d_base; p.v_slots = S.d_slots;
    p.stage_window = 0;
    p.d_lens = chunked ? c.lens() : nullptr; p.old_sub = 1;
    HIP_TRY(launch_prefill_tiled(p, s));
    return MIXATTN_OK;
  }

  // sliding cache: K and V from a staging copy of positions max(0, n_old - (W-1)) .. n_new-1, built from the ring
  // (before it receives the chunk) and the chunk
  const int W = c.window;
  if (!reuse_stage) {
    const int64_t span = std::min<int64_t>(max_old, W - 1) + seq_len;
    S.cache = -1;
    StoreLaunch st;
    st.K = S.K; st.V = S.V; st.v_as_f16 = 1;
    st.d_base = S.d_base; st.d_slots = S.d_slots; st.window = 0;
    st.stage_window = W;
    set_source(st);
    if (chunked) {  // writer (readers past the first chunk always reuse): lengths do not include the chunk yet
      st.d_n_old = c.lens(); st.old_sub = 0;
      st.Kold = c.K; st.Vold = c.V; st.old_base = c.d_base; st.old_slots = c.d_slots; st.old_window = W;
    }
    st.batch = L->batch; st.Hkv = L->Hkv; st.D = L->D; st.elem = L->elem;
    st.max_slots = (int)span;
    HIP_TRY(launch_store_tiled(st, s));
    remember_stage();
  }
  p.Kt = S.K; p.k_base = S.d_base; p.k_slots = S.d_slots;
  p.Vt = S.V; p.v_base = S.d_base; p.v_slots = S.d_slots;
  p.stage_window = W;
  p.d_lens = chunked ? c.lens() : nullptr;
  p.old_sub = writer ? 0 : 1;
  HIP_TRY(launch_prefill_tiled(p, s));
  if (writer) {
    int e = commit();
    if (e != MIXATTN_OK) return e;
  }
  return MIXATTN_OK;
}

int mixattn_prefill(mixattn_layout* L, int layer, const void* q, const void* k, const void* v, void* out,
                    int seq_len, void* stream) {
  if (!L || !q || !out) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  if (seq_len < 1) return MIXATTN_ERR_ORDER;
  return prefill_impl(L, layer, q, k, v, out, nullptr, seq_len, stream);
}

int mixattn_prefill_varlen(mixattn_layout* L, int layer, const void* q, const void* k, const void* v, void* out,
                           const int32_t* seq_lens, void* stream) {
  if (!L || !q || !out || !seq_lens) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  int max_len = 0;
  for (int b = 0; b < L->batch; ++b) {
    if (seq_lens[b] < 0) return MIXATTN_ERR_ORDER;
    max_len = std::max(max_len, seq_lens[b]);
  }
  if (max_len < 1) return MIXATTN_ERR_ORDER;
  return prefill_impl(L, layer, q, k, v, out, seq_lens, max_len, stream);
}

int mixattn_load_kv(mixattn_layout* L, int layer, const void* k, const void* v, const int32_t* seq_lens,
                    void* stream) {
  if (!L || !k || !v || !seq_lens) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  Cache& c = L->caches[L->layer_cache[layer]];
  if (c.writer != layer) return MIXATTN_ERR_NOT_WRITER;
  std::vector<int64_t> first(L->batch);
  int64_t run = 0;
  int max_len = 0;
  for (int b = 0; b < L->batch; ++b) {
    if (held(c, b) != 0) return MIXATTN_ERR_ORDER;
    if (seq_lens[b] < 0) return MIXATTN_ERR_ORDER;
    if (c.kind == MIXATTN_FULL && seq_lens[b] > L->capacity[b]) return MIXATTN_ERR_CAPACITY;
    first[b] = run;
    run += seq_lens[b];
    max_len = std::max(max_len, seq_lens[b]);
  }
  hipStream_t s = (hipStream_t)stream;
  if (c.paged) {
    std::vector<int64_t> want(seq_lens, seq_lens + L->batch);
    const int pe = reserve_pages(L, c, want, s);
    if (pe != MIXATTN_OK) return pe;
  }
  retire_stage(L, c);
  // per-sequence tables travel in the arguments of a small kernel: stream-ordered behind any earlier user of them
  HIP_TRY(launch_set_seq_tables(L->d_stage_src, L->d_stage_lens, first.data(), seq_lens, L->batch, s));
  StoreLaunch st;
  st.K = c.K; st.V = c.V; st.d_base = c.d_base; st.d_slots = c.d_slots; st.window = c.window;
  st.pages = c.page_table();
  st.k_src = k; st.v_src = v; st.d_src_first = L->d_stage_src; st.d_src_len = L->d_stage_lens; st.uniform_len = 0;
  st.d_n_old = c.lens(); st.old_sub = 0;  // 0, or idle
  st.batch = L->batch; st.Hkv = L->Hkv; st.D = L->D; st.elem = L->elem;
  st.max_slots = std::max(1, c.window > 0 ? std::min(max_len, c.window) : max_len);
  HIP_TRY(L->tiled ? launch_store_tiled(st, s) : launch_store_rowmajor(st, s));
  HIP_TRY(launch_advance_lens(c.lens(), L->d_stage_lens, 0, L->batch, s));
  for (int b = 0; b < L->batch; ++b)
    if (seq_lens[b] > 0 || !idle(c, b)) c.len[b] = seq_lens[b];  // an idle sequence given nothing stays idle
  c.plan_key = -1;
  return MIXATTN_OK;
}

int mixattn_n_caches(const mixattn_layout* L) { return L ? (int)L->caches.size() : MIXATTN_ERR_NULL; }

int mixattn_cache_of(const mixattn_layout* L, int layer, int* cache_index, int* is_writer) {
  if (!L) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  const int ci = L->layer_cache[layer];
  if (cache_index) *cache_index = ci;
  if (is_writer) *is_writer = L->caches[ci].writer == layer ? 1 : 0;
  return MIXATTN_OK;
}

int mixattn_seq_len(const mixattn_layout* L, int cache_index, int b, int64_t* n) {
  if (!L || !n) return MIXATTN_ERR_NULL;
  if (cache_index < 0 || cache_index >= (int)L->caches.size() || b < 0 || b >= L->batch) return MIXATTN_ERR_LAYER;
  *n = held(L->caches[cache_index], b);
  return MIXATTN_OK;
}

int mixattn_slot_of(const mixattn_layout* L, int cache_index, int64_t pos, int64_t* slot) {
  if (!L || !slot) return MIXATTN_ERR_NULL;
  if (cache_index < 0 || cache_index >= (int)L->caches.size()) return MIXATTN_ERR_LAYER;
  const Cache& c = L->caches[cache_index];
  return mixattn_slot_for(c.kind, c.window, pos, slot);
}

int mixattn_read_cache(mixattn_layout* L, int cache_index, int b, int kv_head, int64_t slot, void* k_row,
                       void* v_row) {
  if (!L) return MIXATTN_ERR_NULL;
  if (cache_index < 0 || cache_index >= (int)L->caches.size() || b < 0 || b >= L->batch || kv_head < 0 ||
      kv_head >= L->Hkv)
    return MIXATTN_ERR_LAYER;
  const Cache& c = L->caches[cache_index];
  const int64_t limit = c.kind == MIXATTN_SLIDING ? c.window : L->capacity[b];
  if (slot < 0 || slot >= limit) return MIXATTN_ERR_LAYER;
  HIP_TRY(hipDeviceSynchronize());
  if (c.paged) {
    // the page that holds the slot, addressed as a one-page cache of its own
    const int64_t page_tokens = (int64_t)kBlockKeys << c.page_shift;
    if (slot / page_tokens >= (int64_t)c.seq_pages[b].size()) return MIXATTN_ERR_LAYER;
    const int64_t pg = c.seq_pages[b][slot / page_tokens];
    HIP_TRY(launch_gather_row(c.K, c.V, (pg * L->Hkv) << c.page_shift, (int32_t)page_tokens, kv_head,
                              slot % page_tokens, L->D, L->elem, true, L->d_readback, nullptr));
  } else {
    HIP_TRY(launch_gather_row(c.K, c.V, c.base[b], c.slots[b], kv_head, slot, L->D, L->elem, L->tiled, L->d_readback,
                              nullptr));
  }
  HIP_TRY(hipDeviceSynchronize());
  const size_t row = (size_t)L->D * L->elem;
  if (k_row) HIP_TRY(hipMemcpy(k_row, L->d_readback, row, hipMemcpyDeviceToHost));
  if (v_row) HIP_TRY(hipMemcpy(v_row, (const char*)L->d_readback + row, row, hipMemcpyDeviceToHost));
  return MIXATTN_OK;
}

int mixattn_read_device_lens(mixattn_layout* L, int cache_index, int32_t* lens) {
  if (!L || !lens) return MIXATTN_ERR_NULL;
  if (cache_index < 0 || cache_index >= (int)L->caches.size()) return MIXATTN_ERR_LAYER;
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(lens, L->caches[cache_index].lens(), sizeof(int32_t) * L->batch, hipMemcpyDeviceToHost));
  return MIXATTN_OK;
}

int64_t mixattn_kv_bytes_allocated(const mixattn_layout* L) {
  if (!L) return MIXATTN_ERR_NULL;
  int64_t t = 0;
  for (const auto& c : L->caches) t += 2 * c.total_elems * L->elem;
  return t;
}

int64_t mixattn_kv_bytes_live(const mixattn_layout* L) {
  if (!L) return MIXATTN_ERR_NULL;
  int64_t tok = 0;
  for (const auto& c : L->caches)
    for (int b = 0; b < L->batch; ++b) tok += c.window > 0 ? std::min<int64_t>(held(c, b), c.window) : held(c, b);
  return tok * 2 * L->Hkv * L->D * L->elem;
}

int64_t mixattn_step_read_bytes(const mixattn_layout* L, int layer) {
  if (!L) return MIXATTN_ERR_NULL;
  if (layer < 0 || layer >= L->n_layers) return MIXATTN_ERR_LAYER;
  const Cache& c = L->caches[L->layer_cache[layer]];
  const int aw = layer_attn_window(L, layer);
  int64_t tok = 0;
  for (int b = 0; b < L->batch; ++b) tok += tokens_read(c, held(c, b), aw);
  return tok * 2 * L->Hkv * L->D * L->elem;
}

int mixattn_set_param(mixattn_layout* L, int param, int64_t value) {
  if (!L) return MIXATTN_ERR_NULL;
  switch (param) {
    case MIXATTN_PARAM_CHUNK_KEYS:
      if (value < 0 || value % kBlockKeys != 0 || value > (int64_t)1 << 30) return MIXATTN_ERR_PARAM;
      L->chunk_keys = value;
      return MIXATTN_OK;
    case MIXATTN_PARAM_TEST_FAIL_ALLOC:
      if (value < 0) return MIXATTN_ERR_PARAM;
      g_fail_alloc_in = value;
      return MIXATTN_OK;
    case MIXATTN_PARAM_PREFILL_SIMPLE:
      if (value != 0 && value != 1) return MIXATTN_ERR_PARAM;
      L->prefill_simple = value;
      return MIXATTN_OK;
    case MIXATTN_PARAM_PREFILL_WAVES:
      if (value != 0 && value != 4 && value != 8) return MIXATTN_ERR_PARAM;
      L->prefill_waves = value;
      return MIXATTN_OK;
    case MIXATTN_PARAM_PREFILL_HEADS:
      if (value != 0 && value != 1 && value != 2 && value != 4) return MIXATTN_ERR_PARAM;
      L->prefill_heads = value;
      return MIXATTN_OK;
    case MIXATTN_PARAM_BALANCED:
      if (value < 0 || value > 2) return MIXATTN_ERR_PARAM;
      L->balanced = value;
      return MIXATTN_OK;
    default: return MIXATTN_ERR_PARAM;
  }
}

int mixattn_get_param(const mixattn_layout* L, int param, int64_t* value) {
  if (!L || !value) return MIXATTN_ERR_NULL;
  switch (param) {
    case MIXATTN_PARAM_CHUNK_KEYS: *value = L->chunk_keys; return MIXATTN_OK;
    case MIXATTN_PARAM_TEST_FAIL_ALLOC: *value = g_fail_alloc_in; return MIXATTN_OK;
    case MIXATTN_PARAM_PREFILL_SIMPLE: *value = L->prefill_simple; return MIXATTN_OK;
    case MIXATTN_PARAM_PREFILL_WAVES: *value = L->prefill_waves; return MIXATTN_OK;
    case MIXATTN_PARAM_PREFILL_HEADS: *value = L->prefill_heads; return MIXATTN_OK;
    case MIXATTN_PARAM_BALANCED: *value = L->balanced; return MIXATTN_OK;
    default: return MIXATTN_ERR_PARAM;
  }
}

}  // extern "C"
