// Host side of librlkv: argument validation, arena planning, the C-ABI entry points.
// All validation runs before the first HIP call, so the error paths work without a GPU.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "rlkv_internal.h"

using namespace rlkv;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }
inline int round_up_tile(int x) { return (x + kTile - 1) / kTile * kTile; }

// Byte offsets of every region inside the arena.
struct Plan {
  size_t full_mask, active, gate, store_off, cap_pad, slotpos_off, len, v_wide, slot_pos, append_cnt;
  size_t lists, part_o, part_m, part_l, block_table, staging, prefill_split, kv;
  size_t list_stride;        // bytes between the work-list blocks of consecutive layers
  int staging_tiles;         // staging tiles per (sequence, KV head) pair for prefill chunks
  int table_stride;          // block-table entries per sequence (0 = contiguous stores)
  size_t total;
  size_t kv_bytes;           // K/V stores only
  int64_t slot_pos_elems;
  int n_compressed;          // compressed (layer, head) count
};

int resolve_kernel(const rlkv_config_t* c) {
  if (c->kernel != RLKV_KERNEL_AUTO) return c->kernel;
  return c->dtype == RLKV_BF16 ? RLKV_KERNEL_MFMA : RLKV_KERNEL_VALU;
}

bool config_valid(const rlkv_config_t* c) {
  if (!c || !c->full_mask || !c->max_len) return false;
  if (c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->batch < 1) return false;
  if (c->n_q_heads % c->n_kv_heads != 0) return false;
  if (c->n_q_heads / c->n_kv_heads > kMaxGroup) return false;
  if (c->head_dim != kHeadDim) return false;
  if (c->sink < 0 || c->recent < 1) return false;
  if ((int64_t)c->sink + c->recent > (1 << 24)) return false;
  if (c->dtype != RLKV_F32 && c->dtype != RLKV_BF16) return false;
  if (c->kernel != RLKV_KERNEL_AUTO && c->kernel != RLKV_KERNEL_VALU && c->kernel != RLKV_KERNEL_MFMA) return false;
  if (c->kernel == RLKV_KERNEL_MFMA && c->dtype != RLKV_BF16) return false;
  if (c->device < 0) return false;
  if ((int64_t)c->batch * c->n_kv_heads > 65535) return false;   // pairs index one grid dimension of several launches
  for (int b = 0; b < c->batch; ++b)
    if (c->max_len[b] < 1 || c->max_len[b] > (1 << 24)) return false;
  for (int i = 0; i < c->n_layers * c->n_kv_heads; ++i)
    if (c->full_mask[i] > 1) return false;
  if (c->page_tokens != 0) {
    const int p = c->page_tokens;
    if (p < kTile || p > 65536 || (p & (p - 1)) != 0) return false;
    if (c->pool_pages < 1 || c->pool_pages > (1 << 24)) return false;
    if (resolve_kernel(c) != RLKV_KERNEL_MFMA) return false;      // paging exists for the tiled layout only
  }
  if (c->prefill_tokens < 0 || c->prefill_tokens > (1 << 20)) return false;
  if (c->prefill_tokens > 0 && resolve_kernel(c) != RLKV_KERNEL_MFMA) return false;
  if (c->decode_wgs_per_cu < 0 || c->decode_wgs_per_cu > 8) return false;
  if (c->prefill_min_share_tiles < 0 || c->prefill_min_share_tiles > (1 << 20)) return false;
  if (c->prefill_two_group_only < 0 || c->prefill_two_group_only > 1) return false;
  return true;
}

// Pages a sequence of n tokens holds.
int pages_for(int n, int page_tokens) { return (n + page_tokens - 1) / page_tokens; }

// Layout of a layer's work-list block: [ListHeader][WgDesc x n_wg][PairDesc x n_pairs] (see rlkv_internal.h).
size_t list_pair_offset(int n_wg) { return align_up(sizeof(ListHeader) + (size_t)n_wg * sizeof(WgDesc)); }
size_t list_block_bytes(int n_wg, int n_pairs) { return align_up(list_pair_offset(n_wg) + (size_t)n_pairs * sizeof(PairDesc)); }

void make_plan(const rlkv_config_t* c, Plan* p) {
  const size_t L = c->n_layers, H = c->n_kv_heads, B = c->batch;
  const size_t G = c->n_q_heads / c->n_kv_heads;
  const size_t W = (size_t)c->sink + c->recent;
  const size_t row = (size_t)c->head_dim * (c->dtype == RLKV_F32 ? 4 : 2);
  size_t n_comp = 0;
  for (size_t i = 0; i < L * H; ++i) n_comp += c->full_mask[i] ? 0 : 1;
  p->n_compressed = (int)n_comp;
  p->slot_pos_elems = (int64_t)(n_comp * B * W);
  const size_t n_pairs = B * H;
  const size_t slots = kMaxWorkgroups + n_pairs;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  p->full_mask = take(L * H);
  p->active = take(B);
  p->gate = take(L * H * sizeof(float));
  p->store_off = take(L * B * H * sizeof(int64_t));
  p->cap_pad = take(B * sizeof(int32_t));
  p->slotpos_off = take(L * H * sizeof(int64_t));
  p->len = take(2 * L * B * sizeof(int32_t));
  p->v_wide = take(L * sizeof(int32_t));              // (between len and slot_pos: zeroed with the lengths)
  p->slot_pos = take((size_t)p->slot_pos_elems * sizeof(int32_t));
  p->append_cnt = take(2 * B * sizeof(int32_t));      // token counts, then the prefill's sequence order
  p->list_stride = list_block_bytes(kMaxWorkgroups, (int)n_pairs);
  p->lists = take(L * p->list_stride);
  p->part_o = take(2 * slots * G * kHeadDim * sizeof(float));   // two sets: full / local pass of gated heads
  p->part_m = take(2 * slots * G * sizeof(float));
  p->part_l = take(2 * slots * G * sizeof(float));
  p->table_stride = 0;
  if (c->page_tokens > 0)
    for (size_t b = 0; b < B; ++b) p->table_stride = std::max(p->table_stride, pages_for(c->max_len[b], c->page_tokens));
  p->block_table = take(B * (size_t)p->table_stride * sizeof(int32_t));
  p->staging_tiles = (c->prefill_tokens + kTile - 1) / kTile;
  p->staging = take(n_pairs * (size_t)p->staging_tiles * kTileBytes);
  p->prefill_split = take(c->prefill_tokens > 0 ? kPrefillSplitSlots * kPrefillSplitSlotBytes : 0);
  p->kv = o;
  size_t sum_full = 0;   // tokens of one full head over all sequences (paged: of its pool)
  if (c->page_tokens > 0) {
    sum_full = (size_t)c->pool_pages * c->page_tokens;
  } else {
    for (size_t b = 0; b < B; ++b) sum_full += (size_t)round_up_tile(c->max_len[b]);
  }
  const size_t comp_tokens = (size_t)round_up_tile((int)W) * B;
  size_t kv = 0;
  for (size_t i = 0; i < L * H; ++i) kv += 2 * row * (c->full_mask[i] ? sum_full : comp_tokens);
  p->kv_bytes = kv;
  p->total = align_up(o + kv);
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

}  // namespace

// ---- static scratch of the allocation-free entry point (rlkv_decode_attention_noalloc) --------------------
// The split-K partials of that call live here instead of in the arena: one row per (partial slot, query head)
// of kHeadDim accumulator values, plus the row's maximum and normaliser.  Every GPU the library runs on holds its
// own copy of the array until the process ends.  In host code the array's name is only a stand-in: the device
// address comes from hipGetSymbolAddress, once per device, and is what kernels and copies are given.
constexpr int kStaticRows = 16384;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) float scratch[(size_t)kStaticRows * (kHeadDim + 2)];     // 8.1 MiB
static float* g_scratch_ptr[kMaxDevices];           // per device, nullptr = not looked up yet
static std::mutex& scratch_lock() { static std::mutex m; return m; }

// Device address of `scratch` on `device`, which must be the current device.  nullptr on failure.
static float* scratch_on_device(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> g(scratch_lock());
  if (!g_scratch_ptr[device]) {
    float* ptr = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[device] = ptr;
  }
  return g_scratch_ptr[device];
}

struct rlkv_cache {
  rlkv_config_t cfg;
  std::vector<uint8_t> mask;        // host copy [L][Hkv]
  std::vector<int32_t> max_len;     // host copy [B]
  std::vector<int32_t> len_host;    // host mirror of the lengths [L][B]
  std::vector<int32_t> wl_slack;    // [L] tokens the layer's work list is still valid for; -1 = rebuild
  std::vector<int64_t> decode_calls; // [L] decode launches so far (fused or not): the clock of the rebuild schedule
  std::vector<uint8_t> step_ready;  // [L] a fused step was prepared (rlkv_append_decode_prepare) and no launch has run since
  int64_t lists_built = 0;          // work lists planned and sent so far
  std::vector<uint8_t> parity;      // [L] which copy of the device lengths is current
  std::vector<uint8_t> active;      // [B] host copy of the active-slot table
  std::vector<float> gate;          // [L][Hkv] host copy of the Eq. 1 gates
  std::vector<uint8_t> layer_gated; // [L] some full head of the layer has a gate below 1
  std::vector<uint32_t> merge_words; // [L][pairs] (first partial slot << 12) | partials of the layer's work list; empty if too many pairs
  int n_cu;                         // compute units of the device
  int min_share_tiles;              // a divided prefill workgroup's share is at least this many tiles
  bool allow_narrow;                // prefill may pick the one-group kernel form for a layer that does not blend
  DeviceView dv;
  Plan plan;
  char* arena;
  bool owns_arena;
  // paged full heads: the block table and the free list live on the host, the device copy of the
  // table follows through launch_table_update
  std::vector<int32_t> free_pages;       // stack of free page indices
  std::vector<int32_t> pages_held;       // [B] pages the sequence holds
  std::vector<int32_t> table_host;       // [B][table_stride]
  // work lists are planned on the host and copied over: host copies of the tables the records need,
  // and pinned staging slots (one per layer up to a budget) with an event each that tells when
  // the slot's last copy has run
  std::vector<int64_t> store_off_host;   // [L][B][Hkv]
  std::vector<int32_t> cap_pad_host;     // [B]
  std::vector<int32_t> plan_rounds, plan_begin, plan_first, plan_count;   // scratch of the planner
  // One block of pinned host memory, cut into two rings of staging slots.  Every slot has an event that tells
  // when the last copy out of it has run, so a slot is rewritten only after the device has read it.
  char* pinned = nullptr;
  size_t pinned_bytes = 0;
  struct Ring {
    char* base = nullptr;
    size_t slot_bytes = 0;
    int n = 0, next = 0;
    std::vector<hipEvent_t> events;
    std::vector<uint8_t> busy;
  };
  Ring list_ring;                        // work lists (one slot per layer up to a budget)
  Ring small_ring;                       // token counts, the active table, the gates
  hipStream_t last_stream = nullptr;     // the stream of the latest call that queued work
  std::vector<int32_t> new_len;          // [2B] host staging: new lengths for reserve_pages, counts + order for prefill
  std::vector<hipEvent_t> prof_events;   // start/stop pairs, created by rlkv_profile_enable
  int prof_used = 0;                     // pairs recorded so far
};

// Pinned staging blocks are kept for the life of the process and handed from one cache to the
// next: mapping and unmapping pinned host memory is slow and disturbs work in flight.
struct PinnedBlock { char* ptr; size_t bytes; };
static std::vector<PinnedBlock>& pinned_pool() { static std::vector<PinnedBlock> pool; return pool; }
static std::mutex& pinned_pool_lock() { static std::mutex m; return m; }

static char* acquire_pinned(size_t bytes, size_t* got) {
  {
    std::lock_guard<std::mutex> g(pinned_pool_lock());
    std::vector<PinnedBlock>& pool = pinned_pool();
    for (size_t i = 0; i < pool.size(); ++i)
      if (pool[i].bytes >= bytes) {
        PinnedBlock b = pool[i];
        pool.erase(pool.begin() + i);
        *got = b.bytes;
        return b.ptr;
      }
  }
  void* host = nullptr;
  if (hipHostMalloc(&host, bytes, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  *got = bytes;
  return static_cast<char*>(host);
}

static void release_host_staging(rlkv_cache_t* cache) {
  for (rlkv_cache::Ring* r : {&cache->list_ring, &cache->small_ring}) {
    for (hipEvent_t ev : r->events) (void)hipEventDestroy(ev);
    r->events.clear();
  }
  if (cache->pinned) {
    std::lock_guard<std::mutex> g(pinned_pool_lock());
    pinned_pool().push_back(PinnedBlock{cache->pinned, cache->pinned_bytes});
  }
  cache->pinned = nullptr;
}

// The next slot of a ring, once the copy that last read it has run (it has, unless the host is a whole
// round of slots ahead of the device); nullptr on a HIP error.
static char* ring_take(rlkv_cache::Ring& r, int* slot) {
  *slot = r.next;
  r.next = (r.next + 1) % r.n;
  if (r.busy[*slot] && hipEventSynchronize(r.events[*slot]) != hipSuccess) return nullptr;
  r.busy[*slot] = 0;
  return r.base + (size_t)*slot * r.slot_bytes;
}
// Marks the slot as read by the copies queued on `s` so far.
static bool ring_sent(rlkv_cache::Ring& r, int slot, hipStream_t s) {
  if (hipEventRecord(r.events[slot], s) != hipSuccess) return false;
  r.busy[slot] = 1;
  return true;
}
// Copies `bytes` of host memory to the device through a pinned slot: the caller's memory is free again
// when this returns, whatever the stream is doing.
static bool send_small(rlkv_cache_t* cache, void* dst, const void* src, size_t bytes, hipStream_t s) {
  int slot;
  char* stage = ring_take(cache->small_ring, &slot);
  if (!stage || bytes > cache->small_ring.slot_bytes) return false;
  memcpy(stage, src, bytes);
  if (hipMemcpyAsync(dst, stage, bytes, hipMemcpyHostToDevice, s) != hipSuccess) return false;
  return ring_sent(cache->small_ring, slot, s);
}

// Waits for everything this handle has queued (on the stream it was last used on).
static bool wait_for_cache(rlkv_cache_t* cache) { return hipStreamSynchronize(cache->last_stream) == hipSuccess; }

static void drop_profile_events(rlkv_cache_t* cache) {
  for (hipEvent_t ev : cache->prof_events) (void)hipEventDestroy(ev);
  cache->prof_events.clear();
  cache->prof_used = 0;
}

extern "C" {

size_t rlkv_cache_required_bytes(const rlkv_config_t* cfg) {
  if (!config_valid(cfg)) return 0;
  Plan p;
  make_plan(cfg, &p);
  return p.total;
}

rlkv_status_t rlkv_cache_create(const rlkv_config_t* cfg, rlkv_cache_t** out) {
  if (!out) return RLKV_ERR_INVALID_ARG;
  *out = nullptr;
  if (!config_valid(cfg)) return RLKV_ERR_INVALID_ARG;
  Plan p;
  make_plan(cfg, &p);
  if (cfg->arena) {
    if (reinterpret_cast<uintptr_t>(cfg->arena) % kAlign != 0) return RLKV_ERR_INVALID_ARG;
    if (cfg->arena_bytes < p.total) return RLKV_ERR_OOM;
  }
  rlkv_cache* c = new (std::nothrow) rlkv_cache();
  if (!c) return RLKV_ERR_OOM;
  c->cfg = *cfg;
  const int L = cfg->n_layers, H = cfg->n_kv_heads, B = cfg->batch;
  c->mask.assign(cfg->full_mask, cfg->full_mask + (size_t)L * H);
  c->max_len.assign(cfg->max_len, cfg->max_len + B);
  c->len_host.assign((size_t)L * B, 0);
  c->wl_slack.assign((size_t)L, -1);
  c->decode_calls.assign((size_t)L, 0);
  c->step_ready.assign((size_t)L, 0);
  c->parity.assign((size_t)L, 0);
  c->active.assign((size_t)B, 1);
  c->gate.assign((size_t)L * H, 1.f);
  c->layer_gated.assign((size_t)L, 0);
  if (B * H <= kMergeArgPairs) c->merge_words.assign((size_t)L * B * H, 0);
  if (cfg->page_tokens > 0) {
    c->free_pages.resize((size_t)cfg->pool_pages);
    for (int i = 0; i < cfg->pool_pages; ++i) c->free_pages[i] = cfg->pool_pages - 1 - i;   // page 0 on top
    c->pages_held.assign((size_t)B, 0);
    c->table_host.assign((size_t)B * p.table_stride, 0);
  }
  c->new_len.assign((size_t)2 * B, 0);
  c->cfg.full_mask = c->mask.data();
  c->cfg.max_len = c->max_len.data();
  c->cfg.kernel = resolve_kernel(cfg);
  c->plan = p;
  c->owns_arena = false;
  c->arena = nullptr;

  // ---- first HIP calls ------------------------------------------------------------
  if (hipSetDevice(cfg->device) != hipSuccess) { delete c; return RLKV_ERR_HIP; }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, cfg->device) != hipSuccess) { delete c; return RLKV_ERR_HIP; }
  if (cfg->arena) {
    c->arena = static_cast<char*>(cfg->arena);
  } else {
    void* ptr = nullptr;
    if (hipMalloc(&ptr, p.total) != hipSuccess) { (void)hipGetLastError(); delete c; return RLKV_ERR_OOM; }
    c->arena = static_cast<char*>(ptr);
    c->owns_arena = true;
  }

  if (!scratch_on_device(cfg->device)) {     // set-up of the allocation-free entry point, once per device
    if (c->owns_arena) (void)hipFree(c->arena);
    delete c;
    return RLKV_ERR_HIP;
  }
  c->n_cu = prop.multiProcessorCount;
  // Measured on the Qwen shape, one sequence: dividing beats the narrow form from about 85 tiles per share on
  // (the shares' accumulators go through memory and a merge kernel follows).
  c->min_share_tiles = cfg->prefill_min_share_tiles > 0 ? cfg->prefill_min_share_tiles : 80;
  c->allow_narrow = cfg->prefill_two_group_only == 0;
  // measured best: one 4-wave workgroup per CU (see decode_mfma.hip)
  const int wgs_per_cu = cfg->decode_wgs_per_cu > 0 ? cfg->decode_wgs_per_cu : 1;
  int n_wg = prop.multiProcessorCount * wgs_per_cu;
  if (n_wg > kMaxWorkgroups) n_wg = kMaxWorkgroups;
  if (n_wg < 1) n_wg = 1;

  DeviceView& dv = c->dv;
  dv.n_layers = L; dv.n_q_heads = cfg->n_q_heads; dv.n_kv_heads = H; dv.group = cfg->n_q_heads / H;
  dv.batch = B; dv.sink = cfg->sink; dv.recent = cfg->recent; dv.window = cfg->sink + cfg->recent;
  dv.window_pad = round_up_tile(dv.window);
  dv.dtype = cfg->dtype; dv.kernel = c->cfg.kernel;
  dv.row_bytes = cfg->head_dim * (cfg->dtype == RLKV_F32 ? 4 : 2);
  dv.n_pairs = B * H; dv.n_wg = n_wg;
  char* a = c->arena;
  dv.full_mask = reinterpret_cast<uint8_t*>(a + p.full_mask);
  dv.active = reinterpret_cast<uint8_t*>(a + p.active);
  dv.gate = reinterpret_cast<float*>(a + p.gate);
  dv.store_off = reinterpret_cast<int64_t*>(a + p.store_off);
  dv.cap_pad = reinterpret_cast<int32_t*>(a + p.cap_pad);
  dv.slotpos_off = reinterpret_cast<int64_t*>(a + p.slotpos_off);
  dv.len = reinterpret_cast<int32_t*>(a + p.len);
  dv.slot_pos = reinterpret_cast<int32_t*>(a + p.slot_pos);
  dv.v_wide = reinterpret_cast<int32_t*>(a + p.v_wide);
  dv.append_cnt = reinterpret_cast<int32_t*>(a + p.append_cnt);
  dv.list_base = a + p.lists;
  dv.list_stride = (int64_t)p.list_stride;
  dv.list_pair_off = (int32_t)list_pair_offset(n_wg);
  dv.part_o = reinterpret_cast<float*>(a + p.part_o);
  dv.part_m = reinterpret_cast<float*>(a + p.part_m);
  dv.part_l = reinterpret_cast<float*>(a + p.part_l);
  {
    const int64_t slots = kMaxWorkgroups + (int64_t)B * H;
    dv.part_set_ml = slots * dv.group;
    dv.part_set_o = dv.part_set_ml * kHeadDim;
  }
  dv.kv_base = a + p.kv;
  dv.block_table = reinterpret_cast<int32_t*>(a + p.block_table);
  dv.table_stride = p.table_stride;
  dv.page_shift = -1; dv.page_mask = 0; dv.page_bytes = 0;
  if (cfg->page_tokens > 0) {
    const int tiles = cfg->page_tokens / kTile;
    dv.page_shift = 0;
    while ((1 << dv.page_shift) < tiles) ++dv.page_shift;
    dv.page_mask = tiles - 1;
    dv.page_bytes = (int64_t)tiles * kTileBytes;
  }

  // host-built tables
  std::vector<int32_t> cap_pad(B);
  size_t sum_full_bytes = 0;
  std::vector<size_t> seq_off(B);
  for (int b = 0; b < B; ++b) {
    cap_pad[b] = round_up_tile(cfg->max_len[b]);
    seq_off[b] = sum_full_bytes;
    sum_full_bytes += (size_t)cap_pad[b] * dv.row_bytes * 2;
  }
  if (cfg->page_tokens > 0) {
    // a full head's store is its pool: one offset for all sequences, pages through the block table
    for (int b = 0; b < B; ++b) seq_off[b] = 0;
    sum_full_bytes = (size_t)cfg->pool_pages * (size_t)dv.page_bytes;
  }
  const size_t comp_bytes = (size_t)dv.window_pad * dv.row_bytes * 2;
  std::vector<int64_t> store_off((size_t)L * B * H), slotpos_off((size_t)L * H);
  size_t o = 0;
  int64_t sp = 0;
  for (int l = 0; l < L; ++l) {
    for (int h = 0; h < H; ++h) {
      const bool full = c->mask[(size_t)l * H + h] != 0;
      for (int b = 0; b < B; ++b)
        store_off[((size_t)l * B + b) * H + h] = (int64_t)(o + (full ? seq_off[b] : comp_bytes * b));
      o += full ? sum_full_bytes : comp_bytes * B;
      slotpos_off[(size_t)l * H + h] = full ? -1 : sp;
      if (!full) sp += (int64_t)B * dv.window;
    }
  }
  c->store_off_host = store_off;
  c->cap_pad_host = cap_pad;
  c->plan_rounds.resize((size_t)B * H);
  c->plan_first.resize((size_t)B * H);
  c->plan_count.resize((size_t)B * H);
  c->plan_begin.resize((size_t)n_wg + 1);
  bool ok = true;
  {
    rlkv_cache::Ring& lr = c->list_ring;
    rlkv_cache::Ring& sr = c->small_ring;
    lr.slot_bytes = list_block_bytes(n_wg, B * H);
    const size_t budget = (size_t)64 << 20;
    size_t slots = L;
    if (slots * lr.slot_bytes > budget) slots = budget / lr.slot_bytes;
    if (slots < 2) slots = 2;
    lr.n = (int)slots;
    sr.slot_bytes = align_up(std::max({(size_t)2 * B * sizeof(int32_t), (size_t)L * H * sizeof(float), (size_t)B}));
    sr.n = 64;
    c->pinned = acquire_pinned(lr.slot_bytes * lr.n + sr.slot_bytes * sr.n, &c->pinned_bytes);
    ok &= c->pinned != nullptr;
    lr.base = c->pinned;
    sr.base = c->pinned + lr.slot_bytes * lr.n;
    for (rlkv_cache::Ring* r : {&lr, &sr}) {
      r->busy.assign((size_t)r->n, 0);
      for (int i = 0; ok && i < r->n; ++i) {
        hipEvent_t ev;
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess) r->events.push_back(ev);
        else ok = false;
      }
    }
  }
  ok &= hipMemcpy(a + p.full_mask, c->mask.data(), c->mask.size(), hipMemcpyHostToDevice) == hipSuccess;
  ok &= hipMemcpy(a + p.active, c->active.data(), c->active.size(), hipMemcpyHostToDevice) == hipSuccess;
  ok &= hipMemcpy(a + p.gate, c->gate.data(), c->gate.size() * sizeof(float), hipMemcpyHostToDevice) == hipSuccess;
  ok &= hipMemcpy(a + p.store_off, store_off.data(), store_off.size() * 8, hipMemcpyHostToDevice) == hipSuccess;
  ok &= hipMemcpy(a + p.cap_pad, cap_pad.data(), cap_pad.size() * 4, hipMemcpyHostToDevice) == hipSuccess;
  ok &= hipMemcpy(a + p.slotpos_off, slotpos_off.data(), slotpos_off.size() * 8, hipMemcpyHostToDevice) == hipSuccess;
  // lengths, staged counts and work lists start at zero; ring slots start empty (-1)
  ok &= hipMemset(a + p.len, 0, p.slot_pos - p.len) == hipSuccess;
  if (p.append_cnt > p.slot_pos) ok &= hipMemset(a + p.slot_pos, 0xff, p.append_cnt - p.slot_pos) == hipSuccess;
  ok &= hipMemset(a + p.append_cnt, 0, p.part_o - p.append_cnt) == hipSuccess;
  if (p.staging > p.block_table) ok &= hipMemset(a + p.block_table, 0, p.staging - p.block_table) == hipSuccess;
  ok &= hipStreamSynchronize(nullptr) == hipSuccess;     // the fills above ran on the null stream
  if (!ok) {
    release_host_staging(c);
    if (c->owns_arena) (void)hipFree(c->arena);
    delete c;
    return RLKV_ERR_HIP;
  }
  *out = c;
  return RLKV_OK;
}

rlkv_status_t rlkv_cache_destroy(rlkv_cache_t* cache) {
  if (!cache) return RLKV_ERR_INVALID_ARG;
  rlkv_status_t st = RLKV_OK;
  drop_profile_events(cache);
  (void)hipSetDevice(cache->cfg.device);
  (void)wait_for_cache(cache);           // a copy out of the pinned staging may still be queued
  release_host_staging(cache);
  if (cache->owns_arena && cache->arena) {
    if (hipFree(cache->arena) != hipSuccess) st = RLKV_ERR_HIP;
  }
  delete cache;
  return st;
}

rlkv_status_t rlkv_cache_reset(rlkv_cache_t* cache, int32_t seq, void* stream) {
  if (!cache) return RLKV_ERR_INVALID_ARG;
  if (seq < -1 || seq >= cache->cfg.batch) return RLKV_ERR_INVALID_ARG;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  cache->last_stream = as_stream(stream);
  if (launch_reset(cache->dv, seq, cache->plan.slot_pos_elems, as_stream(stream)) != hipSuccess) return RLKV_ERR_HIP;
  const int L = cache->cfg.n_layers, B = cache->cfg.batch;
  for (int l = 0; l < L; ++l)
    for (int b = 0; b < B; ++b)
      if (seq < 0 || b == seq) cache->len_host[(size_t)l * B + b] = 0;
  for (int l = 0; l < L; ++l) cache->wl_slack[l] = -1;
  if (cache->cfg.page_tokens > 0) {
    // the pages go back to the free list at once; whoever gets them next writes them in stream
    // order, after every kernel that still reads them for this sequence
    for (int b = 0; b < B; ++b) {
      if (seq >= 0 && b != seq) continue;
      const int32_t* row = cache->table_host.data() + (size_t)b * cache->plan.table_stride;
      for (int i = cache->pages_held[b] - 1; i >= 0; --i) cache->free_pages.push_back(row[i]);
      cache->pages_held[b] = 0;
    }
  }
  return RLKV_OK;
}

// Paged caches: gives every sequence the pages it needs to hold new_len[b] tokens (new_len = the
// layer's lengths after the append about to be launched) and sends the new block-table entries
// to the device on `s`.  RLKV_ERR_CAPACITY, with nothing changed, if the free list is too short.
static rlkv_status_t reserve_pages(rlkv_cache_t* cache, const std::vector<int32_t>& new_len, hipStream_t s) {
  const int P = cache->cfg.page_tokens;
  if (P <= 0) return RLKV_OK;
  const int B = cache->cfg.batch, stride = cache->plan.table_stride;
  size_t want = 0;
  for (int b = 0; b < B; ++b) {
    const int need = pages_for(new_len[b], P);
    if (need > cache->pages_held[b]) want += (size_t)(need - cache->pages_held[b]);
  }
  if (want == 0) return RLKV_OK;
  if (want > cache->free_pages.size()) return RLKV_ERR_CAPACITY;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  TableUpdates up;
  up.n = 0;
  for (int b = 0; b < B; ++b) {
    const int need = pages_for(new_len[b], P);
    while (cache->pages_held[b] < need) {
      const int32_t page = cache->free_pages.back();
      cache->free_pages.pop_back();
      const int idx = b * stride + cache->pages_held[b]++;
      cache->table_host[idx] = page;
      up.index[up.n] = idx;
      up.value[up.n] = page;
      if (++up.n == kTableUpdateMax) {
        if (launch_table_update(cache->dv, up, s) != hipSuccess) return RLKV_ERR_HIP;
        up.n = 0;
      }
    }
  }
  if (launch_table_update(cache->dv, up, s) != hipSuccess) return RLKV_ERR_HIP;
  return RLKV_OK;
}

// What rlkv_prefill_attention adds to a ragged append: attention of the chunk's queries, run after
// every capacity check has passed and before the chunk's rows go into the stores.
struct PrefillArgs {
  const void* q;
  void* out;
  float softmax_scale;
};

static rlkv_status_t append_impl(rlkv_cache_t* cache, int32_t layer, const void* k, const void* v,
                                 const int32_t* n_tokens, int32_t uniform, int32_t stride, void* stream,
                                 const PrefillArgs* prefill = nullptr) {
  if (!cache || !k || !v) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  const int B = cache->cfg.batch;
  int max_tok = 0;
  if (n_tokens) {
    if (stride < 1) return RLKV_ERR_INVALID_ARG;
    for (int b = 0; b < B; ++b) {
      if (n_tokens[b] < 0 || n_tokens[b] > stride) return RLKV_ERR_INVALID_ARG;
      if (n_tokens[b] > max_tok) max_tok = n_tokens[b];
    }
  } else {
    if (uniform < 1) return RLKV_ERR_INVALID_ARG;
    max_tok = uniform;
  }
  int32_t* lh = cache->len_host.data() + (size_t)layer * B;
  auto tokens_of = [&](int b) -> int { return n_tokens ? n_tokens[b] : (cache->active[b] ? uniform : 0); };
  for (int b = 0; b < B; ++b)
    if ((int64_t)lh[b] + tokens_of(b) > cache->max_len[b]) return RLKV_ERR_CAPACITY;
  if (max_tok == 0) return RLKV_OK;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  hipStream_t s = as_stream(stream);
  if (cache->cfg.page_tokens > 0) {
    for (int b = 0; b < B; ++b) cache->new_len[b] = lh[b] + tokens_of(b);
    if (rlkv_status_t st = reserve_pages(cache, cache->new_len, s)) return st;
  }
  cache->last_stream = s;
  if (prefill) {
    // counts, then the sequences ordered by the keys their chunk attends over, longest first: the
    // prefill kernel hands its longest workgroups out first
    std::vector<int32_t>& stage = cache->new_len;
    stage.resize((size_t)2 * B);
    for (int b = 0; b < B; ++b) { stage[b] = n_tokens[b]; stage[B + b] = b; }
    // (sequences without a chunk last: the rows of the grid that do something then come first, which is
    // what the scratch slots of divided workgroups are counted by)
    std::stable_sort(stage.begin() + B, stage.end(), [&](int32_t x, int32_t y) {
      if ((n_tokens[x] > 0) != (n_tokens[y] > 0)) return n_tokens[x] > 0;
      return (int64_t)lh[x] + n_tokens[x] > (int64_t)lh[y] + n_tokens[y];
    });
    if (!send_small(cache, cache->dv.append_cnt, stage.data(), (size_t)2 * B * sizeof(int32_t), s)) return RLKV_ERR_HIP;
  } else if (n_tokens) {
    if (!send_small(cache, cache->dv.append_cnt, n_tokens, (size_t)B * sizeof(int32_t), s)) return RLKV_ERR_HIP;
  }
  const int par = cache->parity[layer];
  if (prefill) {
    const bool record = (size_t)cache->prof_used * 2 + 1 < cache->prof_events.size();
    hipEvent_t e0 = record ? cache->prof_events[2 * cache->prof_used] : nullptr;
    hipEvent_t e1 = record ? cache->prof_events[2 * cache->prof_used + 1] : nullptr;
    // The kernel form and the division of long workgroups: rlkv_plan_prefill_form (a blending layer always takes
    // the single-group form, undivided).
    bool narrow = cache->layer_gated[layer] != 0;
    int n_split = 1, n_full = 0, split_rows = 0;      // split_rows: grid rows of full heads that have a chunk (they come first)
    {
      const int H = cache->cfg.n_kv_heads;
      for (int h = 0; h < H; ++h) n_full += cache->mask[(size_t)layer * H + h] ? 1 : 0;
    }
    if (!narrow) {
      int32_t nw = 0, ns = 1;
      if (rlkv_plan_prefill_form(cache->n_cu, cache->cfg.n_q_heads, cache->cfg.n_kv_heads, n_full, B, n_tokens, lh,
                                 cache->min_share_tiles, cache->allow_narrow ? 1 : 0, &nw, &ns) != 0)
        return RLKV_ERR_INVALID_ARG;
      narrow = nw != 0;
      n_split = ns;
    }
    int32_t dealt_rows = 0;
    {
      int32_t heavy = 0;
      if (rlkv_plan_prefill_rows(n_full, B, n_tokens, lh, &dealt_rows, &heavy) != 0) return RLKV_ERR_INVALID_ARG;
      split_rows = heavy;
    }
    if (launch_prefill_mfma(cache->dv, layer, narrow, len_of(cache->dv, par, layer), prefill->q,
                            k, v, prefill->out, stride,
                            max_tok, prefill->softmax_scale * 1.44269504088896340736f, cache->arena + cache->plan.staging,
                            cache->plan.staging_tiles, n_split,
                            reinterpret_cast<float*>(cache->arena + cache->plan.prefill_split), split_rows, dealt_rows,
                            cache->mask.data() + (size_t)layer * cache->cfg.n_kv_heads, s, e0,
                            e1) != hipSuccess)
      return RLKV_ERR_HIP;
    if (record) ++cache->prof_used;
  }
  if (launch_append(cache->dv, layer, len_of(cache->dv, par, layer), len_of(cache->dv, par ^ 1, layer), k, v,
                    uniform, stride, n_tokens != nullptr, max_tok, s) != hipSuccess)
    return RLKV_ERR_HIP;
  cache->parity[layer] = par ^ 1;
  for (int b = 0; b < B; ++b) lh[b] += tokens_of(b);
  // the work list tracks growth as one number per layer: uniform appends keep it valid
  int32_t& slack = cache->wl_slack[layer];
  slack = (!n_tokens && slack >= max_tok) ? slack - max_tok : -1;
  return RLKV_OK;
}

// Makes sure the layer's work list covers the current lengths plus `growth` more tokens.  The list
// is planned here, on the host, from the mirror of the lengths (see share_plan.hip), written into
// a pinned staging slot and copied to the device on `s`: no kernel, no synchronisation.
static rlkv_status_t ensure_worklist(rlkv_cache_t* cache, int32_t layer, int growth, hipStream_t s) {
  if (cache->wl_slack[layer] >= growth) return RLKV_OK;
  const DeviceView& dv = cache->dv;
  const int B = dv.batch, H = dv.n_kv_heads, n_pairs = dv.n_pairs, n_wg = dv.n_wg;
  const int32_t* lh = cache->len_host.data() + (size_t)layer * B;
  const uint8_t* mask = cache->mask.data() + (size_t)layer * H;
  int32_t* rounds = cache->plan_rounds.data();
  for (int pi = 0; pi < n_pairs; ++pi) {
    const int b = pi / H, h = pi % H;
    const int limit = mask[h] ? cache->cap_pad_host[b] : dv.window;       // what the store can ever hold
    const int n_fut = lh[b] + kWorklistSlack < limit ? lh[b] + kWorklistSlack : limit;
    rounds[pi] = cache->active[b] ? (n_fut + kTile * kRound - 1) / (kTile * kRound) : 0;   // inactive slots are not attended
  }
  int32_t* wg_begin = cache->plan_begin.data();
  int32_t* seg_first = cache->plan_first.data();
  int32_t* seg_count = cache->plan_count.data();
  plan_shares(rounds, n_pairs, n_wg, wg_begin, seg_first, seg_count);

  int slot;
  char* base = ring_take(cache->list_ring, &slot);
  if (!base) return RLKV_ERR_HIP;
  ListHeader* hd = reinterpret_cast<ListHeader*>(base);
  WgDesc* wd = reinterpret_cast<WgDesc*>(base + sizeof(ListHeader));
  PairDesc* pd = reinterpret_cast<PairDesc*>(base + dv.list_pair_off);
  memset(hd, 0, sizeof(ListHeader));          // grow = 0: the lengths in the records are the current ones
  int32_t us = 0;
  for (int pi = 0; pi < n_pairs; ++pi) {
    const int b = pi / H, h = pi % H;
    const bool full = mask[h] != 0;
    PairDesc& d = pd[pi];
    d.koff = cache->store_off_host[((size_t)layer * B + b) * H + h];
    d.cap = full ? cache->cap_pad_host[b] : dv.window_pad;
    d.n_build = lh[b];
    d.unit_start = us;
    us += rounds[pi] ? rounds[pi] + kPairOverheadUnits : 0;
    d.unit_end = us;
    d.wg_first = seg_first[pi];
    d.full = full ? 1 : 0;
    d.gate = full ? cache->gate[(size_t)layer * H + h] : 1.f;
    d.n_seg = seg_count[pi];
    if (!cache->merge_words.empty())
      cache->merge_words[(size_t)layer * n_pairs + pi] = ((uint32_t)(seg_first[pi] + pi) << 12) | (uint32_t)seg_count[pi];
  }
  int pi = 0;
  for (int w = 0; w < n_wg; ++w) {
    WgDesc& d = wd[w];
    d.u_begin = wg_begin[w];
    d.u_end = wg_begin[w + 1];
    d.pad = 0;
    if (d.u_begin >= d.u_end) {
      d.first_pair = 0;
      d.u_begin = d.u_end = 0;
      d.first = PairDesc{0, 0, 0, 0, 0, 0, 0, 1.f, 0};
    } else {
      while (pd[pi].unit_end <= d.u_begin) ++pi;      // the pair that holds the share's first unit
      d.first_pair = pi;
      d.first = pd[pi];
    }
  }
  const size_t bytes = (size_t)dv.list_pair_off + (size_t)n_pairs * sizeof(PairDesc);
  bool ok = hipMemcpyAsync(dv.list_base + layer * dv.list_stride, base, bytes, hipMemcpyHostToDevice, s) == hipSuccess;
  ok = ok && ring_sent(cache->list_ring, slot, s);
  if (!ok) return RLKV_ERR_HIP;
  // A list serves kWorklistSlack tokens of growth.  The layers' rebuilds are spread over that many steps instead of
  // all falling into one: layer l is due when its count of decode launches plus l * slack / L is a multiple of the
  // slack, and a list planned at any other time (the first one, or after a reset or a change of the active slots)
  // only lives until then.
  const int64_t phase = (cache->decode_calls[layer] + (int64_t)layer * kWorklistSlack / dv.n_layers) % kWorklistSlack;
  cache->wl_slack[layer] = kWorklistSlack - (int32_t)phase;
  ++cache->lists_built;
  return RLKV_OK;
}

rlkv_status_t rlkv_append(rlkv_cache_t* cache, int32_t layer, const void* k, const void* v, int32_t n_tokens,
                          void* stream) {
  return append_impl(cache, layer, k, v, nullptr, n_tokens, n_tokens, stream);
}

rlkv_status_t rlkv_append_ragged(rlkv_cache_t* cache, int32_t layer, const void* k, const void* v,
                                 const int32_t* n_tokens, int32_t stride_tokens, void* stream) {
  if (!n_tokens) return RLKV_ERR_INVALID_ARG;
  return append_impl(cache, layer, k, v, n_tokens, 0, stride_tokens, stream);
}

rlkv_status_t rlkv_prefill_attention(rlkv_cache_t* cache, int32_t layer, const void* q, const void* k, const void* v,
                                     const int32_t* n_tokens, int32_t stride_tokens, void* out, float softmax_scale,
                                     void* stream) {
  if (!cache || !q || !k || !v || !n_tokens || !out) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return RLKV_ERR_INVALID_ARG;
  if (stride_tokens < 1) return RLKV_ERR_INVALID_ARG;
  if (cache->cfg.prefill_tokens <= 0) return RLKV_ERR_STATE;
  if (stride_tokens > cache->cfg.prefill_tokens) return RLKV_ERR_INVALID_ARG;
  const PrefillArgs args{q, out, softmax_scale};
  return append_impl(cache, layer, k, v, n_tokens, 0, stride_tokens, stream, &args);
}

// Decode attention of one layer with the kernels looking for their tables and partials in `dv` (the cache's own
// view, or a copy whose partials point elsewhere).
// Is `s` recording into a graph?  (A failing query counts as "no".)
static bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
  return st != hipStreamCaptureStatusNone;
}

// Decode attention of one layer with the kernels looking for their tables and partials in `dv` (the cache's own
// view, or a copy whose partials point elsewhere).
static rlkv_status_t decode_with_view(rlkv_cache_t* cache, const DeviceView& dv, int32_t layer, const void* q, void* out,
                                      float softmax_scale, hipStream_t s) {
  cache->last_stream = s;
  const float scale_log2 = softmax_scale * 1.44269504088896340736f;
  if (rlkv_status_t st = ensure_worklist(cache, layer, 0, s)) return st;
  const bool record = (size_t)cache->prof_used * 2 + 1 < cache->prof_events.size();
  hipEvent_t e0 = record ? cache->prof_events[2 * cache->prof_used] : nullptr;
  hipEvent_t e1 = record ? cache->prof_events[2 * cache->prof_used + 1] : nullptr;
  const bool gated = cache->layer_gated[layer] != 0;
  hipError_t e = dv.kernel == RLKV_KERNEL_MFMA
                     ? launch_decode_mfma(dv, layer, gated, q, out, scale_log2, nullptr, nullptr, s, e0, e1)
                     : launch_decode_valu(dv, layer, gated, q, out, scale_log2, s, e0, e1);
  if (e != hipSuccess) return RLKV_ERR_HIP;
  if (record) ++cache->prof_used;
  ++cache->decode_calls[layer];
  const uint32_t* words = (cache->merge_words.empty() || cache->layer_gated[layer])
                              ? nullptr : cache->merge_words.data() + (size_t)layer * dv.n_pairs;
  if (launch_combine(dv, layer, out, s, 0, nullptr, words) != hipSuccess) return RLKV_ERR_HIP;
  return RLKV_OK;
}

// Argument and state checks shared by the decode entry points (host only).
static rlkv_status_t decode_checks(rlkv_cache_t* cache, int32_t layer, const void* q, void* out, float softmax_scale) {
  if (!cache || !q || !out) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return RLKV_ERR_INVALID_ARG;
  const int B = cache->cfg.batch;
  const int32_t* lh = cache->len_host.data() + (size_t)layer * B;
  int n_active = 0;
  for (int b = 0; b < B; ++b) {
    if (!cache->active[b]) continue;
    ++n_active;
    if (lh[b] < 1) return RLKV_ERR_STATE;
  }
  if (n_active == 0) return RLKV_ERR_STATE;
  return RLKV_OK;
}

rlkv_status_t rlkv_decode_attention(rlkv_cache_t* cache, int32_t layer, const void* q, void* out,
                                    float softmax_scale, void* stream) {
  if (rlkv_status_t st = decode_checks(cache, layer, q, out, softmax_scale)) return st;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  return decode_with_view(cache, cache->dv, layer, q, out, softmax_scale, as_stream(stream));
}

rlkv_status_t rlkv_decode_attention_noalloc(rlkv_cache_t* cache, int32_t layer, const void* q, void* out,
                                            float softmax_scale, void* stream) {
  if (rlkv_status_t st = decode_checks(cache, layer, q, out, softmax_scale)) return st;
  // rows of partials the launch can write: one per (workgroup or pair, query head), twice that in a layer that blends
  const DeviceView& own = cache->dv;
  const int64_t slots = (int64_t)own.n_wg + own.n_pairs;
  const int64_t rows_per_set = slots * own.group;
  const int64_t rows = rows_per_set * (cache->layer_gated[layer] ? 2 : 1);
  if (rows > kStaticRows) return RLKV_ERR_TOO_LARGE;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  float* ptr = scratch_on_device(cache->cfg.device);     // looked up at rlkv_cache_create; a table read here
  if (!ptr) return RLKV_ERR_HIP;
  DeviceView dv = own;
  dv.part_o = ptr;                                        // [2][rows_per_set][head_dim]
  dv.part_m = ptr + 2 * rows_per_set * kHeadDim;          // [2][rows_per_set]
  dv.part_l = dv.part_m + 2 * rows_per_set;               // [2][rows_per_set]
  dv.part_set_ml = rows_per_set;
  dv.part_set_o = rows_per_set * kHeadDim;
  return decode_with_view(cache, dv, layer, q, out, softmax_scale, as_stream(stream));
}

rlkv_status_t rlkv_set_active(rlkv_cache_t* cache, const uint8_t* active, void* stream) {
  if (!cache) return RLKV_ERR_INVALID_ARG;
  const int B = cache->cfg.batch;
  std::vector<uint8_t> next((size_t)B, 1);
  if (active)
    for (int b = 0; b < B; ++b) {
      if (active[b] > 1) return RLKV_ERR_INVALID_ARG;
      next[b] = active[b];
    }
  if (next == cache->active) return RLKV_OK;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  cache->active = next;
  cache->last_stream = as_stream(stream);
  if (!send_small(cache, cache->dv.active, cache->active.data(), (size_t)B, as_stream(stream))) return RLKV_ERR_HIP;
  for (int l = 0; l < cache->cfg.n_layers; ++l) cache->wl_slack[l] = -1;   // the work lists name the active slots
  return RLKV_OK;
}

rlkv_status_t rlkv_set_gates(rlkv_cache_t* cache, const float* gates, void* stream) {
  if (!cache) return RLKV_ERR_INVALID_ARG;
  const int L = cache->cfg.n_layers, H = cache->cfg.n_kv_heads;
  std::vector<float> next((size_t)L * H, 1.f);
  if (gates)
    for (int i = 0; i < L * H; ++i) {
      if (!(gates[i] >= 0.f && gates[i] <= 1.f)) return RLKV_ERR_INVALID_ARG;
      next[i] = cache->mask[i] ? gates[i] : 1.f;       // a compressed head has no full history to mix in
    }
  if (next == cache->gate) return RLKV_OK;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  cache->gate = next;
  cache->last_stream = as_stream(stream);
  if (!send_small(cache, cache->dv.gate, cache->gate.data(), cache->gate.size() * sizeof(float), as_stream(stream)))
    return RLKV_ERR_HIP;
  for (int l = 0; l < L; ++l) {
    cache->layer_gated[l] = 0;
    for (int h = 0; h < H; ++h)
      if (cache->mask[(size_t)l * H + h] && cache->gate[(size_t)l * H + h] < 1.f) cache->layer_gated[l] = 1;
    cache->wl_slack[l] = -1;      // the work-list records carry the gates
  }
  return RLKV_OK;
}

rlkv_status_t rlkv_append_decode_prepare(rlkv_cache_t* cache, int32_t layer, void* stream) {
  if (!cache) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  const int B = cache->cfg.batch;
  int32_t* lh = cache->len_host.data() + (size_t)layer * B;
  int n_active = 0;
  for (int b = 0; b < B; ++b) {
    if (!cache->active[b]) continue;
    ++n_active;
    if ((int64_t)lh[b] + 1 > cache->max_len[b]) return RLKV_ERR_CAPACITY;
  }
  if (n_active == 0) return RLKV_ERR_STATE;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  hipStream_t s = as_stream(stream);
  if (stream_is_capturing(s)) return RLKV_ERR_STATE;     // this half copies tables: it is not to be recorded
  cache->last_stream = s;
  if (cache->cfg.page_tokens > 0) {
    for (int b = 0; b < B; ++b) cache->new_len[b] = lh[b] + (cache->active[b] ? 1 : 0);
    if (rlkv_status_t st = reserve_pages(cache, cache->new_len, s)) return st;
  }
  if (rlkv_status_t st = ensure_worklist(cache, layer, 1, s)) return st;
  // the mirrors take the step now; the launch (or the replay of a recorded launch) performs it on the device
  for (int b = 0; b < B; ++b) lh[b] += cache->active[b] ? 1 : 0;
  cache->wl_slack[layer] -= 1;
  ++cache->decode_calls[layer];
  cache->step_ready[layer] = 1;
  return RLKV_OK;
}

rlkv_status_t rlkv_append_decode_launch(rlkv_cache_t* cache, int32_t layer, const void* k, const void* v, const void* q,
                                        void* out, float softmax_scale, void* stream) {
  if (!cache || !k || !v || !q || !out) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return RLKV_ERR_INVALID_ARG;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  hipStream_t s = as_stream(stream);
  const bool capturing = stream_is_capturing(s);
  // a launch that runs now consumes a prepared step; one that is only recorded runs at every replay, each of which
  // the caller prepares
  if (!capturing) {
    if (!cache->step_ready[layer]) return RLKV_ERR_STATE;
    cache->step_ready[layer] = 0;
    cache->last_stream = s;
  }
  const float scale_log2 = softmax_scale * 1.44269504088896340736f;
  const bool record = !capturing && (size_t)cache->prof_used * 2 + 1 < cache->prof_events.size();
  hipEvent_t e0 = record ? cache->prof_events[2 * cache->prof_used] : nullptr;
  hipEvent_t e1 = record ? cache->prof_events[2 * cache->prof_used + 1] : nullptr;
  const bool tiled = cache->dv.kernel == RLKV_KERNEL_MFMA;
  if (tiled) {
    if (launch_decode_mfma(cache->dv, layer, cache->layer_gated[layer] != 0, q, out, scale_log2, k, v, s, e0, e1) !=
        hipSuccess)
      return RLKV_ERR_HIP;
  } else {
    // row-major stores (vector-ALU kernel): the append is a launch of its own; it takes its lengths from the work
    // list, the attention kernel counts the appended token on top of the growth counter, the merge kernel
    // advances the counter - three launches whose arguments are the same at every step
    if (launch_append(cache->dv, layer, len_of(cache->dv, 0, layer), len_of(cache->dv, 1, layer), k, v, 1, 1, false, 1,
                      s, true) != hipSuccess)
      return RLKV_ERR_HIP;
    if (launch_decode_valu(cache->dv, layer, cache->layer_gated[layer] != 0, q, out, scale_log2, s, e0, e1, 1) !=
        hipSuccess)
      return RLKV_ERR_HIP;
  }
  if (record) ++cache->prof_used;
  // (a recorded launch outlives the work list it was recorded under, so its merge kernel reads the pair records
  // from memory instead of taking them as arguments)
  const uint32_t* words = (capturing || cache->merge_words.empty() || cache->layer_gated[layer])
                              ? nullptr : cache->merge_words.data() + (size_t)layer * cache->dv.n_pairs;
  // (the merge kernel of the tiled layout also looks at the appended V rows, for the fp16 range flag of prefill)
  if (launch_combine(cache->dv, layer, out, s, 1, tiled ? v : nullptr, words) != hipSuccess) return RLKV_ERR_HIP;
  return RLKV_OK;
}

rlkv_status_t rlkv_append_decode(rlkv_cache_t* cache, int32_t layer, const void* k, const void* v, const void* q,
                                 void* out, float softmax_scale, void* stream) {
  if (!cache || !k || !v || !q || !out) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return RLKV_ERR_INVALID_ARG;
  if (rlkv_status_t st = rlkv_append_decode_prepare(cache, layer, stream)) return st;
  return rlkv_append_decode_launch(cache, layer, k, v, q, out, softmax_scale, stream);
}

int64_t rlkv_worklists_built(const rlkv_cache_t* cache) { return cache ? cache->lists_built : -1; }

rlkv_status_t rlkv_profile_enable(rlkv_cache_t* cache, int32_t max_records) {
  if (!cache || max_records < 1 || max_records > (1 << 20)) return RLKV_ERR_INVALID_ARG;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  drop_profile_events(cache);
  cache->prof_events.reserve((size_t)max_records * 2);
  for (int i = 0; i < max_records * 2; ++i) {
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) { drop_profile_events(cache); return RLKV_ERR_HIP; }
    cache->prof_events.push_back(ev);
  }
  return RLKV_OK;
}

rlkv_status_t rlkv_profile_collect(rlkv_cache_t* cache, float* kernel_ms, int32_t* n_records) {
  if (!cache || !kernel_ms || !n_records) return RLKV_ERR_INVALID_ARG;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  if (!wait_for_cache(cache)) return RLKV_ERR_HIP;
  rlkv_status_t st = RLKV_OK;
  for (int i = 0; i < cache->prof_used; ++i) {
    if (hipEventElapsedTime(&kernel_ms[i], cache->prof_events[2 * i], cache->prof_events[2 * i + 1]) != hipSuccess)
      st = RLKV_ERR_HIP;
  }
  *n_records = cache->prof_used;
  drop_profile_events(cache);
  return st;
}

rlkv_status_t rlkv_get_lengths(rlkv_cache_t* cache, int32_t layer, int32_t* out) {
  if (!cache || !out) return RLKV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= cache->cfg.n_layers) return RLKV_ERR_INVALID_ARG;
  if (hipSetDevice(cache->cfg.device) != hipSuccess) return RLKV_ERR_HIP;
  if (!wait_for_cache(cache)) return RLKV_ERR_HIP;
  const int B = cache->cfg.batch;
  if (hipMemcpy(out, len_of(cache->dv, cache->parity[layer], layer), (size_t)B * 4, hipMemcpyDeviceToHost) !=
      hipSuccess)
    return RLKV_ERR_HIP;
  return RLKV_OK;
}

rlkv_status_t rlkv_get_slot_positions(rlkv_cache_t* cache, int32_t layer, int32_t kv_head, int32_t seq,
                                      int32_t* out) {
  if (!cache || !out) return RLKV_ERR_INVALID_ARG;
  const rlkv_config_t& c = cache->cfg;
  if (layer < 0 || layer >= c.n_layers || kv_head < 0 || kv_head >= c.n_kv_heads || seq < 0 || seq >= c.batch)
    return RLKV_ERR_INVALID_ARG;
  if (cache->mask[(size_t)layer * c.n_kv_heads + kv_head]) return RLKV_ERR_INVALID_ARG;
  // offset of this head's block: count the compressed heads before it
  int64_t idx = 0;
  for (int i = 0; i < layer * c.n_kv_heads + kv_head; ++i) idx += cache->mask[i] ? 0 : 1;
  const int W = c.sink + c.recent;
  const int64_t off = (idx * c.batch + seq) * W;
  if (hipSetDevice(c.device) != hipSuccess) return RLKV_ERR_HIP;
  if (!wait_for_cache(cache)) return RLKV_ERR_HIP;
  if (hipMemcpy(out, cache->dv.slot_pos + off, (size_t)W * 4, hipMemcpyDeviceToHost) != hipSuccess)
    return RLKV_ERR_HIP;
  return RLKV_OK;
}

size_t rlkv_resident_bytes(const rlkv_cache_t* cache) { return cache ? cache->plan.kv_bytes : 0; }

int64_t rlkv_pool_pages_free(const rlkv_cache_t* cache) {
  if (!cache || cache->cfg.page_tokens <= 0) return -1;
  return (int64_t)cache->free_pages.size();
}

rlkv_status_t rlkv_pool_shuffle(rlkv_cache_t* cache, uint64_t seed) {
  if (!cache) return RLKV_ERR_INVALID_ARG;
  if (cache->cfg.page_tokens <= 0) return RLKV_ERR_STATE;
  // Fisher-Yates with a 64-bit mix (splitmix) as the random source
  uint64_t x = seed;
  auto next = [&]() {
    x += 0x9e3779b97f4a7c15ull;
    uint64_t z = x;
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
  };
  std::vector<int32_t>& f = cache->free_pages;
  for (size_t i = f.size(); i > 1; --i) std::swap(f[i - 1], f[next() % i]);
  return RLKV_OK;
}

rlkv_status_t rlkv_probe_stream_read(const void* buf, size_t bytes, void* sink, int32_t workgroups, void* stream) {
  if (!buf || !sink || workgroups < 1 || workgroups > (1 << 20)) return RLKV_ERR_INVALID_ARG;
  if (launch_stream_read(buf, bytes, sink, workgroups, as_stream(stream)) != hipSuccess) return RLKV_ERR_HIP;
  return RLKV_OK;
}

int32_t rlkv_cache_kernel(const rlkv_cache_t* cache) { return cache ? cache->cfg.kernel : -1; }

const char* rlkv_status_string(rlkv_status_t status) {
  switch (status) {
    case RLKV_OK: return "ok";
    case RLKV_ERR_INVALID_ARG: return "invalid argument";
    case RLKV_ERR_OOM: return "out of memory / arena too small";
    case RLKV_ERR_CAPACITY: return "append exceeds max_len or the page pool";
    case RLKV_ERR_STATE: return "decode on an empty sequence, or a call this cache was not created for";
    case RLKV_ERR_HIP: return "HIP runtime error";
    case RLKV_ERR_TOO_LARGE: return "the call needs more split-K scratch than the static buffer of the allocation-free entry point holds";
  }
  return "unknown status";
}

}  // extern "C"
