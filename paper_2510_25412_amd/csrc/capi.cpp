// C ABI of libsymphony_kv.so (declared in include/symphony_kv.h): glue between the host
// file-system state, the batch-descriptor builder and the HIP kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/symphony_kv.h"
#include "desc.hpp"
#include "kernels.hpp"
#include "kvfs.hpp"
#include "sched.hpp"

using namespace symkv;

namespace {
constexpr int kStages = 4;          // pinned staging buffers in rotation
constexpr int kMaxTimed = 4096;     // timed launches kept per kernel id
constexpr int64_t kStaticBlobWords = 1 << 20;      // largest descriptor blob (32-bit words) sym_pred_batch_static accepts; every staging
                                                  // buffer of a device context has this size from sym_init on
inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
// memcpy of `bytes` bytes that tolerates an empty source (the data() of an empty vector may be null)
inline void copy_bytes(void* dst, const void* src, size_t bytes) {
  if (bytes) std::memcpy(dst, src, bytes);
}
// The planner settings of a shape when the caller gives none.
sym_tuning default_tuning(const sym_config* cfg) {
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  const bool bf16 = cfg->dtype == SYM_BF16;
  sym_tuning t;
  t.decode_mfma = (bf16 && G == 8) ? 1 : 0;   // 8 query heads per kv head are bound by vector issue on the VALU path
  t.min_units = 4;
  t.prefill_min = 16;
  t.share_min_lips = 4;
  t.share_min_pages = 8;
  t.tile_rows = 256;
  t.row_tokens = bf16 ? std::min<int>(ROW_TOKENS_MAX, 16 / G) : 1;
  t.range_cost = 3;                            // measured: a range start costs about 3 units
  t.bin_tolerance = 3;
  t.bin_waves = 8;
  t.fuse_append = 1;
  t.mix_lead = 0;
  t.mix_spread = 50;
  t.share_tiles = 512;
  return t;
}
}  // namespace

// A batch planned by sym_pred_begin: where its parts lie in the device copy of the blob, until every layer has run.
struct OpenPred {
  bool open = false;
  int64_t words = 0, cow_off = 0, slots_off = 0;   // blob size; offsets of the copy list and of the slot map in it
  int32_t n_cow = 0, n_append = 0;                 // page copies; rows for the append kernel (0 when the attention kernel appends them all)
  bool copies_first = false;
  int64_t partials = 0;                            // partial slots behind the blob in the workspace
  std::vector<uint8_t> done;                       // per layer: sym_pred_layer has run
  int32_t n_done = 0;
};

struct sym_ctx {
  sym_config cfg;
  int32_t G = 1;
  int32_t n_layers = 1;
  int64_t layer_bytes = 0;            // bytes of one layer of the pool: n_pages * page_bytes
  OpenPred pred;
  int64_t page_bytes = 0;
  float scale_log2e = 0.f;
  int32_t max_waves = 0, min_units = 4, range_cost = 3;
  int32_t decode_mode = 0;                           // 1 = decode ranges on the matrix cores
  int32_t share_min_lips = 4, share_min_pages = 8;   // decode LIPs / common full pages needed to read a prefix once
  int32_t tile_rows = 256;                     // query rows of an MFMA tile: 128 or 256
  int32_t prefill_min = 16, tile_tokens = 0;   // LIPs with >= prefill_min new tokens use the MFMA tile kernel (bf16 only)
  int32_t row_tokens = 1;                      // new tokens of one LIP per decode row (bf16: up to 16 / G, at most 4)
  int32_t fuse_append = 1;                     // 1: the attention kernel appends the tokens of single-token LIPs itself
  int32_t mix_lead = 0, mix_spread = 50;       // where decode workgroups sit among the tile workgroups of a launch (percent)
  int32_t share_tiles = 512;                   // shared-prefix tiles a batch is cut into (by key chunk), about
  int32_t bin_waves = 8;                       // wavefronts per decode bin (workgroup) of a batch without tiles: 4 or 8
  int32_t bin_tolerance = 3;                   // percent of imbalance between the decode bins that is accepted before ranges are split
  std::mutex mu;
  std::string err;
  Kvfs* fs = nullptr;
  AppendPlan plan;
  GatherPlan gplan;
  SwapPlan splan;
  std::vector<uint8_t*> host_chunks;   // pinned memory of the host slots, kHostChunk pages each
  int64_t pages_offloaded = 0, pages_restored = 0;
  BatchDesc desc;
  int32_t desc_hdr[DESC_HEADER_WORDS] = {};   // header of the last descriptor built for a launch (its words lie in pinned memory)
  std::vector<const int32_t*> tables;
  std::vector<int64_t> len_after;
  std::vector<int32_t> scratch_words;
  // pinned staging ring (device contexts only)
  int32_t* stage[kStages] = {nullptr, nullptr, nullptr, nullptr};
  int64_t stage_words[kStages] = {0, 0, 0, 0};
  hipEvent_t stage_ev[kStages];
  bool stage_pending[kStages] = {false, false, false, false};
  int stage_next = 0;
  int fail_staging = 0;                // test hook: this many coming staging reservations fail (sym_test_fail_staging)
  uint8_t* static_scratch = nullptr;   // this device's copy of the library's file-scope scratch array (sym_pred_batch_static)
  // profiling
  int prof_mask = 0, prof_stride = 1;
  int64_t prof_seen[SYM_K_COUNT] = {0, 0, 0, 0, 0};
  std::vector<hipEvent_t> ev_start[SYM_K_COUNT], ev_stop[SYM_K_COUNT];
  int ev_used[SYM_K_COUNT] = {0, 0, 0, 0, 0};
  // counters
  int64_t pred_batches = 0, kernel_launches = 0;
  int64_t host_ns_plan = 0, host_ns_pred = 0;   // time inside sym_pred_batch: planning + descriptor; whole call
};

namespace {

int fail(sym_ctx* c, int code, const std::string& msg) {
  c->err = msg;
  return code;
}
int fail_hip(sym_ctx* c, hipError_t e, const char* what) {
  c->err = std::string(what) + ": " + hipGetErrorString(e);
  return SYM_EHIP;
}

uint8_t* pool_of(const sym_ctx* c, int32_t layer) { return (uint8_t*)c->cfg.pool + (int64_t)layer * c->layer_bytes; }
// Calls that change file-system state (or stage anything) are refused between sym_pred_begin and the batch's last layer:
// the descriptor on the device describes the files as they are.
int refuse_if_open(sym_ctx* c, const char* what) {
  if (!c->pred.open) return SYM_OK;
  return fail(c, SYM_EBUSY, std::string(what) + ": a batch begun with sym_pred_begin has layers left (run them, or sym_pred_end)");
}

bool shape_ok(const sym_config* cfg) {
  if (!cfg) return false;
  const int es = cfg->dtype == SYM_F32 ? 4 : cfg->dtype == SYM_BF16 ? 2 : 0;
  if (es == 0 || cfg->head_dim * es != 256 || cfg->page_tokens != 16) return false;
  if (cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return false;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  return G == 1 || G == 2 || G == 4 || G == 8;
}

// 32-bit words of the host-to-device blob of one batch: descriptor + copies + slots.
int64_t blob_words_bound(const sym_ctx* c, int64_t n_lips, int64_t T, int64_t entries) {
  // bins: a segment (and at most one merge entry) per (row, kv head) and per piece of a split range (no more pieces than
  // partial slots for them: 2 * tokens per row * wavefront slots), an in-bin merge list per workgroup of at least 4 wavefronts
  const int64_t bins = (T * c->cfg.n_kv_heads + 2 * (int64_t)c->row_tokens * c->max_waves + 2) * (SEG_WORDS + MERGE_WORDS) +
                       ((int64_t)c->max_waves / 4 + 1) * LMERGE_WORDS;
  // the order table of a launch with tiles and bins: a word per tile (chunks of at least 16 tokens of a LIP per kv
  // head; up to 8 key chunks of a shared prefix per LIP and kv head) and per 8 bins
  const int64_t order = (T / 16 + 9 * n_lips) * c->cfg.n_kv_heads + (int64_t)c->max_waves / 32 + 8;
  return bins + order + DESC_HEADER_WORDS + T * ROW_WORDS + (int64_t)c->max_waves * (WAVE_WORDS + ROW_TOKENS_MAX * MERGE_WORDS) + entries +
         (T + 8 * n_lips) * c->cfg.n_kv_heads * 2 + n_lips * (1 + c->cfg.n_kv_heads * (MERGE_WORDS + 8 * TILE_WORDS)) +
         n_lips + 1 + 3 * n_lips + T + 64;
}
// Partial-result slots of the workspace: a wave boundary cuts at most one (row, head) range (<= 2
// pieces per wave, each a partial per token of the row); the rest is for the partials of
// shared-prefix tiles and of their members' own ranges.
int64_t partial_slots(const sym_ctx* c) { return (2 * ROW_TOKENS_MAX + 10) * (int64_t)c->max_waves + 1; }
// The fewest slots with which every batch can be described: the cut pieces alone.
int64_t min_partial_slots(const sym_ctx* c) { return 2 * (int64_t)c->row_tokens * c->max_waves + 1; }
int64_t partial_bytes_for(const sym_ctx* c, int64_t np) {
  return align_up(np * c->G * 2 * 4, 256) + align_up(np * c->G * c->cfg.head_dim * 4, 256);
}
int64_t partial_bytes(const sym_ctx* c) { return partial_bytes_for(c, partial_slots(c)); }

// Device scratch of one batch: [descriptor words][partial max/sum][partial accumulators].  Either the
// caller's workspace (as many partial slots as partial_slots says) or the library's static array
// (as many as fit behind the descriptor).
struct Scratch {
  uint8_t* base;
  int64_t bytes;
  int64_t partials;
};
Scratch workspace_of(const sym_ctx* c) { return Scratch{(uint8_t*)c->cfg.workspace, c->cfg.workspace_bytes, partial_slots(c)}; }
// fuse_append: the batch's single-token LIPs are appended by the attention kernel itself (bins only)
DescParams desc_params(const sym_ctx* c, int64_t partials, bool fuse_append = false) {
  DescParams p{c->cfg.n_q_heads, c->cfg.n_kv_heads, c->cfg.page_tokens, c->max_waves, c->min_units, c->range_cost, c->prefill_min,
               c->tile_tokens, c->share_min_lips, c->share_min_pages, (int32_t)std::min<int64_t>(partials, 0x7fffffff), c->row_tokens};
  // the vector-unit decode kernel (up to 4 query heads per kv head, unless the matrix cores are asked for) works on bins
  p.bin_waves = (c->G < 8 && !c->decode_mode) ? c->bin_waves : 0;
  p.fuse_append = (fuse_append && p.bin_waves && c->fuse_append) ? 1 : 0;
  p.bin_tolerance = c->bin_tolerance;
  p.mix_lead = c->mix_lead;
  p.mix_spread = c->mix_spread;
  p.share_tiles = c->share_tiles;
  return p;
}

// Pinned staging.  A call that changes host state first RESERVES room for the most it may stage
// (stage_reserve: every buffer of the ring grows to that size now), then commits, then takes the
// ring's next buffer (stage_acquire): no allocation can fail after the commit, so a call that
// fails for want of pinned memory leaves the file system as it was.
// may_alloc = false: never allocates; buffers that are too small are SYM_ENOSPC.
int stage_reserve(sym_ctx* c, int64_t words, bool may_alloc = true) {
  if (c->fail_staging > 0) {           // test hook (sym_test_fail_staging)
    --c->fail_staging;
    return fail(c, SYM_EHIP, "staging reservation failed (test hook)");
  }
  if (c->cfg.device < 0) return SYM_OK;          // host-only context: nothing is staged
  for (int i = 0; i < kStages; ++i) {
    if (c->stage_words[i] >= words) continue;
    if (!may_alloc) return fail(c, SYM_ENOSPC, "batch too large for the preallocated staging buffers");
    if (c->stage_pending[i]) {
      hipError_t e = hipEventSynchronize(c->stage_ev[i]);
      if (e != hipSuccess) return fail_hip(c, e, "hipEventSynchronize(stage)");
      c->stage_pending[i] = false;
    }
    const int64_t cap = std::max<int64_t>(words * 3 / 2, 1 << 16);
    int32_t* fresh = nullptr;
    hipError_t e = hipHostMalloc((void**)&fresh, (size_t)cap * 4, hipHostMallocDefault);
    if (e != hipSuccess) return fail_hip(c, e, "hipHostMalloc(stage)");
    if (c->stage[i]) (void)hipHostFree(c->stage[i]);
    c->stage[i] = fresh;
    c->stage_words[i] = cap;
  }
  return SYM_OK;
}
// The ring's next buffer (reserved before: it has room for `words`); waits for the copy that last used it.
int stage_acquire(sym_ctx* c, int64_t words, int* idx) {
  const int i = c->stage_next;
  if (c->stage_words[i] < words) return fail(c, SYM_EINVAL, "staging buffer was not reserved");      // a bug of the caller
  if (c->stage_pending[i]) {
    hipError_t e = hipEventSynchronize(c->stage_ev[i]);
    if (e != hipSuccess) return fail_hip(c, e, "hipEventSynchronize(stage)");
    c->stage_pending[i] = false;
  }
  c->stage_next = (i + 1) % kStages;
  *idx = i;
  return SYM_OK;
}

// Brackets a launch with a pair of events when the kernel id is being profiled.  attached = true: the
// events are not recorded here but handed to the launch (start() / stop()), which attaches them to
// the dispatch itself, so they bracket the kernel's execution and not its launch overhead.
struct Timed {
  sym_ctx* c;
  int id;
  hipStream_t st;
  bool on, attached;
  hipEvent_t start() const { return on && attached ? c->ev_start[id][c->ev_used[id]] : nullptr; }
  hipEvent_t stop() const { return on && attached ? c->ev_stop[id][c->ev_used[id]] : nullptr; }
  Timed(sym_ctx* ctx, int kid, hipStream_t s, bool attach = false, bool allow = true) : c(ctx), id(kid), st(s), on(false), attached(attach) {
    ++c->kernel_launches;
    if (!allow || !((c->prof_mask >> id) & 1) || c->ev_used[id] >= kMaxTimed) return;
    if (c->prof_seen[id]++ % c->prof_stride != 0) return;          // every prof_stride-th launch is timed
    if ((int)c->ev_start[id].size() <= c->ev_used[id]) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return;
      if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return;
      }
      c->ev_start[id].push_back(a);
      c->ev_stop[id].push_back(b);
    }
    on = attached || hipEventRecord(c->ev_start[id][c->ev_used[id]], st) == hipSuccess;
  }
  ~Timed() {
    if (on && (attached || hipEventRecord(c->ev_stop[id][c->ev_used[id]], st) == hipSuccess)) ++c->ev_used[id];
  }
};

// Launches attention (decode + merge) for the descriptor in c->desc, already copied to the scratch `ws`.
// timed = false: no profiling events (they are created on demand, and this call may not allocate).
int launch_attention(sym_ctx* c, const Scratch& ws, int64_t blob_words, const void* q, float* out, hipStream_t st, bool timed = true,
                     const void* k_new = nullptr, const void* v_new = nullptr, int32_t layer = 0) {
  const BatchDesc& d = c->desc;
  if (d.n_waves == 0 && d.n_tiles == 0) return SYM_OK;
  const int32_t* hdr = c->desc_hdr;
  // scratch: [descriptor words][partial max/sum][partial accumulators]
  const int32_t* dw = (const int32_t*)ws.base;
  uint8_t* base = ws.base + align_up(blob_words * 4, 256);
  const int64_t np = ws.partials;
  float* part_ml = (float*)base;
  float* part_acc = (float*)(base + align_up(np * c->G * 2 * 4, 256));
  DecodeArgs a;
  a.pool = pool_of(c, layer);
  a.page_bytes = c->page_bytes;
  a.q = q;
  a.out = out;
  a.part_acc = part_acc;
  a.part_ml = part_ml;
  a.rows = dw + hdr[H_OFF_ROWS];
  a.waves = dw + hdr[H_OFF_WAVES];
  a.pt = dw + hdr[H_OFF_PT];
  a.n_waves = d.n_waves;
  a.Hq = c->cfg.n_q_heads;
  a.Hkv = c->cfg.n_kv_heads;
  a.scale_log2e = c->scale_log2e;
  a.segs = dw + hdr[H_OFF_SEGS];
  a.lmerge = dw + hdr[H_OFF_LMERGE];
  a.n_bins = d.n_bins;
  a.bin_waves = d.bin_waves;
  // the attention kernel requests a chunk of these rows with every segment's query rows, used or not: when it appends
  // nothing, the query rows (no smaller) stand in
  a.k_new = d.n_fused > 0 ? k_new : q;
  a.v_new = d.n_fused > 0 ? v_new : q;
  if (d.n_fused > 0 && (!k_new || !v_new)) return fail(c, SYM_EINVAL, "attention launch: rows to append are missing");
  PrefillArgs pa;
  pa.pool = pool_of(c, layer);
  pa.page_bytes = c->page_bytes;
  pa.q = q;
  pa.out = out;
  pa.tiles = dw + hdr[H_OFF_TILES];
  pa.pt = dw + hdr[H_OFF_PT];
  pa.members = dw + hdr[H_OFF_MEMBERS];
  pa.part_acc = part_acc;
  pa.part_ml = part_ml;
  pa.tile_first = 0;
  pa.n_tiles = d.n_tiles;
  pa.xcd_off = dw + H_XCD_OFF;
  pa.tile_blocks = d.tile_blocks;
  pa.tile_rows = d.tile_rows;
  pa.Hq = c->cfg.n_q_heads;
  pa.Hkv = c->cfg.n_kv_heads;
  pa.scale_log2e = c->scale_log2e;
  pa.small_shared_only = d.small_shared_only;
  pa.group_map = hdr[H_N_GROUPS] > 0 ? dw + hdr[H_OFF_GROUPS] : nullptr;
  pa.n_groups = hdr[H_N_GROUPS];
  {
    Timed t(c, SYM_K_ATTN, st, true, timed);
    // rows that hold several new tokens exist for the matrix-core decode kernel only
    hipError_t e = launch_attn(a, pa, c->cfg.dtype, (c->decode_mode || d.max_row_tokens > 1) ? 1 : 0, st, t.start(), t.stop());
    if (e != hipSuccess) return fail_hip(c, e, "attention launch");
  }
  if (d.n_merge > 0) {
    MergeArgs m{part_acc, part_ml, dw + hdr[H_OFF_MERGE], out, d.n_merge};
    Timed t(c, SYM_K_MERGE, st, false, timed);
    hipError_t e = launch_merge(m, c->G, c->cfg.head_dim, st);
    if (e != hipSuccess) return fail_hip(c, e, "merge launch");
  }
  return SYM_OK;
}

// One prologue launch: the first copy_words words of the pinned buffer c->stage[si] (the descriptor, or the whole blob of
// a batch) are copied to `dev_words` (default: the start of the workspace); `n_cow` page copies from the list `cow` and the
// append of `n_tokens` rows k, v by the slot map `slots` (both lists in pinned or device memory) go to layer `layer`.
int launch_prologue(sym_ctx* c, int si, int64_t copy_words, const int32_t* cow, int n_cow, const int32_t* slots, int32_t n_tokens,
                    const void* k, const void* v, hipStream_t st, uint8_t* dev_words = nullptr, bool timed = true, int32_t layer = 0) {
  PrologueArgs a;
  a.pool = pool_of(c, layer);
  a.page_bytes = c->page_bytes;
  a.k_new = k;
  a.v_new = v;
  a.slots = slots;
  a.cow = cow;
  a.host_words = si >= 0 ? c->stage[si] : nullptr;
  a.dev_words = (int32_t*)(dev_words ? dev_words : (uint8_t*)c->cfg.workspace);
  a.copy_words = copy_words;
  a.n_tokens = n_tokens;
  a.Hkv = c->cfg.n_kv_heads;
  a.n_cow = n_cow;
  a.append_blocks = a.copy_blocks = 0;
  Timed t(c, SYM_K_PROLOGUE, st, false, timed);
  hipError_t e = symkv::launch_prologue(a, st);
  if (e != hipSuccess) return fail_hip(c, e, "prologue launch");
  return SYM_OK;
}
// Records the event that lets the staging buffer be reused.
int stage_release(sym_ctx* c, int si, hipStream_t st) {
  hipError_t e = hipEventRecord(c->stage_ev[si], st);
  if (e != hipSuccess) return fail_hip(c, e, "hipEventRecord(stage)");
  c->stage_pending[si] = true;
  return SYM_OK;
}

// Host slots live in pinned chunks of kHostChunk pages each, allocated when first needed.
constexpr int64_t kHostChunk = 1024;
int ensure_host_slots(sym_ctx* c, int64_t n_slots) {
  while ((int64_t)c->host_chunks.size() * kHostChunk < n_slots) {
    uint8_t* p = nullptr;
    hipError_t e = hipHostMalloc((void**)&p, (size_t)(kHostChunk * c->page_bytes * c->n_layers), hipHostMallocDefault);
    if (e != hipSuccess) return fail_hip(c, e, "hipHostMalloc(host slots)");
    c->host_chunks.push_back(p);
  }
  return SYM_OK;
}
// a host slot holds the page's bytes of every layer, layer after layer
uint8_t* host_slot(const sym_ctx* c, int32_t s) { return c->host_chunks[s / kHostChunk] + (int64_t)(s % kHostChunk) * c->page_bytes * c->n_layers; }

constexpr int64_t kSwapChunk = 1 << 18;                               // pages per swap launch
int64_t swap_stage_words(int64_t pages) { return 4 * std::min(pages, kSwapChunk); }
int64_t move_chunk(const sym_ctx* c) { return std::min<int64_t>((c->cfg.workspace_bytes / 4 - 64) / 2, 1 << 20); }   // tokens per move launch
int64_t move_stage_words(const sym_ctx* c, int64_t tokens) { return 2 * std::min(tokens, std::max<int64_t>(move_chunk(c), 0)) + 4; }

// Carries out the page copies of c->splan ((page, slot) pairs when to_host, (slot, page) otherwise).
int run_swaps(sym_ctx* c, bool to_host, hipStream_t st) {
  const std::vector<int32_t>& pr = c->splan.pairs;
  const int64_t n = (int64_t)pr.size() / 2;
  const int64_t cap = kSwapChunk;
  for (int64_t off = 0; off < n; off += cap) {
    const int64_t cnt = std::min(cap, n - off);
    int si, rc;
    if ((rc = stage_acquire(c, 4 * cnt, &si))) return rc;
    uint64_t* list = (uint64_t*)c->stage[si];
    for (int64_t i = 0; i < cnt; ++i) {
      const int32_t a = pr[2 * (off + i)], b = pr[2 * (off + i) + 1];
      list[2 * i] = (uint64_t)(to_host ? a : b);
      list[2 * i + 1] = (uint64_t)(uintptr_t)host_slot(c, to_host ? b : a);
    }
    for (int32_t l = 0; l < c->n_layers; ++l) {
      SwapArgs sa{pool_of(c, l), c->page_bytes, list, (int32_t)cnt, to_host ? 1 : 0, (int64_t)l * c->page_bytes};
      Timed t(c, SYM_K_SWAP, st);
      hipError_t e = launch_swap(sa, st);
      if (e != hipSuccess) return fail_hip(c, e, "swap launch");
    }
    if ((rc = stage_release(c, si, st))) return rc;
  }
  (to_host ? c->pages_offloaded : c->pages_restored) += n;
  return SYM_OK;
}

// Carries out the copies of c->gplan on the device: the move list goes through pinned staging
// into the workspace (bulk copy by the prologue kernel), chunk by chunk, then the move kernel.
int run_moves(sym_ctx* c, hipStream_t st) {
  const std::vector<int32_t>& mv = c->gplan.moves;
  const int64_t n = (int64_t)mv.size() / 2;
  const int64_t cap = move_chunk(c);
  for (int64_t off = 0; off < n; off += cap) {
    const int64_t cnt = std::min(cap, n - off);
    int si, rc;
    if ((rc = stage_acquire(c, 2 * cnt + 4, &si))) return rc;
    copy_bytes(c->stage[si], mv.data() + 2 * off, (size_t)cnt * 8);
    if ((rc = launch_prologue(c, si, 2 * cnt, nullptr, 0, nullptr, 0, nullptr, nullptr, st)) || (rc = stage_release(c, si, st))) return rc;
    for (int32_t l = 0; l < c->n_layers; ++l) {
      MoveArgs ma{pool_of(c, l), c->page_bytes, (const int32_t*)c->cfg.workspace, cnt, c->cfg.n_kv_heads};
      Timed t(c, SYM_K_MOVE, st);
      hipError_t e = launch_move(ma, st);
      if (e != hipSuccess) return fail_hip(c, e, "move launch");
    }
  }
  return SYM_OK;
}

// Builds c->desc from caller-supplied page tables (lock held).  Returns words or a negative status.
int64_t desc_from_flat(sym_ctx* c, int32_t n_lips, const int32_t* n_tokens, const int32_t* page_table_flat,
                       const int64_t* pt_offsets, const int64_t* lengths, const std::function<int32_t*(int64_t)>& alloc) {
  c->tables.resize(n_lips);
  for (int32_t b = 0; b < n_lips; ++b) {
    if (lengths[b] < 1) return fail(c, SYM_EINVAL, "length must be >= 1");
    const int64_t np = (lengths[b] + c->cfg.page_tokens - 1) / c->cfg.page_tokens;
    if (pt_offsets[b + 1] - pt_offsets[b] < np) return fail(c, SYM_EINVAL, "page table shorter than the length needs");
    c->tables[b] = page_table_flat + pt_offsets[b];
    for (int64_t i = 0; i < np; ++i)
      if (c->tables[b][i] < 0 || c->tables[b][i] >= c->cfg.n_pages) return fail(c, SYM_EINVAL, "page id out of range");
  }
  const DescParams prm = desc_params(c, partial_slots(c));
  c->desc.alloc = alloc;
  const int rc = build_desc(prm, n_lips, n_tokens, lengths, c->tables.data(), &c->desc);
  c->desc.alloc = nullptr;
  if (rc) return fail(c, rc, "build_desc: bad batch or no room for the descriptor");
  std::memcpy(c->desc_hdr, c->desc.words, sizeof(c->desc_hdr));
  return c->desc.n_words;
}

// The host half of a batch (lock held, arguments checked): validates, reserves staging, commits the append, builds the
// descriptor straight into a pinned staging buffer with copy list and slot map behind it.  `ws` is the device scratch
// the batch will use; no_alloc = true: nothing is allocated on the way (staging buffers as sym_init made them) and a
// batch that does not fit is refused before anything changes.
struct PlannedBatch {
  int si = -1;
  int64_t dwords = 0, words = 0, cow_off = 0, slots_off = 0;
  int32_t n_cow = 0, n_append = 0;
  int64_t wait_ns = 0;
  int64_t partials = 0;      // partial slots of this batch's scratch (see below)
};
// Partial slots of a batch in the caller's workspace: everything behind the descriptor's bound, not just the minimum the
// context was sized for (the slots left over after the cut pieces decide how many files may share a prefix, and into how
// many key chunks it is cut).  Capped so that slot * G * D stays far inside 32 bits.
int64_t partials_behind(const sym_ctx* c, const Scratch& ws, int64_t bound_words) {
  const int64_t slot_bytes = (int64_t)c->G * (2 + c->cfg.head_dim) * 4;
  const int64_t fit = (ws.bytes - align_up(bound_words * 4, 256) - 512) / slot_bytes;
  return std::max(ws.partials, std::min<int64_t>(fit, 1 << 20));
}
int pred_plan_locked(sym_ctx* c, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens, const Scratch& ws, bool no_alloc,
                     PlannedBatch* pb) {
  const int P = c->cfg.page_tokens;
  // sizes after the append, for the checks that must precede any state change
  int64_t T = 0, entries = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    const KvFile* f = c->fs->file_of(kv[b]);
    if (!f) return fail(c, SYM_EBADF, "pred_batch: bad file handle");
    if (n_tokens[b] < 1) return fail(c, SYM_EINVAL, "pred_batch: n_tokens must be >= 1");
    T += n_tokens[b];
    entries += (f->len + n_tokens[b] + P - 1) / P;
  }
  const int64_t bound = blob_words_bound(c, n_lips, T, entries);
  if (no_alloc && bound > kStaticBlobWords) return fail(c, SYM_ENOSPC, "pred_batch_static: batch too large (descriptor beyond the static limit)");
  const int64_t partials = no_alloc ? ws.partials : partials_behind(c, ws, bound);
  pb->partials = partials;
  if (align_up(bound * 4, 256) + partial_bytes_for(c, partials) > ws.bytes) return fail(c, SYM_ENOSPC, "workspace too small for this batch");
  int rc;
  if ((rc = stage_reserve(c, bound, !no_alloc))) return rc;      // the last thing that can fail for want of memory
  c->plan.clear();
  if ((rc = c->fs->append(n_lips, kv, n_tokens, &c->plan, &c->err))) return rc;
  c->tables.resize(n_lips);
  c->len_after.resize(n_lips);
  for (int32_t b = 0; b < n_lips; ++b) {
    const KvFile* f = c->fs->file_of(kv[b]);
    c->tables[b] = f->pages.data();
    c->len_after[b] = f->len;
  }
  const DescParams prm = desc_params(c, partials, true);
  // The descriptor is built straight into the pinned staging buffer; copy list and slot map follow it.
  const int64_t tail_words = (int64_t)c->plan.cow.size() + (int64_t)c->plan.slots.size() + 4;
  int si = -1;
  c->desc.alloc = [&](int64_t words) -> int32_t* {
    const auto w0 = std::chrono::steady_clock::now();
    if (stage_acquire(c, words + tail_words, &si)) return nullptr;      // may wait for the GPU: not host work
    pb->wait_ns = std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - w0).count();
    return c->stage[si];
  };
  rc = build_desc(prm, n_lips, n_tokens, c->len_after.data(), c->tables.data(), &c->desc);
  c->desc.alloc = nullptr;
  if (rc) return fail(c, rc, "pred_batch: descriptor build failed");   // not reached: sizes were checked against their bounds above
  std::memcpy(c->desc_hdr, c->desc.words, sizeof(c->desc_hdr));
  pb->si = si;
  pb->dwords = align_up(c->desc.n_words, 4);
  pb->cow_off = pb->dwords;
  pb->slots_off = pb->cow_off + (int64_t)c->plan.cow.size();
  pb->words = pb->slots_off + (int64_t)c->plan.slots.size();
  copy_bytes(c->stage[si] + pb->cow_off, c->plan.cow.data(), c->plan.cow.size() * 4);
  copy_bytes(c->stage[si] + pb->slots_off, c->plan.slots.data(), c->plan.slots.size() * 4);
  if (c->desc.n_fused > 0) {           // tokens that the attention kernel appends itself: the append kernel skips them
    int32_t* sl = c->stage[si] + pb->slots_off;
    int64_t t = 0;
    for (int32_t b = 0; b < n_lips; t += n_tokens[b], ++b)
      if (c->desc.fused[b]) sl[t] = -1;
  }
  pb->n_cow = (int)(c->plan.cow.size() / 3);
  // rows for the append kernel: none when the attention kernel appends every token of the batch itself
  pb->n_append = c->desc.n_fused == (int32_t)c->plan.slots.size() ? 0 : (int32_t)c->plan.slots.size();
  return SYM_OK;
}

// sym_pred_batch and sym_pred_batch_static (lock held, arguments checked): one layer, one call.
int pred_batch_locked(sym_ctx* c, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens, const void* q, const void* k_new,
                      const void* v_new, float* out, hipStream_t st, const Scratch& ws, bool no_alloc) {
  const auto t_begin = std::chrono::steady_clock::now();
  PlannedBatch pb;
  int rc;
  if ((rc = pred_plan_locked(c, n_lips, kv, n_tokens, ws, no_alloc, &pb))) return rc;
  const Scratch used{ws.base, ws.bytes, pb.partials};
  const auto t_planned = std::chrono::steady_clock::now();
  const int32_t* cow = c->stage[pb.si] + pb.cow_off;
  const int32_t* slots = c->stage[pb.si] + pb.slots_off;
  int n_cow = pb.n_cow;
  if (c->plan.copies_first) {       // an append of this batch overwrites slots that a copy of this batch reads: copies in a launch of their own
    if ((rc = launch_prologue(c, pb.si, 0, cow, n_cow, nullptr, 0, nullptr, nullptr, st, ws.base, !no_alloc))) return rc;
    n_cow = 0;
  }
  // descriptor to the device; page copies and the appends the attention kernel does not do itself, read from the pinned buffer
  if ((rc = launch_prologue(c, pb.si, pb.dwords, cow, n_cow, slots, pb.n_append, k_new, v_new, st, ws.base, !no_alloc)) ||
      (rc = stage_release(c, pb.si, st)))
    return rc;
  ++c->pred_batches;
  rc = launch_attention(c, used, pb.words, q, out, st, !no_alloc, k_new, v_new);
  const auto t_end = std::chrono::steady_clock::now();
  const auto ns = [](auto d) { return (int64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(d).count(); };
  c->host_ns_plan += ns(t_planned - t_begin) - pb.wait_ns;
  c->host_ns_pred += ns(t_end - t_begin) - pb.wait_ns;
  return rc;
}

}  // namespace

extern "C" {

int64_t sym_page_bytes(const sym_config* cfg) {
  if (!shape_ok(cfg)) return 0;
  return (int64_t)cfg->n_kv_heads * 2 * cfg->page_tokens * 256;
}

int sym_tuning_defaults(const sym_config* cfg, sym_tuning* out) {
  if (!shape_ok(cfg) || !out) return SYM_EINVAL;
  *out = default_tuning(cfg);
  return SYM_OK;
}

int64_t sym_workspace_bytes(const sym_config* cfg, int64_t max_lips, int64_t max_tokens, int64_t max_table_entries) {
  if (!shape_ok(cfg)) return 0;
  sym_ctx tmp;
  tmp.cfg = *cfg;
  tmp.G = cfg->n_q_heads / cfg->n_kv_heads;
  tmp.max_waves = cfg->decode_waves > 0 ? cfg->decode_waves : 8192;
  tmp.row_tokens = ROW_TOKENS_MAX;
  return align_up(blob_words_bound(&tmp, max_lips, max_tokens, max_table_entries) * 4, 256) + partial_bytes(&tmp) + 256;
}

int sym_init(const sym_config* cfg, sym_ctx** out) {
  if (!out) return SYM_EINVAL;
  *out = nullptr;
  if (!shape_ok(cfg) || cfg->n_pages < 1 || cfg->n_pages >= (1LL << 27) || cfg->n_layers < 0 || cfg->n_layers > 1024) return SYM_EINVAL;
  if (cfg->device >= 0 && (!cfg->pool || !cfg->workspace || cfg->workspace_bytes < 4096)) return SYM_EINVAL;
  if (cfg->free_order) {   // must be a permutation
    std::vector<uint8_t> seen((size_t)cfg->n_pages, 0);
    for (int64_t i = 0; i < cfg->n_pages; ++i) {
      const int32_t p = cfg->free_order[i];
      if (p < 0 || p >= cfg->n_pages || seen[p]) return SYM_EINVAL;
      seen[p] = 1;
    }
  }
  const sym_tuning tun = cfg->tuning ? *cfg->tuning : default_tuning(cfg);
  sym_ctx* c = new sym_ctx();
  c->cfg = *cfg;
  c->cfg.free_order = nullptr;
  c->cfg.tuning = nullptr;
  c->G = cfg->n_q_heads / cfg->n_kv_heads;
  c->page_bytes = sym_page_bytes(cfg);
  c->n_layers = std::max(1, cfg->n_layers);
  c->layer_bytes = cfg->n_pages * c->page_bytes;
  const float scale = cfg->softmax_scale != 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  c->scale_log2e = scale * 1.4426950408889634f;
  c->fs = new Kvfs(cfg->n_pages, cfg->page_tokens, cfg->free_order);
  c->max_waves = cfg->decode_waves > 0 ? cfg->decode_waves : 2048;
  if (cfg->device >= 0) {
    hipError_t e = hipSetDevice(cfg->device);
    int cus = 0;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device);
    int n_ev = 0;                                  // staging events created so far
    while (n_ev < kStages && e == hipSuccess)
      if ((e = hipEventCreateWithFlags(&c->stage_ev[n_ev], hipEventDisableTiming)) == hipSuccess) ++n_ev;
    // for the entry point that allocates nothing: this device's address of the library's static scratch
    // array (the device is current here), and staging buffers that hold its largest descriptor
    if (e == hipSuccess) e = static_scratch_address(cfg->device, &c->static_scratch);
    for (int i = 0; i < kStages && e == hipSuccess; ++i) {
      e = hipHostMalloc((void**)&c->stage[i], (size_t)kStaticBlobWords * 4, hipHostMallocDefault);
      if (e == hipSuccess) c->stage_words[i] = kStaticBlobWords;
    }
    if (e != hipSuccess) {
      for (int i = 0; i < kStages; ++i)
        if (c->stage[i]) (void)hipHostFree(c->stage[i]);
      for (int i = 0; i < n_ev; ++i) (void)hipEventDestroy(c->stage_ev[i]);
      delete c->fs;
      delete c;
      return SYM_EHIP;
    }
    // two wavefronts per SIMD; with 8 query heads per kv head a range of the VALU kernel takes two wavefronts
    if (cfg->decode_waves <= 0) c->max_waves = std::max(cus, 1) * ((c->G == 8 && !tun.decode_mfma) ? 4 : 8);
  }
  c->max_waves = std::min(c->max_waves, 1 << 16);
  c->min_units = std::max(1, tun.min_units);
  c->decode_mode = (tun.decode_mfma && cfg->dtype == SYM_BF16) ? 1 : 0;
  c->prefill_min = std::max(2, tun.prefill_min);
  c->share_min_lips = std::max(0, tun.share_min_lips);   // 0 = never group
  c->share_min_pages = std::max(2, tun.share_min_pages);
  c->tile_rows = tun.tile_rows == 128 ? 128 : 256;
  c->tile_tokens = cfg->dtype == SYM_BF16 ? c->tile_rows / c->G : 0;   // new tokens (or sharing members) per tile
  // a short draft (2 .. prefill_min - 1 new tokens) shares one pass over its file: 16 MFMA columns = tokens x heads
  c->row_tokens = cfg->dtype == SYM_BF16 ? std::max(1, std::min(tun.row_tokens, std::min<int>(ROW_TOKENS_MAX, 16 / c->G))) : 1;
  c->range_cost = std::max(0, tun.range_cost);
  c->bin_tolerance = std::max(0, tun.bin_tolerance);
  c->bin_waves = tun.bin_waves == 4 ? 4 : 8;
  c->fuse_append = tun.fuse_append ? 1 : 0;
  c->mix_lead = std::min(std::max(tun.mix_lead, 0), 100);
  c->mix_spread = std::min(std::max(tun.mix_spread, 0), 100 - c->mix_lead);
  c->share_tiles = std::min(std::max(tun.share_tiles, 1), 1 << 16);
  if (cfg->device >= 0 && cfg->workspace_bytes < partial_bytes(c) + 4096) {
    sym_destroy(c);
    return SYM_ENOSPC;
  }
  *out = c;
  return SYM_OK;
}

void sym_destroy(sym_ctx* c) {
  if (!c) return;
  if (c->cfg.device >= 0) {
    for (int i = 0; i < kStages; ++i) {
      if (c->stage_pending[i]) (void)hipEventSynchronize(c->stage_ev[i]);
      if (c->stage[i]) (void)hipHostFree(c->stage[i]);
      (void)hipEventDestroy(c->stage_ev[i]);
    }
    for (uint8_t* p : c->host_chunks) (void)hipHostFree(p);
    for (int k = 0; k < SYM_K_COUNT; ++k)
      for (size_t i = 0; i < c->ev_start[k].size(); ++i) {
        (void)hipEventDestroy(c->ev_start[k][i]);
        (void)hipEventDestroy(c->ev_stop[k][i]);
      }
  }
  delete c->fs;
  delete c;
}

const char* sym_strerror(sym_ctx* c) { return c ? c->err.c_str() : "null context"; }

sym_kv sym_kv_open(sym_ctx* c, const char* name) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  return c->fs->open(name);
}

sym_kv sym_kv_fork(sym_ctx* c, sym_kv parent) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_fork")) return busy;
  const int32_t h = c->fs->fork(parent);
  if (h < 0) c->err = h == SYM_EBUSY ? "kv_fork: file is offloaded" : "kv_fork: bad handle";
  return h;
}

int sym_kv_remove(sym_ctx* c, sym_kv kv) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_remove")) return busy;
  const int rc = c->fs->remove(kv);
  if (rc) c->err = "kv_remove: bad handle";
  return rc;
}

int sym_kv_close(sym_ctx* c, sym_kv kv) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_close")) return busy;
  const int rc = c->fs->close(kv);
  if (rc) c->err = "kv_close: bad handle";
  return rc;
}

int64_t sym_kv_len(sym_ctx* c, sym_kv kv) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  return c->fs->len(kv);
}

int sym_kv_truncate(sym_ctx* c, int32_t n, const sym_kv* kv, const int64_t* new_len) {
  if (!c || n < 0 || (n > 0 && (!kv || !new_len))) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_truncate")) return busy;
  for (int32_t i = 0; i < n; ++i) {          // validate everything first: all or nothing
    const KvFile* f = c->fs->file_of(kv[i]);
    if (!f) return fail(c, SYM_EBADF, "kv_truncate: bad handle");
    if (f->waiting) return fail(c, SYM_EBUSY, "kv_truncate: file is offloaded");
    if (new_len[i] < 0 || new_len[i] > f->len) return fail(c, SYM_EINVAL, "kv_truncate: length beyond the file");
    for (int32_t j = 0; j < i; ++j)
      if (c->fs->file_of(kv[j]) == f) return fail(c, SYM_EBUSY, "kv_truncate: file listed twice");
  }
  for (int32_t i = 0; i < n; ++i) (void)c->fs->truncate(kv[i], new_len[i]);
  return SYM_OK;
}

int64_t sym_kv_pages(sym_ctx* c, sym_kv kv, int32_t* out, int64_t cap) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  const KvFile* f = c->fs->file_of(kv);
  if (!f) return fail(c, SYM_EBADF, "kv_pages: bad handle");
  const int64_t n = (int64_t)f->pages.size();
  if (out) copy_bytes(out, f->pages.data(), (size_t)std::min(n, std::max<int64_t>(cap, 0)) * 4);
  return n;
}

int32_t sym_page_refcount(sym_ctx* c, int32_t page) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  return c->fs->refcount(page);
}

int64_t sym_free_pages(sym_ctx* c) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  return c->fs->free_pages();
}

int sym_get_stats(sym_ctx* c, sym_stats* s) {
  if (!c || !s) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  s->pages_total = c->fs->n_pages();
  s->pages_free = c->fs->free_pages();
  s->pages_shared = c->fs->count_shared();
  s->cow_copies = c->fs->cow_copies;
  s->pages_allocated = c->fs->pages_allocated;
  s->tokens_appended = c->fs->tokens_appended;
  s->pred_batches = c->pred_batches;
  s->kernel_launches = c->kernel_launches;
  s->files = c->fs->count_files();
  s->handles = c->fs->count_handles();
  s->host_ns_plan = c->host_ns_plan;
  s->host_ns_pred = c->host_ns_pred;
  s->tokens_moved = c->fs->tokens_moved;
  s->pages_referenced = c->fs->pages_referenced;
  s->pages_offloaded = c->pages_offloaded;
  s->pages_restored = c->pages_restored;
  s->host_slots = c->fs->host_slots();
  s->last_batch_tiles = c->desc_hdr[H_N_TILES];
  s->last_batch_shared_rows = c->desc_hdr[H_N_MEMBERS];
  return SYM_OK;
}

int sym_plan_append(sym_ctx* c, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens, int32_t* cow_out,
                    int64_t cow_cap, int32_t* n_cow, int32_t* slots_out) {
  if (!c || n_lips < 0 || (n_lips > 0 && (!kv || !n_tokens))) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "plan_append")) return busy;
  if (cow_out && cow_cap < n_lips) return fail(c, SYM_EINVAL, "plan_append: cow_cap must be >= n_lips");
  c->plan.clear();
  const int rc = c->fs->append(n_lips, kv, n_tokens, &c->plan, &c->err);
  if (rc) return rc;
  if (n_cow) *n_cow = (int32_t)(c->plan.cow.size() / 3);
  if (cow_out) copy_bytes(cow_out, c->plan.cow.data(), c->plan.cow.size() * 4);
  if (slots_out) copy_bytes(slots_out, c->plan.slots.data(), c->plan.slots.size() * 4);
  return SYM_OK;
}

int sym_plan_copies_first(sym_ctx* c) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  return c->plan.copies_first ? 1 : 0;
}

int64_t sym_build_desc(sym_ctx* c, int32_t n_lips, const int32_t* n_tokens, const int32_t* page_table_flat,
                       const int64_t* pt_offsets, const int64_t* lengths, int32_t* words_out, int64_t cap) {
  if (!c || n_lips < 0 || (n_lips > 0 && (!n_tokens || !page_table_flat || !pt_offsets || !lengths))) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  const int64_t n = desc_from_flat(c, n_lips, n_tokens, page_table_flat, pt_offsets, lengths, [c](int64_t words) {
    c->scratch_words.resize((size_t)words);
    return c->scratch_words.data();
  });
  if (n < 0) return n;
  if (words_out) copy_bytes(words_out, c->desc.words, (size_t)std::min(n, std::max<int64_t>(cap, 0)) * 4);
  return n;
}

int sym_kv_append(sym_ctx* c, sym_kv kv, int32_t n, const void* k, const void* v, void* stream) {
  if (!c || !k || !v) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->cfg.device < 0) return fail(c, SYM_EINVAL, "host-only context");
  int rc;
  if ((rc = refuse_if_open(c, "kv_append"))) return rc;
  hipStream_t st = (hipStream_t)stream;
  if ((int64_t)n + 3 + 64 > c->cfg.workspace_bytes / 4) return fail(c, SYM_ENOSPC, "workspace too small");
  if ((rc = stage_reserve(c, (int64_t)std::max(n, 0) + 3))) return rc;      // before any state change
  c->plan.clear();
  if ((rc = c->fs->append(1, &kv, &n, &c->plan, &c->err))) return rc;
  const int64_t words = (int64_t)c->plan.cow.size() + (int64_t)c->plan.slots.size();
  int si;
  if ((rc = stage_acquire(c, words, &si))) return rc;
  copy_bytes(c->stage[si], c->plan.cow.data(), c->plan.cow.size() * 4);
  copy_bytes(c->stage[si] + c->plan.cow.size(), c->plan.slots.data(), c->plan.slots.size() * 4);
  const int64_t layer_rows = (int64_t)n * c->cfg.n_kv_heads * 256;           // bytes of one layer's rows in k and in v
  for (int32_t l = 0; l < c->n_layers; ++l)
    if ((rc = launch_prologue(c, si, 0, c->stage[si], (int)(c->plan.cow.size() / 3), c->stage[si] + c->plan.cow.size(), n,
                              (const uint8_t*)k + l * layer_rows, (const uint8_t*)v + l * layer_rows, st, nullptr, true, l)))
      return rc;
  return stage_release(c, si, st);
}

int sym_kv_extract(sym_ctx* c, int32_t n_files, const sym_kv* src, const int64_t* idx_off, const int64_t* idx, sym_kv* out,
                   void* stream) {
  if (!c || n_files < 0) return SYM_EINVAL;
  if (n_files == 0) return SYM_OK;
  if (!src || !idx_off || !out || (idx_off[n_files] > 0 && !idx)) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_extract")) return busy;
  const int64_t none = 0;
  if (!idx) idx = &none;
  int64_t need = 0;                                       // all files or none: plan them all, count the fresh pages
  c->gplan.reset();
  for (int32_t i = 0; i < n_files; ++i) {
    const int64_t k = c->fs->gather_need(1, src + i, idx_off + i, idx, &c->gplan, &c->err);
    if (k < 0) return (int)k;
    need += k;
  }
  if (need > c->fs->free_pages()) return fail(c, SYM_ENOSPC, "page pool exhausted");
  if (int rc = stage_reserve(c, move_stage_words(c, idx_off[n_files] - idx_off[0]))) return rc;      // before any state change
  for (int32_t i = 0; i < n_files; ++i) out[i] = c->fs->gather_commit(&c->gplan, i);
  return c->cfg.device < 0 ? SYM_OK : run_moves(c, (hipStream_t)stream);
}

sym_kv sym_kv_merge(sym_ctx* c, int32_t m, const sym_kv* files, void* stream) {
  if (!c || m < 0 || (m > 0 && !files)) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_merge")) return busy;
  int64_t tokens = 0;
  for (int32_t i = 0; i < m; ++i) tokens += std::max<int64_t>(c->fs->len(files[i]), 0);
  if (int rc = stage_reserve(c, move_stage_words(c, tokens))) return rc;      // before any state change
  const sym_kv h = c->fs->gather(m, files, nullptr, nullptr, &c->gplan, &c->err);
  if (h < 0 || c->cfg.device < 0) return h;
  const int rc = run_moves(c, (hipStream_t)stream);
  return rc ? rc : h;
}

int sym_kv_offload(sym_ctx* c, int32_t n, const sym_kv* kv, void* stream) {
  if (!c || n < 0 || (n > 0 && !kv)) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_offload")) return busy;
  int rc;
  // Host memory and staging first, so that running out of either changes nothing: at most every
  // page of the files leaves, into the lowest free slots.
  int64_t pages = 0;
  for (int32_t b = 0; b < n; ++b) {
    const KvFile* f = c->fs->file_of(kv[b]);
    if (f) pages += (int64_t)f->pages.size();
  }
  if ((rc = stage_reserve(c, swap_stage_words(pages)))) return rc;
  if (c->cfg.device >= 0 && (rc = ensure_host_slots(c, std::max(c->fs->host_slots(), c->fs->host_slots_in_use() + pages)))) return rc;
  if ((rc = c->fs->offload(n, kv, &c->splan, &c->err))) return rc;
  if (c->cfg.device < 0) {
    c->pages_offloaded += (int64_t)c->splan.pairs.size() / 2;
    return SYM_OK;
  }
  return run_swaps(c, true, (hipStream_t)stream);
}

int sym_kv_restore(sym_ctx* c, int32_t n, const sym_kv* kv, void* stream) {
  if (!c || n < 0 || (n > 0 && !kv)) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (int busy = refuse_if_open(c, "kv_restore")) return busy;
  int64_t pages = 0;
  for (int32_t b = 0; b < n; ++b) {
    const KvFile* f = c->fs->file_of(kv[b]);
    if (f) pages += (int64_t)f->pages.size();
  }
  if (int rs = stage_reserve(c, swap_stage_words(pages))) return rs;      // before any state change
  const int rc = c->fs->restore(n, kv, &c->splan, &c->err);
  if (rc || c->cfg.device < 0) {
    if (!rc) c->pages_restored += (int64_t)c->splan.pairs.size() / 2;
    return rc;
  }
  return run_swaps(c, false, (hipStream_t)stream);
}

int sym_kv_waiting(sym_ctx* c, sym_kv kv) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  return c->fs->waiting(kv);
}

int64_t sym_last_swaps(sym_ctx* c, int32_t* out, int64_t cap) {
  if (!c || cap < 0) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  const int64_t n = (int64_t)c->splan.pairs.size() / 2;
  if (out) copy_bytes(out, c->splan.pairs.data(), (size_t)std::min(n, cap) * 8);
  return n;
}

int64_t sym_last_moves(sym_ctx* c, int32_t* out, int64_t cap) {
  if (!c || cap < 0) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  const int64_t n = (int64_t)c->gplan.moves.size() / 2;
  if (out) copy_bytes(out, c->gplan.moves.data(), (size_t)std::min(n, cap) * 8);
  return n;
}

int sym_pred_batch(sym_ctx* c, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens, const void* q,
                   const void* k_new, const void* v_new, float* out, void* stream) {
  if (!c || n_lips < 0) return SYM_EINVAL;
  if (n_lips == 0) return SYM_OK;
  if (!kv || !n_tokens || !q || !k_new || !v_new || !out) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->cfg.device < 0) return fail(c, SYM_EINVAL, "host-only context");
  if (c->n_layers != 1) return fail(c, SYM_EINVAL, "pred_batch: a context with several layers runs its batches with sym_pred_begin / sym_pred_layer");
  if (int busy = refuse_if_open(c, "pred_batch")) return busy;
  return pred_batch_locked(c, n_lips, kv, n_tokens, q, k_new, v_new, out, (hipStream_t)stream, workspace_of(c), false);
}

int sym_pred_batch_static(sym_ctx* c, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens, const void* q,
                          const void* k_new, const void* v_new, float* out, void* stream) {
  if (!c || n_lips < 0) return SYM_EINVAL;
  if (n_lips == 0) return SYM_OK;
  if (!kv || !n_tokens || !q || !k_new || !v_new || !out) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->cfg.device < 0) return fail(c, SYM_EINVAL, "host-only context");
  if (!c->static_scratch) return fail(c, SYM_EHIP, "the static scratch array has no address on this device");
  if (c->n_layers != 1) return fail(c, SYM_EINVAL, "pred_batch_static: single-layer contexts only");
  if (int busy = refuse_if_open(c, "pred_batch_static")) return busy;
  // partial slots: what fits behind the largest descriptor this entry point accepts
  Scratch ws{c->static_scratch, kStaticScratchBytes, 0};
  const int64_t slot_bytes = (int64_t)c->G * (2 + c->cfg.head_dim) * 4;
  ws.partials = (ws.bytes - kStaticBlobWords * 4 - 1024) / slot_bytes;
  if (ws.partials < min_partial_slots(c)) return fail(c, SYM_ENOSPC, "pred_batch_static: this shape's partial results do not fit the static scratch");
  return pred_batch_locked(c, n_lips, kv, n_tokens, q, k_new, v_new, out, (hipStream_t)stream, ws, true);
}

int64_t sym_static_scratch_bytes(void) { return kStaticScratchBytes; }

int sym_pred_batch_raw(sym_ctx* c, int32_t n_lips, const int32_t* n_tokens, const int32_t* page_table_flat,
                       const int64_t* pt_offsets, const int64_t* lengths, const void* q, float* out, void* stream) {
  if (!c || n_lips < 0) return SYM_EINVAL;
  if (n_lips == 0) return SYM_OK;
  if (!q || !out || !n_tokens || !page_table_flat || !pt_offsets || !lengths) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->cfg.device < 0) return fail(c, SYM_EINVAL, "host-only context");
  int si = -1;
  const int64_t dwords = desc_from_flat(c, n_lips, n_tokens, page_table_flat, pt_offsets, lengths, [&](int64_t words) -> int32_t* {
    if (align_up(words * 4, 256) + partial_bytes(c) > c->cfg.workspace_bytes) return nullptr;
    return (stage_reserve(c, words + 4) || stage_acquire(c, words + 4, &si)) ? nullptr : c->stage[si];
  });
  if (dwords < 0) return (int)dwords;
  hipStream_t st = (hipStream_t)stream;
  int rc;
  if ((rc = launch_prologue(c, si, dwords, nullptr, 0, nullptr, 0, nullptr, nullptr, st)) || (rc = stage_release(c, si, st))) return rc;
  ++c->pred_batches;
  return launch_attention(c, workspace_of(c), dwords, q, out, st);
}

int sym_pred_begin(sym_ctx* c, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens, void* stream) {
  if (!c || n_lips < 1 || !kv || !n_tokens) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->cfg.device < 0) return fail(c, SYM_EINVAL, "host-only context");
  int rc;
  if ((rc = refuse_if_open(c, "pred_begin"))) return rc;
  const auto t_begin = std::chrono::steady_clock::now();
  PlannedBatch pb;
  if ((rc = pred_plan_locked(c, n_lips, kv, n_tokens, workspace_of(c), false, &pb))) return rc;
  // the whole blob (descriptor, copy list, slot map) goes to the device once; the layers read it there
  hipStream_t st = (hipStream_t)stream;
  if ((rc = launch_prologue(c, pb.si, pb.words, nullptr, 0, nullptr, 0, nullptr, nullptr, st)) || (rc = stage_release(c, pb.si, st))) return rc;
  OpenPred& o = c->pred;
  o.open = true;
  o.words = pb.words;
  o.cow_off = pb.cow_off;
  o.slots_off = pb.slots_off;
  o.n_cow = pb.n_cow;
  o.n_append = pb.n_append;
  o.copies_first = c->plan.copies_first;
  o.partials = pb.partials;
  o.done.assign((size_t)c->n_layers, 0);
  o.n_done = 0;
  ++c->pred_batches;
  const int64_t ns = std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t_begin).count() - pb.wait_ns;
  c->host_ns_plan += ns;
  c->host_ns_pred += ns;
  return SYM_OK;
}

int sym_pred_layer(sym_ctx* c, int32_t layer, const void* q, const void* k_new, const void* v_new, float* out, void* stream) {
  if (!c || !q || !k_new || !v_new || !out) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  OpenPred& o = c->pred;
  if (!o.open) return fail(c, SYM_EINVAL, "pred_layer: no batch is open (sym_pred_begin first)");
  if (layer < 0 || layer >= c->n_layers) return fail(c, SYM_EINVAL, "pred_layer: no such layer");
  if (o.done[layer]) return fail(c, SYM_EBUSY, "pred_layer: this layer of the batch has already run");
  const auto t_begin = std::chrono::steady_clock::now();
  hipStream_t st = (hipStream_t)stream;
  const Scratch ws{(uint8_t*)c->cfg.workspace, c->cfg.workspace_bytes, o.partials};
  const int32_t* cow = (const int32_t*)ws.base + o.cow_off;          // the device copy of the blob
  const int32_t* slots = (const int32_t*)ws.base + o.slots_off;
  int rc, n_cow = o.n_cow;
  if (o.copies_first && n_cow > 0) {
    if ((rc = launch_prologue(c, -1, 0, cow, n_cow, nullptr, 0, nullptr, nullptr, st, nullptr, true, layer))) return rc;
    n_cow = 0;
  }
  if (n_cow > 0 || o.n_append > 0)
    if ((rc = launch_prologue(c, -1, 0, cow, n_cow, slots, o.n_append, k_new, v_new, st, nullptr, true, layer))) return rc;
  rc = launch_attention(c, ws, o.words, q, out, st, true, k_new, v_new, layer);
  if (rc) return rc;
  o.done[layer] = 1;
  if (++o.n_done == c->n_layers) o.open = false;                      // the batch is complete
  c->host_ns_pred += std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t_begin).count();
  return SYM_OK;
}

int sym_pred_end(sym_ctx* c) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  c->pred.open = false;
  return SYM_OK;
}

int sym_test_fail_staging(sym_ctx* c, int32_t count) {
  if (!c || count < 0) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  c->fail_staging = count;
  return SYM_OK;
}

int sym_kv_read_layer(sym_ctx* c, sym_kv kv, int32_t layer, int64_t start, int32_t n, void* k_out, void* v_out, void* stream) {
  if (!c || !k_out || !v_out || n < 0 || start < 0) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->cfg.device < 0) return fail(c, SYM_EINVAL, "host-only context");
  if (layer < 0 || layer >= c->n_layers) return fail(c, SYM_EINVAL, "kv_read: no such layer");
  const KvFile* f = c->fs->file_of(kv);
  if (!f) return fail(c, SYM_EBADF, "kv_read: bad handle");
  if (f->waiting) return fail(c, SYM_EBUSY, "kv_read: file is offloaded");
  if (start + n > f->len) return fail(c, SYM_EINVAL, "kv_read: range beyond the file");
  if (n == 0) return SYM_OK;
  if (int busy = refuse_if_open(c, "kv_read")) return busy;
  if ((int64_t)n + 64 > c->cfg.workspace_bytes / 4) return fail(c, SYM_ENOSPC, "workspace too small");
  const int P = c->cfg.page_tokens;
  int si, rc;
  if ((rc = stage_reserve(c, n)) || (rc = stage_acquire(c, n, &si))) return rc;
  for (int32_t i = 0; i < n; ++i) {
    const int64_t t = start + i;
    c->stage[si][i] = f->pages[t / P] * P + (int32_t)(t % P);
  }
  hipStream_t st = (hipStream_t)stream;
  GatherArgs ga{pool_of(c, layer), c->page_bytes, c->stage[si], n, c->cfg.n_kv_heads};
  hipError_t e = launch_gather(ga, k_out, v_out, st);
  if (e != hipSuccess) return fail_hip(c, e, "gather launch");
  return stage_release(c, si, st);
}

int sym_kv_read(sym_ctx* c, sym_kv kv, int64_t start, int32_t n, void* k_out, void* v_out, void* stream) {
  return sym_kv_read_layer(c, kv, 0, start, n, k_out, v_out, stream);
}

sym_sched* sym_sched_create(int32_t max_batch, double max_wait_us, double weight, double a_us, double c_us) {
  if (max_batch < 1 || !(max_wait_us >= 0.0) || !(weight > 0.0 && weight <= 1.0) || !(a_us >= 0.0) || !(c_us >= 0.0)) return nullptr;
  return reinterpret_cast<sym_sched*>(new BatchTimer(max_batch, max_wait_us, weight, a_us, c_us));
}
void sym_sched_destroy(sym_sched* s) { delete reinterpret_cast<BatchTimer*>(s); }
void sym_sched_arrive(sym_sched* s, double now_us) {
  if (s) reinterpret_cast<BatchTimer*>(s)->arrive(now_us);
}
int32_t sym_sched_decide(sym_sched* s, double now_us, int gpu_idle) {
  return s ? reinterpret_cast<BatchTimer*>(s)->decide(now_us, gpu_idle != 0) : 0;
}
void sym_sched_fired(sym_sched* s, int32_t n) {
  if (s) reinterpret_cast<BatchTimer*>(s)->fired(n);
}
void sym_sched_done(sym_sched* s, int32_t n, double service_us) {
  if (s && n > 0) reinterpret_cast<BatchTimer*>(s)->done(n, service_us);
}
double sym_sched_next_deadline(sym_sched* s) {
  return s ? reinterpret_cast<BatchTimer*>(s)->next_deadline() : std::numeric_limits<double>::infinity();
}
int sym_sched_state(sym_sched* s, double* rate, double* target, double* a_us, double* c_us, int64_t* pending) {
  if (!s) return SYM_EINVAL;
  const BatchTimer* t = reinterpret_cast<const BatchTimer*>(s);
  if (rate) *rate = t->rate();
  if (target) *target = t->target();
  if (a_us) *a_us = t->a();
  if (c_us) *c_us = t->c();
  if (pending) *pending = t->pending();
  return SYM_OK;
}

int sym_profile_enable(sym_ctx* c, int mask) {
  if (!c) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  c->prof_mask = mask & 0xff;
  c->prof_stride = std::max(1, (mask >> 8) & 0xffff);
  for (int k = 0; k < SYM_K_COUNT; ++k) c->prof_seen[k] = 0;
  return SYM_OK;
}

int sym_profile_read(sym_ctx* c, int kid, double* total_ms, int64_t* launches) {
  if (!c || kid < 0 || kid >= SYM_K_COUNT) return SYM_EINVAL;
  std::lock_guard<std::mutex> lk(c->mu);
  double tot = 0;
  for (int i = 0; i < c->ev_used[kid]; ++i) {
    hipError_t e = hipEventSynchronize(c->ev_stop[kid][i]);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev_start[kid][i], c->ev_stop[kid][i]);
    if (e != hipSuccess) return fail_hip(c, e, "profile_read");
    tot += ms;
  }
  if (total_ms) *total_ms = tot;
  if (launches) *launches = c->ev_used[kid];
  c->ev_used[kid] = 0;
  return SYM_OK;
}

int sym_calib_read(const void* src, int64_t bytes, void* out8, void* stream) {
  if (!src || !out8 || bytes <= 0 || bytes % 16) return SYM_EINVAL;
  return launch_calib_read(src, bytes, out8, (hipStream_t)stream) == hipSuccess ? SYM_OK : SYM_EHIP;
}
int sym_calib_mfma(float* out, int32_t blocks, int32_t iters, void* stream) {
  if (!out || blocks < 1 || blocks > 65536 || iters < 1) return SYM_EINVAL;
  return launch_calib_mfma(out, blocks, iters, (hipStream_t)stream) == hipSuccess ? SYM_OK : SYM_EHIP;
}
int sym_calib_copy(void* dst, const void* src, int64_t bytes, void* stream) {
  if (!dst || !src || bytes <= 0 || bytes % 16) return SYM_EINVAL;
  return launch_calib_copy(dst, src, bytes, (hipStream_t)stream) == hipSuccess ? SYM_OK : SYM_EHIP;
}

}  // extern "C"
