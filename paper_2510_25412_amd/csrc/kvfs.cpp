// KV-cache file system host state (paper section 4.2).  See kvfs.hpp.
#include "kvfs.hpp"

#include <algorithm>
#include <numeric>

#include "../../include/symphony_kv.h"

namespace symkv {

Kvfs::Kvfs(int64_t n_pages, int32_t page_tokens, const int32_t* free_order)
    : n_pages_(n_pages), P_(page_tokens), refcount_(n_pages, 0), order_(n_pages), rank_(n_pages) {
  if (free_order) {
    std::copy(free_order, free_order + n_pages, order_.begin());
  } else {
    std::iota(order_.begin(), order_.end(), 0);
  }
  for (int64_t r = 0; r < n_pages; ++r) rank_[order_[r]] = (int32_t)r;
  for (int s = 0; s < 16; ++s)
    if ((1 << s) == page_tokens) page_shift_ = s;
  free_ranks_.fill(n_pages);
}

const KvFile* Kvfs::file_of(int32_t h) const {
  if (h < 0 || h >= (int32_t)handle_file_.size() || handle_file_[h] < 0) return nullptr;
  return &files_[handle_file_[h]];
}

int32_t Kvfs::alloc_page() {
  int32_t p = order_[free_ranks_.pop_lowest()];   // lowest rank, whatever the release order
  refcount_[p] = 1;
  ++pages_allocated;
  return p;
}

void Kvfs::drop_ref(int32_t p) {
  if (--refcount_[p] == 0) free_ranks_.insert(rank_[p]);
}

namespace {
void erase_ref(std::vector<std::pair<int32_t, int32_t>>& v, int32_t file_id, int32_t idx) {
  auto it = std::find(v.begin(), v.end(), std::make_pair(file_id, idx));
  if (it != v.end()) {
    *it = v.back();
    v.pop_back();
  }
}
}  // namespace

// Drops the file's table entries from index keep on.
void Kvfs::release_entries(int32_t id, size_t keep) {
  KvFile& f = files_[id];
  for (size_t i = keep; i < f.pages.size(); ++i) {
    const int32_t e = f.pages[i];
    if (e >= 0) {
      if (f.waiting) {
        auto w = waiters_.find(e);
        erase_ref(w->second, id, (int32_t)i);
        if (w->second.empty()) waiters_.erase(w);
      }
      drop_ref(e);
    } else {                                  // on the host: the slot is free once nobody refers to it
      auto r = host_refs_.find(-e - 1);
      erase_ref(r->second, id, (int32_t)i);
      if (r->second.empty()) {
        host_refs_.erase(r);
        free_slots_.push(-e - 1);
      }
    }
  }
  f.pages.resize(keep);
}

int32_t Kvfs::new_file() {
  int32_t id;
  if (!free_file_ids_.empty()) {
    id = free_file_ids_.back();
    free_file_ids_.pop_back();
  } else {
    id = (int32_t)files_.size();
    files_.emplace_back();
  }
  KvFile& f = files_[id];
  f.len = 0;
  f.pages.clear();
  f.handles.clear();
  f.name.clear();
  f.named = false;
  f.alive = true;
  f.waiting = false;
  return id;
}

int32_t Kvfs::new_handle(int32_t file_id) {
  int32_t h;
  if (!free_handles_.empty()) {
    h = free_handles_.top();               // lowest free handle slot
    free_handles_.pop();
  } else {
    h = (int32_t)handle_file_.size();
    handle_file_.push_back(-1);
  }
  handle_file_[h] = file_id;
  files_[file_id].handles.push_back(h);
  return h;
}

void Kvfs::drop_file(int32_t id) {
  KvFile& f = files_[id];
  release_entries(id, 0);
  f.len = 0;
  f.waiting = false;
  for (int32_t h : f.handles) {
    handle_file_[h] = -1;
    free_handles_.push(h);
  }
  f.handles.clear();
  if (f.named) names_.erase(f.name);
  f.alive = false;
  free_file_ids_.push_back(id);
}

int32_t Kvfs::open(const char* name) {
  if (name) {
    auto it = names_.find(name);
    if (it != names_.end()) return new_handle(it->second);   // second handle, same file
  }
  int32_t id = new_file();
  if (name) {
    files_[id].name = name;
    files_[id].named = true;
    names_[name] = id;
  }
  return new_handle(id);
}

int32_t Kvfs::fork(int32_t parent) {
  const KvFile* pf = file_of(parent);
  if (!pf) return SYM_EBADF;
  if (pf->waiting) return SYM_EBUSY;
  int32_t pid = handle_file_[parent];
  int32_t id = new_file();                  // may grow files_: re-read the parent by index
  KvFile& child = files_[id];
  const KvFile& par = files_[pid];
  child.pages = par.pages;
  child.len = par.len;
  for (int32_t p : child.pages) ++refcount_[p];
  return new_handle(id);
}

int Kvfs::remove(int32_t h) {
  if (!file_of(h)) return SYM_EBADF;
  drop_file(handle_file_[h]);
  return SYM_OK;
}

int Kvfs::close(int32_t h) {
  if (!file_of(h)) return SYM_EBADF;
  int32_t id = handle_file_[h];
  KvFile& f = files_[id];
  f.handles.erase(std::find(f.handles.begin(), f.handles.end(), h));
  handle_file_[h] = -1;
  free_handles_.push(h);
  if (!f.named && f.handles.empty()) drop_file(id);   // nobody can reach it any more
  return SYM_OK;
}

int64_t Kvfs::len(int32_t h) const {
  const KvFile* f = file_of(h);
  return f ? f->len : (int64_t)SYM_EBADF;
}

int Kvfs::truncate(int32_t h, int64_t new_len) {
  if (!file_of(h)) return SYM_EBADF;
  KvFile& f = files_[handle_file_[h]];
  if (f.waiting) return SYM_EBUSY;
  if (new_len < 0 || new_len > f.len) return SYM_EINVAL;
  release_entries(handle_file_[h], (size_t)((new_len + P_ - 1) / P_));
  f.len = new_len;
  return SYM_OK;
}

int64_t Kvfs::pages_needed(int32_t n, const int32_t* handles, const int32_t* n_tokens, std::string* err) {
  pending_.clear();
  seen_files_.clear();
  int64_t need = 0;
  for (int32_t b = 0; b < n; ++b) {
    const KvFile* f = file_of(handles[b]);
    if (!f) {
      if (err) *err = "bad file handle in batch";
      return SYM_EBADF;
    }
    if (n_tokens[b] < 1) {
      if (err) *err = "n_tokens must be >= 1";
      return SYM_EINVAL;
    }
    if (f->waiting) {
      if (err) *err = "file is offloaded";
      return SYM_EBUSY;
    }
    int32_t id = handle_file_[handles[b]];
    if (std::find(seen_files_.begin(), seen_files_.end(), id) != seen_files_.end()) {
      if (err) *err = "same file twice in one batch";
      return SYM_EBUSY;
    }
    seen_files_.push_back(id);
    int64_t L = f->len;
    if (L % P_ != 0) {
      int32_t last = f->pages.back();
      int64_t rc = (int64_t)refcount_[last];
      auto it = pending_.find(last);
      if (it != pending_.end()) rc += it->second;
      if (rc > 1) {                        // shared, partly filled: this LIP copies it
        ++need;
        pending_[last] -= 1;
      }
    }
    need += (L + n_tokens[b] + P_ - 1) / P_ - (L + P_ - 1) / P_;
  }
  return need;
}

int Kvfs::append(int32_t n, const int32_t* handles, const int32_t* n_tokens, AppendPlan* plan, std::string* err) {
  int64_t need = pages_needed(n, handles, n_tokens, err);
  if (need < 0) return (int)need;
  if (need > free_pages()) {
    if (err) *err = "page pool exhausted";
    return SYM_ENOSPC;
  }
  for (int32_t b = 0; b < n; ++b) {
    KvFile& f = files_[handle_file_[handles[b]]];
    int32_t r = (int32_t)(f.len % P_);
    if (r != 0 && refcount_[f.pages.back()] > 1) {
      int32_t src = f.pages.back();
      int32_t dst = alloc_page();
      --refcount_[src];
      f.pages.back() = dst;
      ++cow_copies;
      if (plan) {
        plan->cow.push_back(src);
        plan->cow.push_back(dst);
        plan->cow.push_back(r);
      }
    } else if (r != 0 && plan && !plan->copies_first) {
      // appending in place into a partly filled page: were more of its slots than this file sees
      // copied out earlier in this batch?
      const int32_t page = f.pages.back();
      for (size_t c = 0; c < plan->cow.size(); c += 3)
        if (plan->cow[c] == page && plan->cow[c + 2] > r) {
          plan->copies_first = true;
          break;
        }
    }
    for (int32_t i = 0; i < n_tokens[b]; ++i) {
      if (f.len % P_ == 0) f.pages.push_back(alloc_page());
      if (plan) plan->slots.push_back(f.pages.back() * P_ + (int32_t)(f.len % P_));
      ++f.len;
    }
    tokens_appended += n_tokens[b];
  }
  return SYM_OK;
}

int64_t Kvfs::gather_need(int32_t n_seg, const int32_t* seg_handle, const int64_t* seg_off, const int64_t* idx, GatherPlan* plan,
                          std::string* err) {
  std::vector<int32_t>& src = plan->src;
  std::vector<int32_t>& shared = plan->shared;
  const size_t s0 = src.size(), h0 = shared.size();
  plan->bounds.push_back((int64_t)s0);
  plan->bounds.push_back((int64_t)h0);
  for (int32_t s = 0; s < n_seg; ++s) {
    const KvFile* f = file_of(seg_handle[s]);
    if (!f) {
      if (err) *err = "extract/merge: bad file handle";
      return SYM_EBADF;
    }
    if (f->waiting) {
      if (err) *err = "extract/merge: file is offloaded";
      return SYM_EBUSY;
    }
    const int64_t lo = idx ? seg_off[s] : 0, hi = idx ? seg_off[s + 1] : f->len;
    if (hi < lo || (int64_t)(src.size() - s0) + (hi - lo) > (int64_t)0x7fffffff) {
      if (err) *err = "extract/merge: bad segment bounds or result too long";
      return SYM_EINVAL;
    }
    const size_t at = src.size();
    src.resize(at + (size_t)(hi - lo));
    int32_t* out = src.data() + at;
    const int32_t* pages = f->pages.data();
    const int64_t len = f->len;
    const int sh = page_shift_;                            // page size is a power of two on the device path
    for (int64_t j = lo; j < hi; ++j) {
      const int64_t i = idx ? idx[j] : j;
      if ((uint64_t)i >= (uint64_t)len) {
        src.resize(at);
        if (err) *err = "extract: token index outside the file";
        return SYM_EINVAL;
      }
      *out++ = sh >= 0 ? (pages[i >> sh] << sh) + (int32_t)(i & (P_ - 1)) : pages[i / P_] * P_ + (int32_t)(i % P_);
    }
  }
  const int64_t n = (int64_t)(src.size() - s0), np = (n + P_ - 1) / P_;
  shared.resize(h0 + (size_t)np, -1);
  int64_t need = 0;
  for (int64_t d = 0; d < np; ++d) {
    const int64_t base = (int64_t)s0 + d * P_, c = std::min<int64_t>(P_, n - d * P_);
    const int32_t first = src[base];
    bool same = first % P_ == 0;
    for (int64_t k = 1; k < c && same; ++k) same = src[base + k] == first + (int32_t)k;
    if (same) shared[h0 + d] = first / P_;
    else ++need;
  }
  return need;
}

int32_t Kvfs::gather_commit(GatherPlan* plan, int32_t k) {
  const bool last = (size_t)(2 * k + 2) >= plan->bounds.size();
  const int64_t s0 = plan->bounds[2 * k], h0 = plan->bounds[2 * k + 1];
  const int64_t n = (last ? (int64_t)plan->src.size() : plan->bounds[2 * k + 2]) - s0;
  const int64_t np = (last ? (int64_t)plan->shared.size() : plan->bounds[2 * k + 3]) - h0;
  const int32_t* src = plan->src.data() + s0;
  const int32_t* shared = plan->shared.data() + h0;
  const int32_t id = new_file();
  files_[id].pages.reserve((size_t)np);
  for (int64_t d = 0; d < np; ++d) {
    if (shared[d] >= 0) {
      ++refcount_[shared[d]];
      files_[id].pages.push_back(shared[d]);
      ++plan->pages_shared;
      ++pages_referenced;
    } else {
      const int32_t dst = alloc_page();
      files_[id].pages.push_back(dst);
      const int64_t base = d * P_, c = std::min<int64_t>(P_, n - base);
      const size_t at = plan->moves.size();
      plan->moves.resize(at + (size_t)(2 * c));
      int32_t* mv = plan->moves.data() + at;
      for (int64_t t = 0; t < c; ++t) {
        mv[2 * t] = src[base + t];
        mv[2 * t + 1] = dst * P_ + (int32_t)t;
      }
      tokens_moved += c;
    }
  }
  files_[id].len = n;
  return new_handle(id);
}

int32_t Kvfs::gather(int32_t n_seg, const int32_t* seg_handle, const int64_t* seg_off, const int64_t* idx, GatherPlan* plan,
                     std::string* err) {
  plan->reset();
  const int64_t need = gather_need(n_seg, seg_handle, seg_off, idx, plan, err);
  if (need < 0) return (int32_t)need;
  if (need > free_pages()) {
    if (err) *err = "page pool exhausted";
    return SYM_ENOSPC;
  }
  return gather_commit(plan, 0);
}

int Kvfs::waiting(int32_t h) const {
  const KvFile* f = file_of(h);
  return f ? (f->waiting ? 1 : 0) : SYM_EBADF;
}

int Kvfs::check_swap_args(int32_t n, const int32_t* handles, bool want_waiting, std::string* err) {
  seen_files_.clear();
  for (int32_t b = 0; b < n; ++b) {
    const KvFile* f = file_of(handles[b]);
    if (!f) {
      if (err) *err = "offload/restore: bad file handle";
      return SYM_EBADF;
    }
    const int32_t id = handle_file_[handles[b]];
    if (f->waiting != want_waiting || std::find(seen_files_.begin(), seen_files_.end(), id) != seen_files_.end()) {
      if (err) *err = want_waiting ? "restore: file is not offloaded, or named twice" : "offload: file already offloaded, or named twice";
      return SYM_EBUSY;
    }
    seen_files_.push_back(id);
  }
  return SYM_OK;
}

int Kvfs::offload(int32_t n, const int32_t* handles, SwapPlan* plan, std::string* err) {
  plan->pairs.clear();
  const int rc = check_swap_args(n, handles, false, err);
  if (rc) return rc;
  for (int32_t b = 0; b < n; ++b) {
    const int32_t id = handle_file_[handles[b]];
    KvFile& f = files_[id];
    f.waiting = true;
    for (size_t i = 0; i < f.pages.size(); ++i) {
      const int32_t p = f.pages[i];
      RefList& w = waiters_[p];
      w.emplace_back(id, (int32_t)i);
      if (w.size() != refcount_[p]) continue;
      int32_t s;                                  // every reader waits: the page leaves for the lowest free slot
      if (!free_slots_.empty()) {
        s = free_slots_.top();
        free_slots_.pop();
      } else {
        s = n_slots_++;
      }
      for (const auto& r : w) files_[r.first].pages[r.second] = -(s + 1);
      host_refs_[s] = std::move(w);
      waiters_.erase(p);
      refcount_[p] = 0;
      free_ranks_.insert(rank_[p]);
      plan->pairs.push_back(p);
      plan->pairs.push_back(s);
    }
  }
  return SYM_OK;
}

int Kvfs::restore(int32_t n, const int32_t* handles, SwapPlan* plan, std::string* err) {
  plan->pairs.clear();
  const int rc = check_swap_args(n, handles, true, err);
  if (rc) return rc;
  pending_.clear();                               // distinct host slots of the files
  for (int32_t id : seen_files_)
    for (int32_t e : files_[id].pages)
      if (e < 0) pending_[-e - 1] = 1;
  if ((int64_t)pending_.size() > free_pages()) {
    if (err) *err = "page pool exhausted";
    return SYM_ENOSPC;
  }
  for (int32_t b = 0; b < n; ++b) {
    const int32_t id = handle_file_[handles[b]];
    files_[id].waiting = false;
    for (size_t i = 0; i < files_[id].pages.size(); ++i) {
      const int32_t e = files_[id].pages[i];
      if (e >= 0) {                               // never left, or already back through another entry
        auto w = waiters_.find(e);
        if (w != waiters_.end()) {
          erase_ref(w->second, id, (int32_t)i);
          if (w->second.empty()) waiters_.erase(w);
        }
        continue;
      }
      const int32_t s = -e - 1;
      const int32_t q = alloc_page();
      RefList refs = std::move(host_refs_[s]);
      host_refs_.erase(s);
      RefList still;
      for (const auto& r : refs) {
        files_[r.first].pages[r.second] = q;
        if (files_[r.first].waiting) still.push_back(r);
      }
      refcount_[q] = (uint32_t)refs.size();
      if (!still.empty()) waiters_[q] = std::move(still);
      free_slots_.push(s);
      plan->pairs.push_back(s);
      plan->pairs.push_back(q);
    }
  }
  return SYM_OK;
}

int64_t Kvfs::count_shared() const {
  int64_t c = 0;
  for (uint32_t r : refcount_) c += r > 1;
  return c;
}
int64_t Kvfs::count_files() const {
  int64_t c = 0;
  for (const KvFile& f : files_) c += f.alive;
  return c;
}
int64_t Kvfs::count_handles() const {
  int64_t c = 0;
  for (int32_t f : handle_file_) c += f >= 0;
  return c;
}

}  // namespace symkv
