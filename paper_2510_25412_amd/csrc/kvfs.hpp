// Host-side state of the KV-cache file system (paper section 4.2): files as page lists,
// per-page reference counts, copy-on-write forks, a ranked set of free pages.  Pure C++, no
// HIP: the integer state is what tests compare bit for bit with the CPU model.
#pragma once
#include <cstdint>
#include <functional>
#include <queue>
#include <string>
#include <unordered_map>
#include <vector>

namespace symkv {

struct KvFile {
  int64_t len = 0;
  std::vector<int32_t> pages;      // page ids; -(slot + 1) for a page that is on the host
  bool waiting = false;            // offloaded: its thread waits for I/O (paper section 4.3)
  std::vector<int32_t> handles;
  std::string name;
  bool named = false;
  bool alive = false;
};

// The set of free ranks with "take the lowest" in a few instructions: a bitmap of the ranks and
// a summary bitmap with one bit per 64-rank word (a 3,000,000-page pool has 733 summary words; the
// scan for the first non-empty one starts at a hint that only moves down when a rank is returned).
class RankSet {
 public:
  void fill(int64_t n) {                      // ranks 0 .. n-1 all free
    l0_.assign((size_t)((n + 63) / 64), ~0ull);
    if (n % 64) l0_.back() = (1ull << (n % 64)) - 1;
    l1_.assign((l0_.size() + 63) / 64, 0);
    for (size_t w = 0; w < l0_.size(); ++w)
      if (l0_[w]) l1_[w >> 6] |= 1ull << (w & 63);
    count_ = n;
    hint_ = 0;
  }
  int64_t size() const { return count_; }
  int32_t pop_lowest() {                      // the caller has checked size() > 0
    size_t i = hint_;
    while (!l1_[i]) ++i;
    hint_ = i;
    const size_t w = i * 64 + (size_t)__builtin_ctzll(l1_[i]);
    const int b = __builtin_ctzll(l0_[w]);
    l0_[w] &= l0_[w] - 1;
    if (!l0_[w]) l1_[i] &= ~(1ull << (w & 63));
    --count_;
    return (int32_t)(w * 64 + (size_t)b);
  }
  void insert(int32_t r) {
    const size_t w = (size_t)r >> 6;
    l0_[w] |= 1ull << (r & 63);
    l1_[w >> 6] |= 1ull << (w & 63);
    if ((w >> 6) < hint_) hint_ = w >> 6;
    ++count_;
  }

 private:
  std::vector<uint64_t> l0_, l1_;
  int64_t count_ = 0;
  size_t hint_ = 0;
};

// Result of planning a batch of appends (reused between calls: no per-call allocation once warm).
struct AppendPlan {
  std::vector<int32_t> cow;       // (src, dst, r) triples: copy slots [0, r) of src into dst
  std::vector<int32_t> slots;     // per new token: page * P + slot
  // Copies and appends of one batch normally touch disjoint bytes (files that share a partly filled
  // page see the same number of tokens in it: the copies take the slots below, the appends the slots
  // from there on) and may run in any order.  Not so after a truncate or an extract left a sharer
  // that sees FEWER tokens of the page: when the files that see more have copied the page and left,
  // it appends in place, into slots that their copies still have to read.  Then the copies go first.
  bool copies_first = false;
  void clear() { cow.clear(); slots.clear(); copies_first = false; }
};

// Result of building a file out of tokens of existing files (extract / merge).
struct GatherPlan {
  std::vector<int32_t> moves;     // (source, destination) pairs of token slots (page * P + slot) to copy
  int64_t pages_shared = 0;       // destination pages that reference an existing page instead
  // scratch of the planning pass, one stretch per planned file
  std::vector<int32_t> src;       // source slot of every destination token
  std::vector<int32_t> shared;    // per destination page, the page it references or -1
  std::vector<int64_t> bounds;    // per planned file: where its stretch of src / of shared begins
  void reset() { moves.clear(); src.clear(); shared.clear(); bounds.clear(); pages_shared = 0; }
};

// Page copies of an offload ((page, host slot) pairs, device to host) or of a restore ((host
// slot, page) pairs, host to device), in the order they must happen.
struct SwapPlan {
  std::vector<int32_t> pairs;
};

class Kvfs {
 public:
  Kvfs(int64_t n_pages, int32_t page_tokens, const int32_t* free_order);

  int32_t open(const char* name);                 // handle or negative status
  int32_t fork(int32_t parent);
  int remove(int32_t h);
  int close(int32_t h);
  int64_t len(int32_t h) const;
  int truncate(int32_t h, int64_t new_len);   // drop tokens from new_len on; frees pages no longer needed
  const KvFile* file_of(int32_t h) const;

  // Pages a batch would allocate, LIPs in batch order; negative status on a bad argument.
  int64_t pages_needed(int32_t n, const int32_t* handles, const int32_t* n_tokens, std::string* err);
  // Two-phase: validate + count, then commit.  On error nothing changes.
  int append(int32_t n, const int32_t* handles, const int32_t* n_tokens, AppendPlan* plan, std::string* err);

  // extract / merge (paper section 4.2): a new anonymous file of the tokens of n_seg segments, one
  // after the other.  Segment s takes from file seg_handle[s]: with idx, the tokens
  // idx[seg_off[s]] .. idx[seg_off[s+1] - 1] (any order, repeats allowed); without, the whole
  // file in order.  A destination page that is slots 0, 1, 2, ... of one existing page
  // references that page; every other one is a fresh page and its tokens go into plan->moves.
  // gather_need validates one file and adds it to the plan's scratch; returns the fresh pages it
  // needs or a negative status.  gather_commit builds planned file k from that scratch (the
  // caller has checked that the pages are free), appends its copies to plan->moves and returns
  // the handle.  gather = one file, both steps, with the free-page check (on error nothing changed).
  int64_t gather_need(int32_t n_seg, const int32_t* seg_handle, const int64_t* seg_off, const int64_t* idx, GatherPlan* plan,
                      std::string* err);
  int32_t gather_commit(GatherPlan* plan, int32_t k);
  int32_t gather(int32_t n_seg, const int32_t* seg_handle, const int64_t* seg_off, const int64_t* idx, GatherPlan* plan,
                 std::string* err);

  // offload / restore (paper section 4.3: the KV cache of a thread that waits for I/O moves to CPU
  // memory and comes back when the wait ends).  A waiting file cannot be read or written
  // (SYM_EBUSY) but can be removed.  A page leaves when EVERY reference to it belongs to a waiting
  // file: lowest free host slot, all referencing entries become -(slot + 1), the page is freed.
  // restore brings each host slot of the files back into a fresh page and rewrites every entry
  // that referenced the slot, also those of files still waiting.  All or nothing.
  int offload(int32_t n, const int32_t* handles, SwapPlan* plan, std::string* err);
  int restore(int32_t n, const int32_t* handles, SwapPlan* plan, std::string* err);
  int waiting(int32_t h) const;                 // 1, 0 or a negative status
  int64_t host_slots() const { return n_slots_; }   // host slots ever created (ids 0 .. n - 1)
  int64_t host_slots_in_use() const { return (int64_t)host_refs_.size(); }

  int32_t refcount(int32_t page) const { return page < 0 || page >= n_pages_ ? -1 : (int32_t)refcount_[page]; }
  int64_t free_pages() const { return free_ranks_.size(); }
  int64_t n_pages() const { return n_pages_; }
  int32_t page_tokens() const { return P_; }

  int64_t cow_copies = 0, pages_allocated = 0, tokens_appended = 0, tokens_moved = 0, pages_referenced = 0;
  int64_t count_shared() const;
  int64_t count_files() const;
  int64_t count_handles() const;

 private:
  int32_t alloc_page();
  void release_entries(int32_t file_id, size_t keep);
  void drop_ref(int32_t page);
  int check_swap_args(int32_t n, const int32_t* handles, bool want_waiting, std::string* err);
  int32_t new_handle(int32_t file_id);
  int32_t new_file();
  void drop_file(int32_t file_id);

  int64_t n_pages_;
  int32_t P_;
  int page_shift_ = -1;                     // log2(P_) when P_ is a power of two, else -1
  std::vector<uint32_t> refcount_;
  std::vector<int32_t> order_, rank_;       // rank -> page, page -> rank
  RankSet free_ranks_;
  std::vector<KvFile> files_;
  std::vector<int32_t> free_file_ids_;
  std::vector<int32_t> handle_file_;        // handle -> file id or -1
  std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> free_handles_;
  std::unordered_map<std::string, int32_t> names_;
  typedef std::vector<std::pair<int32_t, int32_t>> RefList;          // (file id, table index) entries
  std::unordered_map<int32_t, RefList> waiters_;    // resident page -> entries of waiting files that reference it
  std::unordered_map<int32_t, RefList> host_refs_;  // host slot -> entries that reference it
  std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> free_slots_;
  int32_t n_slots_ = 0;
  std::unordered_map<int32_t, int32_t> pending_;   // scratch of pages_needed
  std::vector<int32_t> seen_files_;                 // scratch of append
};

}  // namespace symkv
