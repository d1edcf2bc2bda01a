// Batch-descriptor builder (host, integer work only).  See desc.hpp.
#include "desc.hpp"

#include <algorithm>
#include <cstring>

#include "../../include/symphony_kv.h"

namespace symkv {

int build_desc(const DescParams& prm, int32_t n_lips, const int32_t* n_tokens, const int64_t* len_after,
               const int32_t* const* tables, BatchDesc* out) {
  const int32_t P = prm.page_tokens, H = prm.n_kv_heads, G = prm.n_q_heads / H;
  auto is_prefill = [&](int32_t b) { return prm.tile_tokens > 0 && n_tokens[b] >= prm.prefill_min; };
  // Tiles of a batch with prefill chunks have prm.tile_tokens new tokens (256 query rows by default:
  // eight wavefronts share one staging of K/V); a batch whose only tiles are shared prefixes (few
  // members per group) keeps 128-row tiles, two workgroups per CU.
  bool any_prefill = false;
  for (int32_t b = 0; b < n_lips && !any_prefill; ++b) any_prefill = n_tokens[b] >= 1 && is_prefill(b);
  const int32_t TQ = any_prefill ? prm.tile_tokens : std::min(prm.tile_tokens, 128 / G);
  // A decode row holds up to RT consecutive new tokens of one LIP (a short draft to verify):
  // they share one pass over the file's pages.
  const int32_t RT = std::max(1, std::min(prm.row_tokens, (int32_t)ROW_TOKENS_MAX));
  int32_t max_nt = 1;
  int64_t n_rows = 0, entries = 0, n_tiles = 0, n_tok_total = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    if (n_tokens[b] < 1 || len_after[b] < n_tokens[b] || len_after[b] > (int64_t)0x7fffffff) return SYM_EINVAL;
    if (is_prefill(b)) n_tiles += (int64_t)((n_tokens[b] + TQ - 1) / TQ) * H;
    else {
      n_rows += (n_tokens[b] + RT - 1) / RT;
      max_nt = std::max(max_nt, std::min(RT, n_tokens[b]));
    }
    n_tok_total += n_tokens[b];
    entries += (len_after[b] + P - 1) / P;
  }
  if (n_tok_total > 0x7fffffff / (2 * H) || entries > 0x3fffffff || n_tiles > 0x0fffffff) return SYM_EINVAL;

  // ---- sharing groups: single-token LIPs whose files begin with the same pages.  Same page id
  // means same bytes, so the group's common FULL pages can be read once for all members.
  std::vector<int32_t>& share_start = out->share_start;   // per LIP: pages covered by the group (0 = none)
  std::vector<int32_t>& share_base = out->share_base;     // per LIP: first shared partial of its member tile
  std::vector<int32_t>& share_k = out->share_k;           // per LIP: members in its tile
  std::vector<int32_t>& share_ml = out->share_ml;         // per LIP: its index among them
  std::vector<int32_t>& share_nc = out->share_nc;         // per LIP: key chunks of the common prefix
  std::vector<int32_t>& member_rows = out->member_rows;   // q rows of the members, tile after tile
  std::vector<int32_t>& stiles = out->shared_tiles;       // (first lip, member offset, K, C, NC, partial base) per member tile
  share_start.assign(n_lips, 0);
  share_base.assign(n_lips, 0);
  share_k.assign(n_lips, 0);
  share_ml.assign(n_lips, 0);
  share_nc.assign(n_lips, 0);
  member_rows.clear();
  stiles.clear();
  int64_t n_shared_partials = 0, n_shared_tiles = 0;
  // Partial slots: a wave boundary cuts one (row, head), whose two pieces leave a partial per token
  // of the row; the rest is split between the prefix partials of sharing groups and the
  // members' own ranges (one partial per (member, head), never more than the former).
  const int64_t shared_budget = std::max<int64_t>(0, ((int64_t)prm.max_partials - 2 * (int64_t)RT * prm.max_waves) / 2);
  const int32_t tile_lips = TQ;                             // members of a shared-prefix tile (rows = members x G)
  if (prm.share_min_lips > 0 && tile_lips > 0) {
    auto& cand = out->by_first_page;
    cand.clear();
    std::vector<int32_t>& qrow_of = out->qrow_of;            // token index of each LIP's first row
    qrow_of.resize(n_lips);
    int64_t tok = 0;
    for (int32_t b = 0; b < n_lips; tok += n_tokens[b], ++b) {
      qrow_of[b] = (int32_t)tok;
      if (n_tokens[b] == 1 && (len_after[b] - 1) / P >= prm.share_min_pages) cand.emplace_back(tables[b][0], b);
    }
    std::sort(cand.begin(), cand.end());
    // First pass: groups and their common page counts (the second pass sizes the key chunks).
    // Files that start with the same page are candidates; inside such a run, take the first
    // unassigned file as representative, measure how many leading pages every other one has in
    // common with it (limited to full pages), and keep the k closest files that maximise the
    // pages saved, (k - 1) * common pages.  Files left over get another round among themselves.
    auto& groups = out->groups;                               // (offset into grp_members, count, C) triples
    auto& gm = out->grp_members;
    auto& lcp = out->lcp;                                     // (common pages, index into cand) of the round
    groups.clear();
    gm.clear();
    int64_t base_tiles = 0;
    for (size_t lo = 0; lo < cand.size();) {
      size_t hi = lo + 1;
      while (hi < cand.size() && cand[hi].first == cand[lo].first) ++hi;
      size_t left = hi - lo;                                  // unassigned files of the run
      for (size_t rep = lo; rep < hi && (int32_t)left >= prm.share_min_lips; ++rep) {
        if (cand[rep].first < 0) continue;                    // already assigned
        const int32_t b0 = cand[rep].second;
        const int64_t full0 = (len_after[b0] - 1) / P;        // full pages of the file before the call
        lcp.clear();
        for (size_t i = rep; i < hi; ++i) {
          if (cand[i].first < 0) continue;
          const int32_t b = cand[i].second;
          const int64_t lim = std::min<int64_t>(full0, (len_after[b] - 1) / P);
          const int32_t* t = tables[b];
          const int64_t c = i == rep ? lim : std::mismatch(t, t + lim, tables[b0]).first - t;
          lcp.emplace_back((int32_t)(c & ~(int64_t)1), (int32_t)i);      // whole 32-token blocks
        }
        std::sort(lcp.begin(), lcp.end(), [](const std::pair<int32_t, int32_t>& x, const std::pair<int32_t, int32_t>& y) {
          return x.first != y.first ? x.first > y.first : x.second < y.second;
        });
        int64_t best = 0;
        size_t best_k = 0;
        for (size_t k = (size_t)prm.share_min_lips; k <= lcp.size(); ++k) {
          const int64_t c = lcp[k - 1].first;
          if (c < prm.share_min_pages) break;
          if ((int64_t)(k - 1) * c > best) {
            best = (int64_t)(k - 1) * c;
            best_k = k;
          }
        }
        if (best_k == 0) {                                    // nothing worth sharing with this file
          cand[rep].first = -1;
          --left;
          continue;
        }
        const int32_t C = lcp[best_k - 1].first;
        std::sort(lcp.begin(), lcp.begin() + best_k, [](const std::pair<int32_t, int32_t>& x, const std::pair<int32_t, int32_t>& y) { return x.second < y.second; });
        groups.insert(groups.end(), {(int32_t)gm.size(), (int32_t)best_k, C});
        for (size_t k = 0; k < best_k; ++k) {
          gm.push_back(cand[lcp[k].second].second);
          cand[lcp[k].second].first = -1;
        }
        left -= best_k;
        base_tiles += (int64_t)((best_k + tile_lips - 1) / tile_lips) * H;
      }
      lo = hi;
    }
    if (!groups.empty()) {
      const int64_t target = std::max(1, prm.share_tiles);    // default 512: about two workgroups per CU
      int32_t nc_want = (int32_t)std::max<int64_t>(1, std::min<int64_t>(8, (target + base_tiles - 1) / base_tiles));
      // every member leaves one partial per kv head and key chunk: the same number of chunks for all groups
      // that the partial slots can hold (not the wanted number for the first groups and none for the last)
      int64_t members_total = 0;
      for (size_t gi = 0; gi < groups.size(); gi += 3) members_total += groups[gi + 1];
      nc_want = (int32_t)std::max<int64_t>(1, std::min<int64_t>(nc_want, shared_budget / std::max<int64_t>(1, members_total * H)));
      for (size_t gi = 0; gi < groups.size(); gi += 3) {
        const int32_t lo = groups[gi], K = groups[gi + 1], C = groups[gi + 2];
        // pages per key chunk are even (whole 32-token blocks): rounding up can leave the last chunks empty
        // (66 pages in 8 chunks of 10: the 8th would be [66, 66)), so the count follows from the size
        auto chunks_of = [C](int32_t n) { const int32_t cp = ((C + n - 1) / n + 1) & ~1; return (C + cp - 1) / cp; };
        int32_t nc = chunks_of(std::max(1, std::min(nc_want, C / 8)));
        while (nc > 1 && n_shared_partials + (int64_t)K * H * nc > shared_budget) nc = chunks_of(nc - 1);   // partial slots must fit
        if (n_shared_partials + (int64_t)K * H * nc > shared_budget) continue;            // no room: plain rows
        for (int32_t i = 0; i < K; i += tile_lips) {
          const int32_t k = std::min(tile_lips, K - i);
          const int32_t moff = (int32_t)member_rows.size();
          for (int32_t j = 0; j < k; ++j) {
            const int32_t b = gm[lo + i + j];
            member_rows.push_back(qrow_of[b]);
            share_start[b] = C;
            share_base[b] = (int32_t)n_shared_partials;
            share_k[b] = k;
            share_ml[b] = j;
            share_nc[b] = nc;
          }
          stiles.insert(stiles.end(), {gm[lo + i], moff, k, C, nc, (int32_t)n_shared_partials});
          n_shared_partials += (int64_t)k * H * nc;
          n_shared_tiles += (int64_t)H * nc;
        }
      }
    }
  }
  n_tiles += n_shared_tiles;

  // ---- units of the decode kernel
  int64_t total_units = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    if (is_prefill(b)) continue;
    for (int32_t i = 0; i < n_tokens[b]; i += RT) {
      const int64_t vis_last = len_after[b] - n_tokens[b] + std::min(i + RT, n_tokens[b]);   // what the row's last token sees
      total_units += ((vis_last + P - 1) / P - share_start[b]) * H;
    }
  }
  // bins (whole ranges per workgroup, pieces combined through LDS) for the vector-unit kernel; the global
  // cut for the matrix-core decode kernel, which rows of several tokens need
  const bool bins = prm.bin_waves > 0 && max_nt == 1 && total_units > 0;
  // a bin is a workgroup: eight wavefronts, or four when the launch has tiles of 128 query rows (four-wavefront workgroups)
  const int32_t W = !bins ? 0 : n_tiles > 0 ? (TQ * G != 256 ? 4 : 8) : (prm.bin_waves == 4 ? 4 : 8);
  const int64_t max_bins = std::max<int64_t>(1, prm.max_waves / std::max(W, 1));
  int64_t nw = (total_units + prm.min_units_per_wave - 1) / prm.min_units_per_wave;
  nw = std::max<int64_t>(1, std::min<int64_t>(nw, prm.max_waves));
  if (total_units == 0) nw = 0;
  int64_t n_bins = 0;
  if (bins) {
    n_bins = (total_units + (int64_t)prm.min_units_per_wave * W - 1) / ((int64_t)prm.min_units_per_wave * W);
    n_bins = std::max<int64_t>(1, std::min<int64_t>(n_bins, max_bins));
    nw = n_bins * W;
  }
  const int64_t n_members = (int64_t)member_rows.size();

  // A member of a shared-prefix group reads only the pages after the common ones; those are read by
  // the group's tiles through the table of each tile's first member.  So the common pages of every
  // other member stay out of the descriptor (256 forks of 128-page prefixes: 128 KB that would
  // cross PCIe for nothing); its table offset is moved back by the pages left out, so that page
  // index i >= its first own page still finds entry i.
  std::vector<uint8_t>& full_table = out->full_table;
  full_table.assign((size_t)n_lips, 1);
  for (int32_t b = 0; b < n_lips; ++b)
    if (share_start[b] > 0) full_table[b] = 0;
  for (size_t s = 0; s < stiles.size(); s += 6) full_table[stiles[s]] = 1;
  for (int32_t b = 0; b < n_lips; ++b)
    if (!full_table[b]) entries -= share_start[b];

  // ---- rows, planned before the allocation (the bins are made of them)
  std::vector<int32_t>& rows_tmp = out->rows_tmp;
  rows_tmp.resize((size_t)n_rows * ROW_WORDS);
  out->fused.assign((size_t)n_lips, 0);
  int32_t n_fused = 0;
  {
    int64_t r = 0, e = 0, tok = 0;
    for (int32_t b = 0; b < n_lips; ++b) {
      const int64_t skip = full_table[b] ? 0 : share_start[b];
      const int64_t e_lip = e - skip;
      e += (len_after[b] + P - 1) / P - skip;
      if (!is_prefill(b)) {
        for (int32_t i = 0; i < n_tokens[b]; i += RT, ++r) {
          const int32_t nt = std::min(RT, n_tokens[b] - i);
          rows_tmp[r * ROW_WORDS + 0] = (int32_t)e_lip;                                    // page-table offset
          rows_tmp[r * ROW_WORDS + 1] = (int32_t)(len_after[b] - n_tokens[b] + i + 1);   // tokens the row's first token sees
          rows_tmp[r * ROW_WORDS + 2] = (int32_t)(tok + i);                               // q / out row of its first token
          rows_tmp[r * ROW_WORDS + 3] = share_start[b] | ((nt - 1) << ROW_NT_SHIFT);      // first page of the row's own range; tokens - 1
        }
        // the attention kernel can append a LIP's token itself when it is the LIP's only one (nobody else reads it in this launch)
        if (bins && prm.fuse_append && n_tokens[b] == 1) {
          out->fused[b] = 1;
          ++n_fused;
        }
      }
      tok += n_tokens[b];
    }
  }
  out->row_lip.clear();
  if (bins && n_fused > 0) {
    out->row_lip.reserve((size_t)n_rows);
    for (int32_t b = 0; b < n_lips; ++b)
      if (!is_prefill(b))
        for (int32_t i = 0; i < n_tokens[b]; i += RT) out->row_lip.push_back(b);
  }
  auto trow_nt = [&](int64_t rr) { return (rows_tmp[rr * ROW_WORDS + 3] >> ROW_NT_SHIFT) + 1; };
  auto trow_pages = [&](int64_t rr) { return (rows_tmp[rr * ROW_WORDS + 1] + trow_nt(rr) - 1 + P - 1) / P; };   // pages its last token sees
  auto trow_first = [&](int64_t rr) { return rows_tmp[rr * ROW_WORDS + 3] & ROW_PAGE_MASK; };

  // ---- bins: segments (whole ranges, or pieces of ranges too long for a bin), handed to the bins longest first
  std::vector<int32_t>& seg_tmp = out->seg_tmp;          // SEG_WORDS per segment, in (row, head, page) order
  std::vector<int32_t>& item_bin = out->item_bin;        // bin of every segment
  int64_t n_segs = 0, n_split_partials = 0, n_split_merge = 0;
  const int64_t alpha = prm.range_cost;
  if (bins) {
    const int64_t total_cost = total_units + alpha * n_rows * H;
    auto& order = out->item_order;
    auto& heap = out->bin_heap;
    auto emit = [&](int64_t row, int32_t g, int32_t pb, int32_t pe, int32_t np, int32_t dest, int32_t bin) {
      const int32_t rec[SEG_WORDS] = {rows_tmp[row * ROW_WORDS + 0], g, pb, pe, rows_tmp[row * ROW_WORDS + 1], rows_tmp[row * ROW_WORDS + 2] * prm.n_q_heads + g * G, dest,
                                      (pe == np && !out->row_lip.empty() && out->fused[out->row_lip[row]]) ? (rows_tmp[row * ROW_WORDS + 1] - 1) % P : -1};
      seg_tmp.insert(seg_tmp.end(), rec, rec + SEG_WORDS);
      item_bin.push_back(bin);
    };
    // Plan A, when there are several ranges per bin (short files, the members of forked prefixes): whole ranges, handed to
    // the bins longest first; nothing is split, so no range leaves partials in device memory because of the bins.
    bool planned = false;
    if (n_rows * H >= 3 * n_bins) {
      seg_tmp.clear();
      item_bin.clear();
      n_split_partials = n_split_merge = 0;
      for (int64_t row = 0; row < n_rows; ++row) {
        const int32_t np = trow_pages(row), p0 = trow_first(row);
        for (int32_t g = 0; g < H; ++g) {
          emit(row, g, p0, np, np, p0 > 0 ? (int32_t)n_split_partials : -1, 0);        // the members of a shared prefix always leave partials
          if (p0 > 0) {
            ++n_split_partials;
            ++n_split_merge;
          }
        }
      }
      n_segs = (int64_t)seg_tmp.size() / SEG_WORDS;
      // longest first by counting sort on the page count (rows come in, the H ranges of a row are equal)
      int32_t longest = 0;
      for (int64_t row = 0; row < n_rows; ++row) longest = std::max(longest, trow_pages(row) - trow_first(row));
      order.assign((size_t)longest + 2, 0);                    // order[c] = rows with more than c pages, after the prefix sum
      for (int64_t row = 0; row < n_rows; ++row) ++order[longest - (trow_pages(row) - trow_first(row)) + 1];
      for (int32_t c = 0; c <= longest; ++c) order[c + 1] += order[c];
      auto& sorted = out->tile_tmp;                            // rows, longest first (scratch that the tile list reuses later)
      sorted.resize((size_t)n_rows);
      for (int64_t row = 0; row < n_rows; ++row) sorted[order[longest - (trow_pages(row) - trow_first(row))]++] = (int32_t)row;
      heap.clear();
      for (int64_t b = 0; b < n_bins; ++b) heap.emplace_back(0, (int32_t)b);
      auto worse = [](const std::pair<int64_t, int32_t>& x, const std::pair<int64_t, int32_t>& y) { return x > y; };   // min-heap on (load, bin)
      int64_t worst = 0;
      for (int32_t row : sorted) {
        const int64_t c = trow_pages(row) - trow_first(row) + alpha;
        for (int32_t g = 0; g < H; ++g) {
          std::pop_heap(heap.begin(), heap.end(), worse);
          heap.back().first += c;
          item_bin[(size_t)row * H + g] = heap.back().second;
          worst = std::max(worst, heap.back().first);
          std::push_heap(heap.begin(), heap.end(), worse);
        }
      }
      planned = worst * n_bins * 100 <= total_cost * (100 + prm.bin_tolerance);
    }
    // Plan B: the units in (row, head, page) order are cut into n_bins * W contiguous ranges of equal cost, one per wavefront,
    // exactly like the global cut (on a virtual axis where every range occupies range_cost + pages, wavefront k starts at
    // total * k / (n_bins * W); a start inside the overhead part of a range snaps to its first page), and every W consecutive
    // wavefronts are a bin.  A range that a BIN boundary divides becomes one segment per part, each leaving a partial in
    // device memory (at most n_bins - 1 ranges); what the wavefront boundaries inside a bin divide is combined through LDS.
    out->wave_pos.clear();
    if (!planned && n_bins > 1) {
      seg_tmp.clear();
      item_bin.clear();
      n_split_partials = n_split_merge = 0;
      auto& wpos = out->wave_pos;                        // (segment, page) where every wavefront starts
      wpos.reserve((size_t)nw * 2);
      int64_t k = 0, vstart = 0;
      int32_t bin = 0;
      for (int64_t row = 0; row < n_rows; ++row) {
        const int32_t np = trow_pages(row), p0 = trow_first(row);
        for (int32_t g = 0; g < H; ++g) {
          const int64_t vend = vstart + alpha + (np - p0);
          const size_t first_seg = seg_tmp.size() / SEG_WORDS;
          int32_t pb = p0;
          for (; k < nw && total_cost * k / nw < vend; ++k) {
            const int32_t at = p0 + (int32_t)std::max<int64_t>(0, total_cost * k / nw - vstart - alpha);
            if (k % W == 0) {                            // a bin begins here
              if (at > pb) {
                emit(row, g, pb, at, np, 0, bin);
                pb = at;
              }
              bin = (int32_t)(k / W);
            }
            wpos.push_back((int32_t)(seg_tmp.size() / SEG_WORDS));      // the segment that is emitted next holds page `at`
            wpos.push_back(at);
          }
          emit(row, g, pb, np, np, 0, bin);
          const size_t n_here = seg_tmp.size() / SEG_WORDS - first_seg;
          const bool partial = n_here > 1 || p0 > 0;
          for (size_t i = 0; i < n_here; ++i) seg_tmp[(first_seg + i) * SEG_WORDS + S_DEST] = partial ? (int32_t)(n_split_partials + i) : -1;
          if (partial) {
            n_split_partials += (int64_t)n_here;
            ++n_split_merge;
          }
          vstart = vend;
        }
      }
      n_segs = (int64_t)seg_tmp.size() / SEG_WORDS;
      planned = true;
    }
    // One bin (a small batch): every range is a segment of it, cut between its wavefronts only.
    if (!planned) {
      seg_tmp.clear();
      item_bin.clear();
      n_split_partials = n_split_merge = 0;
      for (int64_t row = 0; row < n_rows; ++row) {
        const int32_t np = trow_pages(row), p0 = trow_first(row);
        for (int32_t g = 0; g < H; ++g) {
          emit(row, g, p0, np, np, p0 > 0 ? (int32_t)n_split_partials : -1, 0);
          if (p0 > 0) {
            ++n_split_partials;
            ++n_split_merge;
          }
        }
      }
      n_segs = (int64_t)seg_tmp.size() / SEG_WORDS;
    }
  }

  const int64_t off_rows = DESC_HEADER_WORDS;
  const int64_t off_waves = off_rows + n_rows * ROW_WORDS;
  const int64_t off_merge = off_waves + nw * WAVE_WORDS;
  // a merge entry per token of a cut (row, head) (at most one cut per wave boundary) and per (member row, head)
  // (a cut (row, head) has a wave boundary inside it, and there are no more of them than (row, head)s);
  // with bins: one per (row, head) that is split between bins or belongs to a shared prefix
  const int64_t merge_cap = bins ? n_split_merge : std::min<int64_t>(nw, n_rows * H) * max_nt + n_members * H;
  const int64_t off_pt = off_merge + merge_cap * MERGE_WORDS;
  const int64_t off_ptoff = off_pt + entries;
  const int64_t off_tiles = off_ptoff + n_lips + 1;
  const int64_t off_members = off_tiles + n_tiles * TILE_WORDS;
  const int64_t off_segs = off_members + n_members;
  const int64_t off_lmerge = off_segs + (bins ? (n_segs + 2) * SEG_WORDS : 0);       // two spare records: the kernel looks ahead
  // the order table of a launch with tiles and bins: a word per group of 8 workgroups (no more tile groups than tiles)
  const int64_t off_groups = off_lmerge + (bins ? n_bins * LMERGE_WORDS : 0);
  const int64_t groups_cap = (bins && n_tiles > 0) ? n_tiles + (n_bins + 7) / 8 : 0;
  const int64_t total = off_groups + groups_cap;
  if (total > 0x7fffffff) return SYM_EINVAL;
  int32_t* const w = out->alloc ? out->alloc(total) : nullptr;   // the caller's buffer (pinned staging memory on the GPU path)
  if (!w) return SYM_ENOSPC;
  out->words = w;
  out->n_words = total;
  std::memset(w, 0, DESC_HEADER_WORDS * sizeof(int32_t));

  // ---- rows, prefill tiles, page table
  int32_t* rows = w + off_rows;
  int32_t* pt = w + off_pt;
  int32_t* ptoff = w + off_ptoff;
  int32_t* tiles = w + off_tiles;
  int64_t e = 0, tok = 0, ti = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    const int64_t skip = full_table[b] ? 0 : share_start[b];      // leading pages left out (see above)
    const int64_t e_lip = e - skip;
    ptoff[b] = (int32_t)e_lip;
    int64_t np = (len_after[b] + P - 1) / P;
    if (np > skip) std::memcpy(pt + e, tables[b] + skip, (size_t)(np - skip) * sizeof(int32_t));
    e += np - skip;
    if (is_prefill(b)) {
      // order (kv head, token tile): the tiles that read the same K/V are neighbours
      for (int32_t g = 0; g < H; ++g)
        for (int32_t t0 = 0; t0 < n_tokens[b]; t0 += TQ, ++ti) {
          int32_t* t = tiles + ti * TILE_WORDS;
          std::memset(t, 0, TILE_WORDS * sizeof(int32_t));
          t[T_TBL] = (int32_t)e_lip;                                // page-table offset
          t[T_LEN] = (int32_t)(len_after[b] - n_tokens[b]);         // file length before the call
          t[T_QROW] = (int32_t)(tok + t0);                          // q / out row of the tile's first token
          t[T_COUNT] = std::min<int32_t>(TQ, n_tokens[b] - t0);     // tokens in the tile
          t[T_HEAD] = g;
          t[T_AUX] = t0;                                            // token offset inside the chunk
          t[T_KIND] = TILE_PREFILL;
        }
    }
    tok += n_tokens[b];
  }
  ptoff[n_lips] = (int32_t)e;
  if (n_rows > 0) std::memcpy(rows, rows_tmp.data(), (size_t)n_rows * ROW_WORDS * sizeof(int32_t));

  // ---- cut the unit sequence into nw ranges of equal cost; number the partial results.
  // Cost of a range = its units + range_cost per (row, head) it starts in (the end-of-range
  // combine and the restart of the pipeline are not free).  On a virtual axis where every
  // (row, head) occupies range_cost + pages, wave k ends at total * (k+1) / nw; a cut that
  // falls into the overhead part of a (row, head) snaps to its first page.
  int32_t* waves = w + off_waves;
  int32_t* merge = w + off_merge;
  auto row_nt = [&](int64_t rr) { return (rows[rr * ROW_WORDS + 3] >> ROW_NT_SHIFT) + 1; };
  auto row_pages = [&](int64_t rr) { return (rows[rr * ROW_WORDS + 1] + row_nt(rr) - 1 + P - 1) / P; };   // pages its last token sees
  auto row_first = [&](int64_t rr) { return rows[rr * ROW_WORDS + 3] & ROW_PAGE_MASK; };
  int32_t part = 0;
  int32_t n_merge = 0;        // (row, head) ranges that need a merge
  if (bins) {
    // ---- bins: segment list bin by bin, wave records, in-bin merge lists, merge entries of split ranges
    int32_t* segs = w + off_segs;
    int32_t* lmerge = w + off_lmerge;
    std::memset(lmerge, 0, (size_t)n_bins * LMERGE_WORDS * sizeof(int32_t));
    auto& first = out->bin_first;                         // first segment of every bin in the final order
    first.assign((size_t)n_bins + 1, 0);
    for (int64_t i = 0; i < n_segs; ++i) ++first[item_bin[i] + 1];
    for (int64_t b = 0; b < n_bins; ++b) first[b + 1] += first[b];
    auto& pos = out->item_order;                          // reused: next free place of every bin
    pos.assign(first.begin(), first.end() - 1);
    for (int64_t i = 0; i < n_segs; ++i)                  // (row, head, page) order is kept inside a bin
      std::memcpy(segs + (int64_t)pos[item_bin[i]]++ * SEG_WORDS, seg_tmp.data() + i * SEG_WORDS, SEG_WORDS * sizeof(int32_t));
    std::memset(segs + n_segs * SEG_WORDS, 0, 2 * SEG_WORDS * sizeof(int32_t));
    // merge entries of the ranges that leave partials, in (row, head) order = the order of their partial numbers
    for (int64_t i = 0; i < n_segs; ++i) {
      const int32_t* sg = seg_tmp.data() + i * SEG_WORDS;
      if (sg[S_DEST] < 0) continue;
      const bool first_piece = i == 0 || sg[-SEG_WORDS + S_DEST] < 0 || sg[-SEG_WORDS + S_QROW] != sg[S_QROW];
      if (first_piece) {
        int32_t* it = merge + (int64_t)n_merge++ * MERGE_WORDS;
        std::memset(it, 0, MERGE_WORDS * sizeof(int32_t));
        it[0] = sg[S_DEST];
        it[2] = sg[S_QROW];
        it[6] = 1;
      }
      ++merge[(int64_t)(n_merge - 1) * MERGE_WORDS + 1];
    }
    part = (int32_t)n_split_partials;
    // Inside a bin the wavefronts cut the bin's segments like the global cut does the batch: on a virtual axis where every
    // segment occupies range_cost + pages, wavefront k of the Wb that get work starts at total * k / Wb (snapped to the
    // segment's first page inside the overhead part).  Wb <= pages of the bin, so no two cuts fall on one page and the
    // pieces of a cut segment lie in consecutive wavefronts.  A piece that is not its whole segment goes to an LDS slot:
    // 2 * wavefront for a wavefront's first piece, 2 * wavefront + 1 for its last; the list of cut segments (segment,
    // slot of the first piece, its wavefront, pieces) tells the workgroup what to combine when all are done.
    for (int64_t b = 0; b < n_bins; ++b) {
      const int64_t s0 = first[b], s1 = first[b + 1];
      int64_t pages = 0;
      for (int64_t i = s0; i < s1; ++i) pages += segs[i * SEG_WORDS + S_PE] - segs[i * SEG_WORDS + S_PB];
      const int64_t vt = pages + alpha * (s1 - s0);
      const int64_t Wb = out->wave_pos.empty() ? std::min<int64_t>(W, pages) : W;
      int32_t* bw = waves + b * W * WAVE_WORDS;
      std::memset(bw, 0, (size_t)W * WAVE_WORDS * sizeof(int32_t));
      int32_t* lm = lmerge + b * LMERGE_WORDS;
      lm[1] = (int32_t)s0;                              // the bin's segments (the kernel walks them for the appends that ride along)
      lm[2] = (int32_t)s1;
      int64_t k = 0, vstart = 0;
      if (!out->wave_pos.empty()) {                     // the wavefronts' starts come from the cut of the whole batch
        for (; k < W; ++k) {
          bw[k * WAVE_WORDS + 0] = out->wave_pos[(size_t)(b * W + k) * 2];
          bw[k * WAVE_WORDS + 1] = out->wave_pos[(size_t)(b * W + k) * 2 + 1];
        }
      }
      for (int64_t i = s0; i < s1 && k < Wb; ++i) {
        const int32_t pb = segs[i * SEG_WORDS + S_PB], pe = segs[i * SEG_WORDS + S_PE];
        const int64_t vend = vstart + alpha + (pe - pb);
        while (k < Wb && vt * k / Wb < vend) {
          const int64_t o = vt * k / Wb - vstart;
          int32_t* ww = bw + k * WAVE_WORDS;
          ww[0] = (int32_t)i;
          ww[1] = pb + (int32_t)std::max<int64_t>(0, o - alpha);
          ++k;
        }
        vstart = vend;
      }
      for (int64_t kk = 0; kk < Wb; ++kk) {
        int32_t* ww = bw + kk * WAVE_WORDS;
        int64_t i = ww[0];
        int32_t p = ww[1];
        const int64_t ei = kk + 1 < Wb ? ww[WAVE_WORDS + 0] : s1;
        const int32_t ep = kk + 1 < Wb ? ww[WAVE_WORDS + 1] : 0;
        {                                   // ids of the first pages: their loads need no table lookup
          const int32_t* sg = segs + i * SEG_WORDS;
          for (int t = 0; t < 3; ++t) ww[4 + t] = pt[sg[S_TBL] + std::min(p + t, sg[S_PE] - 1)];
        }
        int64_t units = 0;
        int32_t piece = 0;
        while (i < s1) {
          const int32_t* sg = segs + i * SEG_WORDS;
          const int32_t end = (i == ei) ? ep : sg[S_PE];      // the next wavefront may start inside this segment
          if (end > p) {
            if (!(p == sg[S_PB] && end == sg[S_PE])) {        // a piece of a cut segment
              if (p == sg[S_PB]) {                             // its first piece: a new entry
                int32_t* en = lm + 4 + 4 * lm[0]++;
                en[0] = (int32_t)i;
                en[1] = (int32_t)(piece == 0 ? 2 * kk : 2 * kk + 1);
                en[2] = (int32_t)kk;
                en[3] = 0;
              }
              ++lm[4 + 4 * (lm[0] - 1) + 3];
            }
            units += end - p;
            ++piece;
          }
          if (i == ei) break;
          ++i;
          p = i < s1 ? segs[i * SEG_WORDS + S_PB] : 0;
        }
        ww[2] = (int32_t)units;
      }
    }
  } else {
    const int64_t vtotal = total_units + alpha * n_rows * H;
    {
      int64_t k = 0, vstart = 0;     // next boundary to place; virtual start of the current (row, head)
      for (int64_t row = 0; row < n_rows && k < nw; ++row) {
        const int32_t np = row_pages(row), p0 = row_first(row);
        for (int32_t g = 0; g < H && k < nw; ++g) {
          const int64_t vend = vstart + alpha + (np - p0);
          while (k < nw && vtotal * k / nw < vend) {
            const int64_t o = vtotal * k / nw - vstart;
            int32_t* ww = waves + k * WAVE_WORDS;
            ww[0] = (int32_t)row;
            ww[1] = g;
            ww[2] = p0 + (int32_t)std::max<int64_t>(0, o - alpha);
            ++k;
          }
          vstart = vend;
        }
      }
    }
    for (int64_t k = 0; k < nw; ++k) {
      int32_t* ww = waves + k * WAVE_WORDS;
      int64_t row = ww[0];
      int32_t g = ww[1], p = ww[2];
      // the range ends where the next one starts (or at the end of the batch)
      const int64_t erow = k + 1 < nw ? ww[WAVE_WORDS + 0] : n_rows;
      const int32_t eg = k + 1 < nw ? ww[WAVE_WORDS + 1] : 0, ep = k + 1 < nw ? ww[WAVE_WORDS + 2] : 0;
      ww[4] = part;
      {                                   // ids of the first pages: their loads need no table lookup
        const int32_t np0 = row_pages(row);
        const int32_t* t0 = pt + rows[row * ROW_WORDS + 0];
        for (int i = 0; i < 3; ++i) ww[5 + i] = t0[std::min(p + i, np0 - 1)];
      }
      int64_t units = 0;
      while (row < erow || (row == erow && (g < eg || (g == eg && p < ep)))) {
        const int32_t np = row_pages(row), p0 = row_first(row);
        const int32_t cnt = (row == erow && g == eg) ? ep - p : np - p;
        if (!(p == 0 && cnt == np)) {                            // a whole (row, g) needs no partial
          const int32_t nt = row_nt(row);                        // a piece leaves one partial per token of the row
          if (p == p0) {                                         // first piece of this (row, g)
            for (int32_t t = 0; t < nt; ++t, ++n_merge) {
              int32_t* it = merge + (int64_t)n_merge * MERGE_WORDS;
              std::memset(it, 0, MERGE_WORDS * sizeof(int32_t));
              it[0] = part + t;
              it[2] = (rows[row * ROW_WORDS + 2] + t) * prm.n_q_heads + g * G;
              it[6] = nt;                                        // distance between the token's pieces
            }
          }
          for (int32_t t = 0; t < nt; ++t) ++merge[(int64_t)(n_merge - 1 - t) * MERGE_WORDS + 1];
          part += nt;
        }
        units += cnt;
        p += cnt;
        if (p == np) {
          if (++g == H) {
            g = 0;
            ++row;
          }
          p = row < n_rows ? row_first(row) : 0;
        }
      }
      ww[3] = (int32_t)units;
    }

  }

  // ---- shared-prefix tiles and the extra partials of their members' merge entries
  const int32_t shared_base = part;
  int32_t max_shared_rows = 0;
  if (!stiles.empty()) {
    int32_t* members = w + off_members;
    std::memcpy(members, member_rows.data(), member_rows.size() * sizeof(int32_t));
    for (size_t s = 0; s < stiles.size(); s += 6) {
      const int32_t b0 = stiles[s], moff = stiles[s + 1], k = stiles[s + 2], C = stiles[s + 3], nc = stiles[s + 4], base = stiles[s + 5];
      const int32_t cp = ((C + nc - 1) / nc + 1) & ~1;        // pages per key chunk, even
      for (int32_t g = 0; g < H; ++g)
        for (int32_t c = 0; c < nc; ++c, ++ti) {
          int32_t* t = tiles + ti * TILE_WORDS;
          std::memset(t, 0, TILE_WORDS * sizeof(int32_t));
          t[T_TBL] = ptoff[b0];
          t[T_QROW] = moff;                                    // offset into the member list
          t[T_COUNT] = k;
          max_shared_rows = std::max(max_shared_rows, k * G);
          t[T_HEAD] = g;
          t[T_AUX] = shared_base + base + (g * nc + c) * k;    // first partial of this tile
          t[T_KIND] = TILE_SHARED;
          t[T_PAGE0] = std::min(c * cp, C);
          t[T_PAGE1] = std::min((c + 1) * cp, C);
        }
    }
  }
  // ---- the tile list in 8 shares of equal cost, one per XCD
  int32_t tile_blocks = 0;
  {
    int32_t* xo = w + H_XCD_OFF;
    for (int x = 0; x <= 8; ++x) xo[x] = 0;
    if (n_tiles > 0) {
      auto cost = [&](const int32_t* t) -> int64_t {
        return t[T_KIND] == TILE_SHARED ? (t[T_PAGE1] - t[T_PAGE0] + 1) / 2 + 1
                                        : ((int64_t)t[T_LEN] + t[T_AUX] + t[T_COUNT] + 31) / 32 + 1;
      };
      // groups = runs of tiles with the same page table and kv head, split so that none exceeds 1/16 of the work
      int64_t total = 0;
      for (int64_t i = 0; i < n_tiles; ++i) total += cost(tiles + i * TILE_WORDS);
      const int64_t cap = std::max<int64_t>(1, total / 16);
      auto& groups = out->tile_groups;                    // (cost, first tile); the next group's first tile ends it
      groups.clear();
      int64_t acc = 0;
      for (int64_t i = 0; i < n_tiles; ++i) {
        const int32_t* t = tiles + i * TILE_WORDS;
        const bool same = i > 0 && t[T_TBL] == t[-TILE_WORDS + T_TBL] && t[T_HEAD] == t[-TILE_WORDS + T_HEAD] && t[T_KIND] == t[-TILE_WORDS + T_KIND];
        if (!same || acc >= cap) {
          groups.emplace_back(0, (int32_t)i);
          acc = 0;
        }
        acc += cost(t);
        groups.back().first += cost(t);
      }
      const size_t ng = groups.size();
      auto& order = out->tile_order;                      // group indices, heaviest first
      order.resize(ng);
      for (size_t i = 0; i < ng; ++i) order[i] = (int32_t)i;
      std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return groups[x].first > groups[y].first; });
      int64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      std::vector<int32_t> share_of(ng);
      int32_t count[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int32_t gi : order) {
        int best = 0;
        for (int x = 1; x < 8; ++x)
          if (load[x] < load[best]) best = x;
        share_of[gi] = best;
        load[best] += groups[gi].first;
        const int32_t gend = (size_t)gi + 1 < ng ? groups[gi + 1].second : (int32_t)n_tiles;
        count[best] += gend - groups[gi].second;
      }
      for (int x = 0; x < 8; ++x) xo[x + 1] = xo[x] + count[x];
      // rewrite the list share by share (groups in heaviest-first order inside a share)
      auto& tmp = out->tile_tmp;
      tmp.assign(tiles, tiles + n_tiles * TILE_WORDS);
      int32_t pos[8];
      for (int x = 0; x < 8; ++x) pos[x] = xo[x];
      for (int32_t gi : order) {
        const int32_t gend = (size_t)gi + 1 < ng ? groups[gi + 1].second : (int32_t)n_tiles;
        const int32_t n = gend - groups[gi].second;
        std::memcpy(tiles + (int64_t)pos[share_of[gi]] * TILE_WORDS, tmp.data() + (int64_t)groups[gi].second * TILE_WORDS,
                    (size_t)n * TILE_WORDS * sizeof(int32_t));
        pos[share_of[gi]] += n;
      }
      for (int x = 0; x < 8; ++x) tile_blocks = std::max(tile_blocks, 8 * count[x]);
    }
    w[H_TILE_BLOCKS] = tile_blocks;
  }
  if (groups_cap > 0) {
    // Tiles come longest first and decode groups all cost the same.  Default: the decode groups go among the first
    // half of the tile groups, so that some CUs stream K/V from HBM for decode ranges while the others keep the
    // matrix cores busy, and no decode group starts late and becomes the tail of the grid.
    const int64_t T = tile_blocks / 8, D = (n_bins + 7) / 8;
    const int64_t lead = T * std::min(std::max(prm.mix_lead, 0), 100) / 100;
    const int64_t spread = std::min(T - lead, (T * std::min(std::max(prm.mix_spread, 0), 100) + 99) / 100);
    const int64_t gs = spread + D;                       // groups of the mixed stretch
    int32_t* gm = w + off_groups;
    int64_t t = 0, d = 0;
    for (int64_t j = 0; j < T + D; ++j) {
      const int64_t jj = j - lead;
      const bool dec = jj >= 0 && jj < gs && (jj + 1) * D / gs > jj * D / gs;
      gm[j] = dec ? ~(int32_t)d++ : (int32_t)t++;
    }
    w[H_N_GROUPS] = (int32_t)(T + D);
    w[H_OFF_GROUPS] = (int32_t)off_groups;
  }

  // every (member row, head): extra partials first + i * stride, i < count
  if (n_members > 0) {
    // merge entries are sorted by word 2 (q row * Hq + first head), as are the LIPs by q row
    int64_t tk = 0;
    int32_t mi = 0;
    for (int32_t b = 0; b < n_lips; tk += n_tokens[b], ++b) {
      if (share_start[b] == 0) continue;
      for (int32_t g = 0; g < H; ++g) {
        const int32_t key = (int32_t)tk * prm.n_q_heads + g * G;
        while (mi < n_merge && merge[(int64_t)mi * MERGE_WORDS + 2] < key) ++mi;
        int32_t* it = merge + (int64_t)mi * MERGE_WORDS;     // exists: a member row never writes final output itself
        it[3] = shared_base + share_base[b] + g * share_nc[b] * share_k[b] + share_ml[b];
        it[4] = share_k[b];
        it[5] = share_nc[b];
      }
    }
  }
  const int32_t n_partials = shared_base + (int32_t)n_shared_partials;
  if (n_partials > prm.max_partials) return SYM_ENOSPC;

  w[H_N_ROWS] = (int32_t)n_rows;
  w[H_N_WAVES] = (int32_t)nw;
  w[H_N_PARTIALS] = n_partials;
  w[H_N_LIPS] = n_lips;
  w[H_N_TILES] = (int32_t)n_tiles;
  w[H_N_MERGE] = n_merge;
  w[H_OFF_ROWS] = (int32_t)off_rows;
  w[H_OFF_WAVES] = (int32_t)off_waves;
  w[H_OFF_MERGE] = (int32_t)off_merge;
  w[H_OFF_PT] = (int32_t)off_pt;
  w[H_OFF_PTOFF] = (int32_t)off_ptoff;
  w[H_OFF_TILES] = (int32_t)off_tiles;
  w[H_OFF_MEMBERS] = (int32_t)off_members;
  w[H_N_MEMBERS] = (int32_t)n_members;
  w[H_N_SHARED_TILES] = (int32_t)n_shared_tiles;
  w[H_TOTAL_WORDS] = (int32_t)total;
  w[H_TOTAL_UNITS_LO] = (int32_t)(total_units & 0xffffffff);
  w[H_TOTAL_UNITS_HI] = (int32_t)(total_units >> 32);
  w[H_N_SEGS] = (int32_t)(bins ? n_segs : 0);
  w[H_OFF_SEGS] = (int32_t)off_segs;
  w[H_N_BINS] = (int32_t)n_bins;
  w[H_BIN_WAVES] = W;
  w[H_OFF_LMERGE] = (int32_t)off_lmerge;
  out->n_bins = (int32_t)n_bins;
  out->bin_waves = W;
  out->n_segs = (int32_t)(bins ? n_segs : 0);
  out->n_fused = n_fused;
  out->n_rows = (int32_t)n_rows;
  out->n_waves = (int32_t)nw;
  out->n_partials = n_partials;
  out->n_merge = n_merge;
  out->n_lips = n_lips;
  out->n_tiles = (int32_t)n_tiles;
  out->total_units = total_units;
  out->max_row_tokens = max_nt;
  out->tile_blocks = tile_blocks;
  out->tile_rows = TQ * G;
  out->small_shared_only = (n_tiles > 0 && !any_prefill && max_shared_rows > 0 && max_shared_rows <= 64) ? 1 : 0;
  return SYM_OK;
}

}  // namespace symkv
