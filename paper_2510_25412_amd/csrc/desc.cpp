// Batch-descriptor builder (host, integer work only).  See desc.hpp.
#include "desc.hpp"

#include <algorithm>
#include <cstring>

#include "../../include/symphony_kv.h"

namespace symkv {

int build_desc(const DescParams& prm, int32_t n_lips, const int32_t* n_tokens, const int64_t* len_after,
               const int32_t* const* tables, BatchDesc* out) {
  const int32_t P = prm.page_tokens, H = prm.n_kv_heads;
  // A LIP with at least prefill_min new tokens goes to the tile kernel (tile_tokens new tokens x
  // all query heads of one kv head per tile); every other new token is a row of the decode kernel.
  const int32_t TQ = prm.tile_tokens;
  auto is_prefill = [&](int32_t b) { return TQ > 0 && n_tokens[b] >= prm.prefill_min; };
  int64_t n_rows = 0, entries = 0, n_tiles = 0, n_tok_total = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    if (n_tokens[b] < 1 || len_after[b] < n_tokens[b] || len_after[b] > (int64_t)0x7fffffff) return SYM_EINVAL;
    if (is_prefill(b)) n_tiles += (int64_t)((n_tokens[b] + TQ - 1) / TQ) * H;
    else n_rows += n_tokens[b];
    n_tok_total += n_tokens[b];
    entries += (len_after[b] + P - 1) / P;
  }
  if (n_tok_total > 0x7fffffff / (2 * H) || entries > 0x3fffffff || n_tiles > 0x0fffffff) return SYM_EINVAL;

  // ---- section sizes known up front: rows, page table, offsets
  int64_t total_units = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    if (is_prefill(b)) continue;
    for (int32_t i = 0; i < n_tokens[b]; ++i) {
      int64_t vis = len_after[b] - n_tokens[b] + i + 1;
      total_units += ((vis + P - 1) / P) * H;
    }
  }
  int64_t nw = (total_units + prm.min_units_per_wave - 1) / prm.min_units_per_wave;
  nw = std::max<int64_t>(1, std::min<int64_t>(nw, prm.max_waves));
  if (total_units == 0) nw = 0;

  std::vector<int32_t>& w = out->words;
  const int64_t off_rows = DESC_HEADER_WORDS;
  const int64_t off_waves = off_rows + n_rows * ROW_WORDS;
  const int64_t off_merge = off_waves + nw * WAVE_WORDS;
  const int64_t off_pt = off_merge + nw * MERGE_WORDS;      // at most one cut (row, head) per wave boundary
  const int64_t off_ptoff = off_pt + entries;
  const int64_t off_tiles = off_ptoff + n_lips + 1;
  const int64_t total = off_tiles + n_tiles * TILE_WORDS;
  if (total > 0x7fffffff) return SYM_EINVAL;
  w.resize((size_t)total);
  std::memset(w.data(), 0, DESC_HEADER_WORDS * sizeof(int32_t));

  // ---- rows, tiles, page table
  int32_t* rows = w.data() + off_rows;
  int32_t* pt = w.data() + off_pt;
  int32_t* ptoff = w.data() + off_ptoff;
  int32_t* tiles = w.data() + off_tiles;
  int64_t r = 0, e = 0, tok = 0, ti = 0;
  for (int32_t b = 0; b < n_lips; ++b) {
    ptoff[b] = (int32_t)e;
    const int64_t e_lip = e;
    int64_t np = (len_after[b] + P - 1) / P;
    std::memcpy(pt + e, tables[b], (size_t)np * sizeof(int32_t));
    e += np;
    if (is_prefill(b)) {
      // order (kv head, token tile): the tiles that read the same K/V are neighbours
      for (int32_t g = 0; g < H; ++g)
        for (int32_t t0 = 0; t0 < n_tokens[b]; t0 += TQ, ++ti) {
          int32_t* t = tiles + ti * TILE_WORDS;
          t[0] = (int32_t)e_lip;                                   // page-table offset
          t[1] = (int32_t)(len_after[b] - n_tokens[b]);            // file length before the call
          t[2] = (int32_t)(tok + t0);                              // q / out row of the tile's first token
          t[3] = std::min<int32_t>(TQ, n_tokens[b] - t0);          // tokens in the tile
          t[4] = g;
          t[5] = t0;                                               // token offset inside the chunk
          t[6] = t[7] = 0;
        }
    } else {
      for (int32_t i = 0; i < n_tokens[b]; ++i, ++r) {
        rows[r * ROW_WORDS + 0] = (int32_t)e_lip;                                    // page-table offset
        rows[r * ROW_WORDS + 1] = (int32_t)(len_after[b] - n_tokens[b] + i + 1);   // visible tokens
        rows[r * ROW_WORDS + 2] = (int32_t)(tok + i);                               // q / out row
        rows[r * ROW_WORDS + 3] = b;
      }
    }
    tok += n_tokens[b];
  }
  ptoff[n_lips] = (int32_t)e;

  // ---- cut the unit sequence into nw ranges of equal cost; number the partial results.
  // Cost of a range = its units + range_cost per (row, head) it starts in (the end-of-range
  // combine and the restart of the pipeline are not free).  On a virtual axis where every
  // (row, head) occupies range_cost + pages, wave k ends at total * (k+1) / nw; a cut that
  // falls into the overhead part of a (row, head) snaps to its first page.
  int32_t* waves = w.data() + off_waves;
  int32_t* merge = w.data() + off_merge;
  auto row_pages = [&](int64_t rr) { return (rows[rr * ROW_WORDS + 1] + P - 1) / P; };
  const int64_t alpha = prm.range_cost;
  const int64_t vtotal = total_units + alpha * n_rows * H;
  {
    int64_t k = 0, vstart = 0;     // next boundary to place; virtual start of the current (row, head)
    for (int64_t row = 0; row < n_rows && k < nw; ++row) {
      const int32_t np = row_pages(row);
      for (int32_t g = 0; g < H && k < nw; ++g) {
        const int64_t vend = vstart + alpha + np;
        while (k < nw && vtotal * k / nw < vend) {
          const int64_t o = vtotal * k / nw - vstart;
          int32_t* ww = waves + k * WAVE_WORDS;
          ww[0] = (int32_t)row;
          ww[1] = g;
          ww[2] = (int32_t)std::max<int64_t>(0, o - alpha);
          ++k;
        }
        vstart = vend;
      }
    }
  }
  int32_t part = 0;
  int32_t n_merge = 0;        // (row, head) ranges that were cut and need a merge
  for (int64_t k = 0; k < nw; ++k) {
    int32_t* ww = waves + k * WAVE_WORDS;
    int64_t row = ww[0];
    int32_t g = ww[1], p = ww[2];
    // the range ends where the next one starts (or at the end of the batch)
    const int64_t erow = k + 1 < nw ? ww[WAVE_WORDS + 0] : n_rows;
    const int32_t eg = k + 1 < nw ? ww[WAVE_WORDS + 1] : 0, ep = k + 1 < nw ? ww[WAVE_WORDS + 2] : 0;
    ww[4] = part;
    ww[5] = rows[row * ROW_WORDS + 1];
    ww[6] = rows[row * ROW_WORDS + 2];
    ww[7] = rows[row * ROW_WORDS + 0];
    for (int i = 0; i < 4; ++i) ww[8 + i] = 0;
    {                                   // ids of the first pages: their loads need no table lookup
      const int32_t np0 = row_pages(row);
      const int32_t* t0 = pt + rows[row * ROW_WORDS + 0];
      for (int i = 0; i < 3; ++i) ww[8 + i] = t0[std::min(p + i, np0 - 1)];
    }
    int64_t units = 0;
    while (row < erow || (row == erow && (g < eg || (g == eg && p < ep)))) {
      const int32_t np = row_pages(row);
      const int32_t cnt = (row == erow && g == eg) ? ep - p : np - p;
      if (!(p == 0 && cnt == np)) {                            // a whole (row, g) needs no partial
        if (p == 0) {                                          // first piece of a cut (row, g)
          int32_t* it = merge + (int64_t)n_merge * MERGE_WORDS;
          it[0] = part;
          it[1] = 0;
          it[2] = rows[row * ROW_WORDS + 2] * prm.n_q_heads + g * (prm.n_q_heads / H);
          it[3] = 0;
          ++n_merge;
        }
        ++merge[(int64_t)(n_merge - 1) * MERGE_WORDS + 1];
        ++part;
      }
      units += cnt;
      p += cnt;
      if (p == np) {
        p = 0;
        if (++g == H) {
          g = 0;
          ++row;
        }
      }
    }
    ww[3] = (int32_t)units;
  }

  w[H_N_ROWS] = (int32_t)n_rows;
  w[H_N_WAVES] = (int32_t)nw;
  w[H_N_PARTIALS] = part;
  w[H_N_LIPS] = n_lips;
  w[H_N_TILES] = (int32_t)n_tiles;
  w[H_N_MERGE] = n_merge;
  w[H_OFF_ROWS] = (int32_t)off_rows;
  w[H_OFF_WAVES] = (int32_t)off_waves;
  w[H_OFF_MERGE] = (int32_t)off_merge;
  w[H_OFF_PT] = (int32_t)off_pt;
  w[H_OFF_PTOFF] = (int32_t)off_ptoff;
  w[H_OFF_TILES] = (int32_t)off_tiles;
  w[H_TOTAL_WORDS] = (int32_t)total;
  w[H_TOTAL_UNITS_LO] = (int32_t)(total_units & 0xffffffff);
  w[H_TOTAL_UNITS_HI] = (int32_t)(total_units >> 32);
  out->n_rows = (int32_t)n_rows;
  out->n_waves = (int32_t)nw;
  out->n_partials = part;
  out->n_merge = n_merge;
  out->n_lips = n_lips;
  out->n_tiles = (int32_t)n_tiles;
  out->total_units = total_units;
  return SYM_OK;
}

}  // namespace symkv
