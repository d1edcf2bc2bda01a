// Batch-descriptor builder: turns the pending pred calls of one batch (paper section 4.4:
// the inference scheduler aggregates pred calls into one GPU batch) into the integer work
// description of the attention launch.  Pure host code, no HIP.
//
// Three kinds of work come out of a batch:
//  * prefill tiles: a LIP that brings many new tokens (a prefill chunk) is cut into tiles of
//    tile_tokens new tokens x one kv head for the MFMA tile kernel;
//  * shared-prefix tiles: decode LIPs whose files start with the same pages (forks of one prefix,
//    paper Fig. 1 / section 4.2) are grouped; the common full pages are read ONCE per group by
//    the tile kernel (rows = members x query heads of the group), leaving partial results;
//  * decode rows: every other new token is a "row" with a visible length (file tokens
//    0 .. len_before + i); a member of a sharing group is a row that starts after the common pages.
//    A LIP that brings a few new tokens (a short draft to verify, paper section 4.1) packs up to
//    row_tokens consecutive ones into one row: they share a single pass over the file, each
//    with its own visible length.
// Workgroups are handed to the 8 XCDs of the GPU round-robin, and each XCD has its own L2.  The
// tile list is therefore cut into 8 shares of equal cost (32-token K/V blocks to walk): tiles that
// read the same K/V (same file, same kv head) stay together in one share, longest first; workgroup
// b runs tile b / 8 of share b % 8.
// The work of the decode kernel is measured in units of one (page, kv head) = one 8 KiB K+V
// slab; the units of all rows, ordered (row, kv head, page), are cut into n_waves contiguous
// ranges of equal cost, one per wavefront, whatever the raggedness of the files.  A range
// that covers only part of a (row, kv head) produces a partial result (running max, sum,
// unnormalised accumulator) and an entry in the merge list; a range covering a whole
// (row, kv head) writes the final output directly and has no partial.
#pragma once
#include <cstdint>
#include <functional>
#include <utility>
#include <vector>

namespace symkv {

enum { DESC_HEADER_WORDS = 32, ROW_WORDS = 4, WAVE_WORDS = 8, MERGE_WORDS = 8, TILE_WORDS = 12 };
// header word indices
enum {
  H_N_ROWS = 0, H_N_WAVES, H_N_PARTIALS, H_N_LIPS, H_N_TILES,
  H_OFF_ROWS, H_OFF_WAVES, H_OFF_MERGE, H_OFF_PT, H_OFF_PTOFF, H_OFF_TILES, H_TOTAL_WORDS,
  H_TOTAL_UNITS_LO, H_TOTAL_UNITS_HI, H_N_MERGE, H_OFF_MEMBERS, H_N_MEMBERS, H_N_SHARED_TILES,
  H_TILE_BLOCKS = 18,     // workgroups of the tile part of the launch = 8 * (tiles of the fullest share)
  H_XCD_OFF = 20          // 9 words: share x of the tile list is [H_XCD_OFF + x, H_XCD_OFF + x + 1)
};
// tile words
enum { T_TBL = 0, T_LEN, T_QROW, T_COUNT, T_HEAD, T_AUX, T_KIND, T_PAGE0, T_PAGE1 };
enum { TILE_PREFILL = 0, TILE_SHARED = 1 };
// word 3 of a row (and word 11 of a wave record): first page of the row's own range in the low
// bits, (new tokens in the row) - 1 above them
enum { ROW_NT_SHIFT = 28, ROW_PAGE_MASK = (1 << ROW_NT_SHIFT) - 1, ROW_TOKENS_MAX = 4 };

struct BatchDesc {
  // The packed descriptor (header first) is written straight into memory the caller hands out
  // once the size is known: alloc(n_words) returns room for n_words words, or nullptr.
  std::function<int32_t*(int64_t)> alloc;
  int32_t* words = nullptr;
  int64_t n_words = 0;
  int32_t n_rows = 0, n_waves = 0, n_partials = 0, n_lips = 0, n_merge = 0, n_tiles = 0;
  int32_t tile_blocks = 0;      // workgroups the tile part of the launch needs
  int32_t tile_rows = 0;        // query rows of this batch's tiles (128 or 256)
  int32_t small_shared_only = 0;   // 1: every tile is a shared-prefix tile with at most 64 live rows
  int32_t max_row_tokens = 1;   // > 1: some row holds several new tokens (needs the matrix-core decode kernel)
  int64_t total_units = 0;
  // scratch of the builder, kept between calls
  std::vector<std::pair<int32_t, int32_t>> by_first_page, lcp;
  std::vector<int32_t> tile_tmp, tile_order;
  std::vector<uint8_t> full_table;   // per LIP: its whole page table goes into the descriptor (see build_desc)
  std::vector<std::pair<int64_t, int32_t>> tile_groups;
  std::vector<int32_t> share_start, share_base, share_k, share_ml, share_nc, member_rows, shared_tiles, qrow_of, groups, grp_members;
};

struct DescParams {
  int32_t n_q_heads, n_kv_heads, page_tokens;
  int32_t max_waves;          // wavefront slots of the decode launch
  int32_t min_units_per_wave; // do not cut finer than this (keeps partial traffic small)
  int32_t range_cost;         // cost of starting a (row, head) range, in units, when balancing
  int32_t prefill_min;        // LIPs with at least this many new tokens use the tile kernel
  int32_t tile_tokens;        // new tokens per tile (0 = no tile kernel for this shape)
  int32_t share_min_lips;     // decode LIPs that must share a prefix to form a group (0 = never group)
  int32_t share_min_pages;    // common full pages a group must have
  int32_t max_partials;       // partial-result slots the workspace holds
  int32_t row_tokens;         // new tokens of one LIP a decode row may hold (1 = a row per token)
};

// n_tokens[b] new tokens of LIP b; len_after[b] = file length including them; LIP b's page
// ids are tables[b][0 .. ceil(len_after/P)).  Returns 0 or a negative status.
int build_desc(const DescParams& prm, int32_t n_lips, const int32_t* n_tokens, const int64_t* len_after,
               const int32_t* const* tables, BatchDesc* out);

}  // namespace symkv
