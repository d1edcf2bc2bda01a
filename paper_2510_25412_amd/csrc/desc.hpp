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
// slab.  Two ways of handing the units to wavefronts:
//  * the global cut (matrix-core decode kernel: 8 query heads per kv head, rows of several draft
//    tokens): the units of all rows, ordered (row, kv head, page), are cut into n_waves contiguous
//    ranges of equal cost, one per wavefront, whatever the raggedness of the files.  A range
//    that covers only part of a (row, kv head) produces a partial result (running max, sum,
//    unnormalised accumulator) in device memory and an entry in the merge list (a kernel of its
//    own combines them); a range covering a whole (row, kv head) writes the final output directly.
//  * bins (the vector-unit decode kernel): every workgroup of bin_waves wavefronts is a bin that
//    receives WHOLE (row, kv head) ranges, as "segments", balanced over the bins longest first; only a
//    range longer than a bin's share (or ranges too few to balance) is split into several segments,
//    each of which leaves a partial result in device memory like above.  Inside a bin the
//    wavefronts cut the bin's segments into equal contiguous parts and combine the pieces of a cut
//    segment through LDS at the end of the workgroup: a plain decode batch needs no merge launch.
//    The segment that holds a row's last page can also carry the append of the row's new token: the
//    wavefront that reads that page takes the token's K/V rows from k_new / v_new and writes them
//    into the pool itself, so no append launch has to precede the attention launch.
#pragma once
#include <cstdint>
#include <functional>
#include <utility>
#include <vector>

namespace symkv {

enum { DESC_HEADER_WORDS = 48, ROW_WORDS = 4, WAVE_WORDS = 8, MERGE_WORDS = 8, TILE_WORDS = 12, SEG_WORDS = 8, LMERGE_WORDS = 32 };
// header word indices
enum {
  H_N_ROWS = 0, H_N_WAVES, H_N_PARTIALS, H_N_LIPS, H_N_TILES,
  H_OFF_ROWS, H_OFF_WAVES, H_OFF_MERGE, H_OFF_PT, H_OFF_PTOFF, H_OFF_TILES, H_TOTAL_WORDS,
  H_TOTAL_UNITS_LO, H_TOTAL_UNITS_HI, H_N_MERGE, H_OFF_MEMBERS, H_N_MEMBERS, H_N_SHARED_TILES,
  H_TILE_BLOCKS = 18,     // workgroups of the tile part of the launch = 8 * (tiles of the fullest share)
  H_XCD_OFF = 20,         // 9 words: share x of the tile list is [H_XCD_OFF + x, H_XCD_OFF + x + 1)
  // bins (0 everywhere when the batch uses the global cut)
  H_N_SEGS = 32, H_OFF_SEGS, H_N_BINS, H_BIN_WAVES, H_OFF_LMERGE,
  // order of the workgroups of a launch that holds tiles and decode bins: one word per group of eight workgroups
  // (one per XCD): g >= 0 = tile group g, g < 0 = decode group ~g
  H_N_GROUPS = 37, H_OFF_GROUPS
};
// segment words: page-table offset, kv head, first page, end page | tokens the row sees, q/out row * Hq + first
// query head of the kv head, destination (-1 = the final output rows; otherwise a partial slot in device memory), slot of the row's last
// page that receives the row's new token (-1 = the token is not appended by the attention kernel)
enum { S_TBL = 0, S_HEAD, S_PB, S_PE, S_VIS, S_QROW, S_DEST, S_APPEND };
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
  int32_t n_bins = 0, bin_waves = 0, n_segs = 0;   // bins in use (0 = the global cut)
  int32_t n_fused = 0;          // new tokens whose append the attention kernel carries out itself
  std::vector<uint8_t> fused;   // per LIP: 1 = its (single) new token is one of them
  // scratch of the builder, kept between calls
  std::vector<std::pair<int32_t, int32_t>> by_first_page, lcp;
  std::vector<int32_t> tile_tmp, tile_order;
  std::vector<uint8_t> full_table;   // per LIP: its whole page table goes into the descriptor (see build_desc)
  std::vector<std::pair<int64_t, int32_t>> tile_groups;
  std::vector<int32_t> share_start, share_base, share_k, share_ml, share_nc, member_rows, shared_tiles, qrow_of, groups, grp_members;
  std::vector<int32_t> rows_tmp, row_lip, seg_tmp, item_order, item_bin, bin_first, wave_pos;
  std::vector<int64_t> bin_load;
  std::vector<std::pair<int64_t, int32_t>> bin_heap;
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
  int32_t bin_waves = 0;      // != 0: bins (the vector-unit decode kernel) unless a row holds several tokens; as many bins as
                              //   max_waves fills with workgroups of 8 wavefronts (4 beside tiles of 128 query rows; a batch
                              //   without tiles: 4 if this is 4, else 8)
  int32_t bin_tolerance = 3;  // percent by which the fullest bin may exceed the mean before ranges are split finer
  int32_t fuse_append = 0;    // 1: single-token LIPs are appended by the attention kernel (bins only)
  // order of a launch with tiles and decode bins, in percent of the tile groups: `mix_lead` tile groups first, then
  // all decode groups spread evenly among the next `mix_spread`, then the other tile groups
  int32_t mix_lead = 0, mix_spread = 50;
  int32_t share_tiles = 512;  // shared prefixes are cut by key chunk (up to 8 chunks) until the batch has about this many tiles
};

// n_tokens[b] new tokens of LIP b; len_after[b] = file length including them; LIP b's page
// ids are tables[b][0 .. ceil(len_after/P)).  Returns 0 or a negative status.
int build_desc(const DescParams& prm, int32_t n_lips, const int32_t* n_tokens, const int64_t* len_after,
               const int32_t* const* tables, BatchDesc* out);

}  // namespace symkv
