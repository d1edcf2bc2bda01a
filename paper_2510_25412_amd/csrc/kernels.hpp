// Argument blocks and launch functions of the HIP kernels (see kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace symkv {

struct DecodeArgs {
  const uint8_t* pool;
  int64_t page_bytes;
  const void* q;            // [rows][Hq][D] storage dtype
  float* out;               // [rows][Hq][D]
  float* part_acc;          // [n_partials][G][D]
  float* part_ml;           // [n_partials][G][2] (max in log2 units, sum)
  const int32_t* rows;      // [n_rows][4]: page-table offset, visible tokens, q/out row, lip
  const int32_t* waves;     // [n_waves][8]: row, kv head, page, units, first partial, ids of the first
                            //   range's first three pages
  const int32_t* pt;        // flattened page tables
  int32_t n_waves, Hq, Hkv;
  float scale_log2e;        // softmax scale * log2(e)
  // bins (the vector-unit decode kernel): `waves` then holds bin_waves records per bin: first segment, first
  // page, units, 0, ids of the first three pages
  const int32_t* segs;      // [n_segs + 2][8]: page-table offset, kv head, first page, end page, visible tokens,
                            //   q/out row * Hq + first query head, destination (-1 output, else partial slot), slot of the appended token or -1
  const int32_t* lmerge;    // [n_bins][32]: count, then (segment, LDS slot of its first piece, that piece's wavefront,
                            //   pieces) per segment the bin's cut divided, from word 4 on
  int32_t n_bins, bin_waves;
  const void* k_new;        // [rows][Hkv][D]: rows of the new tokens, for segments that append (else unused)
  const void* v_new;
};

struct PrefillArgs {
  const uint8_t* pool;
  int64_t page_bytes;
  const void* q;            // [tokens][Hq][128] bf16
  float* out;               // [tokens][Hq][128]
  const int32_t* tiles;     // [n_tiles][12]: page-table offset, length before, first q/out row (or offset
                            //   into members), tokens (or members) in the tile, kv head, token offset in the
                            //   chunk (or first partial slot), kind (0 prefill, 1 shared prefix), first page,
                            //   end page, 0, 0, 0
  const int32_t* pt;        // flattened page tables
  const int32_t* members;   // q rows of the members of shared-prefix tiles
  float* part_acc;          // partial results (shared-prefix tiles)
  float* part_ml;
  const int32_t* xcd_off;   // [9]: workgroup b runs tile xcd_off[b % 8] + b / 8 if that is below xcd_off[b % 8 + 1]
  int32_t tile_blocks;      // workgroups of the tile part of the launch (multiple of 8)
  int32_t tile_first, n_tiles;   // the launch covers tiles [tile_first, tile_first + n_tiles)
  int32_t tile_rows;             // query rows per tile: 128 (four wavefronts per workgroup) or 256 (eight)
  int32_t Hq, Hkv;
  float scale_log2e;
  int32_t small_shared_only;     // every tile is a shared-prefix tile of at most 64 query rows (members x heads per kv head)
  const int32_t* group_map;      // a launch with tiles and decode bins: per group of 8 workgroups, tile group g or ~(decode group)
  int32_t n_groups;
};

struct MergeArgs {
  const float* part_acc;
  const float* part_ml;
  const int32_t* items;     // [n_items][8]: first partial, pieces, q row * Hq + first head, then the extra
                            //   pieces of a shared prefix: first, stride, count; 0, 0
  float* out;
  int32_t n_items;
};

struct PrologueArgs {
  uint8_t* pool;
  int64_t page_bytes;
  const void* k_new;            // device [n_tokens][Hkv][row]
  const void* v_new;
  const int32_t* slots;         // pinned host [n_tokens]: page * P + slot
  const int32_t* cow;           // pinned host [n_cow][3]: src, dst, slots
  const int32_t* host_words;    // pinned host: descriptor words to copy
  int32_t* dev_words;           // device workspace
  int64_t copy_words;
  int32_t n_tokens, Hkv, n_cow;
  int32_t append_blocks, copy_blocks;   // filled by launch_prologue
};

struct GatherArgs {
  const uint8_t* pool;
  int64_t page_bytes;
  const int32_t* slots;         // pinned host or device [n_tokens]
  int32_t n_tokens, Hkv;
};

struct MoveArgs {
  uint8_t* pool;
  int64_t page_bytes;
  const int32_t* moves;         // device [n_tokens][2]: source, destination token slot (page * P + slot)
  int64_t n_tokens;
  int32_t Hkv;
};

struct SwapArgs {
  uint8_t* pool;
  int64_t page_bytes;
  const uint64_t* list;         // pinned host [n_pages][2]: page id, address of the page's host slot
  int32_t n_pages;
  int32_t to_host;              // 1 = pool -> host slots, 0 = host slots -> pool
  int64_t host_offset;          // byte offset inside every host slot (a slot holds the page's bytes of every layer)
};

// Size of the file-scope device array that stands in for the workspace in sym_pred_batch_static, and
// its address on `device` (looked up once per device, with that device current during the lookup).
constexpr int64_t kStaticScratchBytes = 64ll << 20;
hipError_t static_scratch_address(int device, uint8_t** ptr);

// decode_mode: 0 = VALU decode kernel, 1 = decode ranges on the matrix cores (bf16 storage only)
// ev0 / ev1 (both or neither): events attached to the first / last dispatch of the launch (kernel start, kernel end)
hipError_t launch_attn(const DecodeArgs& da, const PrefillArgs& pa, int dtype, int decode_mode, hipStream_t st,
                       hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
hipError_t launch_merge(const MergeArgs& a, int G, int D, hipStream_t st);
hipError_t launch_prologue(PrologueArgs a, hipStream_t st);
hipError_t launch_gather(const GatherArgs& a, void* k_out, void* v_out, hipStream_t st);
hipError_t launch_move(const MoveArgs& a, hipStream_t st);
hipError_t launch_swap(const SwapArgs& a, hipStream_t st);
hipError_t launch_calib_read(const void* src, int64_t bytes, void* out8, hipStream_t st);
hipError_t launch_calib_copy(void* dst, const void* src, int64_t bytes, hipStream_t st);
hipError_t launch_calib_mfma(float* out, int blocks, int iters, hipStream_t st);

}  // namespace symkv
