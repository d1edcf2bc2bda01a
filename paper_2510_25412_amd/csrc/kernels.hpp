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
  const int32_t* rows;      // [n_rows][4]: lip, visible tokens, q/out row, 0
  const int32_t* waves;     // [n_waves][6]: row, kv head, page, units, first partial, 0
  const int32_t* pt;        // flattened page tables
  const int32_t* ptoff;     // [n_lips + 1]
  int32_t n_waves, Hq, Hkv;
  float scale_log2e;        // softmax scale * log2(e)
};

struct MergeArgs {
  const float* part_acc;
  const float* part_ml;
  const int32_t* merge_off; // [n_rows * Hkv + 1]
  const int32_t* rows;
  float* out;
  int32_t Hq, Hkv, D;
};

struct AppendArgs {
  uint8_t* pool;
  int64_t page_bytes;
  const void* k_new;        // [n_tokens][Hkv][row]
  const void* v_new;
  const int32_t* slots;     // [n_tokens]: page * P + slot
  int32_t n_tokens, Hkv;
};

struct CowArgs {
  uint8_t* pool;
  int64_t page_bytes;
  const int32_t* cow;       // [n][3]: src, dst, slots
  int32_t Hkv;
};

hipError_t launch_decode(const DecodeArgs& a, int dtype, hipStream_t st);
hipError_t launch_merge(const MergeArgs& a, int n_rows, hipStream_t st);
hipError_t launch_append(const AppendArgs& a, hipStream_t st);
hipError_t launch_gather(const AppendArgs& a, void* k_out, void* v_out, hipStream_t st);
hipError_t launch_cow(const CowArgs& a, int n_cow, hipStream_t st);
hipError_t launch_calib_read(const void* src, int64_t bytes, void* out8, hipStream_t st);
hipError_t launch_calib_copy(void* dst, const void* src, int64_t bytes, hipStream_t st);

}  // namespace symkv
