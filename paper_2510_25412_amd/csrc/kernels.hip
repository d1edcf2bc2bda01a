// HIP kernels (gfx950 / CDNA4) of the pred hot path: copy-on-write page copy, KV append,
// page-table-indirected decode attention with per-lane online softmax, split merge, plus
// a file gather used by tests and two calibration kernels of known traffic.
//
// Geometry shared by all kernels (also stated in include/symphony_kv.h): a K or V row of
// one token and one kv head is 256 bytes; a (page, kv head) slab is [K|V][row half 0|1]
// [16 tokens][128 bytes], 8 KiB, so 8 tokens of one row half are 1 KiB contiguous.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdint>
#include <mutex>

#include "kernels.hpp"

namespace symkv {

namespace {

constexpr int kP = 16;              // tokens per page
constexpr int kRowBytes = 256;      // bytes of one K or V row (one token, one kv head)
constexpr int kHalfBytes = 128;     // a row half
constexpr int kBlk = kP * kRowBytes;   // 4096: K (or V) of one (page, head)
constexpr int kSlab = 2 * kBlk;        // 8192: K+V of one (page, head)
constexpr int kWavesPerBlock = 4;
constexpr float kTau = 8.0f;        // the running max may lag the true max by up to 2^kTau

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Sum over the 8 lanes of a lane octet (lanes 8k .. 8k+7): three DPP adds.
__device__ __forceinline__ float octet_sum(float x) {
  x += as_f32(__builtin_amdgcn_update_dpp(0, as_u32(x), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
  x += as_f32(__builtin_amdgcn_update_dpp(0, as_u32(x), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
  x += as_f32(__builtin_amdgcn_update_dpp(0, as_u32(x), 0x141, 0xf, 0xf, false));   // row_half_mirror
  return x;
}

// Value of the lane 8 away inside the 16-lane row (lane ^ 8): DPP row rotate by 8.
__device__ __forceinline__ float row_xor8(float x) {
  return as_f32(__builtin_amdgcn_update_dpp(0, as_u32(x), 0x128, 0xf, 0xf, false));   // row_ror:8
}

// max / sum of x over the lane pairs (l, l ^ 32) and (l, l ^ 16), in every lane, with the lane-swap instructions: swapping
// the upper 32 lanes of x with the lower 32 of a copy leaves one register holding the lower half twice and the other the
// upper half twice (likewise the odd and even rows of 16 lanes), so combining the two needs no select.
__device__ __forceinline__ float pair32_max(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(as_u32(x), as_u32(x), false, false);
  return fmaxf(as_f32(sw[0]), as_f32(sw[1]));
}
__device__ __forceinline__ float pair16_max(float x) {
  const auto sw = __builtin_amdgcn_permlane16_swap(as_u32(x), as_u32(x), false, false);
  return fmaxf(as_f32(sw[0]), as_f32(sw[1]));
}
__device__ __forceinline__ float pair32_sum(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(as_u32(x), as_u32(x), false, false);
  return as_f32(sw[0]) + as_f32(sw[1]);
}
__device__ __forceinline__ float pair16_sum(float x) {
  const auto sw = __builtin_amdgcn_permlane16_swap(as_u32(x), as_u32(x), false, false);
  return as_f32(sw[0]) + as_f32(sw[1]);
}

// Element-type traits.  A lane holds, per row half, one 16-byte chunk of a K/V row.
struct ElemBF16 {
  static constexpr int kDimsPerChunk = 8;
  // dot of one 16-byte chunk of K with the matching chunk of q, accumulated into s
  static __device__ __forceinline__ float dot(const uint4& k, const uint4& q, float s) {
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), s, false);
    return s;
  }
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = as_f32(v.x << 16); f[1] = as_f32(v.x & 0xffff0000u);
    f[2] = as_f32(v.y << 16); f[3] = as_f32(v.y & 0xffff0000u);
    f[4] = as_f32(v.z << 16); f[5] = as_f32(v.z & 0xffff0000u);
    f[6] = as_f32(v.w << 16); f[7] = as_f32(v.w & 0xffff0000u);
  }
};
struct ElemF32 {
  static constexpr int kDimsPerChunk = 4;
  static __device__ __forceinline__ float dot(const uint4& k, const uint4& q, float s) {
    s = __builtin_fmaf(as_f32(k.x), as_f32(q.x), s);
    s = __builtin_fmaf(as_f32(k.y), as_f32(q.y), s);
    s = __builtin_fmaf(as_f32(k.z), as_f32(q.z), s);
    s = __builtin_fmaf(as_f32(k.w), as_f32(q.w), s);
    return s;
  }
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = as_f32(v.x); f[1] = as_f32(v.y); f[2] = as_f32(v.z); f[3] = as_f32(v.w);
  }
};

struct PageRegs {
  uint4 k[4];   // index = row_half * 2 + token_half
  uint4 v[4];
};

// ---------------------------------------------------------------------------------------
// Decode attention.  One wavefront per work range; lane = (r = lane/8: token slot within a
// half page, j = lane%8: which 16-byte chunk of each row half).  Every lane keeps its own
// running max / sum / accumulators over the tokens it sees (2 per page), so the page loop
// has no cross-lane traffic except the 8-lane score reduction; the 8 token slots are
// combined once, when a (row, kv head) range ends; a range that is only part of its (row, kv
// head) leaves a partial result for the merge kernel.
// ---------------------------------------------------------------------------------------
// decode_bins (below) is the form for up to 4 query heads per kv head.  decode_ranges is the form for 8
// heads per kv head on the vector units (whose 8 x 16 accumulators do not fit one wavefront's
// registers twice per SIMD): GT = query heads per kv head, G = GT / 2 = heads per wavefront, a
// workgroup of TWO wavefronts per range; wavefront 0 fetches the K half of every page,
// wavefront 1 the V half, they exchange them through LDS (written and read in the same
// lane-linear 1 KiB runs, so without bank conflicts), and every page is still read from HBM once.
// ---------------------------------------------------------------------------------------
// Decode ranges in bins (the VALU kernel for up to 4 query heads per kv head).  A workgroup of W
// wavefronts is a bin: the host hands it a list of segments (whole (row, kv head) ranges, or pieces of
// ranges too long for one bin) and cuts that list into W contiguous parts of equal cost, one per
// wavefront.  A wavefront walks its part as ONE page stream: a LOAD cursor runs two pages ahead of the
// COMPUTE cursor through the same unit sequence, across segment boundaries (starting every segment
// with its own chain of dependent loads, segment record -> page ids -> K/V, would cost several memory
// latencies per segment, a third of the time at 10 pages per range), so the K/V stream never drains;
// the query rows of the next segment are fetched one segment ahead.  At a boundary the compute side only
// combines its 8 token slots, hands the result on and switches to the next segment's registers.
// Where a result goes: a piece that is its whole segment writes the segment's destination (the final
// output rows, or a partial slot in device memory when the segment is only part of its range or the row has a
// shared prefix); a piece of a segment that the bin's cut divided goes to an LDS slot, and when all
// wavefronts of the bin are done they combine those pieces (merge_bin_pieces) into the destination.
// The append of a row's new token can ride along (segment word S_APPEND): the wavefront that reads
// the row's last page replaces the token's slot in its registers with the rows of k_new / v_new and
// writes them into the pool afterwards; nobody else reads that page in this launch.
// ---------------------------------------------------------------------------------------
template <typename E, int G>
struct BinLds {
  static constexpr int kAcc = G * 16 * E::kDimsPerChunk;      // accumulator floats of a piece: G heads x D dims
  static constexpr int kSlot = kAcc + 2 * G;                   // + (max, sum) per head
};

// After the barrier: wavefront `wib` of the bin combines the pieces of cut segments wib, wib + W, ... of the bin's list.
// Lane owns accumulator entries e * 64 + lane of the G * D values (head = entry / D).
template <typename E, int G>
__device__ __forceinline__ void merge_bin_pieces(const DecodeArgs& a, const int bin, const int W, const int wib, const float* lds) {
  constexpr int D = 16 * E::kDimsPerChunk, VL = G * D / 64, SLOT = BinLds<E, G>::kSlot, ACC = BinLds<E, G>::kAcc;
  const int lane = threadIdx.x & 63;
  const int32_t* lm = a.lmerge + (int64_t)bin * 32;
  const int cnt = __builtin_amdgcn_readfirstlane(lm[0]);
  for (int k = wib; k < cnt; k += W) {
    const int seg = __builtin_amdgcn_readfirstlane(lm[4 + 4 * k + 0]);
    const int s0 = __builtin_amdgcn_readfirstlane(lm[4 + 4 * k + 1]);
    const int w0 = __builtin_amdgcn_readfirstlane(lm[4 + 4 * k + 2]);
    const int n = __builtin_amdgcn_readfirstlane(lm[4 + 4 * k + 3]);
    const int32_t* sr = a.segs + (int64_t)seg * 8;
    const int qh = __builtin_amdgcn_readfirstlane(sr[5]);        // q row * Hq + first query head
    const int dest = __builtin_amdgcn_readfirstlane(sr[6]);
    float M[G], ls[G], o[VL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      M[h] = -__builtin_inff();
      ls[h] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < VL; ++e) o[e] = 0.f;
    for (int i = 0; i < n; ++i) {
      const float* sl = lds + (int64_t)(i == 0 ? s0 : 2 * (w0 + i)) * SLOT;
      float sc[G], wt[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float mi = sl[ACC + 2 * h], li = sl[ACC + 2 * h + 1];
        const float mn = fmaxf(M[h], mi);
        sc[h] = __builtin_amdgcn_exp2f(M[h] - mn);      // 0 for the first piece (M = -inf)
        wt[h] = __builtin_amdgcn_exp2f(mi - mn);
        ls[h] = ls[h] * sc[h] + li * wt[h];
        M[h] = mn;
      }
#pragma unroll
      for (int e = 0; e < VL; ++e) o[e] = o[e] * sc[(e * 64) / D] + sl[e * 64 + lane] * wt[(e * 64) / D];
    }
    if (dest < 0) {
      float* out = a.out + (int64_t)qh * D;
#pragma unroll
      for (int e = 0; e < VL; ++e) out[e * 64 + lane] = o[e] / ls[(e * 64) / D];
    } else {
      float* pa = a.part_acc + (int64_t)dest * G * D;
#pragma unroll
      for (int e = 0; e < VL; ++e) pa[e * 64 + lane] = o[e];
      if (lane < G) {
        float mm = M[0], ll = ls[0];
#pragma unroll
        for (int hh = 1; hh < G; ++hh) {
          mm = (lane == hh) ? M[hh] : mm;
          ll = (lane == hh) ? ls[hh] : ll;
        }
        a.part_ml[((int64_t)dest * G + lane) * 2 + 0] = mm;
        a.part_ml[((int64_t)dest * G + lane) * 2 + 1] = ll;
      }
    }
  }
}

template <typename E, int G>
__device__ __forceinline__ void decode_bins(const DecodeArgs& a, const int bin, const int W, float* lds) {
  constexpr int C = E::kDimsPerChunk;    // dims per 16-byte chunk
  constexpr int DPL = 2 * C;             // dims per lane
  constexpr int D = 16 * C;              // head dim
  constexpr int SLOT = BinLds<E, G>::kSlot, ACC = BinLds<E, G>::kAcc;
  if (bin >= a.n_bins) return;           // the whole workgroup
  const int lane = threadIdx.x & 63;
  const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));      // wavefront within the bin
  const int r = lane >> 3, j = lane & 7;
  auto sload = [&](const int32_t* ptr) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(*ptr); };
  const int32_t* ww = a.waves + ((int64_t)bin * W + wib) * 8;
  int remaining = sload(ww + 2);

  if (remaining > 0) {
  // Segment record: [0] page-table offset, [1] kv head, [2] first page, [3] end page (what the load side needs),
  // [4] tokens the row sees, [5] q row * Hq + first query head, [6] destination, [7] slot of the appended token or -1.
  // compute cursor: the segment being accumulated.  The wave record carries the id of the first page, so the first
  // K/V loads go out while the segment record (one more scalar round trip) is still on its way.
  int seg = sload(ww + 0), p = sload(ww + 1);
  const int pid_first = sload(ww + 4);
  const int32_t* sr = a.segs + (int64_t)seg * 8;
  int pe = sload(sr + 3), vis = sload(sr + 4), qh = sload(sr + 5);
  int dest = sload(sr + 6), app = sload(sr + 7), tbl = sload(sr + 0);
  bool from_start = p == sload(sr + 2);                  // the piece begins where its segment begins
  // load cursor: the unit whose K/V is requested next (two pages ahead of the compute cursor)
  int lseg = seg, lg = sload(sr + 1), lp = p, lpe = pe, ltbl = sload(sr + 0), lrem = remaining;
  // record of the segment after the load cursor's (fetched a whole segment ahead of its use; the list ends with spare records)
  int n_tbl = 0, n_g = 0, n_pb = 0, n_pe = 0;
  auto fetch_next_seg = [&](int ss) __attribute__((always_inline)) {
    const int32_t* q4 = a.segs + (int64_t)ss * 8;
    n_tbl = sload(q4 + 0);
    n_g = sload(q4 + 1);
    n_pb = sload(q4 + 2);
    n_pe = sload(q4 + 3);
  };
  fetch_next_seg(lseg + 1);
  // record of segment seg + 1 as the compute side needs it
  int c_pe = 0, c_vis = 0, c_qh = 0, c_dest = 0, c_app = 0, c_tbl = 0;
  auto fetch_compute_next_seg = [&]() __attribute__((always_inline)) {
    const int32_t* q8 = a.segs + (int64_t)(seg + 1) * 8;
    c_pe = sload(q8 + 3);
    c_vis = sload(q8 + 4);
    c_qh = sload(q8 + 5);
    c_dest = sload(q8 + 6);
    c_app = sload(q8 + 7);
    c_tbl = sload(q8 + 0);
  };

  const uint8_t* pool_lane = a.pool + lane * 16;
  // Requests the K/V of the next unit into R and advances the load cursor; past the last unit: page 0, head 0 (valid
  // memory that every wavefront touches, never used).
  int next_pid = pid_first;
  auto load_next = [&](PageRegs& R) __attribute__((always_inline)) {
    const bool valid = lrem > 0;
    const uint8_t* base = pool_lane + (int64_t)(valid ? lg : 0) * kSlab + (int64_t)(valid ? next_pid : 0) * a.page_bytes;
    if (valid) {
      --lrem;
      if (++lp == lpe) {
        ++lseg;
        ltbl = n_tbl;
        lg = n_g;
        lp = n_pb;
        lpe = n_pe;
        fetch_next_seg(lseg + 1);
      }
      next_pid = lrem > 0 ? sload(a.pt + ltbl + lp) : 0;     // id of the unit after this one, used one page later
    }
    // every load is unconditional and off one base address: no control-flow join between a load and its use, so the
    // waits can be for exactly the older page while the newer one is in flight
#pragma unroll
    for (int x = 0; x < 4; ++x) R.k[x] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)(base + x * 1024)));
#pragma unroll
    for (int x = 0; x < 4; ++x) R.v[x] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)(base + kBlk + x * 1024)));
  };

  // q chunks of this lane for the G heads of the current segment
  u32x4_t q[G][2];
  // The append that rides along: the K and V rows of the row's new token (2 x 256 bytes in k_new / v_new) are requested
  // with the query rows, one 16-byte chunk per lane (lanes 0..15: K, 16..31: V; the upper half of the wavefront repeats
  // them), whenever a segment begins: the load is unconditional like every load of the stream (for a segment that appends
  // nothing the chunk is never used; k_new / v_new then point at the query rows, which are no smaller).
  u32x4_t nr;
  auto load_q = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const uint8_t* qp = (const uint8_t*)a.q + (int64_t)(qh + h) * kRowBytes + j * 16;
      q[h][0] = *(const u32x4_t*)qp;
      q[h][1] = *(const u32x4_t*)(qp + kHalfBytes);
    }
    nr = *(const u32x4_t*)((const uint8_t*)((lane & 16) ? a.v_new : a.k_new) + (int64_t)(qh / G) * kRowBytes + (lane & 15) * 16);
  };
  fetch_compute_next_seg();
  load_q();

  float m[G], l[G], acc[G][DPL];
  auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m[h] = -1e30f;
      l[h] = 0.f;
#pragma unroll
      for (int d = 0; d < DPL; ++d) acc[h][d] = 0.f;
    }
  };
  reset_state();
  int piece = 0;                                         // pieces this wavefront has finished

  // tokens of page index pi (absolute, within the row) that exist: the row's last page may be ragged
  auto compute = [&](PageRegs& R, int pi) __attribute__((always_inline)) {
    const int nvalid = vis - pi * kP;          // >= 1; >= 16 for a full page
    if (nvalid < kP) {
      // ragged last page: slots past the file's end hold whatever was there before (possibly
      // NaN patterns); their weight is 0, but 0 * NaN is NaN, so clear their V chunks
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        if ((hf * 8 + r) >= nvalid) {
          R.v[hf] = make_uint4(0, 0, 0, 0);
          R.v[2 + hf] = make_uint4(0, 0, 0, 0);
        }
    }
    float s[2][G];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const bool valid = (hf * 8 + r) < nvalid;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float x = E::dot(R.k[hf], __builtin_bit_cast(uint4, q[h][0]), 0.f);
        x = E::dot(R.k[2 + hf], __builtin_bit_cast(uint4, q[h][1]), x);
        x = octet_sum(x) * a.scale_log2e;
        s[hf][h] = valid ? x : -__builtin_inff();
      }
    }
    bool need = false;
#pragma unroll
    for (int h = 0; h < G; ++h) need |= fmaxf(s[0][h], s[1][h]) > m[h] + kTau;
    if (__builtin_amdgcn_ballot_w64(need) != 0) {     // rare after the first page
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float mn = fmaxf(m[h], fmaxf(s[0][h], s[1][h]));
        const float al = __builtin_amdgcn_exp2f(m[h] - mn);
        l[h] *= al;
#pragma unroll
        for (int d = 0; d < DPL; ++d) acc[h][d] *= al;
        m[h] = mn;
      }
    }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      float pw[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        pw[h] = __builtin_amdgcn_exp2f(s[hf][h] - m[h]);
        l[h] += pw[h];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float vf[C];
        E::unpack(R.v[i * 2 + hf], vf);
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int e = 0; e < C; ++e) acc[h][i * C + e] = __builtin_fmaf(pw[h], vf[e], acc[h][i * C + e]);
      }
    }
  };

  // End of a piece: combine the 8 token slots (lanes with equal j).  Per head: common max M, rescale, total sum.  The
  // G*DPL accumulators are then reduced with a halving exchange (lane bit 5, 4, 3 in turn: keep one half of the list,
  // send the other), so lane (r, j) ends up owning the fully reduced values r*V/8 .. r*V/8 + V/8 - 1 of the list.
  // Then the compute cursor moves on.
  auto finish_piece = [&]() __attribute__((always_inline)) {
    const bool whole = from_start && p == pe;            // the piece is its whole segment
    const int64_t out_row = (int64_t)qh * D;
    const int f_dest = dest;
    // The segment after this one: its query rows are requested now, so that they arrive while the exchange
    // below runs (q is not needed any more for this piece).
    const bool more = remaining > 0;
    if (more) {
      ++seg;
      pe = c_pe;
      vis = c_vis;
      qh = c_qh;
      dest = c_dest;
      app = c_app;
      tbl = c_tbl;
      fetch_compute_next_seg();
      load_q();
    }
    constexpr int V = G * DPL;
    float vals[V];
    float lsum[G], Mh[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float M = m[h];
      M = fmaxf(M, row_xor8(M));
      M = pair16_max(M);
      M = pair32_max(M);
      const float f = __builtin_amdgcn_exp2f(m[h] - M);
      float ls = l[h] * f;
      ls += row_xor8(ls);
      ls = pair16_sum(ls);
      ls = pair32_sum(ls);
      lsum[h] = ls;
      Mh[h] = M;
#pragma unroll
      for (int d = 0; d < DPL; ++d) vals[h * DPL + d] = acc[h][d] * f;
    }
    {
      // lane bits 5 and 4: the lane-swap instructions do "keep one, send the other" in one go: after swapping the upper
      // 32 lanes of x with the lower 32 of y, x + y is x summed over the lane pairs (l, l + 32) in the lower half and y
      // summed in the upper half; likewise with the odd and even rows of 16 lanes
#pragma unroll
      for (int i = 0; i < V / 2; ++i) {
        const auto sw = __builtin_amdgcn_permlane32_swap(as_u32(vals[i]), as_u32(vals[i + V / 2]), false, false);
        vals[i] = as_f32(sw[0]) + as_f32(sw[1]);
      }
#pragma unroll
      for (int i = 0; i < V / 4; ++i) {
        const auto sw = __builtin_amdgcn_permlane16_swap(as_u32(vals[i]), as_u32(vals[i + V / 4]), false, false);
        vals[i] = as_f32(sw[0]) + as_f32(sw[1]);
      }
      const bool b3 = (lane & 8) != 0;
#pragma unroll
      for (int i = 0; i < V / 8; ++i) {
        const float keep = b3 ? vals[i + V / 8] : vals[i], send = b3 ? vals[i] : vals[i + V / 8];
        vals[i] = keep + row_xor8(send);
      }
    }
    // lane (r, j) now holds list entries idx = r * V/8 + t: head idx / DPL, lane-local dim idx % DPL
    if (whole && f_dest < 0) {
#pragma unroll
      for (int t = 0; t < V / 8; ++t) {
        const int idx = r * (V / 8) + t, h = idx / DPL, dl = idx % DPL;
        float ls = lsum[0];
#pragma unroll
        for (int hh = 1; hh < G; ++hh) ls = (h == hh) ? lsum[hh] : ls;
        a.out[out_row + h * D + (dl / C) * (D / 2) + j * C + (dl % C)] = vals[t] / ls;
      }
    } else {
      // unnormalised accumulator, max and sum: to the segment's partial slot in device memory, or to this wavefront's LDS
      // slot (two separate stretches of code: one pointer that may be either would make every store a flat store, and
      // with flat stores outstanding the waits for the K/V loads could no longer count)
      float mm = Mh[0], ll = lsum[0];
#pragma unroll
      for (int hh = 1; hh < G; ++hh) {
        mm = (lane == hh) ? Mh[hh] : mm;
        ll = (lane == hh) ? lsum[hh] : ll;
      }
      if (whole) {
        float* pa = a.part_acc + (int64_t)f_dest * G * D;
#pragma unroll
        for (int t = 0; t < V / 8; ++t) {
          const int idx = r * (V / 8) + t, h = idx / DPL, dl = idx % DPL;
          pa[h * D + (dl / C) * (D / 2) + j * C + (dl % C)] = vals[t];
        }
        if (lane < G) {
          a.part_ml[((int64_t)f_dest * G + lane) * 2 + 0] = mm;
          a.part_ml[((int64_t)f_dest * G + lane) * 2 + 1] = ll;
        }
      } else {
        float* pl = lds + (piece == 0 ? 2 * wib : 2 * wib + 1) * SLOT;
#pragma unroll
        for (int t = 0; t < V / 8; ++t) {
          const int idx = r * (V / 8) + t, h = idx / DPL, dl = idx % DPL;
          pl[h * D + (dl / C) * (D / 2) + j * C + (dl % C)] = vals[t];
        }
        if (lane < G) {
          pl[ACC + lane * 2 + 0] = mm;
          pl[ACC + lane * 2 + 1] = ll;
        }
      }
    }
    ++piece;
    if (more) {                                          // the next segment (the piece ended with its own)
      p = sload(a.segs + (int64_t)seg * 8 + 2);
      from_start = true;
      reset_state();
    }
  };
  // one unit: accumulate the page, move the compute cursor, close the piece at the end of the segment or of the wavefront's work
  auto do_unit = [&](PageRegs& R) __attribute__((always_inline)) {
    if (app >= 0 && p + 1 == pe) {
      // The segment's last page is the row's last page, and its slot `app` is the new token's, still unwritten in the pool:
      // the lanes that hold that slot take the token's chunks (K row halves from lanes j and 8 + j of `nr`, V from
      // 16 + j and 24 + j) and write them into the pool, where this wavefront is the page's only reader in this launch.
      const u32x4_t k0 = {(uint32_t)__shfl((int)nr.x, j), (uint32_t)__shfl((int)nr.y, j), (uint32_t)__shfl((int)nr.z, j), (uint32_t)__shfl((int)nr.w, j)};
      const u32x4_t k1 = {(uint32_t)__shfl((int)nr.x, 8 + j), (uint32_t)__shfl((int)nr.y, 8 + j), (uint32_t)__shfl((int)nr.z, 8 + j), (uint32_t)__shfl((int)nr.w, 8 + j)};
      const u32x4_t v0 = {(uint32_t)__shfl((int)nr.x, 16 + j), (uint32_t)__shfl((int)nr.y, 16 + j), (uint32_t)__shfl((int)nr.z, 16 + j), (uint32_t)__shfl((int)nr.w, 16 + j)};
      const u32x4_t v1 = {(uint32_t)__shfl((int)nr.x, 24 + j), (uint32_t)__shfl((int)nr.y, 24 + j), (uint32_t)__shfl((int)nr.z, 24 + j), (uint32_t)__shfl((int)nr.w, 24 + j)};
      uint8_t* dst = const_cast<uint8_t*>(a.pool) + (int64_t)sload(a.pt + tbl + p) * a.page_bytes + (int64_t)(qh / G % a.Hkv) * kSlab +
                     app * kHalfBytes + j * 16;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)                     // (register indices stay compile-time constants)
        if ((app >> 3) == hf && r == (app & 7)) {
          R.k[hf] = __builtin_bit_cast(uint4, k0);
          R.k[2 + hf] = __builtin_bit_cast(uint4, k1);
          R.v[hf] = __builtin_bit_cast(uint4, v0);
          R.v[2 + hf] = __builtin_bit_cast(uint4, v1);
          *(u32x4_t*)dst = k0;
          *(u32x4_t*)(dst + kP * kHalfBytes) = k1;
          *(u32x4_t*)(dst + kBlk) = v0;
          *(u32x4_t*)(dst + kBlk + kP * kHalfBytes) = v1;
        }
    }
    compute(R, p);
    ++p;
    --remaining;
    if (p == pe || remaining == 0) finish_piece();
  };

  PageRegs A, B;
  load_next(A);
  while (remaining > 0) {
    load_next(B);
    do_unit(A);
    load_next(A);
    if (remaining > 0) do_unit(B);
  }
  }
  __syncthreads();                                       // every piece of the bin is in LDS (or went straight to its destination)
  merge_bin_pieces<E, G>(a, bin, W, wib, lds);
}

template <typename E, int GT, int G>
__device__ __forceinline__ void decode_ranges(const DecodeArgs& a, const int block, uint8_t (*plds)[kSlab], const int wpb = kWavesPerBlock) {
  constexpr bool kPair = G < GT;
  const int hs = kPair ? (int)(threadIdx.x >> 6) : 0;      // which wavefront of the pair
  const int h0 = hs * G;                                    // first head (within the group) of this wavefront
  constexpr int C = E::kDimsPerChunk;    // dims per 16-byte chunk
  constexpr int DPL = 2 * C;             // dims per lane
  constexpr int D = 16 * C;              // head dim
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(kPair ? block : block * wpb + (int)(threadIdx.x >> 6));
  if (wv >= a.n_waves) return;
  const int r = lane >> 3, j = lane & 7;

  const int32_t* ww = a.waves + wv * 8;
  int row = __builtin_amdgcn_readfirstlane(ww[0]);
  int g = __builtin_amdgcn_readfirstlane(ww[1]);
  int p = __builtin_amdgcn_readfirstlane(ww[2]);
  int remaining = __builtin_amdgcn_readfirstlane(ww[3]);
  int part = __builtin_amdgcn_readfirstlane(ww[4]);
  // ids of the first range's first three pages (no table lookup before the first loads)
  int pid0 = __builtin_amdgcn_readfirstlane(ww[5]);
  int pid1 = __builtin_amdgcn_readfirstlane(ww[6]);
  int pid2 = __builtin_amdgcn_readfirstlane(ww[7]);
  int tbl_off = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 0]);
  int vis = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 1]);
  int qrow = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 2]);
  int pstart = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 3]);   // first page of the row's own range (pages before it
                                                                       // are a shared prefix handled by the tile kernel)
  bool first_range = true;

  while (remaining > 0) {
    const int np = (vis + kP - 1) / kP;
    const int cnt = min(remaining, np - p);
    const int32_t* tbl = a.pt + tbl_off + p;

    // q chunks of this lane for the G heads of kv head g
    uint4 q[G][2];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const uint8_t* qp = (const uint8_t*)a.q + ((int64_t)qrow * a.Hq + g * GT + h0 + h) * kRowBytes + j * 16;
      q[h][0] = *(const uint4*)qp;
      q[h][1] = *(const uint4*)(qp + kHalfBytes);
    }
    float m[G], l[G], acc[G][DPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m[h] = -1e30f;
      l[h] = 0.f;
#pragma unroll
      for (int d = 0; d < DPL; ++d) acc[h][d] = 0.f;
    }

    const uint8_t* slab0 = a.pool + (int64_t)g * kSlab + lane * 16;
    // tokens of page index pi (absolute, within the row) that exist: the row's last page may be ragged
    auto compute = [&](PageRegs& R, int pi) {
      const int nvalid = vis - pi * kP;          // >= 1; >= 16 for a full page
      if (nvalid < kP) {
        // ragged last page: slots past the file's end hold whatever was there before (possibly
        // NaN patterns); their weight is 0, but 0 * NaN is NaN, so clear their V chunks
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
          if ((hf * 8 + r) >= nvalid) {
            R.v[hf] = make_uint4(0, 0, 0, 0);
            R.v[2 + hf] = make_uint4(0, 0, 0, 0);
          }
      }
      float s[2][G];
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const bool valid = (hf * 8 + r) < nvalid;
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float x = E::dot(R.k[hf], q[h][0], 0.f);
          x = E::dot(R.k[2 + hf], q[h][1], x);
          x = octet_sum(x) * a.scale_log2e;
          s[hf][h] = valid ? x : -__builtin_inff();
        }
      }
      bool need = false;
#pragma unroll
      for (int h = 0; h < G; ++h) need |= fmaxf(s[0][h], s[1][h]) > m[h] + kTau;
      if (__builtin_amdgcn_ballot_w64(need) != 0) {     // rare after the first page
#pragma unroll
        for (int h = 0; h < G; ++h) {
          const float mn = fmaxf(m[h], fmaxf(s[0][h], s[1][h]));
          const float al = __builtin_amdgcn_exp2f(m[h] - mn);
          l[h] *= al;
#pragma unroll
          for (int d = 0; d < DPL; ++d) acc[h][d] *= al;
          m[h] = mn;
        }
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float pw[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
          pw[h] = __builtin_amdgcn_exp2f(s[hf][h] - m[h]);
          l[h] += pw[h];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float vf[C];
          E::unpack(R.v[i * 2 + hf], vf);
#pragma unroll
          for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < C; ++e) acc[h][i * C + e] = __builtin_fmaf(pw[h], vf[e], acc[h][i * C + e]);
        }
      }
    };

    // Page ids come through the scalar cache, two pages ahead of their K/V loads.  Every load in
    // the loop is unconditional, so the loop body has no control-flow join between a prefetch and
    // its use and the compiler can wait for exactly the older page while the newer one is in
    // flight.  Past the end of the range the prefetch is pointed at page 0 of the pool (valid
    // memory that every wave touches, so it stays in L2) and its data is never used.
    const int last = cnt - 1;
    if (!first_range) {
      pid0 = tbl[0];
      pid1 = tbl[min(1, last)];
      pid2 = tbl[min(2, last)];
    }
    first_range = false;
    static_assert(kPair, "one wavefront per range is decode_stream's job");
    {
      // this wavefront's half (K or V) of a page: 4 lane-linear 1 KiB runs -> registers -> LDS
      const uint8_t* half0 = slab0 + hs * kBlk;
      auto load_half = [&](uint4 (&st)[4], int pid) {
        const uint8_t* base = half0 + (int64_t)pid * a.page_bytes;
#pragma unroll
        for (int x = 0; x < 4; ++x) st[x] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)(base + x * 1024)));
      };
      int id1 = cnt > 1 ? pid1 : 0, id2 = cnt > 2 ? pid2 : 0;
      uint4 sa[4], sb[4];                    // pages k and k+1 in flight
      load_half(sa, pid0);
      load_half(sb, id1);
      for (int k = 0; k < cnt; k += 2) {
        // page k
        {
          uint8_t* buf = plds[0] + hs * kBlk + lane * 16;
#pragma unroll
          for (int x = 0; x < 4; ++x) *(uint4*)(buf + x * 1024) = sa[x];
          __syncthreads();                   // both halves of page k are in LDS; the other buffer is free again
          load_half(sa, id2);
          id2 = k + 4 <= last ? tbl[k + 4] : 0;
          PageRegs R;
          const uint8_t* rb = plds[0] + lane * 16;
#pragma unroll
          for (int x = 0; x < 4; ++x) R.k[x] = *(const uint4*)(rb + x * 1024);
#pragma unroll
          for (int x = 0; x < 4; ++x) R.v[x] = *(const uint4*)(rb + kBlk + x * 1024);
          compute(R, p + k);
        }
        // page k + 1 (both wavefronts take the same branch: cnt is the same for the pair)
        {
          uint8_t* buf = plds[1] + hs * kBlk + lane * 16;
#pragma unroll
          for (int x = 0; x < 4; ++x) *(uint4*)(buf + x * 1024) = sb[x];
          __syncthreads();
          id1 = k + 3 <= last ? tbl[k + 3] : 0;
          load_half(sb, id1);
          if (k + 1 < cnt) {
            PageRegs R;
            const uint8_t* rb = plds[1] + lane * 16;
#pragma unroll
            for (int x = 0; x < 4; ++x) R.k[x] = *(const uint4*)(rb + x * 1024);
#pragma unroll
            for (int x = 0; x < 4; ++x) R.v[x] = *(const uint4*)(rb + kBlk + x * 1024);
            compute(R, p + k + 1);
          }
        }
      }
      __syncthreads();                       // the next range of this pair reuses both buffers
    }

    // ---- end of a (row, kv head) range: combine the 8 token slots (lanes with equal j).
    // Per head: common max M, rescale, total sum.  The G*DPL accumulators are then reduced with
    // a halving exchange (lane bit 5, 4, 3 in turn: keep one half of the list, send the other), so
    // lane (r, j) ends up owning the fully reduced values r*V/8 .. r*V/8 + V/8 - 1 of the list.
    const bool whole = (p == 0 && cnt == np);
    constexpr int V = G * DPL;
    float vals[V];
    float lsum[G], Mh[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float M = m[h];
      M = fmaxf(M, row_xor8(M));
      M = fmaxf(M, __shfl_xor(M, 16));
      M = fmaxf(M, __shfl_xor(M, 32));
      const float f = __builtin_amdgcn_exp2f(m[h] - M);
      float ls = l[h] * f;
      ls += row_xor8(ls);
      ls += __shfl_xor(ls, 16);
      ls += __shfl_xor(ls, 32);
      lsum[h] = ls;
      Mh[h] = M;
#pragma unroll
      for (int d = 0; d < DPL; ++d) vals[h * DPL + d] = acc[h][d] * f;
    }
    {
      const bool b5 = (lane & 32) != 0, b4 = (lane & 16) != 0, b3 = (lane & 8) != 0;
#pragma unroll
      for (int i = 0; i < V / 2; ++i) {
        const float keep = b5 ? vals[i + V / 2] : vals[i], send = b5 ? vals[i] : vals[i + V / 2];
        vals[i] = keep + __shfl_xor(send, 32);
      }
#pragma unroll
      for (int i = 0; i < V / 4; ++i) {
        const float keep = b4 ? vals[i + V / 4] : vals[i], send = b4 ? vals[i] : vals[i + V / 4];
        vals[i] = keep + __shfl_xor(send, 16);
      }
#pragma unroll
      for (int i = 0; i < V / 8; ++i) {
        const float keep = b3 ? vals[i + V / 8] : vals[i], send = b3 ? vals[i] : vals[i + V / 8];
        vals[i] = keep + row_xor8(send);
      }
    }
    // lane (r, j) now holds list entries idx = r * V/8 + t: head idx / DPL, lane-local dim idx % DPL
    const int64_t out_row = ((int64_t)qrow * a.Hq + g * GT + h0) * D;
    if (whole) {
#pragma unroll
      for (int t = 0; t < V / 8; ++t) {
        const int idx = r * (V / 8) + t, h = idx / DPL, dl = idx % DPL;
        float ls = lsum[0];
#pragma unroll
        for (int hh = 1; hh < G; ++hh) ls = (h == hh) ? lsum[hh] : ls;
        a.out[out_row + h * D + (dl / C) * (D / 2) + j * C + (dl % C)] = vals[t] / ls;
      }
    } else {
      float* pa = a.part_acc + ((int64_t)part * GT + h0) * D;
#pragma unroll
      for (int t = 0; t < V / 8; ++t) {
        const int idx = r * (V / 8) + t, h = idx / DPL, dl = idx % DPL;
        pa[h * D + (dl / C) * (D / 2) + j * C + (dl % C)] = vals[t];
      }
      if (lane < G) {
        float mm = Mh[0], ll = lsum[0];
#pragma unroll
        for (int hh = 1; hh < G; ++hh) {
          mm = (lane == hh) ? Mh[hh] : mm;
          ll = (lane == hh) ? lsum[hh] : ll;
        }
        a.part_ml[((int64_t)part * GT + h0 + lane) * 2 + 0] = mm;
        a.part_ml[((int64_t)part * GT + h0 + lane) * 2 + 1] = ll;
      }
    }
    if (!whole) ++part;
    remaining -= cnt;
    p += cnt;
    if (p == np) {
      if (++g == a.Hkv) {
        g = 0;
        ++row;
        if (remaining > 0) {
          tbl_off = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 0]);
          vis = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 1]);
          qrow = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 2]);
          pstart = __builtin_amdgcn_readfirstlane(a.rows[row * 4 + 3]);
        }
      }
      p = pstart;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Prefill-chunk attention on the matrix cores (bf16 storage, D = 128).  One workgroup of 4
// wavefronts per tile = (LIP, kv head, TQ = 128/G consecutive new tokens): 128 query rows
// (token, head of the group), 32 per wavefront.  The file's K/V is walked in blocks of 32 tokens
// (two pages), staged through LDS and shared by the 4 wavefronts.  The same kernel serves
// shared-prefix tiles: 128 rows = the decode rows (members x heads) of LIPs whose files begin
// with the same pages; it reads those pages once for all of them and leaves partial results.
//
// Everything is computed transposed so that what belongs to one query row lives in one lane:
//   S^T[token][row] = K · Q^T      v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers)
//   O^T[dim][row]  += V^T · P^T    v_mfma_f32_32x32x16_f16,  A = V^T from LDS, B = P (registers)
// In both results a lane's column is its query row (lane % 32), so the running max, the sum and
// the rescale factor are lane-local, and the 16 scores a lane holds are, in register order,
// exactly the 8+8 token slots it must supply as the B operand of the two PV steps.  The two
// lanes of a row (lane, lane ^ 32) hold different tokens / dims and share only the max.
// P is rounded to fp16 (2^-11; bf16's 2^-8 would not fit a 2e-3 bar on rows with few keys) and
// the softmax sum adds the rounded weights, so the output is an exact weighted mean of V rows
// for slightly perturbed weights.  V is converted bf16 -> fp16 while it is transposed into LDS:
// packing the same dim of two neighbouring tokens into one register IS the transposition.
// ---------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kKvBlock = 32;              // tokens per K/V block
constexpr int kKLds = kKvBlock * kRowBytes;      // 8 KiB: K block, 16-byte chunks, xor-swizzled
constexpr int kVRow = 80;                 // bytes per dim row of V^T in LDS (64 + 16 pad: conflict-free reads)
constexpr int kVLds = 128 * kVRow;        // 10 KiB

template <int G, int TW, bool SPLIT>
__device__ __forceinline__ void tile_block(const PrefillArgs& a, const int block, uint8_t (*lds)[kKLds + kVLds]) {
  // TW = wavefronts of the workgroup (4 or 8); a tile has 32 * TW query rows that share one staging
  // of every K/V block, so K/V bytes read per flop (from L2, and written to LDS) halve with TW = 8.
  // (Two 32-row column tiles per wavefront instead, four wavefronts per 256-row tile, halve the LDS
  // reads per flop but need ~510 registers, one wavefront per SIMD: measured 1.5x slower, also with
  // the pipelined block loop below.)
  constexpr int CT = 1;
  // workgroups go round-robin over the 8 XCDs; the tile list comes in 8 shares of equal cost in which
  // tiles that read the same K/V are neighbours (one L2 per XCD), longest first
  const int tile = a.xcd_off[block % 8] + block / 8;
  if (tile >= a.xcd_off[block % 8 + 1]) return;
  const int32_t* tw = a.tiles + (int64_t)(a.tile_first + tile) * 12;
  const int tbl_off = tw[0], g = tw[4], count = tw[3];
  const bool shared = tw[6] != 0;
  const int32_t* tbl = a.pt + tbl_off;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int col = lane & 31, hf = lane >> 5;
  // prefill chunk: `count` new tokens from chunk offset t0 on a file of L tokens; row tl sees
  // tokens 0 .. L + t0 + tl.  shared prefix: `count` decode rows (q rows in the member list) that
  // all see the same full pages [page0, page1) of the group's first file.
  const int L = tw[1], t0 = tw[5];
  const int kv_end = shared ? tw[8] * kP : L + t0 + count;       // tokens the tile's last row sees
  const int mask_from = shared ? kv_end : L + t0 + 1;            // first token some row may not see
  const int kb0 = shared ? tw[7] / 2 : 0;                        // first 32-token block (page0 is even)
  const int nblk = (kv_end + kKvBlock - 1) / kKvBlock;
  const int last_page = max((kv_end + kP - 1) / kP - 1, 0);
  // A shared-prefix tile of four wavefronts with at most 64 live rows would keep two of them busy, each alone
  // with the whole chain of a block (operand reads, eight chained score MFMAs, weights, PV) in every step.
  // Such a tile is split by key block instead: wavefronts 0 and 1 take the rows for the even blocks,
  // wavefronts 2 and 3 the same rows for the odd blocks, and each does half of a block's chain per
  // step (scores and weights of its block in one step, PV in the next); the two halves are combined
  // through LDS at the end like two pieces of a split range.
  // (A kernel of its own, chosen by the host when every tile of the batch is such a tile: with both block
  // loops in one kernel the register allocator spills inside them.)
  static_assert(!SPLIT || TW == 4, "only four-wavefront tiles are split");
  constexpr bool split = SPLIT;
  const int pair = split ? (wv >> 1) : 0;
  const int wvr = split ? (wv & 1) : wv;                         // which 32 rows of the tile
  const bool wave_live = wvr * 32 * CT < count * G;              // a wavefront whose rows are all padding only stages

  int tl[CT], h[CT], qrow[CT], vis[CT];
  bf16x8_t q[CT][8];             // Q of this lane's rows: 8 k-steps of 16 dims, this lane supplies dims 16*ks + 8*hf .. +8
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int rho = (wvr * CT + ct) * 32 + col;    // query row of this lane inside the tile
    tl[ct] = rho / G;                              // token (prefill) or member (shared prefix) of the row
    h[ct] = rho % G;
    const int tlc = min(tl[ct], count - 1);        // rows past the tile's last token/member repeat it (never written)
    qrow[ct] = shared ? a.members[tw[2] + tlc] : tw[2] + tlc;
    vis[ct] = shared ? kv_end : L + t0 + tlc + 1;  // tokens this row sees
    const uint8_t* qp = (const uint8_t*)a.q + ((int64_t)qrow[ct] * a.Hq + g * G + h[ct]) * kRowBytes + hf * 16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) q[ct][ks] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(qp + ks * 32));
  }

  // ---- staging roles
  // K: thread copies chunk c = tid (and tid + 256 with four wavefronts) of the block: token c/16, dim chunk c%16
  // V: thread takes tokens (4*q4 + 2*up, +1) of page pg, dim chunk vc: VD dims x 2 tokens
  constexpr int VD = TW == 4 ? 8 : 4;                       // dims per thread
  const int up = tid & 1, q4 = (tid >> 1) & 3, vc = (tid >> 3) & (128 / VD - 1), pg = tid >> (TW == 4 ? 7 : 8);
  // K/V of the blocks in flight (loaded three blocks ahead of their use): three register sets
  uint4 ka0, ka1, va0, va1, kb0r, kb1r, vb0, vb1, kc0, kc1, vc0, vc1;
  const uint8_t* slab = a.pool + (int64_t)g * kSlab;
  // Which of the block's two pages a thread stages is the same for its whole wavefront, so the page
  // ids come through the scalar cache and the page base is scalar arithmetic; what differs per
  // thread is a fixed offset inside the page, computed once.
  const int wvu = __builtin_amdgcn_readfirstlane(wv);
  const int k_page = TW == 4 ? 0 : (wvu >> 2);            // chunk tid: page of the block (chunk tid + 256: the other one)
  const int v_page = TW == 4 ? (wvu >> 1) : (wvu >> 2);
  const int kt = (tid >> 4) & 15, kdc = tid & 15;
  const int k_off = (kdc >> 3) * (kP * kHalfBytes) + kt * kHalfBytes + (kdc & 7) * 16;
  const int dbyte = vc * VD * 2;                            // byte offset of the thread's dims in the 256-byte row
  const int v_off = kBlk + (dbyte >> 7) * (kP * kHalfBytes) + (4 * q4 + 2 * up) * kHalfBytes + (dbyte & 127);
  auto page_base = [&](int pi) {
    const int pid = __builtin_amdgcn_readfirstlane(tbl[min(pi, last_page)]);
    return slab + (int64_t)pid * a.page_bytes;
  };
  auto issue_loads = [&](int kb, uint4& k0, uint4& k1, uint4& v0, uint4& v1) {
    const uint8_t* pk = page_base(2 * kb + k_page);
    // four-wavefront tiles are shared-prefix tiles, and each of those streams K/V of its own (nobody reads a
    // line twice): nontemporal loads.  Prefill tiles share their stream with seven neighbours through L2.
    auto ld16 = [&](const uint8_t* q16) {
      if constexpr (TW == 4) return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)q16));
      else return *(const uint4*)q16;
    };
    k0 = ld16(pk + k_off);
    if constexpr (TW == 4) k1 = ld16(page_base(2 * kb + 1) + k_off);
    const uint8_t* p = (TW == 4 ? page_base(2 * kb + v_page) : pk) + v_off;
    if constexpr (TW == 4) {
      v0 = ld16(p);
      v1 = ld16(p + kHalfBytes);
    } else {
      const uint2 x0 = *(const uint2*)p, x1 = *(const uint2*)(p + kHalfBytes);
      v0.x = x0.x; v0.y = x0.y;
      v1.x = x1.x; v1.y = x1.y;
    }
  };
  auto k_dst = [&](uint8_t* base, int c) {
    const int t = c >> 4, dc = c & 15;
    return base + (t * 16 + (dc ^ (t & 15))) * 16;
  };
  auto store_lds = [&](int kb, uint8_t* base, const uint4& k0, const uint4& k1, const uint4& v0, const uint4& v1) {
    *(uint4*)k_dst(base, tid) = k0;
    if constexpr (TW == 4) *(uint4*)k_dst(base, tid + 256) = k1;
    // tokens past the end of what the tile may see are cleared (their weight is 0, 0 * NaN is not);
    // only the last block can hold such tokens
    const int tok = kb * kKvBlock + pg * 16 + 4 * q4 + 2 * up;
    const bool tail = kb * kKvBlock + kKvBlock > kv_end;
    const bool ok0 = !tail || tok < kv_end, ok1 = !tail || tok + 1 < kv_end;
    uint8_t* vb = base + kKLds + (2 * pg + (q4 & 1)) * 16 + (q4 >> 1) * 8 + up * 4 + vc * VD * kVRow;
    auto put = [&](int e, uint32_t lo_word0, uint32_t lo_word1, bool high) {
      const uint32_t x0 = high ? (lo_word0 & 0xffff0000u) : (lo_word0 << 16);
      const uint32_t x1 = high ? (lo_word1 & 0xffff0000u) : (lo_word1 << 16);
      const float f0 = ok0 ? as_f32(x0) : 0.f, f1 = ok1 ? as_f32(x1) : 0.f;
      *(uint32_t*)(vb + e * kVRow) = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f0, f1));
    };
    put(0, v0.x, v1.x, false); put(1, v0.x, v1.x, true);
    put(2, v0.y, v1.y, false); put(3, v0.y, v1.y, true);
    if constexpr (TW == 4) {
      put(4, v0.z, v1.z, false); put(5, v0.z, v1.z, true);
      put(6, v0.w, v1.w, false); put(7, v0.w, v1.w, true);
    }
  };

  f32x16_t O[CT][4];
  float m[CT], l[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    m[ct] = -1e30f;
    l[ct] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) O[ct][db][v] = 0.f;
  }

  // The block loop is software-pipelined over three LDS buffers.  One step: block kb + 1 (loaded three
  // steps ago) goes from registers to LDS, the loads of block kb + 4 are issued into the same
  // registers, then the matrix cores start S^T = K Q^T of block kb + 1 while the vector units do the
  // softmax arithmetic of block kb, and O^T += V^T P^T of block kb follows.  So the MFMAs of one block
  // run under the vector work of its neighbour inside one wavefront, not only across wavefronts.
  // All loads and all blocks are unconditional: past the end the last pages are loaded again and
  // every token is masked, so the loop (unrolled by three) has no control-flow join between a load
  // and its use.  One barrier per step: the buffer a step writes was last read two steps earlier.
  auto k_operands = [&](const uint8_t* base, bf16x8_t (&kk)[8]) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kk[ks] = *(const bf16x8_t*)(base + (col * 16 + ((2 * ks + hf) ^ (col & 15))) * 16);
  };
  auto scores = [&](const bf16x8_t (&kk)[8]) {
    f32x16_t S;
#pragma unroll
    for (int v = 0; v < 16; ++v) S[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kk[ks], q[0][ks], S, 0, 0, 0);
    return S;
  };
  f32x16_t Sc;                   // scores of the current block (computed one step ahead)
  float mx_cur = 0.f;            // their row maximum in log2 units, both lanes of the row agreeing
  // Causal mask and row maximum of the scores in Sc (block kb), done as soon as the scores exist, at the
  // end of the step before the one that uses them: the exchange between the two lanes of a row goes
  // through the LDS pipe, and there it must not queue behind the sixteen operand reads of its own step
  // with the MFMAs waiting for the branch that needs it.
  // value v of a lane is token 8*(v/4) + 4*hf + v%4 of the block
  // scores stay unscaled; the scale (softmax scale * log2 e, positive) goes into one fma with the max
  auto mask_and_max = [&](const int kb) __attribute__((always_inline)) {
    const int tok0 = kb * kKvBlock + 4 * hf;
    const bool edge = kb * kKvBlock + kKvBlock > mask_from;      // the block reaches the causal edge of some row
    float mx = -__builtin_inff();
    if (edge) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int tok = tok0 + 8 * (v >> 2) + (v & 3);
        Sc[v] = tok < vis[0] ? Sc[v] : -__builtin_inff();
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, Sc[v]);
    mx_cur = fmaxf(mx, __shfl_xor(mx, 32)) * a.scale_log2e;
  };
  auto step = [&](const int kb, uint8_t* cur, uint8_t* nxt, uint4& k0, uint4& k1, uint4& v0, uint4& v1) {
    store_lds(kb + 1, nxt, k0, k1, v0, v1);
    __syncthreads();           // block kb + 1 is in LDS; everyone is done with the block that was in `nxt` before
    issue_loads(kb + 4, k0, k1, v0, v1);
    if (!wave_live) return;

    // operands of both MFMA phases are requested from LDS up front: the latency is paid once per step
    bf16x8_t kk[8];
    k_operands(nxt, kk);
    const uint8_t* vbase = cur + kKLds + col * kVRow + hf * 16;
    f16x8_t vv[4][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < 4; ++db) vv[db][ks] = *(const f16x8_t*)(vbase + db * 32 * kVRow + ks * 32);
    __builtin_amdgcn_sched_barrier(0);

    // the block's row maximum was found at the end of the step before (mask_and_max)
    const float mx = mx_cur;
    if (__builtin_amdgcn_ballot_w64(mx > m[0] + kTau) != 0) {     // rare after the first block
      const float mn = fmaxf(m[0], mx);
      const float al = __builtin_amdgcn_exp2f(m[0] - mn);
      l[0] *= al;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[0][db][v] *= al;
      m[0] = mn;
    }
    // From here to the end of the step there is no branch: the scores of block kb + 1 (eight MFMAs)
    // run under the exponentials of block kb; then the weights of the block's first 16 tokens, their
    // O^T += V^T P^T MFMAs (four independent accumulators), and the second 16 tokens' weights while those run.
    const f32x16_t Sn = scores(kk);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      uint32_t pw[4];
#pragma unroll
      for (int u = 0; u < 8; u += 2) {
        const int v = 8 * ks + u;
        const auto pk = __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(__builtin_fmaf(Sc[v], a.scale_log2e, -m[0])),
                                                   __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[v + 1], a.scale_log2e, -m[0])));
        l[0] = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, pk), f16x2_t{(_Float16)1.0f, (_Float16)1.0f}, l[0], false);
        pw[u >> 1] = __builtin_bit_cast(uint32_t, pk);
      }
      const f16x8_t P = __builtin_bit_cast(f16x8_t, make_uint4(pw[0], pw[1], pw[2], pw[3]));
#pragma unroll
      for (int db = 0; db < 4; ++db) O[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vv[db][ks], P, O[0][db], 0, 0, 0);
    }
    // issue order of this stretch: one MFMA, then a few vector instructions, sixteen times (the first
    // eight MFMAs are the scores of the next block, which depend on nothing computed here)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 4, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x402, 2, 0);
    }
    Sc = Sn;
    mask_and_max(kb + 1);
  };

  // A tile split by key block (see `split` above).  The pair whose block it is computes scores, maximum and
  // weights of block kb + 1 (K in `nxt`) in step kb and the PV product of that block (V^T then in `cur`) in
  // step kb + 1, while the other pair does the same one block later: the buffers are read in the same steps
  // as in the unsplit loop, so three of them and one barrier per step still do.
  uint32_t pwc[2][4] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
  auto first_half = [&](const int kb, const uint8_t* kbuf) {
    bf16x8_t kk[8];
    k_operands(kbuf, kk);
    Sc = scores(kk);
    mask_and_max(kb);
    const float mx = mx_cur;
    if (__builtin_amdgcn_ballot_w64(mx > m[0] + kTau) != 0) {
      const float mn = fmaxf(m[0], mx);
      const float al = __builtin_amdgcn_exp2f(m[0] - mn);
      l[0] *= al;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[0][db][v] *= al;
      m[0] = mn;
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int u = 0; u < 8; u += 2) {
        const int v = 8 * ks + u;
        const auto pk = __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(__builtin_fmaf(Sc[v], a.scale_log2e, -m[0])),
                                                   __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[v + 1], a.scale_log2e, -m[0])));
        l[0] = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, pk), f16x2_t{(_Float16)1.0f, (_Float16)1.0f}, l[0], false);
        pwc[ks][u >> 1] = __builtin_bit_cast(uint32_t, pk);
      }
  };
  auto second_half = [&](const uint8_t* vbuf) {
    const uint8_t* vbase = vbuf + kKLds + col * kVRow + hf * 16;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const f16x8_t P = __builtin_bit_cast(f16x8_t, make_uint4(pwc[ks][0], pwc[ks][1], pwc[ks][2], pwc[ks][3]));
#pragma unroll
      for (int db = 0; db < 4; ++db)
        O[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8_t*)(vbase + db * 32 * kVRow + ks * 32), P, O[0][db], 0, 0, 0);
    }
  };
  auto step_split = [&](const int kb, const uint8_t* cur, uint8_t* nxt, uint4& k0, uint4& k1, uint4& v0, uint4& v1) {
    store_lds(kb + 1, nxt, k0, k1, v0, v1);
    __syncthreads();
    issue_loads(kb + 5, k0, k1, v0, v1);
    if (!wave_live) return;
    if (((kb - kb0) & 1) == pair) second_half(cur);
    else first_half(kb + 1, nxt);
  };

  if constexpr (SPLIT) {
    // This kernel has registers to spare: a fourth set of staging registers (and a fourth LDS buffer, so that
    // the loop unrolled by four addresses them statically) puts the loads four blocks ahead of their use.
    // These tiles each stream K/V of their own, and what bounds them is the bytes in flight.
    uint4 kd0, kd1, vd0, vd1;
    issue_loads(kb0, ka0, ka1, va0, va1);
    issue_loads(kb0 + 1, kb0r, kb1r, vb0, vb1);
    issue_loads(kb0 + 2, kc0, kc1, vc0, vc1);
    issue_loads(kb0 + 3, kd0, kd1, vd0, vd1);
    store_lds(kb0, lds[0], ka0, ka1, va0, va1);
    __syncthreads();
    issue_loads(kb0 + 4, ka0, ka1, va0, va1);
    if (wave_live && pair == 0) first_half(kb0, lds[0]);
    for (int kb = kb0; kb < nblk; kb += 4) {
      step_split(kb, lds[0], lds[1], kb0r, kb1r, vb0, vb1);
      step_split(kb + 1, lds[1], lds[2], kc0, kc1, vc0, vc1);
      step_split(kb + 2, lds[2], lds[3], kd0, kd1, vd0, vd1);
      step_split(kb + 3, lds[3], lds[0], ka0, ka1, va0, va1);
    }
    // the odd blocks' half (wavefronts 2, 3) goes to the even blocks' (wavefronts 0, 1) through LDS: per
    // lane maximum, sum and the 64 accumulator values
    __syncthreads();
    float* xch = (float*)lds[0] + (wvr * 66) * 64 + lane;
    if (pair == 1) {
      xch[0] = m[0];
      xch[64] = l[0];
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) xch[(2 + db * 16 + v) * 64] = O[0][db][v];
    }
    __syncthreads();
    if (pair == 1) return;
    {
      const float m1 = xch[0], l1 = xch[64];
      const float mn = fmaxf(m[0], m1);
      const float a0 = __builtin_amdgcn_exp2f(m[0] - mn), a1 = __builtin_amdgcn_exp2f(m1 - mn);
      l[0] = l[0] * a0 + l1 * a1;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[0][db][v] = O[0][db][v] * a0 + xch[(2 + db * 16 + v) * 64] * a1;
      m[0] = mn;
    }
  } else {
  issue_loads(kb0, ka0, ka1, va0, va1);
  issue_loads(kb0 + 1, kb0r, kb1r, vb0, vb1);
  issue_loads(kb0 + 2, kc0, kc1, vc0, vc1);
  store_lds(kb0, lds[0], ka0, ka1, va0, va1);
  __syncthreads();
  issue_loads(kb0 + 3, ka0, ka1, va0, va1);
  if (wave_live) {
    bf16x8_t kk[8];
    k_operands(lds[0], kk);
    Sc = scores(kk);
    mask_and_max(kb0);
  }
  for (int kb = kb0; kb < nblk; kb += 3) {
    step(kb, lds[0], lds[1], kb0r, kb1r, vb0, vb1);
    step(kb + 1, lds[1], lds[2], kc0, kc1, vc0, vc1);
    step(kb + 2, lds[2], lds[0], ka0, ka1, va0, va1);
  }
  }

#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const float lt = l[ct] + __shfl_xor(l[ct], 32);
    if (tl[ct] < count) {
      if (!shared) {
        const float inv = 1.0f / lt;
        float* o = a.out + ((int64_t)qrow[ct] * a.Hq + g * G + h[ct]) * 128 + 4 * hf;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int vb = 0; vb < 4; ++vb)
            *(float4*)(o + db * 32 + vb * 8) = make_float4(O[ct][db][4 * vb] * inv, O[ct][db][4 * vb + 1] * inv, O[ct][db][4 * vb + 2] * inv, O[ct][db][4 * vb + 3] * inv);
      } else {
        // partial result of member tl for the merge kernel: unnormalised accumulator, max, sum
        const int64_t part = (int64_t)t0 + tl[ct];           // t0 = first partial slot of this tile
        float* o = a.part_acc + (part * G + h[ct]) * 128 + 4 * hf;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int vb = 0; vb < 4; ++vb)
            *(float4*)(o + db * 32 + vb * 8) = make_float4(O[ct][db][4 * vb], O[ct][db][4 * vb + 1], O[ct][db][4 * vb + 2], O[ct][db][4 * vb + 3]);
        if (hf == 0) {
          a.part_ml[(part * G + h[ct]) * 2 + 0] = m[ct];
          a.part_ml[(part * G + h[ct]) * 2 + 1] = lt;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Decode ranges on the matrix cores (bf16 storage).  With 8 query heads per kv head the VALU
// decode kernel above is bound by vector issue, not by HBM (8 flop per KV byte in plain fp32
// FMAs); the 8 heads of a group are a small query tile, so here one wavefront per range feeds
// them to 16x16x32 MFMAs (16 columns, GT of them used):
//   S^T[16 tokens][16 heads] = K · Q^T     A = K rows straight from global memory (64 B per token and
//                                          k-step, no LDS), B = Q (registers), per page
//   O^T[128 dims][16 heads] += V^T · P^T    per two pages (k = 32 tokens); V^T through a wavefront-private
//                                          LDS buffer, written by the wavefront itself while it converts
//                                          bf16 -> fp16 (pairs of neighbouring tokens packed = the transpose)
// A lane's column is a head in both results, so max / sum / rescale factor are lane-local; the
// four lane groups of a head hold different tokens and share only the (lagging) running max.
// No barrier anywhere: the LDS buffer is private to the wavefront.
// A row may hold nt <= 16 / GT consecutive new tokens of one LIP (a short draft being verified,
// paper section 4.1): column c is then (token c / GT, head c % GT), token t sees vis + t file
// tokens, and the page loop runs to the last token's limit: one pass over K/V for all of them.
// ---------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
constexpr int kVtRow = 80;                    // bytes per dim row of V^T (32 tokens fp16 + 16 pad)
constexpr int kVtLds = 128 * kVtRow;          // 10 KiB per wavefront

template <int GT>
__device__ __forceinline__ void decode_mfma_ranges(const DecodeArgs& a, const int block, uint8_t* vlds) {
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(block * kWavesPerBlock + (int)(threadIdx.x >> 6));
  if (wv >= a.n_waves) return;
  const int col = lane & 15, grp = lane >> 4;        // query column, lane group (tokens 4*grp .. 4*grp+3 of a page)
  const int head = col % GT;                          // columns past nt * GT repeat earlier ones; their results are ignored
  const int vq4 = lane >> 4, vc = lane & 15;          // V staging role: tokens 4*vq4 .. +3 of a page, dim chunk vc
  auto sload = [&](const int32_t* ptr) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(*ptr); };

  // As in the VALU kernel, the wavefront's units form ONE stream: a load cursor runs ahead of the compute
  // cursor through the same sequence of (row, kv head) ranges, in steps of a pair of pages (a pair never
  // straddles two ranges: the last pair of a range with an odd number of pages has one page), so the
  // K/V loads of the next range are in flight while the current one is finished and written out.
  const int32_t* ww = a.waves + wv * 8;
  // compute cursor: the range being accumulated
  int row = sload(ww + 0), g = sload(ww + 1), p = sload(ww + 2);
  int remaining = sload(ww + 3);
  int part = sload(ww + 4);
  const int tbl0 = sload(a.rows + row * 4 + 0);
  int vis = sload(a.rows + row * 4 + 1), qrow = sload(a.rows + row * 4 + 2);
  int pstart = sload(a.rows + row * 4 + 3);
  int nt = (pstart >> 28) + 1;                        // new tokens in the row
  pstart &= 0x0fffffff;
  int np = (vis + nt - 1 + kP - 1) / kP;              // pages the row's last token sees
  // load cursor: the pair whose K/V is requested next
  int lg = g, lrow = row, lp = p, lnp = np, ltbl = tbl0, lpstart = pstart, lrem = remaining;
  int id0 = sload(ww + 5), id1 = sload(ww + 6);       // page ids of that pair (the first pair's come with the wave record)
  // record of the row after the load cursor's, fetched a whole row ahead (one past the last row: valid words, never used)
  int n_tbl = 0, n_np = 0, n_pstart = 0;
  auto fetch_next_row = [&](int rr) __attribute__((always_inline)) {
    n_tbl = sload(a.rows + rr * 4 + 0);
    const int v = sload(a.rows + rr * 4 + 1), ps = sload(a.rows + rr * 4 + 3);
    n_pstart = ps & 0x0fffffff;
    n_np = (v + (ps >> 28) + kP - 1) / kP;
  };
  fetch_next_row(row + 1);
  // record of row + 1 as the compute side needs it
  int c_nvis = 0, c_nqrow = 0, c_nps = 0;
  auto fetch_compute_next_row = [&]() __attribute__((always_inline)) {
    c_nvis = sload(a.rows + (row + 1) * 4 + 1);
    c_nqrow = sload(a.rows + (row + 1) * 4 + 2);
    c_nps = sload(a.rows + (row + 1) * 4 + 3);
  };
  fetch_compute_next_row();

  // K of a page as the A operand: token col, chunk 4*ks + grp of its row (row half ks/2, chunk 4*(ks%2) + grp)
  const int k_off = col * kHalfBytes + grp * 16;
  // V of a page for the staging: tokens 4*vq4 + u, chunk vc
  const int v_off = kBlk + (vc >> 3) * (kP * kHalfBytes) + (4 * vq4) * kHalfBytes + (vc & 7) * 16;
  auto load_page = [&](uint4 (&kk)[4], uint4 (&vv)[4], const uint8_t* slab, int pid) __attribute__((always_inline)) {
    const uint8_t* base = slab + (int64_t)pid * a.page_bytes;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      kk[ks] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)(base + k_off + (ks >> 1) * (kP * kHalfBytes) + (ks & 1) * 64)));
#pragma unroll
    for (int u = 0; u < 4; ++u)
      vv[u] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t*)(base + v_off + u * kHalfBytes)));
  };
  // Requests the next pair and moves the load cursor; every load is unconditional (a page that does not
  // exist, also past the end of the wavefront's work, is page 0 of the pool and is never used).
  auto load_next_pair = [&](uint4 (&k0)[4], uint4 (&v0)[4], uint4 (&k1)[4], uint4 (&v1)[4]) __attribute__((always_inline)) {
    const int take = min(2, min(lrem, lnp - lp));
    const uint8_t* slab = a.pool + (int64_t)(take > 0 ? lg : 0) * kSlab;
    load_page(k0, v0, slab, take > 0 ? id0 : 0);
    load_page(k1, v1, slab, take > 1 ? id1 : 0);
    if (take > 0) {
      lrem -= take;
      lp += take;
      if (lp == lnp) {                                 // the range after: next head of the row, or the next row
        if (++lg == a.Hkv) {
          lg = 0;
          ++lrow;
          ltbl = n_tbl;
          lnp = n_np;
          lpstart = n_pstart;
          fetch_next_row(lrow + 1);
        }
        lp = lpstart;
      }
      const int t2 = min(2, min(lrem, lnp - lp));      // ids of the pair after this one, used one pair later
      id0 = t2 > 0 ? sload(a.pt + ltbl + lp) : 0;
      id1 = t2 > 1 ? sload(a.pt + ltbl + lp + 1) : 0;
    }
  };

  // state of the range being accumulated
  int tok = 0;                                        // this column's token within the row
  bf16x8_t q[4];                                      // Q^T operand: this lane's (token, head), dims 32*ks + 8*grp .. +8
  auto load_q = [&]() __attribute__((always_inline)) {
    tok = min(col / GT, nt - 1);
    const uint8_t* qp = (const uint8_t*)a.q + ((int64_t)(qrow + tok) * a.Hq + g * GT + head) * kRowBytes + grp * 16;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) q[ks] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(qp + ks * 64));
  };
  f32x4_t O[8];
  float m = -1e30f, l = 0.f;
  auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int db = 0; db < 8; ++db) O[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    m = -1e30f;
    l = 0.f;
  };
  reset_state();
  load_q();
  int p_first = p;                                    // first page of the piece being accumulated

  // scores of one page: 4 tokens (4*grp + v) x this lane's head; tokens past nvalid masked
  auto scores = [&](const uint4 (&kk)[4], int nvalid, float (&sc)[4]) __attribute__((always_inline)) {
    f32x4_t S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kk[ks]), q[ks], S, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 4; ++v) sc[v] = (4 * grp + v) < nvalid ? S[v] : -__builtin_inff();
  };
  // V of one page -> fp16, transposed, into the wavefront's LDS buffer (half pg of every dim row)
  auto stage_v = [&](const uint4 (&vv)[4], int nvalid, int pg) __attribute__((always_inline)) {
    const uint32_t w[4][4] = {{vv[0].x, vv[0].y, vv[0].z, vv[0].w}, {vv[1].x, vv[1].y, vv[1].z, vv[1].w},
                              {vv[2].x, vv[2].y, vv[2].z, vv[2].w}, {vv[3].x, vv[3].y, vv[3].z, vv[3].w}};
    bool ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) ok[u] = (4 * vq4 + u) < nvalid;      // slots past the file's end may hold anything
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float f[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t x = (e & 1) ? (w[u][e >> 1] & 0xffff0000u) : (w[u][e >> 1] << 16);
        f[u] = ok[u] ? as_f32(x) : 0.f;
      }
      const int d = vc * 8 + e;
      uint2 pk;
      pk.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f[0], f[1]));
      pk.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(f[2], f[3]));
      *(uint2*)(vlds + d * kVtRow + ((vq4 ^ ((d >> 4) & 3)) * 16) + pg * 8) = pk;
    }
  };
  // two pages (32 tokens): scores, softmax weights, O^T += V^T P^T
  auto compute2 = [&](const uint4 (&kA)[4], const uint4 (&vA)[4], const uint4 (&kB)[4], const uint4 (&vB)[4], int piA, bool haveB) __attribute__((always_inline)) {
    // tokens of the page visible to this column's token; slots that hold file tokens at all
    const int nvA = vis + tok - piA * kP, nvB = haveB ? nvA - kP : 0;
    const int nsA = vis + nt - 1 - piA * kP, nsB = haveB ? nsA - kP : 0;
    float sA[4], sB[4];
    scores(kA, nvA, sA);
    scores(kB, nvB, sB);
    stage_v(vA, nsA, 0);
    stage_v(vB, nsB, 1);
    const float mx = fmaxf(fmaxf(fmaxf(sA[0], sA[1]), fmaxf(sA[2], sA[3])), fmaxf(fmaxf(sB[0], sB[1]), fmaxf(sB[2], sB[3]))) * a.scale_log2e;
    if (__builtin_amdgcn_ballot_w64(mx > m + kTau) != 0) {       // rare after the first pages
      float mn = fmaxf(m, mx);
      mn = fmaxf(mn, __shfl_xor(mn, 16));
      mn = fmaxf(mn, __shfl_xor(mn, 32));                        // all four lane groups of the head agree
      const float al = __builtin_amdgcn_exp2f(m - mn);
      l *= al;
#pragma unroll
      for (int db = 0; db < 8; ++db)
#pragma unroll
        for (int v = 0; v < 4; ++v) O[db][v] *= al;
      m = mn;
    }
    uint32_t pw[4];
#pragma unroll
    for (int v = 0; v < 4; v += 2) {
      const auto pa = __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(__builtin_fmaf(sA[v], a.scale_log2e, -m)),
                                                 __builtin_amdgcn_exp2f(__builtin_fmaf(sA[v + 1], a.scale_log2e, -m)));
      const auto pb = __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(__builtin_fmaf(sB[v], a.scale_log2e, -m)),
                                                 __builtin_amdgcn_exp2f(__builtin_fmaf(sB[v + 1], a.scale_log2e, -m)));
      l = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, pa), f16x2_t{(_Float16)1.0f, (_Float16)1.0f}, l, false);
      l = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, pb), f16x2_t{(_Float16)1.0f, (_Float16)1.0f}, l, false);
      pw[v >> 1] = __builtin_bit_cast(uint32_t, pa);
      pw[2 + (v >> 1)] = __builtin_bit_cast(uint32_t, pb);
    }
    const f16x8_t P = __builtin_bit_cast(f16x8_t, make_uint4(pw[0], pw[1], pw[2], pw[3]));
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const f16x8_t vt = *(const f16x8_t*)(vlds + (db * 16 + col) * kVtRow + ((grp ^ (db & 3)) * 16));
      O[db] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vt, P, O[db], 0, 0, 0);
    }
  };

  // End of a piece: the four lane groups of a head add up their sums, O^T is complete; the compute cursor
  // moves to the next range first, so that its query rows are on their way while this piece is written.
  auto finish_piece = [&]() __attribute__((always_inline)) {
    const bool whole = (p_first == 0 && p == np);
    const int64_t o_row = (int64_t)(qrow + tok) * a.Hq + g * GT + head;
    const int64_t o_slot = (int64_t)(part + tok) * GT + head;     // a piece leaves one partial per token of the row
    const bool o_live = col < nt * GT;
    if (!whole) part += nt;
    const bool more = remaining > 0;
    if (more) {
      if (++g == a.Hkv) {
        g = 0;
        ++row;
        vis = c_nvis;
        qrow = c_nqrow;
        nt = (c_nps >> 28) + 1;
        pstart = c_nps & 0x0fffffff;
        np = (vis + nt - 1 + kP - 1) / kP;
        fetch_compute_next_row();
      }
      load_q();
    }
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (o_live) {
      if (whole) {
        const float inv = 1.0f / l;
        float* o = a.out + o_row * 128 + 4 * grp;
#pragma unroll
        for (int db = 0; db < 8; ++db) *(float4*)(o + db * 16) = make_float4(O[db][0] * inv, O[db][1] * inv, O[db][2] * inv, O[db][3] * inv);
      } else {
        float* o = a.part_acc + o_slot * 128 + 4 * grp;
#pragma unroll
        for (int db = 0; db < 8; ++db) *(float4*)(o + db * 16) = make_float4(O[db][0], O[db][1], O[db][2], O[db][3]);
        if (grp == 0) {
          a.part_ml[o_slot * 2 + 0] = m;
          a.part_ml[o_slot * 2 + 1] = l;
        }
      }
    }
    if (more) {
      p = pstart;
      p_first = p;
      reset_state();
    }
  };
  // one pair of the stream: accumulate it, move the compute cursor, close the piece at the end of the range or of the wavefront's work
  auto do_pair = [&](const uint4 (&kA)[4], const uint4 (&vA)[4], const uint4 (&kB)[4], const uint4 (&vB)[4]) __attribute__((always_inline)) {
    const int took = max(1, min(2, min(remaining, np - p)));     // >= 1 whatever the descriptor says: the loop ends
    compute2(kA, vA, kB, vB, p, took > 1);
    p += took;
    remaining -= took;
    if (p == np || remaining == 0) finish_piece();
  };

  // pair k in registers while pair k + 1 is in flight
  uint4 kA[4], vA[4], kB[4], vB[4], kC[4], vC[4], kD[4], vD[4];
  load_next_pair(kA, vA, kB, vB);
  load_next_pair(kC, vC, kD, vD);
  while (remaining > 0) {
    do_pair(kA, vA, kB, vB);
    load_next_pair(kA, vA, kB, vB);
    if (remaining > 0) do_pair(kC, vC, kD, vD);
    load_next_pair(kC, vC, kD, vD);
  }
}

template <int GT>
__global__ __launch_bounds__(256, 2) void decode_mfma_kernel(DecodeArgs da) {
  __shared__ __align__(16) uint8_t vlds[kWavesPerBlock][kVtLds];
  decode_mfma_ranges<GT>(da, blockIdx.x, vlds[threadIdx.x >> 6]);
}

// ---------------------------------------------------------------------------------------
// The attention launch of a batch: workgroups that run tiles (prefill chunks and shared prefixes)
// and workgroups that run decode ranges (one wavefront per range) in ONE grid, so the two kinds of
// work fill the GPU together and there is no launch boundary between them.
// ---------------------------------------------------------------------------------------
template <typename E, int G, int TW, bool SPLIT = false>
__global__ __launch_bounds__(64 * TW, 8 / TW) void attn_kernel(DecodeArgs da, PrefillArgs pa) {
  // Workgroups come in groups of eight (one per XCD, which the tile order relies on).  The host's table says what a
  // group runs: tile group g (g >= 0) or decode group ~g.  By default the decode groups are spread among the
  // first half of the tile groups, so that some CUs stream K/V from HBM for decode ranges while the others keep
  // the matrix cores busy: the two kinds of work are bound by different units.  (Measured on the mixed batch:
  // 1.85 ms against 1.91 ms with all tiles first; spread over the whole grid: 2.02 ms.  A CU that runs decode
  // ranges alone has only its eight wavefronts' loads in flight, so the gain is small.)
  const uint32_t j = blockIdx.x >> 3, x = blockIdx.x & 7;
  const int32_t g = pa.group_map ? __builtin_amdgcn_readfirstlane(pa.group_map[j]) : (int32_t)j;   // no table: tiles only
  const bool is_decode = g < 0;
  // LDS: the K/V buffers of a tile workgroup, or the piece slots of a decode bin (a workgroup is one or the other)
  constexpr int kTileLds = E::kDimsPerChunk == 8 ? (SPLIT ? 4 : 3) * (kKLds + kVLds) : 0;      // tiles exist for bf16 storage only
  constexpr int kBinLds = G < 8 ? 2 * TW * BinLds<E, G < 8 ? G : 1>::kSlot * 4 : 0;
  constexpr int kLds = kTileLds > kBinLds ? kTileLds : (kBinLds > 16 ? kBinLds : 16);
  __shared__ __align__(16) uint8_t lds[kLds];
  if constexpr (E::kDimsPerChunk == 8) {
    if (!is_decode) {
      tile_block<G, TW, SPLIT>(pa, (int)(g * 8 + x), (uint8_t(*)[kKLds + kVLds])lds);
      return;
    }
  }
  if constexpr (G < 8) {
    if (is_decode) decode_bins<E, G>(da, (int)(~g * 8 + x), TW, (float*)lds);
  }
}

// A batch without tiles (plain decode): the decode bins alone, W wavefronts per bin.
template <typename E, int G, int W>
__global__ __launch_bounds__(64 * W, 8 / W) void decode_only_kernel(DecodeArgs da) {
  __shared__ __align__(16) float lds[2 * W * BinLds<E, G>::kSlot];
  decode_bins<E, G>(da, (int)blockIdx.x, W, lds);
}

// Decode ranges for 8 query heads per kv head: one workgroup of two wavefronts per range.
template <typename E>
__global__ __launch_bounds__(128, 2) void decode_pair_kernel(DecodeArgs da) {
  __shared__ __align__(16) uint8_t plds[2][kSlab];
  decode_ranges<E, 8, 4>(da, blockIdx.x, plds);
}

// ---------------------------------------------------------------------------------------
// Merge of partial results, one wavefront per (row, kv head) that was cut:
//   out = sum_i acc_i 2^(m_i - M) / sum_i l_i 2^(m_i - M),  M = max_i m_i.
// The G*D accumulator values of a piece form one flat list; lane owns entries e*64 + lane.  All
// loads of a group of 4 pieces are issued before any is used (indices past the end re-read the
// last piece with weight 0), so the kernel costs one memory round trip per group after the entry.  A row that belongs
// to a shared-prefix group has extra pieces: the partials the tile kernel left for the prefix.
// ---------------------------------------------------------------------------------------
template <int G, int D>
__global__ __launch_bounds__(kWavesPerBlock * 64) void merge_kernel(MergeArgs a) {
  const int lane = threadIdx.x & 63;
  const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
  if (item >= a.n_items) return;
  const int32_t* it = a.items + item * 8;
  const int first = __builtin_amdgcn_readfirstlane(it[0]);
  const int own = __builtin_amdgcn_readfirstlane(it[1]);
  const int64_t out_row = (int64_t)__builtin_amdgcn_readfirstlane(it[2]) * D;   // (q row * Hq + first head) * D
  // pieces own .. own + xcount - 1 are the partials of the row's shared prefix: xfirst + i * xstride
  const int xfirst = __builtin_amdgcn_readfirstlane(it[3]);
  const int xstride = __builtin_amdgcn_readfirstlane(it[4]);
  const int pieces = own + __builtin_amdgcn_readfirstlane(it[5]);
  const int ostride = __builtin_amdgcn_readfirstlane(it[6]);      // distance between own pieces (tokens in the row)
  auto slot = [&](int i) -> int64_t {
    i = min(i, pieces - 1);
    return i < own ? first + (int64_t)i * ostride : xfirst + (int64_t)(i - own) * xstride;
  };
  constexpr int VL = G * D / 64;
  const float* ml0 = a.part_ml;
  const float* pa0 = a.part_acc + lane;
  float Mx[G], ls[G], o[VL];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    Mx[h] = -__builtin_inff();
    ls[h] = 0.f;
  }
#pragma unroll
  for (int e = 0; e < VL; ++e) o[e] = 0.f;
  // groups of 4 pieces: all their loads (max, sum, accumulator) are issued together, one memory round
  // trip per group; the running maximum is carried from group to group (most rows have one group)
  for (int i0 = 0; i0 < pieces; i0 += 4) {
    float mv[4][G], lv[4][G], t[4][VL];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t ii = slot(i0 + u);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        mv[u][h] = ml0[(ii * G + h) * 2];
        lv[u][h] = ml0[(ii * G + h) * 2 + 1];
      }
#pragma unroll
      for (int e = 0; e < VL; ++e) t[u][e] = pa0[ii * G * D + e * 64];
    }
    float sc[G];                                  // factor that brings what was summed so far to the new maximum
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mn = Mx[h];
#pragma unroll
      for (int u = 0; u < 4; ++u) mn = fmaxf(mn, mv[u][h]);
      sc[h] = __builtin_amdgcn_exp2f(Mx[h] - mn);     // 0 for the first group (Mx = -inf)
      Mx[h] = mn;
      ls[h] *= sc[h];
    }
#pragma unroll
    for (int e = 0; e < VL; ++e) o[e] *= sc[(e * 64) / D];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float w[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        w[h] = (i0 + u < pieces) ? __builtin_amdgcn_exp2f(mv[u][h] - Mx[h]) : 0.f;
        ls[h] = __builtin_fmaf(lv[u][h], w[h], ls[h]);
      }
#pragma unroll
      for (int e = 0; e < VL; ++e) o[e] = __builtin_fmaf(t[u][e], w[(e * 64) / D], o[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < VL; ++e) a.out[out_row + e * 64 + lane] = o[e] / ls[(e * 64) / D];
}

// ---------------------------------------------------------------------------------------
// Prologue of a batch, one launch: (1) KV append, one thread per 16-byte chunk of a new K or
// V row; (2) copy-on-write page copies, one block per copy: slots [0, r) of every (head, K/V,
// row half) of page src into page dst; (3) the batch descriptor copied from pinned host memory
// into the device workspace for the attention kernel that follows.  The three parts touch
// disjoint bytes (a copy covers slots below r, appends write slots from r on), so they need
// no ordering among themselves.  Slot map and copy list are read straight from the pinned
// host buffer.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prologue_kernel(PrologueArgs a) {
  int blk = blockIdx.x;
  if (blk < a.append_blocks) {
    const int64_t tid = (int64_t)blk * 256 + threadIdx.x;
    const int64_t total = (int64_t)a.n_tokens * a.Hkv * 32;
    if (tid >= total) return;
    const int c = tid & 15;                 // chunk within the row
    const int kv = (tid >> 4) & 1;
    const int64_t th = tid >> 5;            // token * Hkv + head
    const int g = (int)(th % a.Hkv);
    const int64_t t = th / a.Hkv;
    const int slot = a.slots[t];
    if (slot < 0) return;                   // this token is appended by the attention kernel
    const int page = slot / kP, ts = slot % kP;
    const uint8_t* src = (const uint8_t*)(kv ? a.v_new : a.k_new) + th * kRowBytes + c * 16;
    uint8_t* dst = a.pool + (int64_t)page * a.page_bytes + (int64_t)g * kSlab + kv * kBlk +
                   (c >> 3) * (kP * kHalfBytes) + ts * kHalfBytes + (c & 7) * 16;
    *(uint4*)dst = *(const uint4*)src;
    return;
  }
  blk -= a.append_blocks;
  if (blk < a.n_cow) {
    const int src = a.cow[blk * 3 + 0], dst = a.cow[blk * 3 + 1], r = a.cow[blk * 3 + 2];
    const uint8_t* s = a.pool + (int64_t)src * a.page_bytes;
    uint8_t* d = a.pool + (int64_t)dst * a.page_bytes;
    const int per_seg = r * (kHalfBytes / 16);           // 16-byte chunks per (head, K/V, half)
    const int n_seg = a.Hkv * 4;
    for (int x = threadIdx.x; x < n_seg * per_seg; x += 256) {
      const int seg = x / per_seg, w = x % per_seg;
      const int64_t off = (int64_t)seg * (kP * kHalfBytes) + w * 16;
      *(uint4*)(d + off) = *(const uint4*)(s + off);
    }
    return;
  }
  blk -= a.n_cow;
  // 16 bytes per thread, enough blocks that the whole descriptor is one round trip to the host
  const uint4* src = (const uint4*)a.host_words;
  uint4* dst = (uint4*)a.dev_words;
  const int64_t n16 = (a.copy_words + 3) / 4;          // the staging buffer is padded to 16 bytes
  for (int64_t i = (int64_t)blk * 256 + threadIdx.x; i < n16; i += (int64_t)a.copy_blocks * 256) dst[i] = src[i];
}

// Inverse of append for a list of token slots: pool -> contiguous [n][Hkv][row].
__global__ void gather_kernel(GatherArgs a, uint8_t* k_out, uint8_t* v_out) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)a.n_tokens * a.Hkv * 32;
  if (tid >= total) return;
  const int c = tid & 15;
  const int kv = (tid >> 4) & 1;
  const int64_t th = tid >> 5;
  const int g = (int)(th % a.Hkv);
  const int64_t t = th / a.Hkv;
  const int slot = a.slots[t];
  const int page = slot / kP, ts = slot % kP;
  const uint8_t* src = a.pool + (int64_t)page * a.page_bytes + (int64_t)g * kSlab + kv * kBlk +
                       (c >> 3) * (kP * kHalfBytes) + ts * kHalfBytes + (c & 7) * 16;
  uint8_t* dst = (kv ? v_out : k_out) + th * kRowBytes + c * 16;
  *(uint4*)dst = *(const uint4*)src;
}

// extract / merge (paper section 4.2): K and V rows of whole tokens copied from one slot of the
// pool to another, bit for bit.  A token is Hkv * 4 pieces of 128 bytes (kv head, K/V, row half);
// a thread moves 16 bytes, eight neighbouring threads one piece, so every access is a full
// 128-byte line.  Sources are pages of existing files, destinations fresh pages: disjoint.
__global__ __launch_bounds__(256) void move_kernel(MoveArgs a) {
  const int per_tok = a.Hkv * 32;                                   // 16-byte chunks per token
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= a.n_tokens * per_tok) return;
  const int64_t t = tid / per_tok;
  const int x = (int)(tid % per_tok);
  const int s = a.moves[2 * t], d = a.moves[2 * t + 1];
  const int64_t in_page = (int64_t)(x >> 3) * (kP * kHalfBytes) + (x & 7) * 16;
  const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)(a.pool + (int64_t)(s / kP) * a.page_bytes + in_page + (s % kP) * kHalfBytes));
  *(u32x4_t*)(a.pool + (int64_t)(d / kP) * a.page_bytes + in_page + (d % kP) * kHalfBytes) = v;
}

// offload / restore (paper section 4.3): whole pages between the pool and pinned host memory, over
// the host link.  Four workgroups per page, 16 bytes per thread and pass; the list (page id, host
// address) is read from pinned memory by every workgroup for itself.
constexpr int kSwapSplit = 4;
__global__ __launch_bounds__(256) void swap_kernel(SwapArgs a) {
  const int e = blockIdx.x / kSwapSplit, part = blockIdx.x % kSwapSplit;
  const int64_t page = (int64_t)a.list[2 * e];
  uint8_t* host = (uint8_t*)a.list[2 * e + 1] + a.host_offset;
  uint8_t* dev = a.pool + page * a.page_bytes;
  const int64_t n16 = a.page_bytes / 16, per = (n16 + kSwapSplit - 1) / kSwapSplit;
  const int64_t lo = part * per, hi = min(n16, lo + per);
  const u32x4_t* src = (const u32x4_t*)(a.to_host ? dev : host);
  u32x4_t* dst = (u32x4_t*)(a.to_host ? host : dev);
  for (int64_t i = lo + threadIdx.x; i < hi; i += 4 * 256) {      // four loads in flight per thread
    u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < hi) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < hi) dst[i + u * 256] = v[u];
  }
}

// ---------------------------------------------------------------------------------------
// Calibration: streaming read (reduced so that the loads are live) and plain copy.
// ---------------------------------------------------------------------------------------
// Read: every wave streams its own contiguous span with nontemporal 16-byte loads, 16 KiB in
// flight per wave (the access pattern that reads fastest on this part).
__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4_t* __restrict__ src, int64_t n16, unsigned long long* out) {
  constexpr int U = 16;
  uint32_t acc = 0;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  const int64_t per = n16 / nwaves / (64 * U) * (64 * U);
  const u32x4_t* p = src + wave * per + lane;
  for (int64_t k = 0; k < per; k += 64 * U) {
    u32x4_t a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(p + k + u * 64);
#pragma unroll
    for (int u = 0; u < U; ++u) acc += a[u].x ^ a[u].y ^ a[u].z ^ a[u].w;
  }
  // the tail that does not divide evenly (none when bytes is a multiple of grid * 64 KiB)
  for (int64_t i = nwaves * per + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x) {
    u32x4_t a0 = src[i];
    acc += a0.x ^ a0.y ^ a0.z ^ a0.w;
  }
  if (acc == 0x9e3779b9u) atomicAdd(out, 1ull);      // practically never: keeps the loads alive
}
__global__ __launch_bounds__(256) void calib_copy_kernel(uint4* dst, const uint4* src, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Matrix-core rate that this part sustains: every wavefront (8 per workgroup, two per SIMD, as in the
// tile kernel) issues 16 independent-enough 32x32x16 bf16 MFMAs per iteration on four accumulators,
// operands in registers, nothing else in the loop.  flops = blocks * 8 * iters * 16 * 32768.
__global__ __launch_bounds__(512, 1) void calib_mfma_kernel(float* out, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8_t x[4], y[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // values of mixed sign and exponent, different in every lane and register
      const uint32_t hsh = (uint32_t)(threadIdx.x * 8 + e + 131 * i + 977 * blockIdx.x) * 2654435761u;
      x[i][e] = (__bf16)(((int)(hsh >> 20) - 2048) * (1.0f / 2048.0f));
      y[i][e] = (__bf16)(((int)((hsh >> 8) & 4095) - 2048) * (1.0f / 2048.0f));
    }
  f32x16_t acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[(i + r) & 3], y[i], acc[i], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) sum += acc[i][v];
  out[(int64_t)blockIdx.x * 512 + threadIdx.x] = sum + (float)lane;
}

template <typename E>
hipError_t launch_attn_g(const DecodeArgs& da, const PrefillArgs& pa, int decode_mode, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const int G = da.Hq / da.Hkv;
  // With events: they are attached to the dispatches themselves (start of the first kernel of the
  // attention launch, end of the last), so the interval holds kernel time and nothing else.
  auto launch = [&](auto kernel, dim3 g, dim3 b, hipEvent_t s, hipEvent_t e, auto... args) {
    if (s || e) hipExtLaunchKernelGGL(kernel, g, b, 0, st, s, e, 0, args...);
    else hipLaunchKernelGGL(kernel, g, b, 0, st, args...);
  };
  // decode ranges: matrix cores (mode 1), the two-wavefront VALU kernel for 8 heads (mode 2), or the
  // VALU kernel fused into the tile launch (mode 0)
  const int mode = (E::kDimsPerChunk == 8 && decode_mode == 1) ? 1 : (G == 8 ? 2 : 0);
  PrefillArgs ps = pa;
  ps.tile_first = 0;
  const int tile_blocks = ps.n_tiles > 0 ? ps.tile_blocks : 0;
  // eight-wavefront workgroups when the tiles have 256 query rows (and no tile is there: four)
  const int tw = (ps.n_tiles > 0 && ps.tile_rows == 256) ? 8 : 4;
  // every tile a shared-prefix tile with at most 64 live rows: the kernel that splits them by key block
  const bool split_tiles = E::kDimsPerChunk == 8 && tw == 4 && ps.n_tiles > 0 && ps.small_shared_only != 0;
  // mode 0: one workgroup per bin; the host made the bins for workgroups of this size
  if (mode == 0 && da.n_bins > 0 && (tile_blocks > 0 ? da.bin_waves != tw : (da.bin_waves != 4 && da.bin_waves != 8))) return hipErrorInvalidValue;
  const int decode_blocks = mode == 0 ? da.n_bins : 0;
  const int tile_groups = (tile_blocks + 7) / 8, decode_groups = (decode_blocks + 7) / 8;
  const dim3 grid((tile_groups + decode_groups) * 8), block(256), block8(512);
  // tiles and bins in one grid: the host's order table must cover it; tiles alone run in list order
  if (tile_groups > 0 && decode_groups > 0 && (!ps.group_map || ps.n_groups != tile_groups + decode_groups)) return hipErrorInvalidValue;
  if (decode_groups == 0) ps.group_map = nullptr;
  if (ps.n_tiles > 0 && ps.tile_rows != 128 && ps.tile_rows != 256) return hipErrorInvalidValue;
  const bool second = da.n_waves > 0 && mode != 0;          // decode ranges in a launch of their own
  const hipEvent_t e_first = second ? nullptr : ev1;
  const hipEvent_t s_second = grid.x > 0 ? nullptr : ev0;
#define SYM_ATTN_CASE(GG) \
  case GG: \
    if (tw == 8) launch(attn_kernel<E, GG, 8>, grid, block8, ev0, e_first, da, ps); \
    else if (split_tiles) launch(attn_kernel<E, GG, 4, true>, grid, block, ev0, e_first, da, ps); \
    else launch(attn_kernel<E, GG, 4>, grid, block, ev0, e_first, da, ps); \
    break;
  if (tile_blocks == 0 && mode == 0 && da.n_bins > 0) {      // plain decode: the lean kernel
    const dim3 dgrid(da.n_bins), dblock(64 * da.bin_waves);
#define SYM_DECODE_CASE(GG) \
  case GG: \
    if (da.bin_waves == 8) launch(decode_only_kernel<E, GG, 8>, dgrid, dblock, ev0, ev1, da); \
    else launch(decode_only_kernel<E, GG, 4>, dgrid, dblock, ev0, ev1, da); \
    break;
    switch (G) {
      SYM_DECODE_CASE(1) SYM_DECODE_CASE(2) SYM_DECODE_CASE(4)
      default: return hipErrorInvalidValue;
    }
#undef SYM_DECODE_CASE
    return hipGetLastError();
  }
  if (grid.x > 0) switch (G) {
    SYM_ATTN_CASE(1) SYM_ATTN_CASE(2) SYM_ATTN_CASE(4) SYM_ATTN_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef SYM_ATTN_CASE
  if (da.n_waves > 0 && mode == 2) launch(decode_pair_kernel<E>, dim3(da.n_waves), dim3(128), s_second, ev1, da);
  if (da.n_waves > 0 && mode == 1) {
    const dim3 dgrid((da.n_waves + kWavesPerBlock - 1) / kWavesPerBlock);
    switch (G) {
      case 1: launch(decode_mfma_kernel<1>, dgrid, block, s_second, ev1, da); break;
      case 2: launch(decode_mfma_kernel<2>, dgrid, block, s_second, ev1, da); break;
      case 4: launch(decode_mfma_kernel<4>, dgrid, block, s_second, ev1, da); break;
      case 8: launch(decode_mfma_kernel<8>, dgrid, block, s_second, ev1, da); break;
      default: return hipErrorInvalidValue;
    }
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Scratch memory of the entry point that allocates nothing (sym_pred_batch_static): descriptor
// words + partial results live in this file-scope array instead of the caller's workspace.
// Every GPU the library runs on holds its own copy at its own address, until the process ends;
// host code never uses the array's name as an address: it asks the runtime once per device for
// the address and passes that to the kernels like any other workspace.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

}  // namespace

hipError_t static_scratch_address(int device, uint8_t** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static uint8_t* addr[kMaxDevices] = {};
  if (device < 0 || device >= kMaxDevices || !ptr) return hipErrorInvalidValue;
  std::lock_guard<std::mutex> lk(mu);
  if (!addr[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device && (e = hipSetDevice(device)) != hipSuccess) return e;
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (cur != device) (void)hipSetDevice(cur);
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[device] = (uint8_t*)p;
  }
  *ptr = addr[device];
  return hipSuccess;
}

hipError_t launch_attn(const DecodeArgs& da, const PrefillArgs& pa, int dtype, int decode_mode, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (da.n_waves <= 0 && pa.n_tiles <= 0) return hipSuccess;
  if (dtype == 0) return pa.n_tiles > 0 ? hipErrorInvalidValue : launch_attn_g<ElemF32>(da, pa, 0, st, ev0, ev1);
  return launch_attn_g<ElemBF16>(da, pa, decode_mode, st, ev0, ev1);
}

hipError_t launch_merge(const MergeArgs& a, int G, int D, hipStream_t st) {
  if (a.n_items <= 0) return hipSuccess;
  const dim3 grid((a.n_items + kWavesPerBlock - 1) / kWavesPerBlock), block(kWavesPerBlock * 64);
#define SYM_MERGE_CASE(GG, DD) \
  if (G == GG && D == DD) { hipLaunchKernelGGL((merge_kernel<GG, DD>), grid, block, 0, st, a); return hipGetLastError(); }
  SYM_MERGE_CASE(1, 64) SYM_MERGE_CASE(2, 64) SYM_MERGE_CASE(4, 64) SYM_MERGE_CASE(8, 64)
  SYM_MERGE_CASE(1, 128) SYM_MERGE_CASE(2, 128) SYM_MERGE_CASE(4, 128) SYM_MERGE_CASE(8, 128)
#undef SYM_MERGE_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_prologue(PrologueArgs a, hipStream_t st) {
  const int64_t total = (int64_t)a.n_tokens * a.Hkv * 32;
  a.append_blocks = (int32_t)((total + 255) / 256);
  a.copy_blocks = a.copy_words > 0 ? (int32_t)std::min<int64_t>(((a.copy_words + 3) / 4 + 255) / 256, 256) : 0;   // >= 1: also for one, two or three words
  const int64_t blocks = (int64_t)a.append_blocks + a.n_cow + a.copy_blocks;
  if (blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(prologue_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_gather(const GatherArgs& a, void* k_out, void* v_out, hipStream_t st) {
  if (a.n_tokens <= 0) return hipSuccess;
  const int64_t total = (int64_t)a.n_tokens * a.Hkv * 32;
  hipLaunchKernelGGL(gather_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, (uint8_t*)k_out, (uint8_t*)v_out);
  return hipGetLastError();
}

hipError_t launch_move(const MoveArgs& a, hipStream_t st) {
  if (a.n_tokens <= 0) return hipSuccess;
  const int64_t blocks = (a.n_tokens * a.Hkv * 32 + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(move_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_swap(const SwapArgs& a, hipStream_t st) {
  if (a.n_pages <= 0) return hipSuccess;
  hipLaunchKernelGGL(swap_kernel, dim3((unsigned)a.n_pages * kSwapSplit), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_calib_read(const void* src, int64_t bytes, void* out8, hipStream_t st) {
  hipLaunchKernelGGL(calib_read_kernel, dim3(256 * 4), dim3(256), 0, st, (const u32x4_t*)src, bytes / 16, (unsigned long long*)out8);
  return hipGetLastError();
}
hipError_t launch_calib_mfma(float* out, int blocks, int iters, hipStream_t st) {
  hipLaunchKernelGGL(calib_mfma_kernel, dim3(blocks), dim3(512), 0, st, out, iters);
  return hipGetLastError();
}
hipError_t launch_calib_copy(void* dst, const void* src, int64_t bytes, hipStream_t st) {
  hipLaunchKernelGGL(calib_copy_kernel, dim3(256 * 8), dim3(256), 0, st, (uint4*)dst, (const uint4*)src, bytes / 16);
  return hipGetLastError();
}

}  // namespace symkv
