// Internal definitions shared by the host API and the gfx950 kernels of librlkv.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "rlkv.h"

namespace rlkv {

constexpr int kTile = 32;          // tokens per scheduling tile (and per MFMA step)
constexpr int kHeadDim = 128;      // the only head_dim the kernels are written for
constexpr int kMaxGroup = 16;      // query heads per KV head
constexpr int kMaxWorkgroups = 2048;  // upper bound of the split-K grid (sizes the scratch)
constexpr int kBlock = 256;        // threads per workgroup (4 wavefronts)
constexpr int kRound = 4;          // tiles per scheduling unit: one tile for each wavefront of a workgroup
constexpr int kPairOverheadUnits = 1;  // units at the head of every pair that carry no tiles (a label for its start)
constexpr int kRoundCost = 2;          // cost model of the share partition, in half rounds: one round of tiles ...
constexpr int kPairStartCost = 3;      // ... and the start of a pair (pipeline restart on a new store, Q load,
                                       // merge, output write): about 1.5 rounds, from per-workgroup timestamps
constexpr int kWorklistSlack = 32; // tokens a work list stays valid for after it was built

// Work-list records, written by the host (share_plan.hip, ensure_worklist) and read by the attention and merge
// kernels with wave-uniform (scalar) loads.  A workgroup's record embeds the record of its
// first pair, so one load level separates the kernel start from the first K/V tile load.
// The list of a layer is one block of device memory, [ListHeader][WgDesc x n_wg][PairDesc x n_pairs], written by
// a single copy out of a pinned staging slot of the same layout.
struct ListHeader {      // 64 bytes
  int32_t grow;          // tokens every active sequence has gained since the list was planned.  The copy that
                         // brings a new list sets it to 0; the kernels that append advance it (the merge kernel
                         // behind a fused step by 1, a uniform multi-token append by its token count), so that a
                         // decode launch needs no per-step argument and a captured step can be replayed
  int32_t pad[15];
};
struct PairDesc {        // 40 bytes
  int64_t koff;          // byte offset of the pair's K store from kv_base
  int32_t cap;           // token capacity of the store (the V store starts cap rows later)
  int32_t n_build;       // cached tokens of the sequence when the list was built
  int32_t unit_start;    // first scheduling unit of the pair in the end-to-end numbering
  int32_t unit_end;      // one past its last unit.  The first kPairOverheadUnits units of a pair hold
                         // no tiles; every later unit is kRound consecutive tiles of its store
  int32_t wg_first;      // first workgroup that holds units of the pair; its partial slots are wg + pair index
  int32_t full;          // 1 = full head, 0 = compressed
  float gate;            // Eq. 1 gate of a full head: out = gate * full + (1 - gate) * local; 1 = plain
  int32_t n_seg;         // workgroups that hold units of the pair (wg_first .. wg_first + n_seg - 1)
};
struct WgDesc {          // 56 bytes
  int32_t first_pair;    // pair that holds the workgroup's first tile
  int32_t u_begin, u_end;  // the workgroup's share of units [u_begin, u_end); empty if u_begin >= u_end
  int32_t pad;
  PairDesc first;        // copy of pair_desc[first_pair]
};

// Everything a kernel needs to find its data; passed by value as a kernel argument.
struct DeviceView {
  int32_t n_layers, n_q_heads, n_kv_heads, group, batch;
  int32_t sink, recent, window;   // window = sink + recent
  int32_t window_pad;             // window rounded up to a whole tile
  int32_t dtype, kernel;
  int32_t row_bytes;              // head_dim * element size
  int32_t n_pairs;                // batch * n_kv_heads
  int32_t n_wg;                   // grid size of the split-K kernel

  const uint8_t* full_mask;       // [n_layers][n_kv_heads]
  uint8_t* active;                // [batch] 1 = the slot takes part in uniform appends and in decode
  float* gate;                    // [n_layers][n_kv_heads] Eq. 1 gates (1 = plain full attention)
  const int64_t* store_off;       // [n_layers][batch][n_kv_heads] byte offset of the K store
  const int32_t* cap_pad;         // [batch] padded token capacity of a full store
  const int64_t* slotpos_off;     // [n_layers][n_kv_heads] element offset into slot_pos, -1 = full
  int32_t* len;                   // [2][n_layers][batch] cached tokens, double buffered: a kernel that
                                  // appends reads one copy and writes the other, so no workgroup
                                  // can see a length another one has already advanced
  int32_t* slot_pos;              // per compressed (layer, head): [batch][window]
  int32_t* v_wide;                // [n_layers] 1 once a V value of magnitude >= 65536 (or Inf / NaN) has gone into the
                                  // layer's stores or staging (tiled layout): prefill then takes V as bf16
  int32_t* append_cnt;            // [2][batch] staging: per-sequence token counts; sequence order of a prefill
  char* list_base;                // [n_layers] work-list blocks of list_stride bytes (see ListHeader)
  int64_t list_stride;
  int32_t list_pair_off;          // byte offset of the PairDesc array inside a block
  float* part_o;                  // [n_wg + n_pairs][group][head_dim]
  float* part_m;                  // [n_wg + n_pairs][group]  (log2 domain maxima)
  float* part_l;                  // [n_wg + n_pairs][group]
  int64_t part_set_o, part_set_ml; // element offsets of the second partial set (local attention of gated heads)
  char* kv_base;                  // start of the K/V stores

  // Paged full heads (Sec. 4.3).  store_off of a full head is then the offset of its pool, the
  // same for every sequence, and tile t of sequence b lives at
  //   pool + block_table[b][t >> page_shift] * page_bytes + (t & page_mask) * kTileBytes.
  int32_t page_shift;             // log2(tiles per page); -1 = contiguous stores
  int32_t page_mask;              // tiles per page - 1
  int32_t table_stride;           // block-table entries per sequence
  int64_t page_bytes;             // bytes of one page (K and V)
  int32_t* block_table;           // [batch][table_stride] page index, shared by all layers and heads
};

// Block-table entries that change, passed by value to a one-block kernel (no host-to-device copy
// on the append path).
constexpr int kTableUpdateMax = 96;
struct TableUpdates {
  int32_t n;
  int32_t index[kTableUpdateMax];   // element index into block_table
  int32_t value[kTableUpdateMax];   // page
};

// ---- store addressing ------------------------------------------------------------
// Row-major layout (VALU kernel): row `slot` of K (or V) at slot * row_bytes.
//
// Tiled layout (MFMA kernel, bf16): the store is cut into tiles so that lane l of a
// wavefront reading 16 bytes at tile_base + step * 1024 + l * 16 receives exactly its
// MFMA operand:
//   K, per 16 slots (4 KiB, two per tile):  [chunk = d / 8 : 16][slot % 16 : 16][d % 8 : 8]
//      -> step s in 0..3 covers chunks 4s..4s+3; lane l = (chunk % 4) * 16 + slot % 16
//         holds row slot%16, k-group chunk%4 of a 16x16x32 A operand.
//   V, per 32 slots (8 KiB):  [dblk = d / 16 : 8][kb : 4][d % 16 : 16][e : 8]
//      with slot % 32 = half * 16 + kb * 4 + r and e = half * 4 + r
//      -> step dblk; lane l = kb * 16 + d % 16 holds column d%16, k-group kb of a
//         16x16x32 B operand whose k index runs over the 32 slots of the tile in the
//         same order the score tile leaves them in the accumulator registers.
// K and V tiles of the same 32 slots sit next to each other (16 KiB: K then V), so the 16
// loads a wavefront issues per tile fall into one contiguous block.  Offsets are relative
// to the start of the pair's store.
constexpr int kTileBytes = 16384;
__host__ __device__ inline int64_t tiled_k_offset(int slot, int chunk) {
  return (int64_t)(slot >> 5) * kTileBytes + ((slot >> 4) & 1) * 4096 + chunk * 256 + (slot & 15) * 16;
}
__host__ __device__ inline int64_t tiled_v_offset(int slot, int d) {
  const int st = slot & 31;
  const int half = st >> 4, kb = (st & 15) >> 2, r = st & 3;
  return (int64_t)(slot >> 5) * kTileBytes + 8192 + (d >> 4) * 1024 + (kb * 16 + (d & 15)) * 16 + (half * 4 + r) * 2;
}

// bf16 bits whose value lies beyond the fp16 range (exponent field >= 127 + 16; Inf and NaN included)
__host__ __device__ inline bool bf16_beyond_fp16(uint32_t bits) { return (bits & 0x7f80u) >= 0x4780u; }

// The parts of a layer's work-list block.
__host__ __device__ inline ListHeader* list_header(const DeviceView& dv, int layer) {
  return reinterpret_cast<ListHeader*>(dv.list_base + layer * dv.list_stride);
}
__host__ __device__ inline WgDesc* wg_desc_of(const DeviceView& dv, int layer) {
  return reinterpret_cast<WgDesc*>(dv.list_base + layer * dv.list_stride + sizeof(ListHeader));
}
__host__ __device__ inline PairDesc* pair_desc_of(const DeviceView& dv, int layer) {
  return reinterpret_cast<PairDesc*>(dv.list_base + layer * dv.list_stride + dv.list_pair_off);
}

// Lengths of `layer` in copy `parity` (0 / 1).
__host__ __device__ inline int32_t* len_of(const DeviceView& dv, int parity, int layer) {
  return dv.len + ((int64_t)parity * dv.n_layers + layer) * dv.batch;
}

// ---- launchers (defined next to their kernels) -------------------------------------
// `len_in` is the current copy of the layer's lengths; kernels that append write the
// advanced lengths to `len_out` (the other copy).  A uniform append also adds its token count to the
// layer's ListHeader::grow.  `from_list` (a uniform append of one token, the first launch of a decode step that
// can be recorded): the lengths are taken from the layer's work list and its growth counter instead, both copies
// of the table take the new lengths, and the counter is left to the merge kernel of the step (advance = 1).
hipError_t launch_append(const DeviceView& dv, int layer, const int32_t* len_in, int32_t* len_out,
                         const void* k, const void* v, int n_tokens_uniform, int stride_tokens, bool ragged,
                         int max_tokens, hipStream_t stream, bool from_list = false);
hipError_t launch_reset(const DeviceView& dv, int seq, int64_t slot_pos_elems, hipStream_t stream);
hipError_t launch_table_update(const DeviceView& dv, const TableUpdates& up, hipStream_t stream);
// Host-side plan of the shares (share_plan.hip): rounds[p] = rounds of tiles of pair p (0 = none).
// Fills wg_begin[0 .. n_wg] (share w = units [wg_begin[w], wg_begin[w + 1])), seg_first[p] / seg_count[p]
// (the workgroups that hold units of pair p); returns the number of workgroups used.
int plan_shares(const int32_t* rounds, int n_pairs, int n_wg, int32_t* wg_begin, int32_t* seg_first,
                int32_t* seg_count);
// ev_start / ev_stop (both or neither): events that receive the kernel's own begin and end
// timestamps (the dispatch's completion signal), for the measurement aid.
// `gated`: some full head of the layer has a gate below 1 (two passes for those heads).
// `appended`: tokens appended by the step's own append launch that the growth counter does not count yet (0 or 1).
hipError_t launch_decode_valu(const DeviceView& dv, int layer, bool gated, const void* q, void* out,
                              float scale_log2, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop,
                              int appended = 0);
// k_new / v_new non-null: fused single-token append (rows [batch][n_kv_heads][1][head_dim]); the advanced
// lengths are written to both copies of the length table, and the merge kernel that follows must be launched
// with advance = 1.
hipError_t launch_decode_mfma(const DeviceView& dv, int layer, bool gated,
                              const void* q, void* out, float scale_log2, const void* k_new, const void* v_new,
                              hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);
// merge_words (host, [n_pairs], optional): per pair (first partial slot << 12) | partials, as planned for the
// work list now on the device; with it and at most kMergeArgPairs pairs the merge kernel takes these from its
// arguments instead of from the pair records (not for a layer with gates: their records carry more).
// advance: tokens to add to the layer's ListHeader::grow (1 behind a fused append + decode launch).
constexpr int kMergeArgPairs = 512;
hipError_t launch_combine(const DeviceView& dv, int layer, void* out, hipStream_t stream, int advance,
                          const void* v_new = nullptr, const uint32_t* merge_words = nullptr);
// Prefill attention of one chunk (counts in dv.append_cnt, lengths before the chunk in len_in):
// stages the chunk's K/V as tiles in `staging` (staging_tiles tiles per pair), then attends.
// `gated`: the kernel form with one column group of queries per wavefront, the only one that can blend
// (Eq. 1: causal and local attention of a full head with a gate below 1).
// `n_split` > 1 (other form only): the unmasked tiles of every full head's workgroup are divided among
// n_split workgroups, which leave their shares in `split_out` (kPrefillSplitSlotBytes per divided
// workgroup; at most kPrefillSplitSlots: split_rows (the grid's first rows: full heads of sequences
// that have a chunk) x blocks x n_split) for a merge kernel that follows.
constexpr int kPrefillSplitSlots = 1024;
constexpr int kPrefillArgHeads = 64;      // KV heads of a layer whose class lists travel in the prefill kernels' arguments
constexpr size_t kPrefillSplitSlotBytes = 256 * (size_t)(kHeadDim + 2) * sizeof(float);
hipError_t launch_prefill_mfma(const DeviceView& dv, int layer, bool gated, const int32_t* len_in, const void* q,
                               const void* k, const void* v, void* out, int stride_tokens, int max_tokens,
                               float scale_log2, char* staging, int staging_tiles, int n_split, float* split_out,
                               int split_rows, int dealt_rows,
                               const uint8_t* mask_row /* host, [n_kv_heads]: the layer's mask */,
                               hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

// Measurement aid: reads `bytes` (whole 16 KiB blocks) of `buf` once with `workgroups` workgroups.
hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, hipStream_t stream);

// ---- small device helpers -----------------------------------------------------------
__device__ inline float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace rlkv
