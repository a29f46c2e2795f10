// Append + evict: writes the new K/V rows of one layer into the head-mixed cache.
//
// Full heads store position p at row p.  Compressed heads are a fixed-size store of
// `sink` never-evicted slots followed by a ring of `recent` slots (paper Sec. 4.3: fixed
// size circular buffer, sink + local; App. B: only the first-S and recent-R tokens are
// kept): position p < S lives in slot p, position p >= S in slot S + (p - S) mod R, where
// it overwrites position p - R.
//
// The kernel is destination driven: every thread owns 16-byte units of the store, asks
// "which appended position ends up in my slot?" (the largest one that maps to it), and
// copies that row only.  A multi-token append therefore writes survivors only and gives
// the same store as the same tokens appended one at a time, whatever the write order.
#include "rlkv_internal.h"

namespace rlkv {
namespace {

struct TileRange { int first, count; };

__device__ inline TileRange tiles_of(int slot_lo, int slot_hi /* exclusive */) {
  if (slot_hi <= slot_lo) return {0, 0};
  const int t0 = slot_lo / kTile, t1 = (slot_hi - 1) / kTile;
  return {t0, t1 - t0 + 1};
}

// Appended position that ends in `slot` after the append, or -1 if the slot is untouched.
__device__ inline int source_position(bool full, int slot, int len_old, int len_new, int S, int R) {
  int p;
  if (full || slot < S) {
    p = slot;
  } else {
    const int r = slot - S;
    if (r >= R) return -1;                       // padding slot behind the ring
    const int last = len_new - 1 - S;            // ring index space of the newest position
    if (last < r) return -1;
    p = S + r + R * ((last - r) / R);            // largest p < len_new with (p - S) % R == r
  }
  return (p >= len_old && p < len_new) ? p : -1;
}

__device__ inline void len_in_out_both(const DeviceView& dv, int layer, int b, int len_new) {
  len_of(dv, 0, layer)[b] = len_new;
  len_of(dv, 1, layer)[b] = len_new;
}

template <int KERNEL, typename T>
__global__ __launch_bounds__(kBlock) void append_kernel(DeviceView dv, int layer, const int32_t* __restrict__ len_in,
                                                        int32_t* __restrict__ len_out, const T* __restrict__ k_new,
                                                        const T* __restrict__ v_new, int n_uniform,
                                                        int stride_tokens, int ragged, int from_list) {
  const int pair = blockIdx.y;
  const int b = pair / dv.n_kv_heads, h = pair % dv.n_kv_heads;
  const int job = blockIdx.x;
  const int S = dv.sink, R = dv.recent;
  // a uniform append skips inactive slots; a ragged append states its counts explicitly
  const int n_tok = ragged ? dv.append_cnt[b] : (dv.active[b] ? n_uniform : 0);
  int len_old;
  if (from_list) {
    // The append of a decode step whose launches carry no per-step argument (so that they can be recorded and
    // replayed): the length is the pair's length when the layer's work list was planned plus the list's growth
    // counter, which the merge kernel behind the attention kernel advances; nobody reads the length tables
    // here, so both copies take the new length.
    len_old = pair_desc_of(dv, layer)[pair].n_build + list_header(dv, layer)->grow;
    if (n_tok > 0 && job == 0 && h == 0 && threadIdx.x == 0) len_in_out_both(dv, layer, b, len_old + n_tok);
  } else {
    // lengths are double buffered: read the current copy, the block of (job 0, head 0) writes
    // the advanced length of its sequence to the other copy
    len_old = len_in[b];
    if (job == 0 && h == 0 && threadIdx.x == 0) len_out[b] = len_old + n_tok;
    // a uniform append keeps the layer's work list valid: every active sequence has grown by the same count
    if (!ragged && job == 0 && pair == 0 && threadIdx.x == 0) list_header(dv, layer)->grow += n_uniform;
  }
  const int len_new = len_old + n_tok;
  const bool full = dv.full_mask[layer * dv.n_kv_heads + h] != 0;

  int tile = -1;
  if (n_tok > 0) {
    if (full) {
      const TileRange t = tiles_of(len_old, len_new);
      if (job < t.count) tile = t.first + job;
    } else {
      // up to three slot ranges change: new sinks, and the ring range (which may wrap)
      const TileRange ta = tiles_of(len_old < S ? len_old : S, len_new < S ? len_new : S);
      const int p0 = len_old > S ? len_old : S;
      const int c = len_new - p0;                 // positions that go to the ring
      TileRange tb = {0, 0}, tc = {0, 0};
      if (c >= R) {
        tb = tiles_of(S, S + R);
      } else if (c > 0) {
        const int r0 = (p0 - S) % R;
        const int r1 = r0 + c;
        tb = tiles_of(S + r0, S + (r1 < R ? r1 : R));
        if (r1 > R) tc = tiles_of(S, S + r1 - R);
      }
      int j = job;
      if (j < ta.count) tile = ta.first + j;
      else if ((j -= ta.count) < tb.count) tile = tb.first + j;
      else if ((j -= tb.count) < tc.count) tile = tc.first + j;
    }
  }

  if (tile >= 0) {
    constexpr int kChunks = kHeadDim * sizeof(T) / 16;    // 16-byte chunks per row
    constexpr int kElems = 16 / sizeof(T);                // elements per chunk
    const int64_t koff = dv.store_off[((int64_t)layer * dv.batch + b) * dv.n_kv_heads + h];
    const int cap = full ? dv.cap_pad[b] : dv.window_pad;
    char* kst = dv.kv_base + koff;
    char* vst = kst + (int64_t)cap * dv.row_bytes;    // row-major layout only
    // tiled layout: start of this block's tile (through the block table for a paged full head)
    char* tile_base = kst + (int64_t)tile * kTileBytes;
    if (KERNEL == RLKV_KERNEL_MFMA && full && dv.page_shift >= 0)
      tile_base = kst + dv.block_table[(int64_t)b * dv.table_stride + (tile >> dv.page_shift)] * dv.page_bytes +
                  (int64_t)(tile & dv.page_mask) * kTileBytes;
    const int64_t src_head = ((int64_t)b * dv.n_kv_heads + h) * stride_tokens;
    int32_t* slot_pos = nullptr;
    if (!full) slot_pos = dv.slot_pos + dv.slotpos_off[layer * dv.n_kv_heads + h] + (int64_t)b * dv.window;

    // K rows (both layouts) and V rows (row-major layout): one 16-byte chunk per unit
    for (int u = threadIdx.x; u < kTile * kChunks; u += kBlock) {
      const int slot = tile * kTile + u / kChunks, chunk = u % kChunks;
      const int p = source_position(full, slot, len_old, len_new, S, R);
      if (p < 0) continue;
      const int64_t src = ((src_head + (p - len_old)) * kHeadDim + chunk * kElems) * sizeof(T);
      const uint4 kv = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(k_new) + src);
      if (KERNEL == RLKV_KERNEL_MFMA) {
        *reinterpret_cast<uint4*>(tile_base + tiled_k_offset(slot & (kTile - 1), chunk)) = kv;
      } else {
        const int64_t dst = (int64_t)slot * dv.row_bytes + chunk * 16;
        *reinterpret_cast<uint4*>(kst + dst) = kv;
        *reinterpret_cast<uint4*>(vst + dst) =
            *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(v_new) + src);
      }
      if (slot_pos && chunk == 0) slot_pos[slot] = p;
    }

    if (KERNEL == RLKV_KERNEL_MFMA) {
      // V, tiled layout: a unit is the 16 bytes that hold one d of eight slots.
      const uint16_t* vsrc = reinterpret_cast<const uint16_t*>(v_new);
      for (int u = threadIdx.x; u < 8 * 64; u += kBlock) {
        const int dblk = u >> 6, kb = (u >> 4) & 3, dn = u & 15;
        const int d = dblk * 16 + dn;
        uint16_t vals[8];
        unsigned have = 0;
        bool wide = false;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int slot = tile * kTile + (e >> 2) * 16 + kb * 4 + (e & 3);
          const int p = source_position(full, slot, len_old, len_new, S, R);
          if (p >= 0) {
            vals[e] = vsrc[(src_head + (p - len_old)) * kHeadDim + d];
            wide |= bf16_beyond_fp16(vals[e]);
            have |= 1u << e;
          } else {
            vals[e] = 0;
          }
        }
        if (wide) dv.v_wide[layer] = 1;      // the prefill kernel takes this layer's V as bf16 from now on
        char* dst = tile_base + tiled_v_offset(kb * 4, d);   // e = 0 of this unit
        if (have == 0xffu) {
          uint4 w;
          w.x = vals[0] | ((uint32_t)vals[1] << 16);
          w.y = vals[2] | ((uint32_t)vals[3] << 16);
          w.z = vals[4] | ((uint32_t)vals[5] << 16);
          w.w = vals[6] | ((uint32_t)vals[7] << 16);
          *reinterpret_cast<uint4*>(dst) = w;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (have & (1u << e)) reinterpret_cast<uint16_t*>(dst)[e] = vals[e];
        }
      }
    }
  }

}

__global__ void reset_kernel(DeviceView dv, int seq, int64_t slot_pos_elems) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n_len = (int64_t)2 * dv.n_layers * dv.batch;     // both copies
  if (i < n_len) {
    if (seq < 0 || i % dv.batch == seq) dv.len[i] = 0;
  }
  if (seq < 0 && i < dv.n_layers) dv.v_wide[i] = 0;     // an empty cache holds no value beyond the fp16 range
  if (i < slot_pos_elems) {
    // slot_pos is [compressed (layer, head)][batch][window]
    const int b = (int)((i / dv.window) % dv.batch);
    if (seq < 0 || b == seq) dv.slot_pos[i] = -1;
  }
}

__global__ void table_update_kernel(DeviceView dv, TableUpdates up) {
  const int i = threadIdx.x;
  if (i < up.n) dv.block_table[up.index[i]] = up.value[i];
}

}  // namespace

hipError_t launch_table_update(const DeviceView& dv, const TableUpdates& up, hipStream_t stream) {
  if (up.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(table_update_kernel, dim3(1), dim3(kTableUpdateMax), 0, stream, dv, up);
  return hipGetLastError();
}

hipError_t launch_append(const DeviceView& dv, int layer, const int32_t* len_in, int32_t* len_out,
                         const void* k, const void* v, int n_tokens_uniform, int stride_tokens, bool ragged,
                         int max_tokens, hipStream_t stream, bool from_list) {
  // Tiles a pair can touch: a range of c >= 1 slots touches at most (c + 30) / 32 + 1 tiles;
  // a full head has one range, a compressed head up to three (new sinks, ring, wrapped
  // ring) whose sizes add up to at most max_tokens.  One token touches one tile.
  const int jobs = max_tokens <= 1 ? 1 : (max_tokens + 3 * (kTile - 2)) / kTile + 3;
  const dim3 grid(jobs, dv.n_pairs), block(kBlock);
  if (dv.dtype == RLKV_F32) {
    hipLaunchKernelGGL((append_kernel<RLKV_KERNEL_VALU, float>), grid, block, 0, stream, dv, layer,
                       len_in, len_out, (const float*)k, (const float*)v, n_tokens_uniform, stride_tokens, (int)ragged, (int)from_list);
  } else if (dv.kernel == RLKV_KERNEL_MFMA) {
    hipLaunchKernelGGL((append_kernel<RLKV_KERNEL_MFMA, uint16_t>), grid, block, 0, stream, dv, layer,
                       len_in, len_out, (const uint16_t*)k, (const uint16_t*)v, n_tokens_uniform, stride_tokens, (int)ragged, (int)from_list);
  } else {
    hipLaunchKernelGGL((append_kernel<RLKV_KERNEL_VALU, uint16_t>), grid, block, 0, stream, dv, layer,
                       len_in, len_out, (const uint16_t*)k, (const uint16_t*)v, n_tokens_uniform, stride_tokens, (int)ragged, (int)from_list);
  }
  return hipGetLastError();
}

hipError_t launch_reset(const DeviceView& dv, int seq, int64_t slot_pos_elems, hipStream_t stream) {
  int64_t n = (int64_t)2 * dv.n_layers * dv.batch;
  if (slot_pos_elems > n) n = slot_pos_elems;
  if (n == 0) return hipSuccess;
  const int block = 256;
  hipLaunchKernelGGL(reset_kernel, dim3((unsigned)((n + block - 1) / block)), dim3(block), 0, stream, dv, seq,
                     slot_pos_elems);
  return hipGetLastError();
}

}  // namespace rlkv
