// Prefill (chunked prefill) attention for mixed heads, MFMA variant (tiled bf16 stores).
//
// One chunk of T new positions per sequence attends over the positions already cached plus the
// chunk itself, under the two masks of paper Sec. 3.1 (App. B: prefilling applies them as mask
// matrices): a full head uses the causal mask, j <= i; a compressed head the local mask,
// j <= i and (j < S or i - j < R).  Here nothing is materialised: a query block walks only the
// tiles its mask rows can touch and masks inside the tile.
//
// Keys and values come from two places, both in the tiled MFMA-operand layout:
//   - the store: positions before the chunk (all of them for a full head; for a compressed head
//     the sink slots and, while the chunk's first R queries still reach back, the ring slots,
//     whose positions are read from the slot table);
//   - a staging buffer holding the chunk's own K/V, tiled by stage_chunk_kernel.  A compressed
//     head's ring cannot hold a chunk longer than R, and early queries of the chunk need keys that
//     later ones evict, so the chunk is attended from the staging buffer and appended afterwards.
//
// Work split and the two loops of a wavefront: see the comment on prefill_mfma_kernel below.
// Scores use the same instruction and operand layouts as the decode kernel; a column of the score
// tile is a (position, head) pair instead of a head.  For the weights x V product the hot loop sends
// both operands to the matrix cores as fp16 (V converted on its way into LDS, exact for magnitudes in
// [2^-14, 65536), at most 2^-24 absolute below; tiles with larger values are taken as bf16); the
// general loop keeps the decode kernel's two-part bf16 weights.
#include <type_traits>

#include "mfma_tile.h"
#include "prefill_deal.h"

namespace rlkv {
namespace {


// Tiles re-read by many query blocks: ordinary (cached) loads.
__device__ __forceinline__ void load_tile_cached(TileRegs& r, const char* tile_base, int lane) {
  const char* kb = tile_base + lane * 16;
  const char* vb = kb + 8192;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int s = 0; s < 4; ++s) r.k[hf][s].u = *reinterpret_cast<const uint4*>(kb + hf * 4096 + s * 1024);
#pragma unroll
  for (int j = 0; j < 8; ++j) r.v[j].u = *reinterpret_cast<const uint4*>(vb + j * 1024);
}

// Scores of one 32-slot tile against one group's Q operands, unscaled.
__device__ __forceinline__ void raw_scores(const TileRegs& t, const Frag (&qb)[4], float (&raw)[8]) {
  floatx4 s0 = floatx4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[0][s].v, qb[s].v, s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[1][s].v, qb[s].v, s1, 0, 0, 0);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) raw[e] = e < 4 ? s0[e] : s1[e - 4];
}

// Eight fp32 weights as two bf16 operands: the head keeps the top 16 bits of each weight
// (truncated, one byte permute per pair), the remainder p - head is exact in fp32 and is rounded
// to bf16; together they carry ~16 mantissa bits.
__device__ __forceinline__ void split_weights(const float (&p)[8], Frag& hi, Frag& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t b0 = __float_as_uint(p[2 * k]), b1 = __float_as_uint(p[2 * k + 1]);
    h[k] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);            // {b1.hi16, b0.hi16}
    const float r0 = p[2 * k] - __uint_as_float(b0 & 0xffff0000u);
    const float r1 = p[2 * k + 1] - __uint_as_float(b1 & 0xffff0000u);
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 r = {(__bf16)r0, (__bf16)r1};
    l[k] = *reinterpret_cast<uint32_t*>(&r);
  }
  hi.u = make_uint4(h[0], h[1], h[2], h[3]);
  lo.u = make_uint4(l[0], l[1], l[2], l[3]);
}

// The weights of the hot loop go to the matrix cores as one fp16 operand (11 significant bits, against
// 8 for bf16), which needs V in fp16 as well: the threads that move a tile into LDS convert its V
// half on the way.  A bf16 value converts exactly while its magnitude lies in [2^-14, 65536); smaller
// ones lose at most 2^-24 absolute.  Larger ones do not occur here: the kernels that write V into the
// stores and the staging buffer raise the layer's v_wide flag when they see one, and the hot loop
// then takes V as stored.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t x) {
  const auto h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(x << 16), __uint_as_float(x & 0xffff0000u));
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ uint4 bf16x8_to_f16x8(uint4 w) {
  return make_uint4(bf16x2_to_f16x2(w.x), bf16x2_to_f16x2(w.y), bf16x2_to_f16x2(w.z), bf16x2_to_f16x2(w.w));
}

// Eight fp32 weights (at most 2^(kSlack + kWeightShift) < 65504) as one fp16 operand, truncated: the
// normaliser is accumulated from the same operand, so the common part of the truncation cancels.
__device__ __forceinline__ void half_weights(const float (&p)[8], Frag& ph) {
  uint32_t h[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) h[k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[2 * k], p[2 * k + 1]));
  ph.u = make_uint4(h[0], h[1], h[2], h[3]);
}

// All weights of this kernel carry a factor 2^kWeightShift (it cancels between the accumulators and
// the normaliser): it keeps fp16 weights as small as 2^-30 of the reference maximum representable.
constexpr float kWeightShift = 6.f;

// Online-softmax state of one 16-column group.  In the general loop the weights go to the matrix
// cores as in the decode kernel, a bf16 head plus a bf16 remainder (~16 mantissa bits; a single
// bf16 weight measurably misses the 1e-2 bar).  This kernel is bound by its vector instruction count, so the
// normaliser is accumulated by the matrix cores too, from the same two parts against a tile of
// ones: it then arrives in the accumulator layout and needs no cross-lane sums.
struct GroupState {
  float m;          // reference maximum of column lane%16 (log2 domain; same in all four k-groups)
  float ref;        // what the exponent subtracts: m (0 while m is -inf) minus kWeightShift
  float thr;        // a raw score above this makes the reference move: (m + slack) / scale
  floatx4 l;        // normaliser of columns 4*(lane/16) + r (accumulator layout)
  floatx4 o[8];     // O[column 4*(lane/16) + r][d = 16*j + lane%16]
};

// This file is compiled with -fno-honor-nans: fmaxf would otherwise first quiet a possible signalling
// NaN in every operand (three instructions per maximum); scores are never NaN here, and -inf (a masked
// score, an empty running maximum) is still honoured.
__device__ __forceinline__ float max2(float a, float b) { return fmaxf(a, b); }
__device__ __forceinline__ float max8(const float (&v)[8]) {
  return fmaxf(fmaxf(fmaxf(fmaxf(v[0], v[1]), v[2]), fmaxf(fmaxf(v[3], v[4]), v[5])), fmaxf(v[6], v[7]));
}

// The reference maximum only moves when a score outgrows it by more than 2^kSlack; what depends on it
// is kept beside it, so that a tile costs one comparison and no arithmetic on the reference.
constexpr float kSlack = 8.f;
__device__ __forceinline__ void set_reference(GroupState& st, float m_new, float scale) {
  st.m = m_new;
  st.ref = (m_new == -INFINITY ? 0.f : m_new) - kWeightShift;
  st.thr = (m_new + kSlack) / scale;       // -inf while no key has been seen: any score moves it
}

// Maximum over the four lanes that hold the same column (lane, lane^16, lane^32, lane^48), with
// the gfx950 row swaps instead of LDS permutes.
__device__ __forceinline__ float column_max(float v) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  u32x2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = max2(__uint_as_float(a[0]), __uint_as_float(a[1]));
  u32x2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return max2(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// Folds the masked raw scores `sc` of one tile (-inf = does not count) into the group's state;
// `scale` (> 0, log2 domain) is applied inside the exponent's fused multiply-add.
__device__ __forceinline__ void group_update(const TileRegs& t, const float (&sc)[8], float scale, GroupState& st,
                                             int kb, const Frag& ones) {
  // The reference maximum only moves when some column's scores outgrow it by more than 2^kSlack:
  // until then the weights are simply larger than 1 (fp32 accumulators and the two-part bf16 split
  // are relative, so nothing is lost) and the accumulators need no rescaling.  Every lane holds its
  // column's reference, so the test needs the lane's own eight scores only; the column's maximum
  // (two cross-lane steps) is formed when the test fires.
  const float mx_lane = max8(sc);
  if (__any(mx_lane > st.thr)) {
    const float mx = column_max(mx_lane) * scale;
    const float m_new = fmaxf(st.m, mx);
    // a column that has seen no key yet still has a zero accumulator: factor 1
    const float alpha = st.m == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(st.m - m_new);
    set_reference(st, m_new, scale);
    if (__any(alpha != 1.f)) {
      // the accumulators hold columns 4*kb + r: fetch their factors from lanes 0..15
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float a = __shfl(alpha, kb * 4 + r);
        st.l[r] *= a;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.o[j][r] *= a;
      }
    }
  }
  float p[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e], scale, -st.ref));
  Frag phi, plo;
  split_weights(p, phi, plo);
  st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi.v, ones.v, st.l, 0, 0, 0);
  st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo.v, ones.v, st.l, 0, 0, 0);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    st.o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi.v, t.v[j].v, st.o[j], 0, 0, 0);
    st.o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo.v, t.v[j].v, st.o[j], 0, 0, 0);
  }
}

// Copies the chunk's K/V rows (row-major [batch][n_kv_heads][stride][128]) into tiles of the MFMA
// layout: staging tile t of a pair holds chunk rows 32 t .. 32 t + 31; rows past the sequence's
// count are written as zeros, so a staged tile never holds stale bits.
__global__ __launch_bounds__(kBlock) void stage_chunk_kernel(DeviceView dv, int layer, const uint16_t* __restrict__ k_new,
                                                             const uint16_t* __restrict__ v_new, int stride_tokens,
                                                             char* __restrict__ staging, int staging_tiles) {
  const int pair = blockIdx.y, tile = blockIdx.x;
  const int b = pair / dv.n_kv_heads;
  const int t = dv.append_cnt[b];
  if (tile * kTile >= t) return;
  char* tile_base = staging + ((int64_t)pair * staging_tiles + tile) * kTileBytes;
  const int64_t src_head = (int64_t)pair * stride_tokens;
  for (int u = threadIdx.x; u < kTile * 16; u += kBlock) {          // K: one 16-byte chunk of a row per unit
    const int slot = u >> 4, chunk = u & 15;
    const int row = tile * kTile + slot;
    uint4 kv = make_uint4(0, 0, 0, 0);
    if (row < t) kv = *reinterpret_cast<const uint4*>(k_new + (src_head + row) * kHeadDim + chunk * 8);
    *reinterpret_cast<uint4*>(tile_base + tiled_k_offset(slot, chunk)) = kv;
  }
  for (int u = threadIdx.x; u < 8 * 64; u += kBlock) {              // V: one d of eight slots per unit
    const int dblk = u >> 6, kb = (u >> 4) & 3, dn = u & 15;
    const int d = dblk * 16 + dn;
    uint32_t w[4];
    bool wide = false;
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      uint32_t pack = 0;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int e = 2 * e2 + k;
        const int row = tile * kTile + (e >> 2) * 16 + kb * 4 + (e & 3);
        const uint32_t val = row < t ? v_new[(src_head + row) * kHeadDim + d] : 0u;
        wide |= bf16_beyond_fp16(val);
        pack |= val << (16 * k);
      }
      w[e2] = pack;
    }
    if (wide) dv.v_wide[layer] = 1;        // seen by the attention kernel that follows on the stream
    *reinterpret_cast<uint4*>(tile_base + tiled_v_offset(kb * 4, d)) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Grid row y of the prefill kernels -> (sequence, KV head): the pairs of full heads first, then those of
// compressed heads, each class by descending sequence length (the host-sorted order behind the counts).
// The heads of each class come with the kernel arguments (heads.n_full >= 0; one load instead of two loops of
// dependent loads over the layer's mask at the start of every workgroup), unless the layer has more heads
// than fit there.
struct PrefillHeads {
  int32_t n_full;                          // full heads of the layer; -1: not given, read the mask
  int32_t heavy_rows;                      // leading grid rows that are full heads of sequences with a chunk
  int32_t dealt_rows;                      // of those, the leading ones that go one row per XCD (see prefill_deal)
  int32_t head[2][kPrefillArgHeads];       // [0]: the full heads in ascending order, [1]: the compressed ones
};
__device__ __forceinline__ void pair_of_grid_row(const DeviceView& dv, int layer, int y, const PrefillHeads& heads,
                                                 int& b, int& h, bool& full) {
  if (heads.n_full >= 0) {
    const int n_full_pairs = dv.batch * heads.n_full;
    full = y < n_full_pairs;
    const int per_seq = full ? heads.n_full : dv.n_kv_heads - heads.n_full;
    const int yy = full ? y : y - n_full_pairs;
    b = dv.append_cnt[dv.batch + yy / per_seq];
    h = heads.head[full ? 0 : 1][yy % per_seq];
    return;
  }
  int n_full_heads = 0;
  for (int i = 0; i < dv.n_kv_heads; ++i) n_full_heads += dv.full_mask[layer * dv.n_kv_heads + i] ? 1 : 0;
  const int n_full_pairs = dv.batch * n_full_heads;
  const bool want_full = y < n_full_pairs;
  const int per_seq = want_full ? n_full_heads : dv.n_kv_heads - n_full_heads;
  const int yy = want_full ? y : y - n_full_pairs;
  b = dv.append_cnt[dv.batch + yy / per_seq];
  h = 0;
  for (int i = 0, k = yy % per_seq; i < dv.n_kv_heads; ++i) {
    if ((dv.full_mask[layer * dv.n_kv_heads + i] != 0) == want_full) {
      if (k == 0) { h = i; break; }
      --k;
    }
  }
  full = want_full;
}

// Split prefill (few long workgroups: one or two sequences, few full heads): the unmasked tiles of a
// full head's workgroup are divided among gridDim.z workgroups, each of which leaves its 256 columns'
// unnormalised accumulators, normalisers and reference maxima in a slot of scratch memory
// ([256][128] O, then [256] m, then [256] l, fp32); prefill_merge_kernel combines them.
constexpr int kSplitCols = 256;
constexpr int kSplitSlotFloats = kSplitCols * (kHeadDim + 2);
constexpr int kMergeColsPerGroup = 8;      // columns a workgroup of the merge kernel combines

constexpr int kPrefillWaves = 8;                 // wavefronts per workgroup: two per SIMD
constexpr int kPrefillBlock = kPrefillWaves * 64;



// A workgroup = one (sequence, KV head) pair x 8 wavefronts, two per SIMD so that one wavefront's
// vector work (exponentials, weight split, maxima) runs beside the other's matrix work.  Each
// wavefront owns NG 16-column groups of the workgroup's (position, head) columns, flattened
// position-major across the whole workgroup.
//
// GATED (some full head of the layer has an Eq. 1 gate below 1): a wavefront owns one column group
// instead of two, and its second accumulator set holds the local attention (sink + recent
// positions) of the same columns; the scores of a tile are computed once for both, and the output
// is gate * causal + (1 - gate) * local.
//
// Two loops.  The hot one takes the tiles that every query of the workgroup sees whole: those of a
// full head that lie wholly before the workgroup's first query (nearly all of a prefill's work),
// and for a compressed head its complete sink tiles and the chunk tiles before the first query
// that no query's recent band has left yet.  The eight wavefronts walk them together, every tile is
// fetched from memory once per workgroup into LDS (one barrier per tile; K straight into LDS, V
// through registers) and read from there as MFMA operands; no masks.  The general one takes everything else (partly filled
// tiles, a compressed head's ring, the causal diagonal and the band's edge, the sink and band tiles
// of a gated head), each wavefront on its own, with per-slot positions and masks.
template <bool PAGED, bool GATED>
__global__ __launch_bounds__(kPrefillBlock) void prefill_mfma_kernel(DeviceView dv, int layer,
                                                                     const int32_t* __restrict__ len_in,
                                                                     const uint16_t* __restrict__ q,
                                                                     uint16_t* __restrict__ out, int stride_tokens,
                                                                     float scale_log2,
                                                                     const char* __restrict__ staging,
                                                                     int staging_tiles, float* __restrict__ split_out,
                                                                     PrefillHeads heads) {
  // LDS: the K halves of four tiles (filled by loads that go from memory straight into LDS, two tiles ahead)
  // and the V halves of two (through registers: V is converted on the way).
  __shared__ uint4 sm_k[4][kTileBytes / 32];
  __shared__ uint4 sm_v[2][kTileBytes / 32];
  // Workgroups are handed out in grid order, and each XCD takes the rows dealt to it (prefill_deal) in
  // order: the long ones go first - the pairs of full heads before those of compressed heads, long
  // sequences before short ones, and within a pair the later query blocks (more keys under the
  // causal mask) before the earlier ones - so that the short ones fill the end.
  int b, h;
  bool full;
  int bx = blockIdx.x, by = blockIdx.y;
  if (gridDim.z == 1) prefill_deal((int)(blockIdx.x + gridDim.x * blockIdx.y), (int)gridDim.x, (int)gridDim.y, heads.dealt_rows,
                                    heads.heavy_rows, bx, by);   // (a divided launch keeps the plain order: its merge kernel indexes by it)
  pair_of_grid_row(dv, layer, by, heads, b, h, full);
  const int pair = b * dv.n_kv_heads + h;
  const int block_x = gridDim.x - 1 - bx;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int hd = lane & 15;     // score layout: column; operand layouts: row / column
  const int kb = lane >> 4;     // k-group of the operand layouts; slot quad of the score layout
  const int G = dv.group, S = dv.sink, R = dv.recent;
  constexpr int NG = GATED ? 1 : 2;                      // column groups of queries per wavefront
  constexpr int LOCAL = NG;                              // index of the first local accumulator set (GATED)
  constexpr int kWaveCols = 16 * NG;
  const int wg_positions = kPrefillWaves * kWaveCols / G;    // chunk positions per workgroup
  const int t = dv.append_cnt[b];          // chunk length of this sequence
  const int n_old = len_in[b];             // positions cached before the chunk
  const int c_wg = block_x * wg_positions; // the workgroup's first chunk index
  if (c_wg >= t) return;
  const int c_last = (c_wg + wg_positions < t ? c_wg + wg_positions : t) - 1;   // its last one
  // share z of Z of a divided workgroup; grid plane 0, handed out first, holds the last share, the longest one
  // (it also takes the masked tiles)
  const int Z = gridDim.z, z = Z - 1 - (int)blockIdx.z;
  if (!full && blockIdx.z > 0) return;       // a compressed head's workgroup is short: never divided
  const bool split = !GATED && full && Z > 1;
  const float gate = (GATED && full) ? dv.gate[layer * dv.n_kv_heads + h] : 1.f;
  const bool mix = GATED && full && gate < 1.f;          // this head blends causal and local attention

  // This wavefront's columns: kWaveCols of the workgroup's flattened (position, head) pairs.
  const int col0 = wave * kWaveCols;
  const int c0 = c_wg + col0 / G;                                        // first chunk index it touches
  const int c_hi_raw = c_wg + (col0 + kWaveCols - 1) / G;
  const int c_hi = c_hi_raw < c_last ? c_hi_raw : c_last;               // last one
  const bool busy = c0 <= c_last;                                        // it has at least one query
  Frag qb[NG][4];               // Q as the B operand of the score MFMA
  int qpos[NG];                 // absolute position of the lane's column, -1 = no such query
  int g_lo[NG], g_hi[NG];       // positions a group holds
  bool g_on[NG];
#pragma unroll
  for (int cg = 0; cg < NG; ++cg) {
    const int col = col0 + 16 * cg + hd;
    const int cl = col / G, hh = col - cl * G;
    const bool valid = c_wg + cl <= c_last;
    qpos[cg] = valid ? n_old + c_wg + cl : -1;
    const int64_t qrow = ((int64_t)b * dv.n_q_heads + h * G + hh) * stride_tokens + c_wg + cl;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint4 qv = make_uint4(0, 0, 0, 0);
      if (valid)
        qv = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(q) + (qrow * kHeadDim + s * 32 + kb * 8) * 2);
      qb[cg][s].u = qv;
    }
    const int cl_lo = (col0 + 16 * cg) / G, cl_hi = (col0 + 16 * cg + 15) / G;
    g_on[cg] = c_wg + cl_lo <= c_last;
    g_lo[cg] = n_old + c_wg + cl_lo;
    g_hi[cg] = n_old + (c_wg + cl_hi < c_last ? c_wg + cl_hi : c_last);
  }

  TileMap<PAGED> store;
  store.base = dv.kv_base + dv.store_off[((int64_t)layer * dv.batch + b) * dv.n_kv_heads + h];
  store.paged = PAGED && full;
  if (PAGED) {
    store.row = dv.block_table + (int64_t)b * dv.table_stride;
    store.page_bytes = dv.page_bytes;
    store.shift = dv.page_shift;
    store.mask = dv.page_mask;
    store.last = dv.table_stride - 1;
  }
  const char* stage = staging + (int64_t)pair * staging_tiles * kTileBytes;
  const int32_t* slot_pos = nullptr;
  if (!full) slot_pos = dv.slot_pos + dv.slotpos_off[layer * dv.n_kv_heads + h] + (int64_t)b * dv.window;

  const int n_st = full ? n_old : (n_old < dv.window ? n_old : dv.window);     // store slots that hold data
  const int sink_in_chunk = S - n_old;       // chunk indices below this are sink positions

  // Hot tiles (same for all wavefronts of the workgroup): tiles in which every slot counts for every
  // query of the workgroup.  Full head: the store's complete tiles and the staging tiles wholly before
  // the workgroup's first query.  Compressed head: the store's complete sink tiles, and the staging
  // tiles wholly before the first query that also lie wholly inside the recent band of the last one
  // (a chunk is usually longer than the band, so these are most of what such a head attends over).
  // A blending head also feeds its local accumulators from the tiles that hold sink positions or
  // reach into the recent band of that first query: those take the general loop.  (A softmax scale
  // that is not positive, unusual, takes the general loop throughout.)
  const bool hot = scale_log2 > 0.f;
  int hs_lo = 0, hs_hi = 0;                  // hot store tiles [hs_lo, hs_hi)
  int stg_lo = 0, stg_hi = 0;                // hot staging tiles [stg_lo, stg_hi)
  if (hot) {
    stg_hi = c_wg / kTile;
    if (full) {
      hs_hi = n_st / kTile;
    } else {
      hs_hi = (S < n_st ? S : n_st) / kTile;
      const int band_first = c_last - R + 1;               // first chunk index the last query still sees
      stg_lo = band_first > 0 ? (band_first + kTile - 1) / kTile : 0;
      if (stg_lo > stg_hi) stg_lo = stg_hi;
    }
  }
  if (mix) {
    const int sink_slots = S < n_st ? S : n_st;
    const int band_first = n_old + c_wg - R + 1;         // first position of the first query's band
    hs_lo = (sink_slots + kTile - 1) / kTile;
    if (hs_lo > hs_hi) hs_lo = hs_hi;
    const int before_band = band_first > 0 ? band_first / kTile : 0;
    if (hs_hi > before_band) hs_hi = before_band;
    if (hs_hi < hs_lo) hs_hi = hs_lo;
    const int before_band_stage = c_wg - R + 1 > 0 ? (c_wg - R + 1) / kTile : 0;
    if (stg_hi > before_band_stage) stg_hi = before_band_stage;
    if (sink_in_chunk > 0) stg_hi = 0;                   // the chunk itself still holds sink positions
  }
  const int hot_store = hs_hi - hs_lo;
  const int n_plain_all = hot_store + stg_hi - stg_lo;
  // (a divided workgroup: share z of Z of them; the last share also takes the general tiles)
  const int plain_lo = split ? (int)((int64_t)n_plain_all * z / Z) : 0;
  const int n_plain = split ? (int)((int64_t)n_plain_all * (z + 1) / Z) - plain_lo : n_plain_all;
  auto plain_address = [&](int i0) -> const char* {
    const int i = i0 + plain_lo;
    return i < hot_store ? store.at(hs_lo + i) : stage + (int64_t)(stg_lo + i - hot_store) * kTileBytes;
  };

  // General tiles of this wavefront: store tiles [0, n_store), then staging tiles [0, n_stage).
  int n_store;
  if (full) {
    n_store = (n_st + kTile - 1) / kTile;
  } else {
    // the ring matters only while the wavefront's first query still reaches positions before the chunk
    const int reach = c0 < R ? n_st : (S < n_st ? S : n_st);
    n_store = (reach + kTile - 1) / kTile;
  }
  const int n_stage = c_hi / kTile + 1;
  const int total = busy && (!split || z == Z - 1) ? n_store + n_stage : 0;
  const int band_lo = c0 - R + 1;            // first chunk index inside the recent band of the wavefront's first query
  auto needed = [&](int x) {
    if (x < n_store) return x < hs_lo || x >= hs_hi;
    const int j = x - n_store;
    if (j >= stg_lo && j < stg_hi) return false;
    if (full) return true;
    const int first = j * kTile;
    return first < sink_in_chunk || first + kTile - 1 >= band_lo;
  };
  auto next_needed = [&](int x) {
    while (x < total && !needed(x)) ++x;
    return x;
  };
  auto address = [&](int x) -> const char* {
    return x < n_store ? store.at(x) : stage + (int64_t)(x - n_store) * kTileBytes;
  };

  Frag ones;
  ones.u = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);      // eight bf16 1.0
  GroupState st[2];             // NG causal sets; GATED: st[1] is the local set of group 0
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    set_reference(st[k], -INFINITY, 1.f);
    st[k].l = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) st[k].o[j] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  // The softmax scale rides in the exponent's multiply-add.  A negative one (unusual) would turn the
  // running maximum into a minimum, and zero times the -inf of a masked score is not a number, so
  // those two are applied to the scores up front instead.
  const float pre_scale = scale_log2 > 0.f ? 1.f : scale_log2;
  const float exp_scale = scale_log2 > 0.f ? scale_log2 : 1.f;

  // ---- hot loop: the whole workgroup, tiles through LDS ---------------------------------------
  // Thread i moves 16 bytes of the tile's K half and 16 of its V half.  The loop exists in two forms.
  // The usual one (HALF) puts V into LDS as fp16 and sends the weights to the matrix cores as one
  // fp16 operand.  The other one, for a layer whose v_wide flag is up (some V value beyond the fp16
  // range has been appended since the cache was last empty; unusual), takes V as stored, with
  // two-part bf16 weights.
  auto hot_loop = [&](auto half_tag) {
    constexpr bool HALF = decltype(half_tag)::value;
    uint4 next_v = make_uint4(0, 0, 0, 0);      // the next tile's V as fp16, when the loop body has converted it already
    bool next_ready = false;
    auto put = [&](int x, const uint4& v16) {
      if (HALF) {
        sm_v[x & 1][tid] = next_ready ? next_v : bf16x8_to_f16x8(v16);
        next_ready = false;
      } else {
        sm_v[x & 1][tid] = v16;
      }
    };
    // Buffer loads: the tile's address travels in scalar registers (a descriptor made per tile) and the
    // per-thread offset is one fixed vector register, so no vector address registers are written while
    // earlier loads are still in flight (which the compiler answers with a wait for all of them).
    const int thread_off = tid * 16;
    // The K half goes from memory straight into LDS (lane i of a wavefront fills bytes 16 i .. 16 i + 15 behind
    // the wavefront's base, which is the tile's own order): no registers, no LDS store instruction.  Both
    // halves of a tile are asked for two tiles ahead; the compiler makes every wavefront wait for its loads into
    // LDS before the next barrier (the K half therefore has one iteration to arrive), the V half, which
    // passes through registers to be converted, is waited for where it is used, an iteration later.
    auto fetch = [&](int x, int slot, uint4& v16) {
      const __amdgpu_buffer_rsrc_t rsrc =
          __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(plain_address(x)), 0, kTileBytes, 0x00020000);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(&sm_k[slot & 3][wave * 64]), 16,
                                               thread_off, 0, 0, 0);
      const u32x4 vv = __builtin_amdgcn_raw_buffer_load_b128(rsrc, thread_off, 8192, 0);
      v16 = make_uint4(vv[0], vv[1], vv[2], vv[3]);
    };
    Frag ones_op = ones;
    if (HALF) ones_op.u = make_uint4(0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);    // eight fp16 1.0
    // One tile.  c1 holds this thread's 16 bytes of V of tile x + 1, asked for an iteration ago; the loads of
    // tile x + 2 are issued here, K into LDS, V into f1.  Two iterations ahead, in two register sets that
    // swap roles: the workgroups of a pair walk its tiles at about the same time, so most of these loads find
    // their line still on its way from HBM, and one iteration (about a microsecond) does not cover that.
    auto step = [&](int x, uint4& c1, uint4& f1) {
      __syncthreads();          // tile x is complete in its buffers; nobody reads the buffers written next any more
      const uint4* kbuf = sm_k[x & 3];
      const uint4* vbuf = sm_v[x & 1];
      TileRegs tr;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)                      // (also by a wavefront without queries: no branch here)
#pragma unroll
        for (int s = 0; s < 4; ++s) tr.k[hf][s].u = kbuf[(hf * 4 + s) * 64 + lane];
#pragma unroll
      for (int j = 0; j < 8; ++j) tr.v[j].u = vbuf[j * 64 + lane];
      fetch(x + 2 < n_plain ? x + 2 : n_plain - 1, x + 2, f1);   // (past the end: the last tile again, unused)
      if (busy) {
        float sc[NG][8], mx[NG];
        bool grow = false;
#pragma unroll
        for (int cg = 0; cg < NG; ++cg) {
          raw_scores(tr, qb[cg], sc[cg]);
          // (every lane holds its column's reference: the test needs the lane's own scores only)
          mx[cg] = max8(sc[cg]);
          grow |= mx[cg] > st[cg].thr;
        }
        if (__any(grow)) {
          // a maximum moved by more than the slack (rare): new references, accumulators rescaled
#pragma unroll
          for (int cg = 0; cg < NG; ++cg) {
            const float m_new = fmaxf(st[cg].m, column_max(mx[cg]) * exp_scale);
            const float alpha = st[cg].m == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(st[cg].m - m_new);
            set_reference(st[cg], m_new, exp_scale);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float a = __shfl(alpha, kb * 4 + r);
              st[cg].l[r] *= a;
#pragma unroll
              for (int j = 0; j < 8; ++j) st[cg].o[j][r] *= a;
            }
          }
        }
        if constexpr (HALF && NG == 2) {
          // Two column groups, written out in issue order: a wavefront's own vector instructions run
          // beside its matrix instructions (those of another wavefront of the SIMD do not), so the
          // exponentials of the second group sit between the matrix instructions of the first, and the
          // fp16 conversion of the next tile's V between those of the second.  The scheduling barriers
          // keep the compiler from gathering each kind again.
          const float ref0 = st[0].ref, ref1 = st[1].ref;
          float p[8];
          Frag ph0, ph1;
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][e], exp_scale, -ref0));
          half_weights(p, ph0);
          __builtin_amdgcn_sched_barrier(0);
          st[0].l = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph0.h, ones_op.h, st[0].l, 0, 0, 0);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            p[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[1][j], exp_scale, -ref1));
            __builtin_amdgcn_sched_barrier(0);
            st[0].o[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph0.h, tr.v[j].h, st[0].o[j], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
          half_weights(p, ph1);
          __builtin_amdgcn_sched_barrier(0);
          st[1].l = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph1.h, ones_op.h, st[1].l, 0, 0, 0);
          uint32_t hw[4];
          const uint32_t gw[4] = {c1.x, c1.y, c1.z, c1.w};
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            if (j < 4) hw[j] = bf16x2_to_f16x2(gw[j]);
            __builtin_amdgcn_sched_barrier(0);
            st[1].o[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph1.h, tr.v[j].h, st[1].o[j], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
          next_v = make_uint4(hw[0], hw[1], hw[2], hw[3]);
          next_ready = true;
        } else if constexpr (HALF && NG == 1) {
          // One column group: the fp16 conversion of the next tile's V sits between the matrix instructions.
          const float ref0 = st[0].ref;
          float p[8];
          Frag ph0;
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[0][e], exp_scale, -ref0));
          half_weights(p, ph0);
          __builtin_amdgcn_sched_barrier(0);
          st[0].l = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph0.h, ones_op.h, st[0].l, 0, 0, 0);
          uint32_t hw[4];
          const uint32_t gw[4] = {c1.x, c1.y, c1.z, c1.w};
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            if (j < 4) hw[j] = bf16x2_to_f16x2(gw[j]);
            __builtin_amdgcn_sched_barrier(0);
            st[0].o[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph0.h, tr.v[j].h, st[0].o[j], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
          next_v = make_uint4(hw[0], hw[1], hw[2], hw[3]);
          next_ready = true;
        } else
#pragma unroll
        for (int cg = 0; cg < NG; ++cg) {
          const float m_ref = st[cg].ref;
          float p[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[cg][e], exp_scale, -m_ref));
          if (HALF) {
            Frag ph;
            half_weights(p, ph);
            st[cg].l = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph.h, ones_op.h, st[cg].l, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 8; ++j)
              st[cg].o[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph.h, tr.v[j].h, st[cg].o[j], 0, 0, 0);
          } else {
            Frag phi, plo;
            split_weights(p, phi, plo);
            st[cg].l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi.v, ones_op.v, st[cg].l, 0, 0, 0);
            st[cg].l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo.v, ones_op.v, st[cg].l, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              st[cg].o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi.v, tr.v[j].v, st[cg].o[j], 0, 0, 0);
              st[cg].o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo.v, tr.v[j].v, st[cg].o[j], 0, 0, 0);
            }
          }
        }
      }
      put(x + 1, c1);           // (after the last tile: a copy of it into the buffer nobody reads any more)
    };
    uint4 a1, b1;
    fetch(0, 0, a1);
    put(0, a1);
    fetch(1 < n_plain ? 1 : 0, 1, a1);
    for (int x = 0; x < n_plain; x += 2) {
      step(x, a1, b1);
      if (x + 1 < n_plain) step(x + 1, b1, a1);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt 0: no load into LDS is left in flight behind the loop
  };
  if (n_plain > 0) {
    if (dv.v_wide[layer] == 0) hot_loop(std::true_type{});
    else hot_loop(std::false_type{});
  }
  if (!busy) return;            // no barrier lies ahead

  // ---- general loop: this wavefront alone, tiles straight from memory -------------------------
  // One tile: mask the scores of each column group and fold the tile into its softmax state.
  auto process = [&](TileRegs& tr, int x) {
    const bool from_store = x < n_store;
    const int tile = from_store ? x : x - n_store;
    const int held = from_store ? n_st : t;                     // slots of this source that hold a position
    const bool complete = tile * kTile + kTile <= held;         // every slot of the tile does
    // position held by each of the lane's eight slots (-1 = the slot holds nothing)
    int pos[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int slot = tile * kTile + (e >> 2) * 16 + kb * 4 + (e & 3);
      int p = from_store ? slot : n_old + slot;
      if (from_store && !full) p = slot_pos[slot < held ? slot : held - 1];
      pos[e] = slot < held ? p : -1;
    }
    if (from_store && !complete) {
      // slots of the store that were never written may hold anything: clear their V operands
      uint32_t msk[4];
#pragma unroll
      for (int jw = 0; jw < 4; ++jw)
        msk[jw] = (pos[2 * jw] >= 0 ? 0x0000ffffu : 0u) | (pos[2 * jw + 1] >= 0 ? 0xffff0000u : 0u);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        tr.v[j].u.x &= msk[0]; tr.v[j].u.y &= msk[1]; tr.v[j].u.z &= msk[2]; tr.v[j].u.w &= msk[3];
      }
    }
    // positions this tile can hold (store tiles of a compressed head: anything before the chunk)
    const int p_first = from_store ? (full ? tile * kTile : 0) : n_old + tile * kTile;
    const int p_last = from_store ? (full ? tile * kTile + kTile - 1 : n_old - 1) : n_old + tile * kTile + kTile - 1;
#pragma unroll
    for (int cg = 0; cg < NG; ++cg) {
      if (!g_on[cg]) continue;
      if (p_first > g_hi[cg]) continue;                                        // wholly above the causal diagonal
      if (!full && p_first >= S && p_last < g_lo[cg] - R + 1) continue;        // wholly before the recent band
      float raw[8], sc[8];
      tile_scores(tr, qb[cg], pre_scale, raw);
      const int i = qpos[cg];
      // a full head's tile at or below every query of the group needs no masking (columns that
      // stand for no query compute on zeros and are never written out)
      if (full && complete && p_last <= g_lo[cg]) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sc[e] = raw[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int p = pos[e];
          const bool on = p >= 0 && p <= i && (full || p < S || i - p < R);
          sc[e] = on ? raw[e] : -INFINITY;
        }
      }
      group_update(tr, sc, exp_scale, st[cg], kb, ones);
      if (GATED && mix && (p_first < S || p_last >= g_lo[cg] - R + 1)) {
        // the same scores under the local mask, into the group's second accumulator set
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int p = pos[e];
          const bool on = p >= 0 && p <= i && (p < S || i - p < R);
          sc[e] = on ? raw[e] : -INFINITY;
        }
        group_update(tr, sc, exp_scale, st[GATED ? LOCAL : 0], kb, ones);
      }
    }
  };
  {
    TileRegs tr;
    for (int x = next_needed(0); x < total; x = next_needed(x + 1)) {
      load_tile_cached(tr, address(x), lane);
      process(tr, x);
    }
  }

  if (split) {
    float* slot = split_out + (((int64_t)by * gridDim.x + bx) * Z + z) * kSplitSlotFloats;
#pragma unroll
    for (int cg = 0; cg < NG; ++cg) {
      if (kb == 0) slot[kSplitCols * kHeadDim + col0 + 16 * cg + hd] = st[cg].m;      // the lane's own column
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int col = col0 + 16 * cg + kb * 4 + r;
        if (hd == 0) slot[kSplitCols * (kHeadDim + 1) + col] = st[cg].l[r];
#pragma unroll
        for (int j = 0; j < 8; ++j) slot[col * kHeadDim + j * 16 + hd] = st[cg].o[j][r];
      }
    }
    return;
  }
  // out[b][head][c][d] = O / l (blended with the local result for a gated head); the accumulator
  // rows of group cg are its columns 4 kb + r
#pragma unroll
  for (int cg = 0; cg < NG; ++cg) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = col0 + 16 * cg + kb * 4 + r;
      const int cl = col / G, hh = col - cl * G;
      if (c_wg + cl <= c_last) {
        const int64_t orow = ((int64_t)b * dv.n_q_heads + h * G + hh) * stride_tokens + c_wg + cl;
        const float inv = 1.f / st[cg].l[r];
        const float inv_local = mix ? 1.f / st[GATED ? LOCAL : 0].l[r] : 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          float res = st[cg].o[j][r] * inv;
          if (GATED && mix) res = gate * res + (1.f - gate) * (st[GATED ? LOCAL : 0].o[j][r] * inv_local);
          out[orow * kHeadDim + j * 16 + hd] = f32_to_bf16_rne(res);
        }
      }
    }
  }
}

// Combines the shares of a divided workgroup: weights 2^(m_z - max m) on each share's accumulators and
// normaliser (every share's weights carry the same 2^kWeightShift, which cancels).  A share that saw no
// key has m = -inf and counts for nothing; the last share always holds the query's own position.
__global__ __launch_bounds__(kSplitCols) void prefill_merge_kernel(DeviceView dv, int layer, const float* __restrict__ split_out,
                                                                   int Z, uint16_t* __restrict__ out, int stride_tokens,
                                                                   PrefillHeads heads) {
  int b, h;
  bool full;
  pair_of_grid_row(dv, layer, blockIdx.y, heads, b, h, full);
  const int G = dv.group;
  const int wg_positions = kSplitCols / G;
  const int t = dv.append_cnt[b];
  const int c_wg = (gridDim.x - 1 - blockIdx.x) * wg_positions;
  if (c_wg >= t) return;
  const int c_last = (c_wg + wg_positions < t ? c_wg + wg_positions : t) - 1;
  const float* slot0 = split_out + ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * Z * kSplitSlotFloats;
  // eight columns per workgroup, four per thread: the loads behind the four outputs are independent, so
  // their latencies overlap, and there are still thousands of workgroups
  const int d = threadIdx.x & (kHeadDim - 1);
  constexpr int kPer = kMergeColsPerGroup / 2;
  float M[kPer], num[kPer], den[kPer];
  int col[kPer];
  bool on[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    col[i] = blockIdx.z * kMergeColsPerGroup + 2 * i + (threadIdx.x >> 7);
    on[i] = c_wg + col[i] / G <= c_last;
    M[i] = -INFINITY;
    num[i] = den[i] = 0.f;
  }
  for (int zz = 0; zz < Z; ++zz) {
    const float* sl = slot0 + (int64_t)zz * kSplitSlotFloats;
#pragma unroll
    for (int i = 0; i < kPer; ++i)
      if (on[i]) M[i] = fmaxf(M[i], sl[kSplitCols * kHeadDim + col[i]]);
  }
  for (int zz = 0; zz < Z; ++zz) {
    const float* sl = slot0 + (int64_t)zz * kSplitSlotFloats;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      if (!on[i]) continue;
      const float m = sl[kSplitCols * kHeadDim + col[i]];
      const float w = m == -INFINITY ? 0.f : exp2f(m - M[i]);
      num[i] += w * sl[col[i] * kHeadDim + d];
      den[i] += w * sl[kSplitCols * (kHeadDim + 1) + col[i]];
    }
  }
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    if (!on[i]) continue;
    const int cl = col[i] / G, hh = col[i] - cl * G;
    const int64_t orow = ((int64_t)b * dv.n_q_heads + h * G + hh) * stride_tokens + c_wg + cl;
    out[orow * kHeadDim + d] = f32_to_bf16_rne(num[i] / den[i]);
  }
}

}  // namespace

hipError_t launch_prefill_mfma(const DeviceView& dv, int layer, bool gated, const int32_t* len_in, const void* q,
                               const void* k, const void* v, void* out, int stride_tokens, int max_tokens,
                               float scale_log2, char* staging, int staging_tiles, int n_split, float* split_out,
                               int split_rows, int dealt_rows, const uint8_t* mask_row, hipStream_t stream,
                               hipEvent_t ev_start, hipEvent_t ev_stop) {
  PrefillHeads heads;
  heads.n_full = -1;
  heads.heavy_rows = split_rows;
  heads.dealt_rows = dealt_rows;
  if (mask_row && dv.n_kv_heads <= kPrefillArgHeads) {
    int nf = 0, nc = 0;
    for (int i = 0; i < dv.n_kv_heads; ++i) {
      if (mask_row[i]) heads.head[0][nf++] = i;
      else heads.head[1][nc++] = i;
    }
    heads.n_full = nf;
  }
  const int tiles = (max_tokens + kTile - 1) / kTile;
  hipLaunchKernelGGL(stage_chunk_kernel, dim3(tiles, dv.n_pairs), dim3(kBlock), 0, stream, dv, layer, (const uint16_t*)k,
                     (const uint16_t*)v, stride_tokens, staging, staging_tiles);
  if (hipError_t e = hipGetLastError()) return e;
  if (gated || n_split < 1 || !split_out) n_split = 1;         // (the blending form is never divided)
  const int per_block = kPrefillWaves * 16 * (gated ? 1 : 2) / dv.group;      // chunk positions per workgroup
  const dim3 grid((max_tokens + per_block - 1) / per_block, dv.n_pairs, n_split), block(kPrefillBlock);
#define RLKV_LAUNCH(PG, GT)                                                                                          \
  hipExtLaunchKernelGGL((prefill_mfma_kernel<PG, GT>), grid, block, 0, stream, ev_start, ev_stop, 0, dv, layer, len_in, \
                        (const uint16_t*)q, (uint16_t*)out, stride_tokens, scale_log2, (const char*)staging,       \
                        staging_tiles, split_out, heads)
  if (dv.page_shift >= 0) { if (gated) RLKV_LAUNCH(true, true); else RLKV_LAUNCH(true, false); }
  else                    { if (gated) RLKV_LAUNCH(false, true); else RLKV_LAUNCH(false, false); }
#undef RLKV_LAUNCH
  if (hipError_t e = hipGetLastError()) return e;
  if (n_split > 1 && split_rows > 0)
    hipLaunchKernelGGL(prefill_merge_kernel, dim3(grid.x, split_rows, kSplitCols / kMergeColsPerGroup), dim3(kSplitCols), 0, stream, dv, layer,
                       (const float*)split_out, n_split, (uint16_t*)out, stride_tokens, heads);
  return hipGetLastError();
}

}  // namespace rlkv
