// Split-K decode attention, MFMA variant (tiled bf16 stores).
//
// Same operation as the vector-ALU variant (softmax attention of the G query heads of a
// group over the rows a store holds; paper Sec. 3.1 Eq. 1 at gate 0/1, Sec. 3.3), with the
// two contractions on the matrix cores:
//   scores  S[slot][head] = sum_d K[slot][d] * Q[head][d]   v_mfma_f32_16x16x32_bf16,
//                           A = K tile (16 slots x 32 d), B = Q^T (heads padded to 16)
//   output  O[head][d]    = sum_slot P[head][slot] * V[slot][d]   same instruction,
//                           A = P (k runs over the 32 slots of a tile), B = V tile
// The score accumulator leaves lane l holding head l%16 and slots 4*(l/16)..+3 of each
// 16-slot half, which is exactly the A-operand register layout, so P never moves between
// lanes.  The stores are laid out (see rlkv_internal.h) so that every 128-bit load per lane
// is one contiguous kilobyte per wavefront and lands directly in operand registers: no
// LDS staging, no transposes, and the wavefronts of a workgroup run independently until
// the merge.  P is split into a bf16 head and a bf16 remainder (two MFMAs per V block) so
// the weights carry ~16 mantissa bits; the matrix cores are idle most of the time anyway.
//
// The kernel is latency-lean at its start: a workgroup learns its share and its first store
// from one wave-uniform record and at once issues the loads of Q and of its first tile.
// Each wavefront keeps one tile (16 KiB) in flight behind the one it works on; with one
// workgroup per CU that is 64 KiB in flight per CU, which measurement shows is where this
// part's HBM streams best (more in flight lowers the achieved bandwidth).
//
// Gated heads (GATED = true; paper Sec. 3.1, Eq. 1): a full head with gate g < 1 returns
// g * full + (1 - g) * local attention.  The local positions (first S, last R) are a subset of
// the full ones, so the same pass keeps a second accumulator that only the tiles touching
// those ranges update; the scores of a tile are computed once for both.
//
// Fused single-token append (FUSED = true): the kernel also performs this step's append.
// Every sequence grows by one position; the wavefront that owns the tile holding the new
// slot of a pair writes the new K/V row into the store (sink slot, ring slot - evicting
// position p - R - or next row of a full head) before it loads that tile; each lane writes
// exactly the bytes it later loads, so no other wavefront ever depends on the write.  No
// workgroup reads a length from the table: a pair's length is its length when the work list was
// planned plus the list's growth counter (ListHeader::grow), which this kernel only reads - the
// merge kernel that follows advances it - so the kernel needs no grid-wide fence, takes no
// per-step argument, and a captured launch can be replayed.  The new lengths are written to
// both copies of the length table for the kernels that do read it.
#include "mfma_tile.h"

namespace rlkv {
namespace {

// Online-softmax update and P.V accumulation of one tile into `st`.  A slot counts if it
// lies in the valid prefix [0, n_eff) and, for the local attention of a gated head (LOCAL),
// also in the sink range [0, keep_lo) or the recent range [keep_from, n_eff).  Clears the V
// operands of slots that do not count (they may hold anything).
template <bool LOCAL>
__device__ __forceinline__ void tile_accumulate(TileRegs& t, const float (&raw)[8], Softmax& st, int tile, int n_eff,
                                                int kb, int keep_lo = 0, int keep_from = 0) {
  auto counts = [&](int slot) { return slot < n_eff && (!LOCAL || slot < keep_lo || slot >= keep_from); };
  float sc[8];
  const int slot0 = tile * kTile + kb * 4;
  const bool ragged_tile = tile * kTile + kTile > n_eff ||
                           (LOCAL && tile * kTile + kTile > keep_lo && tile * kTile < keep_from);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int slot = slot0 + (e >> 2) * 16 + (e & 3);
    sc[e] = (!ragged_tile || counts(slot)) ? raw[e] : -INFINITY;
  }
  if (ragged_tile) {
    uint32_t msk[4];
#pragma unroll
    for (int jw = 0; jw < 4; ++jw) {
      const int e0 = 2 * jw, e1 = 2 * jw + 1;
      const int sl0 = slot0 + (e0 >> 2) * 16 + (e0 & 3), sl1 = slot0 + (e1 >> 2) * 16 + (e1 & 3);
      msk[jw] = (counts(sl0) ? 0x0000ffffu : 0u) | (counts(sl1) ? 0xffff0000u : 0u);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      t.v[j].u.x &= msk[0]; t.v[j].u.y &= msk[1]; t.v[j].u.z &= msk[2]; t.v[j].u.w &= msk[3];
    }
  }
  softmax_pv(t, sc, st, kb);
}

// One tile of a head: full attention into st_full and, for a gated head (Eq. 1), the local
// attention into st_local when the tile touches the sink or the recent range.  The scores
// are computed once; the full update runs first because its V clearing (slots past the
// prefix) is a subset of the local one.
template <bool GATED>
__device__ __forceinline__ void process_tile(TileRegs& t, const Frag (&qb)[4], Softmax& st_full, Softmax& st_local,
                                             bool two_sets, int tile, int n_eff, float scale_log2, int kb, int keep_lo,
                                             int keep_from) {
  float raw[8];
  tile_scores(t, qb, scale_log2, raw);
  tile_accumulate<false>(t, raw, st_full, tile, n_eff, kb);
  if (GATED && two_sets && (tile * kTile < keep_lo || tile * kTile + kTile > keep_from))
    tile_accumulate<true>(t, raw, st_local, tile, n_eff, kb, keep_lo, keep_from);
}

// The gated variant carries two accumulator sets: it is built for one wavefront per SIMD (the
// configuration the library launches), which leaves it 512 registers.
template <bool FUSED, bool GATED, bool PAGED>
__global__ __launch_bounds__(kBlock, 1) void decode_mfma_kernel(DeviceView dv, int layer,
                                                                const uint16_t* __restrict__ q,
                                                                uint16_t* __restrict__ out, float scale_log2,
                                                                const uint16_t* __restrict__ k_new,
                                                                const uint16_t* __restrict__ v_new) {
  __shared__ float sm_o[4][kMaxGroup][kHeadDim];
  __shared__ float sm_m[4][kMaxGroup];
  __shared__ float sm_l[4][kMaxGroup];

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // shares so that its L2 and TLBs see one compact slice of the stores.
  const int n_wg = gridDim.x;
  const int wg = (n_wg & 7) == 0 ? (blockIdx.x & 7) * (n_wg >> 3) + (blockIdx.x >> 3) : blockIdx.x;
  const WgDesc* __restrict__ wdp = wg_desc_of(dv, layer) + wg;
  const int grow = list_header(dv, layer)->grow;     // tokens since the list was planned (asked for beside the record)
  const int u_begin = wdp->u_begin, u_end = wdp->u_end;
  // The record this workgroup will start the next layer's launch with: asked for now, so that it is in
  // L2 by then (its record is the first thing a workgroup waits for).  Looked at only at the very end.
  uint32_t warm = 0;
  if (threadIdx.x == 0 && layer + 1 < dv.n_layers)
    warm = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(wdp) + dv.list_stride);
  if (u_begin >= u_end) return;
  int pi = wdp->first_pair;
  PairDesc pd = wdp->first;
  const PairDesc* __restrict__ pairs = pair_desc_of(dv, layer);

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int hd = lane & 15;     // score layout: head; operand layouts: row / column
  const int kb = lane >> 4;     // k-group of the operand layouts; slot quad of the score layout
  const int G = dv.group;

  for (int u = u_begin; u < u_end;) {
    // segment = the units [u, seg_end) of pair pi = tiles [tile_lo, tile_hi) of its store
    const int ps = pd.unit_start, pe = pd.unit_end;
    const int seg_end = u_end < pe ? u_end : pe;
    // the first unit(s) of a pair carry no tiles (they stand for its fixed cost)
    const int r_lo = u - ps > kPairOverheadUnits ? u - ps - kPairOverheadUnits : 0;
    const int r_hi = seg_end - ps > kPairOverheadUnits ? seg_end - ps - kPairOverheadUnits : 0;
    const int tile_lo = r_lo * kRound;
    const bool whole_pair = u == ps && seg_end == pe;
    const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
    const int n_old = pd.n_build + grow;
    const int n = FUSED ? n_old + 1 : n_old;
    const bool full = pd.full != 0;
    const int n_eff = full ? n : (n < dv.window ? n : dv.window);
    TileMap<PAGED> store;
    store.base = dv.kv_base + pd.koff;
    store.paged = PAGED && full;
    if (PAGED) {
      store.row = dv.block_table + (int64_t)b * dv.table_stride;
      store.page_bytes = dv.page_bytes;
      store.shift = dv.page_shift;
      store.mask = dv.page_mask;
      store.last = dv.table_stride - 1;
    }
    // the list was built with room to grow: tiles past the valid prefix are still empty
    const int tiles_valid = (n_eff + kTile - 1) / kTile;
    const int tile_hi = r_hi * kRound < tiles_valid ? r_hi * kRound : tiles_valid;

    if (FUSED) {
      // whoever owns tile 0 of head 0 publishes the new length, in both copies of the table (nobody reads
      // either during this launch)
      if (h == 0 && tile_lo == 0 && tid == 0) { len_of(dv, 0, layer)[b] = n; len_of(dv, 1, layer)[b] = n; }
      // position n_old goes to slot_new (sink / ring / next row of a full head)
      const int slot_new = (full || n_old < dv.sink) ? n_old : dv.sink + (n_old - dv.sink) % dv.recent;
      const int tile_new = slot_new >> 5;
      if (tile_new >= tile_lo && tile_new < tile_hi && ((tile_new - tile_lo) & 3) == wave) {
        // This wavefront will read the tile that holds the new slot: it writes the row first.
        // Every 16-byte unit below is written by the lane that later loads it, so program
        // order makes the loads see the new row.
        const int st = slot_new & 31, hf = st >> 4;
        char* tile_base = store.at(tile_new);
        const int64_t src = ((int64_t)b * dv.n_kv_heads + h) * kHeadDim;
        // (all loads of the new row first, then the stores: one memory latency instead of two in a row
        // for the one wavefront per pair that does this, and whose workgroup waits for it at the merge)
        const bool k_lane = hd == (st & 15);            // K: the lanes that hold row slot % 16
        const bool v_lane = kb == ((st & 15) >> 2);     // V: the lanes that hold this slot's k-group
        uint4 kn[4];
        uint16_t vn[8];
#pragma unroll
        for (int s = 0; s < 4; ++s)
          kn[s] = k_lane ? *reinterpret_cast<const uint4*>(k_new + src + (s * 4 + kb) * 8) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) vn[j] = v_lane ? v_new[src + j * 16 + hd] : (uint16_t)0;
        if (k_lane) {
#pragma unroll
          for (int s = 0; s < 4; ++s) *reinterpret_cast<uint4*>(tile_base + hf * 4096 + s * 1024 + lane * 16) = kn[s];
        }
        if (v_lane) {
          const int e = hf * 4 + (st & 3);
#pragma unroll
          for (int j = 0; j < 8; ++j)
            *reinterpret_cast<uint16_t*>(tile_base + 8192 + j * 1024 + lane * 16 + e * 2) = vn[j];
        }
        if (lane == 0 && !full)
          dv.slot_pos[dv.slotpos_off[layer * dv.n_kv_heads + h] + (int64_t)b * dv.window + slot_new] = n_old;
      }
    }

    // Q as the B operand of the score MFMA: column = head, k-group kb, step s
    Frag qb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (hd < G) {
        const int64_t qrow = (int64_t)b * dv.n_q_heads + h * G + hd;
        qb[s].u = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(q) +
                                                  (qrow * kHeadDim + s * 32 + kb * 8) * 2);
      } else {
        qb[s].u = make_uint4(0, 0, 0, 0);
      }
    }
    // each wavefront keeps one tile in flight behind the one it is working on
    int tile = tile_lo + wave;
    TileRegs ra, rb;
    if (tile < tile_hi) load_tile(ra, store.at(tile), lane);
    // address of the tile after this one; looked up one iteration ahead so that a block-table
    // read never sits between a wavefront and its next loads
    const char* next_base = store.at(tile + kRound);
    // the next pair's record, for the (rare) share that crosses a pair boundary
    PairDesc pd_next = pd;
    if (seg_end < u_end) pd_next = pairs[pi + 1];     // fetched early, looked at after the segment

    // Eq. 1 gate: a full head with gate < 1 also accumulates its local attention (sink + recent
    // positions) over the same tiles; out = gate * full + (1 - gate) * local.
    const bool two_sets = GATED && full && pd.gate < 1.f;
    const int keep_lo = dv.sink, keep_from = n - dv.recent;          // local: slot < S or slot >= n - R
    Softmax st[GATED ? 2 : 1];
#pragma unroll
    for (int k = 0; k < (GATED ? 2 : 1); ++k) {
      st[k].m = -INFINITY;
      st[k].l = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) st[k].o[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    // Two register images that swap roles, and the last tile of the segment outside the steady state:
    // inside it the loads of the next tile are unconditional, so the work on the current one waits for
    // its own loads only and the next tile's stay in flight beside it.  (With one loop and a conditional
    // load the compiler has to wait for every load in flight before the work, the next tile's included.)
    auto work = [&](TileRegs& t, int tl) {
      process_tile<GATED>(t, qb, st[0], st[GATED ? 1 : 0], two_sets, tl, n_eff, scale_log2, kb, keep_lo, keep_from);
    };
    if constexpr (GATED) {
      // (the variant with two accumulator sets has no registers left for that and keeps the one loop)
      while (tile < tile_hi) {
        if (tile + kRound < tile_hi) load_tile(rb, next_base, lane);
        next_base = store.at(tile + 2 * kRound);
        work(ra, tile);
        ra = rb;
        tile += kRound;
      }
    } else
    for (;;) {
      if (tile + kRound >= tile_hi) {
        if (tile < tile_hi) work(ra, tile);
        break;
      }
      load_tile(rb, next_base, lane);
      next_base = store.at(tile + 2 * kRound);
      work(ra, tile);
      tile += kRound;
      if (tile + kRound >= tile_hi) {
        work(rb, tile);
        break;
      }
      load_tile(ra, next_base, lane);
      next_base = store.at(tile + 2 * kRound);
      work(rb, tile);
      tile += kRound;
    }

    float held[(kMaxGroup * kHeadDim) / kBlock];                     // full-attention results of a whole pair
#pragma unroll
    for (int set = 0; set < (GATED ? 2 : 1); ++set) {
      if (set == 1 && !two_sets) break;
      const Softmax& ss = st[set];
      float l = ss.l;
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);

      __syncthreads();   // the previous merge has finished reading LDS
      if (kb == 0 && hd < G) { sm_m[wave][hd] = ss.m; sm_l[wave][hd] = l; }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int g = kb * 4 + r;
        if (g < G) {
#pragma unroll
          for (int j = 0; j < 8; ++j) sm_o[wave][g][j * 16 + hd] = ss.o[j][r];
        }
      }
      __syncthreads();
      int it = 0;
      for (int idx = tid; idx < G * kHeadDim; idx += kBlock, ++it) {
        const int g = idx / kHeadDim, d = idx % kHeadDim;
        float M = sm_m[0][g];
#pragma unroll
        for (int w = 1; w < 4; ++w) M = fmaxf(M, sm_m[w][g]);
        float O = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float sc = exp2_or_zero(sm_m[w][g], M);
          O += sc * sm_o[w][g][d];
          L += sc * sm_l[w][g];
        }
        if (whole_pair) {
          float res = O / L;
          if (two_sets) {
            if (set == 0) { held[it] = res; continue; }
            res = pd.gate * held[it] + (1.f - pd.gate) * res;
          }
          const int64_t oi = ((int64_t)b * dv.n_q_heads + h * G + g) * kHeadDim + d;
          out[oi] = f32_to_bf16_rne(res);
        } else {
          const int64_t slot = (int64_t)wg + pi;
          dv.part_o[set * dv.part_set_o + (slot * G + g) * kHeadDim + d] = O;
          if (d == 0) {
            dv.part_m[set * dv.part_set_ml + slot * G + g] = M;
            dv.part_l[set * dv.part_set_ml + slot * G + g] = L;
          }
        }
      }
    }
    u = seg_end;
    ++pi;
    pd = pd_next;
    if (u < u_end)
      while (pd.unit_end <= u) pd = pairs[++pi];       // pairs of inactive slots own no units
  }
  asm volatile("" ::"v"(warm));                        // keeps the load above alive
}

}  // namespace

hipError_t launch_decode_mfma(const DeviceView& dv, int layer, bool gated, const void* q, void* out, float scale_log2,
                              const void* k_new, const void* v_new, hipStream_t stream, hipEvent_t ev_start,
                              hipEvent_t ev_stop) {
  const dim3 grid(dv.n_wg), block(kBlock);
  // (the plain launch when no timestamps are asked for: that form can be recorded into a graph)
#define RLKV_LAUNCH(F, GT, PG)                                                                                    \
  do {                                                                                                            \
    if (ev_start || ev_stop)                                                                                      \
      hipExtLaunchKernelGGL((decode_mfma_kernel<F, GT, PG>), grid, block, 0, stream, ev_start, ev_stop, 0, dv,    \
                            layer, (const uint16_t*)q, (uint16_t*)out, scale_log2, (const uint16_t*)k_new,       \
                            (const uint16_t*)v_new);                                                              \
    else                                                                                                          \
      hipLaunchKernelGGL((decode_mfma_kernel<F, GT, PG>), grid, block, 0, stream, dv, layer, (const uint16_t*)q,  \
                         (uint16_t*)out, scale_log2, (const uint16_t*)k_new, (const uint16_t*)v_new);             \
  } while (0)
#define RLKV_PICK(F, GT) do { if (dv.page_shift >= 0) RLKV_LAUNCH(F, GT, true); else RLKV_LAUNCH(F, GT, false); } while (0)
  if (k_new) { if (gated) RLKV_PICK(true, true); else RLKV_PICK(true, false); }
  else       { if (gated) RLKV_PICK(false, true); else RLKV_PICK(false, false); }
#undef RLKV_PICK
#undef RLKV_LAUNCH
  return hipGetLastError();
}

}  // namespace rlkv
