// Host side of the work list: where the end-to-end sequence of scheduling units is cut into one
// contiguous share per workgroup.  Runs on the host from the library's mirror of the lengths (the
// records are then copied to the device), so a rebuild costs the GPU a small copy and no kernel.
//
// Cost model (paper Sec. 4.3: the residual cost of a compressed head is its sW/L tokens, so a
// share's cost is what it reads plus what it restarts): kRoundCost per round of tiles plus
// kPairStartCost for every pair that starts in the share - the load pipeline restarts on a new
// store, Q is loaded, a merge and an output or partial write follow; about 1.5 rounds by
// per-workgroup timestamps.  A pair that continues from the previous workgroup pays no start.
// The plan is the in-order greedy deal at the smallest capacity that needs no more workgroups than
// the grid has; greedy is optimal for a contiguous partition once the capacity is fixed.
#include <algorithm>
#include <vector>

#include "prefill_deal.h"
#include "rlkv_internal.h"

namespace rlkv {

// Deals the rounds out at capacity `cap`; returns the number of workgroups used.  With wg_begin /
// seg_first / seg_count non-null also records the shares.
static int deal_rounds(const int32_t* rounds, int n_pairs, int cap, int32_t* wg_begin, int32_t* seg_first,
                       int32_t* seg_count) {
  const int per_fresh = cap / kRoundCost;                  // rounds a workgroup takes of a pair it does not start
  int w = 0, used = 0, us = 0;                             // us: first unit of the pair in the end-to-end numbering
  for (int p = 0; p < n_pairs; ++p) {
    const int r = rounds[p];
    if (seg_first) { seg_first[p] = 0; seg_count[p] = 0; }
    if (r == 0) continue;                                  // inactive slot
    if (used > 0 && cap - used < kPairStartCost + kRoundCost) {
      ++w;
      used = 0;
      if (wg_begin) wg_begin[w] = us;
    }
    if (seg_first) seg_first[p] = w;
    used += kPairStartCost;
    int take = (cap - used) / kRoundCost;
    if (take > r) take = r;
    used += take * kRoundCost;
    const int rest = r - take;
    if (rest > 0) {
      const int more = (rest + per_fresh - 1) / per_fresh;          // further workgroups, the last one partly filled
      if (wg_begin)
        for (int k = 0; k < more; ++k) wg_begin[w + 1 + k] = us + kPairOverheadUnits + take + k * per_fresh;
      w += more;
      used = (rest - (more - 1) * per_fresh) * kRoundCost;
    }
    if (seg_count) seg_count[p] = w - seg_first[p] + 1;
    us += r + kPairOverheadUnits;
  }
  return w + 1;
}

int plan_shares(const int32_t* rounds, int n_pairs, int n_wg, int32_t* wg_begin, int32_t* seg_first,
                int32_t* seg_count) {
  int64_t cost = 0, units = 0;
  int longest = 0;
  for (int p = 0; p < n_pairs; ++p)
    if (rounds[p] > 0) {
      cost += (int64_t)rounds[p] * kRoundCost + kPairStartCost;
      units += rounds[p] + kPairOverheadUnits;
      if (rounds[p] > longest) longest = rounds[p];
    }
  for (int w = 0; w <= n_wg; ++w) wg_begin[w] = (int32_t)units;      // workgroups the deal does not reach stay empty
  wg_begin[0] = 0;
  if (units == 0) {
    for (int p = 0; p < n_pairs; ++p) seg_first[p] = seg_count[p] = 0;
    return 0;
  }
  // feasible for sure: the whole list in one workgroup; look upward from the average
  int64_t cap = (cost + n_wg - 1) / n_wg;
  if (cap < kPairStartCost + kRoundCost) cap = kPairStartCost + kRoundCost;
  while (deal_rounds(rounds, n_pairs, (int)cap, nullptr, nullptr, nullptr) > n_wg) {
    // the average is nearly always within a few steps of the answer; widen the stride if not
    const int64_t step = cap / 64 > 0 ? cap / 64 : 1;
    int64_t probe = cap + step;
    if (step > 1 && deal_rounds(rounds, n_pairs, (int)probe, nullptr, nullptr, nullptr) <= n_wg) {
      // overshot: walk the last stride one by one
      ++cap;
      while (deal_rounds(rounds, n_pairs, (int)cap, nullptr, nullptr, nullptr) > n_wg) ++cap;
      break;
    }
    cap = probe;
  }
  return deal_rounds(rounds, n_pairs, (int)cap, wg_begin, seg_first, seg_count);
}

}  // namespace rlkv

extern "C" int32_t rlkv_plan_shares(const int32_t* rounds, int32_t n_pairs, int32_t n_workgroups, int32_t* wg_begin,
                                    int32_t* seg_first, int32_t* seg_count) {
  if (!rounds || !wg_begin || !seg_first || !seg_count || n_pairs < 1 || n_workgroups < 1) return -1;
  for (int p = 0; p < n_pairs; ++p)
    if (rounds[p] < 0 || rounds[p] > (1 << 24)) return -1;
  return rlkv::plan_shares(rounds, n_pairs, n_workgroups, wg_begin, seg_first, seg_count);
}

extern "C" int32_t rlkv_plan_prefill_form(int32_t n_compute_units, int32_t n_q_heads, int32_t n_kv_heads,
                                          int32_t n_full_heads, int32_t batch, const int32_t* n_tokens,
                                          const int32_t* cached, int32_t min_share_tiles, int32_t allow_narrow,
                                          int32_t* narrow, int32_t* n_split) {
  if (!n_tokens || !cached || !narrow || !n_split) return -1;
  if (n_compute_units < 1 || n_kv_heads < 1 || n_q_heads < n_kv_heads || n_q_heads % n_kv_heads != 0) return -1;
  if (n_full_heads < 0 || n_full_heads > n_kv_heads || batch < 1 || min_share_tiles < 1) return -1;
  using namespace rlkv;
  const int G = n_q_heads / n_kv_heads, per_block = G < 256 ? 256 / G : 1;     // chunk positions per workgroup
  int64_t blocks = 0, n_active = 0;
  int max_tok = 0, min_tiles = INT32_MAX;      // min_tiles: cached tiles of the shortest sequence that has a chunk
  for (int b = 0; b < batch; ++b) {
    if (n_tokens[b] < 0 || cached[b] < 0) return -1;
    if (n_tokens[b] == 0) continue;
    blocks += (n_tokens[b] + per_block - 1) / per_block;
    ++n_active;
    if (n_tokens[b] > max_tok) max_tok = n_tokens[b];
    if (cached[b] / kTile < min_tiles) min_tiles = cached[b] / kTile;
  }
  *narrow = 0;
  *n_split = 1;
  const int64_t long_wgs = blocks * (n_full_heads ? n_full_heads : n_kv_heads);
  if (n_active == 0 || 2 * long_wgs > n_compute_units) return 0;
  // (Dividing when the long workgroups need more than one round was measured and lost: three sequences of
  // the Qwen shape, 342 workgroups, 4.53 -> 4.76 ms per 16384 tokens.)
  constexpr int kMaxSplit = 8;
  const int64_t rows = (int64_t)((max_tok + per_block - 1) / per_block) * n_active * n_full_heads;   // slots per share
  for (int zc = 2; zc <= kMaxSplit && n_full_heads > 0; ++zc) {
    if (long_wgs * zc > n_compute_units || rows * zc > kPrefillSplitSlots || min_tiles / zc < min_share_tiles) break;
    *n_split = zc;
  }
  if (*n_split == 1 && allow_narrow) *narrow = 1;
  return 0;
}

extern "C" int32_t rlkv_plan_prefill_rows(int32_t n_full_heads, int32_t batch, const int32_t* n_tokens,
                                          const int32_t* cached, int32_t* dealt_rows, int32_t* heavy_rows) {
  if (!n_tokens || !cached || !dealt_rows || !heavy_rows || n_full_heads < 0 || batch < 1) return -1;
  // work of a full head's grid row: its queries times the keys each attends over on average, plus a constant
  // per query for what a workgroup costs beside its unmasked tiles; sequences in the order of the grid
  // (those with a chunk first, then by cached + chunk length, longest first; stable)
  std::vector<int32_t> order;
  for (int b = 0; b < batch; ++b) {
    if (n_tokens[b] < 0 || cached[b] < 0) return -1;
    if (n_tokens[b] > 0) order.push_back(b);
  }
  std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
    return (int64_t)cached[x] + n_tokens[x] > (int64_t)cached[y] + n_tokens[y];
  });
  const int heavy = (int)order.size() * n_full_heads;
  auto work = [&](int row) {
    const int32_t b = order[row / n_full_heads];
    return (double)n_tokens[b] * ((double)cached[b] + 0.5 * n_tokens[b] + 600.0);
  };
  int dealt = 0;
  while (dealt + 8 <= heavy && work(dealt + 7) >= 0.85 * work(dealt)) dealt += 8;
  *dealt_rows = dealt;
  *heavy_rows = heavy;
  return 0;
}

extern "C" int32_t rlkv_plan_prefill_block(int32_t linear_index, int32_t grid_x, int32_t grid_y, int32_t dealt_rows,
                                           int32_t heavy_rows, int32_t* block_x, int32_t* block_y) {
  if (!block_x || !block_y || grid_x < 1 || grid_y < 1 || linear_index < 0 ||
      (int64_t)linear_index >= (int64_t)grid_x * grid_y)
    return -1;
  int bx = 0, by = 0;
  rlkv::prefill_deal(linear_index, grid_x, grid_y, dealt_rows, heavy_rows, bx, by);
  *block_x = bx;
  *block_y = by;
  return 0;
}
