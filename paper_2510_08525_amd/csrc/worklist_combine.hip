// Work-list build and split-K merge for decode attention over the head-mixed cache.
//
// One work list covers both head types: every (sequence, KV head) pair contributes
// ceil(n_eff / 32) tiles, n_eff = n for a full head and min(n, sink + recent) for a
// compressed one (the residual cost s*W/L of Sec. 4.3).  A workgroup's four wavefronts
// take one tile each per round, and a wavefront's time is set by the number of rounds it
// waits for, so the unit of scheduling is the round: ceil(tiles / 4) units per pair, behind one
// unit that carries no tiles and marks the pair's start.  The units of all pairs are laid end to
// end and cut into contiguous shares, one per workgroup, so a tiny compressed head costs a
// workgroup exactly its rounds and nothing idles behind a long full head.
//
// Where to cut: a share costs kRoundCost per round plus kPairStartCost for every pair that starts
// in it (the load pipeline restarts on a new store, Q is loaded, a merge and an output or partial
// write follow; about 1.5 rounds by per-workgroup timestamps).  The kernel looks for the smallest
// capacity for which dealing the rounds out in order, never beyond the capacity, needs no more
// workgroups than the grid has - candidates from the average cost upward, one per thread - and
// then deals once more to record the shares.  A workgroup whose share crosses pair boundaries
// emits one partial per pair it touches, in slot (workgroup index + pair index); the workgroups
// of a pair are consecutive, and the merge below walks them in ascending order, so the result is
// deterministic.
//
// A list is built for the lengths of the moment plus `slack` tokens of growth, so the
// decode steps that follow (one token per sequence each) reuse it; the attention kernels
// skip tiles that are still empty.  The host rebuilds it when the slack is used up.
#include "rlkv_internal.h"

namespace rlkv {
namespace {

// Walks the pairs in order and deals their rounds to workgroups of capacity `cap` (cost units:
// kRoundCost per round, kPairStartCost where a pair starts; a pair that continues into the next
// workgroup pays no start there).  Returns the number of workgroups used.  With EMIT, records the
// shares: close(w, u) = workgroup w ends at unit u (and w + 1 begins there), begin(p, w) / end(p, w) =
// pair p starts in workgroup w / its last round lies in workgroup w.
template <bool EMIT, typename Close, typename Begin, typename End>
__device__ int deal_rounds(const int* rounds, const int* unit_start, int n_pairs, int cap, Close close, Begin begin,
                           End end) {
  int w = 0, used = 0;
  for (int p = 0; p < n_pairs; ++p) {
    const int r = rounds[p];
    if (r == 0) continue;                                  // inactive slot
    const int us = unit_start[p];
    if (used > 0 && cap - used < kPairStartCost + kRoundCost) {
      if (EMIT) close(w, us);
      ++w;
      used = 0;
    }
    if (EMIT) begin(p, w);
    used += kPairStartCost;
    int done = 0;
    for (;;) {
      int take = (cap - used) / kRoundCost;
      if (take > r - done) take = r - done;
      done += take;
      used += take * kRoundCost;
      if (done == r) break;
      if (EMIT) close(w, us + kPairOverheadUnits + done);  // the pair goes on in the next workgroup
      ++w;
      used = 0;
    }
    if (EMIT) end(p, w);
  }
  return w + 1;
}

__global__ __launch_bounds__(1024) void build_worklist_kernel(DeviceView dv, int layer,
                                                              const int32_t* __restrict__ len_in, int slack) {
  __shared__ int scan[1024];
  __shared__ int carry;
  __shared__ int rounds[kGreedyMaxPairs];      // rounds of tiles per pair (0 = inactive)
  __shared__ int seg_first[kGreedyMaxPairs];   // first workgroup of the pair
  __shared__ int seg_count[kGreedyMaxPairs];   // workgroups that hold units of the pair
  __shared__ int best_cap, cost_total;
  const int tid = threadIdx.x;
  const bool greedy = dv.n_pairs <= kGreedyMaxPairs;
  int* unit_start = dv.unit_start + (int64_t)layer * (dv.n_pairs + 1);
  if (tid == 0) { carry = 0; unit_start[0] = 0; best_cap = 0x7fffffff; cost_total = 0; }
  __syncthreads();
  for (int base = 0; base < dv.n_pairs; base += 1024) {
    const int pi = base + tid;
    int units = 0;
    if (pi < dv.n_pairs) {
      const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
      const int n = len_in[b];
      const bool full = dv.full_mask[layer * dv.n_kv_heads + h] != 0;
      const int limit = full ? dv.cap_pad[b] : dv.window;     // what the store can ever hold
      const int n_fut = n + slack < limit ? n + slack : limit;
      units = (n_fut + kTile * kRound - 1) / (kTile * kRound) + kPairOverheadUnits;
      if (!dv.active[b]) units = 0;        // inactive slots are not attended
      if (greedy) {
        rounds[pi] = units ? units - kPairOverheadUnits : 0;
        if (units) atomicAdd(&cost_total, (units - kPairOverheadUnits) * kRoundCost + kPairStartCost);
      }
    }
    scan[tid] = units;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {           // inclusive scan
      const int add = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += add;
      __syncthreads();
    }
    if (pi < dv.n_pairs) unit_start[pi + 1] = carry + scan[tid];
    __syncthreads();
    if (tid == 1023) carry += scan[1023];
    __syncthreads();
  }
  const int total = carry;
  __threadfence_block();
  __syncthreads();
  WgDesc* wd = dv.wg_desc + (int64_t)layer * kMaxWorkgroups;
  auto nop2 = [](int, int) {};

  if (greedy) {
    // Smallest workgroup capacity whose greedy deal fits the grid: candidates from the average cost
    // upward, one per thread, each an independent sequential walk over the pairs.
    int lowest = (cost_total + dv.n_wg - 1) / dv.n_wg;
    if (lowest < kPairStartCost + kRoundCost) lowest = kPairStartCost + kRoundCost;
    for (int base = 0; best_cap == 0x7fffffff; base += 256) {
      if (tid < 256) {
        const int cap = lowest + base + tid;
        if (deal_rounds<false>(rounds, unit_start, dv.n_pairs, cap, nop2, nop2, nop2) <= dv.n_wg) atomicMin(&best_cap, cap);
      }
      __syncthreads();
    }
    // the shares themselves: one more walk, by one thread
    for (int w = tid; w < dv.n_wg; w += 1024) { wd[w].u_begin = 0; wd[w].u_end = 0; wd[w].first_pair = 0; wd[w].pad = 0; }
    __syncthreads();
    if (tid == 0) {
      int first_unit = 0;
      for (int p = 0; p < dv.n_pairs; ++p) if (rounds[p]) { first_unit = unit_start[p]; break; }
      wd[0].u_begin = first_unit;
      const int used_wgs = deal_rounds<true>(
          rounds, unit_start, dv.n_pairs, best_cap,
          [&](int w, int u) { wd[w].u_end = u; wd[w + 1].u_begin = u; },
          [&](int p, int w) { seg_first[p] = w; },
          [&](int p, int w) { seg_count[p] = w - seg_first[p] + 1; });
      wd[used_wgs - 1].u_end = total;
      if (total == 0) { wd[0].u_begin = 0; wd[0].u_end = 0; }
    }
    __threadfence_block();
    __syncthreads();
  }

  int per_wg = (total + dv.n_wg - 1) / dv.n_wg;      // equal unit counts: the fallback for very many pairs
  if (per_wg < 1) per_wg = 1;
  auto describe = [&](int pi) {
    const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
    const bool full = dv.full_mask[layer * dv.n_kv_heads + h] != 0;
    PairDesc d;
    d.koff = dv.store_off[((int64_t)layer * dv.batch + b) * dv.n_kv_heads + h];
    d.cap = full ? dv.cap_pad[b] : dv.window_pad;
    d.n_build = len_in[b];
    d.unit_start = unit_start[pi];
    d.unit_end = unit_start[pi + 1];
    d.full = full ? 1 : 0;
    d.gate = full ? dv.gate[layer * dv.n_kv_heads + h] : 1.f;
    if (greedy) {
      d.wg_first = d.unit_end > d.unit_start ? seg_first[pi] : 0;
      d.n_seg = d.unit_end > d.unit_start ? seg_count[pi] : 0;
    } else {
      d.wg_first = d.unit_end > d.unit_start ? d.unit_start / per_wg : 0;
      d.n_seg = d.unit_end > d.unit_start ? (d.unit_end - 1) / per_wg - d.wg_first + 1 : 0;
    }
    return d;
  };
  PairDesc* pd = dv.pair_desc + (int64_t)layer * dv.n_pairs;
  for (int pi = tid; pi < dv.n_pairs; pi += 1024) pd[pi] = describe(pi);
  // every workgroup's share and the pair that holds its first tile
  for (int w = tid; w < dv.n_wg; w += 1024) {
    WgDesc d;
    if (greedy) {
      d.u_begin = wd[w].u_begin;
      d.u_end = wd[w].u_end;
    } else {
      const int t = w * per_wg;
      d.u_begin = t;
      d.u_end = t + per_wg < total ? t + per_wg : total;
    }
    d.pad = 0;
    if (d.u_begin >= d.u_end) {
      d.first_pair = 0;
      d.u_begin = d.u_end = 0;
      d.first = PairDesc{0, 0, 0, 0, 0, 0, 0, 1.f, 0};
    } else {
      int lo = 0, hi = dv.n_pairs;     // the pair with unit_start[lo] <= u_begin < unit_start[lo + 1]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (unit_start[mid] <= d.u_begin) lo = mid; else hi = mid;
      }
      d.first_pair = lo;
      d.first = describe(lo);
    }
    wd[w] = d;
  }
}

// One block per (pair, query head of the group), one thread per output dimension.
template <typename T>
__global__ __launch_bounds__(kHeadDim) void combine_kernel(DeviceView dv, int layer, T* __restrict__ out) {
  __shared__ float sm_scale[kHeadDim];
  __shared__ float sm_red[2];
  const int pi = blockIdx.x, g = blockIdx.y, d = threadIdx.x;
  const PairDesc pd = dv.pair_desc[(int64_t)layer * dv.n_pairs + pi];
  const int nseg = pd.n_seg;
  if (nseg <= 1) return;                // no units (inactive slot), or a single workgroup wrote the final output itself
  const int G = dv.group;
  const int64_t slot0 = (int64_t)pd.wg_first + pi;       // partial slots of this pair are consecutive
  // a gated full head (Eq. 1) has two sets of partials: full attention and local attention
  const int n_sets = (pd.full && pd.gate < 1.f) ? 2 : 1;
  float r = 0.f;
  for (int set = 0; set < n_sets; ++set) {
    const float* part_m = dv.part_m + set * dv.part_set_ml;
    const float* part_l = dv.part_l + set * dv.part_set_ml;
    const float* part_o = dv.part_o + set * dv.part_set_o;
    __syncthreads();
    constexpr int kFew = 16;
    if (nseg <= kFew) {
      // The usual case, a handful of partials: every load is issued before anything is waited for
      // (this kernel is a chain of memory latencies and little else), one barrier, same ascending
      // order of accumulation as the general path below.
      const float* po = part_o + (slot0 * G + g) * kHeadDim + d;
      float o[kFew];
#pragma unroll
      for (int j = 0; j < kFew; ++j) o[j] = j < nseg ? po[(int64_t)j * G * kHeadDim] : 0.f;
      float mw = -INFINITY, lw = 0.f;
      if (d < nseg) { mw = part_m[(slot0 + d) * G + g]; lw = part_l[(slot0 + d) * G + g]; }
      if (d < 64) {                       // the first wavefront holds all the (m, l) pairs in lanes 0 .. nseg - 1
        float M = mw;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
        const float sc = mw == -INFINITY ? 0.f : exp2f(mw - M);
        float ls = sc * lw;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) ls += __shfl_xor(ls, off);
        if (d < kFew) sm_scale[d] = sc;
        if (d == 0) sm_red[0] = ls;
      }
      __syncthreads();
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < kFew; ++j) acc += sm_scale[j] * o[j];      // scale is 0 beyond nseg
      const float res = acc / sm_red[0];
      r = n_sets == 1 ? res : (set == 0 ? pd.gate * res : r + (1.f - pd.gate) * res);
      continue;
    }
    // maximum over the partial maxima
    float M = -INFINITY;
    for (int i = d; i < nseg; i += kHeadDim) M = fmaxf(M, part_m[(slot0 + i) * G + g]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    if ((d & 63) == 0) sm_red[d >> 6] = M;
    __syncthreads();
    M = fmaxf(sm_red[0], sm_red[1]);
    float acc = 0.f, L = 0.f;
    for (int base = 0; base < nseg; base += kHeadDim) {       // chunks of 128 partials, ascending order
      __syncthreads();
      const int i = base + d;
      float sc = 0.f, ls = 0.f;
      if (i < nseg) {
        const float mw = part_m[(slot0 + i) * G + g];
        sc = mw == -INFINITY ? 0.f : exp2f(mw - M);
        ls = sc * part_l[(slot0 + i) * G + g];
      }
      sm_scale[d] = sc;
      // normaliser: fixed-order tree over the chunk
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) ls += __shfl_xor(ls, off);
      __syncthreads();
      if ((d & 63) == 0) sm_red[d >> 6] = ls;
      __syncthreads();
      L += sm_red[0] + sm_red[1];
      const int cnt = nseg - base < kHeadDim ? nseg - base : kHeadDim;
      const float* po = part_o + ((slot0 + base) * G + g) * kHeadDim + d;
      int j = 0;
      for (; j + 4 <= cnt; j += 4) {
        const float a0 = po[(int64_t)(j + 0) * G * kHeadDim], a1 = po[(int64_t)(j + 1) * G * kHeadDim];
        const float a2 = po[(int64_t)(j + 2) * G * kHeadDim], a3 = po[(int64_t)(j + 3) * G * kHeadDim];
        acc += sm_scale[j] * a0; acc += sm_scale[j + 1] * a1; acc += sm_scale[j + 2] * a2; acc += sm_scale[j + 3] * a3;
      }
      for (; j < cnt; ++j) acc += sm_scale[j] * po[(int64_t)j * G * kHeadDim];
    }
    const float res = acc / L;
    r = n_sets == 1 ? res : (set == 0 ? pd.gate * res : r + (1.f - pd.gate) * res);
  }
  const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
  const int64_t o = ((int64_t)b * dv.n_q_heads + h * G + g) * kHeadDim + d;
  if (sizeof(T) == 4) reinterpret_cast<float*>(out)[o] = r;
  else reinterpret_cast<uint16_t*>(out)[o] = f32_to_bf16_rne(r);
}

}  // namespace

hipError_t launch_build_worklist(const DeviceView& dv, int layer, const int32_t* len_in, int slack,
                                 hipStream_t stream) {
  hipLaunchKernelGGL(build_worklist_kernel, dim3(1), dim3(1024), 0, stream, dv, layer, len_in, slack);
  return hipGetLastError();
}

hipError_t launch_combine(const DeviceView& dv, int layer, void* out, hipStream_t stream) {
  if (dv.dtype == RLKV_F32)
    hipLaunchKernelGGL(combine_kernel<float>, dim3(dv.n_pairs, dv.group), dim3(kHeadDim), 0, stream, dv, layer, (float*)out);
  else
    hipLaunchKernelGGL(combine_kernel<uint16_t>, dim3(dv.n_pairs, dv.group), dim3(kHeadDim), 0, stream, dv, layer,
                       (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace rlkv
