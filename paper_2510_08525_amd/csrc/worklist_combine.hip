// Work-list build and split-K merge for decode attention over the head-mixed cache.
//
// One work list covers both head types: every (sequence, KV head) pair contributes
// ceil(n_eff / 32) tiles, n_eff = n for a full head and min(n, sink + recent) for a
// compressed one (the residual cost s*W/L of Sec. 4.3).  A workgroup's four wavefronts
// take one tile each per round, and a wavefront's time is set by the number of rounds it
// waits for, so the unit of scheduling is the round: ceil(tiles / 4) units per pair, plus
// kPairOverheadUnits that stand for the pair's fixed cost (pipeline restart, Q load, merge, output write).  The
// units of all pairs are laid end to end and cut into equal contiguous shares, one per
// workgroup, so a tiny compressed head costs a workgroup exactly its rounds and nothing
// idles behind a long full head.  A workgroup whose share crosses pair boundaries emits one partial per
// pair it touches, in slot (workgroup index + pair index); the merge below walks them in
// ascending workgroup order, so the result is deterministic.
//
// A list is built for the lengths of the moment plus `slack` tokens of growth, so the
// decode steps that follow (one token per sequence each) reuse it; the attention kernels
// skip tiles that are still empty.  The host rebuilds it when the slack is used up.
#include "rlkv_internal.h"

namespace rlkv {
namespace {

__global__ __launch_bounds__(1024) void build_worklist_kernel(DeviceView dv, int layer,
                                                              const int32_t* __restrict__ len_in, int slack) {
  __shared__ int scan[1024];
  __shared__ int carry;
  const int tid = threadIdx.x;
  int* unit_start = dv.unit_start + (int64_t)layer * (dv.n_pairs + 1);
  if (tid == 0) { carry = 0; unit_start[0] = 0; }
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
  int per_wg = (total + dv.n_wg - 1) / dv.n_wg;
  if (per_wg < 1) per_wg = 1;
  __threadfence_block();
  __syncthreads();
  auto describe = [&](int pi) {
    const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
    const bool full = dv.full_mask[layer * dv.n_kv_heads + h] != 0;
    PairDesc d;
    d.koff = dv.store_off[((int64_t)layer * dv.batch + b) * dv.n_kv_heads + h];
    d.cap = full ? dv.cap_pad[b] : dv.window_pad;
    d.n_build = len_in[b];
    d.unit_start = unit_start[pi];
    d.unit_end = unit_start[pi + 1];
    d.per_wg = per_wg;
    d.full = full ? 1 : 0;
    d.gate = full ? dv.gate[layer * dv.n_kv_heads + h] : 1.f;
    d.pad = 0;
    return d;
  };
  PairDesc* pd = dv.pair_desc + (int64_t)layer * dv.n_pairs;
  for (int pi = tid; pi < dv.n_pairs; pi += 1024) pd[pi] = describe(pi);
  // every workgroup's share and the pair that holds its first tile
  WgDesc* wd = dv.wg_desc + (int64_t)layer * kMaxWorkgroups;
  for (int w = tid; w < dv.n_wg; w += 1024) {
    WgDesc d;
    const int t = w * per_wg;
    d.u_begin = t;
    d.u_end = t + per_wg < total ? t + per_wg : total;
    d.pad = 0;
    if (t >= total) {
      d.first_pair = 0;
      d.u_begin = d.u_end = 0;
      d.first = PairDesc{0, 0, 0, 0, 0, per_wg, 0, 1.f, 0};
    } else {
      int lo = 0, hi = dv.n_pairs;     // the pair with unit_start[lo] <= t < unit_start[lo + 1]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (unit_start[mid] <= t) lo = mid; else hi = mid;
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
  const int per_wg = pd.per_wg;
  const int ts = pd.unit_start, te = pd.unit_end;
  if (te <= ts) return;
  const int w0 = ts / per_wg, w1 = (te - 1) / per_wg;
  if (w0 == w1) return;                 // a single workgroup wrote the final output itself
  const int G = dv.group;
  const int nseg = w1 - w0 + 1;
  const int64_t slot0 = (int64_t)w0 + pi;       // partial slots of this pair are consecutive
  // a gated full head (Eq. 1) has two sets of partials: full attention and local attention
  const int n_sets = (pd.full && pd.gate < 1.f) ? 2 : 1;
  float r = 0.f;
  for (int set = 0; set < n_sets; ++set) {
    const float* part_m = dv.part_m + set * dv.part_set_ml;
    const float* part_l = dv.part_l + set * dv.part_set_ml;
    const float* part_o = dv.part_o + set * dv.part_set_o;
    __syncthreads();
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
