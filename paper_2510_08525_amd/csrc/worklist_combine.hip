// Work-list build and split-K merge for decode attention over the head-mixed cache.
//
// One work list covers both head types: every (sequence, KV head) pair contributes
// ceil(n_eff / 32) tiles, n_eff = n for a full head and min(n, sink + recent) for a
// compressed one (the residual cost s*W/L of Sec. 4.3).  The tiles of all pairs are
// laid end to end and cut into equal contiguous shares, one per workgroup, so a tiny
// compressed head costs a workgroup exactly its tiles and nothing idles behind a long
// full head.  A workgroup whose share crosses pair boundaries emits one partial per
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
  int* tile_start = dv.tile_start + (int64_t)layer * (dv.n_pairs + 1);
  if (tid == 0) { carry = 0; tile_start[0] = 0; }
  __syncthreads();
  for (int base = 0; base < dv.n_pairs; base += 1024) {
    const int pi = base + tid;
    int tiles = 0;
    if (pi < dv.n_pairs) {
      const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
      const int n = len_in[b];
      const bool full = dv.full_mask[layer * dv.n_kv_heads + h] != 0;
      const int limit = full ? dv.cap_pad[b] : dv.window;     // what the store can ever hold
      const int n_fut = n + slack < limit ? n + slack : limit;
      tiles = (n_fut + kTile - 1) / kTile;
    }
    scan[tid] = tiles;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {           // inclusive scan
      const int add = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += add;
      __syncthreads();
    }
    if (pi < dv.n_pairs) tile_start[pi + 1] = carry + scan[tid];
    __syncthreads();
    if (tid == 1023) carry += scan[1023];
    __syncthreads();
  }
  const int total = carry;
  int per_wg = (total + dv.n_wg - 1) / dv.n_wg;
  if (per_wg < kMinTilesPerWg) per_wg = kMinTilesPerWg;
  const int active = (total + per_wg - 1) / per_wg;
  int* meta = dv.wl_meta + layer * 4;
  if (tid == 0) { meta[0] = total; meta[1] = per_wg; meta[2] = active; meta[3] = 0; }
  __threadfence_block();
  __syncthreads();
  // first pair of every workgroup: the pair pi with tile_start[pi] <= w*per_wg < tile_start[pi+1]
  int* first = dv.wg_first_pair + (int64_t)layer * dv.n_wg;
  for (int w = tid; w < dv.n_wg; w += 1024) {
    const int t = w * per_wg;
    int lo = 0, hi = dv.n_pairs;     // answer in [lo, hi)
    if (t >= total) { first[w] = dv.n_pairs; continue; }
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (tile_start[mid] <= t) lo = mid; else hi = mid;
    }
    first[w] = lo;
  }
}

// One block per (pair, query head of the group), one thread per output dimension.
template <typename T>
__global__ __launch_bounds__(kHeadDim) void combine_kernel(DeviceView dv, int layer, T* __restrict__ out) {
  __shared__ float sm_scale[kHeadDim];
  __shared__ float sm_red[2];
  const int pi = blockIdx.x, g = blockIdx.y, d = threadIdx.x;
  const int* tile_start = dv.tile_start + (int64_t)layer * (dv.n_pairs + 1);
  const int per_wg = dv.wl_meta[layer * 4 + 1];
  const int ts = tile_start[pi], te = tile_start[pi + 1];
  if (te <= ts) return;
  const int w0 = ts / per_wg, w1 = (te - 1) / per_wg;
  if (w0 == w1) return;                 // a single workgroup wrote the final output itself
  const int G = dv.group;
  const int nseg = w1 - w0 + 1;
  const int64_t slot0 = (int64_t)w0 + pi;       // partial slots of this pair are consecutive
  // maximum over the partial maxima
  float M = -INFINITY;
  for (int i = d; i < nseg; i += kHeadDim) M = fmaxf(M, dv.part_m[(slot0 + i) * G + g]);
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
      const float mw = dv.part_m[(slot0 + i) * G + g];
      sc = mw == -INFINITY ? 0.f : exp2f(mw - M);
      ls = sc * dv.part_l[(slot0 + i) * G + g];
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
    const float* po = dv.part_o + ((slot0 + base) * G + g) * kHeadDim + d;
    int j = 0;
    for (; j + 4 <= cnt; j += 4) {
      const float a0 = po[(int64_t)(j + 0) * G * kHeadDim], a1 = po[(int64_t)(j + 1) * G * kHeadDim];
      const float a2 = po[(int64_t)(j + 2) * G * kHeadDim], a3 = po[(int64_t)(j + 3) * G * kHeadDim];
      acc += sm_scale[j] * a0; acc += sm_scale[j + 1] * a1; acc += sm_scale[j + 2] * a2; acc += sm_scale[j + 3] * a3;
    }
    for (; j < cnt; ++j) acc += sm_scale[j] * po[(int64_t)j * G * kHeadDim];
  }
  const float r = acc / L;
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
