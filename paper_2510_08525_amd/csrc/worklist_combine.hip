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
#include "rlkv_internal.h"

namespace rlkv {
namespace {

__global__ __launch_bounds__(1024) void build_worklist_kernel(DeviceView dv, int layer) {
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
      const int n = dv.len[layer * dv.batch + b];
      const bool full = dv.full_mask[layer * dv.n_kv_heads + h] != 0;
      const int n_eff = full ? n : (n < dv.window ? n : dv.window);
      tiles = (n_eff + kTile - 1) / kTile;
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

// One block per pair, one thread per output dimension.
template <typename T>
__global__ __launch_bounds__(kHeadDim) void combine_kernel(DeviceView dv, int layer, T* __restrict__ out) {
  const int pi = blockIdx.x, d = threadIdx.x;
  const int* tile_start = dv.tile_start + (int64_t)layer * (dv.n_pairs + 1);
  const int per_wg = dv.wl_meta[layer * 4 + 1];
  const int ts = tile_start[pi], te = tile_start[pi + 1];
  if (te <= ts) return;
  const int w0 = ts / per_wg, w1 = (te - 1) / per_wg;
  if (w0 == w1) return;                 // a single workgroup wrote the final output itself
  const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
  const int G = dv.group;
  for (int g = 0; g < G; ++g) {
    float M = -INFINITY;
    for (int w = w0; w <= w1; ++w) M = fmaxf(M, dv.part_m[(int64_t)(w + pi) * G + g]);
    float acc = 0.f, L = 0.f;
    for (int w = w0; w <= w1; ++w) {
      const int64_t slot = w + pi;
      const float mw = dv.part_m[slot * G + g];
      const float sc = mw == -INFINITY ? 0.f : exp2f(mw - M);
      L += sc * dv.part_l[slot * G + g];
      acc += sc * dv.part_o[(slot * G + g) * kHeadDim + d];
    }
    const float r = acc / L;
    const int64_t o = ((int64_t)b * dv.n_q_heads + h * G + g) * kHeadDim + d;
    if (sizeof(T) == 4) reinterpret_cast<float*>(out)[o] = r;
    else reinterpret_cast<uint16_t*>(out)[o] = f32_to_bf16_rne(r);
  }
}

}  // namespace

hipError_t launch_build_worklist(const DeviceView& dv, int layer, hipStream_t stream) {
  hipLaunchKernelGGL(build_worklist_kernel, dim3(1), dim3(1024), 0, stream, dv, layer);
  return hipGetLastError();
}

hipError_t launch_combine(const DeviceView& dv, int layer, void* out, hipStream_t stream) {
  if (dv.dtype == RLKV_F32)
    hipLaunchKernelGGL(combine_kernel<float>, dim3(dv.n_pairs), dim3(kHeadDim), 0, stream, dv, layer, (float*)out);
  else
    hipLaunchKernelGGL(combine_kernel<uint16_t>, dim3(dv.n_pairs), dim3(kHeadDim), 0, stream, dv, layer,
                       (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace rlkv
