// Split-K merge for decode attention over the head-mixed cache.
//
// A workgroup of the attention kernel whose share does not cover a whole pair leaves one partial
// (m, l, O) per pair it touches, in slot (workgroup index + pair index).  The workgroups of a pair
// are consecutive, and this kernel walks them in ascending order, so the result is deterministic.
#include <string.h>

#include "rlkv_internal.h"

namespace rlkv {
namespace {

// One block per (pair, query head of the group), one thread per output dimension.
// v_new (tiled bf16 caches, after a fused append + decode step): the V rows that step appended.  This
// kernel has time to spare, so it is the one that looks whether any of them lies beyond the fp16 range
// and raises the layer's flag for the prefill kernel (a test inside the attention kernel's append
// cost it 2 us per launch).
//
// IN_ARGS (a layer without gates, at most kMergeArgPairs pairs): what the kernel needs of a pair's record
// - its first partial slot and its number of partials - comes as one word per pair among the kernel
// arguments instead of from the record in memory, which takes one memory latency out of a kernel that
// is a chain of three of them.
struct MergeWords {
  uint32_t w[kMergeArgPairs];     // (first slot << 12) | partials
};
template <typename T, bool IN_ARGS>
__global__ __launch_bounds__(kHeadDim) void combine_kernel(DeviceView dv, int layer, T* __restrict__ out,
                                                           const uint16_t* __restrict__ v_new, MergeWords words,
                                                           int advance) {
  __shared__ float sm_scale[kHeadDim];
  __shared__ float sm_red[2];
  const int pi = blockIdx.x, g = blockIdx.y, d = threadIdx.x;
  // behind a fused append + decode launch: the list's growth counter follows the lengths (no kernel reads it
  // while this one runs; the next launch that does comes after it on the stream)
  if (advance != 0 && pi == 0 && g == 0 && d == 0) list_header(dv, layer)->grow += advance;
  PairDesc pd;
  if (IN_ARGS) {
    const uint32_t word = words.w[pi];
    pd.n_seg = (int32_t)(word & 0xfffu);
    pd.wg_first = (int32_t)(word >> 12) - pi;
    pd.full = 0;
    pd.gate = 1.f;
  } else {
    pd = pair_desc_of(dv, layer)[pi];
  }
  // The two loads of the range test are asked for here, side by side, and looked at (range_test) once the loads
  // of the partials are on their way too; the empty asm marks the place up to which the compiler must have issued
  // them (left alone it makes the second wait for the first, and the partials for both).
  const bool look = v_new != nullptr && g == 0;
  uint32_t act = 0, vn = 0;
  if (look) {
    act = dv.active[pi / dv.n_kv_heads];
    vn = v_new[(int64_t)pi * kHeadDim + d];
  }
  auto range_test = [&]() {
    asm volatile("" : "+v"(act), "+v"(vn));
    if (look && act != 0 && bf16_beyond_fp16(vn)) dv.v_wide[layer] = 1;
  };
  const int nseg = pd.n_seg;
  if (nseg <= 1) {                      // no units (inactive slot), or a single workgroup wrote the final output itself
    range_test();
    return;
  }
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
      if (set == 0) range_test();
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
    if (set == 0) range_test();
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

hipError_t launch_combine(const DeviceView& dv, int layer, void* out, hipStream_t stream, int advance, const void* v_new,
                          const uint32_t* merge_words) {
  const dim3 grid(dv.n_pairs, dv.group), block(kHeadDim);
  const uint16_t* vn = (dv.dtype != RLKV_F32 && dv.kernel == RLKV_KERNEL_MFMA) ? (const uint16_t*)v_new : nullptr;
  MergeWords words;
  const bool in_args = merge_words != nullptr && dv.n_pairs <= kMergeArgPairs;
  if (in_args) memcpy(words.w, merge_words, (size_t)dv.n_pairs * sizeof(uint32_t));
  if (dv.dtype == RLKV_F32) {
    if (in_args) hipLaunchKernelGGL((combine_kernel<float, true>), grid, block, 0, stream, dv, layer, (float*)out, vn, words, advance);
    else hipLaunchKernelGGL((combine_kernel<float, false>), grid, block, 0, stream, dv, layer, (float*)out, vn, words, advance);
  } else {
    if (in_args) hipLaunchKernelGGL((combine_kernel<uint16_t, true>), grid, block, 0, stream, dv, layer, (uint16_t*)out, vn, words, advance);
    else hipLaunchKernelGGL((combine_kernel<uint16_t, false>), grid, block, 0, stream, dv, layer, (uint16_t*)out, vn, words, advance);
  }
  return hipGetLastError();
}

}  // namespace rlkv
