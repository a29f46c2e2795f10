// Split-K decode attention, vector-ALU variant (row-major stores; fp32 and bf16).
//
// For every (sequence, KV head) pair the kernel computes ordinary softmax attention of
// the G query heads of the group over the rows the store holds (paper Sec. 3.1 Eq. 1 with
// the gate at 0 or 1; Sec. 3.3: compressed heads run full attention over their
// compressed cache).  A store's valid rows are always the prefix [0, n_eff), and softmax
// attention does not depend on the order of the rows, so ring slots are read in slot
// order.
//
// Mapping: a wavefront reads whole rows with 128-bit loads (16 lanes cover a 256-byte
// bf16 row, 32 lanes a 512-byte fp32 row); every lane keeps the 8 (4) elements of its
// column chunk of Q for all heads of the group, so a K/V row is loaded once per group.
// Dot products are reduced across the lanes of a row with DPP row rotations; each group
// of lanes that shares a row index runs its own online softmax, and the streams are
// merged at the end of the segment (lane groups by shuffles, wavefronts through LDS).
#include "rlkv_internal.h"

namespace rlkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ inline float dpp_mov(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane receives the total.
__device__ inline float row_sum16(float x) {
  x += dpp_mov<0x128>(x);  // row_ror:8
  x += dpp_mov<0x124>(x);  // row_ror:4
  x += dpp_mov<0x122>(x);  // row_ror:2
  x += dpp_mov<0x121>(x);  // row_ror:1
  return x;
}

// Element types.  `Q` is what a lane keeps of a query row (its column chunk) and `dot` the lane's part of
// <q, k> for one K row as loaded: fp32 multiplies and adds the unpacked elements; bf16 leaves both rows packed
// and takes two products per instruction (v_dot2c_f32_bf16: exact products, fp32 accumulation), which spares
// the unpacking of K and half of the multiply-adds - this kernel is bound by its vector instruction count.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerLane = 4;
  struct Q { float f[4]; };
  __device__ static void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static Q query(const uint4& r) { Q q; unpack(r, q.f); return q; }
  __device__ static float dot(const Q& q, const uint4& k) {
    float kf[4];
    unpack(k, kf);
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) d = fmaf(q.f[e], kf[e], d);
    return d;
  }
};
template <> struct Elem<uint16_t> {
  static constexpr int kPerLane = 8;
  struct Q { uint4 packed; };
  __device__ static void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static Q query(const uint4& r) { return Q{r}; }
  __device__ static float dot(const Q& q, const uint4& k) {
    float d = 0.f;
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.packed.x), __builtin_bit_cast(bf16x2, k.x), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.packed.y), __builtin_bit_cast(bf16x2, k.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.packed.z), __builtin_bit_cast(bf16x2, k.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.packed.w), __builtin_bit_cast(bf16x2, k.w), d, false);
    return d;
  }
};

__device__ inline float exp2_or_zero(float m, float ref) {
  // 2^(m - ref) with the convention that an empty stream (m = -inf) weighs nothing
  return m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - ref);
}

template <typename T, int GB>
__global__ __launch_bounds__(kBlock) void decode_valu_kernel(DeviceView dv, int layer,
                                                             const T* __restrict__ q, T* __restrict__ out,
                                                             float scale_log2, int appended) {
  constexpr int EPL = Elem<T>::kPerLane;        // elements per lane per 128-bit load
  constexpr int LPR = kHeadDim / EPL;           // lanes per row
  constexpr int RPL = 64 / LPR;                 // rows per wavefront load
  constexpr int U = 4;                          // row loads in flight per K and per V
  constexpr int kBatches = kTile / (RPL * U);

  __shared__ float sm_o[4][GB][kHeadDim];
  __shared__ float sm_m[4][GB];
  __shared__ float sm_l[4][GB];

  const int wg = blockIdx.x;
  const WgDesc* __restrict__ wdp = wg_desc_of(dv, layer) + wg;
  // tokens since the list was planned (`appended`: by this step's append launch, not counted there yet)
  const int grow = list_header(dv, layer)->grow + appended;
  const int u_begin = wdp->u_begin, u_end = wdp->u_end;
  if (u_begin >= u_end) return;
  int pi = wdp->first_pair;
  PairDesc pd = wdp->first;
  const PairDesc* __restrict__ pairs = pair_desc_of(dv, layer);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane % LPR, rg = lane / LPR;
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
    PairDesc pd_next = pd;
    if (seg_end < u_end) pd_next = pairs[pi + 1];     // fetched early, looked at after the segment

    const int b = pi / dv.n_kv_heads, h = pi % dv.n_kv_heads;
    const int n = pd.n_build + grow;
    const bool full = pd.full != 0;
    const int n_eff = full ? n : (n < dv.window ? n : dv.window);
    const char* kst = dv.kv_base + pd.koff;
    const char* vst = kst + (int64_t)pd.cap * dv.row_bytes;
    // the list was built with room to grow: tiles past the valid prefix are still empty
    const int tiles_valid = (n_eff + kTile - 1) / kTile;
    const int tile_hi = r_hi * kRound < tiles_valid ? r_hi * kRound : tiles_valid;

    for (int gb = 0; gb < G; gb += GB) {
      const int gcount = G - gb < GB ? G - gb : GB;
      typename Elem<T>::Q qf[GB];
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        uint4 r = make_uint4(0, 0, 0, 0);                  // (no such head: zeros, in either element type)
        if (g < gcount) {
          const int64_t qrow = (int64_t)b * dv.n_q_heads + h * G + gb + g;
          r = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(q) + (qrow * kHeadDim + c * EPL) * sizeof(T));
        }
        qf[g] = Elem<T>::query(r);
      }

      // Eq. 1 gate: a full head with gate < 1 takes a second, local pass over the tiles of this
      // segment that hold sink or recent positions; out = gate * full + (1 - gate) * local.
      const bool two_pass = full && pd.gate < 1.f;
      const int keep_lo = dv.sink, keep_from = n - dv.recent;        // local pass: row < S or row >= n - R
      const int sink_tiles = (keep_lo + kTile - 1) / kTile;
      const int recent_tile0 = keep_from > 0 ? keep_from / kTile : 0;
      float held[(GB * kHeadDim + kBlock - 1) / kBlock];             // full-pass results of a whole-pair segment
      for (int pass = 0; pass < (two_pass ? 2 : 1); ++pass) {
      float m[GB], l[GB], acc[GB][EPL];
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
      }

      for (int tile = tile_lo + wave; tile < tile_hi; tile += 4) {
        if (pass == 1 && tile >= sink_tiles && tile < recent_tile0) {
          tile += (recent_tile0 - tile - 1) / 4 * 4;                   // hop over the evicted middle
          continue;
        }
        const int tok0 = tile * kTile;
#pragma unroll 1
        for (int bt = 0; bt < kBatches; ++bt) {
          uint4 kr[U], vr[U];
          bool valid[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int tok = tok0 + (bt * U + u) * RPL + rg;
            valid[u] = tok < n_eff && (pass == 0 || tok < keep_lo || tok >= keep_from);
            const int tc = valid[u] ? tok : n_eff - 1;       // stay inside the valid prefix
            const int64_t off = (int64_t)tc * dv.row_bytes + c * 16;
            // rows are read once per step: stream them past the caches
            const u32x4 kk = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kst + off));
            const u32x4 vv = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vst + off));
            kr[u] = make_uint4(kk.x, kk.y, kk.z, kk.w);
            vr[u] = make_uint4(vv.x, vv.y, vv.z, vv.w);
          }
          float s[U][GB];
#pragma unroll
          for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int g = 0; g < GB; ++g) {
              float d = Elem<T>::dot(qf[g], kr[u]);
              d = row_sum16(d);
              if (LPR == 32) d += __shfl_xor(d, 16);
              s[u][g] = valid[u] ? d * scale_log2 : -INFINITY;
            }
          }
          float p[U][GB];
#pragma unroll
          for (int g = 0; g < GB; ++g) {
            float mx = s[0][g];
#pragma unroll
            for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][g]);
            const float m_new = fmaxf(m[g], mx);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m[g] - m_ref);   // 2^-inf = 0 for a fresh stream
            m[g] = m_new;
            float ps_ = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
              p[u][g] = __builtin_amdgcn_exp2f(s[u][g] - m_ref);
              ps_ += p[u][g];
            }
            l[g] = l[g] * alpha + ps_;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
          }
#pragma unroll
          for (int u = 0; u < U; ++u) {
            float vf[EPL];
            Elem<T>::unpack(vr[u], vf);
#pragma unroll
            for (int g = 0; g < GB; ++g)
#pragma unroll
              for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p[u][g], vf[e], acc[g][e]);
          }
        }
      }

      // merge the lane groups of the wavefront (they hold the same column chunk)
#pragma unroll
      for (int mask = LPR; mask < 64; mask <<= 1) {
#pragma unroll
        for (int g = 0; g < GB; ++g) {
          const float mo = __shfl_xor(m[g], mask);
          const float M = fmaxf(m[g], mo);
          const float a = exp2_or_zero(m[g], M), bsc = exp2_or_zero(mo, M);
          l[g] = l[g] * a + __shfl_xor(l[g], mask) * bsc;
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] = acc[g][e] * a + __shfl_xor(acc[g][e], mask) * bsc;
          m[g] = M;
        }
      }
      __syncthreads();   // previous segment's readers are done with the LDS buffers
      if (rg == 0) {
#pragma unroll
        for (int g = 0; g < GB; ++g) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) sm_o[wave][g][c * EPL + e] = acc[g][e];
          if (c == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
        }
      }
      __syncthreads();
      // merge the four wavefronts; emit the final output or a partial for the combine pass
      int it = 0;
      for (int idx = tid; idx < gcount * kHeadDim; idx += kBlock, ++it) {
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
          const int64_t o = ((int64_t)b * dv.n_q_heads + h * G + gb + g) * kHeadDim + d;
          float r = O / L;
          if (two_pass) {
            if (pass == 0) { held[it] = r; continue; }
            r = pd.gate * held[it] + (1.f - pd.gate) * r;
          }
          if (sizeof(T) == 4) reinterpret_cast<float*>(out)[o] = r;
          else reinterpret_cast<uint16_t*>(out)[o] = f32_to_bf16_rne(r);
        } else {
          const int64_t slot = (int64_t)wg + pi;
          dv.part_o[pass * dv.part_set_o + (slot * G + gb + g) * kHeadDim + d] = O;
          if (d == 0) {
            dv.part_m[pass * dv.part_set_ml + slot * G + gb + g] = M;
            dv.part_l[pass * dv.part_set_ml + slot * G + gb + g] = L;
          }
        }
      }
      }   // pass
    }
    u = seg_end;
    ++pi;
    pd = pd_next;
    if (u < u_end)
      while (pd.unit_end <= u) pd = pairs[++pi];       // pairs of inactive slots own no units
  }
}

template <typename T>
hipError_t launch_t(const DeviceView& dv, int layer, const void* q, void* out, float scale_log2,
                    hipStream_t stream, hipEvent_t e0, hipEvent_t e1, int appended) {
  const dim3 grid(dv.n_wg), block(kBlock);
  const T* qp = (const T*)q;
  T* op = (T*)out;
  const int G = dv.group;
  // (without events: the plain launch, which a stream capture can record)
#define RLKV_LAUNCH_VALU(GB)                                                                                         \
  do {                                                                                                               \
    if (e0 || e1)                                                                                                    \
      hipExtLaunchKernelGGL((decode_valu_kernel<T, GB>), grid, block, 0, stream, e0, e1, 0, dv, layer, qp, op,      \
                            scale_log2, appended);                                                                   \
    else                                                                                                             \
      hipLaunchKernelGGL((decode_valu_kernel<T, GB>), grid, block, 0, stream, dv, layer, qp, op, scale_log2,        \
                         appended);                                                                                  \
  } while (0)
  if (G <= 1) RLKV_LAUNCH_VALU(1);
  else if (G <= 2) RLKV_LAUNCH_VALU(2);
  else if (G <= 4) RLKV_LAUNCH_VALU(4);
  else if (G == 7) RLKV_LAUNCH_VALU(7);
  else RLKV_LAUNCH_VALU(8);
#undef RLKV_LAUNCH_VALU
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_valu(const DeviceView& dv, int layer, bool /*gated: decided per pair*/,
                              const void* q, void* out, float scale_log2, hipStream_t stream, hipEvent_t ev_start,
                              hipEvent_t ev_stop, int appended) {
  return dv.dtype == RLKV_F32 ? launch_t<float>(dv, layer, q, out, scale_log2, stream, ev_start, ev_stop, appended)
                              : launch_t<uint16_t>(dv, layer, q, out, scale_log2, stream, ev_start, ev_stop, appended);
}

}  // namespace rlkv
