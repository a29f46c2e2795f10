// Pieces shared by the MFMA attention kernels (decode and prefill): the register image of a
// 32-slot K/V tile of the tiled store layout, its loads, the score contraction, the online-softmax
// state, and the map from a tile index to its address (contiguous or paged store).
#pragma once

#include "rlkv_internal.h"

namespace rlkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

union Frag {
  uint4 u;
  bf16x8 v;
  f16x8 h;
  u32x4 w;
};

struct TileRegs {
  Frag k[2][4];   // [16-slot half][32-wide d step]
  Frag v[8];      // [16-wide d block]
};

// K/V rows are read exactly once per step: non-temporal loads keep them from displacing
// anything in the caches on the way (measured: +12 % achieved HBM bandwidth).
__device__ __forceinline__ void load_tile(TileRegs& r, const char* tile_base, int lane) {
  const char* kb = tile_base + lane * 16;
  const char* vb = kb + 8192;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int s = 0; s < 4; ++s) r.k[hf][s].w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + hf * 4096 + s * 1024));
#pragma unroll
  for (int j = 0; j < 8; ++j) r.v[j].w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + j * 1024));
}

__device__ __forceinline__ float exp2_or_zero(float m, float ref) {
  return m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - ref);
}

// Online-softmax state of one wavefront for one (pair, share) segment.
struct Softmax {
  float m;          // running maximum of head lane%16 (log2 domain; same in all four k-groups)
  float l;          // this lane's share of the normaliser
  floatx4 o[8];     // O[head 4*(lane/16) + r][d = 16*j + lane%16]
};

// Raw scores of one 32-slot tile: lane l receives head l%16, slots 4*(l/16)..+3 of each half.
__device__ __forceinline__ void tile_scores(const TileRegs& t, const Frag (&qb)[4], float scale_log2, float (&raw)[8]) {
  floatx4 s0 = floatx4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[0][s].v, qb[s].v, s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[1][s].v, qb[s].v, s1, 0, 0, 0);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) raw[e] = (e < 4 ? s0[e] : s1[e - 4]) * scale_log2;
}

// Online-softmax update of `st` with the masked scores `sc` of one tile (-inf = does not count;
// layout as tile_scores leaves them) and accumulation of P.V.  The 16 columns of the score tile
// are heads (decode) or (query position, head) pairs (prefill); lane l tracks column l%16.  P is
// split into a bf16 head and a bf16 remainder so the weights carry ~16 mantissa bits.
__device__ __forceinline__ void softmax_pv(const TileRegs& t, const float (&sc)[8], Softmax& st, int kb) {
  float mx = sc[0];
#pragma unroll
  for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[e]);
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(st.m, mx);
  const float m_ref = m_new == -INFINITY ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_ref);
  st.m = m_new;
  float p[8], psum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    p[e] = __builtin_amdgcn_exp2f(sc[e] - m_ref);
    psum += p[e];
  }
  st.l = st.l * alpha + psum;
  bf16x8 phi, plo;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    phi[e] = (__bf16)p[e];
    plo[e] = (__bf16)(p[e] - (float)phi[e]);
  }
  if (__any(alpha != 1.f)) {
    // the output accumulator holds heads 4*kb + r: fetch their factors from lanes 0..15
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float a = __shfl(alpha, kb * 4 + r);
#pragma unroll
      for (int j = 0; j < 8; ++j) st.o[j][r] *= a;
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    st.o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi, t.v[j].v, st.o[j], 0, 0, 0);
    st.o[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo, t.v[j].v, st.o[j], 0, 0, 0);
  }
}

// Where the tiles of one pair's store live.  Contiguous store: tile t at base + t * 16 KiB.
// Paged full head (PAGED; Sec. 4.3): base is the head's pool and the sequence's block-table row
// names the page of every run of 2^shift tiles.  The tile index is the same in all lanes of a
// wavefront, so the table entry comes through a scalar load.
template <bool PAGED>
struct TileMap {
  char* base;
  const int32_t* row;     // block-table row of the sequence (paged pairs only)
  int64_t page_bytes;
  int shift, mask, last;  // last = highest valid index into row
  bool paged;
  __device__ __forceinline__ char* at(int tile) const {
    if (PAGED && paged) {
      int idx = __builtin_amdgcn_readfirstlane(tile) >> shift;
      idx = idx < last ? idx : last;      // look-ahead may run past the row: stay inside it
      return base + row[idx] * page_bytes + (int64_t)(tile & mask) * kTileBytes;
    }
    return base + (int64_t)tile * kTileBytes;
  }
};

}  // namespace rlkv
