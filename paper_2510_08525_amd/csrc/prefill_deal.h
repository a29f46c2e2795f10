// Which (x, y) block of a prefill attention launch a workgroup works on, given its linear index in the grid.
// Shared by the kernel and the host-side planning entry point (which exists so that this arithmetic can be
// checked without a GPU).
#pragma once
#include <hip/hip_runtime.h>

namespace rlkv {

// Workgroups are dealt to the 8 XCDs in turn by their linear index, and each XCD has an L2 of its own.  All the
// workgroups of a grid row (one sequence, one KV head) read the same tiles, so whole rows are kept on one XCD
// where that leaves the XCDs equally loaded.  The rows come sorted: first the `heavy` rows (full heads of
// sequences that have a chunk, long to short), then the light ones (compressed heads, sequences without a
// chunk); the host names the leading `dealt` heavy rows (a multiple of 8) whose groups of 8 are alike enough
// to go one row per XCD.  Each XCD takes, in this order: its rows of the dealt heavy rows (row y on XCD
// y % 8); its eighth of the workgroups of the other heavy rows, dealt one by one; its rows of the light rows,
// likewise; its eighth of the up to 7 light rows left over.  The two parts dealt one by one form one list
// dealt in turn, so every XCD ends up with exactly the workgroups the hardware hands it: a bijection of the
// grid's (x, y) plane for any grid size and any counts.  `lin` = blockIdx.x + gx * blockIdx.y of a gx x gy
// grid; returns the (x, y) block index to work on.
__host__ __device__ inline void prefill_deal(int lin, int gx, int gy, int dealt, int heavy, int& bx, int& by) {
  const int k = lin & 7;
  int idx = lin >> 3;
  const int F = heavy < gy ? (heavy > 0 ? heavy : 0) : gy;
  const int A = (dealt < F ? (dealt > 0 ? dealt : 0) : F) & ~7;
  const int ra = A >> 3, rc = (gy - F) >> 3;            // whole rows per XCD of either class
  const int n_b = (F - A) * gx;                         // workgroups of the heavy rows dealt one by one
  const int c_a = ra * gx, c_c = rc * gx;
  const int c_b = (n_b - k + 7) >> 3;                   // how many of them come to this XCD
  if (idx < c_a) { by = (idx / gx) * 8 + k; bx = idx % gx; return; }
  idx -= c_a;
  if (idx < c_b) { const int w = idx * 8 + k; by = A + w / gx; bx = w % gx; return; }
  idx -= c_b;
  if (idx < c_c) { by = F + (idx / gx) * 8 + k; bx = idx % gx; return; }
  idx -= c_c;
  const int w = (c_b + idx) * 8 + k - n_b;              // the dealt list goes on with the light rows left over
  by = F + 8 * rc + w / gx;
  bx = w % gx;
}

}  // namespace rlkv
