/* CPU oracle for decode attention over a head-mixed KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct code written from the
 * paper's statement of the method; it keeps the COMPLETE K/V history of every head and
 * applies the definition (no ring buffer, no tiling, no online softmax).  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may build or call it.  It shares
 * no code, header, table or helper with the HIP library.
 *
 * What is computed, and where the paper states it:
 *   - full head      : softmax(scale * q.K^T) V over all cached positions 0..n-1
 *                      (Sec. 3.1, Eq. 1 with gate = 1; "scaled dot product attention").
 *   - compressed head: the same attention restricted to the retained tokens, i.e. the
 *                      first S sink positions and the last R positions
 *                      (Sec. 3.1 local mask with constant initial sink tokens and recent
 *                      tokens; Sec. 3.3 last paragraph; App. B "Local Attention
 *                      Implementation": first-S sink + recent-R local tokens).
 *   - GQA            : the full/compressed choice is per KV head and every query head of
 *                      the group follows it (Sec. 3.1: one gate per KV head).
 *   - gated mixture  : gate * full + (1 - gate) * local per KV head (Sec. 3.1, Eq. 1), the form
 *                      used while the gates are still continuous (rollouts of Sec. 3.2).
 *   - prefill        : row i of the causal mask (full head) or of the local mask (compressed
 *                      head: j <= i and (j < S or i - j < R)), blended by the gate (Sec. 3.1
 *                      Eq. 1; App. B: mask matrices for prefilling).
 *   - ring slots     : the compressed store is a fixed-size circular buffer of
 *                      S + R slots (Sec. 4.3 "Inference Efficiency").  The slot rule
 *                      itself (sinks in slots 0..S-1, position p >= S in slot
 *                      S + (p-S) mod R) is this build's reading; attention does not
 *                      depend on it, only the index check does.
 *
 * Pins (tests/test_oracle_pins.py): all-full == library softmax attention; compressed
 * == full while n <= S+R; zero keys -> uniform weights -> closed-form mean of the
 * position set; a dominating key at an evicted / retained position; weights >= 0 and
 * sum to 1; explicit-mask brute force; ring simulation == closed form == position set;
 * gated mixture == the same blend of two library attentions, gate 1 / 0 == full / local;
 * prefill == library attention under explicit mask matrices, == the decode oracle row by row,
 * zero keys -> closed-form mean of the mask row.  The fp32 instantiations (decode, gated
 * decode, prefill) are each pinned to the same library attention and to their fp64 twins.
 * Every exported function is pinned by at least one of those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Position set of a head at cached length n (positions 0..n-1, newest = n-1):
 * full -> every position; compressed -> j < S (sink) or j >= n - R (recent, newest
 * included).  Union without duplicates, so n <= S+R keeps everything. */
int rlkv_oracle_in_position_set(int is_full, int64_t j, int64_t n, int S, int R)
{
    if (j < 0 || j >= n) return 0;
    if (is_full) return 1;
    return (j < S) || (j >= n - R);
}

static inline double load_elem(int dtype, const void* base, int64_t idx)
{
    if (dtype == 0) return (double)((const float*)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t*)base)[idx] << 16;   /* bf16 -> fp32, exact */
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

#define REAL double
#define REAL_EXP exp
#define FN(name) name##_f64
#include "attend_body.inc"
#undef REAL
#undef REAL_EXP
#undef FN

#define REAL float
#define REAL_EXP expf
#define FN(name) name##_f32
#include "attend_body.inc"
#undef REAL
#undef REAL_EXP
#undef FN

/* Ring-buffer index oracle: append positions 0..n_tokens-1 one at a time into a store
 * of S sink slots followed by R ring slots; slot_pos[s] = position held by slot s, or
 * -1 if the slot was never written.  Returns the cached length (= n_tokens). */
int64_t rlkv_oracle_ring_simulate(int S, int R, int64_t n_tokens, int32_t* slot_pos)
{
    for (int s = 0; s < S + R; ++s) slot_pos[s] = -1;
    int64_t len = 0;
    for (int64_t p = 0; p < n_tokens; ++p) {
        int slot;
        if (p < S) slot = (int)p;                 /* sinks are never evicted */
        else       slot = S + (int)((p - S) % R); /* overwrites position p - R, if any */
        slot_pos[slot] = (int32_t)p;
        ++len;
    }
    return len;
}

int rlkv_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
