// Host-side description of the sequence split and of the workspace each operation uses.
// One place computes the sizes so that cottn_workspace_bytes() and the launchers agree.
#pragma once
#include <stddef.h>

namespace cottn {

// G segments of seg_rows rows (a whole number of chunks of C rows) per (batch, head).
struct SeqPlan {
  int C;
  int G;
  int seg_rows;
};

bool make_plan(int op, int B, int H, int N, int dk, int dv, int chunk, int dtype, SeqPlan* plan);

inline size_t round_up_256(size_t x) { return (x + 255) & ~size_t(255); }

// Workspace layouts (all fp32; a state is dk x dv: row-major [d_key][d_value] on the
// bidirectional and fp32 paths; the 16-bit causal kernels, which alone read what they write
// here, keep each state in 16x16 tiles of 256 consecutive floats in accumulator-register order,
// device_common.h: tiled_state_offset):
//   causal forward   G > 1: [units][G][dk][dv]   segment totals, turned in place into the
//                            state at each segment start
//   causal backward  G > 1: the same array for the forward-time states, a second one for
//                            the reverse-time states; always: [units][G] partial sums of ds
//   bidirectional forward : [units][G][dk][dv]   segment totals, slot 0 becomes the full state
//   bidirectional backward: two arrays [units][G][dk][dv], totals of Kh^T V and of Qh^T dO,
//                            slot 0 becomes the full matrix when the combine kernel runs; per
//                            unit max(G, dk*dv/256) partial sums of ds (the totals kernel
//                            leaves G, the combine kernel dk*dv/256)
inline size_t state_array_bytes(int B, int H, int dk, int dv, int G) {
  return round_up_256(size_t(B) * H * G * dk * dv * sizeof(float));
}
inline size_t ds_partials_bytes(int B, int H, int G) {
  return round_up_256(size_t(B) * H * G * sizeof(float));
}

inline size_t workspace_bytes_for(int op, int B, int H, int dk, int dv, const SeqPlan& p) {
  switch (op) {
    case 0: return p.G > 1 ? state_array_bytes(B, H, dk, dv, p.G) : 0;
    case 1: return (p.G > 1 ? 2 * state_array_bytes(B, H, dk, dv, p.G) : 0) + ds_partials_bytes(B, H, p.G);
    case 2: return state_array_bytes(B, H, dk, dv, p.G);
    case 3: return 2 * state_array_bytes(B, H, dk, dv, p.G) +
                   ds_partials_bytes(B, H, p.G > dk * dv / 256 ? p.G : dk * dv / 256);
    default: return 0;
  }
}

}  // namespace cottn
