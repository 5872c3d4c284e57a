// The work plan of a grouped launch of the persistent GEMM (GemmPlan in kernels.h), computed by one wave
// at the end of the grouping kernel, which has the groups' sizes in its lanes: lane g looks at group g.
#pragma once
#include "kernels.h"

namespace moe {

// Every tile is cut into p.slices K slices.  Ranges: the item list is cut where the estimated cost reaches
// 1/8, 2/8, ... of the total; a full tile costs 1 (its K loop), a remainder tile of r rows
// max(0.5, its share of the MFMAs): measured, a tile of at most 64 rows takes half the time of a full one,
// bound by the weight tile's way in from HBM.
__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}

// count: the rows of group `lane` (any value in lanes past the last group).
__device__ __forceinline__ void make_plan(const PlanParams &p, int lane, int count) {
  GemmPlan *out = p.out;
  const bool active = lane < p.n_groups && ((p.mask >> lane) & 1ull);
  const int cnt = active ? count : 0;
  const int mf = p.equal_heights ? (cnt + kPpTileRows - 1) / kPpTileRows : cnt / kPpTileRows;
  const int rem = p.equal_heights ? 0 : cnt % kPpTileRows, hr = rem ? 1 : 0;
  const float c_r = hr ? fmaxf(0.5f, 0.08f + 0.92f * (float)((rem + 63) / 64) * 0.25f) : 0.0f;
  const int s_f = p.slices > 0 ? p.slices : 1, s_r = s_f;
  const int items = p.ntn * (mf * s_f + hr * s_r);
  const float cost = p.ntn * ((float)mf + c_r);
  int item_end = items;
  float cost_end = cost;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const int oi = __shfl_up(item_end, s);
    const float oc = __shfl_up(cost_end, s);
    if (lane >= s) { item_end += oi; cost_end += oc; }
  }
  const int n_items = __shfl(item_end, 63);
  const float total = __shfl(cost_end, 63);
  out->item_begin[lane + 1] = item_end;
  if (lane == 0) {
    out->item_begin[0] = 0;
    out->n_items = n_items;
    out->s_full = s_f;
    out->s_rem = s_r;
    out->xcd_begin[0] = 0;
    out->xcd_begin[8] = n_items;
  }
  // boundary j: in the group whose cost range holds j/8 of the total, at the same fraction of its items
  // (a group's range begins exactly where the one before it ends: no target falls between two groups)
  const float prev_end = __shfl_up(cost_end, 1);
  const float cost_begin = lane ? prev_end : 0.0f;
  for (int j = 1; j < 8; ++j) {
    const float target = total * (float)j * 0.125f;
    const bool here = cost > 0.0f && cost_begin <= target && target < cost_end;
    const unsigned long long who = __ballot(here);
    if (who == 0) {   // (rounding at the very end of the list, or nothing to do at all)
      if (lane == 0) out->xcd_begin[j] = n_items;
    } else if (lane == __ffsll((long long)who) - 1) {
      int at = item_end - items + (int)((target - cost_begin) / cost * (float)items);
      out->xcd_begin[j] = at < item_end ? at : item_end;
    }
  }
  out->queue[lane] = 0;
  out->queue[lane + 64] = 0;
}

}  // namespace moe
