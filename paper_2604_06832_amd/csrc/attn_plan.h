// How the attention phase of the streaming forward kernel is dealt out when it stays inside each XCD (host and device).
#pragma once
#include "common.h"

namespace bd {

// CT column tiles per XCD (all of one kv head), each spread over NCH of the XCD's WX workgroups.
struct AttnLocalPlan { int CT, NCH, WX; };
__host__ __device__ inline bool attn_local_plan(int nwg, int n_xcd, int n_kv, int n_ct, AttnLocalPlan& p) {
  if (n_xcd <= 0 || nwg % n_xcd != 0) return false;
  const int total = n_kv * n_ct;
  if (total % n_xcd != 0) return false;
  p.CT = total / n_xcd;
  p.WX = nwg / n_xcd;
  if (p.CT > kWavesPerWG || (p.CT & (p.CT - 1)) != 0 || n_ct % p.CT != 0 || p.WX % p.CT != 0) return false;
  p.NCH = p.WX / p.CT;
  return p.NCH <= 64;
}

}  // namespace bd
