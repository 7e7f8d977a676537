// Translation unit of the large-M prefill kernels (prefill.h) and the host sequence that runs one chunk of prompt
// rows through all layers.
#include <cmath>

#include "launch.h"
#include "prefill.h"

namespace bd {
namespace {

// Tile shapes per phase (rows per workgroup = 32*WN, k-steps per stage BKS, tokens per workgroup = 32*TW), picked by
// measurement at 1024 rows: gate/up 128 rows x 128 tokens x 2 k-steps, down and O 64 x 64 x 4, QKV 64 x 64 x 2 (the
// phases with 2048-2560 output rows need the smaller token tile to put two workgroups on every CU).
template <int PH, int WN, int BKS, int TW>
int launch_pf_gemm(hipStream_t s, PfGemmArgs a, int n_rows) {
  static bool attr_set = false;
  constexpr int lds = pf_gemm_lds<WN, BKS, TW>();
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<PH, WN, BKS, TW>), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  a.NT = n_rows / 16;
  a.RG = ceil_div(a.NT, 2 * WN);
  a.TG = ceil_div(a.MTc, 2 * TW);
  const int grid = ceil_div(a.RG, 8) * 8 * a.TG;
  hipLaunchKernelGGL((pf_gemm_kernel<PH, WN, BKS, TW>), dim3(grid), dim3(kPfThreads), lds, s, a);
  return check_launch();
}

template <int PH, int WN, int BKS, int TW, int NST, int OCC>
int launch_pf_gemm_direct(hipStream_t s, PfGemmArgs a, int n_rows) {
  static bool attr_set = false;
  constexpr int lds = pf_gemm_direct_lds<WN, BKS, TW, NST>();
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_direct_kernel<PH, WN, BKS, TW, NST, OCC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  static_assert(OCC * lds <= 160 * 1024, "workgroups per CU bounded by LDS");
  if (a.KS % BKS != 0) return BD_E_ARG;
  a.NT = n_rows / 16;
  a.RG = ceil_div(a.NT, 2 * WN);
  a.TG = ceil_div(a.MTc, 2 * TW);
  if (a.SK < 1 || (a.KS / BKS) % a.SK != 0) return BD_E_ARG;
  const int grid = ceil_div(a.RG, 8) * 8 * a.TG * a.SK;
  hipLaunchKernelGGL((pf_gemm_direct_kernel<PH, WN, BKS, TW, NST, OCC>), dim3(grid), dim3(kPfThreads), lds, s, a);
  return check_launch();
}

// K splits (at most kPfSplit) that divide n_it pipeline iterations evenly.
int skinny_split(int n_it) {
  for (int sk = kPfSplit; sk > 1; --sk)
    if (n_it % sk == 0) return sk;
  return 1;
}

}  // namespace

// One chunk of c.rows rows (prompt rows from prompt row c.off, or the tokens of a decode block) at cache position c.n0:
// all layers, K/V into the cache, no LM head.  The kernels work on whole tiles of 16 rows: the rows that pad the last tile are zero on entry, take part
// in every product and write nothing to the cache.  The device-side length is advanced by the caller.
int launch_prefill_chunk(hipStream_t s, const PfChunk& c) {
  const int rows = c.rows;
  const int MTc = ceil_div(rows, 16);
  const int mc = MTc * 16;
  const DevState* skip = c.skippable ? c.st : nullptr;
  if (c.block) {
    hipLaunchKernelGGL(pf_block_embed_kernel, dim3(rows), dim3(kWGThreads), 0, s, c.x, c.H, c.ids, c.mask,
                       c.seed_tokens, c.seed_mask, c.st, c.skippable, c.mask_id, c.table, c.vocab);
  } else {
    hipLaunchKernelGGL(embed_kernel, dim3(rows), dim3(kWGThreads), 0, s, c.x, c.H, c.embeds, c.n_embed, c.ids, c.off,
                       (const uint8_t*)nullptr, c.mask_id, c.table, c.vocab);
  }
  BD_TRY(check_launch());
  if (mc > rows) {
    hipLaunchKernelGGL(zero_rows_kernel, dim3(mc - rows), dim3(kWGThreads), 0, s, c.x + (size_t)rows * c.H, c.H, skip);
    BD_TRY(check_launch());
  }
  hipLaunchKernelGGL(rope_table_kernel, dim3(mc), dim3(64), 0, s, c.rope, c.st, c.D / 2, c.rope_theta, c.quad_W);
  BD_TRY(check_launch());
  // Up to 128 rows: the products are bound by how fast the weights arrive, not by the matrix cores.  Tiles of 32 rows x
  // 64 tokens put 2.5 to 8 times as many workgroups on the chip as the tiles above, each with a deep direct-to-LDS
  // pipeline (84 to 132 KiB in flight per CU), and the two projections with few output rows split K over workgroups.
  // (65 to 128 rows: two token groups per row group, the second of which finds the weights in its XCD's L2.)
  const bool skinny = MTc <= 8 && !c.staged;
  PfGemmArgs g{};
  g.MTc = MTc; g.Mvalid = rows; g.rs = c.rs; g.rope = c.rope; g.x = c.x; g.q = c.q; g.max_kb = c.max_kb; g.n0 = c.n0;
  g.act = c.act; g.H = c.H; g.QD = c.QD; g.KVD = c.KVD; g.D = c.D; g.n_q = c.n_q;
  g.SK = 1;
  g.st = c.st; g.skippable = c.skippable; g.pages = c.pages;
  int parts = 0;                                   // K splits of the last down projection still to be added to x
  auto norm = [&](const float* gain, const float* kparts, int n_kparts) -> int {
    if (skinny) hipLaunchKernelGGL(pf_norm_row_kernel, dim3(mc), dim3(kPfThreads), 0, s, c.x, c.H, c.rms_eps, c.xb, MTc, c.rs, gain, kparts, n_kparts, skip);
    else hipLaunchKernelGGL(pf_norm_kernel, dim3(mc / 4), dim3(kPfThreads), 0, s, c.x, c.H, c.rms_eps, c.xb, MTc, c.rs, gain, kparts, n_kparts, skip);
    return check_launch();
  };
  for (int l = 0; l < c.L; ++l) {
    const u16* wl = c.w + (size_t)l * c.layer_elems;
    g.Kc = c.Kc + (size_t)l * c.kv_layer_elems;
    g.Vc = c.Vc + (size_t)l * c.kv_layer_elems;
    // e4m3 weights: the norm gains go into the activation copy and the row scales onto the accumulators (as in decode)
    const float* ws = c.fp8 ? c.wscale + (size_t)l * c.wscale_layer : nullptr;
    BD_TRY(norm(c.fp8 ? c.gains + (size_t)(2 * l) * c.H : nullptr, c.part, parts));
    parts = 0;
    g.w = reinterpret_cast<const bf16x8*>(wl + c.w_off[0]); g.KS = ceil_div(c.H, 32);
    g.xin = reinterpret_cast<const bf16x8*>(c.xb);
    g.wscale = ws ? ws + c.wscale_off[0] : nullptr;
    // (every phase: the direct-to-LDS kernel when K is a whole number of stages, else the register-staged one)
    if (skinny && g.KS % 4 == 0) BD_TRY((launch_pf_gemm_direct<PH_QKV, 1, 4, 2, 6, 1>(s, g, c.NQKV)));
    else if (!c.staged && g.KS % 2 == 0) BD_TRY((launch_pf_gemm_direct<PH_QKV, 2, 2, 2, 2, 4>(s, g, c.NQKV)));
    else BD_TRY((launch_pf_gemm<PH_QKV, 2, 2, 2>(s, g, c.NQKV)));
    {
      PfAttnArgs t{};
      t.q = c.q; t.Kc = g.Kc; t.Vc = g.Vc; t.max_kb = c.max_kb; t.n0 = c.n0; t.Mc = mc; t.n_q = c.n_q;
      t.n_kv = c.n_kv; t.scale_log2e = 1.4426950408889634f / std::sqrt((float)c.D); t.out = c.ap; t.MTc = MTc;
      t.mode = c.mode; t.Mvalid = rows; t.st = c.st; t.skippable = c.skippable; t.pages = c.pages;
      const int items = t.n_q * (mc / 16);                    // one item per workgroup, its four wavefronts share the blocks
      const bool quad = c.mode >= 2;
      // (few rows: query tiles of a head share a workgroup, the keys are dealt to kPfAttnChunks workgroups, a second
      // kernel sums the chunks)
      const bool split = skinny && MTc <= 4 && c.apart != nullptr;
      if (split) {
        t.n_chunks = kPfAttnChunks;
        t.part = c.apart;
        const int grid = t.n_kv * ceil_div(mc / 16, kPfAttnTiles) * (t.n_q / t.n_kv) * kPfAttnChunks;
        if (c.D == 128 && quad) hipLaunchKernelGGL((pf_attn_split_kernel<128, kPfAttnTiles, true>), dim3(grid), dim3(256), 0, s, t);
        else if (c.D == 128) hipLaunchKernelGGL((pf_attn_split_kernel<128, kPfAttnTiles>), dim3(grid), dim3(256), 0, s, t);
        else if (quad) hipLaunchKernelGGL((pf_attn_split_kernel<64, kPfAttnTiles, true>), dim3(grid), dim3(256), 0, s, t);
        else hipLaunchKernelGGL((pf_attn_split_kernel<64, kPfAttnTiles>), dim3(grid), dim3(256), 0, s, t);
        BD_TRY(check_launch());
        if (c.D == 128) hipLaunchKernelGGL((pf_attn_merge_kernel<128, kPfAttnChunks>), dim3(items * 2), dim3(256), 0, s, t);
        else hipLaunchKernelGGL((pf_attn_merge_kernel<64, kPfAttnChunks>), dim3(items), dim3(256), 0, s, t);
      } else if (c.D == 128 && quad) hipLaunchKernelGGL((pf_attn_kernel<128, 4, true>), dim3(items), dim3(256), 0, s, t);
      else if (c.D == 128) hipLaunchKernelGGL((pf_attn_kernel<128, 4>), dim3(items), dim3(256), 0, s, t);
      else if (quad) hipLaunchKernelGGL((pf_attn_kernel<64, 4, true>), dim3(items), dim3(256), 0, s, t);
      else hipLaunchKernelGGL((pf_attn_kernel<64, 4>), dim3(items), dim3(256), 0, s, t);
      BD_TRY(check_launch());
    }
    g.w = reinterpret_cast<const bf16x8*>(wl + c.w_off[1]); g.KS = ceil_div(c.QD, 32);
    g.xin = reinterpret_cast<const bf16x8*>(c.ap);
    g.wscale = ws ? ws + c.wscale_off[1] : nullptr;
    int o_parts = 0;
    if (skinny && g.KS % 2 == 0) {
      // K split over workgroups like the down projection below; the norm that follows adds the splits
      g.SK = skinny_split(g.KS / 2); g.part = g.SK > 1 ? c.part : nullptr;
      BD_TRY((launch_pf_gemm_direct<PH_O, 1, 2, 2, 12, 1>(s, g, c.H)));
      o_parts = g.SK > 1 ? g.SK : 0;
      g.SK = 1; g.part = nullptr;
    } else if (!c.staged && g.KS % 4 == 0) {
      BD_TRY((launch_pf_gemm_direct<PH_O, 2, 4, 2, 2, 2>(s, g, c.H)));
    } else {
      BD_TRY((launch_pf_gemm<PH_O, 2, 4, 2>(s, g, c.H)));
    }
    BD_TRY(norm(c.fp8 ? c.gains + (size_t)(2 * l + 1) * c.H : nullptr, o_parts > 0 ? c.part : nullptr, o_parts));
    g.w = reinterpret_cast<const bf16x8*>(wl + c.w_off[2]); g.KS = ceil_div(c.H, 32);
    g.xin = reinterpret_cast<const bf16x8*>(c.xb);
    g.wscale = ws ? ws + c.wscale_off[2] : nullptr;
    // gate/up: 256 rows x 128 tokens per workgroup (a 128 x 64 tile per wavefront), one k-step per stage: 97 us for the
    // 3B shape against 110 us with 128 x 128 tiles and 136 us with the register-staged kernel
    if (skinny && g.KS % 2 == 0) BD_TRY((launch_pf_gemm_direct<PH_GU, 3, 2, 2, 7, 1>(s, g, 2 * c.F)));
    else if (!c.staged) BD_TRY((launch_pf_gemm_direct<PH_GU, 8, 1, 4, 2, 2>(s, g, 2 * c.F)));
    else BD_TRY((launch_pf_gemm<PH_GU, 4, 2, 4>(s, g, 2 * c.F)));
    g.w = reinterpret_cast<const bf16x8*>(wl + c.w_off[3]); g.KS = ceil_div(c.F, 32);
    g.xin = reinterpret_cast<const bf16x8*>(c.act);
    g.wscale = ws ? ws + c.wscale_off[3] : nullptr;
    // down: K split four ways over workgroups with 128 x 128 tiles when K divides; the next norm adds the splits
    if (skinny && g.KS % 2 == 0) {
      g.SK = skinny_split(g.KS / 2); g.part = g.SK > 1 ? c.part : nullptr;
      BD_TRY((launch_pf_gemm_direct<PH_DOWN, 1, 2, 2, 12, 1>(s, g, c.H)));
      parts = g.SK > 1 ? g.SK : 0;
      g.SK = 1; g.part = nullptr;
    } else if (!c.staged && g.KS % (2 * kPfSplit) == 0) {
      g.SK = kPfSplit; g.part = c.part;
      BD_TRY((launch_pf_gemm_direct<PH_DOWN, 4, 2, 4, 2, 2>(s, g, c.H)));
      g.SK = 1; g.part = nullptr;
      parts = kPfSplit;
    } else {
      BD_TRY((launch_pf_gemm<PH_DOWN, 2, 4, 2>(s, g, c.H)));
    }
  }
  if (parts > 0) {
    // the last layer's splits: the same kernel completes the residual stream (its other outputs are not used)
    BD_TRY(norm(nullptr, c.part, parts));
  }
  return BD_OK;
}

}  // namespace bd
