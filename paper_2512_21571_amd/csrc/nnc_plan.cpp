// Analytic tile chooser: see nnc_plan.h for the model (paper Section 3.2.2).
#include "nnc_plan.h"

#include <algorithm>
#include <cmath>

namespace nnc {

Machine machine_mi355x(int cus) {
  Machine m{};
  m.cus = cus > 0 ? cus : 256;
  m.lds_bytes = 160 * 1024;
  m.vgprs_per_wave = 256;
  // measured on these kernels, not datasheet values: inside a pass the GEMMs stream at 5.8 TB/s
  // once every CU has work
  m.hbm_bytes_per_us = 5.8e6;
  m.launch_us = 5.0;
  // whole prompt passes with and without k slices on the large tiles (0.6B .. 8B layer shapes, 768 ..
  // 4096 tokens): slices pay (4 - 9 %) while the partials are a few tens of MB and cost 2 - 3 % once
  // they are not; the second rate is the one at which the model stops choosing the losing launches
  m.fold_cached_bytes = 48e6;
  m.fold_bytes_per_us = 2.0e6;
  // the weight-streaming GEMM alone, launches back to back, 200 (rows, k, batch, row tiles,
  // k slices) combinations of the five model shapes: least-squares / best-pick fit
  m.stream_bytes_per_us = 6.4e6;
  m.cu_bytes_per_us = 58e3;
  m.skinny_launch_us = 2.5;
  m.skinny_round_us = 0.6;
  // prompt GEMM, time per k step with two workgroups per CU, measured at the 4B / 8B shapes:
  // 0.48 us for 128 x 128 tiles (16 matrix-core instructions per wave), 0.726 for 192 x 128 (24),
  // 0.865 for 256 x 128 (32): least-squares line through the three; a lone workgroup on a CU
  // takes 0.78 x that
  m.pg_c1 = 0.0241;
  m.pg_c0 = 0.110;
  m.pg_solo = 0.78;
  // the 256 x 256 tile, one workgroup per CU: 0.77 us per k step (64 matrix-core instructions per
  // wave), measured on the 8B gate|up and down projections at 4080 tokens
  m.pg_big = 0.77;
  m.pg_big12 = 0.62;  // the 192 x 256 tile (48 per wave): the 8B QKV projection
  // the register-ring kernel of the 64-row tiles: 0.26 us per k step with 4 matrix-core
  // instructions per wave (64 x 64), 0.37 with 8 (64 x 128)
  m.rg_c1 = 0.0275;
  m.rg_c0 = 0.150;
  return m;
}

namespace {
int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct PgTile {
  int code, nt, tt;
  bool lds_direct;  // three LDS stages filled by direct copies; else register ring, two stages
  int wgs_per_cu;   // resident workgroups per CU the kernel is built for
};
// every block tile the prompt GEMM kernels are instantiated for, plus one that is not (256 x 256
// with two workgroups per CU: it shows the capacity constraints at work and is never chosen)
const PgTile kPgTiles[] = {{1, 16, 8, true, 2}, {4, 12, 8, true, 2}, {2, 8, 8, true, 2}, {0, 4, 8, false, 2},
                           {3, 4, 4, false, 2}, {5, 16, 16, true, 1}, {6, 12, 16, true, 1}, {-1, 16, 16, true, 2}};
}  // namespace

PrefillGemmPlan plan_prefill_gemm(const Machine& mc, int n_tiles, int KT, int col_tiles, int n_tokens, int pieces,
                                  int epi, int max_k_slices) {
  PrefillGemmPlan best{};
  best.tile = -1;
  best.t_us = 1e30;
  const double W = (double)n_tiles * KT * 1024.0, X = (double)col_tiles * KT * 1024.0;
  const double N = (double)n_tiles * 16.0;
  const double out_bytes = epi == PLAN_EPI_STORE ? n_tokens * N * 4.0
                           : epi == PLAN_EPI_RESID ? n_tokens * N * 8.0  // read-modify-write of the residual stream
                                                   : n_tokens * (N / 2.0) * 2.0 * pieces;
  for (const PgTile& t : kPgTiles) {
    const int wgs_per_cu = t.wgs_per_cu;
    ++best.candidates;
    // capacity: staged operands of the resident workgroups in LDS; accumulators and two sets of
    // fragments (one for the ring kernels) in the wave's registers
    const int stages = t.lds_direct ? 3 : 2;
    const int lds = stages * (t.nt + t.tt) * 1024 * wgs_per_cu;
    const int wi = t.nt / 2, wj = t.tt / 2;
    const int regs = wi * wj * 4 + (t.lds_direct ? 2 : 1) * (wi + wj) * 4 + (t.lds_direct ? 0 : 8 * (t.nt / 4 + t.tt / 4) * 4);
    // (a wave alone on its SIMD has the accumulation registers on top of the ordinary ones)
    if (lds > mc.lds_bytes || regs > mc.vgprs_per_wave * (wgs_per_cu == 1 ? 2 : 1) || t.code < 0) {
      ++best.rejected_by_capacity;
      continue;
    }
    const int ks_max = epi != PLAN_EPI_RESID ? 1 : std::max(1, max_k_slices);
    // a slice shorter than the register ring (or, for the tiles with three LDS stages in flight,
    // than a few times their pipeline) gains nothing
    const int kts_min = !t.lds_direct ? 8 : wgs_per_cu == 1 ? 32 : 16;
    for (int ks = 1; ks <= ks_max; ++ks) {
      const int kts = ceil_div(KT, ks);
      if (ks > 1 && kts < kts_min) break;
      const int slices = ceil_div(KT, kts);
      if (slices != ks) continue;            // same launch as a smaller ks
      const int wgs = ceil_div(n_tiles, t.nt) * ceil_div(col_tiles, t.tt) * slices;
      const int slots = wgs_per_cu * mc.cus;
      const int full = wgs / slots, rem = wgs - full * slots;
      const double t2 = wgs_per_cu == 1 ? (t.nt == 16 ? mc.pg_big : mc.pg_big12)
                        : t.lds_direct  ? mc.pg_c0 + mc.pg_c1 * wi * wj
                                        : mc.rg_c0 + mc.rg_c1 * wi * wj;
      const double t1 = mc.pg_solo * t2;
      const double t_comp = wgs_per_cu == 1 ? kts * t2 * (full + (rem ? 1 : 0))
                                            : kts * (full * t2 + (rem == 0 ? 0.0 : rem <= mc.cus ? t1 : t2));
      const double fold = (slices - 1) * n_tokens * N * 4.0 * 2.0;  // partials written, then read by the norm kernel
      const double t_mem = (W + X) / mc.hbm_bytes_per_us;
      const double t_fold = fold / (fold <= mc.fold_cached_bytes ? mc.hbm_bytes_per_us : mc.fold_bytes_per_us);
      const double total = std::max(t_comp, t_mem) + out_bytes / mc.hbm_bytes_per_us + t_fold + mc.launch_us;
      if (total < best.t_us * 0.999) {
        best.tile = t.code; best.nt = t.nt; best.tt = t.tt;
        best.k_slices = slices; best.kts_per_split = slices > 1 ? kts : 0;
        best.workgroups = wgs;
        best.t_comp_us = t_comp; best.t_mem_us = t_mem; best.t_us = total;
      }
    }
  }
  return best;
}

SkinnyGemmPlan plan_skinny_gemm(const Machine& mc, int n_tiles, int KT, int ncols, int nseq, int rt_choices,
                                int max_k_slices) {
  SkinnyGemmPlan best{};
  best.rt = 0;
  best.t_us = 1e30;
  const double W = (double)n_tiles * KT * 1024.0;
  // operand bytes per k tile: one 16-byte group per (k / 8 or k / 4, column), i.e. 64 bytes per
  // column, and the kernel loads whole blocks of 16 columns
  const double x_per_kt = 64.0 * ((ncols + 15) / 16 * 16);
  for (int rt = 1; rt <= 8; ++rt) {
    if (!((rt_choices >> rt) & 1) || n_tiles % rt) continue;
    for (int ks = 1; ks <= std::max(1, max_k_slices); ++ks) {
      const int kts = ceil_div(KT, ks);
      if (ks > 1 && kts < 8) break;  // at least two k tiles per wave
      const int slices = ceil_div(KT, kts);
      if (slices != ks) continue;
      const int wgs = n_tiles / rt * slices;
      // T_mem, level 1: what the busiest CU pulls through its vector memory path.  A workgroup
      // reads its rt x kts weight tiles once, and the operand of its k slice once for all its
      // row tiles; the operand comes from L2, but it crosses the same per-CU path as the
      // weights, and with 48 operand columns a workgroup of one row tile moves three operand
      // bytes per weight byte.  Measured: a CU sustains 58 GB/s on this access pattern whether
      // one workgroup or three share it.
      const int per_cu = ceil_div(wgs, mc.cus);
      const double wg_bytes = (double)rt * kts * 1024.0 + kts * x_per_kt;
      const double t_cu = per_cu * wg_bytes / mc.cu_bytes_per_us;
      // T_mem, level 2: the weights from HBM; fewer workgroups than CUs cannot draw the full rate
      const double cover = std::min(1.0, (double)wgs / mc.cus);
      const double t_hbm = W / (mc.stream_bytes_per_us * std::sqrt(cover));
      // epilogue: the four waves' partial tiles meet in LDS two row tiles at a time (one at a
      // time for an odd count), one round after the other, for every workgroup a CU runs
      const int rounds = rt % 2 == 0 ? rt / 2 : rt;
      const double t_epi = mc.skinny_round_us * rounds * per_cu;
      // partial sums: written per slice and read once more by the consumer, a norm kernel of one
      // workgroup per sequence that runs at an eighth of the streaming rate at best
      const double fold = slices > 1 ? slices * (double)n_tiles * 16.0 * nseq * 4.0 * 2.0 / (mc.hbm_bytes_per_us / 8.0) : 0.0;
      const double total = std::max(t_cu, t_hbm) + t_epi + fold + mc.skinny_launch_us;
      if (total < best.t_us * 0.999) {
        best.rt = rt; best.k_slices = slices; best.kts_per_split = kts; best.workgroups = wgs;
        best.t_mem_us = t_hbm; best.t_operand_us = t_cu; best.t_us = total;
      }
    }
  }
  return best;
}

}  // namespace nnc
