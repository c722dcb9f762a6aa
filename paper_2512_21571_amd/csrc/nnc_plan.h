// Analytic choice of tile sizes for the GEMM launches (host code only).
//
// The paper's Auto Schedule picks tile sizes by solving a small optimisation problem instead of
// tuning by hand (Section 3.2.2, parametric optimisation): integer tile variables per loop and
// memory level, buffer sizes and traffic derived from them, capacity constraints per storage
// level, and the objective  minimise max(T_mem, T_comp)  with T_comp taken from a linear
// regression of the micro-kernel's time and T_mem = traffic / bandwidth.  Here the search space is
// the handful of block tiles the kernels are instantiated for (x the k slices a launch may use),
// so "solving" is enumeration; the model is the paper's:
//   variables    block tile (NT x TT 16-row / 16-column tiles at the LDS level), k slices
//   constraints  LDS bytes of the staged operands x resident workgroups <= LDS per CU;
//                accumulator + fragment registers per wave <= the register file share
//   T_comp       k steps x micro-kernel time per k step (linear in the matrix-core
//                instructions per wave: c0 + c1 x WI x WJ, measured), summed over the rounds in
//                which the launch's workgroups occupy the chip (a last round with at most one
//                workgroup per CU runs faster per step than a full one)
//   T_mem        (weights + activations + outputs + k-slice partials) / streaming bandwidth
//   objective    max(T_comp, T_mem) + epilogue traffic time + launch time
#pragma once
#include <stdint.h>

namespace nnc {

struct Machine {
  int cus;                // compute units
  int lds_bytes;          // LDS per CU
  int vgprs_per_wave;     // with two waves per SIMD
  double hbm_bytes_per_us;       // streaming rate these kernels reach
  double launch_us;       // start-to-end time of a kernel with nothing to do
  // k-slice partials of a prompt GEMM (written by its epilogue, read back by the next norm kernel):
  // at the streaming rate while all of them stay in the caches, at fold_bytes_per_us beyond that
  double fold_cached_bytes, fold_bytes_per_us;
  // the weight-streaming GEMM of decode passes: streaming rate of the whole chip, bytes a CU moves
  // through its vector memory path (weights + operand), launch-to-launch overhead, one round of
  // the cross-wave reduction in the epilogue
  double stream_bytes_per_us, cu_bytes_per_us, skinny_launch_us, skinny_round_us;
  // micro-kernel regression of the LDS-staged prompt GEMM, per k step of 32 with two workgroups per
  // CU: c0 + c1 * (matrix-core instructions per wave and k step) microseconds; one workgroup
  // alone on a CU takes `solo` times that
  double pg_c0, pg_c1, pg_solo;
  double pg_big, pg_big12;  // microseconds per k step of the 256 x 256 / 192 x 256 tile (one workgroup per CU)
  double rg_c0, rg_c1;  // the same regression for the register-ring kernel of the 64-row tiles
};
Machine machine_mi355x(int cus);

enum { PLAN_EPI_STORE = 0, PLAN_EPI_RESID = 1, PLAN_EPI_SWIGLU = 2 };

struct PrefillGemmPlan {
  int tile;            // launch_gemm_prefill shape code (0: 64x128, 1: 256x128, 2: 128x128, 3: 64x64, 4: 192x128, 5: 256x256, 6: 192x256)
  int nt, tt;          // block tile in 16-row / 16-column tiles
  int k_slices;        // workgroups that share one output tile's k range
  int kts_per_split;   // k tiles per slice (0: one slice)
  int workgroups;
  double t_comp_us, t_mem_us, t_us;
  int candidates, rejected_by_capacity;
};
// n_tiles: output rows / 16; KT: k / 32; col_tiles: operand column tiles (token tiles x pieces);
// n_tokens, pieces: of the block; epi: PLAN_EPI_*; max_k_slices: 1 if the launch may not split k.
PrefillGemmPlan plan_prefill_gemm(const Machine& mc, int n_tiles, int KT, int col_tiles, int n_tokens, int pieces,
                                  int epi, int max_k_slices);

struct SkinnyGemmPlan {
  int rt;              // 16-row tiles per workgroup
  int k_slices;
  int kts_per_split;
  int workgroups;
  double t_mem_us;      // weights from HBM
  double t_operand_us;  // weights + operand through the busiest CU's vector memory path
  double t_us;
};
// Weight-streaming GEMM of decode passes: n_tiles x KT tiles of 1 KiB, ncols operand columns
// (sequences x pieces) of elem_bytes each, nseq sequences.  rt_choices: bit r set = the kernel is
// instantiated for r row tiles per workgroup.  max_k_slices: 1 if the consumer cannot add partials.
SkinnyGemmPlan plan_skinny_gemm(const Machine& mc, int n_tiles, int KT, int ncols, int nseq, int rt_choices,
                                int max_k_slices);

}  // namespace nnc
