// Internal interface between the host-side step scheduler (nnc_api.hip) and the
// gfx950 kernels (nnc_kernels.hip).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace nnc {

// `dt` arguments of the launchers: the model's element type, 0 = fp32, 1 = bf16, 2 = binary16
// (enum Dtype in nnc_half.h, same values as nnc_dtype in the public header).

// Activation columns one pass may carry: decode batch, or a prompt chunk.
constexpr int MAX_COLS = 64;
// Cached positions one attention workgroup covers.
constexpr int ATT_CHUNK = 64;

// Per-column bookkeeping, resident in device memory so that a captured graph
// never bakes a position, slot or token into a kernel argument.
struct ColState {
  int32_t tok[MAX_COLS];    // token id of the column (token models)
  uint32_t slot[MAX_COLS];  // KV slot the column belongs to
  uint32_t pos[MAX_COLS];   // position the column occupies in its slot
  uint32_t step;            // greedy-loop step counter
  uint32_t pad[3];
};

enum Epilogue { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

// Column -> (slot, position, row of the q|k|v buffer).  st != NULL: decode pass, looked up
// per column, row = column.  st == NULL: prompt block, column c is position pos0 + c of
// `slot` and row row0 + c.
struct ColMap {
  const ColState* st;
  uint32_t slot, pos0;
  int row0;
};

// Skinny GEMM  Y[n, seq] = sum_k W[n, k] * X[k, seq]  over packed operands.
//
// Packed weight layout (both dtypes: 16 rows x KTILE columns per 1 KiB tile,
// KTILE = 32 for bf16 and 16 for fp32, VEC = 8 or 4 elements per lane):
//   Wp[((nt * KT + kt) * 64 + lane) * VEC + j] = W[nt*16 + lane%16][kt*KTILE + (lane/16)*VEC + j]
// i.e. tile (nt, kt) is stored in the order a 64-lane wave feeds it to the
// 16x16 matrix-core instruction as its A operand: every lane issues one
// 16-byte load and a wave reads 1 KiB contiguously.
//
// Packed activation layout (the B operand; NC columns allocated, `ncols` used):
//   Xp[((k / VEC) * NC + col) * VEC + k % VEC]
// bf16 models carry each fp32 activation as `nsplit` bf16 pieces in adjacent
// columns (col = seq * nsplit + piece, piece 0 = rounded value, piece 1 = rounded
// remainder, ...); the pieces' products are summed in the epilogue, which keeps
// activations at fp32 accuracy while the weights stream through the bf16 matrix
// cores untouched.
// The RMSNorm that follows an output / down projection, run in the tail of that GEMM launch
// instead of a kernel of its own: every workgroup stores its partial tile through to memory and
// counts itself done; the last workgroups to finish (one per sequence) wait until all have, then
// each adds the k-slice partials of its sequence to the residual stream (fixed slice order),
// norms the row and writes the packed operand of the next GEMM: what k_rmsnorm_pack computes,
// with the same arithmetic.  counter == NULL: no tail.
struct NormTail {
  uint32_t* counter;   // zero before the launch
  float* x;            // residual stream [sequence][ldx]
  long ldx;
  const float* gain;
  int H;
  float eps;
  void* Xp;            // packed operand out
  int NC, nsplit;
  unsigned spin_limit; // polls of the counter before a waiting workgroup gives up
  unsigned* error;     // set to 1 when one does (the pass's results are then invalid)
};

struct GemmArgs {
  const void* Wp;
  // weight-only 8-bit matrices: one fp32 scale per output row, in the row order of the packed
  // tiles; NULL for matrices in the model's element type.  A k tile is then 16 rows x 64 k (1 KiB
  // of bytes, the lane's 8 values of k sub-tile 0 then its 8 of sub-tile 1) and KT, kts_per_split
  // count those; the operand has two of its 32-wide k tiles per weight tile.
  const float* wscale;
  int n_tiles;        // output rows / 16
  int KT;             // k tiles in the matrix
  int kts_per_split;  // k tiles per blockIdx.y slice
  const void* Xp;
  int NC;     // allocated operand columns
  int ncols;  // used operand columns = nseq * nsplit
  int nsplit;
  int nseq;
  // EPI_STORE: out[kslice * split_stride + seq * ldo + n] = partial y of that k slice
  // (one slice, split_stride unused, for the GEMMs whose consumer wants the full sum).
  float* out;
  long ldo;
  long split_stride;
  // offset added to `out`, in floats, = *step_ptr * step_stride (greedy loop logits log)
  const uint32_t* step_ptr;
  long step_stride;
  // EPI_SWIGLU: rows come in 16-row pairs (gate tile, up tile); the activation
  // silu(gate) * up for feature f is written as the packed operand of the next
  // GEMM (K = number of features), split into nsplit_out pieces.
  void* packed_out;
  int NC_out;
  int nsplit_out;
  // 16-row tiles per workgroup (1, 2, 3, 4 or 6; SwiGLU: 2, 4, 6 or 8; fp32 models: 1, 2 or 4);
  // 0: the launcher's own rule
  int rt;
  NormTail tail;  // EPI_STORE with out = [k slice][sequence][ldo = tail.H] only
};

struct KernelCtx;  // profiling hook, defined in nnc_api.hip

// All launchers enqueue on `s` and return the launch error code.
hipError_t launch_repack(hipStream_t s, bool src_f32, int dst_dt, const void* src, void* dst,
                         int rows, int K, int tile_stride, int tile_offset);
// row-major signed bytes [rows, K] -> byte tiles of 16 rows x 64 k (K a multiple of 64)
hipError_t launch_repack_w8(hipStream_t s, const void* src, void* dst, int rows, int K, int tile_stride,
                            int tile_offset);
hipError_t launch_set_state(hipStream_t s, ColState* st, int ncols, const int32_t* tok,
                            const uint32_t* slot, const uint32_t* pos, uint32_t step);
hipError_t launch_embed(hipStream_t s, int dt, const void* Ep, int H, const ColState* st,
                        int ncols, float* x);
hipError_t launch_rmsnorm_pack(hipStream_t s, int dt, float* x, long ldx, const float* part, int nparts,
                               long part_stride, const float* gain, int H, float eps, int ncols, void* Xp,
                               int NC, int nsplit);
// n 32-bit words = 0 (a fill kernel: safe under graph capture)
hipError_t launch_zero_words(hipStream_t s, uint32_t* p, int n);
hipError_t launch_fold_residual(hipStream_t s, float* x, const float* part, int nparts, long part_stride,
                                size_t n);
hipError_t launch_gemm(hipStream_t s, int dt, int epi, const GemmArgs& a);
hipError_t launch_qknorm_rope_append(hipStream_t s, int dt, float* qkv, int nq, int nkv,
                                     const float* gq, const float* gk, float eps,
                                     const float2* rope, const ColMap& cm, int ncols, void* kc,
                                     void* vc, uint32_t max_batch, uint32_t max_seq, void* qsplit, void* vt,
                                     uint32_t vt_stride);
// Fused QK-norm + RoPE + append inside the batched decode attention (bf16, at most 8 query heads
// per kv head, every column a different slot): what the kernel needs besides the raw projection.
struct AttnFuseArgs {
  const float* gq;
  const float* gk;
  float eps;
  const float2* rope;
  // the raw projection arrives as qkv_slices partial sums (k slices of the QKV GEMM),
  // qkv_slice_stride floats apart; the kernel adds them in slice order (0 or 1: one array)
  int qkv_slices;
  long qkv_slice_stride;
};
bool attn_partial_can_fuse(int dt, int nq, int nkv);
hipError_t launch_attn_partial(hipStream_t s, int dt, const float* qkv, const void* qsplit, int nq, int nkv,
                               void* kc, void* vc, uint32_t max_batch, uint32_t max_seq, const ColMap& cm,
                               int ncols, int grid_chunks, float* partial, int max_chunks,
                               const AttnFuseArgs* fuse, bool one_slot = false);
hipError_t launch_attn_combine(hipStream_t s, int dt, const float* partial, int max_chunks, int nq,
                               const ColMap& cm, int ncols, void* Op, int NC, int nsplit);

// ---- prompt pass on large token blocks (bf16 models): LDS-staged matrix-core GEMM ----
// Y[t, n] = sum_k X[t, k] W[n, k].  W: packed weights (above).  X: bf16 activations in
// fragment order [column tile][k / 32][64 lanes][8]; with `pieces` = 2 every activation is two
// bf16 values (value, remainder) and token tile q occupies column tiles 2q, 2q+1 (the
// epilogue adds their products).  t_tiles counts column tiles = token tiles x pieces.
// epi EPI_STORE: out[t * ldo + n] = y (fp32).  EPI_RESID: out[t * ldo + n] += y.
// EPI_SWIGLU: rows alternate gate / up in 16-row tiles; silu(gate) * up for feature f is
// written as bf16 in fragment order (k = f, k tiles = n_tiles / 2 / 2) into packed_out.
struct PrefillGemmArgs {
  const void* Wp;
  // weight-only 8-bit layers: Wp holds the bytes widened to 16 bits (launch_widen_w8) and the
  // epilogue multiplies every output row by its scale (packed row order); NULL otherwise
  const float* wscale = nullptr;
  int n_tiles, KT;
  const void* Xf;
  int t_tiles;
  float* out;
  long ldo;
  void* packed_out;
  // k split (residual epilogue only, any tile): k tiles per blockIdx.z slice, 0 =
  // one slice.  Slice 0 adds to `out`; slice s > 0 stores its partial sums at part + (s - 1) *
  // part_stride (same row stride as out).
  int kts_per_split = 0;
  float* part = nullptr;
  long part_stride = 0;
};
hipError_t launch_gemm_prefill(hipStream_t s, bool f16, int epi, const PrefillGemmArgs& a, int pieces, int shape);
// packed byte tiles (n_tiles x KT8 of 16 rows x 64 k) -> bf16 tiles of 16 rows x 32 k in the same tile order
// (exact: |byte| <= 127), the operand the block-tile prompt GEMMs copy into LDS
hipError_t launch_widen_w8(hipStream_t s, const void* src, void* dst, int n_tiles, int KT8);
// x[rows, H] += part[0] + ... + part[nparts-1] (written back), then RMSNorm of rows 0..n_rows-1
// as `pieces` bf16 per value in fragment order; rows n_rows .. 16 * token_tiles - 1 of the
// operand are zero-filled.
hipError_t launch_rmsnorm_frag(hipStream_t s, bool f16, float* x, const float* part, int nparts, long part_stride,
                               const float* gain, int H, float eps, int n_rows, int token_tiles, int pieces,
                               void* Xf);
hipError_t launch_v_transpose(hipStream_t s, const void* vc, uint32_t slot, int nkv, uint32_t max_seq, uint32_t n_pos,
                              void* vt, uint32_t S);
hipError_t launch_attn_prefill(hipStream_t s, bool f16, const float* qkv, int nq, int nkv, const void* kc, const void* vt,
                               uint32_t S, uint32_t slot, uint32_t max_seq, uint32_t pos0, int n, int pieces, void* Of,
                               int n_cus, int shape);
hipError_t launch_embed_rows(hipStream_t s, bool f16, const void* Ep, int H, const int32_t* tokens_dev, int n, float* x);
hipError_t launch_argmax(hipStream_t s, const float* logits, long ld, int V, int ncols,
                         const uint32_t* step_ptr, long step_stride, float* scratch_val,
                         int32_t* scratch_idx, int32_t* next);
hipError_t launch_finish_step(hipStream_t s, ColState* st, int ncols, const int32_t* next,
                              int32_t* token_log);
hipError_t launch_kv_read(hipStream_t s, int dt, const void* cache, uint32_t max_seq, int nkv,
                          uint32_t pos0, uint32_t n, float* out);
hipError_t launch_copy_rows(hipStream_t s, const float* src, float* dst, size_t n);

// ---- resident whole-step decode kernel (bf16 models, batch 1) ----
struct MkPlan {
  int nwg;  // resident workgroups: min(compute units, QKV tiles)
  int n_layers, H, nq, nkv, F, V;
  float eps;
  uint32_t max_seq;
  int max_chunks;
  int tok0;             // token fed to the first step
  uint32_t pos0, slot;  // its position and KV slot
  int n_steps;
  unsigned tag_base;    // first exchange tag of this launch (tags must never repeat)
  int ks_o, ks_d;       // k slices of the output / down projections
  int off_att, off_o, off_d;  // first workgroup of the attention / output / down projection units
  unsigned spin_max;    // polls of one wait before the launch gives up (0 = default)
  bool f16;             // binary16 model (else bf16)
};

struct MkBuffers {
  const void* layers;  // device array of per-layer pointer records (mk_fill_layer)
  const void* embed;
  const void* lm_head;
  const float* g_final;
  const float2* rope;
  unsigned* error;  // single word, zero-initialised once
  // exchange buffers of 64-bit (value, tag) words, zero-initialised once
  void *xq, *xatt, *xo, *xop, *xact, *xdp, *xamv, *xami;
  float* logits;       // [n_steps][V] or NULL
  int32_t* token_log;  // [n_steps]
  unsigned long long* trace;  // [nwg][trace_points] or NULL
  int trace_step, trace_points;
};
// Stamps per traced step, 8 per layer: layer start, stage-1 operand ready, q|k|v published,
// attention partials published, attention block output published, stage-4 operand ready,
// activations published, MLP output published; then LM-head operand ready, winners
// published, token known.
inline int mk_trace_points(int n_layers) { return 8 * n_layers + 3; }
// exchange tags one decode step consumes
inline unsigned mk_tags_per_step(int n_layers) { return 5u * (unsigned)n_layers + 1u; }

size_t mk_layer_bytes();
void mk_fill_layer(void* dst, const void* wqkv, const void* wo, const void* wgu, const void* wd, const float* g_in,
                   const float* g_q, const float* g_k, const float* g_post, void* kc, void* vc);
size_t mk_opnd_bytes(const MkPlan& p);
int mk_max_resident_workgroups(const MkPlan& p, int n_cus);
hipError_t launch_decode_resident(hipStream_t s, const MkPlan& p, const MkBuffers& b);

}  // namespace nnc
