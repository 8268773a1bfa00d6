// Internal declarations shared by the host entry points and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "monarchrt.h"

namespace mrt {

// Offset, in tokens, of block-grid index x along one side of the block grid:
//   div == 0:  x * lo          div > 0:  (x / div) * hi + (x % div) * lo
// (the two-level form is needed when that side is (frame, width): Sec. 4.1's (fw, h) and (h, fw)).
struct AxisMap {
  int div;
  int hi, lo;
};
__host__ __device__ inline long long axis_offset(const AxisMap& m, int x) {
  if (m.div == 0) return (long long)x * m.lo;
  const int q = x / m.div;
  return (long long)q * m.hi + (long long)(x - q * m.div) * m.lo;
}

// Geometry and addressing of one call, passed by value to every kernel.
//
// Index names follow App. A: m query tile, n key tile, l query row, j column, k key row,
// i key column, v feature.  nk = n*b1 + k is the flattened (key tile, key row) index the
// joint softmax of L runs over.
struct KParams {
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  mrt_strides qs, ks, vs, os;
  // per-pass intermediates (slabs of `heads in this pass`), see slab_layout()
  void* aL;     // alpha_L [bh][m][j][nk][d]
  void* Y;      // Y       [bh][m][j][nk][d]
  void* aR;     // alpha_R / c_R  [bh][m][nk][j][d]
  float* cL;    // c_L     [bh][m][j][nk]
  float* cmx_out;   // optional outputs of stage L (earlier iterations, any kernel): column maximum of
  float* cinv_out;  //   log L and inverse column sum behind alpha_R / c_R   [bh][m][nk][j]
  float* lse_out;   // optional outputs of the streamed last-iteration stage L kernel: base-2
  float* o32_out;   //   log-sum-exp of every query row's logits [bh][m][j][l] and O in fp32 [bh][m][j][l][d]
  int H;        // heads (to split the flat batch*head index)
  int bh0;      // first flat (batch,head) index of this pass
  int d;
  int b1, b2;
  int c2;       // column tiles
  int ntq, ntk; // query tiles IN THIS PASS (workspace extent), key tiles of the whole grid
  int m0;       // first query tile of this pass
  int c1k;      // key tile rows
  AxisMap rmap, cmap;   // token of block-grid cell (x, y) = axis_offset(rmap, x) + axis_offset(cmap, y)
  // neighbourhood tiles (Sec. 4.2): a tile row is n_f frames x nh grid rows of each, nh < h.
  // nh == 0: tile row a is the contiguous block-grid rows a*b1 .. a*b1 + b1 - 1.
  int nh;       // grid rows of one frame per tile (0 = contiguous rows)
  int nhb;      // tile rows per frame group = h / nh
  int tf_tok;   // tokens from one frame group to the next = n_f * h * w
  int th_tok;   // tokens from one row band to the next = nh * w
  int ct;       // tile rows per causal chunk; 0 = no mask
  int qt0;      // tile row (of the key grid) at which query tile row 0 sits (mask only)
  // regular Monarch under the chunk-causal mask: its one tile straddles every chunk, and the mask
  // is a support constraint on L.  Block row x holds frame x / (rows per frame), so query row l
  // sees the key rows k < visible_key_rows(p, l), a prefix.  rl == 0: nothing hidden.
  int rl;       // block rows per causal chunk
  int rq0;      // block row at which query row 0 sits on the key side (frame offset * rows per frame)
  int cc;       // frames per causal chunk (dense baseline); 0 = no mask
  int qoff;     // absolute frame of query frame 0 (dense baseline)
  int Nq, Nkv;  // tokens per head on the query / key side
  int hw;       // tokens per frame (h*w)
  float scale;
};

// Token offset of row l of tile row a (add the column offset axis_offset(cmap, y) to it).
__host__ __device__ inline long long row_offset(const KParams& p, int a, int l) {
  if (p.nh == 0) return axis_offset(p.rmap, a * p.b1 + l);
  const int fa = a / p.nhb, ha = a - fa * p.nhb;
  const int u = l / p.nh, v = l - u * p.nh;
  return (long long)fa * p.tf_tok + (long long)ha * p.th_tok + (long long)u * p.hw + (long long)v * p.rmap.lo;
}

// Number of visible key-tile ROWS for query tile row a (tile-level chunk-causal reading: key
// tile row a' is visible iff its chunk floor(a' / ct) is not later than the query tile row's
// chunk floor((qt0 + a) / ct); no tile straddles a chunk).
__host__ __device__ inline int visible_key_tile_rows(int a, int c1k, int ct, int qt0) {
  if (ct == 0) return c1k;
  const int rows = ((qt0 + a) / ct + 1) * ct;
  return rows < c1k ? rows : c1k;
}

// Regular Monarch with p.rl > 0: number of leading key rows visible to query row l (the rows of
// every chunk up to and including the query row's own).  May exceed b1; the diagonal k = l is
// always below it.
__host__ __device__ inline int visible_key_rows(const KParams& p, int l) {
  return ((l + p.rq0) / p.rl + 1) * p.rl;
}

// Arguments of the backward kernels: the forward geometry plus gradient buffers.
// k.aL / k.cL / k.Y are the saved intermediates of the iteration being differentiated, k.aR its
// abar (for iterations >= 2).  All gradient buffers are fp32.
struct BwdParams {
  KParams k;
  const void* dO;       // storage dtype, strides k.os
  const float* Anext;   // abar of iteration t+1   [bh][m][nk][j][d]   (stage L backward, t < T)
  const float* cmx;     // max_l log L[l, nk] and 1 / sum_l exp(log L - max) of the L that formed
  const float* cinv;    //   abar of iteration t+1   [bh][m][nk][j]     (matrix-unit stage L backward)
  float* dA;            // d abar: stage L backward (t < T) reads that of t+1, stage R backward writes that of t
  float* daL;           // [bh][m][j][nk][d]
  float* dcL;           // [bh][m][j][nk]
  float* dY;            // [bh][m][j][nk][d]
  float* dQ;            // [batch*heads][N_q][d]
  float* dK;            // [batch*heads][N_kv][d]
  float* dV;
  int accumulate;       // add to dQ (stage L backward) / dK (stage R backward) instead of overwriting
  int dq_from_r;        // matrix-unit stage R backward of the first iteration adds d abar_1 to dQ itself
                        // (one key tile per query tile: nothing to sum over), no separate dQ kernel
  const float* lse;     // row statistics the forward call left ([bh][m][j][l], base-2 log-sum-exp) and its
  const float* o32;     // output in fp32 ([bh][m][j][l][d]): stage L backward at t = T then reads its key range
                        // once (null: it forms the statistics in a sweep of its own)
  int dA1_bf16;         // d abar of the first iteration is held as bf16 (matrix-unit stage R backward on a
                        // bf16 workspace), like that of the later iterations: the dQ kernel widens it
};

struct Plan {
  KParams kp;          // everything but the pointers
  int B, T;
  int Nq, Nkv;
  int dtype, compute;
  int ntq_total, c1q;                         // query tiles / query tile rows of the whole grid
  size_t slab_aL, slab_Y, slab_aR, slab_cL;   // bytes per (batch, head, query tile row)
  size_t slab_bytes() const { return slab_aL + slab_Y + slab_aR + slab_cL; }
  bool f32_path() const { return dtype == MRT_F32 || compute == MRT_COMPUTE_F32; }
};

void set_error(const char* fmt, ...);

// The forward call behind monarch_attn_fwd and monarch_attn_fwd_noalloc (mrt_api.cpp).
mrt_status fwd_run(const void* Q, const void* K, const void* V, void* O, const mrt_problem* p, int b1,
                   int b2, int tile, int iters, int causal_chunk, void* workspace,
                   size_t workspace_bytes, void* hip_stream, bool own_stream_only);

// fp32 SIMT path (mrt_f32.hip)
hipError_t launch_f32_stage_r(const KParams& kp, int dtype, int nbh, bool first, bool last,
                              hipStream_t s);
hipError_t launch_f32_stage_l(const KParams& kp, int dtype, int nbh, bool last, hipStream_t s);
hipError_t launch_f32_dense(const KParams& kp, int dtype, int nbh, hipStream_t s);

// backward pass, fp32 (mrt_bwd_f32.hip)
bool bwd_fits(int b1, int b2, int d);
hipError_t launch_bwd_stage_l(const BwdParams& bp, int dtype, int nbh, bool last, hipStream_t s);
hipError_t launch_bwd_stage_r(const BwdParams& bp, int dtype, int nbh, bool first, bool last,
                              hipStream_t s);
hipError_t launch_bwd_q_first(const BwdParams& bp, int nbh, hipStream_t s);

// backward pass on the bf16 matrix unit for short key ranges (mrt_bwd_bf16.hip)
bool bwd_bf16_fits(const KParams& kp);
size_t bwd_bf16_scratch_bytes(const KParams& kp, int ntq_total);
hipError_t launch_bwd_bf16_stage_l(const BwdParams& bp, int nbh, bool last, bool ws_bf16, void* scratch,
                                   hipStream_t s);
bool bwd_bf16_r_fits(const KParams& kp);
hipError_t launch_bwd_bf16_stage_r(const BwdParams& bp, int nbh, bool first, bool last, bool ws_bf16,
                                   hipStream_t s);

// bf16 MFMA path (mrt_bf16.hip)
hipError_t launch_bf16_stage_r(const KParams& kp, int nbh, bool first, bool last, hipStream_t s);
hipError_t launch_bf16_stage_l(const KParams& kp, int nbh, bool last, hipStream_t s);
bool bf16_stage_l_out_streams(const KParams& kp);   // its last-iteration kernel fills lse_out / o32_out
hipError_t launch_bf16_dense(const KParams& kp, int nbh, hipStream_t s);

}  // namespace mrt
