// Internal declarations shared by the host entry points and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "monarchrt.h"

namespace mrt {

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
  int H;        // heads (to split the flat batch*head index)
  int bh0;      // first flat (batch,head) index of this pass
  int d;
  int b1, b2;
  int c2;       // column tiles
  int ntq, ntk; // query tiles IN THIS PASS (workspace extent), key tiles of the whole grid
  int m0;       // first query tile of this pass
  int c1k;      // key tile rows
  int w;        // grid width = c2*b2
  int fb;       // frames per tile row (b1/h); 0 when no mask
  int cc;       // frames per causal chunk; 0 = no mask
  int qoff;     // absolute frame of query frame 0
  int Nq, Nkv;  // tokens per head on the query / key side
  int hw;       // tokens per frame (h*w)
  float scale;
};

// Number of visible key-tile ROWS for query tile row a (tile-level chunk-causal reading:
// key tile row a' is visible iff floor(a'*fb / cc) <= floor((qoff + a*fb) / cc)).
__host__ __device__ inline int visible_key_tile_rows(int a, int c1k, int fb, int cc, int qoff) {
  if (cc == 0) return c1k;
  int q_chunk = (qoff + a * fb) / cc;
  int rows = ((q_chunk + 1) * cc) / fb;
  return rows < c1k ? rows : c1k;
}

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

// fp32 SIMT path (mrt_f32.hip)
hipError_t launch_f32_stage_r(const KParams& kp, int dtype, int nbh, bool first, bool last,
                              hipStream_t s);
hipError_t launch_f32_stage_l(const KParams& kp, int dtype, int nbh, bool last, hipStream_t s);
hipError_t launch_f32_dense(const KParams& kp, int dtype, int nbh, hipStream_t s);

// bf16 MFMA path (mrt_bf16.hip)
hipError_t launch_bf16_stage_r(const KParams& kp, int nbh, bool first, bool last, hipStream_t s);
hipError_t launch_bf16_stage_l(const KParams& kp, int nbh, bool last, hipStream_t s);
hipError_t launch_bf16_dense(const KParams& kp, int nbh, hipStream_t s);

}  // namespace mrt
