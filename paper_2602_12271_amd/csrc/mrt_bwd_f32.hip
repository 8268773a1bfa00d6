// Backward pass of the operator (gradients w.r.t. Q, K, V) in fp32: operands staged in LDS as
// fp32, contractions on the matrix unit in fp32 (mrt_f32_tiles.hpp), the rest plain ALU code.
//
// Monarch finetuning trains through the refinement iterations (Sec. 4.3), so every iteration
// is differentiated.  With the forward quantities of iteration t (App. A notation)
//   abar_t = alpha_R / c_R          R_t = softmax_i(scale abar_t K)
//   aL_t = R_t K, cL_t = sum_i R_t log R_t          L_t = softmax_(n,k)(scale aL_t Q - cL_t)
// and O = sum_(n,k) L_T (R_T V), the reverse sweep runs, for t = T .. 1,
//   stage L backward (one workgroup per (m, j)):   dL_t -> d aL_t, d cL_t, (d Y), dQ
//   stage R backward (one workgroup per (n, k)):   d aL_t, d cL_t, (d Y) -> dK, dV, d abar_t
// and finally dQ[m,k,j] += sum_n d abar_1[m,n,k,j] (abar_1 is Q itself).
// The forward intermediates of every iteration are recomputed by the forward kernels into the
// workspace before the sweep; softmax factors are rebuilt from them on the fly.
#include "mrt_internal.hpp"
#include "mrt_f32_tiles.hpp"

namespace mrt {

namespace {

constexpr int kMaxTiles = 6;   // 16x16 tiles of dQ[m, :, j, :] per wave (b1 <= 192, d <= 128, 4 waves)
constexpr int kMaxAccT = 3;    // 16x16 tiles of dK / dV of one key block per wave (b2 <= 96, d <= 128)

template <typename T> __device__ inline float ldf(const T* p);
template <> __device__ inline float ldf<float>(const float* p) { return *p; }
template <> __device__ inline float ldf<uint16_t>(const uint16_t* p) {
  return __uint_as_float((uint32_t)(*p) << 16);
}

// ---------------------------------------------------------------------------------------
// stage L backward for one (m, j).  Z[l,c] = scale aL[c].Q[l] - cL[c], L = exp(Z - lse[l]).
//   LAST  (t = T):  dL[l,c] = dO[l].Y[c]
//                   dY[c]  = sum_l L[l,c] dO[l]
//   else  (t < T):  abar_(t+1)[c] = sum_l w[l,c] Q[l] with w[l,c] = L[l,c] / sum_l' L[l',c], so
//                   L[l,c] dL[l,c] = w[l,c] u[l,c],  u[l,c] = dA[c].(Q[l] - abar[c])
//                   dQ[l] += sum_c w[l,c] dA[c]
//   both:           delta[l] = sum_c L dL,  dZ = L dL - L delta[l]
//                   d aL[c] = scale sum_l dZ[l,c] Q[l],  d cL[c] = -sum_l dZ[l,c]
//                   dQ[l] += scale sum_c dZ[l,c] aL[c]
// (w is formed as a softmax over l of log L, which cannot produce 0/0.)
// ---------------------------------------------------------------------------------------
template <typename TIn, bool LAST>
__global__ __launch_bounds__(kThreads) void k_bwd_stage_l(BwdParams bp, int kCH) {
  const KParams& p = bp.k;
  extern __shared__ float sm[];
  const int tid = threadIdx.x;
  const int d = p.d, b1 = p.b1, b2 = p.b2, ld = d + 1, lz = kCH + 1;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;

  float* Qj = sm;                          // [b1][ld]   Q[m, :, j, :]
  float* Xj = Qj + b1 * ld;                // [b1][ld]   dO[m, :, j, :]      (LAST only)
  float* Kc = Xj + (LAST ? b1 * ld : 0);   // [kCH][ld]  aL chunk
  float* Wc = Kc + kCH * ld;               // [kCH][ld]  Y chunk (LAST) or dA chunk
  float* Lc = Wc + kCH * ld;               // [b1][lz]   L (LAST) or w
  float* Uc = Lc + b1 * lz;                // [b1][lz]   L dL, then dZ
  float* lse = Uc + b1 * lz;               // [b1]
  float* delta = lse + b1;                 // [b1]
  float* tc = delta + b1;                  // [kCH]      dA[c].abar[c]
  float* cst = tc + kCH;                   // [2*kCH]    column max / inverse column sum of log L

  const TIn* Qp = (const TIn*)p.Q + b * p.qs.batch + hd * p.qs.head;
  const TIn* dOp = (const TIn*)bp.dO + b * p.os.batch + hd * p.os.head;
  const long long qcol = axis_offset(p.cmap, bq * b2 + j);
  auto qtok = [&](int l) { return row_offset(p, a, l) + qcol; };
  for (int idx = tid; idx < b1 * d; idx += kThreads) {
    const int l = idx / d, v = idx - l * d;
    Qj[l * ld + v] = ldf(Qp + qtok(l) * p.qs.token + v);
    if (LAST) Xj[l * ld + v] = ldf(dOp + qtok(l) * p.os.token + v);
  }
  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const float* aLp = (const float*)p.aL + row0 * d;
  const float* Yp = (const float*)p.Y + row0 * d;
  const float* cLp = p.cL + row0;
  // rows (nk, j) of the [m][nk][j][d] arrays
  const size_t arow0 = ((size_t)bhl * p.ntq + ml) * NKtot * b2;
  auto arow = [&](int nk) { return (arow0 + (size_t)nk * b2 + j) * d; };

  // regular Monarch under the chunk-causal mask: hidden (l, nk) are zeros of L (log L = -inf gives
  // L = w = 0 below, so they drop out of every sum)
  auto hidden = [&](int l, int nk) { return p.rl > 0 && nk >= visible_key_rows(p, l); };

  // ---- pass 0: log-sum-exp of every row l
  float rmax = -INFINITY, rsum = 0.f;
  for (int c0 = 0; c0 < NK; c0 += kCH) {
    const int cn = NK - c0 < kCH ? NK - c0 : kCH;
    __syncthreads();
    for (int idx = tid; idx < cn * d; idx += kThreads) {
      const int c = idx / d, v = idx - c * d;
      Kc[c * ld + v] = aLp[(size_t)(c0 + c) * d + v];
    }
    __syncthreads();
    gemm_tiles(b1, cn, d,
               [&](int l, int v) { return l < b1 && v < d ? Qj[l * ld + v] : 0.f; },
               [&](int v, int c) { return c < cn && v < d ? Kc[c * ld + v] : 0.f; },
               [&](int l, int c, float x) { Lc[l * lz + c] = hidden(l, c0 + c) ? -INFINITY : p.scale * x - cLp[c0 + c]; },
               tid);
    __syncthreads();
    if (tid < b1) {
      float mx = rmax;
      for (int c = 0; c < cn; ++c) mx = fmaxf(mx, Lc[tid * lz + c]);
      float s = rsum * expf(rmax - mx);
      for (int c = 0; c < cn; ++c) s += expf(Lc[tid * lz + c] - mx);
      rmax = mx; rsum = s;
    }
  }
  if (tid < b1) { lse[tid] = rmax + logf(rsum); delta[tid] = 0.f; }

  // dQ[m, :, j, :] accumulates over the chunks in registers: 16x16 tiles (l tile, v tile) dealt
  // to the waves, tile t = wave + kWaves * n in dq[n]
  const int wave = tid >> 6, lane = tid & 63;
  const int tnv = (d + 15) >> 4, qtiles = ((b1 + 15) >> 4) * tnv;
  f32x4 dq[kMaxTiles];
#pragma unroll
  for (int n = 0; n < kMaxTiles; ++n) dq[n] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- pass 1 (delta) and pass 2 (gradients)
  for (int pass = 1; pass <= 2; ++pass) {
    for (int c0 = 0; c0 < NK; c0 += kCH) {
      const int cn = NK - c0 < kCH ? NK - c0 : kCH;
      __syncthreads();
      for (int idx = tid; idx < cn * d; idx += kThreads) {
        const int c = idx / d, v = idx - c * d;
        Kc[c * ld + v] = aLp[(size_t)(c0 + c) * d + v];
        Wc[c * ld + v] = LAST ? Yp[(size_t)(c0 + c) * d + v] : bp.dA[arow(c0 + c) + v];
      }
      if (!LAST && tid < cn) {
        const float* da = bp.dA + arow(c0 + tid);
        const float* ab = bp.Anext + arow(c0 + tid);
        float t = 0.f;
        for (int v = 0; v < d; ++v) t = fmaf(da[v], ab[v], t);
        tc[tid] = t;
      }
      __syncthreads();
      const float* Xrows = LAST ? Xj : Qj;
      gemm_tiles(b1, cn, d,
                 [&](int l, int v) { return l < b1 && v < d ? Qj[l * ld + v] : 0.f; },
                 [&](int v, int c) { return c < cn && v < d ? Kc[c * ld + v] : 0.f; },
                 [&](int l, int c, float x) {                                                            // log L
                   Lc[l * lz + c] = hidden(l, c0 + c) ? -INFINITY : p.scale * x - cLp[c0 + c] - lse[l];
                 }, tid);
      gemm_tiles(b1, cn, d,
                 [&](int l, int v) { return l < b1 && v < d ? Xrows[l * ld + v] : 0.f; },
                 [&](int v, int c) { return c < cn && v < d ? Wc[c * ld + v] : 0.f; },
                 [&](int l, int c, float x) { Uc[l * lz + c] = LAST ? x : x - tc[c]; },                  // dL or u
                 tid);
      __syncthreads();
      if (!LAST) {
        if (tid < cn) {
          float mx = -INFINITY;
          for (int l = 0; l < b1; ++l) mx = fmaxf(mx, Lc[l * lz + tid]);
          float s = 0.f;
          for (int l = 0; l < b1; ++l) s += expf(Lc[l * lz + tid] - mx);
          cst[tid] = mx;
          cst[kCH + tid] = 1.0f / s;           // s >= 1
        }
        __syncthreads();
      }
      // Uc <- L dL ; Lc <- L (LAST) or w (else), keeping L in a register for pass 2
      for (int idx = tid; idx < b1 * cn; idx += kThreads) {
        const int l = idx / cn, c = idx - l * cn;
        const float logl = Lc[l * lz + c];
        const float Lv = expf(logl);
        if (LAST) {
          Lc[l * lz + c] = Lv;
          Uc[l * lz + c] *= Lv;
        } else {
          const float w = expf(logl - cst[c]) * cst[kCH + c];
          Uc[l * lz + c] *= w;
          // pass 2 needs both w (for dQ) and L (for dZ): L delta[l] is subtracted right here
          if (pass == 2) Uc[l * lz + c] -= Lv * delta[l];
          Lc[l * lz + c] = w;
        }
      }
      __syncthreads();
      if (pass == 1) {
        if (tid < b1) {
          float s = 0.f;
          for (int c = 0; c < cn; ++c) s += Uc[tid * lz + c];
          delta[tid] += s;
        }
        continue;
      }
      if (LAST) {
        // dZ = L dL - L delta
        for (int idx = tid; idx < b1 * cn; idx += kThreads) {
          const int l = idx / cn, c = idx - l * cn;
          Uc[l * lz + c] -= Lc[l * lz + c] * delta[l];
        }
        __syncthreads();
      }
      // per-column outputs: d aL, d cL, (d Y)
      gemm_tiles(cn, d, b1,
                 [&](int c, int l) { return c < cn && l < b1 ? Uc[l * lz + c] : 0.f; },
                 [&](int l, int v) { return l < b1 && v < d ? Qj[l * ld + v] : 0.f; },
                 [&](int c, int v, float x) { bp.daL[(row0 + c0 + c) * d + v] = p.scale * x; }, tid);
      if (LAST)
        gemm_tiles(cn, d, b1,
                   [&](int c, int l) { return c < cn && l < b1 ? Lc[l * lz + c] : 0.f; },
                   [&](int l, int v) { return l < b1 && v < d ? Xj[l * ld + v] : 0.f; },
                   [&](int c, int v, float x) { bp.dY[(row0 + c0 + c) * d + v] = x; }, tid);
      if (tid < cn) {
        float s = 0.f;
        for (int l = 0; l < b1; ++l) s += Uc[l * lz + tid];
        bp.dcL[row0 + c0 + tid] = -s;
      }
      // per-row accumulation of dQ
#pragma unroll
      for (int n = 0; n < kMaxTiles; ++n) {
        const int t = wave + kWaves * n;
        if (t < qtiles) {
          const int l0 = 16 * (t / tnv), v0 = 16 * (t % tnv);
          dq[n] = mma16([&](int r, int c) { return l0 + r < b1 && c < cn ? p.scale * Uc[(l0 + r) * lz + c] : 0.f; },
                        [&](int c, int v) { return c < cn && v0 + v < d ? Kc[c * ld + v0 + v] : 0.f; }, cn, dq[n], lane);
          if (!LAST)
            dq[n] = mma16([&](int r, int c) { return l0 + r < b1 && c < cn ? Lc[(l0 + r) * lz + c] : 0.f; },
                          [&](int c, int v) { return c < cn && v0 + v < d ? Wc[c * ld + v0 + v] : 0.f; }, cn, dq[n], lane);
        }
      }
    }
    __syncthreads();
  }
  {
    float* dQp = bp.dQ + (size_t)bh * p.Nq * d;
    const int i = lane & 15, q = lane >> 4;
#pragma unroll
    for (int n = 0; n < kMaxTiles; ++n) {
      const int t = wave + kWaves * n;
      if (t < qtiles) {
        const int l0 = 16 * (t / tnv), v0 = 16 * (t % tnv);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int l = l0 + 4 * q + r, v = v0 + i;
          if (l < b1 && v < d) {
            float* dst = dQp + qtok(l) * d + v;
            *dst = bp.accumulate ? *dst + dq[n][r] : dq[n][r];
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// stage R backward for one key block (n, k), looping over the query tiles m that see it:
//   R = softmax_i(scale abar K),  log R kept (R log R stays finite when R underflows)
//   dR[j,i] = d aL[j].K[i] + d cL[j] (log R[j,i] + 1) (+ d Y[j].V[i] at t = T)
//   dS = R (dR - sum_i R dR)
//   dK[i] += sum_j R[j,i] d aL[j] + scale sum_j dS[j,i] abar[j]      dV[i] += sum_j R[j,i] d Y[j]
//   d abar[j] = scale sum_i dS[j,i] K[i]
// dK and dV are summed over m in registers and written (or added, for t < T) once.
// ---------------------------------------------------------------------------------------
template <typename TIn>
__global__ __launch_bounds__(kThreads) void k_bwd_stage_r(BwdParams bp, int first, int last) {
  const KParams& p = bp.k;
  extern __shared__ float sm[];
  const int tid = threadIdx.x;
  const int d = p.d, b1 = p.b1, b2 = p.b2, ld = d + 1, ls = b2 + 1;
  const int nk = blockIdx.x, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int n = nk / b1, k = nk - n * b1;
  const int an = n / p.c2, bn = n - an * p.c2;
  const int b = bh / p.H, hd = bh - b * p.H;

  float* B1 = sm;                 // [b2][ld]  abar, then d aL, d Y, abar again
  float* B2 = B1 + b2 * ld;       // [b2][ld]  K, V, K again
  float* LR = B2 + b2 * ld;       // [b2][ls]  log R
  float* DR = LR + b2 * ls;       // [b2][ls]  dR, then dS
  float* dcl = DR + b2 * ls;      // [b2]

  const long long krow = row_offset(p, an, k);
  auto ktok = [&](int i) { return krow + axis_offset(p.cmap, bn * b2 + i); };
  const TIn* Qp = (const TIn*)p.Q + b * p.qs.batch + hd * p.qs.head;
  const TIn* Kp = (const TIn*)p.K + b * p.ks.batch + hd * p.ks.head;
  const TIn* Vp = (const TIn*)p.V + b * p.vs.batch + hd * p.vs.head;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int nel = b2 * d;

  // dK and dV of the block accumulate over the query tiles in registers: 16x16 tiles
  // (i tile, v tile) dealt to the waves, tile t = wave + kWaves * n in accK[n] / accV[n]
  const int wave = tid >> 6, lane = tid & 63;
  const int tnv = (d + 15) >> 4, ktiles = ((b2 + 15) >> 4) * tnv;
  f32x4 accK[kMaxAccT], accV[kMaxAccT];
#pragma unroll
  for (int n = 0; n < kMaxAccT; ++n) {
    accK[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    accV[n] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // acc[n] += P^T X for P[jj][i] (b2 x b2, row stride ls) and X[jj][v] (b2 x d, row stride ld)
  auto accumulate_t = [&](f32x4 (&acc)[kMaxAccT], const float* P, const float* X, float mul) {
#pragma unroll
    for (int n = 0; n < kMaxAccT; ++n) {
      const int t = wave + kWaves * n;
      if (t < ktiles) {
        const int i0 = 16 * (t / tnv), v0 = 16 * (t % tnv);
        acc[n] = mma16([&](int r, int jj) { return i0 + r < b2 && jj < b2 ? mul * P[jj * ls + i0 + r] : 0.f; },
                       [&](int jj, int v) { return jj < b2 && v0 + v < d ? X[jj * ld + v0 + v] : 0.f; }, b2,
                       acc[n], lane);
      }
    }
  };
  auto rows_dot = [&](const float* X, const float* Y, auto done) {   // done(jj, i, X[jj].Y[i])
    gemm_tiles(b2, b2, d,
               [&](int jj, int v) { return jj < b2 && v < d ? X[jj * ld + v] : 0.f; },
               [&](int v, int i) { return i < b2 && v < d ? Y[i * ld + v] : 0.f; }, done, tid);
  };

  auto load_rows = [&](float* dst, auto src) {     // dst[j][v] = src(j, v)
    for (int idx = tid; idx < nel; idx += kThreads) {
      const int jj = idx / d, v = idx - jj * d;
      dst[jj * ld + v] = src(jj, v);
    }
  };
  auto load_K = [&]() { load_rows(B2, [&](int i, int v) { return ldf(Kp + ktok(i) * p.ks.token + v); }); };

  for (int ml = 0; ml < p.ntq; ++ml) {
    const int m = p.m0 + ml, a = m / p.c2, bq = m - a * p.c2;
    if (an >= visible_key_tile_rows(a, p.c1k, p.ct, p.qt0)) continue;   // uniform per workgroup
    const long long qrow = row_offset(p, a, k);
    const float* aRp = (const float*)p.aR + (((size_t)bhl * p.ntq + ml) * NKtot + nk) * b2 * d;
    auto load_A = [&]() {
      load_rows(B1, [&](int jj, int v) {
        return first ? ldf(Qp + (qrow + axis_offset(p.cmap, bq * b2 + jj)) * p.qs.token + v)
                     : aRp[(size_t)jj * d + v];
      });
    };
    // rows (j, nk) of the [m][j][nk][d] arrays
    const size_t jrow0 = ((size_t)bhl * p.ntq + ml) * b2;
    auto jrow = [&](int jj) { return (jrow0 + jj) * NKtot + nk; };

    __syncthreads();
    load_A();
    load_K();
    if (tid < b2) dcl[tid] = bp.dcL[jrow(tid)];
    __syncthreads();
    // logits
    rows_dot(B1, B2, [&](int jj, int i, float x) { LR[jj * ls + i] = p.scale * x; });
    __syncthreads();
    if (tid < b2) {
      float mx = -INFINITY;
      for (int i = 0; i < b2; ++i) mx = fmaxf(mx, LR[tid * ls + i]);
      float s = 0.f;
      for (int i = 0; i < b2; ++i) s += expf(LR[tid * ls + i] - mx);
      const float l = mx + logf(s);
      for (int i = 0; i < b2; ++i) LR[tid * ls + i] -= l;         // log R
    }
    __syncthreads();
    // d aL into B1 (K still in B2)
    load_rows(B1, [&](int jj, int v) { return bp.daL[jrow(jj) * d + v]; });
    __syncthreads();
    rows_dot(B1, B2, [&](int jj, int i, float x) { DR[jj * ls + i] = x + dcl[jj] * (LR[jj * ls + i] + 1.0f); });
    __syncthreads();
    // from here on LR holds R itself (log R was only needed for the entropy term above)
    for (int idx = tid; idx < b2 * b2; idx += kThreads) {
      const int jj = idx / b2, i = idx - jj * b2;
      LR[jj * ls + i] = expf(LR[jj * ls + i]);
    }
    __syncthreads();
    accumulate_t(accK, LR, B1, 1.0f);          // dK += R^T d aL
    __syncthreads();
    if (last) {
      load_rows(B1, [&](int jj, int v) { return bp.dY[jrow(jj) * d + v]; });
      load_rows(B2, [&](int i, int v) { return ldf(Vp + ktok(i) * p.vs.token + v); });
      __syncthreads();
      rows_dot(B1, B2, [&](int jj, int i, float x) { DR[jj * ls + i] += x; });
      accumulate_t(accV, LR, B1, 1.0f);        // dV += R^T d Y
      __syncthreads();
    }
    // dS = R (dR - sum_i R dR), in place
    if (tid < b2) {
      float dot = 0.f;
      for (int i = 0; i < b2; ++i) dot = fmaf(LR[tid * ls + i], DR[tid * ls + i], dot);
      for (int i = 0; i < b2; ++i) DR[tid * ls + i] = LR[tid * ls + i] * (DR[tid * ls + i] - dot);
    }
    load_A();
    if (last) load_K();
    __syncthreads();
    // dK += scale dS^T abar ;  d abar = scale dS K
    accumulate_t(accK, DR, B1, p.scale);
    float* dAp = bp.dA + (((size_t)bhl * p.ntq + ml) * NKtot + nk) * b2 * d;
    gemm_tiles(b2, d, b2,
               [&](int jj, int i) { return jj < b2 && i < b2 ? DR[jj * ls + i] : 0.f; },
               [&](int i, int v) { return i < b2 && v < d ? B2[i * ld + v] : 0.f; },
               [&](int jj, int v, float x) { dAp[(size_t)jj * d + v] = p.scale * x; }, tid);
  }
  float* dKp = bp.dK + (size_t)bh * p.Nkv * d;
  float* dVp = bp.dV + (size_t)bh * p.Nkv * d;
  const int li = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int n = 0; n < kMaxAccT; ++n) {
    const int t = wave + kWaves * n;
    if (t < ktiles) {
      const int i0 = 16 * (t / tnv), v0 = 16 * (t % tnv);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = i0 + 4 * lq + r, v = v0 + li;
        if (i < b2 && v < d) {
          const size_t off = (size_t)ktok(i) * d + v;
          dKp[off] = bp.accumulate ? dKp[off] + accK[n][r] : accK[n][r];
          if (last) dVp[off] = accV[n][r];
        }
      }
    }
  }
}

// dQ[m, k, j, :] += sum over the visible key tiles n of d abar_1[m, (n,k), j, :]
__global__ __launch_bounds__(kThreads) void k_bwd_q_first(BwdParams bp) {
  const KParams& p = bp.k;
  const int d = p.d, b1 = p.b1, b2 = p.b2;
  const int k = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int nvis = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2;
  const size_t NKtot = (size_t)p.ntk * b1;
  const float* dAp = bp.dA + ((size_t)bhl * p.ntq + ml) * NKtot * b2 * d;
  float* dQp = bp.dQ + (size_t)bh * p.Nq * d;
  const long long qrow = row_offset(p, a, k);
  if (bp.dA1_bf16) {
    // bf16 terms (d is 64 or 128 there): eight features per lane, four key tiles in flight; the
    // terms are read once and by nobody else (non-temporal loads)
    const unsigned short* dA16 = (const unsigned short*)bp.dA + ((size_t)bhl * p.ntq + ml) * NKtot * b2 * d;
    typedef __attribute__((ext_vector_type(4))) unsigned ux4;
    const ux4* src = (const ux4*)(dA16 + (size_t)k * b2 * d);
    auto ld = [&](size_t at) { return __builtin_nontemporal_load(src + at); };
    const size_t per_n = (size_t)b1 * b2 * d / 8;
    auto add8 = [](f32x4& lo, f32x4& hi, const ux4 x) {
      lo += f32x4{__uint_as_float(x.x << 16), __uint_as_float(x.x & 0xffff0000u),
                  __uint_as_float(x.y << 16), __uint_as_float(x.y & 0xffff0000u)};
      hi += f32x4{__uint_as_float(x.z << 16), __uint_as_float(x.z & 0xffff0000u),
                  __uint_as_float(x.w << 16), __uint_as_float(x.w & 0xffff0000u)};
    };
    for (int idx = threadIdx.x; idx < b2 * d / 8; idx += kThreads) {
      const int jj = (8 * idx) / d, v = 8 * idx - jj * d;
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
      int n = 0;
      for (; n + 4 <= nvis; n += 4) {
        const ux4 x0 = ld((size_t)n * per_n + idx), x1 = ld((size_t)(n + 1) * per_n + idx);
        const ux4 x2 = ld((size_t)(n + 2) * per_n + idx), x3 = ld((size_t)(n + 3) * per_n + idx);
        add8(s0, s1, x0); add8(s0, s1, x1); add8(s0, s1, x2); add8(s0, s1, x3);
      }
      for (; n < nvis; ++n) add8(s0, s1, ld((size_t)n * per_n + idx));
      f32x4* dst = (f32x4*)(dQp + (qrow + axis_offset(p.cmap, bq * b2 + jj)) * d + v);
      dst[0] += s0;
      dst[1] += s1;
    }
    return;
  }
  if (d % 4 == 0) {
    // four features per lane, four key tiles in flight per step (a pure stream: the loads are all
    // there is to hide)
    const f32x4* src = (const f32x4*)(dAp + (size_t)k * b2 * d);
    const size_t per_n = (size_t)b1 * b2 * d / 4;
    for (int idx = threadIdx.x; idx < b2 * d / 4; idx += kThreads) {
      const int jj = (4 * idx) / d, v = 4 * idx - jj * d;
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      int n = 0;
      for (; n + 4 <= nvis; n += 4) {
        const f32x4 x0 = src[(size_t)n * per_n + idx], x1 = src[(size_t)(n + 1) * per_n + idx];
        const f32x4 x2 = src[(size_t)(n + 2) * per_n + idx], x3 = src[(size_t)(n + 3) * per_n + idx];
        s += (x0 + x1) + (x2 + x3);
      }
      for (; n < nvis; ++n) s += src[(size_t)n * per_n + idx];
      f32x4* dst = (f32x4*)(dQp + (qrow + axis_offset(p.cmap, bq * b2 + jj)) * d + v);
      *dst += s;
    }
    return;
  }
  for (int idx = threadIdx.x; idx < b2 * d; idx += kThreads) {
    const int jj = idx / d, v = idx - jj * d;
    float s = 0.f;
    for (int n = 0; n < nvis; ++n) s += dAp[(((size_t)n * b1 + k) * b2 + jj) * d + v];
    dQp[(qrow + axis_offset(p.cmap, bq * b2 + jj)) * d + v] += s;
  }
}

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return hipSuccess;
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

size_t bwd_stage_l_lds(int b1, int d, bool last, int ch) {
  return ((size_t)(last ? 2 : 1) * b1 * (d + 1) + (size_t)2 * ch * (d + 1) + (size_t)2 * b1 * (ch + 1) +
          2 * b1 + 3 * ch) * 4;
}
size_t bwd_stage_r_lds(int b2, int d) {
  return ((size_t)2 * b2 * (d + 1) + (size_t)2 * b2 * (b2 + 1) + b2) * 4;
}
bool bwd_fits(int b1, int b2, int d) {
  const size_t lim = 160 * 1024;
  return bwd_stage_l_lds(b1, d, true, 16) <= lim && bwd_stage_r_lds(b2, d) <= lim &&
         ((b2 + 15) / 16) * ((d + 15) / 16) <= kMaxAccT * kWaves &&
         ((b1 + 15) / 16) * ((d + 15) / 16) <= kMaxTiles * kWaves;
}

hipError_t launch_bwd_stage_l(const BwdParams& bp, int dtype, int nbh, bool last, hipStream_t s) {
  const KParams& kp = bp.k;
  // nk rows per chunk: the largest of 64 / 32 / 16 whose buffers fit on chip
  int ch = 64;
  while (ch > 16 && bwd_stage_l_lds(kp.b1, kp.d, last, ch) > 160 * 1024) ch /= 2;
  const size_t lds = bwd_stage_l_lds(kp.b1, kp.d, last, ch);
  dim3 grid(kp.b2, kp.ntq, nbh);
  hipError_t e;
#define MRT_LAUNCH_BL(T, LASTV)                                                        \
  do {                                                                                 \
    if ((e = allow_lds(k_bwd_stage_l<T, LASTV>, lds)) != hipSuccess) return e;         \
    k_bwd_stage_l<T, LASTV><<<grid, kThreads, lds, s>>>(bp, ch);                          \
  } while (0)
  if (dtype == MRT_F32) { if (last) MRT_LAUNCH_BL(float, true); else MRT_LAUNCH_BL(float, false); }
  else { if (last) MRT_LAUNCH_BL(uint16_t, true); else MRT_LAUNCH_BL(uint16_t, false); }
#undef MRT_LAUNCH_BL
  return hipGetLastError();
}

hipError_t launch_bwd_stage_r(const BwdParams& bp, int dtype, int nbh, bool first, bool last,
                              hipStream_t s) {
  const KParams& kp = bp.k;
  const size_t lds = bwd_stage_r_lds(kp.b2, kp.d);
  dim3 grid(kp.ntk * kp.b1, 1, nbh);
  hipError_t e;
  if (dtype == MRT_F32) {
    if ((e = allow_lds(k_bwd_stage_r<float>, lds)) != hipSuccess) return e;
    k_bwd_stage_r<float><<<grid, kThreads, lds, s>>>(bp, first, last);
  } else {
    if ((e = allow_lds(k_bwd_stage_r<uint16_t>, lds)) != hipSuccess) return e;
    k_bwd_stage_r<uint16_t><<<grid, kThreads, lds, s>>>(bp, first, last);
  }
  return hipGetLastError();
}

hipError_t launch_bwd_q_first(const BwdParams& bp, int nbh, hipStream_t s) {
  const KParams& kp = bp.k;
  dim3 grid(kp.b1, kp.ntq, nbh);
  k_bwd_q_first<<<grid, kThreads, 0, s>>>(bp);
  return hipGetLastError();
}

}  // namespace mrt
