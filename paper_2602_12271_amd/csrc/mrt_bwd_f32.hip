// Backward pass of the operator (gradients w.r.t. Q, K, V), fp32 plain-ALU kernels.
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

namespace mrt {

namespace {

constexpr int kThreads = 256;
constexpr int kCH = 16;        // nk rows per chunk in stage L backward
constexpr int kMaxRows = 96;   // rows per thread in the dQ accumulation (b1 <= 192, d <= 128)
constexpr int kMaxAcc = 48;    // (i, v) elements per thread in the dK / dV accumulation

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
__global__ __launch_bounds__(kThreads) void k_bwd_stage_l(BwdParams bp) {
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
    for (int idx = tid; idx < b1 * cn; idx += kThreads) {
      const int l = idx / cn, c = idx - l * cn;
      float acc = 0.f;
      for (int v = 0; v < d; ++v) acc = fmaf(Qj[l * ld + v], Kc[c * ld + v], acc);
      Lc[l * lz + c] = p.scale * acc - cLp[c0 + c];
    }
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

  const int dp = d <= 64 ? 64 : 128;
  const int ngroups = kThreads / dp;
  const int vt = tid % dp, lg = tid / dp;
  float acc[kMaxRows];
#pragma unroll
  for (int r = 0; r < kMaxRows; ++r) acc[r] = 0.f;

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
      for (int idx = tid; idx < b1 * cn; idx += kThreads) {
        const int l = idx / cn, c = idx - l * cn;
        float z = 0.f, u = 0.f;
        for (int v = 0; v < d; ++v) {
          z = fmaf(Qj[l * ld + v], Kc[c * ld + v], z);
          u = fmaf((LAST ? Xj : Qj)[l * ld + v], Wc[c * ld + v], u);
        }
        Lc[l * lz + c] = p.scale * z - cLp[c0 + c] - lse[l];     // log L[l,c]
        Uc[l * lz + c] = LAST ? u : u - tc[c];                    // dL (LAST) or u
      }
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
      for (int idx = tid; idx < cn * d; idx += kThreads) {
        const int c = idx / d, v = idx - c * d;
        float s = 0.f, y = 0.f;
        for (int l = 0; l < b1; ++l) {
          s = fmaf(Uc[l * lz + c], Qj[l * ld + v], s);
          if (LAST) y = fmaf(Lc[l * lz + c], Xj[l * ld + v], y);
        }
        bp.daL[(row0 + c0 + c) * d + v] = p.scale * s;
        if (LAST) bp.dY[(row0 + c0 + c) * d + v] = y;
      }
      if (tid < cn) {
        float s = 0.f;
        for (int l = 0; l < b1; ++l) s += Uc[l * lz + tid];
        bp.dcL[row0 + c0 + tid] = -s;
      }
      // per-row accumulation of dQ
      if (vt < d) {
#pragma unroll
        for (int r = 0; r < kMaxRows; ++r) {
          const int l = lg + r * ngroups;
          if (l < b1) {
            float s = acc[r];
            for (int c = 0; c < cn; ++c) {
              s = fmaf(p.scale * Uc[l * lz + c], Kc[c * ld + vt], s);
              if (!LAST) s = fmaf(Lc[l * lz + c], Wc[c * ld + vt], s);
            }
            acc[r] = s;
          }
        }
      }
    }
    __syncthreads();
  }
  if (vt < d) {
    float* dQp = bp.dQ + (size_t)bh * p.Nq * d;
#pragma unroll
    for (int r = 0; r < kMaxRows; ++r) {
      const int l = lg + r * ngroups;
      if (l < b1) {
        float* dst = dQp + qtok(l) * d + vt;
        *dst = bp.accumulate ? *dst + acc[r] : acc[r];
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

  float accK[kMaxAcc], accV[kMaxAcc];
#pragma unroll
  for (int r = 0; r < kMaxAcc; ++r) { accK[r] = 0.f; accV[r] = 0.f; }

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
    for (int idx = tid; idx < b2 * b2; idx += kThreads) {
      const int jj = idx / b2, i = idx - jj * b2;
      float s = 0.f;
      for (int v = 0; v < d; ++v) s = fmaf(B1[jj * ld + v], B2[i * ld + v], s);
      LR[jj * ls + i] = p.scale * s;
    }
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
    for (int idx = tid; idx < b2 * b2; idx += kThreads) {
      const int jj = idx / b2, i = idx - jj * b2;
      float s = 0.f;
      for (int v = 0; v < d; ++v) s = fmaf(B1[jj * ld + v], B2[i * ld + v], s);
      DR[jj * ls + i] = s + dcl[jj] * (LR[jj * ls + i] + 1.0f);
    }
    // dK += R^T d aL
#pragma unroll
    for (int r = 0; r < kMaxAcc; ++r) {
      const int idx = tid + r * kThreads;
      if (idx < nel) {
        const int i = idx / d, v = idx - i * d;
        float s = accK[r];
        for (int jj = 0; jj < b2; ++jj) s = fmaf(expf(LR[jj * ls + i]), B1[jj * ld + v], s);
        accK[r] = s;
      }
    }
    __syncthreads();
    if (last) {
      load_rows(B1, [&](int jj, int v) { return bp.dY[jrow(jj) * d + v]; });
      load_rows(B2, [&](int i, int v) { return ldf(Vp + ktok(i) * p.vs.token + v); });
      __syncthreads();
      for (int idx = tid; idx < b2 * b2; idx += kThreads) {
        const int jj = idx / b2, i = idx - jj * b2;
        float s = 0.f;
        for (int v = 0; v < d; ++v) s = fmaf(B1[jj * ld + v], B2[i * ld + v], s);
        DR[jj * ls + i] += s;
      }
#pragma unroll
      for (int r = 0; r < kMaxAcc; ++r) {
        const int idx = tid + r * kThreads;
        if (idx < nel) {
          const int i = idx / d, v = idx - i * d;
          float s = accV[r];
          for (int jj = 0; jj < b2; ++jj) s = fmaf(expf(LR[jj * ls + i]), B1[jj * ld + v], s);
          accV[r] = s;
        }
      }
      __syncthreads();
    }
    // dS = R (dR - sum_i R dR), in place
    if (tid < b2) {
      float dot = 0.f;
      for (int i = 0; i < b2; ++i) dot = fmaf(expf(LR[tid * ls + i]), DR[tid * ls + i], dot);
      for (int i = 0; i < b2; ++i) DR[tid * ls + i] = expf(LR[tid * ls + i]) * (DR[tid * ls + i] - dot);
    }
    load_A();
    if (last) load_K();
    __syncthreads();
    // dK += scale dS^T abar ;  d abar = scale dS K
#pragma unroll
    for (int r = 0; r < kMaxAcc; ++r) {
      const int idx = tid + r * kThreads;
      if (idx < nel) {
        const int i = idx / d, v = idx - i * d;
        float s = 0.f;
        for (int jj = 0; jj < b2; ++jj) s = fmaf(DR[jj * ls + i], B1[jj * ld + v], s);
        accK[r] = fmaf(p.scale, s, accK[r]);
      }
    }
    float* dAp = bp.dA + (((size_t)bhl * p.ntq + ml) * NKtot + nk) * b2 * d;
    for (int idx = tid; idx < nel; idx += kThreads) {
      const int jj = idx / d, v = idx - jj * d;
      float s = 0.f;
      for (int i = 0; i < b2; ++i) s = fmaf(DR[jj * ls + i], B2[i * ld + v], s);
      dAp[idx] = p.scale * s;
    }
  }
  float* dKp = bp.dK + (size_t)bh * p.Nkv * d;
  float* dVp = bp.dV + (size_t)bh * p.Nkv * d;
#pragma unroll
  for (int r = 0; r < kMaxAcc; ++r) {
    const int idx = tid + r * kThreads;
    if (idx < nel) {
      const int i = idx / d, v = idx - i * d;
      const size_t off = (size_t)ktok(i) * d + v;
      dKp[off] = bp.accumulate ? dKp[off] + accK[r] : accK[r];
      if (last) dVp[off] = accV[r];
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

size_t bwd_stage_l_lds(int b1, int d, bool last) {
  return ((size_t)(last ? 2 : 1) * b1 * (d + 1) + (size_t)2 * kCH * (d + 1) + (size_t)2 * b1 * (kCH + 1) +
          2 * b1 + 3 * kCH) * 4;
}
size_t bwd_stage_r_lds(int b2, int d) {
  return ((size_t)2 * b2 * (d + 1) + (size_t)2 * b2 * (b2 + 1) + b2) * 4;
}
bool bwd_fits(int b1, int b2, int d) {
  const size_t lim = 160 * 1024;
  return bwd_stage_l_lds(b1, d, true) <= lim && bwd_stage_r_lds(b2, d) <= lim &&
         (size_t)b2 * d <= (size_t)kMaxAcc * kThreads;
}

hipError_t launch_bwd_stage_l(const BwdParams& bp, int dtype, int nbh, bool last, hipStream_t s) {
  const KParams& kp = bp.k;
  const size_t lds = bwd_stage_l_lds(kp.b1, kp.d, last);
  dim3 grid(kp.b2, kp.ntq, nbh);
  hipError_t e;
#define MRT_LAUNCH_BL(T, LASTV)                                                        \
  do {                                                                                 \
    if ((e = allow_lds(k_bwd_stage_l<T, LASTV>, lds)) != hipSuccess) return e;         \
    k_bwd_stage_l<T, LASTV><<<grid, kThreads, lds, s>>>(bp);                           \
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
