// fp32 path: fp32 arithmetic and fp32 intermediates; the contractions run on the matrix unit in
// fp32 (v_mfma_f32_16x16x4_f32 on fp32 operands held in LDS), everything else is plain ALU code.
//
// Used for f32 storage (the 1e-4 parity class) and, on request, as a device-side
// cross-check for bf16 storage.  Same three stages as the MFMA path:
//   stage R  (one workgroup per (m, n, k)):  Z_R, R = softmax_i, c_L, alpha_L, (Y)
//   stage L  (one workgroup per (m, j)):     Z_L, L = softmax_(n,k), then alpha_R/c_R or O
// Equation references: App. A.1 / A.2 update equations.
#include "mrt_internal.hpp"
#include "mrt_f32_tiles.hpp"

namespace mrt {

namespace {

template <typename T> __device__ inline float ldf(const T* p);
template <> __device__ inline float ldf<float>(const float* p) { return *p; }
template <> __device__ inline float ldf<uint16_t>(const uint16_t* p) {
  return __uint_as_float((uint32_t)(*p) << 16);
}
template <typename T> __device__ inline void stf(T* p, float x);
template <> __device__ inline void stf<float>(float* p, float x) { *p = x; }
template <> __device__ inline void stf<uint16_t>(uint16_t* p, float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------------------------------
// stage R:  for one (m, n, k):
//   Z_R[j,i] = scale * sum_v A[j,v] K[n,k,i,v]        A = Q[m,k,j,:] at t=1 (L = identity),
//                                                      A = alpha_R/c_R from the workspace later
//   R = softmax_i Z_R;  c_L[j] = sum_i R log R;  alpha_L[j,:] = sum_i R[j,i] K[i,:];  Y likewise
// ---------------------------------------------------------------------------------------
template <typename TIn>
__global__ __launch_bounds__(kThreads) void k_f32_stage_r(KParams p, int first, int last) {
  extern __shared__ float sm[];
  const int tid = threadIdx.x;
  const int d = p.d, b1 = p.b1, b2 = p.b2, ld = d + 1, ls = b2 + 1;
  const int nk = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int n = nk / b1, k = nk - n * b1;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int an = n / p.c2, bn = n - an * p.c2;
  if (an >= visible_key_tile_rows(a, p.c1k, p.ct, p.qt0)) return;
  const int b = bh / p.H, hd = bh - b * p.H;

  float* A = sm;
  float* Kb = A + b2 * ld;
  float* S = Kb + b2 * ld;

  // block-grid rows a*b1 + k (queries) and an*b1 + k (keys); columns bq*b2 + j and bn*b2 + i
  const long long qrow = row_offset(p, a, k), krow = row_offset(p, an, k);
  auto qtok = [&](int j) { return qrow + axis_offset(p.cmap, bq * b2 + j); };
  auto ktok = [&](int i) { return krow + axis_offset(p.cmap, bn * b2 + i); };
  const TIn* Qp = (const TIn*)p.Q + b * p.qs.batch + hd * p.qs.head;
  const TIn* Kp = (const TIn*)p.K + b * p.ks.batch + hd * p.ks.head;
  const TIn* Vp = (const TIn*)p.V + b * p.vs.batch + hd * p.vs.head;
  const size_t NKtot = (size_t)p.ntk * b1;
  const float* aRp = (const float*)p.aR + (((size_t)bhl * p.ntq + ml) * NKtot + nk) * b2 * d;

  for (int idx = tid; idx < b2 * d; idx += kThreads) {
    const int j = idx / d, v = idx - j * d;
    A[j * ld + v] = first ? ldf(Qp + qtok(j) * p.qs.token + v) : aRp[idx];
    Kb[j * ld + v] = ldf(Kp + ktok(j) * p.ks.token + v);
  }
  __syncthreads();
  gemm_tiles(b2, b2, d,
             [&](int j, int v) { return j < b2 && v < d ? A[j * ld + v] : 0.f; },
             [&](int v, int i) { return i < b2 && v < d ? Kb[i * ld + v] : 0.f; },
             [&](int j, int i, float x) { S[j * ls + i] = p.scale * x; }, tid);
  __syncthreads();
  if (tid < b2) {
    const int j = tid;
    float mx = -INFINITY;
    for (int i = 0; i < b2; ++i) mx = fmaxf(mx, S[j * ls + i]);
    float sum = 0.f, ent = 0.f;
    for (int i = 0; i < b2; ++i) {
      const float z = S[j * ls + i] - mx;
      const float e = expf(z);
      sum += e;
      ent = fmaf(e, z, ent);
      S[j * ls + i] = e;
    }
    const float inv = 1.0f / sum;
    for (int i = 0; i < b2; ++i) S[j * ls + i] *= inv;
    // sum_i R log R = (sum_i e z)/sum - log(sum)
    p.cL[(((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot + nk] = ent * inv - logf(sum);
  }
  __syncthreads();
  float* aLp = (float*)p.aL + ((((size_t)bhl * p.ntq + ml) * b2) * NKtot + nk) * d;
  float* Yp = (float*)p.Y + ((((size_t)bhl * p.ntq + ml) * b2) * NKtot + nk) * d;
  const size_t jstride = NKtot * d;
  gemm_tiles(b2, d, b2,
             [&](int j, int i) { return j < b2 && i < b2 ? S[j * ls + i] : 0.f; },
             [&](int i, int v) { return i < b2 && v < d ? Kb[i * ld + v] : 0.f; },
             [&](int j, int v, float x) { aLp[j * jstride + v] = x; }, tid);
  if (last) {
    __syncthreads();                  // every wave is done with K: the tile now holds V
    for (int idx = tid; idx < b2 * d; idx += kThreads) {
      const int i = idx / d, v = idx - i * d;
      Kb[i * ld + v] = ldf(Vp + ktok(i) * p.vs.token + v);
    }
    __syncthreads();
    gemm_tiles(b2, d, b2,
               [&](int j, int i) { return j < b2 && i < b2 ? S[j * ls + i] : 0.f; },
               [&](int i, int v) { return i < b2 && v < d ? Kb[i * ld + v] : 0.f; },
               [&](int j, int v, float x) { Yp[j * jstride + v] = x; }, tid);
  }
}

// ---------------------------------------------------------------------------------------
// stage L:  for one (m, j):
//   Z_L[l,nk] = scale * sum_v alpha_L[nk,v] Q[m,l,j,v] - c_L[nk];  L = softmax over visible nk
//   last iteration:   O[l,:]  = sum_nk L[l,nk] Y[nk,:]
//   otherwise:        alpha_R[nk,:]/c_R[nk] = sum_l L[l,nk] Q[l,:] / sum_l L[l,nk]
// The second form is evaluated as a softmax over l of log L[l,nk] (column maximum removed),
// which is the same ratio and cannot underflow to 0/0.
// ---------------------------------------------------------------------------------------
constexpr int kCH = 16;     // nk rows per chunk
constexpr int kMaxTiles = 6;   // 16x16 output tiles per wave in the last stage (b1 <= 192, d <= 128)

template <typename TIn, bool LAST>
__global__ __launch_bounds__(kThreads) void k_f32_stage_l(KParams p) {
  extern __shared__ float sm[];
  const int tid = threadIdx.x;
  const int d = p.d, b1 = p.b1, b2 = p.b2, ld = d + 1, lz = kCH + 1;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;

  float* Qj = sm;                    // [b1][ld]
  float* Kc = Qj + b1 * ld;          // [kCH][ld]
  float* Zc = Kc + kCH * ld;         // [b1][lz]
  float* lse = Zc + b1 * lz;         // [b1]
  float* cmx = lse + b1;             // [kCH]
  float* cinv = cmx + kCH;           // [kCH]

  const TIn* Qp = (const TIn*)p.Q + b * p.qs.batch + hd * p.qs.head;
  const long long qcol = axis_offset(p.cmap, bq * b2 + j);
  auto qtok = [&](int l) { return row_offset(p, a, l) + qcol; };
  for (int idx = tid; idx < b1 * d; idx += kThreads) {
    const int l = idx / d, v = idx - l * d;
    Qj[l * ld + v] = ldf(Qp + qtok(l) * p.qs.token + v);
  }
  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const float* aLp = (const float*)p.aL + row0 * d;
  const float* Yp = (const float*)p.Y + row0 * d;
  const float* cLp = p.cL + row0;

  // regular Monarch under the chunk-causal mask: key rows of later chunks are zeros of L (the
  // first chunk of 16 key rows always holds a visible one, so the running maximum is finite)
  auto hidden = [&](int l, int nk) { return p.rl > 0 && nk >= visible_key_rows(p, l); };

  // pass 1: log-sum-exp of every row l over all visible nk
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
               [&](int l, int c, float x) { Zc[l * lz + c] = hidden(l, c0 + c) ? -INFINITY : p.scale * x - cLp[c0 + c]; },
               tid);
    __syncthreads();
    if (tid < b1) {
      float mx = rmax;
      for (int c = 0; c < cn; ++c) mx = fmaxf(mx, Zc[tid * lz + c]);
      float s = rsum * expf(rmax - mx);
      for (int c = 0; c < cn; ++c) s += expf(Zc[tid * lz + c] - mx);
      rmax = mx; rsum = s;
    }
  }
  if (tid < b1) lse[tid] = rmax + logf(rsum);

  // pass 2
  // O[m, :, j, :] accumulates over the chunks in registers: 16x16 tiles (l tile, v tile) dealt to
  // the waves, tile t = wave + kWaves * n in acc[n]
  const int wave = tid >> 6, lane = tid & 63;
  const int tnv = (d + 15) >> 4, otiles = ((b1 + 15) >> 4) * tnv;
  f32x4 acc[kMaxTiles];
  if (LAST) {
#pragma unroll
    for (int n = 0; n < kMaxTiles; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  float* aRout = (float*)p.aR + ((size_t)bhl * p.ntq + ml) * NKtot * b2 * d;

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
               [&](int l, int c, float x) {
                 const float z = hidden(l, c0 + c) ? -INFINITY : p.scale * x - cLp[c0 + c] - lse[l];   // log L[l,nk]
                 Zc[l * lz + c] = LAST ? expf(z) : z;
               }, tid);
    __syncthreads();
    if (LAST) {
      for (int idx = tid; idx < cn * d; idx += kThreads) {
        const int c = idx / d, v = idx - c * d;
        Kc[c * ld + v] = Yp[(size_t)(c0 + c) * d + v];
      }
      __syncthreads();
#pragma unroll
      for (int n = 0; n < kMaxTiles; ++n) {
        const int t = wave + kWaves * n;
        if (t < otiles) {
          const int l0 = 16 * (t / tnv), v0 = 16 * (t % tnv);
          acc[n] = mma16([&](int r, int c) { return l0 + r < b1 && c < cn ? Zc[(l0 + r) * lz + c] : 0.f; },
                         [&](int c, int v) { return c < cn && v0 + v < d ? Kc[c * ld + v0 + v] : 0.f; }, cn,
                         acc[n], lane);
        }
      }
    } else {
      if (tid < cn) {
        float mx = -INFINITY;
        for (int l = 0; l < b1; ++l) mx = fmaxf(mx, Zc[l * lz + tid]);
        cmx[tid] = mx;
      }
      __syncthreads();
      for (int idx = tid; idx < b1 * cn; idx += kThreads) {
        const int l = idx / cn, c = idx - l * cn;
        Zc[l * lz + c] = expf(Zc[l * lz + c] - cmx[c]);
      }
      __syncthreads();
      if (tid < cn) {
        float s = 0.f;
        for (int l = 0; l < b1; ++l) s += Zc[l * lz + tid];
        cinv[tid] = 1.0f / s;      // s >= 1: the column maximum contributes exp(0)
        if (p.cmx_out) {
          const size_t at = ((size_t)bhl * p.ntq + ml) * NKtot * b2 + (size_t)(c0 + tid) * b2 + j;
          p.cmx_out[at] = cmx[tid];
          p.cinv_out[at] = cinv[tid];
        }
      }
      __syncthreads();
      gemm_tiles(cn, d, b1,
                 [&](int c, int l) { return c < cn && l < b1 ? Zc[l * lz + c] : 0.f; },
                 [&](int l, int v) { return l < b1 && v < d ? Qj[l * ld + v] : 0.f; },
                 [&](int c, int v, float x) { aRout[((size_t)(c0 + c) * b2 + j) * d + v] = x * cinv[c]; }, tid);
    }
  }
  if (LAST) {
    TIn* Op = (TIn*)p.O + b * p.os.batch + hd * p.os.head;
    const int li = lane & 15, lq = lane >> 4;
#pragma unroll
    for (int n = 0; n < kMaxTiles; ++n) {
      const int t = wave + kWaves * n;
      if (t < otiles) {
        const int l0 = 16 * (t / tnv), v0 = 16 * (t % tnv);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int l = l0 + 4 * lq + r, v = v0 + li;
          if (l < b1 && v < d) stf(Op + qtok(l) * p.os.token + v, acc[n][r]);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// dense baseline: softmax(scale Q K^T + mask) V, 16 query rows per workgroup, online softmax
// ---------------------------------------------------------------------------------------
constexpr int kDQ = 16, kDK = 64;

template <typename TIn>
__global__ __launch_bounds__(kThreads) void k_f32_dense(KParams p) {
  extern __shared__ float sm[];
  const int tid = threadIdx.x;
  const int d = p.d, ld = d + 1, lz = kDK + 1;
  const int q0 = blockIdx.x * kDQ, bh = blockIdx.y;
  const int b = bh / p.H, hd = bh - b * p.H;
  float* Qb = sm;                   // [kDQ][ld]
  float* Kc = Qb + kDQ * ld;        // [kDK][ld]
  float* S = Kc + kDK * ld;         // [kDQ][lz]
  float* alpha = S + kDQ * lz;      // [kDQ]
  float* rinv = alpha + kDQ;        // [kDQ]
  const TIn* Qp = (const TIn*)p.Q + b * p.qs.batch + hd * p.qs.head;
  const TIn* Kp = (const TIn*)p.K + b * p.ks.batch + hd * p.ks.head;
  const TIn* Vp = (const TIn*)p.V + b * p.vs.batch + hd * p.vs.head;
  const int qn = p.Nq - q0 < kDQ ? p.Nq - q0 : kDQ;
  for (int idx = tid; idx < kDQ * d; idx += kThreads) {
    const int r = idx / d, v = idx - r * d;
    Qb[r * ld + v] = r < qn ? ldf(Qp + (long long)(q0 + r) * p.qs.token + v) : 0.f;
  }
  const int dp = d <= 64 ? 64 : 128;
  const int ngroups = kThreads / dp;             // 2 or 4
  const int vt = tid % dp, lg = tid / dp;
  float acc[kDQ / 2];
#pragma unroll
  for (int r = 0; r < kDQ / 2; ++r) acc[r] = 0.f;
  float rmax = -INFINITY, rsum = 0.f;            // threads < kDQ
  int q_chunk = 0;
  if (tid < kDQ && p.cc > 0) {
    const int qt = q0 + tid < p.Nq ? q0 + tid : p.Nq - 1;
    q_chunk = (p.qoff + qt / p.hw) / p.cc;
  }
  // keys beyond the last visible chunk of the LAST query row of this block are never needed
  int nkeys = p.Nkv;
  if (p.cc > 0) {
    const int qlast = q0 + qn - 1;
    const long long lim = (long long)((p.qoff + qlast / p.hw) / p.cc + 1) * p.cc * p.hw;
    if (lim < nkeys) nkeys = (int)lim;
  }
  for (int c0 = 0; c0 < nkeys; c0 += kDK) {
    const int cn = nkeys - c0 < kDK ? nkeys - c0 : kDK;
    __syncthreads();
    for (int idx = tid; idx < cn * d; idx += kThreads) {
      const int c = idx / d, v = idx - c * d;
      Kc[c * ld + v] = ldf(Kp + (long long)(c0 + c) * p.ks.token + v);
    }
    __syncthreads();
    for (int idx = tid; idx < kDQ * cn; idx += kThreads) {
      const int r = idx / cn, c = idx - r * cn;
      float s = 0.f;
      for (int v = 0; v < d; ++v) s = fmaf(Qb[r * ld + v], Kc[c * ld + v], s);
      S[r * lz + c] = p.scale * s;
    }
    __syncthreads();
    if (tid < kDQ) {
      float mx = rmax;
      for (int c = 0; c < cn; ++c) {
        const bool vis = p.cc == 0 || ((c0 + c) / p.hw) / p.cc <= q_chunk;
        if (!vis) S[tid * lz + c] = -INFINITY;
        mx = fmaxf(mx, S[tid * lz + c]);
      }
      const float al = (rmax == -INFINITY) ? 0.f : expf(rmax - mx);
      float s = rsum * al;
      for (int c = 0; c < cn; ++c) {
        const float e = (mx == -INFINITY) ? 0.f : expf(S[tid * lz + c] - mx);
        S[tid * lz + c] = e;
        s += e;
      }
      rmax = mx; rsum = s; alpha[tid] = al;
    }
    __syncthreads();
    for (int idx = tid; idx < cn * d; idx += kThreads) {
      const int c = idx / d, v = idx - c * d;
      Kc[c * ld + v] = ldf(Vp + (long long)(c0 + c) * p.vs.token + v);
    }
    __syncthreads();
    if (vt < d) {
#pragma unroll
      for (int r = 0; r < kDQ / 2; ++r) {
        const int row = lg + r * ngroups;
        if (row < kDQ) {
          float s = acc[r] * alpha[row];
          for (int c = 0; c < cn; ++c) s = fmaf(S[row * lz + c], Kc[c * ld + vt], s);
          acc[r] = s;
        }
      }
    }
  }
  __syncthreads();
  if (tid < kDQ) rinv[tid] = rsum > 0.f ? 1.0f / rsum : 0.f;
  __syncthreads();
  if (vt < d) {
    TIn* Op = (TIn*)p.O + b * p.os.batch + hd * p.os.head;
#pragma unroll
    for (int r = 0; r < kDQ / 2; ++r) {
      const int row = lg + r * ngroups;
      if (row < kDQ && row < qn) stf(Op + (long long)(q0 + row) * p.os.token + vt, acc[r] * rinv[row]);
    }
  }
}

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return hipSuccess;
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

size_t f32_stage_r_lds(int b2, int d) { return ((size_t)2 * b2 * (d + 1) + (size_t)b2 * (b2 + 1)) * 4; }
size_t f32_stage_l_lds(int b1, int d) {
  return ((size_t)b1 * (d + 1) + (size_t)kCH * (d + 1) + (size_t)b1 * (kCH + 1) + b1 + 2 * kCH) * 4;
}

hipError_t launch_f32_stage_r(const KParams& kp, int dtype, int nbh, bool first, bool last,
                              hipStream_t s) {
  const size_t lds = f32_stage_r_lds(kp.b2, kp.d);
  dim3 grid(kp.ntk * kp.b1, kp.ntq, nbh);
  hipError_t e;
  if (dtype == MRT_F32) {
    if ((e = allow_lds(k_f32_stage_r<float>, lds)) != hipSuccess) return e;
    k_f32_stage_r<float><<<grid, kThreads, lds, s>>>(kp, first, last);
  } else {
    if ((e = allow_lds(k_f32_stage_r<uint16_t>, lds)) != hipSuccess) return e;
    k_f32_stage_r<uint16_t><<<grid, kThreads, lds, s>>>(kp, first, last);
  }
  return hipGetLastError();
}

hipError_t launch_f32_stage_l(const KParams& kp, int dtype, int nbh, bool last, hipStream_t s) {
  const size_t lds = f32_stage_l_lds(kp.b1, kp.d);
  dim3 grid(kp.b2, kp.ntq, nbh);
  hipError_t e;
#define MRT_LAUNCH_L(T, LASTV)                                                     \
  do {                                                                             \
    if ((e = allow_lds(k_f32_stage_l<T, LASTV>, lds)) != hipSuccess) return e;     \
    k_f32_stage_l<T, LASTV><<<grid, kThreads, lds, s>>>(kp);                       \
  } while (0)
  if (dtype == MRT_F32) { if (last) MRT_LAUNCH_L(float, true); else MRT_LAUNCH_L(float, false); }
  else { if (last) MRT_LAUNCH_L(uint16_t, true); else MRT_LAUNCH_L(uint16_t, false); }
#undef MRT_LAUNCH_L
  return hipGetLastError();
}

hipError_t launch_f32_dense(const KParams& kp, int dtype, int nbh, hipStream_t s) {
  const size_t lds = ((size_t)(kDQ + kDK) * (kp.d + 1) + (size_t)kDQ * (kDK + 1) + 2 * kDQ) * 4;
  dim3 grid((kp.Nq + kDQ - 1) / kDQ, nbh);
  if (dtype == MRT_F32) k_f32_dense<float><<<grid, kThreads, lds, s>>>(kp);
  else k_f32_dense<uint16_t><<<grid, kThreads, lds, s>>>(kp);
  return hipGetLastError();
}

}  // namespace mrt
