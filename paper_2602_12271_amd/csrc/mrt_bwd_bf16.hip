// Backward pass on the bf16 matrix unit (bf16 storage, b1 <= 144 for stage L, b2 <= 64 for stage R,
// head_dim 64 or 128): bf16 MFMA operands, fp32 accumulation and fp32 softmax arithmetic, same
// register layouts as the forward kernels (mrt_bf16.hip).  The workspace arrays are typed by TW:
// fp32 when the fp32 forward kernels recomputed the intermediates (one of the two stages runs the
// fp32 kernels of mrt_bwd_f32.hip), bf16 when every stage runs here and the bf16 forward kernels
// did; operands are rounded to bf16 at the latest when they are staged into LDS.
//
// Stage L backward is split in two kernels per (m, j):
//   rows kernel  (lanes own query rows l):  L, dL, delta, dZ;  dQ[l] += scale dZ aL (+ w dA);
//                writes L (or w) and dZ transposed, as bf16 [nk][l], for the second kernel
//   cols kernel  (lanes own key rows nk):   d aL[nk] = scale sum_l dZ[l,nk] Q[l],
//                d cL[nk] = -sum_l dZ[l,nk], d Y[nk] = sum_l L[l,nk] dO[l]
// so that every contraction has its summation index on the K side of an MFMA.  The rows kernel
// holds the key range in LDS when it has at most 96 rows and streams it in segments otherwise.
#include "mrt_internal.hpp"
#include <type_traits>

#include "mrt_bf16_tiles.hpp"

namespace mrt {

namespace {

constexpr int kBRows = 96;     // key rows / query rows held in LDS
constexpr int kBPad = 8;       // row padding of the LDS tiles (as the forward resident kernels)
constexpr int kLP = 96;        // row pitch (elements) of the transposed L / dZ arrays, b1 <= 96
constexpr int kLPWide = 160;   // the same for 96 < b1 <= 144 (ten query tiles, the last one zeros)
constexpr int kBRowsWide = 144;
__host__ __device__ inline int lp_of(int b1) { return b1 <= kBRows ? kLP : kLPWide; }

// fp32 rows -> bf16 LDS tile: row r of the tile comes from src + rowoff(r); rows >= valid are zero.
template <int D, int LD, int ROWS, int NTHR, typename RowFn>
__device__ inline void stage_rows_f32(u16* dst, const float* src, RowFn rowoff, int valid, int tid) {
  constexpr int CPR = D / 8, TOTAL = ROWS * CPR, N = (TOTAL + NTHR - 1) / NTHR;
  f32x4 lo[N], hi[N];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    int idx = tid + i * NTHR;
    idx = idx < TOTAL ? idx : TOTAL - 1;
    int r = idx / CPR;
    const int c = idx - r * CPR;
    r = r < valid ? r : valid - 1;
    const float* p = src + rowoff(r) + 8 * c;
    lo[i] = *(const f32x4*)p;
    hi[i] = *(const f32x4*)(p + 4);
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int idx = tid + i * NTHR;
    const int r = idx / CPR, c = idx - r * CPR;
    if (idx < TOTAL) {
      const bf16x8 v = pack8(lo[i], hi[i]);
      *(uint4*)(dst + r * LD + 8 * c) = r < valid ? __builtin_bit_cast(uint4, v) : uint4{0u, 0u, 0u, 0u};
    }
  }
}

// Rows of a workspace array into a bf16 LDS tile, whichever type the array is stored in.
// The same copy split into its two halves (see RowRegs): load() issues every global load,
// store() converts and writes the tile.
template <int D, int ROWS, int NTHR>
struct RowRegsF32 {
  static constexpr int CPR = D / 8, TOTAL = ROWS * CPR, N = (TOTAL + NTHR - 1) / NTHR;
  f32x4 lo[N], hi[N];
  int valid;
  template <typename RowFn>
  __device__ inline void load(const float* src, RowFn rowoff, int nvalid, int tid) {
    valid = nvalid;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int idx = tid + i * NTHR;
      idx = idx < TOTAL ? idx : TOTAL - 1;
      int r = idx / CPR;
      const int c = idx - r * CPR;
      r = r < nvalid ? r : nvalid - 1;
      const float* p = src + rowoff(r) + 8 * c;
      lo[i] = *(const f32x4*)p;
      hi[i] = *(const f32x4*)(p + 4);
    }
  }
  template <int LD>
  __device__ inline void store(u16* dst, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int idx = tid + i * NTHR;
      const int r = idx / CPR, c = idx - r * CPR;
      if (idx < TOTAL) {
        const bf16x8 v = pack8(lo[i], hi[i]);
        *(uint4*)(dst + r * LD + 8 * c) = r < valid ? __builtin_bit_cast(uint4, v) : uint4{0u, 0u, 0u, 0u};
      }
    }
  }
};
template <int D, int LD, int ROWS, int NTHR, typename RowFn>
__device__ inline void stage_ws(u16* dst, const float* src, RowFn rowoff, int valid, int tid) {
  stage_rows_f32<D, LD, ROWS, NTHR>(dst, src, rowoff, valid, tid);
}
template <int D, int LD, int ROWS, int NTHR, typename RowFn>
__device__ inline void stage_ws(u16* dst, const u16* src, RowFn rowoff, int valid, int tid) {
  stage_rows_batched<D, LD, ROWS, NTHR>(dst, src, rowoff, valid, tid);
}
__device__ inline float ldw(const float* p) { return *p; }
__device__ inline float ldw(const u16* p) { return __uint_as_float((uint32_t)(*p) << 16); }
// Eight consecutive workspace values (16-byte aligned for bf16, 32 for fp32) as two float vectors.
__device__ inline void ldw8(const float* p, f32x4& lo, f32x4& hi) {
  lo = *(const f32x4*)p;
  hi = *(const f32x4*)(p + 4);
}
__device__ inline void ldw8(const u16* p, f32x4& lo, f32x4& hi) {
  const uint4 v = *(const uint4*)p;
  lo = f32x4{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
             __uint_as_float(v.y & 0xffff0000u)};
  hi = f32x4{__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u), __uint_as_float(v.w << 16),
             __uint_as_float(v.w & 0xffff0000u)};
}

// Bias of keys key0 .. key0 + 3 of a lane whose query row sees the keys below lim (regular Monarch
// under the chunk-causal mask: a hidden key gets -inf like a key beyond the range).
__device__ inline f32x4 mask_bias(f32x4 bi, int key0, int lim) {
#pragma unroll
  for (int r = 0; r < 4; ++r) bi[r] = key0 + r < lim ? bi[r] : -INFINITY;
  return bi;
}

// S^T tiles of one query tile against NTK resident row tiles: out[kt][r] = rows[16kt + 4g + r] . q
template <int D, int NTK, int LD>
__device__ inline void rows_dot(const u16* rows, const bf16x8 (&qv)[D / 32], f32x4 (&out)[NTK], int lane) {
  constexpr int KS1 = D / 32;
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int kt = 0; kt < NTK; ++kt) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks)
      acc = mfma(ld_lds_16B(rows + (16 * kt + c) * LD + 32 * ks + 8 * g), qv[ks], acc);
    out[kt] = acc;
    if (kt % 2 == 1) __builtin_amdgcn_sched_barrier(0);
  }
}

// The same with the LDS reads of the next pair of row tiles issued ahead of the current pair's
// MFMAs (two sets of operand registers).  For kernels that run one wave per SIMD: there nothing else
// hides the latency of an LDS read, and the compiler's own schedule waits for every read right
// before the MFMA that uses it.
template <int D, int NTK, int LD>
__device__ inline void rows_dot_ahead(const u16* rows, const bf16x8 (&qv)[D / 32], f32x4 (&out)[NTK], int lane) {
  constexpr int KS1 = D / 32, NP = (NTK + 1) / 2;
  const int g = lane >> 4, c = lane & 15;
  bf16x8 a[2][2][KS1];
  auto fetch = [&](int kp, bf16x8 (&dst)[2][KS1]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
      if (2 * kp + t < NTK) {
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) dst[t][ks] = ld_lds_16B(rows + (16 * (2 * kp + t) + c) * LD + 32 * ks + 8 * g);
      }
  };
#pragma unroll
  for (int kt = 0; kt < NTK; ++kt) out[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
  fetch(0, a[0]);
#pragma unroll
  for (int kp = 0; kp < NP; ++kp) {
    if (kp + 1 < NP) fetch(kp + 1, a[(kp + 1) & 1]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        if (2 * kp + t < NTK) out[2 * kp + t] = mfma(a[kp & 1][t][ks], qv[ks], out[2 * kp + t]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Second-product step with the contraction slots in natural order (slot (g, e) <-> row 8g + e of
// the 32-row step), for B operands that come from memory rather than from accumulator registers.
template <int D, int NB, int LD>
__device__ inline void pv_step_nat(const u16* vals, const bf16x8 (&pb)[NB], int nb,
                                   f32x4 (&acc)[NB][D / 16], int lane) {
  constexpr int NVT = D / 16, HALF = NVT / 2;
  const int g = lane >> 4, s = lane & 15, e = s >> 2, q = s & 3;
  const u16* base = vals + (8 * g + e) * LD + 8 * q;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    s16x4 lo[HALF], hi[HALF];
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const int vt = h * HALF + i;
      const u16* p0 = base + 32 * (vt >> 1) + 4 * (vt & 1);
      lo[i] = ld_lds_tr(p0);
      hi[i] = ld_lds_tr(p0 + 4 * LD);
    }
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const bf16x8 av =
          __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo[i], hi[i], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
      for (int b = 0; b < NB; ++b)
        if (b < nb) acc[b][h * HALF + i] = mfma(av, pb[b], acc[b][h * HALF + i]);
    }
  }
}

// A lane's D/16 accumulator tiles as fp32: 8 consecutive features at 32q + 8g per pair of tiles.
// The same rows with non-temporal stores: gradients that no later kernel of the call reads or adds
// to (they would only displace the workspace arrays from the caches).
template <int D>
__device__ inline void store_rows_f32_nt(float* row, const f32x4* acc, float mul, int g) {
#pragma unroll
  for (int q = 0; q < D / 32; ++q) {
    f32x4* p = (f32x4*)(row + 32 * q + 8 * g);
    __builtin_nontemporal_store(acc[2 * q] * mul, p);
    __builtin_nontemporal_store(acc[2 * q + 1] * mul, p + 1);
  }
}
template <int D>
__device__ inline void store_rows_f32(float* row, const f32x4* acc, float mul, int g, bool add) {
#pragma unroll
  for (int q = 0; q < D / 32; ++q) {
    f32x4* p = (f32x4*)(row + 32 * q + 8 * g);
    f32x4 a = acc[2 * q] * mul, b = acc[2 * q + 1] * mul;
    if (add) { a += p[0]; b += p[1]; }
    p[0] = a;
    p[1] = b;
  }
}

// A lane's row of D/16 accumulator tiles into a workspace array of either type (overwriting).
template <int D>
__device__ inline void store_ws_row(float* row, const f32x4* acc, float mul, int g) {
  store_rows_f32<D>(row, acc, mul, g, false);
}
template <int D>
__device__ inline void store_ws_row(u16* row, const f32x4* acc, float mul, int g) {
  store_rows<D>(row, acc, mul, g);
}

// Transposed store of one accumulator tile: lane (c, g) holds v[r] for query row l = l16 + c and
// keys nk0 + 4g + r.  The four lanes of a quad (four consecutive query rows) exchange their values
// (two DPP steps on packed bf16 pairs) so that lane c ends up with key nk0 + 4g + (c mod 4) for
// the quad's four rows, and stores them as one 8-byte piece of row nk of the [nk][l] array:
// four store instructions per tile instead of sixteen 2-byte ones.
__device__ inline void store_tile_transposed(u16* arr, int pitch, int nk0, int NK, int l16, f32x4 v, int c, int g) {
  const uint32_t P0 = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
  const uint32_t P1 = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
  const uint32_t X0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)P0, 0xB1, 0xf, 0xf, true);   // lane ^ 1
  const uint32_t X1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)P1, 0xB1, 0xf, 0xf, true);
  const bool odd = c & 1, up = c & 2;
  // keys (c mod 2) and 2 + (c mod 2), rows of the lane pair
  const uint32_t A = odd ? ((X0 >> 16) | (P0 & 0xffff0000u)) : ((P0 & 0xffffu) | (X0 << 16));
  const uint32_t B = odd ? ((X1 >> 16) | (P1 & 0xffff0000u)) : ((P1 & 0xffffu) | (X1 << 16));
  const uint32_t recv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(up ? A : B), 0x4E, 0xf, 0xf, true);   // lane ^ 2
  const uint2 out = up ? uint2{recv, B} : uint2{A, recv};
  const int nk = nk0 + 4 * g + (c & 3);
  if (nk < NK) *(uint2*)(arr + (size_t)nk * pitch + l16 + (c & ~3)) = out;
}

// The gradient arrays that only travel between the kernels of the sweep (d alpha_L, dY, and d abar
// of the iterations t >= 2) are stored in the type TW of the forward intermediates: as bf16 they
// hold exactly the values the consuming kernel would round its matrix operands to anyway.
// ---------------------------------------------------------------------------------------
// stage L backward, rows kernel, one workgroup per (m, j)
// ---------------------------------------------------------------------------------------
// TW: storage type of the forward intermediates alpha_L, Y and abar in the workspace (fp32 when
// the fp32 kernels recomputed them, bf16 when the bf16 forward kernels did).
template <int D, int NTK, bool LAST, typename TW>
__global__ __launch_bounds__(256, 3) void k_bwdm_l_rows(BwdParams bp, u16* Pw, u16* Zw) {
  const KParams& p = bp.k;
  constexpr int LD = D + kBPad, KS1 = D / 32, NVT = D / 16, KS2 = (NTK + 1) / 2, ROWS = 32 * KS2;
  __shared__ __attribute__((aligned(16))) u16 Ks[ROWS * LD];    // alpha_L rows
  __shared__ __attribute__((aligned(16))) u16 Vs[ROWS * LD];    // Y rows (LAST) or d abar rows
  __shared__ __attribute__((aligned(16))) float bias[ROWS];     // -c_L log2(e), -inf beyond NK
  __shared__ __attribute__((aligned(16))) float tcs[ROWS];      // d abar . abar                  (not LAST)
  __shared__ __attribute__((aligned(16))) float cms[ROWS];      // max_l log2 L[l, nk]            (not LAST)
  __shared__ __attribute__((aligned(16))) float cis[ROWS];      // 1 / sum_l 2^(log2 L - max)     (not LAST)

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2, d = D;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;   // <= 16 * NTK
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;
  const int nlt = (b1 + 15) >> 4;

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const TW* aLp = (const TW*)p.aL + row0 * d;
  const TW* Yp = (const TW*)p.Y + row0 * d;
  const float* cLp = p.cL + row0;
  // rows (nk, j) of the [m][nk][j][d] arrays
  const size_t arow0 = ((size_t)bhl * p.ntq + ml) * NKtot * b2;
  auto arow = [&](int nk) { return (long long)((arow0 + (size_t)nk * b2 + j) * d); };
  const long long qcol = axis_offset(p.cmap, bq * b2 + j);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qcol * p.qs.token;
  const u16* dOp = (const u16*)bp.dO + b * p.os.batch + hd * p.os.head + qcol * p.os.token;
  const TokRows qrow = tile_rows(p, a, p.qs.token), orow = tile_rows(p, a, p.os.token);

  stage_ws<D, LD, ROWS, 256>(Ks, aLp, PlainRows{D}, NK, tid);
  if (LAST) {
    stage_ws<D, LD, ROWS, 256>(Vs, Yp, PlainRows{D}, NK, tid);
  } else {
    // d abar rows (fp32) into LDS as bf16; d abar . abar is formed on the way: the D/8 consecutive
    // lanes that share a row hold 8 features each
    constexpr int CPR = D / 8, TOTAL = ROWS * CPR, NI = (TOTAL + 255) / 256;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int idx = tid + i * 256;
      const bool in = idx < TOTAL;
      const int r = (in ? idx : TOTAL - 1) / CPR, ch = idx % CPR;
      const bool ok = in && r < NK;
      const size_t at = (size_t)arow(ok ? r : 0) + 8 * ch;
      f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = lo;
      float t = 0.f;
      if (ok) {
        ldw8((const TW*)bp.dA + at, lo, hi);
        f32x4 alo, ahi;
        ldw8((const TW*)bp.Anext + at, alo, ahi);
#pragma unroll
        for (int e = 0; e < 4; ++e) t = fmaf(lo[e], alo[e], fmaf(hi[e], ahi[e], t));
      }
      t = CPR == 16 ? row16_sum(t) : row8_sum(t);
      if (in) {
        *(uint4*)(Vs + r * LD + 8 * ch) = __builtin_bit_cast(uint4, pack8(lo, hi));
        if (ch == 0) tcs[r] = t;
      }
    }
  }
  for (int i = tid; i < ROWS; i += 256) {
    bias[i] = i < NK ? -cLp[i] * kLog2e : -INFINITY;
    if (!LAST) {
      const size_t at = arow0 + (size_t)(i < NK ? i : 0) * b2 + j;
      cms[i] = i < NK ? bp.cmx[at] * kLog2e : 0.f;
      cis[i] = i < NK ? bp.cinv[at] : 0.f;
    }
  }
  __syncthreads();

  const float scale2 = p.scale * kLog2e;
  float* dQp = bp.dQ + (size_t)bh * p.Nq * d;
  u16* Pt = Pw + row0 * kLP;
  u16* Zt = Zw + row0 * kLP;
  // the cols kernel reads query rows in steps of 32: an odd tile count leaves one tile of zeros
  for (int lt = wave; lt < 2 * ((nlt + 1) / 2); lt += 4) {
    const int l = 16 * lt + c;
    if (lt >= nlt) {
      for (int nk = g; nk < NK; nk += 4) {
        if (LAST) Pt[(size_t)nk * kLP + l] = 0;
        Zt[(size_t)nk * kLP + l] = 0;
      }
      continue;
    }
    const int lc = l < b1 ? l : b1 - 1;
    bf16x8 qv[KS1], xv[KS1];
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) {
      qv[ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
      xv[ks] = LAST ? ld_global_16B(dOp + orow(lc) + 32 * ks + 8 * g) : qv[ks];
    }
    // regular Monarch under the chunk-causal mask: this lane's query row sees the keys below klim
    const int klim = p.rl > 0 ? visible_key_rows(p, lc) : 0x7fffffff;
    f32x4 s[NTK], dl[NTK], z[NTK];
    rows_dot<D, NTK, LD>(Ks, qv, s, lane);
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) z[kt] = s[kt];              // raw logits, for log2 L below
    __builtin_amdgcn_sched_barrier(0);
    rows_dot<D, NTK, LD>(Vs, xv, dl, lane);
    __builtin_amdgcn_sched_barrier(0);
    // L = softmax over nk (exact: the whole key range is resident)
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) {
      const f32x4 bi = mask_bias(*(const f32x4*)(bias + 16 * kt + 4 * g), 16 * kt + 4 * g, klim);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[kt][r] = fmaf(s[kt][r], scale2, bi[r]);
        mx = fmaxf(mx, s[kt][r]);
      }
    }
    mx = xmax(mx);
    float sm = 0.f;
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[kt][r] = exp2_fast(s[kt][r] - mx);
        sm += s[kt][r];
      }
    const float inv = 1.0f / xsum(sm);
    const float lse2 = mx + log2_fast(xsum(sm));              // base-2 log-sum-exp of the row
    const bool live = l < b1;                                  // rows beyond b1 contribute nothing
    // s <- L; wq <- L (LAST) or w = L / sum_l L, formed as 2^(log2 L - column max) / column sum;
    // dl <- L dL (LAST) or w u (else)
    float delta = 0.f;
    f32x4 wq[NTK];
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) {
      const f32x4 bi = mask_bias(*(const f32x4*)(bias + 16 * kt + 4 * g), 16 * kt + 4 * g, klim);
      f32x4 cm = {0.f, 0.f, 0.f, 0.f}, ci = {0.f, 0.f, 0.f, 0.f}, tc = {0.f, 0.f, 0.f, 0.f};
      if (!LAST) {
        cm = *(const f32x4*)(cms + 16 * kt + 4 * g);
        ci = *(const f32x4*)(cis + 16 * kt + 4 * g);
        tc = *(const f32x4*)(tcs + 16 * kt + 4 * g);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float logl = fmaf(z[kt][r], scale2, bi[r]) - lse2;           // log2 L, -inf beyond NK
        const float L = live ? s[kt][r] * inv : 0.f;
        s[kt][r] = L;
        const float w = LAST ? L : (live ? exp2_fast(logl - cm[r]) * ci[r] : 0.f);
        wq[kt][r] = w;
        dl[kt][r] = w * (dl[kt][r] - tc[r]);
        delta += dl[kt][r];
      }
    }
    delta = xsum(delta);
    // dZ, and the transposed copies for the cols kernel
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) dl[kt][r] = dl[kt][r] - s[kt][r] * delta;
      if (LAST) store_tile_transposed(Pt, kLP, 16 * kt, NK, 16 * lt, wq[kt], c, g);   // only dY, at t = T, is formed from it
      store_tile_transposed(Zt, kLP, 16 * kt, NK, 16 * lt, dl[kt], c, g);
    }
    __builtin_amdgcn_sched_barrier(0);
    // dQ[l] = scale sum_nk dZ[l,nk] aL[nk] (+ sum_nk w[l,nk] dA[nk])
    f32x4 o[NVT];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) o[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      const bool has = 2 * st + 1 < NTK;
      const bf16x8 pz = pack8(dl[2 * st] * p.scale, has ? dl[has ? 2 * st + 1 : 0] * p.scale : zero);
      pv_step<D, LD>(Ks + 32 * st * LD, pz, o, lane);
      __builtin_amdgcn_sched_barrier(0);
      if (!LAST) {
        const bf16x8 pw = pack8(wq[2 * st], has ? wq[has ? 2 * st + 1 : 0] : zero);
        pv_step<D, LD>(Vs + 32 * st * LD, pw, o, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (l < b1) store_rows_f32<D>(dQp + (row_offset(p, a, l) + qcol) * d, o, 1.0f, g, bp.accumulate != 0);
  }
}

// ---------------------------------------------------------------------------------------
// stage L backward, rows kernel for key ranges that do not fit LDS: one workgroup per (m, j),
// wave w owns query tile w, the key range is streamed in segments of 64 rows, twice.  The first
// sweep forms the row statistics online (running maximum and sum of the logits for the
// log-sum-exp, and delta[l] = sum_c (L dL)[l, c] against a running maximum of its own, so that the
// column shift of the weights never meets a positive exponent); the second sweep forms L (or w),
// dZ and the dQ products with them.
// ---------------------------------------------------------------------------------------
constexpr int kSegTiles = 4, kSeg = 16 * kSegTiles;
// Segments staged per barrier pair: two segments' loads are in flight together and the exposed
// load latency and the two barriers are paid once per 128 key rows (70 KB of LDS per workgroup,
// two workgroups per compute unit).
// (three or four segments at a time, which the ten-wave variant's LDS would allow, measured no
// faster and slower)
constexpr int kStageSegs = 2, kStage = kSeg * kStageSegs;

// NW waves: 6 for b1 <= 96, 10 for b1 <= 144 (the pitch of the transposed arrays follows).
template <int D, bool LAST, typename TW, int NW>
__global__ __launch_bounds__(64 * NW, 3) void k_bwdm_l_rows_stream(BwdParams bp, u16* Pw, u16* Zw) {
  const KParams& p = bp.k;
  constexpr int LD = D + kBPad, KS1 = D / 32, NVT = D / 16, NTK = kSegTiles, KS2 = NTK / 2;
  constexpr int CPR = D / 8, TOTAL = kStage * CPR, NTMAX = 64 * NW, NI = (TOTAL + NTMAX - 1) / NTMAX;
  constexpr int LP = NW <= 6 ? kLP : kLPWide;
  __shared__ __attribute__((aligned(16))) u16 Ks[kStage * LD];    // alpha_L rows of the segment
  __shared__ __attribute__((aligned(16))) u16 Vs[kStage * LD];    // Y rows (LAST) or d abar rows
  __shared__ __attribute__((aligned(16))) float bias[kStage];     // -c_L log2(e), -inf beyond NK
  __shared__ __attribute__((aligned(16))) float tcs[kStage];      // d abar . abar                  (not LAST)
  __shared__ __attribute__((aligned(16))) float cms[kStage];      // max_l log2 L[l, nk]            (not LAST)
  __shared__ __attribute__((aligned(16))) float cis[kStage];      // 1 / sum_l 2^(log2 L - max)     (not LAST)

  constexpr int nthr = NTMAX;                  // launched with exactly this many threads
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2, d = D;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;
  const int nlt = (b1 + 15) >> 4;

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const TW* aLp = (const TW*)p.aL + row0 * d;
  const TW* Yp = (const TW*)p.Y + row0 * d;
  const float* cLp = p.cL + row0;
  // rows (nk, j) of the [m][nk][j][d] arrays
  const size_t arow0 = ((size_t)bhl * p.ntq + ml) * NKtot * b2;
  const long long qcol = axis_offset(p.cmap, bq * b2 + j);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qcol * p.qs.token;
  const u16* dOp = (const u16*)bp.dO + b * p.os.batch + hd * p.os.head + qcol * p.os.token;
  const TokRows qrow = tile_rows(p, a, p.qs.token), orow = tile_rows(p, a, p.os.token);

  // one segment of the key side into LDS; d abar . abar is formed on the way from the fp32 rows
  auto stage = [&](int k0) {
    const int valid = NK - k0 < kStage ? NK - k0 : kStage;
    stage_ws<D, LD, kStage, NTMAX>(Ks, aLp + (size_t)k0 * d, PlainRows{D}, valid, tid);
    if (LAST) {
      stage_ws<D, LD, kStage, NTMAX>(Vs, Yp + (size_t)k0 * d, PlainRows{D}, valid, tid);
    } else {
      // D/8 consecutive lanes share a row: 8 features each
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int idx = tid + i * nthr;
        const bool in = idx < TOTAL;
        const int r = (in ? idx : TOTAL - 1) / CPR, ch = idx % CPR;
        const bool ok = in && r < valid;
        const size_t at = (arow0 + (size_t)(k0 + (ok ? r : 0)) * b2 + j) * d + 8 * ch;
        f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = lo;
        float t = 0.f;
        if (ok) {
          ldw8((const TW*)bp.dA + at, lo, hi);
          f32x4 alo, ahi;
          ldw8((const TW*)bp.Anext + at, alo, ahi);
#pragma unroll
          for (int e = 0; e < 4; ++e) t = fmaf(lo[e], alo[e], fmaf(hi[e], ahi[e], t));
        }
        t = CPR == 16 ? row16_sum(t) : row8_sum(t);
        if (in) {
          *(uint4*)(Vs + r * LD + 8 * ch) = __builtin_bit_cast(uint4, pack8(lo, hi));
          if (ch == 0) tcs[r] = t;
        }
      }
    }
    if (tid < kStage) {
      const int nk = k0 + tid;
      const bool ok = nk < NK;
      bias[tid] = ok ? -cLp[nk] * kLog2e : -INFINITY;
      if (!LAST) {
        const size_t at = arow0 + (size_t)(ok ? nk : 0) * b2 + j;
        cms[tid] = ok ? bp.cmx[at] * kLog2e : 0.f;
        cis[tid] = ok ? bp.cinv[at] : 0.f;
      }
    }
  };

  const int lt = wave, l = 16 * lt + c;
  const bool tile_live = lt < nlt;           // an odd tile count leaves one wave that only writes zeros
  const bool live = l < b1;
  const int lc = l < b1 ? l : b1 - 1;
  bf16x8 qv[KS1], xv[KS1];
#pragma unroll
  for (int ks = 0; ks < KS1; ++ks) {
    qv[ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
    xv[ks] = LAST ? ld_global_16B(dOp + orow(lc) + 32 * ks + 8 * g) : qv[ks];
  }
  const float scale2 = p.scale * kLog2e;
  // regular Monarch under the chunk-causal mask: this lane's query row sees the keys below klim
  // (key 0 is visible to every row, so the running maxima are finite after the first segment)
  const int klim = p.rl > 0 ? visible_key_rows(p, lc) : 0x7fffffff;

  // ---- sweep 1: lse2[l] and delta[l]
  float mz = -INFINITY, sz = 0.f;            // running maximum / sum of 2^(z - mz)
  float mw = -INFINITY, dw = 0.f;            // the same for the shifted logits, weighted sum of u
  for (int kb = 0; kb < NK; kb += kStage) {
    __syncthreads();
    stage(kb);
    __syncthreads();
    for (int h = 0; h < kStageSegs && kb + h * kSeg < NK; ++h) {
    const int k0 = kb + h * kSeg;
    const u16* Ksh = Ks + h * kSeg * LD;
    const u16* Vsh = Vs + h * kSeg * LD;
    const float *biash = bias + h * kSeg, *tcsh = tcs + h * kSeg, *cmsh = cms + h * kSeg, *cish = cis + h * kSeg;
    if (!tile_live) continue;
    f32x4 s[NTK], dl[NTK];
    rows_dot<D, NTK, LD>(Ksh, qv, s, lane);
    __builtin_amdgcn_sched_barrier(0);
    rows_dot<D, NTK, LD>(Vsh, xv, dl, lane);
    __builtin_amdgcn_sched_barrier(0);
    float mx = -INFINITY, mxw = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) {
      const f32x4 bi = mask_bias(*(const f32x4*)(biash + 16 * kt + 4 * g), k0 + 16 * kt + 4 * g, klim);
      f32x4 cm = {0.f, 0.f, 0.f, 0.f};
      if (!LAST) cm = *(const f32x4*)(cmsh + 16 * kt + 4 * g);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[kt][r] = fmaf(s[kt][r], scale2, bi[r]);
        mx = fmaxf(mx, s[kt][r]);
        if (!LAST) mxw = fmaxf(mxw, s[kt][r] - cm[r]);
      }
    }
    const float mzn = fmaxf(mz, xmax(mx));
    const float mwn = LAST ? mzn : fmaxf(mw, xmax(mxw));
    float ps = 0.f, pd = 0.f;
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) {
      f32x4 cm = {0.f, 0.f, 0.f, 0.f}, ci = {1.f, 1.f, 1.f, 1.f}, tc = {0.f, 0.f, 0.f, 0.f};
      if (!LAST) {
        cm = *(const f32x4*)(cmsh + 16 * kt + 4 * g);
        ci = *(const f32x4*)(cish + 16 * kt + 4 * g);
        tc = *(const f32x4*)(tcsh + 16 * kt + 4 * g);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float e = exp2_fast(s[kt][r] - mzn);
        ps += e;
        const float ew = LAST ? e : exp2_fast(s[kt][r] - cm[r] - mwn) * ci[r];
        pd = fmaf(ew, dl[kt][r] - tc[r], pd);
      }
    }
    sz = fmaf(sz, exp2_fast(mz - mzn), xsum(ps));
    dw = fmaf(dw, exp2_fast((LAST ? mz : mw) - mwn), xsum(pd));
    mz = mzn;
    mw = mwn;
    }
  }
  const float lse2 = mz + log2_fast(sz);
  const float delta = dw * exp2_fast((LAST ? mz : mw) - lse2);

  // ---- sweep 2: L (or w), dZ, their transposed copies, dQ
  float* dQp = bp.dQ + (size_t)bh * p.Nq * d;
  u16* Pt = Pw + row0 * LP;
  u16* Zt = Zw + row0 * LP;
  f32x4 o[NVT];
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt) o[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int kb = 0; kb < NK; kb += kStage) {
    __syncthreads();
    stage(kb);
    __syncthreads();
    for (int h = 0; h < kStageSegs && kb + h * kSeg < NK; ++h) {
    const int k0 = kb + h * kSeg;
    const u16* Ksh = Ks + h * kSeg * LD;
    const u16* Vsh = Vs + h * kSeg * LD;
    const float *biash = bias + h * kSeg, *tcsh = tcs + h * kSeg, *cmsh = cms + h * kSeg, *cish = cis + h * kSeg;
    if (!tile_live) {
      // the cols kernel reads as many query tiles as its template holds (2, 4, 6, or all ten of
      // the wide pitch): the tiles beyond the last query tile are zeros
      if (lt < (NW <= 6 ? 2 * ((nlt + 1) / 2) : NW))
        for (int nk = k0 + g; nk < NK && nk < k0 + kSeg; nk += 4) {
          if (LAST) Pt[(size_t)nk * LP + l] = 0;
          Zt[(size_t)nk * LP + l] = 0;
        }
      continue;
    }
    f32x4 s[NTK], dl[NTK], wq[NTK];
    rows_dot<D, NTK, LD>(Ksh, qv, s, lane);
    __builtin_amdgcn_sched_barrier(0);
    rows_dot<D, NTK, LD>(Vsh, xv, dl, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) {
      const f32x4 bi = mask_bias(*(const f32x4*)(biash + 16 * kt + 4 * g), k0 + 16 * kt + 4 * g, klim);
      f32x4 cm = {0.f, 0.f, 0.f, 0.f}, ci = {0.f, 0.f, 0.f, 0.f}, tc = {0.f, 0.f, 0.f, 0.f};
      if (!LAST) {
        cm = *(const f32x4*)(cmsh + 16 * kt + 4 * g);
        ci = *(const f32x4*)(cish + 16 * kt + 4 * g);
        tc = *(const f32x4*)(tcsh + 16 * kt + 4 * g);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float logl = fmaf(s[kt][r], scale2, bi[r]) - lse2;           // log2 L, -inf beyond NK
        const float L = live ? exp2_fast(logl) : 0.f;
        const float w = LAST ? L : (live ? exp2_fast(logl - cm[r]) * ci[r] : 0.f);
        const float dz = w * (dl[kt][r] - tc[r]) - L * delta;
        wq[kt][r] = w;
        dl[kt][r] = dz;
        const int nk = k0 + 16 * kt + 4 * g + r;
        if (nk < NK) {
          if (LAST) Pt[(size_t)nk * LP + l] = f2bf(w);       // only dY, at t = T, is formed from it
          Zt[(size_t)nk * LP + l] = f2bf(dz);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // dQ[l] += scale sum_nk dZ[l,nk] aL[nk] (+ sum_nk w[l,nk] dA[nk])
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      const bf16x8 pz = pack8(dl[2 * st] * p.scale, dl[2 * st + 1] * p.scale);
      pv_step<D, LD>(Ksh + 32 * st * LD, pz, o, lane);
      __builtin_amdgcn_sched_barrier(0);
      if (!LAST) {
        const bf16x8 pw = pack8(wq[2 * st], wq[2 * st + 1]);
        pv_step<D, LD>(Vsh + 32 * st * LD, pw, o, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    }
  }
  if (tile_live && live)
    store_rows_f32<D>(dQp + (row_offset(p, a, l) + qcol) * d, o, 1.0f, g, bp.accumulate != 0);
}

// Sum of the products of the eight bf16 pairs of two 16-byte pieces.
__device__ inline float dot8_bf16(uint4 a, uint4 b) {
  const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
  float t = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    t = fmaf(__uint_as_float(aw[e] << 16), __uint_as_float(bw[e] << 16), t);
    t = fmaf(__uint_as_float(aw[e] & 0xffff0000u), __uint_as_float(bw[e] & 0xffff0000u), t);
  }
  return t;
}

// ---------------------------------------------------------------------------------------
// The streamed rows kernel for a bf16 workspace, software-pipelined.  Same two sweeps over the key
// range and the same arithmetic as k_bwdm_l_rows_stream, but the segments of 64 key rows travel
// through a ring of two LDS slots behind one set of registers: while the waves work on segment s
// (slot s mod 2), the global loads of segment s + 1 are in flight; they are written to the other
// slot when the wave is done with s, the loads of s + 2 are issued, and one barrier ends the step.
// The loop body has no branch around a load, so the waits count exactly (the transposed stores of
// a step are never waited for), and a step past the end of the range reloads the last segment into
// the slot nobody reads.  d abar . abar, which the first sweep forms on the way from the two rows,
// is kept for the second sweep in this (m, j)'s row of d c_L, which the cols kernel overwrites
// afterwards, so the second sweep does not read abar again.
//
// NQT query tiles (6 for b1 <= 96, 10 for b1 <= 144).  A workgroup of more than four waves has a
// compute unit to itself (its waves do not spread evenly over the SIMDs, so a second one does not
// fit beside it), and six waves leave half of the unit's wave slots empty: with KSPLIT = 2 every
// query tile is owned by two waves, each taking half of a segment's key tiles, twelve waves in
// all.  The two halves' row statistics are merged after the first sweep and their partial dQ rows
// after the second, through LDS.  (KSPLIT = 2 needs every row to see key 32 of the range, which
// holds unless regular Monarch runs under the chunk-causal mask: the host picks KSPLIT = 1 then.)
// ---------------------------------------------------------------------------------------
template <int D, bool LAST, int NQT, int KSPLIT>
__global__ __launch_bounds__(64 * NQT * KSPLIT, 3) void k_bwdm_l_rows_ring(BwdParams bp, u16* Pw, u16* Zw) {
  const KParams& p = bp.k;
  constexpr int NW = NQT * KSPLIT;
  constexpr int LD = D + kBPad, KS1 = D / 32, NVT = D / 16, NTK = kSegTiles / KSPLIT, KS2 = NTK / 2;
  constexpr int NTHR = 64 * NW, CPR = D / 8, TOTAL = kSeg * CPR;
  constexpr int LP = NQT <= 6 ? kLP : kLPWide;
  static_assert(NTK % 2 == 0 && 4 * kSeg * LD * 2 >= (KSPLIT - 1) * NQT * NVT * 64 * 16, "LDS reuse");
  // per slot: alpha_L rows of a segment (Ks), Y rows (LAST) or d abar rows (Vs)
  __shared__ __attribute__((aligned(16))) u16 ring[4 * kSeg * LD];
  u16 (*Ks)[kSeg * LD] = (u16 (*)[kSeg * LD])ring;
  u16 (*Vs)[kSeg * LD] = (u16 (*)[kSeg * LD])(ring + 2 * kSeg * LD);
  // per slot: -c_L log2(e) (-inf beyond NK) | d abar . abar | max_l log2 L[l, nk] | 1 / sum_l 2^(log2 L - max)
  __shared__ __attribute__((aligned(16))) float side[2][4][kSeg];
  __shared__ __attribute__((aligned(16))) f32x4 halves[KSPLIT][NQT][16];   // row statistics of the key halves
  // kFuse: the column side of the stage (d alpha_L, d c_L, dY: k_bwdm_l_cols otherwise) is formed
  // here, from the segment's dZ (and L) left transposed in LDS instead of in global scratch
  // (ten query tiles: only at t < T, where one transposed array and the Q tile fit beside the ring)
  constexpr bool kFuse = (KSPLIT == 2 && NQT == 6) || (NQT == 10 && KSPLIT == 1 && !LAST);
  constexpr int QROWS = 16 * NQT, LPZ = QROWS + 8, KSC = NQT / 2;
  __shared__ __attribute__((aligned(16))) u16 Qs[kFuse ? QROWS * LD : 8];             // Q[m, :, j, :]
  __shared__ __attribute__((aligned(16))) u16 dOs[kFuse && LAST ? QROWS * LD : 8];    // dO[m, :, j, :]
  // dZ as [nk][l] of a segment: two buffers at t < T (the column side of a step then runs beside the
  // next step's row side), one at t = T, where L needs one too
  __shared__ __attribute__((aligned(16))) u16 Zs[kFuse ? (LAST ? 1 : 2) * kSeg * LPZ : 8];
  __shared__ __attribute__((aligned(16))) u16 Ws[kFuse && LAST ? kSeg * LPZ : 8];

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2, d = D;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const int nseg = (NK + kSeg - 1) / kSeg;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const u16* aLp = (const u16*)p.aL + row0 * d;
  const u16* Yp = (const u16*)p.Y + row0 * d;
  const float* cLp = p.cL + row0;
  float* tcp = bp.dcL + row0;                  // d abar . abar between the sweeps
  // rows (nk, j) of the [m][nk][j][d] arrays
  const size_t arow0 = ((size_t)bhl * p.ntq + ml) * NKtot * b2;
  const long long qcol = axis_offset(p.cmap, bq * b2 + j);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qcol * p.qs.token;
  const u16* dOp = (const u16*)bp.dO + b * p.os.batch + hd * p.os.head + qcol * p.os.token;
  const TokRows qrow = tile_rows(p, a, p.qs.token), orow = tile_rows(p, a, p.os.token);

  if constexpr (kFuse) {
    stage_rows_batched<D, LD, QROWS, NTHR>(Qs, Qp, qrow, b1, tid);
    if (LAST) stage_rows_batched<D, LD, QROWS, NTHR>(dOs, dOp, orow, b1, tid);
  }
  // the register set behind the ring
  RowRegs<D, kSeg, NTHR> rA, rB, rC;
  float sc = 0.f;
  // SWEEP 1 also fetches abar (for d abar . abar); SWEEP 2 reads that product back instead
  auto issue = [&](auto sweep, int seg) {
    constexpr int SWEEP = decltype(sweep)::value;
    const int k0 = kSeg * (seg < nseg ? seg : nseg - 1);
    const int valid = NK - k0 < kSeg ? NK - k0 : kSeg;
    rA.load(aLp + (size_t)k0 * d, PlainRows{D}, valid, tid);
    if (LAST) {
      rB.load(Yp + (size_t)k0 * d, PlainRows{D}, valid, tid);
    } else {
      const size_t at0 = (arow0 + (size_t)k0 * b2 + j) * d;
      rB.load((const u16*)bp.dA + at0, PlainRows{(long long)b2 * D}, valid, tid);
      if (SWEEP == 1) rC.load((const u16*)bp.Anext + at0, PlainRows{(long long)b2 * D}, valid, tid);
    }
    // one side value per thread: wave 0 fetches c_L, and for the earlier iterations wave 1 the
    // column maximum, wave 2 the inverse column sum, wave 3 (second sweep) d abar . abar
    const int r = tid & 63;
    const int nkc = k0 + r < NK ? k0 + r : NK - 1;
    const float* sp = cLp + nkc;
    if (!LAST) {
      const size_t at = arow0 + (size_t)nkc * b2 + j;
      sp = wave == 1 ? bp.cmx + at : wave == 2 ? bp.cinv + at : (wave == 3 && SWEEP == 2) ? tcp + nkc : sp;
    }
    sc = *sp;
  };
  auto commit = [&](auto sweep, int seg, int slot) {
    constexpr int SWEEP = decltype(sweep)::value;
    const int k0 = kSeg * (seg < nseg ? seg : nseg - 1);
    const int valid = NK - k0 < kSeg ? NK - k0 : kSeg;
    rA.template store<LD>(Ks[slot], tid);
    rB.template store<LD>(Vs[slot], tid);
    if (!LAST && SWEEP == 1) {
      // the D/8 consecutive lanes that share a row hold 8 features each
#pragma unroll
      for (int i = 0; i < RowRegs<D, kSeg, NTHR>::N; ++i) {
        const int idx = tid + i * NTHR;
        const int r = idx / CPR, ch = idx - r * CPR;
        float t = dot8_bf16(rB.v[i], rC.v[i]);
        t = CPR == 16 ? row16_sum(t) : row8_sum(t);
        if (idx < TOTAL && ch == 0) {
          side[slot][1][r] = r < valid ? t : 0.f;
          if (r < valid) tcp[k0 + r] = t;
        }
      }
    }
    const int r = tid & 63;
    const bool ok = k0 + r < NK;
    const float v = wave == 0 ? (ok ? -sc * kLog2e : -INFINITY) : wave == 1 ? (ok ? sc * kLog2e : 0.f) : (ok ? sc : 0.f);
    const int which = wave == 0 ? 0 : wave == 1 ? 2 : wave == 2 ? 3 : 1;
    const bool wr = wave == 0 || (!LAST && (wave < 3 || (wave == 3 && SWEEP == 2)));
    if (wr) side[slot][which][r] = v;
  };

  // wave -> query tile lt and key half kh: key tiles NTK kh .. NTK kh + NTK - 1 of every segment
  const int kh = wave / NQT, lt = wave - kh * NQT, l = 16 * lt + c;
  const int koff = 16 * NTK * kh;
  const bool live = l < b1;                  // a query tile beyond the last one, or its ragged end: zeros
  const int lc = l < b1 ? l : b1 - 1;
  bf16x8 qv[KS1], xv[KS1];
#pragma unroll
  for (int ks = 0; ks < KS1; ++ks) {
    qv[ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
    xv[ks] = LAST ? ld_global_16B(dOp + orow(lc) + 32 * ks + 8 * g) : qv[ks];
  }
  const float scale2 = p.scale * kLog2e;
  // regular Monarch under the chunk-causal mask: this lane's query row sees the keys below klim
  // (key 0 is visible to every row, so the running maxima are finite after the first segment)
  const int klim = p.rl > 0 ? visible_key_rows(p, lc) : 0x7fffffff;

  // ---- sweep 1: lse2[l] and delta[l]
  float mz = -INFINITY, sz = 0.f;            // running maximum / sum of 2^(z - mz)
  float mw = -INFINITY, dw = 0.f;            // the same for the shifted logits, weighted sum of u
  // t = T after a forward call that left its row statistics: lse2 is there, and delta[l] =
  // sum_nk L[l, nk] (dO[l] . Y[nk]) = dO[l] . O[l], so the first sweep is not needed
  const bool given = LAST && bp.lse != nullptr;
  if (!given) {
    const std::integral_constant<int, 1> sw;
    issue(sw, 0);
    commit(sw, 0, 0);
    issue(sw, 1);
    __syncthreads();
    for (int sg = 0; sg < nseg; ++sg) {
      const int slot = sg & 1, k0 = kSeg * sg + koff;
      const u16* Ksh = Ks[slot] + koff * LD;
      const u16* Vsh = Vs[slot] + koff * LD;
      const float *biash = side[slot][0] + koff, *tcsh = side[slot][1] + koff, *cmsh = side[slot][2] + koff,
                  *cish = side[slot][3] + koff;
      f32x4 s[NTK], dl[NTK];
      rows_dot<D, NTK, LD>(Ksh, qv, s, lane);
      __builtin_amdgcn_sched_barrier(0);
      rows_dot<D, NTK, LD>(Vsh, xv, dl, lane);
      __builtin_amdgcn_sched_barrier(0);
      float mx = -INFINITY, mxw = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < NTK; ++kt) {
        const f32x4 bi = mask_bias(*(const f32x4*)(biash + 16 * kt + 4 * g), k0 + 16 * kt + 4 * g, klim);
        f32x4 cm = {0.f, 0.f, 0.f, 0.f};
        if (!LAST) cm = *(const f32x4*)(cmsh + 16 * kt + 4 * g);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          s[kt][r] = fmaf(s[kt][r], scale2, bi[r]);
          mx = fmaxf(mx, s[kt][r]);
          if (!LAST) mxw = fmaxf(mxw, s[kt][r] - cm[r]);
        }
      }
      const float mzn = fmaxf(mz, xmax(mx));
      const float mwn = LAST ? mzn : fmaxf(mw, xmax(mxw));
      // a wave whose key half has been empty so far (a visible range of fewer than 33 keys under the
      // mask) still has -inf maxima: its exponents are taken against 0 and come out as zeros
      const float mzs = mzn == -INFINITY ? 0.f : mzn, mws = mwn == -INFINITY ? 0.f : mwn;
      float ps = 0.f, pd = 0.f;
#pragma unroll
      for (int kt = 0; kt < NTK; ++kt) {
        f32x4 cm = {0.f, 0.f, 0.f, 0.f}, ci = {1.f, 1.f, 1.f, 1.f}, tc = {0.f, 0.f, 0.f, 0.f};
        if (!LAST) {
          cm = *(const f32x4*)(cmsh + 16 * kt + 4 * g);
          ci = *(const f32x4*)(cish + 16 * kt + 4 * g);
          tc = *(const f32x4*)(tcsh + 16 * kt + 4 * g);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float e = exp2_fast(s[kt][r] - mzs);
          ps += e;
          const float ew = LAST ? e : exp2_fast(s[kt][r] - cm[r] - mws) * ci[r];
          pd = fmaf(ew, dl[kt][r] - tc[r], pd);
        }
      }
      sz = fmaf(sz, exp2_fast(mz - mzs), xsum(ps));
      dw = fmaf(dw, exp2_fast((LAST ? mz : mw) - mws), xsum(pd));
      mz = mzn;
      mw = mwn;
      commit(sw, sg + 1, slot ^ 1);
      issue(sw, sg + 2);
      __syncthreads();
    }
  }
  if (KSPLIT > 1 && !given) {
    // the halves' statistics, merged in the same order by every wave of a tile
    if (g == 0) halves[kh][lt][c] = f32x4{mz, sz, mw, dw};
    __syncthreads();
    f32x4 h = halves[0][lt][c];
    mz = h[0]; sz = h[1]; mw = h[2]; dw = h[3];
#pragma unroll
    for (int q = 1; q < KSPLIT; ++q) {
      h = halves[q][lt][c];
      const float mzn = fmaxf(mz, h[0]), mwn = fmaxf(mw, h[2]);
      sz = fmaf(sz, exp2_fast(mz - mzn), h[1] * exp2_fast(h[0] - mzn));
      dw = fmaf(dw, exp2_fast((LAST ? mz : mw) - (LAST ? mzn : mwn)),
                h[3] * exp2_fast((LAST ? h[0] : h[2]) - (LAST ? mzn : mwn)));
      mz = mzn;
      mw = mwn;
    }
  }
  float lse2 = mz + log2_fast(sz);
  float delta = dw * exp2_fast((LAST ? mz : mw) - lse2);
  if (given) {
    const size_t qr = (((size_t)bhl * p.ntq + ml) * b2 + j) * b1 + lc;
    lse2 = bp.lse[qr];
    const float* orow32 = bp.o32 + qr * D;
    float t = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) {
      const f32x4 o0 = *(const f32x4*)(orow32 + 32 * ks + 8 * g), o1 = *(const f32x4*)(orow32 + 32 * ks + 8 * g + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        t = fmaf((float)xv[ks][e], o0[e], t);
        t = fmaf((float)xv[ks][e + 4], o1[e], t);
      }
    }
    delta = xsum(t);
  }

  // ---- sweep 2: L (or w), dZ, their transposed copies, dQ
  float* dQp = bp.dQ + (size_t)bh * p.Nq * d;
  u16* Pt = Pw + row0 * LP;
  u16* Zt = Zw + row0 * LP;
  f32x4 o[NVT];
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt) o[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  {
    const std::integral_constant<int, 2> sw;
    issue(sw, 0);
    commit(sw, 0, 0);
    issue(sw, 1);
    __syncthreads();
    for (int sg = 0; sg < nseg; ++sg) {
      const int slot = sg & 1, k0 = kSeg * sg + koff;
      const u16* Ksh = Ks[slot] + koff * LD;
      const u16* Vsh = Vs[slot] + koff * LD;
      const float *biash = side[slot][0] + koff, *tcsh = side[slot][1] + koff, *cmsh = side[slot][2] + koff,
                  *cish = side[slot][3] + koff;
      f32x4 s[NTK], dl[NTK], wq[NTK];
      rows_dot<D, NTK, LD>(Ksh, qv, s, lane);
      __builtin_amdgcn_sched_barrier(0);
      rows_dot<D, NTK, LD>(Vsh, xv, dl, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kt = 0; kt < NTK; ++kt) {
        const f32x4 bi = mask_bias(*(const f32x4*)(biash + 16 * kt + 4 * g), k0 + 16 * kt + 4 * g, klim);
        f32x4 cm = {0.f, 0.f, 0.f, 0.f}, ci = {0.f, 0.f, 0.f, 0.f}, tc = {0.f, 0.f, 0.f, 0.f};
        if (!LAST) {
          cm = *(const f32x4*)(cmsh + 16 * kt + 4 * g);
          ci = *(const f32x4*)(cish + 16 * kt + 4 * g);
          tc = *(const f32x4*)(tcsh + 16 * kt + 4 * g);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float logl = fmaf(s[kt][r], scale2, bi[r]) - lse2;           // log2 L, -inf beyond NK
          const float L = live ? exp2_fast(logl) : 0.f;
          const float w = LAST ? L : (live ? exp2_fast(logl - cm[r]) * ci[r] : 0.f);
          const float dz = w * (dl[kt][r] - tc[r]) - L * delta;
          wq[kt][r] = w;
          dl[kt][r] = dz;
          if constexpr (kFuse) {
            const int at = (koff + 16 * kt + 4 * g + r) * LPZ + l;
            Zs[(LAST ? 0 : (sg & 1) * kSeg * LPZ) + at] = f2bf(dz);
            if (LAST) Ws[at] = f2bf(w);
          }
        }
        if constexpr (!kFuse) {
          if (LAST) store_tile_transposed(Pt, LP, k0 + 16 * kt, NK, 16 * lt, wq[kt], c, g);   // only dY is formed from it
          store_tile_transposed(Zt, LP, k0 + 16 * kt, NK, 16 * lt, dl[kt], c, g);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // dQ[l] += scale sum_nk dZ[l,nk] aL[nk] (+ sum_nk w[l,nk] dA[nk])
#pragma unroll
      for (int st = 0; st < KS2; ++st) {
        const bf16x8 pz = pack8(dl[2 * st] * p.scale, dl[2 * st + 1] * p.scale);
        pv_step<D, LD>(Ksh + 32 * st * LD, pz, o, lane);
        __builtin_amdgcn_sched_barrier(0);
        if (!LAST) {
          const bf16x8 pw = pack8(wq[2 * st], wq[2 * st + 1]);
          pv_step<D, LD>(Vsh + 32 * st * LD, pw, o, lane);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      commit(sw, sg + 1, slot ^ 1);
      issue(sw, sg + 2);
      __syncthreads();
      if constexpr (kFuse) {
        // column side of the segment: d alpha_L[nk] = scale sum_l dZ[l, nk] Q[l], d c_L[nk] =
        // -sum_l dZ[l, nk], and at t = T dY[nk] = sum_l L[l, nk] dO[l]; one 16-row nk tile per wave,
        // the duty moving on by four waves every step
        const int duty = (wave + NW - (4 * sg) % NW) % NW;
        if (duty < (LAST ? 8 : 4)) {
          const bool second = duty >= 4;                 // dY
          const int t = duty & 3, nk = kSeg * sg + 16 * t + c;
          const u16* src = (second ? Ws : Zs + (LAST ? 0 : (sg & 1) * kSeg * LPZ)) + (16 * t + c) * LPZ;
          bf16x8 zb[KSC];
          float zsum = 0.f;
#pragma unroll
          for (int st = 0; st < KSC; ++st) {
            zb[st] = ld_lds_16B(src + 32 * st + 8 * g);
#pragma unroll
            for (int e = 0; e < 8; ++e) zsum += (float)zb[st][e];
          }
          zsum = xsum(zsum);
          if (!second && g == 0 && nk < NK) bp.dcL[row0 + nk] = -zsum;
          f32x4 oc[1][NVT];
#pragma unroll
          for (int vt = 0; vt < NVT; ++vt) oc[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
          const u16* tile = second ? dOs : Qs;
#pragma unroll
          for (int st = 0; st < KSC; ++st) {
            const bf16x8 one[1] = {zb[st]};
            pv_step_nat<D, 1, LD>(tile + 32 * st * LD, one, 1, oc, lane);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (nk < NK) {
            if (second) store_ws_row<D>((u16*)bp.dY + (row0 + nk) * d, oc[0], 1.0f, g);
            else store_ws_row<D>((u16*)bp.daL + (row0 + nk) * d, oc[0], p.scale, g);
          }
        }
        if (LAST) __syncthreads();        // one buffer: the next step's row side writes it again
      }
    }
  }
  if constexpr (KSPLIT > 1) {
    // partial dQ rows of the upper key halves, through the ring's LDS (no longer in use)
    f32x4* part = (f32x4*)ring;
    if (kh > 0) {
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) part[(((kh - 1) * NQT + lt) * NVT + vt) * 64 + lane] = o[vt];
    }
    __syncthreads();
    if (kh > 0) return;
#pragma unroll
    for (int q = 1; q < KSPLIT; ++q)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) o[vt] += part[(((q - 1) * NQT + lt) * NVT + vt) * 64 + lane];
  }
  if (live) store_rows_f32<D>(dQp + (row_offset(p, a, l) + qcol) * d, o, 1.0f, g, bp.accumulate != 0);
}

// ---------------------------------------------------------------------------------------
// stage L backward, cols kernel, one workgroup per (m, j)
// ---------------------------------------------------------------------------------------
template <int D, int NLT, bool LAST, typename TW>
__global__ __launch_bounds__(256, NLT <= 6 ? 3 : 2) void k_bwdm_l_cols(BwdParams bp, const u16* Pw, const u16* Zw) {
  const KParams& p = bp.k;
  constexpr int LD = D + kBPad, NVT = D / 16, KS2 = (NLT + 1) / 2, QROWS = 32 * KS2;
  constexpr int LP = NLT <= 6 ? kLP : kLPWide;
  // up to six query tiles: Q and dO side by side; ten: one tile's worth of LDS, used for Q first
  // and for dO afterwards
  constexpr bool kTwoTiles = LAST && NLT <= 6;
  __shared__ __attribute__((aligned(16))) u16 Qs[QROWS * LD];
  __shared__ __attribute__((aligned(16))) u16 Xs_two[kTwoTiles ? QROWS * LD : 8];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2, d = D;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;
  const int nkt = (NK + 15) >> 4;

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const long long qcol = axis_offset(p.cmap, bq * b2 + j);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qcol * p.qs.token;
  const u16* dOp = (const u16*)bp.dO + b * p.os.batch + hd * p.os.head + qcol * p.os.token;
  stage_rows_batched<D, LD, QROWS, 256>(Qs, Qp, tile_rows(p, a, p.qs.token), b1, tid);
  if (kTwoTiles) stage_rows_batched<D, LD, QROWS, 256>(Xs_two, dOp, tile_rows(p, a, p.os.token), b1, tid);
  __syncthreads();

  const u16* Pt = Pw + row0 * LP;
  const u16* Zt = Zw + row0 * LP;
  // d alpha_L[nk] = scale sum_l dZ[l, nk] Q[l], d c_L[nk] = -sum_l dZ[l, nk]
  for (int kt = wave; kt < nkt; kt += 4) {
    const int nk = 16 * kt + c;
    const int nkc = nk < NK ? nk : NK - 1;
    bf16x8 zb[1][KS2];
    float zsum = 0.f;
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      zb[0][st] = ld_global_16B(Zt + (size_t)nkc * LP + 32 * st + 8 * g);
#pragma unroll
      for (int e = 0; e < 8; ++e) zsum += (float)zb[0][st][e];
    }
    zsum = xsum(zsum);
    if (g == 0 && nk < NK) bp.dcL[row0 + nk] = -zsum;
    f32x4 o[1][NVT];
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) o[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      const bf16x8 one[1] = {zb[0][st]};
      pv_step_nat<D, 1, LD>(Qs + 32 * st * LD, one, 1, o, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (nk < NK) store_ws_row<D>((TW*)bp.daL + (row0 + nk) * d, o[0], p.scale, g);
    if constexpr (kTwoTiles) {
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) o[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < KS2; ++st) {
        const bf16x8 one[1] = {ld_global_16B(Pt + (size_t)nkc * LP + 32 * st + 8 * g)};
        pv_step_nat<D, 1, LD>(Xs_two + 32 * st * LD, one, 1, o, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (nk < NK) store_ws_row<D>((TW*)bp.dY + (row0 + nk) * d, o[0], 1.0f, g);
    }
  }
  if constexpr (LAST && !kTwoTiles) {
    // dY[nk] = sum_l L[l, nk] dO[l], with dO in the tile Q has just left
    __syncthreads();
    stage_rows_batched<D, LD, QROWS, 256>(Qs, dOp, tile_rows(p, a, p.os.token), b1, tid);
    __syncthreads();
    for (int kt = wave; kt < nkt; kt += 4) {
      const int nk = 16 * kt + c;
      const int nkc = nk < NK ? nk : NK - 1;
      f32x4 o[1][NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) o[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < KS2; ++st) {
        const bf16x8 one[1] = {ld_global_16B(Pt + (size_t)nkc * LP + 32 * st + 8 * g)};
        pv_step_nat<D, 1, LD>(Qs + 32 * st * LD, one, 1, o, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (nk < NK) store_ws_row<D>((TW*)bp.dY + (row0 + nk) * d, o[0], 1.0f, g);
    }
  }
}

// ---------------------------------------------------------------------------------------
// stage R backward.  Work item = one key block (batch*head, n, k); for each the workgroup (NT waves)
// loops over the query tiles m that see it.  Wave w owns query columns j = 16w + c for the softmax
// side (as the forward stage R) and key rows i = 16w + c for the dK / dV accumulation, whose
// contraction runs over j: R and scale dS pass through LDS transposed ([i][j], bf16) in between.
//
// The grid is persistent: workgroup g takes items g, g + gridDim.x, ...  The global loads of the
// next step (the next query tile, or the next item's K / V and first tile) are issued as soon as
// the current step's operands have moved from the register stage into LDS, so they are in flight
// during the whole of the current step's arithmetic and stores; without that every workgroup of
// the launch alternates between a load burst, arithmetic and a store burst in lockstep.
//
// LW (loader waves; for the shapes whose tiles leave one workgroup per compute unit): the workgroup
// has NT more waves that do nothing but the memory side of the pipeline, i.e. hold the register
// stage, write it to LDS between the step's first two barriers and issue the next step's loads.
// A wave that issues a step's 66 KB of loads sits in the issue for about their transfer time; on
// the arithmetic waves that time is lost (nothing else runs on their SIMDs), on waves of their own
// it overlaps the arithmetic.  Both kinds of waves run the same step sequence and meet at the
// same three barriers per step.
// ---------------------------------------------------------------------------------------
// Five and six waves (64 < b2 <= 96) always run with loader waves, three and two of them (eight
// waves in all: a third wave on a SIMD would leave 168 registers each); at t = T and head_dim 128 their five tiles and two transposed
// arrays exceed LDS, so scale dS^T takes the place of the V tile once V's logit products are done
// (one more barrier per step; the loader waves write V again every step).
template <int NT> constexpr int kLoaderThreads = NT == 5 ? 192 : NT == 6 ? 128 : 64 * NT;
template <int NT, int D, bool LAST, typename TW, bool LW = false>
__global__ __launch_bounds__(64 * NT + (LW ? kLoaderThreads<NT> : 0), LW ? 2 : (LAST ? 1 : 2)) void k_bwdm_r(BwdParams bp, int first, int nitems) {
  const KParams& p = bp.k;
  constexpr int LD = D + kBPad, KS1 = D / 32, NVT = D / 16, KS2 = (NT + 1) / 2, ROWS = 32 * KS2;
  constexpr int LR = ROWS + 8, NTHR = 64 * NT, LTHR = LW ? kLoaderThreads<NT> : NTHR;
  constexpr bool kAlias = LAST && NT >= 5 && D == 128;
  static_assert(!kAlias || (LW && ROWS * LR <= ROWS * LD), "scale dS^T in the V tile");
  __shared__ __attribute__((aligned(16))) u16 Ks[ROWS * LD];              // K[n, k, i, :]
  __shared__ __attribute__((aligned(16))) u16 Vs[LAST ? ROWS * LD : 8];   // V[n, k, i, :]
  __shared__ __attribute__((aligned(16))) u16 As[ROWS * LD];              // abar[m, n, k, j, :]
  __shared__ __attribute__((aligned(16))) u16 Gs[ROWS * LD];              // d alpha_L[m, n, j, k, :]
  __shared__ __attribute__((aligned(16))) u16 Ys[LAST ? ROWS * LD : 8];   // d Y[m, n, j, k, :]
  __shared__ __attribute__((aligned(16))) u16 RT[ROWS * LR];              // R[j, i] as [i][j]
  __shared__ __attribute__((aligned(16))) u16 ST_own[kAlias ? 8 : ROWS * LR];   // scale dS[j, i] as [i][j]
  u16* ST = kAlias ? Vs : ST_own;
  __shared__ float dcls[LW ? ROWS : 1];                                   // d c_L of the step's columns (LW)

  // LW: threads NTHR .. 2 NTHR - 1 are the loader waves; tid is a thread's index within its kind
  const bool loader = LW && (int)threadIdx.x >= NTHR;
  const int tid = loader ? (int)threadIdx.x - NTHR : (int)threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2, d = D;
  const int nkb = p.ntk * b1;                   // key blocks per (batch, head)
  const size_t NKtot = (size_t)p.ntk * b1;
  const int j = 16 * wave + c;                  // query column (softmax side) / key row (dK side)
  const float scale2 = p.scale * kLog2e;

  // one work item: key block nk of (batch, head) slot bhl
  struct Item {
    int w, nk, bhl, bh, k, an, bn, ml0;
    long long krow;
  };
  auto decode = [&](int w) {
    Item it;
    it.w = w;
    it.bhl = w / nkb;
    it.nk = w - it.bhl * nkb;
    it.bh = p.bh0 + it.bhl;
    const int n = it.nk / b1;
    it.k = it.nk - n * b1;
    it.an = n / p.c2;
    it.bn = n - it.an * p.c2;
    it.krow = row_offset(p, it.an, it.k);
    // the query tiles that do not see this key tile form a prefix (a later chunk sees more)
    it.ml0 = 0;
    while (it.ml0 < p.ntq && it.an >= visible_key_tile_rows((p.m0 + it.ml0) / p.c2, p.c1k, p.ct, p.qt0)) ++it.ml0;
    return it;
  };

  // register stages: every global load of a step is issued before the first LDS store
  constexpr bool kF32Ws = sizeof(TW) == 4;
  // (the stages cover the 16 NT rows the waves own; an odd NT leaves 16 more tile rows, which the
  // 32-row steps of the second products read: zeroed once below and never written again)
  constexpr int SROWS = 16 * NT;
  RowRegs<D, SROWS, LTHR> rk;                          // K rows
  RowRegs<D, LAST ? SROWS : 1, LTHR> rv;               // V rows (t = T)
  RowRegs<D, SROWS, LTHR> ra;                          // Q rows, or abar stored as bf16
  RowRegsF32<D, kF32Ws ? SROWS : 1, LTHR> raf;         // abar stored as fp32
  typename std::conditional<kF32Ws, RowRegsF32<D, SROWS, LTHR>, RowRegs<D, SROWS, LTHR>>::type rg;
  typename std::conditional<kF32Ws, RowRegsF32<D, LAST ? SROWS : 1, LTHR>, RowRegs<D, LAST ? SROWS : 1, LTHR>>::type ry;
  auto issue_block = [&](const Item& it) {
    const int b = it.bh / p.H, hd = it.bh - b * p.H;
    const u16* Kp = (const u16*)p.K + b * p.ks.batch + hd * p.ks.head + it.krow * p.ks.token;
    rk.load(Kp, TokRows{0, p.cmap, it.bn * b2, p.ks.token}, b2, tid);
    if (LAST) {
      const u16* Vp = (const u16*)p.V + b * p.vs.batch + hd * p.vs.head + it.krow * p.vs.token;
      rv.load(Vp, TokRows{0, p.cmap, it.bn * b2, p.vs.token}, b2, tid);
    }
  };
  // part 0: abar (or Q) only, part 1: the gradients only, -1: both
  auto issue_tile = [&](const Item& it, int ml, int part = -1) {
    const int m = p.m0 + ml, a = m / p.c2, bq = m - a * p.c2;
    const size_t jrow0 = ((size_t)it.bhl * p.ntq + ml) * b2;
    const int nk = it.nk;
    auto jrow = [&](int jj) { return (long long)(((jrow0 + jj) * NKtot + nk) * d); };
    const size_t ablk = (((size_t)it.bhl * p.ntq + ml) * NKtot + nk) * b2;
    if (part != 1) {
      if (first) {
        const int b = it.bh / p.H, hd = it.bh - b * p.H;
        const u16* Qbase = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head;
        const long long qrow = row_offset(p, a, it.k);
        ra.load(Qbase + qrow * p.qs.token, TokRows{0, p.cmap, bq * b2, p.qs.token}, b2, tid);
      } else if constexpr (kF32Ws) {
        raf.load((const float*)p.aR + ablk * d, PlainRows{D}, b2, tid);
      } else {
        ra.load((const u16*)p.aR + ablk * d, PlainRows{D}, b2, tid);
      }
    }
    if (part != 0) {
      rg.load((const TW*)bp.daL, jrow, b2, tid);
      if (LAST) ry.load((const TW*)bp.dY, jrow, b2, tid);
    }
  };

  Item cur = decode(blockIdx.x);          // the host launches at most nitems workgroups
  int ml = cur.ml0;
  bool newblk = true;
  if constexpr (LW) {
    if (loader) {
      // ---- loader waves: the memory side of every step, the same sequence of steps and barriers
      static_assert(LTHR >= ROWS, "one loader thread per column for d c_L");
      auto dcl_of = [&](const Item& it, int mlx) {
        return bp.dcL[(((size_t)it.bhl * p.ntq + mlx) * b2 + (tid < b2 ? tid : b2 - 1)) * NKtot + it.nk];
      };
      float dcl_r = 0.f;
      issue_block(cur);
      if (ml < p.ntq) {
        if (tid < ROWS) dcl_r = dcl_of(cur, ml);
        issue_tile(cur, ml);
      }
      while (true) {
        const bool has_tile = ml < p.ntq;
        __syncthreads();                       // the arithmetic waves are done with the tiles
        if (newblk) rk.template store<LD>(Ks, tid);
        if (LAST && (newblk || kAlias)) rv.template store<LD>(Vs, tid);
        if (has_tile) {
          if (first || !kF32Ws) ra.template store<LD>(As, tid);
          else raf.template store<LD>(As, tid);
          rg.template store<LD>(Gs, tid);
          if (LAST) ry.template store<LD>(Ys, tid);
          if (tid < ROWS) dcls[tid] = dcl_r;
        }
        const bool item_done = !has_tile || ml + 1 >= p.ntq;
        Item nxt = cur;
        int nml = ml + 1;
        bool more = true;
        if (item_done) {
          const int w2 = cur.w + (int)gridDim.x;
          more = w2 < nitems;
          if (more) {
            nxt = decode(w2);
            nml = nxt.ml0;
          }
        }
        __syncthreads();                       // the tiles are in LDS
        // the next step's loads, in two halves around the arithmetic waves' middle barrier: the
        // wave sits in the issue of each half while the arithmetic waves work
        const bool nxt_tile = more && nml < p.ntq;
        if (item_done && more) issue_block(nxt);
        if (nxt_tile) {
          if (tid < ROWS) dcl_r = dcl_of(nxt, nml);
          issue_tile(nxt, nml, 0);
        }
        if (kAlias && has_tile) __syncthreads();   // (the arithmetic waves are done with the V tile)
        if (has_tile) __syncthreads();         // (the arithmetic waves' barrier between their two halves)
        if (nxt_tile) issue_tile(nxt, nml, 1);
        if (!more) break;
        cur = nxt;
        ml = nml;
        newblk = item_done;
      }
      return;
    }
  } else {
    issue_block(cur);
    if (ml < p.ntq) issue_tile(cur, ml);
  }
  for (int idx = tid; idx < ROWS * LR; idx += NTHR) {
    RT[idx] = 0;
    if (!kAlias) ST[idx] = 0;
  }
  if constexpr (ROWS > SROWS) {
    for (int idx = SROWS * LD + tid; idx < ROWS * LD; idx += NTHR) {
      Ks[idx] = 0; As[idx] = 0; Gs[idx] = 0;
      if (LAST) { Vs[idx] = 0; Ys[idx] = 0; }
    }
  }

  f32x4 oK[1][NVT], oV[1][NVT];
#pragma unroll
  for (int vt = 0; vt < NVT; ++vt) {
    oK[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
    oV[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // dK / dV of a finished item.  With loader waves they are stored after the next step's first
  // barrier, while the loader waves write that step's tiles to LDS (the stores need registers only,
  // and a wave sits in their issue for about their transfer time); otherwise right away.
  bool pend_kv = false;
  int pbh = 0, pbn = 0;
  long long pkrow = 0;
  auto store_kv = [&]() {
    if (j < b2) {
      const long long tok = pkrow + axis_offset(p.cmap, pbn * b2 + j);
      if (first && !bp.accumulate) store_rows_f32_nt<D>(bp.dK + ((size_t)pbh * p.Nkv + tok) * d, oK[0], 1.0f, g);
      else store_rows_f32<D>(bp.dK + ((size_t)pbh * p.Nkv + tok) * d, oK[0], 1.0f, g, bp.accumulate != 0);
      if (LAST) store_rows_f32_nt<D>(bp.dV + ((size_t)pbh * p.Nkv + tok) * d, oV[0], 1.0f, g);
    }
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) {
      oK[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
      oV[0][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    pend_kv = false;
  };

  while (true) {
    const bool has_tile = ml < p.ntq;        // an item no query tile sees only writes its zeros
    __syncthreads();                         // the previous step's reads of the LDS tiles
    if constexpr (LW) {
      if (pend_kv) store_kv();
    }
    float dcl = 0.f;
    if constexpr (!LW) {
      if (newblk) {
        rk.template store<LD>(Ks, tid);
        if (LAST) rv.template store<LD>(Vs, tid);
      }
      if (has_tile) {
        if (first || !kF32Ws) ra.template store<LD>(As, tid);
        else raf.template store<LD>(As, tid);
        rg.template store<LD>(Gs, tid);
        if (LAST) ry.template store<LD>(Ys, tid);
      }
      // c_L's gradient of this lane's column: fetched ahead of the next step's loads, which would
      // otherwise have to land first (loads return in order)
      if (has_tile && j < b2) dcl = bp.dcL[(((size_t)cur.bhl * p.ntq + ml) * b2 + j) * NKtot + cur.nk];
    }
    // the step after this one, and its loads
    const bool item_done = !has_tile || ml + 1 >= p.ntq;
    Item nxt = cur;
    int nml = ml + 1;
    bool more = true;
    if (item_done) {
      const int w2 = cur.w + (int)gridDim.x;
      more = w2 < nitems;
      if (more) {
        nxt = decode(w2);
        nml = nxt.ml0;
        if constexpr (!LW) issue_block(nxt);
      }
    }
    if constexpr (!LW) {
      if (more && nml < p.ntq) issue_tile(nxt, nml);
    }
    __syncthreads();
    if constexpr (LW) {
      if (has_tile) dcl = dcls[j];            // written by the loader waves before the barrier
    }

    if (has_tile) {
      // rows (j, nk) of the [m][j][nk][..] arrays and the (m, nk) block of the [m][nk][j][d] arrays
      const int nk = cur.nk, bhl = cur.bhl, bh = cur.bh, k = cur.k;
      const size_t ablk = (((size_t)bhl * p.ntq + ml) * NKtot + nk) * b2;
      // ---- softmax side: lanes own query column j
      {
        const bool live = j < b2;
        bf16x8 qv[KS1], gv[KS1], yv[KS1];
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) {
          qv[ks] = ld_lds_16B(As + j * LD + 32 * ks + 8 * g);
          gv[ks] = ld_lds_16B(Gs + j * LD + 32 * ks + 8 * g);
          if (LAST) yv[ks] = ld_lds_16B(Ys + j * LD + 32 * ks + 8 * g);
        }
        f32x4 s[NT], dr[NT];
        // (t = T: one workgroup per compute unit, one wave per SIMD: LDS reads issued ahead)
        constexpr bool kAhead = LAST && NT <= 4;       // (beyond four waves the registers are needed elsewhere)
        if constexpr (kAhead) rows_dot_ahead<D, NT, LD>(Ks, qv, s, lane);
        else rows_dot<D, NT, LD>(Ks, qv, s, lane);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kAhead) rows_dot_ahead<D, NT, LD>(Ks, gv, dr, lane);
        else rows_dot<D, NT, LD>(Ks, gv, dr, lane);
        __builtin_amdgcn_sched_barrier(0);
        if (LAST) {
          f32x4 dy[NT];
          if constexpr (kAhead) rows_dot_ahead<D, NT, LD>(Vs, yv, dy, lane);
          else rows_dot<D, NT, LD>(Vs, yv, dy, lane);
#pragma unroll
          for (int it = 0; it < NT; ++it) dr[it] += dy[it];
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (kAlias) {
          __syncthreads();                     // every wave is done with V: its tile now takes scale dS^T
          // columns 16 NT .. ROWS - 1 of the rows this wave writes are read as zeros below
          if constexpr (ROWS > 16 * NT) {
            for (int idx = lane; idx < 16 * (ROWS - 16 * NT); idx += 64)
              ST[(16 * wave + idx / (ROWS - 16 * NT)) * LR + 16 * NT + idx % (ROWS - 16 * NT)] = 0;
          }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int it = 0; it < NT; ++it)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const bool ok = 16 * it + 4 * g + r < b2;
            s[it][r] = ok ? s[it][r] * scale2 : -INFINITY;
            mx = fmaxf(mx, s[it][r]);
          }
        mx = xmax(mx);
        float sum = 0.f;
#pragma unroll
        for (int it = 0; it < NT; ++it)
#pragma unroll
          for (int r = 0; r < 4; ++r) sum += exp2_fast(s[it][r] - mx);
        const float lse2 = mx + log2_fast(xsum(sum));
        // R, dR (with the entropy term), dS
        float dot = 0.f;
#pragma unroll
        for (int it = 0; it < NT; ++it)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const bool ok = live && 16 * it + 4 * g + r < b2;
            const float logr2 = s[it][r] - lse2;                     // log2 R, -inf beyond b2
            const float R = ok ? exp2_fast(logr2) : 0.f;
            const float dR = ok ? dr[it][r] + dcl * fmaf(logr2, kLn2, 1.0f) : 0.f;
            s[it][r] = R;
            dr[it][r] = dR;
            dot = fmaf(R, dR, dot);
          }
        dot = xsum(dot);
#pragma unroll
        for (int it = 0; it < NT; ++it)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float ds = p.scale * s[it][r] * (dr[it][r] - dot);   // scale dS
            dr[it][r] = ds;
            const int i = 16 * it + 4 * g + r;
            RT[i * LR + j] = f2bf(s[it][r]);
            ST[i * LR + j] = f2bf(ds);
          }
        // d abar[j] = sum_i (scale dS[j, i]) K[i]
        f32x4 o[NVT];
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) o[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < KS2; ++st) {
          const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
          const bool has = 2 * st + 1 < NT;
          const bf16x8 pz = pack8(dr[2 * st], has ? dr[has ? 2 * st + 1 : 0] : zero);
          pv_step<D, LD>(Ks + 32 * st * LD, pz, o, lane);
          __builtin_amdgcn_sched_barrier(0);
        }
        // d abar of the first iteration is summed over the key tiles into dQ by the last kernel of
        // the call, from the workspace's storage type (with one key tile per query tile there is
        // nothing to sum: it goes straight into dQ)
        if (live) {
          if (first && bp.dq_from_r) {
            const int m = p.m0 + ml, a = m / p.c2, bq = m - a * p.c2;
            const long long tok = row_offset(p, a, k) + axis_offset(p.cmap, bq * b2 + j);
            store_rows_f32<D>(bp.dQ + ((size_t)bh * p.Nq + tok) * d, o, 1.0f, g, true);
          } else if (first && kF32Ws) {
            store_rows_f32<D>(bp.dA + (ablk + j) * d, o, 1.0f, g, false);
          } else {
            store_ws_row<D>((TW*)bp.dA + (ablk + j) * d, o, 1.0f, g);
          }
        }
      }
      __syncthreads();                               // RT / ST complete

      // ---- accumulation side: lanes own key row i = j
#pragma unroll
      for (int st = 0; st < KS2; ++st) {
        const bf16x8 bR[1] = {ld_lds_16B(RT + j * LR + 32 * st + 8 * g)};
        const bf16x8 bS[1] = {ld_lds_16B(ST + j * LR + 32 * st + 8 * g)};
        pv_step_nat<D, 1, LD>(Gs + 32 * st * LD, bR, 1, oK, lane);     // dK += R^T d alpha_L
        __builtin_amdgcn_sched_barrier(0);
        pv_step_nat<D, 1, LD>(As + 32 * st * LD, bS, 1, oK, lane);     // dK += scale dS^T abar
        __builtin_amdgcn_sched_barrier(0);
        if (LAST) {
          pv_step_nat<D, 1, LD>(Ys + 32 * st * LD, bR, 1, oV, lane);   // dV += R^T d Y
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (item_done) {
      pend_kv = true;
      pbh = cur.bh;
      pbn = cur.bn;
      pkrow = cur.krow;
      if constexpr (!LW) store_kv();
    }
    if (!more) break;
    cur = nxt;
    ml = nml;
    newblk = item_done;
  }
  if (pend_kv) store_kv();
}

}  // namespace

bool bwd_bf16_fits(const KParams& kp) { return kp.b1 <= kBRowsWide && (kp.d == 64 || kp.d == 128); }
size_t bwd_bf16_scratch_bytes(const KParams& kp, int ntq_total) {
  // the transposed L and dZ arrays: (m, j, nk) rows of 96 or 160 bf16 each, two arrays
  return (size_t)ntq_total * kp.b2 * kp.ntk * kp.b1 * lp_of(kp.b1) * 2 * 2;
}

template <int D, bool LAST, typename TW>
static hipError_t launch_rows(const BwdParams& bp, dim3 grid, int nkt, u16* Pw, u16* Zw, hipStream_t s) {
  switch (nkt) {
    case 1: case 2: k_bwdm_l_rows<D, 2, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    case 3: case 4: k_bwdm_l_rows<D, 4, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    case 5: case 6: k_bwdm_l_rows<D, 6, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
template <int D, bool LAST, typename TW>
static hipError_t launch_cols(const BwdParams& bp, dim3 grid, int nlt, const u16* Pw, const u16* Zw,
                              hipStream_t s) {
  switch (nlt) {
    case 1: case 2: k_bwdm_l_cols<D, 2, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    case 3: case 4: k_bwdm_l_cols<D, 4, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    case 5: case 6: k_bwdm_l_cols<D, 6, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    case 7: case 8: case 9: case 10: k_bwdm_l_cols<D, 10, LAST, TW><<<grid, 256, 0, s>>>(bp, Pw, Zw); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

bool bwd_bf16_r_fits(const KParams& kp) { return kp.b2 <= 96 && (kp.d == 64 || kp.d == 128); }

// Workgroups of `kernel` the current device keeps resident at once (its compute units times the
// workgroups of `threads` threads that fit one): the size of a persistent grid.
template <typename K>
static int resident_workgroups(K kernel, int threads) {
  int per_cu = 0, dev = 0, cus = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1)
    per_cu = 1;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  return per_cu * cus;
}

template <int NT, int D, typename TW>
static hipError_t launch_r_nt(const BwdParams& bp, int nitems, bool first, bool last, hipStream_t s) {
  // persistent grid: as many workgroups as stay resident, each striding over the key blocks
  if constexpr (NT >= 5) {
    // 64 < b2 <= 96: loader waves at every iteration, bf16 workspace only
    if constexpr (sizeof(TW) == 2) {
      constexpr int threads = 64 * NT + kLoaderThreads<NT>;
      if (last) {
        static const int resident = resident_workgroups(k_bwdm_r<NT, D, true, TW, true>, threads);
        k_bwdm_r<NT, D, true, TW, true><<<dim3(nitems < resident ? nitems : resident), threads, 0, s>>>(bp, first ? 1 : 0, nitems);
      } else {
        static const int resident = resident_workgroups(k_bwdm_r<NT, D, false, TW, true>, threads);
        k_bwdm_r<NT, D, false, TW, true><<<dim3(nitems < resident ? nitems : resident), threads, 0, s>>>(bp, first ? 1 : 0, nitems);
      }
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  } else if (last) {
    if constexpr (D == 128 && NT >= 3) {
      // five tiles and the two transposed arrays leave one workgroup per compute unit: loader waves
      static const int resident = resident_workgroups(k_bwdm_r<NT, D, true, TW, true>, 128 * NT);
      k_bwdm_r<NT, D, true, TW, true><<<dim3(nitems < resident ? nitems : resident), 128 * NT, 0, s>>>(bp, first ? 1 : 0, nitems);
    } else {
      static const int resident = resident_workgroups(k_bwdm_r<NT, D, true, TW>, 64 * NT);
      k_bwdm_r<NT, D, true, TW><<<dim3(nitems < resident ? nitems : resident), 64 * NT, 0, s>>>(bp, first ? 1 : 0, nitems);
    }
  } else {
    // (t < T keeps two workgroups per compute unit without loader waves: one workgroup with them
    // measured 8 % slower at b2 = 52 and 45 % slower at b2 = 40)
    static const int resident = resident_workgroups(k_bwdm_r<NT, D, false, TW>, 64 * NT);
    k_bwdm_r<NT, D, false, TW><<<dim3(nitems < resident ? nitems : resident), 64 * NT, 0, s>>>(bp, first ? 1 : 0, nitems);
  }
  return hipGetLastError();
}
template <int D, typename TW>
static hipError_t launch_r_d(const BwdParams& bp, int nitems, bool first, bool last, hipStream_t s) {
  switch ((bp.k.b2 + 15) / 16) {
    case 1: return launch_r_nt<1, D, TW>(bp, nitems, first, last, s);
    case 2: return launch_r_nt<2, D, TW>(bp, nitems, first, last, s);
    case 3: return launch_r_nt<3, D, TW>(bp, nitems, first, last, s);
    case 4: return launch_r_nt<4, D, TW>(bp, nitems, first, last, s);
    case 5: return launch_r_nt<5, D, TW>(bp, nitems, first, last, s);
    case 6: return launch_r_nt<6, D, TW>(bp, nitems, first, last, s);
  }
  return hipErrorInvalidValue;
}

// Stage R backward on the matrix unit (b2 <= 64).  ws_bf16: the forward intermediates in the
// workspace are bf16 (written by the bf16 forward kernels) rather than fp32.
hipError_t launch_bwd_bf16_stage_r(const BwdParams& bp, int nbh, bool first, bool last, bool ws_bf16,
                                   hipStream_t s) {
  const KParams& kp = bp.k;
  const long long items = (long long)kp.ntk * kp.b1 * nbh;      // key blocks of the pass
  if (items < 1 || items > 0x7fffffff) return hipErrorInvalidValue;
  const int nitems = (int)items;
  if (ws_bf16)
    return kp.d == 128 ? launch_r_d<128, u16>(bp, nitems, first, last, s)
                       : launch_r_d<64, u16>(bp, nitems, first, last, s);
  return kp.d == 128 ? launch_r_d<128, float>(bp, nitems, first, last, s)
                     : launch_r_d<64, float>(bp, nitems, first, last, s);
}

// Stage L backward on the matrix unit; scratch = bwd_bf16_scratch_bytes() of device memory.
template <int D, typename TW>
static hipError_t launch_l_d(const BwdParams& bp, dim3 grid, int nkt, int nlt, bool last, u16* Pw, u16* Zw,
                             hipStream_t s) {
  hipError_t e;
  if (16 * nkt > kBRows) {
    // key range beyond the resident kernel: streamed, one wave per query tile (always six or ten
    // waves: the staging loops are laid out for the full workgroup)
    if constexpr (sizeof(TW) == 2) {
      // bf16 workspace: the pipelined kernel
      if (nlt <= 6 && bp.k.rl == 0) {
        // twelve waves, and the column side of the stage in the same kernel: no cols launch
        if (last) k_bwdm_l_rows_ring<D, true, 6, 2><<<grid, 768, 0, s>>>(bp, Pw, Zw);
        else k_bwdm_l_rows_ring<D, false, 6, 2><<<grid, 768, 0, s>>>(bp, Pw, Zw);
        return hipGetLastError();
      } else if (nlt <= 6) {
        if (last) k_bwdm_l_rows_ring<D, true, 6, 1><<<grid, 384, 0, s>>>(bp, Pw, Zw);
        else k_bwdm_l_rows_ring<D, false, 6, 1><<<grid, 384, 0, s>>>(bp, Pw, Zw);
      } else {
        if (last) k_bwdm_l_rows_ring<D, true, 10, 1><<<grid, 640, 0, s>>>(bp, Pw, Zw);
        else {
          // t < T: column side in the same kernel
          k_bwdm_l_rows_ring<D, false, 10, 1><<<grid, 640, 0, s>>>(bp, Pw, Zw);
          return hipGetLastError();
        }
      }
    } else if (nlt <= 6) {
      if (last) k_bwdm_l_rows_stream<D, true, TW, 6><<<grid, 384, 0, s>>>(bp, Pw, Zw);
      else k_bwdm_l_rows_stream<D, false, TW, 6><<<grid, 384, 0, s>>>(bp, Pw, Zw);
    } else {
      if (last) k_bwdm_l_rows_stream<D, true, TW, 10><<<grid, 640, 0, s>>>(bp, Pw, Zw);
      else k_bwdm_l_rows_stream<D, false, TW, 10><<<grid, 640, 0, s>>>(bp, Pw, Zw);
    }
    e = hipGetLastError();
  } else {
    e = last ? launch_rows<D, true, TW>(bp, grid, nkt, Pw, Zw, s)
             : launch_rows<D, false, TW>(bp, grid, nkt, Pw, Zw, s);
  }
  if (e != hipSuccess) return e;
  return last ? launch_cols<D, true, TW>(bp, grid, nlt, Pw, Zw, s)
              : launch_cols<D, false, TW>(bp, grid, nlt, Pw, Zw, s);
}

hipError_t launch_bwd_bf16_stage_l(const BwdParams& bp, int nbh, bool last, bool ws_bf16, void* scratch,
                                   hipStream_t s) {
  const KParams& kp = bp.k;
  dim3 grid(kp.b2, kp.ntq, nbh);
  const int nkt = (kp.ntk * kp.b1 + 15) / 16, nlt = (kp.b1 + 15) / 16;
  u16* Pw = (u16*)scratch;
  u16* Zw = Pw + (size_t)nbh * kp.ntq * kp.b2 * kp.ntk * kp.b1 * lp_of(kp.b1);
  if (kp.d == 128)
    return ws_bf16 ? launch_l_d<128, u16>(bp, grid, nkt, nlt, last, Pw, Zw, s)
                   : launch_l_d<128, float>(bp, grid, nkt, nlt, last, Pw, Zw, s);
  return ws_bf16 ? launch_l_d<64, u16>(bp, grid, nkt, nlt, last, Pw, Zw, s)
                 : launch_l_d<64, float>(bp, grid, nkt, nlt, last, Pw, Zw, s);
}

}  // namespace mrt
