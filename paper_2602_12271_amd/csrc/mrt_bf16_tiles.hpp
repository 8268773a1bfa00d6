// Building blocks of the bf16 MFMA kernels (forward and backward): vector types, LDS / global
// access helpers, the transposed LDS read, the second-product step and tile staging.
// See the head of mrt_bf16.hip for the register layouts these assume.
#pragma once
#include <type_traits>
#include <utility>

#include "mrt_internal.hpp"

namespace mrt {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef unsigned short u16;

constexpr int kPad = 16;   // bf16 elements of padding per LDS row: row stride = 8 banks mod 64

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline bf16x8 ld_global_16B(const u16* p) { return as_bf16x8(*(const uint4*)p); }

__device__ inline bf16x8 ld_lds_16B(const u16* p) { return as_bf16x8(*(const uint4*)p); }

// transposed LDS read: the 16 lanes of a group address 4 rows x 16 columns (lane s -> row s/4,
// columns 4(s%4)..+3); lane c receives column c of those 4 rows.
__device__ inline s16x4 ld_lds_tr(const u16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

__device__ inline u16 f2bf(float x) { return __builtin_bit_cast(u16, (__bf16)x); }

__device__ inline bf16x8 pack8(f32x4 a, f32x4 b) {
  bf16x8 r;
  r[0] = (__bf16)a[0]; r[1] = (__bf16)a[1]; r[2] = (__bf16)a[2]; r[3] = (__bf16)a[3];
  r[4] = (__bf16)b[0]; r[5] = (__bf16)b[1]; r[6] = (__bf16)b[2]; r[7] = (__bf16)b[3];
  return r;
}

__device__ inline f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Softmax arithmetic runs in the base-2 domain: logits are multiplied by scale*log2(e) (one
// fma) and exponentiated with the hardware exp2, which saves a multiply per element.
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
__device__ inline float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

// Reductions over the four 16-lane rows of a wave, per lane column (lane & 15): the lanes that hold
// one accumulator column of an MFMA tile.  gfx950's row-swap instructions do the exchange in the
// vector ALU instead of a ds_bpermute through the LDS crossbar: with a = b = x on entry,
// v_permlane16_swap leaves the even rows' values in a and the odd rows' in b (in both rows of each
// pair), v_permlane32_swap the same for the two halves of the wave.  Written as inline assembly (the
// builtin folds the two results into one when both operands are the same value), with the wait
// states a VALU producer / consumer of the swapped registers needs.  All 64 lanes must be active.
__device__ inline void row_swap16(float& a, float& b) {
  asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ inline void row_swap32(float& a, float& b) {
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ inline float xmax(float x) {
  float a = x, b = x;
  row_swap16(a, b);
  a = b = fmaxf(a, b);
  row_swap32(a, b);
  return fmaxf(a, b);
}
__device__ inline float xsum(float x) {
  float a = x, b = x;
  row_swap16(a, b);
  a = b = a + b;
  row_swap32(a, b);
  return a + b;
}

// Maximum / sum over the 16 lanes that share lane >> 4 (one accumulator row of an MFMA tile):
// data-parallel-primitive moves (pairs, quads, mirrored halves of 8, mirrored 16), no LDS traffic.
template <int CTRL>
__device__ inline float dpp_mov(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
__device__ inline float row16_max(float x) {
  x = fmaxf(x, dpp_mov<0xB1>(x));    // quad_perm [1,0,3,2]
  x = fmaxf(x, dpp_mov<0x4E>(x));    // quad_perm [2,3,0,1]
  x = fmaxf(x, dpp_mov<0x141>(x));   // row_half_mirror
  return fmaxf(x, dpp_mov<0x140>(x));  // row_mirror
}
__device__ inline float row16_sum(float x) {
  x += dpp_mov<0xB1>(x);
  x += dpp_mov<0x4E>(x);
  x += dpp_mov<0x141>(x);
  return x + dpp_mov<0x140>(x);
}
// Sum over aligned groups of 8 lanes (the first three steps of the above).
__device__ inline float row8_sum(float x) {
  x += dpp_mov<0xB1>(x);
  x += dpp_mov<0x4E>(x);
  return x + dpp_mov<0x141>(x);
}

// Swizzled LDS tiles (SWZ = true; rows of 128 bf16 = 256 bytes = all 64 banks, NOT padded): the
// 16-byte piece p of row r sits at piece index p ^ swz16(r), swz16(r) = 4 (r mod 4) ^ (r / 4 mod 4).
// Both ways a tile is read are then free of bank conflicts: a matrix operand read of one piece
// column from 8 consecutive rows (ds_read_b128: 8 lanes per clock; swz16 takes 8 different values
// on rows 8a .. 8a + 7) and a transposed read (ds_read_b64_tr_b16: 16 lanes per clock on rows
// 4g .. 4g + 3, four pieces q + 4k each: (q + 4k) ^ swz16 = (q ^ g) + 4 (k ^ e) covers all 16
// pieces).  With padded rows one of the two always conflicts (two- to four-fold).
__device__ inline int swz16(int row) { return ((row & 3) << 2) ^ ((row >> 2) & 3); }
template <int LD, bool SWZ>
__device__ inline int tile_off(int row, int piece) {
  return row * LD + 8 * (SWZ ? piece ^ swz16(row) : piece);
}

// Second product for one 32-key step: acc[vt] += Val^T[phi(vt, .), keys] * P.
// vals points at LDS row `32*step` of a row-major [rows][D + kPad] tile; output feature of
// accumulator row (4g + r) of tile vt is phi = 32(vt/2) + 8g + 4(vt%2) + r.
template <int D, int LD = D + kPad>
__device__ inline void pv_step(const u16* vals, bf16x8 pb, f32x4* acc, int lane) {
  constexpr int NVT = D / 16, HALF = NVT / 2;
  const int g = lane >> 4, s = lane & 15, e = s >> 2, q = s & 3;
  const u16* base = vals + (4 * g + e) * LD + 8 * q;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    s16x4 lo[HALF], hi[HALF];
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const int vt = h * HALF + i;
      const u16* p0 = base + 32 * (vt >> 1) + 4 * (vt & 1);
      lo[i] = ld_lds_tr(p0);
      hi[i] = ld_lds_tr(p0 + 16 * LD);
    }
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      s16x8 a = __builtin_shufflevector(lo[i], hi[i], 0, 1, 2, 3, 4, 5, 6, 7);
      acc[h * HALF + i] = mfma(__builtin_bit_cast(bf16x8, a), pb, acc[h * HALF + i]);
    }
  }
}

// One half of pv_step: tiles h*D/32 .. (h+1)*D/32 - 1 (features 64h' .. of each 32-feature pair
// group) into acc[0 .. D/32).
// DIR = -1: the tile is stored bottom-up (row r at vals - r * LD).
template <int D, int LD = D + kPad, int DIR = 1>
__device__ inline void pv_step_half(const u16* vals, bf16x8 pb, f32x4* acc, int lane, int h) {
  constexpr int HALF = D / 32;
  const int g = lane >> 4, s = lane & 15, e = s >> 2, q = s & 3;
  const u16* base = vals + DIR * (4 * g + e) * LD + 8 * q;
  s16x4 lo[HALF], hi[HALF];
#pragma unroll
  for (int i = 0; i < HALF; ++i) {
    const int vt = h * HALF + i;
    const u16* p0 = base + 32 * (vt >> 1) + 4 * (vt & 1);
    lo[i] = ld_lds_tr(p0);
    hi[i] = ld_lds_tr(p0 + DIR * 16 * LD);
  }
#pragma unroll
  for (int i = 0; i < HALF; ++i) {
    s16x8 a = __builtin_shufflevector(lo[i], hi[i], 0, 1, 2, 3, 4, 5, 6, 7);
    acc[i] = mfma(__builtin_bit_cast(bf16x8, a), pb, acc[i]);
  }
}

// Same for NB probability operands sharing every value-side LDS read (operands >= nb idle).
// vals must be a multiple of 16 rows into its tile when SWZ.
template <int D, int NB, int LD = D + kPad, bool SWZ = false>
__device__ inline void pv_step_multi(const u16* vals, const bf16x8 (&pb)[NB], int nb,
                                     f32x4 (&acc)[NB][D / 16], int lane) {
  constexpr int NVT = D / 16, HALF = NVT / 2;
  const int g = lane >> 4, s = lane & 15, e = s >> 2, q = s & 3;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    s16x4 lo[HALF], hi[HALF];
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const int vt = h * HALF + i;
      // rows 4g + e and 16 + 4g + e (the same swizzle), piece q + 4 (vt / 2), half vt % 2
      const u16* p0 = vals + tile_off<LD, SWZ>(4 * g + e, q + 4 * (vt >> 1)) + 4 * (vt & 1);
      lo[i] = ld_lds_tr(p0);
      hi[i] = ld_lds_tr(p0 + 16 * LD);
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

// Store a lane's D/16 accumulator tiles (scaled) as bf16: 16 bytes per pair of tiles at
// feature 32q + 8g.
template <int D>
__device__ inline void store_rows(u16* row, const f32x4* acc, float mul, int g) {
#pragma unroll
  for (int q = 0; q < D / 32; ++q) {
    bf16x8 o = pack8(acc[2 * q] * mul, acc[2 * q + 1] * mul);
    *(uint4*)(row + 32 * q + 8 * g) = __builtin_bit_cast(uint4, o);
  }
}

// The same row with non-temporal stores: the operator's output, which no later kernel of the call
// reads (it would only displace the workspace arrays from the caches).
template <int D>
__device__ inline void store_rows_nt(u16* row, const f32x4* acc, float mul, int g) {
  typedef __attribute__((ext_vector_type(4))) unsigned ux4;
#pragma unroll
  for (int q = 0; q < D / 32; ++q) {
    bf16x8 o = pack8(acc[2 * q] * mul, acc[2 * q + 1] * mul);
    __builtin_nontemporal_store(__builtin_bit_cast(ux4, o), (ux4*)(row + 32 * q + 8 * g));
  }
}

// Half h of such a row from the D/32 tiles pv_step_half accumulates.
template <int D>
__device__ inline void store_rows_half(u16* row, const f32x4* acc, float mul, int g, int h) {
#pragma unroll
  for (int q = 0; q < D / 64; ++q) {
    bf16x8 o = pack8(acc[2 * q] * mul, acc[2 * q + 1] * mul);
    *(uint4*)(row + 32 * (h * (D / 64) + q) + 8 * g) = __builtin_bit_cast(uint4, o);
  }
}

// Element offset of row r of a tile of a token-indexed tensor (Q, K, V, O): the tile's rows are
// the block-grid indices x0 + r along one side of the block grid.
// A row map is "linear" when consecutive rows are a fixed number of elements apart (one-level axis
// maps; always for the workspace arrays): row r then sits at first() + r * step(), and the host's
// checks keep every offset inside one (batch, head) below 2^31 elements, so that the per-lane part
// of an address is a 32-bit offset from a wave-uniform base.
struct TokRows {
  long long base;      // tokens
  AxisMap m;
  int x0;
  long long tstride;   // elements per token
  __device__ inline long long operator()(int r) const { return (base + axis_offset(m, x0 + r)) * tstride; }
  __device__ inline bool linear() const { return m.div == 0; }
  __device__ inline long long first() const { return (base + (long long)x0 * m.lo) * tstride; }
  __device__ inline unsigned step() const { return (unsigned)m.lo * (unsigned)tstride; }
};
// Rows of tile row a: contiguous block-grid rows, or nh rows of each of the tile's frames.
__device__ inline TokRows tile_rows(const KParams& p, int a, long long tstride) {
  if (p.nh == 0) return TokRows{0, p.rmap, a * p.b1, tstride};
  const int fa = a / p.nhb, ha = a - fa * p.nhb;
  return TokRows{(long long)fa * p.tf_tok + (long long)ha * p.th_tok, AxisMap{p.nh, p.hw, p.rmap.lo}, 0,
                 tstride};
}
// Rows at a fixed stride (the intermediates in the workspace).
struct PlainRows {
  long long stride;
  __device__ inline long long operator()(int r) const { return (long long)r * stride; }
  __device__ inline bool linear() const { return true; }
  __device__ inline long long first() const { return 0; }
  __device__ inline unsigned step() const { return (unsigned)stride; }
};

// Row maps that can say whether their rows are evenly spaced (TokRows, PlainRows); any other
// callable taking a row index is treated as a general map.
template <typename T, typename = void>
struct HasLinear : std::false_type {};
template <typename T>
struct HasLinear<T, std::void_t<decltype(std::declval<const T&>().linear())>> : std::true_type {};

// Cooperative copy of `rows` rows of D bf16 (row r at src + rowoff(r)) into a row-major LDS tile,
// zero-filling rows >= valid.
template <int D, int LD = D + kPad, typename RowFn>
__device__ inline void stage_rows(u16* dst, const u16* src, RowFn rowoff, int rows, int valid,
                                  int tid, int nthr) {
  constexpr int CPR = D / 8;
  for (int idx = tid; idx < rows * CPR; idx += nthr) {
    const int r = idx / CPR, c = idx - r * CPR;
    uint4 v = {0u, 0u, 0u, 0u};
    if (r < valid) v = *(const uint4*)(src + rowoff(r) + 8 * c);
    *(uint4*)(dst + r * LD + 8 * c) = v;
  }
}

// Same copy with compile-time extents, split into its two halves: load() issues every global
// load of the tile (rows beyond `valid` re-read the last valid row), store() writes the tile to
// LDS and zero-fills the missing rows.  A thread has all its loads in flight at once instead of
// one round trip per row, and other loads can be issued between the two calls.
template <int D, int ROWS, int NTHR>
struct RowRegs {
  static constexpr int CPR = D / 8, TOTAL = ROWS * CPR, N = (TOTAL + NTHR - 1) / NTHR;
  uint4 v[N];
  int valid;
  template <typename RowFn>
  __device__ inline void load(const u16* src, RowFn rowoff, int nvalid, int tid) {
    valid = nvalid;
    static_assert(NTHR % CPR == 0, "a thread keeps its column chunk from load to load");
    if constexpr (HasLinear<RowFn>::value) if (rowoff.linear()) {
      // thread t fetches chunk t % CPR of rows t / CPR + i * (NTHR / CPR): one multiply, then a
      // uniform increment per load; rows beyond the last valid one re-read it (clamped offset)
      const u16* base = src + rowoff.first() + 8 * (tid % CPR);
      const unsigned S = rowoff.step(), last = (unsigned)(nvalid - 1) * S, inc = (unsigned)(NTHR / CPR) * S;
      unsigned off = (unsigned)(tid / CPR) * S;
#pragma unroll
      for (int i = 0; i < N; ++i) {
        v[i] = *(const uint4*)(base + (off < last ? off : last));
        off += inc;
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int idx = tid + i * NTHR;
      idx = idx < TOTAL ? idx : TOTAL - 1;
      int r = idx / CPR;
      const int c = idx - r * CPR;
      r = r < nvalid ? r : nvalid - 1;
      v[i] = *(const uint4*)(src + rowoff(r) + 8 * c);
    }
  }
  template <int LD, bool SWZ = false>
  __device__ inline void store(u16* dst, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int idx = tid + i * NTHR;
      const int r = idx / CPR, c = idx - r * CPR;
      if (idx < TOTAL) *(uint4*)(dst + tile_off<LD, SWZ>(r, c)) = r < valid ? v[i] : uint4{0u, 0u, 0u, 0u};
    }
  }
  // Bottom-up: row r at dst - r * LD.
  template <int LD>
  __device__ inline void store_rev(u16* dst, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int idx = tid + i * NTHR;
      const int r = idx / CPR, c = idx - r * CPR;
      if (idx < TOTAL) *(uint4*)(dst - r * LD + 8 * c) = r < valid ? v[i] : uint4{0u, 0u, 0u, 0u};
    }
  }
};

template <int D, int LD, int ROWS, int NTHR, bool SWZ = false, typename RowFn>
__device__ inline void stage_rows_batched(u16* dst, const u16* src, RowFn rowoff, int valid, int tid) {
  RowRegs<D, ROWS, NTHR> r;
  r.load(src, rowoff, valid, tid);
  r.template store<LD, SWZ>(dst, tid);
}


}  // namespace
}  // namespace mrt
