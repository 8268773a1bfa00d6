// bf16 MFMA path for gfx950: bf16 operands, fp32 accumulation, fp32 softmax arithmetic.
//
// Every contraction runs on v_mfma_f32_16x16x32_bf16.  One wave owns 16 "query" rows and keeps
// them as the B operand (N side) of the logit product, so that a logit column -- everything
// the softmax of one query needs -- lives in one lane column (lane & 15) of the accumulators:
//
//   S^T[i, q] = sum_v Key[i, v] Qry[q, v]        A = Key rows from LDS, B = Qry rows in registers
//   lane (g = lane>>4, c = lane&15), register r of tile t holds S^T[16t + 4g + r, c]
//
// Row max / row sum are then in-lane reductions plus two cross-lane steps (xor 16, xor 32).
// The probabilities stay in registers: a lane's 8 values of two adjacent tiles are exactly the
// B operand of the second product once the contraction slots of group g are read as
// key = 32s + 16(e/4) + 4g + (e%4), e = 0..7:
//
//   Out^T[v, q] = sum_i Val^T[v, i] P^T[i, q]    A = Val read transposed from row-major LDS
//
// The A operand of that product needs, per lane, 8 different LDS rows of one column; gfx950's
// ds_read_b64_tr_b16 delivers exactly that from row-major tiles (lane c of a 16-lane group
// receives column c of the 4 rows addressed by the group), so no transposed copy is staged.
// Output rows of the second product are permuted (phi below) so that each lane ends up with 8
// consecutive features and stores 16 bytes.
//
// Stages (App. A.1 / A.2 update equations):
//   stage R      one workgroup per (m, n, k): Z_R, R = softmax_i, c_L, alpha_L = R K, Y = R V
//   stage L out  one workgroup per (m, j): flash loop over nk: L = softmax(Z_L), O = L Y
//   stage L ref  one workgroup per (m, j): alpha_R / c_R of the next iteration; one pass over the
//                logits for key ranges of at most 192 rows (row statistics exchanged between
//                the waves), else a log-sum-exp pass over nk followed by a second pass
#include "mrt_internal.hpp"
#include "mrt_bf16_tiles.hpp"

namespace mrt {

namespace {

// Optional timeline instrumentation (development builds only, -DMRT_TRACE): thread 0 of every
// workgroup stamps the 100 MHz wall clock at phase boundaries into a caller-provided buffer.
#ifdef MRT_TRACE
__device__ unsigned long long* g_trace_buf = nullptr;
#define MRT_STAMP(slot)                                                                          \
  do {                                                                                           \
    if (threadIdx.x == 0 && g_trace_buf) {                                                       \
      const size_t wg = ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;  \
      g_trace_buf[wg * 8 + (slot)] = wall_clock64();                                             \
      if ((slot) == 0) g_trace_buf[wg * 8 + 7] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | (31 << 11)) | ((unsigned long long)__builtin_amdgcn_s_getreg((20) | (0 << 6) | (31 << 11)) << 32); \
    }                                                                                            \
  } while (0)
#else
#define MRT_STAMP(slot) do { } while (0)
#endif

// ---------------------------------------------------------------------------------------
// stage R
// ---------------------------------------------------------------------------------------
// One workgroup = one key block (n, k) against a group of `gs` query tiles: the key (and value)
// rows are staged in LDS once and every query tile of the group that sees key tile n is then
// processed against them without further barriers (the next tile's query-side rows are
// prefetched while the current tile is computed).
// LDS of the last iteration's variant (keys and values resident): the value tile is stored
// bottom-up right after the keys, value row r at LDS row b2 + ROWS - 1 - r.  Rows b2 .. ROWS - 1
// of both tiles (zeros: the matrix tiles read 16 rows at a time) are then the same LDS rows, so the
// pair takes ROWS + b2 rows.  Row padding: 16 elements as everywhere (measured 0.3 us faster than 8
// at b2 = 52), 8 for five or six waves, where it lets a third workgroup onto the compute unit.
template <int NT> constexpr int kPadRV = NT >= 5 ? 8 : kPad;
template <int NT, int D>
inline size_t stage_r_last_lds_bytes(int b2) {
  return (size_t)(32 * ((NT + 1) / 2) + b2) * (D + kPadRV<NT>) * 2;
}

template <int NT, int D, bool FIRST, bool LAST>
__global__ __launch_bounds__(64 * NT, 4) void k_bf16_stage_r(KParams p, int gs) {
  constexpr int LD = D + (LAST ? kPadRV<NT> : kPad), KS1 = D / 32, KS2 = (NT + 1) / 2, ROWS = 32 * KS2, NVT = D / 16;
  constexpr int NTHR = 64 * NT;
  __shared__ __attribute__((aligned(16))) u16 Ks_static[LAST ? 8 : ROWS * LD];
  extern __shared__ __attribute__((aligned(16))) u16 r_lds[];     // LAST only
  u16* Ks = LAST ? r_lds : Ks_static;
  u16* Vtop = r_lds + (p.b2 + ROWS - 1) * LD;                     // value row 0

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  const int nk = blockIdx.x, bhl = blockIdx.z, bh = p.bh0 + bhl;
  const int n = nk / b1, k = nk - n * b1;
  const int an = n / p.c2, bn = n - an * p.c2;
  // query tiles [ml0, ml1) of this group; the hidden ones form a prefix (a later query chunk
  // sees more key tiles)
  int ml0 = blockIdx.y * gs;
  const int ml1 = ml0 + gs < p.ntq ? ml0 + gs : p.ntq;
  while (ml0 < ml1 && an >= visible_key_tile_rows((p.m0 + ml0) / p.c2, p.c1k, p.ct, p.qt0)) ++ml0;
  if (ml0 >= ml1) return;
  const int b = bh / p.H, hd = bh - b * p.H;

  // key block (n, k): block-grid row an*b1 + k, columns bn*b2 + i
  const long long krow = row_offset(p, an, k);
  const u16* Kp = (const u16*)p.K + b * p.ks.batch + hd * p.ks.head + krow * p.ks.token;
  const u16* Vp = (const u16*)p.V + b * p.vs.batch + hd * p.vs.head + krow * p.vs.token;
  const u16* Qbase = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head;
  const size_t NKtot = (size_t)p.ntk * b1;

  MRT_STAMP(0);
  // all loads of the block (keys, values, the first tile's query-side rows) are issued before
  // the first LDS store
  // (the register stages cover the 16 NT rows the waves own; with an odd NT the 32-row steps of the
  // second products read 16 rows more, zeros that no store touches: written once here)
  constexpr int SROWS = 16 * NT;
  RowRegs<D, SROWS, NTHR> rk;
  RowRegs<D, LAST ? SROWS : 1, NTHR> rv;
  rk.load(Kp, TokRows{0, p.cmap, bn * b2, p.ks.token}, b2, tid);
  if constexpr (ROWS > SROWS) {
    for (int idx = tid; idx < (ROWS - SROWS) * LD / 8; idx += NTHR)
      *(uint4*)(Ks + SROWS * LD + 8 * idx) = uint4{0u, 0u, 0u, 0u};
  }

  // query-side rows of this wave (row j = 16*wave + c) go straight to registers: Q[m, k, j, :] in
  // the first iteration (L is the identity), alpha_R / c_R afterwards
  const int j = 16 * wave + c;
  const int jc = j < b2 ? j : b2 - 1;
  bf16x8 qv[KS1], qn[KS1];
  auto load_q = [&](int ml) {
    const u16* arow;
    if (FIRST) {
      const int m = p.m0 + ml, a = m / p.c2, bq = m - a * p.c2;
      arow = Qbase + (row_offset(p, a, k) + axis_offset(p.cmap, bq * b2 + jc)) * p.qs.token;
    } else {
      arow = (const u16*)p.aR + ((((size_t)bhl * p.ntq + ml) * NKtot + nk) * b2 + jc) * D;
    }
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) qn[ks] = ld_global_16B(arow + 32 * ks + 8 * g);
  };
  load_q(ml0);
  if (LAST) rv.load(Vp, TokRows{0, p.cmap, bn * b2, p.vs.token}, b2, tid);
  rk.template store<LD>(Ks, tid);
  __syncthreads();
  MRT_STAMP(1);

  const float scale2 = p.scale * kLog2e;
  for (int ml = ml0; ml < ml1; ++ml) {
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) qv[ks] = qn[ks];
    if (ml + 1 < ml1) load_q(ml + 1);

    // Z_R^T tiles
    f32x4 s[NT];
#pragma unroll
    for (int it = 0; it < NT; ++it) {
      s[it] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks)
        s[it] = mfma(ld_lds_16B(Ks + (16 * it + c) * LD + 32 * ks + 8 * g), qv[ks], s[it]);
      if (it % 2 == 1) __builtin_amdgcn_sched_barrier(0);   // bound the operand reads in flight
    }
    __builtin_amdgcn_sched_barrier(0);
    // softmax over i (rows of the tiles) for column j, and sum_i R log R (base-2 domain inside)
    float mx = -INFINITY;
#pragma unroll
    for (int it = 0; it < NT; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool ok = 16 * it + 4 * g + r < b2;
        const float z = ok ? s[it][r] * scale2 : -INFINITY;
        s[it][r] = z;
        mx = fmaxf(mx, z);
      }
    mx = xmax(mx);
    float sum = 0.f, ent = 0.f;
#pragma unroll
    for (int it = 0; it < NT; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool ok = 16 * it + 4 * g + r < b2;
        const float z = ok ? s[it][r] - mx : 0.f;
        const float e = ok ? exp2_fast(z) : 0.f;
        sum += e;
        ent = fmaf(e, z, ent);
        s[it][r] = e;
      }
    sum = xsum(sum);
    ent = xsum(ent);
    const float inv = 1.0f / sum;
    const size_t row = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot + nk;
    if (g == 0 && j < b2) p.cL[row] = kLn2 * (ent * inv - log2_fast(sum));

    __builtin_amdgcn_sched_barrier(0);
    if (LAST && ml == ml0) {
      // the values, requested with the keys, were still arriving during the first tile's logits and
      // softmax; they are needed from here on
      rv.template store_rev<LD>(Vtop, tid);
      __syncthreads();
    }
    // alpha_L = R K (and Y = R V)
    bf16x8 pb[KS2];
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      const f32x4 lo = s[2 * st] * inv;
      const f32x4 hi = (2 * st + 1 < NT) ? s[(2 * st + 1 < NT) ? 2 * st + 1 : 0] * inv : zero;
      pb[st] = pack8(lo, hi);
    }
    if constexpr (!LAST) {
      f32x4 oK[NVT];
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) oK[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < KS2; ++st) {
        pv_step<D, LD>(Ks + 32 * st * LD, pb[st], oK, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (j < b2) store_rows<D>((u16*)p.aL + row * D, oK, 1.0f, g);
    } else {
      // both products, one half of the features at a time: the same interleaving of key-side and
      // value-side steps with half the live accumulators
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        f32x4 oK[NVT / 2], oV[NVT / 2];
#pragma unroll
        for (int vt = 0; vt < NVT / 2; ++vt) {
          oK[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
          oV[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int st = 0; st < KS2; ++st) {
          pv_step_half<D, LD>(Ks + 32 * st * LD, pb[st], oK, lane, h);
          pv_step_half<D, LD, -1>(Vtop - 32 * st * LD, pb[st], oV, lane, h);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (j < b2) {
          store_rows_half<D>((u16*)p.aL + row * D, oK, 1.0f, g, h);
          store_rows_half<D>((u16*)p.Y + row * D, oV, 1.0f, g, h);
        }
      }
    }
    if (ml == ml0) MRT_STAMP(2);
  }
  MRT_STAMP(3);
}

// ---------------------------------------------------------------------------------------
// flash loop shared by stage L (out), stage L (refine, pass 1) and the dense baseline
// ---------------------------------------------------------------------------------------
constexpr int kHK = 32;    // keys per pipeline step (one register set, one LDS slot)
constexpr int kRing = 4;   // LDS slots
// Row padding of the chunk slots (and of the streamed refine kernel's Q tile) is a template
// parameter PAD of the pieces below: 16 elements as elsewhere (8 measured 1 % slower at the
// KV-cache shapes, and so did unpadded rows with the resident kernels' XOR swizzle).

// Online softmax state of a wave's query tiles.  mrun is the reference the exponentials are taken
// against (the same in the four lanes that share a query): not the running maximum itself but a
// value within kGrow (base-2) of it, raised only when a chunk brings a logit more than kGrow above
// it.  Every probability is then at most 2^kGrow, the ratio sum(p v) / sum(p) does not depend on the
// reference, and the common case of a chunk is free of cross-lane reductions and of rescaling.
constexpr float kGrow = 8.0f;
template <int QT>
struct FlashState {
  float mrun[QT], lrun[QT];   // reference (see above), this lane's partial sum of 2^(z - mrun)
  __device__ inline FlashState() {
#pragma unroll
    for (int q = 0; q < QT; ++q) { mrun[q] = -INFINITY; lrun[q] = 0.f; }
  }
};

// One 32-row chunk of D bf16 held in registers between its global load and its LDS commit, so
// that its load is in flight while earlier chunks are being consumed.  NT = threads of the
// workgroup; the loads are unconditional: rows beyond the last valid one are copies of it (the
// consumer hides them through their bias), and when the pieces do not divide evenly over the
// threads the surplus loads of the last round re-read the last row and are not committed.
template <int D, int NT, int PAD = kPad>
struct ChunkRegs {
  static constexpr int CPR = D / 8, TOTAL = kHK * CPR, N = (TOTAL + NT - 1) / NT;
  static constexpr bool RAGGED = TOTAL % NT != 0;
  s16x8 v[N];
  // nvalid >= 1 rows exist at src.  STREAM: the rows are read once and by nobody else (non-temporal
  // loads: they do not displace what later kernels will look for in the caches)
  template <bool STREAM = false>
  __device__ inline void load(const u16* src, long long stride, int nvalid, int tid) {
    // thread t fetches piece t % CPR of rows t / CPR + i * (NT / CPR): a 32-bit offset from the
    // uniform chunk base, one multiply and then a uniform increment per load
    const u16* base = src + 8 * (tid % CPR);
    const unsigned S = (unsigned)stride, last = (unsigned)(nvalid - 1) * S, inc = (unsigned)(NT / CPR) * S;
    unsigned off = (unsigned)(tid / CPR) * S;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const s16x8* at = (const s16x8*)(base + (off < last ? off : last));
      v[i] = STREAM ? __builtin_nontemporal_load(at) : *at;
      off += inc;
    }
  }
  __device__ inline void commit(u16* dst, int tid) const {
    constexpr int LD = D + PAD;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int idx = tid + i * NT;
      const int r = idx / CPR, c = idx - r * CPR;
      if (!RAGGED || i + 1 < N || idx < TOTAL) *(s16x8*)(dst + r * LD + 8 * c) = v[i];
    }
  }
};

// One 32-key chunk against the wave's QT query tiles (16 queries each), in three stages that the
// streaming loop interleaves across chunks: the logits (MFMA), the online softmax update
// (vector ALU) and, when WITH_V, the rescale + accumulate of the output tiles (MFMA).  NQ, the
// number of tiles the wave owns (the first NQ of its QT), is a compile-time value: a chunk is
// then straight code in which the scheduler can overlap one stage's MFMAs with another's
// softmax arithmetic.
// Every key-side LDS operand is read once and used for all NQ query tiles.

// raw logits: s[q][t] = K tile t (16 keys) x Q tile q, summed over D
template <int D, int QT, int NQ, int PAD>
__device__ inline void flash_qk(const u16* Kc, const bf16x8 (&qv)[QT][D / 32], f32x4 (&s)[QT][2], int lane) {
  constexpr int LD = D + PAD, KS1 = D / 32;
  const int g = lane >> 4, c = lane & 15;
  // both key tiles' operand reads are issued before the first MFMA, and consecutive MFMAs
  // alternate between independent accumulators
  bf16x8 a[2][KS1];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks)
      a[t][ks] = ld_lds_16B(Kc + (16 * t + c) * LD + 32 * ks + 8 * g);
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int t = 0; t < 2; ++t) s[q][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t) s[q][t] = mfma(a[t][ks], qv[q][ks], s[q][t]);
}

// base-2 logits of the chunk in place of the raw products: z = scale * s + bias.  bias[i] is
// added to the scaled logit of key i (-inf for keys beyond the end); when MASKED,
// kchunk[i] > qchunk[q] hides key i from this lane's query of tile q.  Returns whether one of this
// lane's logits lies more than kGrow above its query's reference.
template <int QT, int NQ, bool MASKED>
__device__ inline bool flash_logits(f32x4 (&s)[QT][2], const float* bias, const int* kchunk,
                                    const int (&qchunk)[QT], float scale, const FlashState<QT>& st, int lane) {
  const int g = lane >> 4;
  f32x4 bi[2];
  int4 kc[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    bi[it] = *(const f32x4*)(bias + 16 * it + 4 * g);
    if (MASKED) kc[it] = *(const int4*)(kchunk + 16 * it + 4 * g);
  }
  bool grow = false;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    float zm = -INFINITY;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int kcs[4] = {MASKED ? kc[it].x : 0, MASKED ? kc[it].y : 0, MASKED ? kc[it].z : 0,
                          MASKED ? kc[it].w : 0};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float z = fmaf(s[q][it][r], scale, bi[it][r]);
        if (MASKED && kcs[r] > qchunk[q]) z = -INFINITY;
        s[q][it][r] = z;
        zm = fmaxf(zm, z);
      }
    }
    grow |= zm > st.mrun[q] + kGrow;    // also the first finite logit after mrun = -inf
  }
  return grow;
}

// The rare step: raise every query's reference to its running maximum (the old reference or the
// chunk's largest logit) and rescale its sum and, when WITH_V, its accumulators.
template <int D, int QT, int NQ, bool WITH_V>
__device__ inline void flash_grow(const f32x4 (&s)[QT][2], FlashState<QT>& st, f32x4 (&o)[QT][D / 16]) {
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    float zm = -INFINITY;
#pragma unroll
    for (int it = 0; it < 2; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r) zm = fmaxf(zm, s[q][it][r]);
    const float mnew = fmaxf(st.mrun[q], xmax(zm));
    // mnew == -inf only if every key so far is hidden from this query: the state stays empty
    const float alpha = mnew == -INFINITY ? 1.0f : exp2_fast(st.mrun[q] - mnew);   // mrun = -inf -> 0
    st.lrun[q] *= alpha;
    st.mrun[q] = mnew;
    if (WITH_V) {
#pragma unroll
      for (int vt = 0; vt < D / 16; ++vt) o[q][vt] = o[q][vt] * alpha;
    }
  }
}

// probabilities 2^(z - mrun) of the chunk: added to the running sums and, when WITH_V, packed
// to bf16 for the second product
template <int QT, int NQ, bool WITH_V, bool MASKED>
__device__ inline void flash_exp(f32x4 (&s)[QT][2], FlashState<QT>& st, bf16x8 (&pb)[QT]) {
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    // a reference of -inf (possible only when MASKED: every key so far hidden) gives 2^(-inf - 0) = 0
    const float m = (MASKED && st.mrun[q] == -INFINITY) ? 0.f : st.mrun[q];
    float ps = 0.f;
#pragma unroll
    for (int it = 0; it < 2; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float e = exp2_fast(s[q][it][r] - m);
        s[q][it][r] = e;
        ps += e;
      }
    st.lrun[q] += ps;
    if (WITH_V) pb[q] = pack8(s[q][0], s[q][1]);
  }
}

// o[q] += P[q] V
template <int D, int QT, int NQ, int PAD>
__device__ inline void flash_pv(const u16* Vc, const bf16x8 (&pb)[QT], f32x4 (&o)[QT][D / 16], int lane) {
  constexpr int LD = D + PAD, NVT = D / 16, HALF = NVT / 2;
  const int g = lane >> 4;
  const int sl = lane & 15, e = sl >> 2, qq = sl & 3;
  const u16* base = Vc + (4 * g + e) * LD + 8 * qq;
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
      const bf16x8 av =
          __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo[i], hi[i], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
      for (int q = 0; q < NQ; ++q) o[q][h * HALF + i] = mfma(av, pb[q], o[q][h * HALF + i]);
    }
  }
}

// LDS layout of the chunk pipeline: a ring of kRing slots of kHK rows each (contiguous, so that
// the ring is also one array of kRing * kHK rows)
template <int D, bool WITH_V, int PAD = kPad>
struct FlashLds {
  static constexpr int LD = D + PAD, ROWS = kRing * kHK;
  static constexpr size_t kBytes = (size_t)ROWS * LD * 2 * (WITH_V ? 2 : 1) + ROWS * 8;
  u16* k0;
  u16* v0;
  float* b0;
  int* c0;
  __device__ inline explicit FlashLds(unsigned char* base) {
    u16* p = (u16*)base;
    k0 = p; p += ROWS * LD;
    v0 = p; if (WITH_V) p += ROWS * LD;
    b0 = (float*)p;
    c0 = (int*)(b0 + ROWS);
  }
  __device__ inline u16* K(int slot) const { return k0 + slot * (kHK * LD); }
  __device__ inline u16* V(int slot) const { return v0 + slot * (kHK * LD); }
  __device__ inline float* bias(int slot) const { return b0 + slot * kHK; }
  __device__ inline int* kch(int slot) const { return c0 + slot * kHK; }
};

// One register set of the pipeline: a chunk of keys (and values) between its global load and its
// LDS commit.  meta(key) fetches the value whose negative is the key's bias, and the chunk id of
// the key.  Nothing here is conditional (a chunk beyond the end of the keys is fetched as copies
// of key 0 and committed with a bias of -inf): the pipeline below then runs as straight code in
// which the compiler's wait counts for one register set leave the other set's loads in flight.
template <int D, bool WITH_V, int NT, int PAD = kPad, bool STREAM = false>
struct ChunkFetch {
  ChunkRegs<D, NT, PAD> rk, rv;
  float rb;    // raw per-key value fetched by meta(); turned into the bias at commit time
  int rc, rvalid;
  template <typename Meta>
  __device__ inline void fetch(const u16* kbase, long long kstride, const u16* vbase,
                               long long vstride, int nkeys, int c0, Meta& meta, int tid) {
    const int left = nkeys - c0;                       // <= 0 beyond the end
    const int valid = left < kHK ? left : kHK;
    const int first = left > 0 ? c0 : 0, rows = valid > 0 ? valid : 1;
    rk.template load<STREAM>(kbase + (long long)first * kstride, kstride, rows, tid);
    if (WITH_V) rv.template load<STREAM>(vbase + (long long)first * vstride, vstride, rows, tid);
    rvalid = valid;
    const int k = tid & (kHK - 1);
    meta(first + (k < rows ? k : rows - 1), rb, rc);
  }
  template <bool MASKED>
  __device__ inline void commit(FlashLds<D, WITH_V, PAD>& lds, int slot, int tid) const {
    rk.commit(lds.K(slot), tid);
    if (WITH_V) rv.commit(lds.V(slot), tid);
    // every thread writes key (tid mod kHK)'s entry: the copies agree
    const int k = tid & (kHK - 1);
    lds.bias(slot)[k] = k < rvalid ? -rb * kLog2e : -INFINITY;
    if (MASKED) lds.kch(slot)[k] = rc;
  }
};

// The streaming loop: keys [0, nkeys) of a row-major key array (and value array), kHK at a time,
// through two register sets and a ring of four LDS slots, one barrier per pair of chunks.  While
// chunks c and c+1 are consumed, chunks c+2 and c+3 sit in (or are being written to) the other
// two slots and the loads of chunks c+4 and c+5 are in flight: each register set is committed
// one pair after its loads were issued and reloaded at once, so that a workgroup always has
// loads outstanding.  The slot a commit overwrites was last read in the previous pair, before
// that pair's barrier; the chunk it writes is first read after this pair's barrier.
// The loop body is one run of straight code (chunks are consumed in pairs, an odd last chunk is
// followed by an empty one) for a wave that owns NQ query tiles.
// NSET = 4 keeps four register sets in flight (two pairs ahead), for workgroups that have a compute
// unit to themselves and few registers per set (512 threads): with one workgroup per compute unit
// two chunks in flight do not cover the memory latency at the streaming rate.
template <int D, int QT, int NQ, bool WITH_V, bool MASKED, int NT, int NSET, int PAD, bool STREAM, typename Meta>
__device__ inline void flash_loop_n(const u16* kbase, long long kstride, const u16* vbase,
                                    long long vstride, int nkeys, Meta& meta, FlashLds<D, WITH_V, PAD>& lds,
                                    const bf16x8 (&qv)[QT][D / 32], float scale,
                                    const int (&qchunk)[QT], FlashState<QT>& st,
                                    f32x4 (&o)[QT][D / 16], int tid, int lane) {
  const int npairs = (nkeys + 2 * kHK - 1) / (2 * kHK);
  static_assert(NSET == 2 || NSET == 4, "two or four register sets");
  using Fetch = ChunkFetch<D, WITH_V, NT, PAD, STREAM>;
  Fetch fa, fb;
  auto fetch = [&](Fetch& f, int chunk) {
    f.fetch(kbase, kstride, vbase, vstride, nkeys, chunk * kHK, meta, tid);
  };
  // one pair of chunks (2 pr, 2 pr + 1); fx and fy hold the next pair's chunks, are committed and
  // then reloaded with the chunks NSET + 2 and NSET + 3 ahead
  auto pair = [&](int pr, Fetch& fx, Fetch& fy) {
    const int s0 = 2 * (pr & 1), s1 = s0 ^ 2;    // slots of this pair's chunks / of the next pair's
    // Stages of the two chunks in an order that leaves the scheduler independent work to put
    // under each other: the second chunk's first product next to the first chunk's exponentials,
    // the first chunk's second product next to the second chunk's logits.  Only the rare raise of
    // a reference branches.
    f32x4 sa[QT][2], sb[QT][2];
    bf16x8 pa[QT], pbb[QT];
    if (NQ > 0) {
      flash_qk<D, QT, NQ, PAD>(lds.K(s0), qv, sa, lane);
      const bool ga = flash_logits<QT, NQ, MASKED>(sa, lds.bias(s0), lds.kch(s0), qchunk, scale, st, lane);
      if (__builtin_amdgcn_ballot_w64(ga) != 0) flash_grow<D, QT, NQ, WITH_V>(sa, st, o);
      flash_qk<D, QT, NQ, PAD>(lds.K(s0 + 1), qv, sb, lane);
      flash_exp<QT, NQ, WITH_V, MASKED>(sa, st, pa);
      if (WITH_V) flash_pv<D, QT, NQ, PAD>(lds.V(s0), pa, o, lane);
      const bool gb = flash_logits<QT, NQ, MASKED>(sb, lds.bias(s0 + 1), lds.kch(s0 + 1), qchunk, scale, st, lane);
      if (__builtin_amdgcn_ballot_w64(gb) != 0) flash_grow<D, QT, NQ, WITH_V>(sb, st, o);
    }
    fx.template commit<MASKED>(lds, s1, tid);
    fetch(fx, 2 * pr + NSET + 2);
    if (NQ > 0) {
      flash_exp<QT, NQ, WITH_V, MASKED>(sb, st, pbb);
      if (WITH_V) flash_pv<D, QT, NQ, PAD>(lds.V(s0 + 1), pbb, o, lane);
    }
    fy.template commit<MASKED>(lds, s1 + 1, tid);
    fetch(fy, 2 * pr + NSET + 3);
    __syncthreads();
  };
  fetch(fa, 0);
  fetch(fb, 1);
  fa.template commit<MASKED>(lds, 0, tid);
  fetch(fa, 2);
  fb.template commit<MASKED>(lds, 1, tid);
  fetch(fb, 3);
  if (NSET == 2) {
    __syncthreads();
    for (int pr = 0; pr < npairs; ++pr) pair(pr, fa, fb);
  } else {
    Fetch fc, fd;
    fetch(fc, 4);
    fetch(fd, 5);
    __syncthreads();
    // (an odd number of pairs ends with an empty pair: its chunks lie beyond the keys)
    for (int pr = 0; pr < npairs; pr += 2) {
      pair(pr, fa, fb);
      pair(pr + 1, fc, fd);
    }
  }
}

// nq = query tiles the wave owns (uniform over the wave): QT, QT - 1 or none; every path runs
// the same fetches, commits and barriers.
template <int D, int QT, bool WITH_V, bool MASKED, int NT, int PAD = kPad, int NSET = 2, bool STREAM = false,
          typename Meta>
__device__ inline void flash_loop(const u16* kbase, long long kstride, const u16* vbase,
                                  long long vstride, int nkeys, Meta meta, FlashLds<D, WITH_V, PAD>& lds,
                                  const bf16x8 (&qv)[QT][D / 32], int nq, float scale,
                                  const int (&qchunk)[QT], FlashState<QT>& st,
                                  f32x4 (&o)[QT][D / 16], int tid, int lane) {
  if (nq == QT)
    flash_loop_n<D, QT, QT, WITH_V, MASKED, NT, NSET, PAD, STREAM>(kbase, kstride, vbase, vstride, nkeys, meta, lds, qv, scale,
                                                     qchunk, st, o, tid, lane);
  else if (QT > 1 && nq == QT - 1)
    flash_loop_n<D, QT, (QT > 1 ? QT - 1 : 0), WITH_V, MASKED, NT, NSET, PAD, STREAM>(kbase, kstride, vbase, vstride, nkeys, meta,
                                                                       lds, qv, scale, qchunk, st, o, tid, lane);
  else
    flash_loop_n<D, QT, 0, WITH_V, MASKED, NT, NSET, PAD, STREAM>(kbase, kstride, vbase, vstride, nkeys, meta, lds, qv, scale,
                                                    qchunk, st, o, tid, lane);
}

// Head of a stage L workgroup.  Stage R, which ran just before, worked through the heads in
// ascending order; stage L takes them in DESCENDING order, so that its first workgroups read what
// was written last and is still in the memory-side cache (and stage L's own results for head 0,
// written last, are what the next stage R reads first).  With intermediates of a few hundred MB
// per launch a forward order would find nothing of them left (KV-cache step at 480p, one head
// group: 498 -> 478 us per call).
__device__ inline int last_head_first() { return (int)gridDim.z - 1 - (int)blockIdx.z; }

// Query tiles of a wave: tile q of wave w is l tile (q * nwaves + w); nq of them exist.
template <int QT>
struct WaveTiles {
  int lt[QT];
  int nq;
  __device__ inline WaveTiles(int wave, int nwaves, int ntiles) {
    nq = 0;
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      lt[q] = q * nwaves + wave;
      if (lt[q] < ntiles) nq = q + 1;
    }
  }
};

// stage L, last iteration:  O[m, l, j, :] = sum_nk softmax_nk(scale * alpha_L Q - c_L) Y
// RMASK: regular Monarch under the chunk-causal mask (key rows of later chunks hidden per query row)
// STATS: also leaves every row's base-2 log-sum-exp and the unrounded output (p.lse_out, p.o32_out)
template <int D, int QT, int NT, bool RMASK, bool STATS = false>
__global__ __launch_bounds__(NT, NT == 512 ? 1 : 2) void k_bf16_stage_l_out(KParams p) {
  constexpr int KS1 = D / 32, NVT = D / 16;
  __shared__ __attribute__((aligned(16))) unsigned char smem[FlashLds<D, true>::kBytes];
  FlashLds<D, true> lds(smem);

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = last_head_first(), bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;
  const WaveTiles<QT> wt(wave, NT / 64, (b1 + 15) >> 4);

  const long long qtok0 = axis_offset(p.cmap, bq * b2 + j);   // column j of the tile; rows via qrow / orow
  const TokRows qrow = tile_rows(p, a, p.qs.token), orow = tile_rows(p, a, p.os.token);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qtok0 * p.qs.token;
  bf16x8 qv[QT][KS1];
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    const int l = 16 * wt.lt[q] + c;
    const int lc = l < b1 ? l : b1 - 1;
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks)
      qv[q][ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
  }

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const u16* aLp = (const u16*)p.aL + row0 * D;
  const u16* Yp = (const u16*)p.Y + row0 * D;
  const float* cLp = p.cL + row0;

  FlashState<QT> st;
  f32x4 o[QT][NVT];
  int qchunk[QT];
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    // chunk of this lane's query row (rows beyond b1 take the last row's; they are not stored)
    const int l = 16 * wt.lt[q] + c;
    qchunk[q] = RMASK ? ((l < b1 ? l : b1 - 1) + p.rq0) / p.rl : 0;
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) o[q][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  MRT_STAMP(0);
  auto meta = [&](int key, float& raw, int& chunk) { raw = cLp[key]; chunk = RMASK ? key / p.rl : 0; };
  flash_loop<D, QT, true, RMASK, NT, kPad, (NT == 512 ? 4 : 2), true>(aLp, D, Yp, D, NK, meta, lds, qv, wt.nq,
                                                                 p.scale * kLog2e, qchunk, st, o,
                                     tid, lane);
  MRT_STAMP(1);
  u16* Op = (u16*)p.O + b * p.os.batch + hd * p.os.head + qtok0 * p.os.token;
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    const int l = 16 * wt.lt[q] + c;
    const float lsum = xsum(st.lrun[q]);
    if (q < wt.nq && l < b1) store_rows_nt<D>(Op + orow(l), o[q], 1.0f / lsum, g);
  }
  if constexpr (STATS) {
    // for a backward call that follows: the rows' log-sum-exp and the unrounded output
    const size_t qr0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * b1;
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int l = 16 * wt.lt[q] + c;
      const float lsum = xsum(st.lrun[q]);
      if (q < wt.nq && l < b1) {
        float* row = p.o32_out + (qr0 + l) * D;
        const float inv = 1.0f / lsum;
#pragma unroll
        for (int h = 0; h < D / 32; ++h) {
          *(f32x4*)(row + 32 * h + 8 * g) = o[q][2 * h] * inv;
          *(f32x4*)(row + 32 * h + 8 * g + 4) = o[q][2 * h + 1] * inv;
        }
        if (g == 0) p.lse_out[qr0 + l] = st.mrun[q] + log2_fast(lsum);
      }
    }
  }
  MRT_STAMP(2);
}

// Pass 2 of the refine stage for one (m, j): waves stride over groups of PT adjacent 16-wide nk
// tiles (every LDS read of Q serves all PT tiles).  Qs holds Q[m, :, j, :] row-major (rows >= b1
// zero), lse the base-2 log-sum-exp of every row l.  alpha_L[m, j] and c_L are read from global
// memory (the cache: pass 1 has just streamed them), with the next group's operands in flight
// while the current one is processed.  The result
//   alpha_R[m, nk, j, :] / c_R[m, nk, j] = sum_l w Q[m, l, j, :] / sum_l w,   w = L[l, nk] = 2^z,
// is stored as the next iteration's abar rows.  It is computed one PAIR of l tiles at a time: the
// weights are L[l, nk] itself (no maximum is taken out), so a pair's logits can be turned into
// weights, summed and contracted with its 32 rows of Q at once, and only two tiles of logits per
// key tile are ever live.  A key whose whole column underflows in fp32 (sum of weights 0) is redone
// with the column maximum taken out first (the ratio is unchanged by it).
template <int D, int NLT, int PT, int LD>
__device__ inline void refine_pass2(const KParams& p, const u16* Qs, const float* lse, const u16* aLp,
                                          const float* cLp, u16* aRout, int NK, int j, int wave,
                                          int nwaves, int lane) {
  constexpr int KS1 = D / 32, NVT = D / 16, NP = (NLT + 1) / 2;
  const int g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  const float scale2 = p.scale * kLog2e;
  const int ntiles = (NK + 15) >> 4;
  const int ngroups = (ntiles + PT - 1) / PT;
  bf16x8 kb[PT][KS1], kbn[PT][KS1];
  float cl[PT], cln[PT];
  auto fetch = [&](int grp, bf16x8 (&dst)[PT][KS1], float (&cdst)[PT]) {
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
      const int nk = 16 * (PT * grp + pt) + c;
      const int nkc = nk < NK ? nk : NK - 1;
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks)
        dst[pt][ks] = ld_global_16B(aLp + (size_t)nkc * D + 32 * ks + 8 * g);
      cdst[pt] = cLp[nkc];
    }
  };
  // the groups are taken from the END of the key range backwards: pass 1 has just streamed the
  // range front to back, so its tail is what the caches still hold
  if (wave < ngroups) fetch(ngroups - 1 - wave, kbn, cln);
  for (int grp = ngroups - 1 - wave; grp >= 0; grp -= nwaves) {
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks) kb[pt][ks] = kbn[pt][ks];
      cl[pt] = cln[pt] * kLog2e;    // c_L in the base-2 domain
    }
    if (grp - nwaves >= 0) fetch(grp - nwaves, kbn, cln);
    const int npt = ntiles - PT * grp < PT ? ntiles - PT * grp : PT;   // tiles of this group

    // log2 L[l, nk] of l tile lt for the group's key tiles (rows beyond b1: -inf)
    auto logits = [&](int lt, f32x4 (&z)[PT]) {
      bf16x8 av[KS1];
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks) av[ks] = ld_lds_16B(Qs + (16 * lt + c) * LD + 32 * ks + 8 * g);
      const f32x4 ls = *(const f32x4*)(lse + 16 * lt + 4 * g);
#pragma unroll
      for (int pt = 0; pt < PT; ++pt) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) acc = mfma(av[ks], kb[pt][ks], acc);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const bool ok = 16 * lt + 4 * g + r < b1;
          acc[r] = ok ? fmaf(acc[r], scale2, -cl[pt]) - ls[r] : -INFINITY;
        }
        z[pt] = acc;
      }
    };
    float csum[PT], shift[PT];
    f32x4 o[PT][NVT];
    // pairs in a software pipeline: the next pair's logits (MFMA) are issued ahead of this pair's
    // exponentials (vector ALU), so that the matrix unit works under them
    auto pair_logits = [&](int pr, f32x4 (&zlo)[PT], f32x4 (&zhi)[PT]) {
      logits(2 * pr, zlo);
      if (2 * pr + 1 < NLT) logits(2 * pr + 1, zhi);
    };
    auto run = [&]() {
#pragma unroll
      for (int pt = 0; pt < PT; ++pt) {
        csum[pt] = 0.f;
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) o[pt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      f32x4 zlo[PT], zhi[PT], nlo[PT], nhi[PT];
      pair_logits(0, zlo, zhi);
#pragma unroll
      for (int pr = 0; pr < NP; ++pr) {
        if (pr + 1 < NP) pair_logits(pr + 1, nlo, nhi);
        bf16x8 pb[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
          f32x4 lo, hi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            lo[r] = exp2_fast(zlo[pt][r] - shift[pt]);
            csum[pt] += lo[r];
            if (2 * pr + 1 < NLT) {
              hi[r] = exp2_fast(zhi[pt][r] - shift[pt]);
              csum[pt] += hi[r];
            }
          }
          pb[pt] = pack8(lo, hi);
        }
        pv_step_multi<D, PT, LD>(Qs + 32 * pr * LD, pb, PT, o, lane);
        // keep the scheduler from hoisting every pair's operand reads to the top (register blow-up)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) { zlo[pt] = nlo[pt]; zhi[pt] = nhi[pt]; }
      }
#pragma unroll
      for (int pt = 0; pt < PT; ++pt) csum[pt] = xsum(csum[pt]);
    };
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) shift[pt] = 0.f;
    run();
    bool under = false;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) under |= (pt < npt && csum[pt] == 0.f);
    if (__builtin_expect(__any(under), 0)) {
      float cm[PT];
#pragma unroll
      for (int pt = 0; pt < PT; ++pt) cm[pt] = -INFINITY;
      for (int lt = 0; lt < NLT; ++lt) {
        f32x4 z[PT];
        logits(lt, z);
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
          for (int r = 0; r < 4; ++r) cm[pt] = fmaxf(cm[pt], z[pt][r]);
      }
#pragma unroll
      for (int pt = 0; pt < PT; ++pt) shift[pt] = xmax(cm[pt]);
      run();
    }
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
      const int nk = 16 * (PT * grp + pt) + c;
      if (pt < npt && nk < NK) {
        store_rows<D>(aRout + ((size_t)nk * b2 + j) * D, o[pt], 1.0f / csum[pt], g);
        // the backward pass rebuilds the weights as exp(log L - cmx) * cinv
        if (p.cmx_out != nullptr && g == 0) {
          const size_t at = (size_t)(aRout - (u16*)p.aR) / D + (size_t)nk * b2 + j;
          p.cmx_out[at] = shift[pt] * kLn2;
          p.cinv_out[at] = 1.0f / csum[pt];
        }
      }
    }
  }
}

// stage L, earlier iterations:
//   alpha_R[m, nk, j, :] / c_R[m, nk, j] = sum_l L[l, nk] Q[m, l, j, :] / sum_l L[l, nk]
// with L = softmax_nk(Z_L).  Pass 1 finds the log-sum-exp of every row l (flash loop without
// values); pass 2 recomputes Z_L one 16-wide nk tile per wave with l on the M side, forms
// softmax over l of log L[l, nk] (the same ratio, safe against underflow) and contracts with Q
// read transposed from LDS.
constexpr int kMaxLT = 12;   // l tiles of 16 (b1 <= 192)
constexpr int kRefineHead = 16 * kMaxLT * 4;   // bytes of LDS ahead of the shared region

// NLT = number of 16-row l tiles (compile time, so that the tile loops unroll without guards and
// the scheduler can overlap one tile's LDS reads with another's MFMAs).
template <int D, int QT, int MAXT, int NLT, int PT, int PAD>
__global__ __launch_bounds__(MAXT, 2) void k_bf16_stage_l_refine(KParams p) {
  constexpr int LD = D + PAD, KS1 = D / 32, NVT = D / 16;
  // LDS: the row log-sum-exps, then one region that holds the chunk ring during pass 1 and the
  // Q tile during pass 2 (pass 1 takes its Q operands straight from global memory)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* lse = (float*)smem;                             // [16 * kMaxLT]
  FlashLds<D, false, PAD> lds(smem + kRefineHead);
  u16* Qs = (u16*)(smem + kRefineHead);                  // [32 * ceil(NLT / 2)][LD], rows >= b1 zero

  constexpr int nwaves = MAXT / 64;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  constexpr int nlt = NLT;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = last_head_first(), bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;

  const long long qtok0 = axis_offset(p.cmap, bq * b2 + j);   // column j of the tile; rows via qrow
  const TokRows qrow = tile_rows(p, a, p.qs.token);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qtok0 * p.qs.token;
  MRT_STAMP(0);

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const u16* aLp = (const u16*)p.aL + row0 * D;
  const float* cLp = p.cL + row0;

  // ---- pass 1
  {
    const WaveTiles<QT> wt(wave, nwaves, nlt);
    bf16x8 qv[QT][KS1];
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int l = 16 * wt.lt[q] + c;
      const int lc = l < b1 ? l : b1 - 1;
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks)
        qv[q][ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
    }
    FlashState<QT> st;
    f32x4 odummy[QT][NVT];
    int qchunk[QT];
#pragma unroll
    for (int q = 0; q < QT; ++q) qchunk[q] = 0;
    auto meta = [&](int key, float& raw, int& chunk) { raw = cLp[key]; chunk = 0; };
    flash_loop<D, QT, false, false, MAXT, PAD>(aLp, D, nullptr, 0, NK, meta, lds, qv, wt.nq, p.scale * kLog2e,
                                               qchunk, st, odummy, tid, lane);
    MRT_STAMP(1);
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const float lsum = xsum(st.lrun[q]);
      if (q < wt.nq && g == 0) lse[16 * wt.lt[q] + c] = st.mrun[q] + log2_fast(lsum);   // base 2
    }
  }
  __syncthreads();                 // every wave is done with the chunk ring
  stage_rows_batched<D, LD, 32 * ((NLT + 1) / 2), MAXT>(Qs, Qp, qrow, b1, tid);
  __syncthreads();
  MRT_STAMP(2);

  // ---- pass 2 (alpha_L[m, j] is streamed again, from the cache)
  u16* aRout = (u16*)p.aR + ((size_t)bhl * p.ntq + ml) * NKtot * b2 * D;
  refine_pass2<D, NLT, PT, LD>(p, Qs, lse, aLp, cLp, aRout, NK, j, wave, nwaves, lane);
  MRT_STAMP(6);
}

// ---------------------------------------------------------------------------------------
// stage L for short key ranges (NK <= 96: regular Monarch with b1 <= 96, or one small visible
// tile).  Everything a workgroup needs is loaded once, so there is one memory round trip, an exact
// (not online) softmax, and the footprint (52 KB of LDS, <= 168 registers) lets three workgroups
// share a compute unit: the 52*heads workgroups of the 4680-token chunk run in a single round.
// ---------------------------------------------------------------------------------------
constexpr int kResRows = 96;    // key rows held resident
constexpr int kResPad = 8;      // row padding of the resident tiles of 64 features (128: swizzled, no padding)
// layout of a resident tile: swizzled rows for 128 features, padded rows for 64
template <int D> struct ResTile {
  static constexpr bool SWZ = D == 128;
  static constexpr int LD = SWZ ? D : D + kResPad;
};

// Exact softmax of QT query tiles (nq of them live) against NTK resident key tiles; every key
// operand read from LDS serves all QT tiles.  On return s holds the exponentials (base-2 logits
// minus the column maximum) and sum their column sums.
// RMASK (regular Monarch under the chunk-causal mask): the lane's query row of tile q sees the keys
// below klim[q].
template <int D, int NTK, int LD, bool SWZ, int QT, bool RMASK>
__device__ inline void res_logits(const u16* Ks, const float* bias, const bf16x8 (&qv)[QT][D / 32],
                                  int nq, float scale2, const int (&klim)[QT], f32x4 (&s)[QT][NTK],
                                  float (&sum)[QT], int lane) {
  constexpr int KS1 = D / 32;
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int q = 0; q < QT; ++q)
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt) s[q][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kp = 0; kp < (NTK + 1) / 2; ++kp) {
    bf16x8 a[2][KS1];
#pragma unroll
    for (int t = 0; t < 2; ++t)
      if (2 * kp + t < NTK) {
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks)
          a[t][ks] = ld_lds_16B(Ks + tile_off<LD, SWZ>(16 * (2 * kp + t) + c, 4 * ks + g));
      }
#pragma unroll
    for (int q = 0; q < QT; ++q)
      if (q < nq) {
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
          for (int t = 0; t < 2; ++t)
            if (2 * kp + t < NTK) s[q][2 * kp + t] = mfma(a[t][ks], qv[q][ks], s[q][2 * kp + t]);
      }
    __builtin_amdgcn_sched_barrier(0);   // one pair of key tiles in flight at a time
  }
  f32x4 bi[NTK];
#pragma unroll
  for (int kt = 0; kt < NTK; ++kt) bi[kt] = *(const f32x4*)(bias + 16 * kt + 4 * g);
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[q][kt][r] = fmaf(s[q][kt][r], scale2, bi[kt][r]);      // -inf beyond the last key
        if (RMASK && 16 * kt + 4 * g + r >= klim[q]) s[q][kt][r] = -INFINITY;
        mx = fmaxf(mx, s[q][kt][r]);
      }
    mx = xmax(mx);
    float sm = 0.f;
#pragma unroll
    for (int kt = 0; kt < NTK; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[q][kt][r] = exp2_fast(s[q][kt][r] - mx);
        sm += s[q][kt][r];
      }
    sum[q] = xsum(sm);
  }
}

template <int D, int NTK, bool RMASK>
__global__ __launch_bounds__(256, 3) void k_bf16_stage_l_out_res(KParams p) {
  constexpr int LD = ResTile<D>::LD, KS1 = D / 32, NVT = D / 16, KS2 = (NTK + 1) / 2, ROWS = 32 * KS2;
  constexpr bool SWZ = ResTile<D>::SWZ;
  constexpr int QT = 2;
  __shared__ __attribute__((aligned(16))) u16 Ks[ROWS * LD];
  __shared__ __attribute__((aligned(16))) u16 Vs[ROWS * LD];
  __shared__ __attribute__((aligned(16))) float bias[ROWS];

  const int tid = threadIdx.x, nthr = blockDim.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
  const int lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = last_head_first(), bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;   // <= 16*NTK
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;
  const int nlt = (b1 + 15) >> 4;

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const u16* aLp = (const u16*)p.aL + row0 * D;
  const u16* Yp = (const u16*)p.Y + row0 * D;
  const float* cLp = p.cL + row0;
  const long long qtok0 = axis_offset(p.cmap, bq * b2 + j);   // column j of the tile; rows via qrow / orow
  const TokRows qrow = tile_rows(p, a, p.qs.token);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qtok0 * p.qs.token;
  u16* Op = (u16*)p.O + b * p.os.batch + hd * p.os.head + qtok0 * p.os.token;

  MRT_STAMP(0);
  // this wave's query tiles (2*wave, 2*wave+1) go to registers while the key side goes to LDS
  bf16x8 qv[QT][KS1];
  auto load_q = [&](int pair) {
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int l = 16 * (QT * pair + q) + c;
      const int lc = l < b1 ? l : b1 - 1;
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks)
        qv[q][ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
    }
  };
  const int npairs = (nlt + QT - 1) / QT;      // <= 3 (b1 <= 96): at most one pair per wave
  // every global load of the workgroup is issued before the first LDS store: one memory round
  // trip instead of one per tile.  The loads return in order: alpha_L, c_L and the query rows, which
  // the logits need, are requested first; the values follow and are still arriving while the
  // logits and the softmax are formed (they are committed to LDS only before the second product).
  RowRegs<D, ROWS, 256> rk, rv;
  rk.load(aLp, PlainRows{D}, NK, tid);
  static_assert(ROWS <= 256, "one bias value per thread");
  const float cl = cLp[tid < NK ? tid : NK - 1];
  if (wave < npairs) load_q(wave);
  rv.load(Yp, PlainRows{D}, NK, tid);
  rk.template store<LD, SWZ>(Ks, tid);
  if (tid < ROWS) bias[tid] = tid < NK ? -cl * kLog2e : -INFINITY;
  __syncthreads();
  MRT_STAMP(1);

  const float scale2 = p.scale * kLog2e;
  const int pair = wave;
  const int nq = pair < npairs ? (nlt - QT * pair < QT ? nlt - QT * pair : QT) : 0;
  bf16x8 pb[KS2][QT];
  float sum[QT];
  if (nq > 0) {
    f32x4 s[QT][NTK];
    int klim[QT];
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int l = 16 * (QT * pair + q) + c;
      klim[q] = RMASK ? visible_key_rows(p, l < b1 ? l : b1 - 1) : 0;
    }
    res_logits<D, NTK, LD, SWZ, QT, RMASK>(Ks, bias, qv, nq, scale2, klim, s, sum, lane);
#pragma unroll
    for (int q = 0; q < QT; ++q)
#pragma unroll
      for (int st = 0; st < KS2; ++st) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        const f32x4 hi = (2 * st + 1 < NTK) ? s[q][(2 * st + 1 < NTK) ? 2 * st + 1 : 0] : zero;
        pb[st][q] = pack8(s[q][2 * st], hi);
      }
  }
  __builtin_amdgcn_sched_barrier(0);
  rv.template store<LD, SWZ>(Vs, tid);
  __syncthreads();
  MRT_STAMP(2);
  if (nq > 0) {
    f32x4 o[QT][NVT];
#pragma unroll
    for (int q = 0; q < QT; ++q)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) o[q][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      pv_step_multi<D, QT, LD, SWZ>(Vs + 32 * st * LD, pb[st], nq, o, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
    const TokRows orow = tile_rows(p, a, p.os.token);
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int l = 16 * (QT * pair + q) + c;
      if (q < nq && l < b1) store_rows_nt<D>(Op + orow(l), o[q], 1.0f / sum[q], g);
    }
  }
  MRT_STAMP(3);
}

// Stage L of an earlier iteration for key ranges of at most 64 PT rows, in one pass over the
// logits: wave w owns key tiles PT w .. PT w + PT - 1 and forms their logits against every query
// tile once, with queries on the accumulator rows.  The row statistics of the joint softmax over
// the key range are reduced inside the wave and exchanged between the NW waves through LDS;
// alpha_L goes from global memory straight into the matrix operands, only Q is staged.
template <int D, int NLT, int PT, int NW, bool RMASK>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 2) void k_bf16_stage_l_refine_one(KParams p) {
  constexpr int LD = ResTile<D>::LD, KS1 = D / 32, QROWS = 32 * ((NLT + 1) / 2), LROWS = 16 * NLT;
  constexpr bool SWZ = ResTile<D>::SWZ;
  __shared__ __attribute__((aligned(16))) u16 Qs[QROWS * LD];
  __shared__ __attribute__((aligned(16))) float red_m[NW][LROWS];
  __shared__ __attribute__((aligned(16))) float red_s[NW][LROWS];
  __shared__ __attribute__((aligned(16))) float lse[LROWS];
  __shared__ int redo;

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = last_head_first(), bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;   // <= 64 * PT
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;

  const long long qtok0 = axis_offset(p.cmap, bq * b2 + j);
  const TokRows qrow = tile_rows(p, a, p.qs.token);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qtok0 * p.qs.token;
  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const u16* aLp = (const u16*)p.aL + row0 * D;
  const float* cLp = p.cL + row0;

  MRT_STAMP(0);
  const int tile0 = PT * wave;
  const int ntiles = (NK + 15) >> 4;
  const int npt = ntiles - tile0 < PT ? (ntiles - tile0 > 0 ? ntiles - tile0 : 0) : PT;
  RowRegs<D, QROWS, 64 * NW> rq;
  rq.load(Qp, qrow, b1, tid);
  bf16x8 kb[PT][KS1];
  float cl[PT];
#pragma unroll
  for (int pt = 0; pt < PT; ++pt) {
    const int nk = 16 * (tile0 + pt) + c;
    const int nkc = nk < NK ? nk : NK - 1;
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) kb[pt][ks] = ld_global_16B(aLp + (size_t)nkc * D + 32 * ks + 8 * g);
    cl[pt] = cLp[nkc] * kLog2e;
  }
  rq.template store<LD, SWZ>(Qs, tid);
  __syncthreads();
  MRT_STAMP(1);

  // logits in the base-2 domain: rows 4g + r are queries, column c is key 16 (tile0 + pt) + c
  // (a lambda: the two rare underflow paths below form them a second time)
  const float scale2 = p.scale * kLog2e;
  f32x4 z[PT][NLT];
  auto logits = [&]() {
#pragma unroll
    for (int lt = 0; lt < NLT; ++lt) {
      bf16x8 av[KS1];
#pragma unroll
      for (int ks = 0; ks < KS1; ++ks) av[ks] = ld_lds_16B(Qs + tile_off<LD, SWZ>(16 * lt + c, 4 * ks + g));
#pragma unroll
      for (int pt = 0; pt < PT; ++pt) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (pt < npt) {
#pragma unroll
          for (int ks = 0; ks < KS1; ++ks) acc = mfma(av[ks], kb[pt][ks], acc);
        }
        const bool col = 16 * (tile0 + pt) + c < NK;
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = col ? fmaf(acc[r], scale2, -cl[pt]) : -INFINITY;
        z[pt][lt] = acc;
      }
      if (lt % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (RMASK) {
      // regular Monarch under the chunk-causal mask: key rows of later chunks are zeros of L
#pragma unroll
      for (int lt = 0; lt < NLT; ++lt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int lim = visible_key_rows(p, 16 * lt + 4 * g + r);
#pragma unroll
          for (int pt = 0; pt < PT; ++pt)
            if (16 * (tile0 + pt) + c >= lim) z[pt][lt][r] = -INFINITY;
        }
    }
  };
  logits();
  // This wave's share of every query row's sum of 2^z, relative to a reference the waves then
  // reconcile; the exponentials e = 2^(z - reference) are kept in place of the logits, and a weight
  // is L = 2^(z - lse) = e * 2^(reference - M) / S with M the largest reference of the row and S
  // the row's total relative to it: one exponential per logit.  First with one reference per query
  // tile (the maximum over the tile's 16 rows: six cross-lane steps per tile instead of four per
  // row).  A row whose largest logit lies far below its tile's maximum would lose weights to
  // underflow (e is flushed below 2^-126), so if any row's total comes out below 2^-64 the logits
  // are formed again and the statistics redone with every row's own maximum; with S >= 2^-64 a
  // flushed e stands for a weight below 2^-62.
  auto stats = [&](bool per_row) {
#pragma unroll
    for (int lt = 0; lt < NLT; ++lt) {
      f32x4 vr;
      float vt = -INFINITY;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = z[0][lt][r];
#pragma unroll
        for (int pt = 1; pt < PT; ++pt) v = fmaxf(v, z[pt][lt][r]);
        vr[r] = v;
        vt = fmaxf(vt, v);
      }
      if (per_row) {
#pragma unroll
        for (int r = 0; r < 4; ++r) vr[r] = row16_max(vr[r]);
      } else {
        vt = xmax(row16_max(vt));
#pragma unroll
        for (int r = 0; r < 4; ++r) vr[r] = vt;
      }
      f32x4 sm;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float ref = vr[r] == -INFINITY ? 0.f : vr[r];
        float e = 0.f;
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
          z[pt][lt][r] = exp2_fast(z[pt][lt][r] - ref);
          e += z[pt][lt][r];
        }
        sm[r] = row16_sum(e);
      }
      if (c == 0) {
        *(f32x4*)(&red_m[wave][16 * lt + 4 * g]) = vr;
        *(f32x4*)(&red_s[wave][16 * lt + 4 * g]) = sm;
      }
    }
  };
  // per row: log-sum-exp (base 2) and, in place of every wave's partial sum, the factor that turns
  // that wave's exponentials into weights (zero for the padding rows beyond b1)
  auto combine = [&]() {
    if (tid < LROWS) {
      float M = red_m[0][tid];
#pragma unroll
      for (int w = 1; w < NW; ++w) M = fmaxf(M, red_m[w][tid]);
      const float Ms = M == -INFINITY ? 0.f : M;
      float f[NW], S = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        f[w] = exp2_fast(red_m[w][tid] - Ms);
        S = fmaf(red_s[w][tid], f[w], S);
      }
      lse[tid] = Ms + log2_fast(S);
      const float inv = tid < b1 ? 1.0f / S : 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) red_s[w][tid] = f[w] * inv;
      if (!(S > 0x1p-64f) && tid < b1) redo = 1;
    }
  };
  if (tid == 0) redo = 0;
  stats(false);
  __syncthreads();
  combine();
  __syncthreads();
  if (__builtin_expect(redo, 0)) {            // uniform: read after the barrier
    logits();
    stats(true);
    __syncthreads();
    combine();
    __syncthreads();
  }
  MRT_STAMP(2);
  // weights L[l, nk] as packed bf16 operands, and their column sums c_R
  constexpr int NVT = D / 16, NS2 = (NLT + 1) / 2;
  float csum[PT];
  bf16x8 pb[NS2][PT];
#pragma unroll
  for (int pt = 0; pt < PT; ++pt) csum[pt] = 0.f;
#pragma unroll
  for (int st2 = 0; st2 < NS2; ++st2) {
    const f32x4 f0 = *(const f32x4*)(&red_s[wave][32 * st2 + 4 * g]);
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const f32x4 f1 = 2 * st2 + 1 < NLT ? *(const f32x4*)(&red_s[wave][32 * st2 + 16 + 4 * g]) : zero;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
      const f32x4 lo = z[pt][2 * st2] * f0;
      const f32x4 hi = 2 * st2 + 1 < NLT ? z[pt][2 * st2 + 1 < NLT ? 2 * st2 + 1 : 0] * f1 : zero;
      csum[pt] += (lo[0] + lo[1]) + (lo[2] + lo[3]) + (hi[0] + hi[1]) + (hi[2] + hi[3]);
      pb[st2][pt] = pack8(lo, hi);
    }
  }
  bool under = false;
#pragma unroll
  for (int pt = 0; pt < PT; ++pt) {
    csum[pt] = xsum(csum[pt]);
    under |= (pt < npt && 16 * (tile0 + pt) + c < NK && csum[pt] == 0.f);
  }
  float shift[PT];
#pragma unroll
  for (int pt = 0; pt < PT; ++pt) shift[pt] = 0.f;
  if (__builtin_expect(__any(under), 0)) {
    // a whole column of weights underflowed: the ratio alpha_R / c_R is formed from log2 L relative
    // to the column's maximum instead (logits formed again; rare)
    logits();
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
      float cm = -INFINITY;
#pragma unroll
      for (int lt = 0; lt < NLT; ++lt) {
        const f32x4 ls = *(const f32x4*)(lse + 16 * lt + 4 * g);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          z[pt][lt][r] = 16 * lt + 4 * g + r < b1 ? z[pt][lt][r] - ls[r] : -INFINITY;
          cm = fmaxf(cm, z[pt][lt][r]);
        }
      }
      cm = xmax(cm);
      shift[pt] = cm == -INFINITY ? 0.f : cm;
      csum[pt] = 0.f;
#pragma unroll
      for (int st2 = 0; st2 < NS2; ++st2) {
        f32x4 lo, hi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          lo[r] = exp2_fast(z[pt][2 * st2][r] - shift[pt]);
          csum[pt] += lo[r];
          if (2 * st2 + 1 < NLT) {
            hi[r] = exp2_fast(z[pt][2 * st2 + 1 < NLT ? 2 * st2 + 1 : 0][r] - shift[pt]);
            csum[pt] += hi[r];
          }
        }
        pb[st2][pt] = pack8(lo, hi);
      }
      csum[pt] = xsum(csum[pt]);
    }
  }
  MRT_STAMP(4);
  u16* aRout = (u16*)p.aR + ((size_t)bhl * p.ntq + ml) * NKtot * b2 * D;
  if (npt > 0) {
    f32x4 o[PT][NVT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) o[pt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st2 = 0; st2 < NS2; ++st2) {
      pv_step_multi<D, PT, LD, SWZ>(Qs + 32 * st2 * LD, pb[st2], npt, o, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
    MRT_STAMP(5);
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
      const int nk = 16 * (tile0 + pt) + c;
      if (pt < npt && nk < NK) {
        store_rows<D>(aRout + ((size_t)nk * b2 + j) * D, o[pt], 1.0f / csum[pt], g);
        // the backward pass rebuilds the weights as exp(log L - cmx) * cinv
        if (p.cmx_out != nullptr && g == 0) {
          const size_t at = (size_t)(aRout - (u16*)p.aR) / D + (size_t)nk * b2 + j;
          p.cmx_out[at] = shift[pt] * kLn2;
          p.cinv_out[at] = 1.0f / csum[pt];
        }
      }
    }
  }
  MRT_STAMP(6);
}

// dense baseline: 128 queries per workgroup (4 waves x 2 tiles of 16), flash loop over all
// visible keys
constexpr int kDenseQT = 2, kDenseQ = 64 * kDenseQT;

template <int D>
__global__ __launch_bounds__(256, 2) void k_bf16_dense(KParams p) {
  constexpr int KS1 = D / 32, NVT = D / 16, QT = kDenseQT;
  __shared__ __attribute__((aligned(16))) unsigned char smem[FlashLds<D, true>::kBytes];
  FlashLds<D, true> lds(smem);
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int q0 = blockIdx.x * kDenseQ, bh = blockIdx.y;
  const int b = bh / p.H, hd = bh - b * p.H;
  const int qtiles = (p.Nq - q0 + 15) >> 4;
  const WaveTiles<QT> wt(wave, 4, qtiles < 4 * QT ? qtiles : 4 * QT);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head;
  bf16x8 qv[QT][KS1];
  int qchunk[QT];
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    const int qi = q0 + 16 * wt.lt[q] + c;
    const int qc = qi < p.Nq ? qi : p.Nq - 1;
    qchunk[q] = p.cc > 0 ? (p.qoff + qc / p.hw) / p.cc : 0x7fffffff;
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks)
      qv[q][ks] = ld_global_16B(Qp + (long long)qc * p.qs.token + 32 * ks + 8 * g);
  }
  const u16* Kp = (const u16*)p.K + b * p.ks.batch + hd * p.ks.head;
  const u16* Vp = (const u16*)p.V + b * p.vs.batch + hd * p.vs.head;
  int nkeys = p.Nkv;
  if (p.cc > 0) {
    const int qlast = (q0 + kDenseQ - 1 < p.Nq ? q0 + kDenseQ - 1 : p.Nq - 1);
    const long long lim = (long long)((p.qoff + qlast / p.hw) / p.cc + 1) * p.cc * p.hw;
    if (lim < nkeys) nkeys = (int)lim;
  }
  FlashState<QT> st;
  f32x4 o[QT][NVT];
#pragma unroll
  for (int q = 0; q < QT; ++q)
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt) o[q][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int cc = p.cc, hw = p.hw;
  auto meta = [&](int key, float& raw, int& chunk) { raw = 0.f; chunk = cc > 0 ? (key / hw) / cc : 0; };
  flash_loop<D, QT, true, true, 256>(Kp, p.ks.token, Vp, p.vs.token, nkeys, meta, lds, qv, wt.nq,
                                     p.scale * kLog2e, qchunk, st, o, tid, lane);
  u16* Op = (u16*)p.O + b * p.os.batch + hd * p.os.head;
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    const int qi = q0 + 16 * wt.lt[q] + c;
    const float lsum = xsum(st.lrun[q]);
    if (q < wt.nq && qi < p.Nq)
      store_rows<D>(Op + (long long)qi * p.os.token, o[q], lsum > 0.f ? 1.0f / lsum : 0.f, g);
  }
}

template <int NT, int D>
hipError_t launch_r(const KParams& kp, dim3 grid, int gs, bool first, bool last, hipStream_t s) {
  const size_t lds = last ? stage_r_last_lds_bytes<NT, D>(kp.b2) : 0;
  if (first && last) k_bf16_stage_r<NT, D, true, true><<<grid, 64 * NT, lds, s>>>(kp, gs);
  else if (first) k_bf16_stage_r<NT, D, true, false><<<grid, 64 * NT, 0, s>>>(kp, gs);
  else if (last) k_bf16_stage_r<NT, D, false, true><<<grid, 64 * NT, lds, s>>>(kp, gs);
  else k_bf16_stage_r<NT, D, false, false><<<grid, 64 * NT, 0, s>>>(kp, gs);
  return hipGetLastError();
}

template <int D>
hipError_t launch_r_d(const KParams& kp, dim3 grid, int gs, bool first, bool last, hipStream_t s) {
  switch ((kp.b2 + 15) / 16) {
    case 1: return launch_r<1, D>(kp, grid, gs, first, last, s);
    case 2: return launch_r<2, D>(kp, grid, gs, first, last, s);
    case 3: return launch_r<3, D>(kp, grid, gs, first, last, s);
    case 4: return launch_r<4, D>(kp, grid, gs, first, last, s);
    case 5: return launch_r<5, D>(kp, grid, gs, first, last, s);
    case 6: return launch_r<6, D>(kp, grid, gs, first, last, s);
  }
  return hipErrorInvalidValue;
}

template <int D, int QT, int NT>
hipError_t launch_l_out(const KParams& kp, dim3 grid, hipStream_t s) {
  const bool stats = kp.lse_out != nullptr && kp.o32_out != nullptr;
  if (kp.rl > 0) {
    if (stats) k_bf16_stage_l_out<D, QT, NT, true, true><<<grid, NT, 0, s>>>(kp);
    else k_bf16_stage_l_out<D, QT, NT, true><<<grid, NT, 0, s>>>(kp);
  } else {
    if (stats) k_bf16_stage_l_out<D, QT, NT, false, true><<<grid, NT, 0, s>>>(kp);
    else k_bf16_stage_l_out<D, QT, NT, false><<<grid, NT, 0, s>>>(kp);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// stage L for medium key ranges (96 < NK <= 192, b1 <= 128): still one workgroup per (m, j) and
// three workgroups per compute unit, with ONE 52 KB LDS tile used twice.  Last iteration: the
// tile first holds alpha_L[m, j] (every wave forms the exact softmax of its one or two query
// tiles against all keys and keeps the probabilities as packed bf16 in registers), then Y[m, j]
// (second product).  Earlier iterations: the tile holds alpha_L for the row log-sum-exp, then Q
// for the second pass, which streams alpha_L again from global memory.
// ---------------------------------------------------------------------------------------
constexpr int kMidRows = 192;

// Base-2 logits (bias added, -inf beyond the last key) of one query tile against NTK resident key
// tiles (NTK <= 12), and their column maximum.
template <int D, int NTK, int LD, bool SWZ, bool RMASK>
__device__ inline float mid_logits(const u16* Ks, const float* bias, const bf16x8 (&qv)[D / 32],
                                   float scale2, int klim, f32x4 (&s)[2 * ((NTK + 1) / 2)], int lane) {
  constexpr int KS1 = D / 32, KS2 = (NTK + 1) / 2;
  const int g = lane >> 4, c = lane & 15;
#pragma unroll
  for (int kp = 0; kp < KS2; ++kp) {
    bf16x8 a[2][KS1];
#pragma unroll
    for (int t = 0; t < 2; ++t)
      if (2 * kp + t < NTK) {
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks)
          a[t][ks] = ld_lds_16B(Ks + tile_off<LD, SWZ>(16 * (2 * kp + t) + c, 4 * ks + g));
      }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      if (2 * kp + t < NTK) {
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) acc = mfma(a[t][ks], qv[ks], acc);
      }
      s[2 * kp + t] = acc;
    }
    __builtin_amdgcn_sched_barrier(0);   // one pair of key tiles in flight at a time
  }
  float mx = -INFINITY;
#pragma unroll
  for (int kt = 0; kt < 2 * KS2; ++kt) {
    const f32x4 ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    const f32x4 bi = kt < NTK ? *(const f32x4*)(bias + 16 * kt + 4 * g) : ninf;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      s[kt][r] = fmaf(s[kt][r], scale2, bi[r]);
      if (RMASK && 16 * kt + 4 * g + r >= klim) s[kt][r] = -INFINITY;   // hidden from this query row
      mx = fmaxf(mx, s[kt][r]);
    }
  }
  return xmax(mx);
}

template <int D, int NTK, bool RMASK>
__global__ __launch_bounds__(256, 3) void k_bf16_stage_l_out_mid(KParams p) {
  constexpr int LD = ResTile<D>::LD, KS1 = D / 32, NVT = D / 16, KS2 = (NTK + 1) / 2, ROWS = 32 * KS2;
  constexpr bool SWZ = ResTile<D>::SWZ;
  constexpr int QT = 2;
  __shared__ __attribute__((aligned(16))) u16 tile[ROWS * LD];
  __shared__ __attribute__((aligned(16))) float bias[ROWS];

  const int tid = threadIdx.x, nthr = blockDim.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthr >> 6;
  const int lane = tid & 63, g = lane >> 4, c = lane & 15;
  const int b1 = p.b1, b2 = p.b2;
  const int j = blockIdx.x, ml = blockIdx.y, m = p.m0 + ml, bhl = last_head_first(), bh = p.bh0 + bhl;
  const int a = m / p.c2, bq = m - a * p.c2;
  const int NK = visible_key_tile_rows(a, p.c1k, p.ct, p.qt0) * p.c2 * b1;   // <= 16*NTK
  const size_t NKtot = (size_t)p.ntk * b1;
  const int b = bh / p.H, hd = bh - b * p.H;
  const WaveTiles<QT> wt(wave, nwaves, (b1 + 15) >> 4);      // b1 <= 128: at most two tiles a wave

  const size_t row0 = (((size_t)bhl * p.ntq + ml) * b2 + j) * NKtot;
  const u16* aLp = (const u16*)p.aL + row0 * D;
  const u16* Yp = (const u16*)p.Y + row0 * D;
  const float* cLp = p.cL + row0;
  const long long qtok0 = axis_offset(p.cmap, bq * b2 + j);
  const TokRows qrow = tile_rows(p, a, p.qs.token), orow = tile_rows(p, a, p.os.token);
  const u16* Qp = (const u16*)p.Q + b * p.qs.batch + hd * p.qs.head + qtok0 * p.qs.token;
  u16* Op = (u16*)p.O + b * p.os.batch + hd * p.os.head + qtok0 * p.os.token;

  MRT_STAMP(0);
  bf16x8 qv[QT][KS1];
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    const int l = 16 * wt.lt[q] + c;
    const int lc = l < b1 ? l : b1 - 1;
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) qv[q][ks] = ld_global_16B(Qp + qrow(lc) + 32 * ks + 8 * g);
  }
  stage_rows_batched<D, LD, ROWS, 256, SWZ>(tile, aLp, PlainRows{D}, NK, tid);
  for (int i = tid; i < ROWS; i += nthr) bias[i] = i < NK ? -cLp[i] * kLog2e : -INFINITY;
  __syncthreads();
  MRT_STAMP(1);

  // ---- first product and exact softmax, one query tile at a time
  const float scale2 = p.scale * kLog2e;
  bf16x8 pb[KS2][QT];
  float sum[QT];
#pragma unroll
  for (int q = 0; q < QT; ++q) {
    sum[q] = 1.f;
    if (q < wt.nq) {
      f32x4 s[2 * KS2];
      const int lq = 16 * wt.lt[q] + c;
      const int klim = RMASK ? visible_key_rows(p, lq < b1 ? lq : b1 - 1) : 0;
      const float mx = mid_logits<D, NTK, LD, SWZ, RMASK>(tile, bias, qv[q], scale2, klim, s, lane);
      float sm = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2 * KS2; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          s[kt][r] = exp2_fast(s[kt][r] - mx);
          sm += s[kt][r];
        }
      sum[q] = xsum(sm);
#pragma unroll
      for (int st = 0; st < KS2; ++st) pb[st][q] = pack8(s[2 * st], s[2 * st + 1]);
    } else {
#pragma unroll
      for (int st = 0; st < KS2; ++st) pb[st][q] = bf16x8{};
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();                      // every wave is done with alpha_L
  MRT_STAMP(2);
  stage_rows_batched<D, LD, ROWS, 256, SWZ>(tile, Yp, PlainRows{D}, NK, tid);
  __syncthreads();
  MRT_STAMP(3);

  // ---- second product: both query tiles of the wave share every value read
  if (wt.nq > 0) {
    f32x4 o[QT][NVT];
#pragma unroll
    for (int q = 0; q < QT; ++q)
#pragma unroll
      for (int vt = 0; vt < NVT; ++vt) o[q][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < KS2; ++st) {
      pv_step_multi<D, QT, LD, SWZ>(tile + 32 * st * LD, pb[st], wt.nq, o, lane);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < QT; ++q) {
      const int l = 16 * wt.lt[q] + c;
      if (q < wt.nq && l < b1) store_rows_nt<D>(Op + orow(l), o[q], 1.0f / sum[q], g);
    }
  }
  MRT_STAMP(4);
}

template <int D, int NTK>
hipError_t launch_l_out_mid(const KParams& kp, dim3 grid, hipStream_t s) {
  if (kp.rl > 0) k_bf16_stage_l_out_mid<D, NTK, true><<<grid, 256, 0, s>>>(kp);
  else k_bf16_stage_l_out_mid<D, NTK, false><<<grid, 256, 0, s>>>(kp);
  return hipGetLastError();
}

template <int D>
hipError_t launch_l_out_mid_d(const KParams& kp, dim3 grid, int nkt, hipStream_t s) {
  switch (nkt) {
    case 7: case 8: return launch_l_out_mid<D, 8>(kp, grid, s);
    case 9: case 10: return launch_l_out_mid<D, 10>(kp, grid, s);
    case 11: case 12: return launch_l_out_mid<D, 12>(kp, grid, s);
  }
  return hipErrorInvalidValue;
}

// Streamed refine kernel: always four waves (one per SIMD, so that two workgroups fit a compute
// unit however their waves are dealt to the SIMDs), each owning up to QT query tiles.  The chunk
// ring of pass 1 and the Q tile of pass 2 share one LDS region (at most 56 KB for b1 = 192).
template <int D, int NLT>
hipError_t launch_l_refine(const KParams& kp, dim3 grid, hipStream_t s) {
  constexpr int QT = (NLT + 3) / 4, MAXT = 256, PT = 2, PAD = kPad;
  const size_t tile = (size_t)32 * ((NLT + 1) / 2) * (D + PAD) * 2, ring = FlashLds<D, false, PAD>::kBytes;
  const size_t lds = kRefineHead + (tile > ring ? tile : ring);
  hipError_t e;
  if (lds > 64 * 1024 &&
      (e = hipFuncSetAttribute((const void*)k_bf16_stage_l_refine<D, QT, MAXT, NLT, PT, PAD>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess)
    return e;
  k_bf16_stage_l_refine<D, QT, MAXT, NLT, PT, PAD><<<grid, 256, lds, s>>>(kp);
  return hipGetLastError();
}

template <int D, int NTK>
hipError_t launch_l_out_res(const KParams& kp, dim3 grid, hipStream_t s) {
  if (kp.rl > 0) k_bf16_stage_l_out_res<D, NTK, true><<<grid, 256, 0, s>>>(kp);
  else k_bf16_stage_l_out_res<D, NTK, false><<<grid, 256, 0, s>>>(kp);
  return hipGetLastError();
}

template <int D>
hipError_t launch_l_out_res_d(const KParams& kp, dim3 grid, int nkt, hipStream_t s) {
  switch (nkt) {
    case 1: return launch_l_out_res<D, 1>(kp, grid, s);
    case 2: return launch_l_out_res<D, 2>(kp, grid, s);
    case 3: return launch_l_out_res<D, 3>(kp, grid, s);
    case 4: return launch_l_out_res<D, 4>(kp, grid, s);
    case 5: return launch_l_out_res<D, 5>(kp, grid, s);
    case 6: return launch_l_out_res<D, 6>(kp, grid, s);
  }
  return hipErrorInvalidValue;
}

template <int D>
hipError_t launch_l_refine_d(const KParams& kp, dim3 grid, int nlt, hipStream_t s) {
  switch (nlt) {
    case 1: return launch_l_refine<D, 1>(kp, grid, s);
    case 2: return launch_l_refine<D, 2>(kp, grid, s);
    case 3: return launch_l_refine<D, 3>(kp, grid, s);
    case 4: return launch_l_refine<D, 4>(kp, grid, s);
    case 5: return launch_l_refine<D, 5>(kp, grid, s);
    case 6: return launch_l_refine<D, 6>(kp, grid, s);
    case 7: return launch_l_refine<D, 7>(kp, grid, s);
    case 8: return launch_l_refine<D, 8>(kp, grid, s);
    case 9: return launch_l_refine<D, 9>(kp, grid, s);
    case 10: return launch_l_refine<D, 10>(kp, grid, s);
    case 11: return launch_l_refine<D, 11>(kp, grid, s);
    case 12: return launch_l_refine<D, 12>(kp, grid, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

#ifdef MRT_TRACE
hipError_t set_trace_buffer(void* buf, hipStream_t s) {
  static thread_local unsigned long long* slot[64];
  static thread_local int next = 0;
  slot[next] = (unsigned long long*)buf;
  hipError_t e = hipMemcpyToSymbolAsync(HIP_SYMBOL(g_trace_buf), &slot[next], sizeof(void*), 0,
                                        hipMemcpyHostToDevice, s);
  next = (next + 1) % 64;
  return e;
}
#endif

hipError_t launch_bf16_stage_r(const KParams& kp, int nbh, bool first, bool last, hipStream_t s) {
  // query tiles per workgroup: each key block is then staged once for gs query tiles instead of
  // once per tile.  Measured: 2..3 tiles per workgroup win whenever the launch keeps about a
  // thousand workgroups; more only lengthen the workgroups.
  const long long blocks = (long long)kp.ntk * kp.b1 * kp.ntq * nbh;
  long long gs = blocks / 1024;
  if (gs > 3) gs = 3;
  if (gs > kp.ntq) gs = kp.ntq;
  if (gs < 1) gs = 1;
  dim3 grid(kp.ntk * kp.b1, (kp.ntq + (int)gs - 1) / (int)gs, nbh);
  return kp.d == 128 ? launch_r_d<128>(kp, grid, (int)gs, first, last, s)
                     : launch_r_d<64>(kp, grid, (int)gs, first, last, s);
}

// RMASK: regular Monarch under the chunk-causal mask (a variant of its own, so that the unmasked
// kernel carries neither the mask code nor its registers)
template <int D, int NLT, int PT, int NW>
void launch_refine_one_k(const KParams& kp, dim3 grid, hipStream_t s) {
  if (kp.rl > 0) k_bf16_stage_l_refine_one<D, NLT, PT, NW, true><<<grid, 64 * NW, 0, s>>>(kp);
  else k_bf16_stage_l_refine_one<D, NLT, PT, NW, false><<<grid, 64 * NW, 0, s>>>(kp);
}

template <int D, int PT>
hipError_t launch_l_refine_one(const KParams& kp, dim3 grid, int nlt, hipStream_t s) {
  switch (nlt) {
    case 1: launch_refine_one_k<D, 1, PT, 4>(kp, grid, s); break;
    case 2: launch_refine_one_k<D, 2, PT, 4>(kp, grid, s); break;
    case 3: launch_refine_one_k<D, 3, PT, 4>(kp, grid, s); break;
    case 4: launch_refine_one_k<D, 4, PT, 4>(kp, grid, s); break;
    case 5: launch_refine_one_k<D, 5, PT, 4>(kp, grid, s); break;
    case 6: launch_refine_one_k<D, 6, PT, 4>(kp, grid, s); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
// 7 .. 12 query tiles (one key tile per query tile, so as many key tiles): six waves, two key
// tiles each; an odd tile count runs as the next even one (the extra tile is masked rows)
template <int D>
hipError_t launch_l_refine_one_wide(const KParams& kp, dim3 grid, int nlt, hipStream_t s) {
  switch ((nlt + 1) / 2) {
    case 4: launch_refine_one_k<D, 8, 2, 6>(kp, grid, s); break;
    case 5: launch_refine_one_k<D, 10, 2, 6>(kp, grid, s); break;
    case 6: launch_refine_one_k<D, 12, 2, 6>(kp, grid, s); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// The last iteration's stage L runs the streamed kernel (the one that can leave row statistics
// and an fp32 output for a backward call): same conditions as in launch_bf16_stage_l below.
bool bf16_stage_l_out_streams(const KParams& kp) {
  const int nlt = (kp.b1 + 15) / 16, nk_max = kp.ntk * kp.b1;
  return nlt <= kMaxLT && nk_max > kResRows && !(nk_max <= kMidRows && nlt <= 8);
}

hipError_t launch_bf16_stage_l(const KParams& kp, int nbh, bool last, hipStream_t s) {
  dim3 grid(kp.b2, kp.ntq, nbh);
  const int nlt = (kp.b1 + 15) / 16;
  if (nlt > kMaxLT) return hipErrorInvalidValue;
  const int nk_max = kp.ntk * kp.b1;
  // earlier iterations, key range of at most 192 rows: one pass over the logits (four waves for
  // b1 <= 96, six beyond)
  if (!last && nk_max <= kMidRows && nlt <= 6) {
    if (nk_max <= 128) return kp.d == 128 ? launch_l_refine_one<128, 2>(kp, grid, nlt, s)
                                          : launch_l_refine_one<64, 2>(kp, grid, nlt, s);
    return kp.d == 128 ? launch_l_refine_one<128, 3>(kp, grid, nlt, s)
                       : launch_l_refine_one<64, 3>(kp, grid, nlt, s);
  }
  if (!last && nk_max <= kMidRows && nlt <= kMaxLT)
    return kp.d == 128 ? launch_l_refine_one_wide<128>(kp, grid, nlt, s)
                       : launch_l_refine_one_wide<64>(kp, grid, nlt, s);
  // last iteration, short key ranges: everything resident, three workgroups per compute unit
  if (nk_max <= kResRows) {
    return kp.d == 128 ? launch_l_out_res_d<128>(kp, grid, (nk_max + 15) / 16, s)
                       : launch_l_out_res_d<64>(kp, grid, (nk_max + 15) / 16, s);
  }
  // medium key ranges, last iteration: one LDS tile used twice, still three workgroups per
  // compute unit (the earlier iterations went above)
  if (nk_max <= kMidRows && nlt <= 8)
    return kp.d == 128 ? launch_l_out_mid_d<128>(kp, grid, (nk_max + 15) / 16, s)
                       : launch_l_out_mid_d<64>(kp, grid, (nk_max + 15) / 16, s);
  // long key ranges: streamed.  Workgroups of 4 waves (one per SIMD), each wave owning up to two
  // query tiles, so that two workgroups fit a compute unit whatever order their waves are dealt
  // to the SIMDs in; only b1 > 128 needs a fifth and sixth wave.
  if (!last) return kp.d == 128 ? launch_l_refine_d<128>(kp, grid, nlt, s)
                                : launch_l_refine_d<64>(kp, grid, nlt, s);
  if (nlt <= 4) return kp.d == 128 ? launch_l_out<128, 1, 256>(kp, grid, s)
                                   : launch_l_out<64, 1, 256>(kp, grid, s);
  if (nlt <= 8) return kp.d == 128 ? launch_l_out<128, 2, 256>(kp, grid, s)
                                   : launch_l_out<64, 2, 256>(kp, grid, s);
  return kp.d == 128 ? launch_l_out<128, 2, 512>(kp, grid, s)
                     : launch_l_out<64, 2, 512>(kp, grid, s);
}

hipError_t launch_bf16_dense(const KParams& kp, int nbh, hipStream_t s) {
  dim3 grid((kp.Nq + kDenseQ - 1) / kDenseQ, nbh);
  if (kp.d == 128) k_bf16_dense<128><<<grid, 256, 0, s>>>(kp);
  else k_bf16_dense<64><<<grid, 256, 0, s>>>(kp);
  return hipGetLastError();
}

}  // namespace mrt
