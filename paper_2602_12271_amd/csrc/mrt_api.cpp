// Host side of the C ABI: argument checks, workspace carving, pass scheduling.
// No arithmetic of the method happens here; every step runs in the kernels.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "mrt_internal.hpp"

namespace mrt {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static size_t round256(size_t x) { return (x + 255) & ~size_t(255); }

static mrt_status check_common(const mrt_problem* p) {
  if (!p) { set_error("problem is NULL"); return MRT_ERR_NULL; }
  if (p->batch < 1 || p->heads < 1 || p->f_q < 1 || p->f_kv < 1 || p->h < 1 || p->w < 1) {
    set_error("batch/heads/f_q/f_kv/h/w must be >= 1");
    return MRT_ERR_SHAPE;
  }
  if ((long long)p->batch * p->heads > 65535) {
    set_error("batch*heads = %lld exceeds 65535", (long long)p->batch * p->heads);
    return MRT_ERR_SHAPE;
  }
  if (p->dtype != MRT_F32 && p->dtype != MRT_BF16) { set_error("unknown dtype"); return MRT_ERR_SHAPE; }
  if (p->compute != MRT_COMPUTE_DEFAULT && p->compute != MRT_COMPUTE_F32) {
    set_error("unknown compute mode");
    return MRT_ERR_SHAPE;
  }
  const bool f32 = p->dtype == MRT_F32 || p->compute == MRT_COMPUTE_F32;
  if (f32) {
    if (p->head_dim < 1 || p->head_dim > 128) { set_error("head_dim must be 1..128"); return MRT_ERR_SHAPE; }
  } else if (p->head_dim != 64 && p->head_dim != 128) {
    set_error("bf16 path needs head_dim 64 or 128, got %d", p->head_dim);
    return MRT_ERR_SHAPE;
  }
  long long nq = (long long)p->f_q * p->h * p->w, nkv = (long long)p->f_kv * p->h * p->w;
  if (nq > (1 << 24) || nkv > (1 << 24)) { set_error("more than 2^24 tokens per head"); return MRT_ERR_SHAPE; }
  const mrt_strides* st[4] = {&p->q, &p->k, &p->v, &p->o};
  for (int t = 0; t < 4; ++t) {
    if (st[t]->token < p->head_dim || st[t]->head < 1 || st[t]->batch < 1) {
      set_error("stride set %d: token stride must be >= head_dim, head/batch strides >= 1", t);
      return MRT_ERR_SHAPE;
    }
    // 16-byte vector accesses on the bf16 path need rows aligned to 8 elements
    if (!f32 && (st[t]->token % 8 || st[t]->head % 8 || st[t]->batch % 8)) {
      set_error("stride set %d: bf16 path needs strides that are multiples of 8 elements", t);
      return MRT_ERR_SHAPE;
    }
    // the bf16 kernels address the tokens of one (batch, head) with 32-bit element offsets
    if (!f32 && (t < 1 || t > 2 ? nq : nkv) * st[t]->token >= (1ll << 31)) {
      set_error("stride set %d: tokens x token stride must stay below 2^31 elements on the bf16 path", t);
      return MRT_ERR_UNSUPPORTED;
    }
  }
  if (p->q_frame_offset < 0) { set_error("q_frame_offset < 0"); return MRT_ERR_SHAPE; }
  if ((int)p->assignment < 0 || (int)p->assignment > (int)MRT_ASSIGN_HW_F) {
    set_error("unknown block assignment %d", (int)p->assignment);
    return MRT_ERR_SHAPE;
  }
  if (!(p->scale > 0.0f) || !(p->scale < 1e30f)) { set_error("scale must be positive and finite"); return MRT_ERR_SHAPE; }
  if (p->tile_h < 0) { set_error("tile_h < 0"); return MRT_ERR_SHAPE; }
  if (p->head_groups < 0) { set_error("head_groups < 0"); return MRT_ERR_SHAPE; }
  return MRT_OK;
}

static mrt_status make_plan(const mrt_problem* p, int b1, int b2, int tile, int iters,
                            int causal_chunk, Plan* out) {
  mrt_status st = check_common(p);
  if (st != MRT_OK) return st;
  if (tile != 0 && tile != 1) { set_error("tile must be 0 or 1"); return MRT_ERR_SHAPE; }
  if (iters < 1) { set_error("iters must be >= 1"); return MRT_ERR_SHAPE; }
  if (iters > 64) { set_error("iters > 64"); return MRT_ERR_SHAPE; }
  if (causal_chunk < 0) { set_error("causal_chunk < 0"); return MRT_ERR_SHAPE; }
  if (b1 < 1 || b2 < 1) { set_error("block sizes must be >= 1"); return MRT_ERR_BLOCK; }
  if (b1 > 192 || b2 > 96) {
    set_error("this build supports b1 <= 192 and b2 <= 96 (got %d, %d)", b1, b2);
    return MRT_ERR_UNSUPPORTED;
  }
  Plan pl;
  memset(&pl, 0, sizeof(pl));
  KParams& k = pl.kp;
  // block grid of the chosen assignment (Sec. 4.1): rows x cols per side, and the token offsets
  // of a row / column index.  rpf = rows per frame when the frame is the slowest row axis.
  const int f_q = p->f_q, f_kv = p->f_kv, h = p->h, w = p->w, hw = p->h * p->w;
  int rows_q = 0, rows_k = 0, cols_q = 0, cols_k = 0, rpf = 0;
  static const char* const kNames[] = {"(fh,w)", "(w,fh)", "(fw,h)", "(h,fw)", "(f,hw)", "(hw,f)"};
  const char* aname = kNames[(int)p->assignment];
  switch (p->assignment) {
    case MRT_ASSIGN_FH_W:
      rows_q = f_q * h; rows_k = f_kv * h; cols_q = cols_k = w; rpf = h;
      k.rmap = AxisMap{0, 0, w}; k.cmap = AxisMap{0, 0, 1};
      break;
    case MRT_ASSIGN_W_FH:
      rows_q = rows_k = w; cols_q = f_q * h; cols_k = f_kv * h;
      k.rmap = AxisMap{0, 0, 1}; k.cmap = AxisMap{0, 0, w};
      break;
    case MRT_ASSIGN_FW_H:
      rows_q = f_q * w; rows_k = f_kv * w; cols_q = cols_k = h; rpf = w;
      k.rmap = AxisMap{w, hw, 1}; k.cmap = AxisMap{0, 0, w};
      break;
    case MRT_ASSIGN_H_FW:
      rows_q = rows_k = h; cols_q = f_q * w; cols_k = f_kv * w;
      k.rmap = AxisMap{0, 0, w}; k.cmap = AxisMap{w, hw, 1};
      break;
    case MRT_ASSIGN_F_HW:
      rows_q = f_q; rows_k = f_kv; cols_q = cols_k = hw; rpf = 1;
      k.rmap = AxisMap{0, 0, hw}; k.cmap = AxisMap{0, 0, 1};
      break;
    case MRT_ASSIGN_HW_F:
      rows_q = rows_k = hw; cols_q = f_q; cols_k = f_kv;
      k.rmap = AxisMap{0, 0, 1}; k.cmap = AxisMap{0, 0, hw};
      break;
  }
  if (cols_q != cols_k) {
    set_error("assignment %s has the frame axis on the b2 side: f_q must equal f_kv", aname);
    return MRT_ERR_UNSUPPORTED;
  }
  const int cols = cols_q;
  if (tile == 0) {
    if (p->f_q != p->f_kv) {
      set_error("regular Monarch needs f_q == f_kv (use tile=1 for a KV cache)");
      return MRT_ERR_UNSUPPORTED;
    }
    if (p->tile_h != 0) { set_error("tile_h needs tile = 1"); return MRT_ERR_SHAPE; }
    if (b1 != rows_q || b2 != cols) {
      set_error("regular Monarch with assignment %s needs (b1,b2) = (%d,%d), got (%d,%d)", aname, rows_q, cols, b1, b2);
      return MRT_ERR_BLOCK;
    }
    k.c2 = 1; k.ntq = 1; k.ntk = 1; k.c1k = 1; pl.c1q = 1;
  } else if (p->tile_h > 0) {
    // neighbourhood tiles (n_f, n_h, n_w) = (b1 / n_h, n_h, b2) of Sec. 4.2
    const int nh = p->tile_h;
    if (p->assignment != MRT_ASSIGN_FH_W) {
      set_error("neighbourhood tiles (tile_h > 0) need the (fh,w) assignment");
      return MRT_ERR_UNSUPPORTED;
    }
    if (h % nh || b1 % nh || w % b2) {
      set_error("neighbourhood tiles: tile_h = %d must divide h = %d and b1 = %d, and b2 = %d must divide w = %d",
                nh, h, b1, b2, w);
      return MRT_ERR_BLOCK;
    }
    const int nf = b1 / nh;
    if (f_q % nf || f_kv % nf) {
      set_error("neighbourhood tiles of %d frames do not divide the grids (%d | %d frames)", nf, f_q, f_kv);
      return MRT_ERR_BLOCK;
    }
    k.nh = nh; k.nhb = h / nh; k.tf_tok = nf * hw; k.th_tok = nh * w;
    k.c2 = w / b2;
    k.c1k = (f_kv / nf) * k.nhb;
    pl.c1q = (f_q / nf) * k.nhb;
    k.ntq = pl.c1q * k.c2;
    k.ntk = k.c1k * k.c2;
  } else {
    if (rows_q % b1 || rows_k % b1 || cols % b2) {
      set_error("tile blocks (%d,%d) do not divide the %s grids (%d|%d rows, %d cols)", b1, b2, aname,
                rows_q, rows_k, cols);
      return MRT_ERR_BLOCK;
    }
    k.c2 = cols / b2;
    k.c1k = rows_k / b1;
    pl.c1q = rows_q / b1;
    k.ntq = pl.c1q * k.c2;
    k.ntk = k.c1k * k.c2;
  }
  if (causal_chunk > 0) {
    if (rpf == 0) {
      set_error("a causal mask needs an assignment whose slowest b1 axis is the frame, not %s", aname);
      return MRT_ERR_UNSUPPORTED;
    }
    long long ct = 0, qt0 = 0;
    if (tile == 0) {
      // one tile across every chunk: the mask hides key rows of later chunks from a query row
      // (a support constraint on L); nothing is hidden if query row 0 already sees every row
      const long long rl = (long long)causal_chunk * rpf, r0 = (long long)p->q_frame_offset * rpf;
      if ((r0 / rl + 1) * rl < b1) { k.rl = (int)rl; k.rq0 = (int)r0; }   // rl < b1 <= 192 here
    } else if (k.nh > 0) {
      const int nf = b1 / k.nh;
      if (causal_chunk % nf || p->q_frame_offset % nf) {
        set_error("a tile (%d frames) must not straddle a causal chunk (%d frames, offset %d)", nf,
                  causal_chunk, p->q_frame_offset);
        return MRT_ERR_BLOCK;
      }
      ct = (long long)(causal_chunk / nf) * k.nhb;
      qt0 = (long long)(p->q_frame_offset / nf) * k.nhb;
    } else {
      const long long cr = (long long)causal_chunk * rpf, q0 = (long long)p->q_frame_offset * rpf;
      if (cr % b1 || q0 % b1) {
        set_error("a tile (%d rows, %d rows per frame) must not straddle a causal chunk (%d frames, offset %d)",
                  b1, rpf, causal_chunk, p->q_frame_offset);
        return MRT_ERR_BLOCK;
      }
      ct = cr / b1;
      qt0 = q0 / b1;
    }
    if (ct > (1 << 24) || qt0 > (1 << 24)) { set_error("causal chunk or frame offset too large"); return MRT_ERR_SHAPE; }
    k.ct = (int)ct; k.qt0 = (int)qt0; k.cc = causal_chunk; k.qoff = p->q_frame_offset;
  }
  k.qs = p->q; k.ks = p->k; k.vs = p->v; k.os = p->o;
  k.H = p->heads; k.d = p->head_dim; k.b1 = b1; k.b2 = b2;
  k.Nq = p->f_q * p->h * p->w; k.Nkv = p->f_kv * p->h * p->w; k.hw = p->h * p->w;
  k.scale = p->scale;
  pl.B = p->batch; pl.T = iters; pl.Nq = k.Nq; pl.Nkv = k.Nkv;
  pl.dtype = p->dtype; pl.compute = p->compute;
  const size_t es = pl.f32_path() ? 4 : 2;
  pl.ntq_total = k.ntq;
  // one slab = the intermediates of one query tile row (c2 query tiles) of one (batch, head)
  const size_t rows = (size_t)k.c2 * b1 * b2 * k.ntk;          // (m, j, nk) triples of the row
  pl.slab_aL = round256(rows * k.d * es);
  pl.slab_Y = pl.slab_aL;
  pl.slab_aR = iters >= 2 ? pl.slab_aL : 0;
  pl.slab_cL = round256(rows * sizeof(float));
  *out = pl;
  return MRT_OK;
}

// (batch, head, query tile row) slabs the recommended workspace is sized for
static size_t recommended_slabs(const Plan& pl) {
  // Measured on MI355X: more (batch, head) slabs per pass always won over keeping a pass inside
  // the 256 MB last-level cache (stage L has only ntq*b2 workgroups per head), so the only cap
  // is a bound on the workspace itself.
  const size_t budget = size_t(8) << 30;
  const size_t all = (size_t)pl.B * pl.kp.H * pl.c1q;
  size_t g = budget / pl.slab_bytes();
  if (g >= (size_t)pl.c1q) g -= g % pl.c1q;        // whole heads when at least one fits
  if (g < 1) g = 1;
  return g > all ? all : g;
}

#ifdef MRT_TRACE
hipError_t set_trace_buffer(void* buf, hipStream_t s);
static char* g_trace_base = nullptr;
static size_t g_trace_stride = 0;
static int g_trace_next = 0;
static void trace_next_launch(hipStream_t s) {
  if (g_trace_base) (void)set_trace_buffer(g_trace_base + g_trace_stride * (g_trace_next++), s);
}
#else
static inline void trace_next_launch(hipStream_t) {}
#endif

// ---- optional per-kernel timing (benchmarks only) --------------------------------------
struct ProfRecord { hipEvent_t a, b; int kind, reps; };
static std::atomic<int> g_prof_on{0};   // 0 = off, r > 0 = each launch issued r times inside its bracket
static std::vector<ProfRecord> g_prof;
static std::mutex g_prof_mu;

// Runs `launch` once, or, while profiling, g_prof_on times between two events.  Every kernel of
// this library reads only buffers it does not write, so a repeated launch leaves the same result.
template <class F>
static hipError_t timed_launch(hipStream_t s, int kind, F launch, bool may_time = true) {
  const int reps = may_time ? g_prof_on.load(std::memory_order_relaxed) : 0;
  if (reps <= 0) return launch();
  hipEvent_t a = nullptr, b = nullptr;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return launch();
  (void)hipEventRecord(a, s);
  hipError_t e = hipSuccess;
  for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch();
  (void)hipEventRecord(b, s);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof.push_back({a, b, kind, reps});
  return e;
}

// ---- helper streams for concurrent head groups ------------------------------------------
constexpr int kMaxGroups = 4;
static std::atomic<int> g_max_groups{0};   // process-wide default; 0 = choose per call
struct StreamPool {
  hipStream_t side[kMaxGroups - 1];
  hipEvent_t fork, join[kMaxGroups - 1];
  // Held from the fork record to the last join wait of a call: the pool's events and helper
  // streams belong to one call at a time, so two host threads (or two caller streams) inside
  // multi-group calls on one device never re-record an event another call still has to wait on.
  // A stream wait binds to the record that precedes it, so the next call may re-record the events
  // as soon as this one has enqueued its waits.
  std::mutex in_use;
};
// One pool per device, created on first use and kept for the life of the process.  Streams are
// created with the default priority.
// The fork / join events order streams of one device only: no timing, and no system-scope fence
// (cache write-back to the host's view) when they are recorded; the kernels' own device-scope
// release at their end is what the other stream's kernels need.
constexpr unsigned kForkJoinFlags = hipEventDisableTiming | hipEventDisableSystemFence;
static StreamPool* get_pool() {
  static std::mutex mu;
  static StreamPool* pools[64] = {nullptr};
  static bool failed[64] = {false};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lk(mu);
  if (pools[dev] || failed[dev]) return pools[dev];
  StreamPool* p = new StreamPool();
  bool ok = hipEventCreateWithFlags(&p->fork, kForkJoinFlags) == hipSuccess;
  for (int i = 0; ok && i < kMaxGroups - 1; ++i)
    ok = hipStreamCreateWithFlags(&p->side[i], hipStreamNonBlocking) == hipSuccess &&
         hipEventCreateWithFlags(&p->join[i], kForkJoinFlags) == hipSuccess;
  if (!ok) { failed[dev] = true; delete p; return nullptr; }   // fall back to one stream
  pools[dev] = p;
  return p;
}

// Compute units of the current device (256 on MI355X); queried once per process.
static int compute_units() {
  static const int n = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
      cus = 256;
    return cus;
  }();
  return n;
}

// Head groups a call asks for: the call's own field, else the process-wide default (0 = automatic).
static int requested_groups(const mrt_problem* p) {
  int n = p->head_groups > 0 ? p->head_groups : g_max_groups.load(std::memory_order_relaxed);
  return n > kMaxGroups ? kMaxGroups : n;
}

static mrt_status hip_fail(hipError_t e, const char* what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return MRT_ERR_HIP;
}

}  // namespace mrt

using namespace mrt;

extern "C" {

const char* mrt_status_string(mrt_status s) {
  switch (s) {
    case MRT_OK: return "ok";
    case MRT_ERR_NULL: return "null pointer";
    case MRT_ERR_SHAPE: return "bad shape or stride";
    case MRT_ERR_BLOCK: return "block sizes do not fit the grid";
    case MRT_ERR_UNSUPPORTED: return "not supported by this build";
    case MRT_ERR_WORKSPACE: return "workspace too small";
    case MRT_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

const char* mrt_last_error(void) { return g_err; }

mrt_status monarch_attn_check(const mrt_problem* p, int b1, int b2, int tile, int iters,
                              int causal_chunk) {
  Plan pl;
  return make_plan(p, b1, b2, tile, iters, causal_chunk, &pl);
}

size_t monarch_attn_workspace_min_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters) {
  Plan pl;
  if (make_plan(p, b1, b2, tile, iters, 0, &pl) != MRT_OK) return 0;
  return pl.slab_bytes();
}

size_t monarch_attn_workspace_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters) {
  Plan pl;
  if (make_plan(p, b1, b2, tile, iters, 0, &pl) != MRT_OK) return 0;
  return pl.slab_bytes() * recommended_slabs(pl);
}

}  // extern "C"

namespace mrt {
// The forward call behind both entry points.  own_stream_only: run every launch on the caller's
// stream and create no HIP object (no helper streams, no timing events).
mrt_status fwd_run(const void* Q, const void* K, const void* V, void* O, const mrt_problem* p, int b1,
                   int b2, int tile, int iters, int causal_chunk, void* workspace,
                   size_t workspace_bytes, void* hip_stream, bool own_stream_only) {
  Plan pl;
  mrt_status st = make_plan(p, b1, b2, tile, iters, causal_chunk, &pl);
  if (st != MRT_OK) return st;
  if (!Q || !K || !V || !O || !workspace) { set_error("Q, K, V, O and workspace must be non-NULL"); return MRT_ERR_NULL; }
  if ((uintptr_t)workspace % 256) { set_error("workspace must be 256-byte aligned"); return MRT_ERR_WORKSPACE; }
  if (!pl.f32_path()) {
    const void* ptrs[4] = {Q, K, V, O};
    for (const void* q : ptrs)
      if ((uintptr_t)q % 16) { set_error("bf16 path needs 16-byte aligned tensors"); return MRT_ERR_SHAPE; }
  }
  const size_t slab = pl.slab_bytes();
  if (workspace_bytes < slab) {
    set_error("workspace has %zu bytes, one query tile row of one (batch,head) needs %zu",
              workspace_bytes, slab);
    return MRT_ERR_WORKSPACE;
  }
  // A pass covers G (batch, head) entries x A query tile rows, whatever fits the workspace:
  // all rows of as many heads as possible, or, if not even one head fits, A rows of one head at
  // a time (query tiles are independent: the mini-sequence strategy of Sec. 4.3).
  const int BH = pl.B * pl.kp.H;
  const size_t units = workspace_bytes / slab;
  int G, A;
  if (units >= (size_t)pl.c1q) {
    G = (int)(units / pl.c1q < (size_t)BH ? units / pl.c1q : (size_t)BH);
    A = pl.c1q;
  } else {
    G = 1;
    A = (int)units;
  }
  hipStream_t s = (hipStream_t)hip_stream;

  KParams kp = pl.kp;
  kp.Q = Q; kp.K = K; kp.V = V; kp.O = O;
  char* base = (char*)workspace;
  const size_t per_head = (size_t)A;               // slabs per head inside a pass
  kp.aL = base;
  kp.Y = base + pl.slab_aL * per_head * G;
  kp.aR = base + (pl.slab_aL + pl.slab_Y) * per_head * G;
  kp.cL = (float*)(base + (pl.slab_aL + pl.slab_Y + pl.slab_aR) * per_head * G);

  // Heads are independent, so a pass is cut into up to kMaxGroups head groups whose kernel chains
  // run on helper streams forked from and joined back to the caller's stream: the short tail of
  // one group's launch (workgroup counts are rarely a multiple of what the chip holds) overlaps
  // the next kernel of another group.  Per-kernel timing needs launches that do not overlap.
  // Measured on MI355X: the fork/join costs ~10 us per extra group, so it only pays for launches
  // that run for >= 100 us, and only when a group's chain has several kernels to interleave with
  // the other group's (T >= 2: KV-cache steps -1 ... -4 %; the two-kernel chains of T = 1 lose
  // 1 ... 5 %); small calls run on the caller's stream.
  int want_groups = requested_groups(p);
  if (want_groups == 0) {
    const size_t inter_per_launch = pl.slab_aL * per_head * G;
    want_groups = (inter_per_launch >= (size_t(128) << 20) && pl.T >= 2) ? 2 : 1;
  }
  const bool may_time = !own_stream_only;
  StreamPool* pool = (own_stream_only || g_prof_on.load() || want_groups <= 1) ? nullptr : get_pool();
  std::unique_lock<std::mutex> pool_lock;
  if (pool) pool_lock = std::unique_lock<std::mutex>(pool->in_use);
  mrt_status status = MRT_OK;
  for (int bh0 = 0; bh0 < BH && status == MRT_OK; bh0 += G)
  for (int a0 = 0; a0 < pl.c1q && status == MRT_OK; a0 += A) {
    const int nbh = BH - bh0 < G ? BH - bh0 : G;
    const int na = pl.c1q - a0 < A ? pl.c1q - a0 : A;
    kp.m0 = a0 * pl.kp.c2;
    kp.ntq = na * pl.kp.c2;
    int ngroups = pool ? (nbh < want_groups ? nbh : want_groups) : 1;
    if (ngroups > 1) {
      if (hipEventRecord(pool->fork, s) != hipSuccess) ngroups = 1;
      for (int gi = 1; gi < ngroups; ++gi)
        if (hipStreamWaitEvent(pool->side[gi - 1], pool->fork, 0) != hipSuccess) status = MRT_ERR_HIP;
      if (status != MRT_OK) { set_error("helper stream fork failed"); break; }
    }
    // Two groups: when the heads whose stage L workgroups fill the chip exactly once (two
    // workgroups per compute unit) are at least half of the pass, the first group takes that many
    // and the second the rest, so that the larger group's stage L launches have no part-filled
    // second round (12 heads of 52 columns: 9 + 3, 467 -> 456 us on the 480p KV-cache step);
    // otherwise the heads are split evenly.
    int first_group = 0;
    if (ngroups == 2) {
      const long long wgs_per_head = (long long)na * pl.kp.c2 * pl.kp.b2;
      const int per_round = (int)(2LL * compute_units() / (wgs_per_head > 0 ? wgs_per_head : 1));
      if (per_round < nbh && 2 * per_round >= nbh) first_group = per_round;
    }
    for (int gi = 0; gi < ngroups; ++gi) {
      int lo = (int)((long long)nbh * gi / ngroups), hi = (int)((long long)nbh * (gi + 1) / ngroups);
      if (first_group > 0) { lo = gi == 0 ? 0 : first_group; hi = gi == 0 ? first_group : nbh; }
      hipStream_t gs = gi == 0 ? s : pool->side[gi - 1];
      KParams kg = kp;
      kg.bh0 = bh0 + lo;
      kg.aL = (char*)kp.aL + pl.slab_aL * na * lo;
      kg.Y = (char*)kp.Y + pl.slab_Y * na * lo;
      kg.aR = (char*)kp.aR + pl.slab_aR * na * lo;
      kg.cL = (float*)((char*)kp.cL + pl.slab_cL * na * lo);
      for (int t = 1; t <= pl.T && status == MRT_OK; ++t) {
        const bool first = t == 1, last = t == pl.T;
        hipError_t e;
        trace_next_launch(gs);
        e = timed_launch(gs, MRT_KERNEL_STAGE_R | (first ? MRT_KERNEL_FIRST : 0) | (last ? MRT_KERNEL_LAST : 0), [&] {
          return pl.f32_path() ? launch_f32_stage_r(kg, pl.dtype, hi - lo, first, last, gs)
                               : launch_bf16_stage_r(kg, hi - lo, first, last, gs);
        }, may_time);
        if (e != hipSuccess) { status = hip_fail(e, "stage R launch"); break; }
        trace_next_launch(gs);
        e = timed_launch(gs, MRT_KERNEL_STAGE_L | (last ? MRT_KERNEL_LAST : 0), [&] {
          return pl.f32_path() ? launch_f32_stage_l(kg, pl.dtype, hi - lo, last, gs)
                               : launch_bf16_stage_l(kg, hi - lo, last, gs);
        }, may_time);
        if (e != hipSuccess) { status = hip_fail(e, "stage L launch"); break; }
      }
    }
    // join even after a failed launch, so that the helper streams never run ahead of the caller
    for (int gi = 1; gi < ngroups; ++gi) {
      if (hipEventRecord(pool->join[gi - 1], pool->side[gi - 1]) != hipSuccess ||
          hipStreamWaitEvent(s, pool->join[gi - 1], 0) != hipSuccess) {
        if (status == MRT_OK) { set_error("helper stream join failed"); status = MRT_ERR_HIP; }
      }
    }
  }
  return status;
}
}  // namespace mrt

extern "C" {

mrt_status monarch_attn_fwd(const void* Q, const void* K, const void* V, void* O,
                            const mrt_problem* p, int b1, int b2, int tile, int iters,
                            int causal_chunk, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  return mrt::fwd_run(Q, K, V, O, p, b1, b2, tile, iters, causal_chunk, workspace, workspace_bytes,
                      hip_stream, false);
}

// ---- backward pass -------------------------------------------------------------------------
// Workspace of one (batch, head), sized for fp32 entries (the matrix-unit path stores bf16 in the
// same places): alpha_L and c_L of every iteration, abar and its two column statistics of
// iterations 2..T, Y, the gradient buffers d alpha_L, d c_L, d Y, d abar, the matrix-unit kernels'
// transposed scratch, and (more than 192 key rows per problem or more than eight query tiles, bf16)
// the fp32 output copy and row log-sum-exp that the saving forward call leaves for the sweep.
namespace {
struct BwdLayout {
  size_t rowsD, rowsS;    // bytes of one [m][j][nk][d] / [m][j][nk] array of one head
  size_t rows;            // (m, j, nk) triples of one head
  size_t scratch;         // bytes of the matrix-unit kernels' own arrays of one head (0 if unused)
  size_t rowsO, rowsL;    // bytes of one head's fp32 output copy [m][j][l][d] and row statistics [m][j][l]
                          // (0 unless the streamed last-iteration stage L kernel can leave them)
  size_t per_head;
  int T;
  bool mfma;              // stage L backward runs on the bf16 matrix unit
  size_t off_aL(int t) const { return rowsD * (size_t)(t - 1); }                 // t = 1..T
  size_t off_aR(int t) const { return rowsD * (size_t)(T + t - 2); }             // t = 2..T
  size_t off_Y() const { return rowsD * (size_t)(2 * T - 1); }
  size_t off_daL() const { return rowsD * (size_t)(2 * T); }
  size_t off_dY() const { return rowsD * (size_t)(2 * T + 1); }
  size_t off_dA() const { return rowsD * (size_t)(2 * T + 2); }
  size_t base_S() const { return rowsD * (size_t)(2 * T + 3); }
  size_t off_cL(int t) const { return base_S() + rowsS * (size_t)(t - 1); }
  size_t off_dcL() const { return base_S() + rowsS * (size_t)T; }
  size_t off_cmx(int t) const { return base_S() + rowsS * (size_t)(T + t - 1); }        // t = 2..T
  size_t off_cinv(int t) const { return base_S() + rowsS * (size_t)(2 * T + t - 2); }   // t = 2..T
  size_t off_scratch() const { return base_S() + rowsS * (size_t)(3 * T - 1); }
  size_t off_o32() const { return off_scratch() + scratch; }
  size_t off_lse() const { return off_o32() + rowsO; }
};
BwdLayout bwd_layout(const mrt::Plan& pl, const mrt_problem* p) {
  BwdLayout L;
  const size_t rows = (size_t)pl.kp.c2 * pl.kp.b1 * pl.kp.b2 * pl.kp.ntk * pl.c1q;   // (m, j, nk) triples
  L.rows = rows;
  L.rowsD = mrt::round256(rows * pl.kp.d * sizeof(float));
  L.rowsS = mrt::round256(rows * sizeof(float));
  L.T = pl.T;
  L.mfma = p->dtype == MRT_BF16 && p->compute == MRT_COMPUTE_DEFAULT && mrt::bwd_bf16_fits(pl.kp);
  L.scratch = L.mfma ? mrt::round256(mrt::bwd_bf16_scratch_bytes(pl.kp, pl.ntq_total)) : 0;
  const bool stats = L.mfma && mrt::bwd_bf16_r_fits(pl.kp) && mrt::bf16_stage_l_out_streams(pl.kp);
  L.rowsO = stats ? mrt::round256((size_t)pl.Nq * pl.kp.d * sizeof(float)) : 0;
  L.rowsL = stats ? mrt::round256((size_t)pl.Nq * sizeof(float)) : 0;
  L.per_head = L.off_lse() + L.rowsL;
  return L;
}
mrt_status bwd_plan(const mrt_problem* p, int b1, int b2, int tile, int iters, int causal_chunk,
                    mrt::Plan* pl) {
  mrt_status st = mrt::make_plan(p, b1, b2, tile, iters, causal_chunk, pl);
  if (st != MRT_OK) return st;
  // the fp32 kernels take blocks whose buffers fit LDS; beyond that only shapes that run on the
  // bf16 matrix unit in every stage
  const bool all_mfma = p->dtype == MRT_BF16 && p->compute == MRT_COMPUTE_DEFAULT &&
                        mrt::bwd_bf16_fits(pl->kp) && mrt::bwd_bf16_r_fits(pl->kp);
  if (!mrt::bwd_fits(b1, b2, p->head_dim) && !all_mfma) {
    mrt::set_error("backward pass: blocks (%d,%d) at head_dim %d exceed this build's on-chip buffers", b1, b2,
                   p->head_dim);
    return MRT_ERR_UNSUPPORTED;
  }
  if (iters > 16) { mrt::set_error("backward pass supports at most 16 iterations"); return MRT_ERR_UNSUPPORTED; }
  return MRT_OK;
}
}  // namespace

size_t monarch_attn_bwd_workspace_min_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters) {
  mrt::Plan pl;
  if (bwd_plan(p, b1, b2, tile, iters, 0, &pl) != MRT_OK) return 0;
  return bwd_layout(pl, p).per_head;
}

size_t monarch_attn_bwd_workspace_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters) {
  mrt::Plan pl;
  if (bwd_plan(p, b1, b2, tile, iters, 0, &pl) != MRT_OK) return 0;
  const size_t per = bwd_layout(pl, p).per_head, budget = size_t(16) << 30;
  size_t heads = (size_t)pl.B * pl.kp.H;
  if (per * heads > budget) heads = budget / per > 0 ? budget / per : 1;
  return per * heads;
}

}  // extern "C"

namespace {
// What a call of the backward machinery does: everything (monarch_attn_bwd), only the forward
// intermediates plus O (monarch_attn_fwd_save), or only the reverse sweep over intermediates a
// monarch_attn_fwd_save call left in the workspace (monarch_attn_bwd_saved).
enum BwdMode { kBwdAll, kBwdForwardOnly, kBwdSweepOnly };

mrt_status bwd_run(BwdMode mode, const void* Q, const void* K, const void* V, void* O, const void* dO,
                   float* dQ, float* dK, float* dV, const mrt_problem* p, int b1, int b2, int tile,
                   int iters, int causal_chunk, void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace mrt;
  Plan pl;
  mrt_status st = bwd_plan(p, b1, b2, tile, iters, causal_chunk, &pl);
  if (st != MRT_OK) return st;
  if (!Q || !K || !V || !workspace) { set_error("Q, K, V and workspace must be non-NULL"); return MRT_ERR_NULL; }
  if (mode == kBwdForwardOnly ? !O : (!dO || !dQ || !dK || !dV)) {
    set_error(mode == kBwdForwardOnly ? "O must be non-NULL" : "dO, dQ, dK and dV must be non-NULL");
    return MRT_ERR_NULL;
  }
  if ((uintptr_t)workspace % 256) { set_error("workspace must be 256-byte aligned"); return MRT_ERR_WORKSPACE; }
  const BwdLayout L = bwd_layout(pl, p);
  if (L.mfma) {
    const void* ptrs[2] = {Q, mode == kBwdForwardOnly ? (const void*)O : dO};
    for (const void* q : ptrs)
      if ((uintptr_t)q % 16) { set_error("bf16 path needs 16-byte aligned tensors"); return MRT_ERR_SHAPE; }
  }
  // intermediates handed from one call to the next: every (batch, head) stays in the workspace
  const size_t need = mode == kBwdAll ? L.per_head : L.per_head * (size_t)pl.B * pl.kp.H;
  if (workspace_bytes < need) {
    if (mode == kBwdAll)
      set_error("workspace has %zu bytes, the backward pass of one (batch,head) needs %zu", workspace_bytes, need);
    else
      set_error("workspace has %zu bytes, keeping the intermediates of every (batch,head) needs %zu",
                workspace_bytes, need);
    return MRT_ERR_WORKSPACE;
  }
  const int BH = pl.B * pl.kp.H, T = pl.T;
  const bool bf16_ops = p->dtype == MRT_BF16 && p->compute == MRT_COMPUTE_DEFAULT;
  // every stage on the matrix unit: the forward intermediates can then be bf16 as well
  const bool ws_bf16 = L.mfma && bwd_bf16_r_fits(pl.kp);
  const int G = (int)(workspace_bytes / L.per_head < (size_t)BH ? workspace_bytes / L.per_head : (size_t)BH);
  hipStream_t s = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  // array X of the pass starts at base + off_X * G (every array holds G heads back to back)
  auto arr = [&](size_t off) { return base + off * (size_t)G; };

  // array X of heads [lo, ..) of the pass: every array has room for rowsD (or rowsS) bytes per
  // head; a kernel launched for a group of heads packs them from its base at the stride of what it
  // stores, and so do the groups, so that a head's place does not depend on how the heads were
  // grouped (the call that saves the intermediates and the one that reads them may group differently)
  const size_t headD = L.rows * (size_t)pl.kp.d * (ws_bf16 ? 2 : 4), headS = L.rows * sizeof(float);
  const size_t headO = (size_t)pl.Nq * pl.kp.d * sizeof(float), headL = (size_t)pl.Nq * sizeof(float);
  auto arrD = [&](size_t off, int lo) { return arr(off) + headD * (size_t)lo; };
  auto arrS = [&](size_t off, int lo) { return arr(off) + headS * (size_t)lo; };

  // the whole backward pass of heads [bh0 + lo, bh0 + hi) of a pass, on stream gs
  auto run_heads = [&](int bh0, int lo, int hi, hipStream_t gs) -> mrt_status {
    const int nbh = hi - lo;
    KParams kp = pl.kp;
    kp.Q = Q; kp.K = K; kp.V = V; kp.O = mode == kBwdForwardOnly ? O : nullptr;
    kp.bh0 = bh0 + lo; kp.m0 = 0; kp.ntq = pl.ntq_total;
    kp.Y = arrD(L.off_Y(), lo);
    hipError_t e;
    // forward intermediates of every iteration (the last iteration's stage L only when O is asked
    // for): by the bf16 forward kernels when every backward stage runs on the matrix unit (the
    // arrays then hold bf16), else by the fp32 kernels
    for (int t = 1; t <= T && mode != kBwdSweepOnly; ++t) {
      kp.aL = arrD(L.off_aL(t), lo);
      kp.cL = (float*)arrS(L.off_cL(t), lo);
      kp.aR = t >= 2 ? arrD(L.off_aR(t), lo) : nullptr;
      kp.cmx_out = nullptr; kp.cinv_out = nullptr;
      e = ws_bf16 ? launch_bf16_stage_r(kp, nbh, t == 1, t == T, gs)
                  : launch_f32_stage_r(kp, pl.dtype, nbh, t == 1, t == T, gs);
      if (e != hipSuccess) return hip_fail(e, "backward: forward stage R launch");
      if (t < T) {
        kp.aR = arrD(L.off_aR(t + 1), lo);
        kp.cmx_out = (float*)arrS(L.off_cmx(t + 1), lo);
        kp.cinv_out = (float*)arrS(L.off_cinv(t + 1), lo);
        e = ws_bf16 ? launch_bf16_stage_l(kp, nbh, false, gs) : launch_f32_stage_l(kp, pl.dtype, nbh, false, gs);
        if (e != hipSuccess) return hip_fail(e, "backward: forward stage L launch");
      } else if (mode == kBwdForwardOnly) {
        kp.cmx_out = nullptr; kp.cinv_out = nullptr;
        // the streamed kernel also leaves the rows' log-sum-exp and O in fp32 for the backward call
        if (L.rowsL) {
          kp.lse_out = (float*)(arr(L.off_lse()) + headL * (size_t)lo);
          kp.o32_out = (float*)(arr(L.off_o32()) + headO * (size_t)lo);
        }
        e = ws_bf16 ? launch_bf16_stage_l(kp, nbh, true, gs) : launch_f32_stage_l(kp, pl.dtype, nbh, true, gs);
        kp.lse_out = nullptr; kp.o32_out = nullptr;
        if (e != hipSuccess) return hip_fail(e, "forward stage L launch");
      }
    }
    if (mode == kBwdForwardOnly) return MRT_OK;
    kp.aL = arrD(L.off_aL(T), lo);
    kp.cL = (float*)arrS(L.off_cL(T), lo);
    kp.aR = T >= 2 ? arrD(L.off_aR(T), lo) : nullptr;
    kp.cmx_out = nullptr; kp.cinv_out = nullptr;
    // reverse sweep
    BwdParams bp;
    memset(&bp, 0, sizeof(bp));
    bp.k = kp;
    bp.dO = dO;
    bp.daL = (float*)arrD(L.off_daL(), lo);
    bp.dcL = (float*)arrS(L.off_dcL(), lo);
    bp.dY = (float*)arrD(L.off_dY(), lo);
    bp.dA = (float*)arrD(L.off_dA(), lo);
    bp.dQ = dQ; bp.dK = dK; bp.dV = dV;
    // (64 < b2 <= 96 runs on the matrix unit only with a bf16 workspace, i.e. when stage L does too)
    const bool r_mfma = bf16_ops && bwd_bf16_r_fits(bp.k) && (bp.k.b2 <= 64 || ws_bf16);
    bp.dq_from_r = (r_mfma && kp.ntk == 1) ? 1 : 0;
    bp.dA1_bf16 = (r_mfma && ws_bf16) ? 1 : 0;
    if (mode == kBwdSweepOnly && L.rowsL) {
      bp.lse = (const float*)(arr(L.off_lse()) + headL * (size_t)lo);
      bp.o32 = (const float*)(arr(L.off_o32()) + headO * (size_t)lo);
    }
    for (int t = T; t >= 1; --t) {
      const bool last = t == T;
      bp.k.aL = arrD(L.off_aL(t), lo);
      bp.k.cL = (float*)arrS(L.off_cL(t), lo);
      bp.Anext = last ? nullptr : (const float*)arrD(L.off_aR(t + 1), lo);
      bp.cmx = last ? nullptr : (const float*)arrS(L.off_cmx(t + 1), lo);
      bp.cinv = last ? nullptr : (const float*)arrS(L.off_cinv(t + 1), lo);
      bp.accumulate = last ? 0 : 1;
      e = L.mfma ? launch_bwd_bf16_stage_l(bp, nbh, last, ws_bf16, arr(L.off_scratch()) + L.scratch * (size_t)lo, gs)
                 : launch_bwd_stage_l(bp, pl.dtype, nbh, last, gs);
      if (e != hipSuccess) return hip_fail(e, "backward stage L launch");
      bp.k.aR = t >= 2 ? arrD(L.off_aR(t), lo) : nullptr;
      e = r_mfma ? launch_bwd_bf16_stage_r(bp, nbh, t == 1, last, ws_bf16, gs)
                 : launch_bwd_stage_r(bp, pl.dtype, nbh, t == 1, last, gs);
      if (e != hipSuccess) return hip_fail(e, "backward stage R launch");
    }
    if (!bp.dq_from_r && (e = launch_bwd_q_first(bp, nbh, gs)) != hipSuccess)
      return hip_fail(e, "backward dQ launch");
    return MRT_OK;
  };

  // Heads are independent: as in the forward call, a pass may be cut into head groups whose kernel
  // chains run on helper streams forked from and joined back to the caller's stream, so that the
  // part-filled last round of one group's launch overlaps another group's kernels.  It pays for
  // long calls whose stage L launches are a small multiple of what the chip holds (KV-cache
  // shapes); otherwise the pass runs on the caller's stream.
  int want_groups = requested_groups(p);
  if (want_groups == 0) {
    // stage L backward keeps two workgroups per compute unit resident for b1 <= 96, one beyond:
    // groups pay while a launch is fewer than four rounds of them (measured: 12 heads of the 480p
    // KV-cache step -10 %, 10 heads per pass of the 720p one +5 %)
    const long long l_wgs = (long long)pl.ntq_total * pl.kp.b2 * G, slots = pl.kp.b1 <= 96 ? 512 : 256;
    want_groups = (L.rowsD * (size_t)G >= (size_t(256) << 20) && l_wgs < 4 * slots) ? 2 : 1;
  }
  StreamPool* pool = (g_prof_on.load() || want_groups <= 1) ? nullptr : get_pool();
  std::unique_lock<std::mutex> pool_lock;
  if (pool) pool_lock = std::unique_lock<std::mutex>(pool->in_use);
  mrt_status status = MRT_OK;
  for (int bh0 = 0; bh0 < BH && status == MRT_OK; bh0 += G) {
    const int nbh = BH - bh0 < G ? BH - bh0 : G;
    int ngroups = pool ? (nbh < want_groups ? nbh : want_groups) : 1;
    if (ngroups > 1) {
      if (hipEventRecord(pool->fork, s) != hipSuccess) ngroups = 1;
      for (int gi = 1; gi < ngroups; ++gi)
        if (hipStreamWaitEvent(pool->side[gi - 1], pool->fork, 0) != hipSuccess) status = MRT_ERR_HIP;
      if (status != MRT_OK) { set_error("helper stream fork failed"); break; }
    }
    // the heads are split evenly (the forward call's uneven split, which lets the larger group's
    // stage L launches fill the chip exactly once, does not carry over: the streamed stage L backward
    // kernel holds one workgroup per compute unit; 12 heads of the 480p KV-cache step: 6 + 6 1.76 ms,
    // 9 + 3 1.82, 4 + 8 1.84, 10 + 2 1.93)
    // The saving forward call runs the forward kernels only and takes the forward call's split.
    int first_group = 0;
    if (mode == kBwdForwardOnly && ngroups == 2) {
      const long long wgs_per_head = (long long)pl.ntq_total * pl.kp.b2;
      const int per_round = (int)(2LL * compute_units() / (wgs_per_head > 0 ? wgs_per_head : 1));
      if (per_round < nbh && 2 * per_round >= nbh) first_group = per_round;
    }
    for (int gi = 0; gi < ngroups && status == MRT_OK; ++gi) {
      int lo = (int)((long long)nbh * gi / ngroups), hi = (int)((long long)nbh * (gi + 1) / ngroups);
      if (first_group > 0) { lo = gi == 0 ? 0 : first_group; hi = gi == 0 ? first_group : nbh; }
      status = run_heads(bh0, lo, hi, gi == 0 ? s : pool->side[gi - 1]);
    }
    // join even after a failed launch, so that the helper streams never run ahead of the caller
    for (int gi = 1; gi < ngroups; ++gi) {
      if (hipEventRecord(pool->join[gi - 1], pool->side[gi - 1]) != hipSuccess ||
          hipStreamWaitEvent(s, pool->join[gi - 1], 0) != hipSuccess) {
        if (status == MRT_OK) { set_error("helper stream join failed"); status = MRT_ERR_HIP; }
      }
    }
  }
  return status;
}
}  // namespace

extern "C" {

mrt_status monarch_attn_bwd(const void* Q, const void* K, const void* V, const void* dO, float* dQ,
                            float* dK, float* dV, const mrt_problem* p, int b1, int b2, int tile,
                            int iters, int causal_chunk, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  return bwd_run(kBwdAll, Q, K, V, nullptr, dO, dQ, dK, dV, p, b1, b2, tile, iters, causal_chunk, workspace,
                 workspace_bytes, hip_stream);
}

size_t monarch_attn_bwd_saved_workspace_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters) {
  mrt::Plan pl;
  if (bwd_plan(p, b1, b2, tile, iters, 0, &pl) != MRT_OK) return 0;
  return bwd_layout(pl, p).per_head * (size_t)pl.B * pl.kp.H;
}

mrt_status monarch_attn_fwd_save(const void* Q, const void* K, const void* V, void* O, const mrt_problem* p,
                                 int b1, int b2, int tile, int iters, int causal_chunk, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  return bwd_run(kBwdForwardOnly, Q, K, V, O, nullptr, nullptr, nullptr, nullptr, p, b1, b2, tile, iters,
                 causal_chunk, workspace, workspace_bytes, hip_stream);
}

mrt_status monarch_attn_bwd_saved(const void* Q, const void* K, const void* V, const void* dO, float* dQ,
                                  float* dK, float* dV, const mrt_problem* p, int b1, int b2, int tile,
                                  int iters, int causal_chunk, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
  return bwd_run(kBwdSweepOnly, Q, K, V, nullptr, dO, dQ, dK, dV, p, b1, b2, tile, iters, causal_chunk,
                 workspace, workspace_bytes, hip_stream);
}

mrt_status dense_attn_check(const mrt_problem* p, int causal_chunk) {
  mrt_status st = check_common(p);
  if (st != MRT_OK) return st;
  if (causal_chunk < 0) { set_error("causal_chunk < 0"); return MRT_ERR_SHAPE; }
  return MRT_OK;
}

mrt_status dense_attn_fwd(const void* Q, const void* K, const void* V, void* O,
                          const mrt_problem* p, int causal_chunk, void* hip_stream) {
  mrt_status st = dense_attn_check(p, causal_chunk);
  if (st != MRT_OK) return st;
  if (!Q || !K || !V || !O) { set_error("Q, K, V and O must be non-NULL"); return MRT_ERR_NULL; }
  const bool f32 = p->dtype == MRT_F32 || p->compute == MRT_COMPUTE_F32;
  if (!f32) {
    const void* ptrs[4] = {Q, K, V, O};
    for (const void* q : ptrs)
      if ((uintptr_t)q % 16) { set_error("bf16 path needs 16-byte aligned tensors"); return MRT_ERR_SHAPE; }
  }
  KParams kp;
  memset(&kp, 0, sizeof(kp));
  kp.Q = Q; kp.K = K; kp.V = V; kp.O = O;
  kp.qs = p->q; kp.ks = p->k; kp.vs = p->v; kp.os = p->o;
  kp.H = p->heads; kp.d = p->head_dim;
  kp.Nq = p->f_q * p->h * p->w; kp.Nkv = p->f_kv * p->h * p->w; kp.hw = p->h * p->w;
  kp.cc = causal_chunk; kp.qoff = p->q_frame_offset; kp.scale = p->scale;
  const int BH = p->batch * p->heads;
  hipError_t e = timed_launch((hipStream_t)hip_stream, MRT_KERNEL_DENSE, [&] {
    return f32 ? launch_f32_dense(kp, p->dtype, BH, (hipStream_t)hip_stream)
               : launch_bf16_dense(kp, BH, (hipStream_t)hip_stream);
  });
  if (e != hipSuccess) return hip_fail(e, "dense launch");
  return MRT_OK;
}

#ifdef MRT_TRACE
int mrt_debug_set_trace(void* buf, size_t stride_bytes) {
  mrt::g_trace_base = (char*)buf;
  mrt::g_trace_stride = stride_bytes;
  mrt::g_trace_next = 0;
  return 0;
}
#endif

void mrt_set_head_groups(int n) { g_max_groups.store(n < 0 ? 0 : (n > kMaxGroups ? kMaxGroups : n)); }

void mrt_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on.store(on < 0 ? 0 : (on > 64 ? 64 : on));
}

int mrt_profile_read(float* ms, int* kind, int capacity) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int n = 0;
  for (ProfRecord& r : g_prof) {
    float t = -1.f;
    if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&t, r.a, r.b) == hipSuccess)
      t /= (float)r.reps;
    if (n < capacity) { ms[n] = t; kind[n] = r.kind; ++n; }
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof.clear();
  return n;
}

}  // extern "C"
