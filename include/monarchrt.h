/*
 * monarchrt.h -- C ABI of the MonarchRT attention forward operator for AMD MI355X (gfx950).
 *
 * The library computes, for every (batch, head) independently, the MonarchAttention
 * output of App. A of the MonarchRT paper (arXiv 2602.12271):
 *
 *   regular Monarch (App. A.1, Alg. 1): factors L[j,k,l] (b2 blocks of b1 x b1) and
 *   R[k,j,i] (b1 blocks of b2 x b2) of  M[(l*b2+j),(k*b2+i)] = L[j,l,k] R[k,j,i]  (Sec. 4.2)
 *   are refined for T alternating iterations (R: softmax over i of beta_R / c_R;
 *   L: softmax over k of beta_L - c_L), then O = L (R V);
 *
 *   tiled Monarch (Sec. 4.2, App. A.2, Alg. 2): the same per pair of (query tile m,
 *   key tile n) with tile-local block sizes (b1, b2), the softmax of L taken jointly
 *   over all visible key tiles and key rows (n, k).
 *
 * Token order is row-major (frame, height, width) (App. B.1).  Blocks are one of the six aligned
 * choices of Sec. 4.1 (mrt_assignment): every video axis goes as a whole to the b1 side ("rows",
 * index x) or to the b2 side ("columns", index y); the default gives (frame, height) to b1 and
 * width to b2.  A tile is b1 consecutive rows by b2 consecutive columns (Alg. 2, the
 * "(a l b j)" split): row x = a*b1 + l, column y = b*b2 + j; for the default assignment
 * token = x*w + y.
 *
 * All data pointers are DEVICE pointers owned by the caller.  The library allocates
 * no device memory, orders its kernels after the work already on the given HIP stream and
 * before anything enqueued on it later, and returns without synchronising.  Entry points return a status code; nothing is thrown across the ABI.
 * All argument checks happen on the host before the first launch.
 */
#ifndef MONARCHRT_H
#define MONARCHRT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MRT_OK = 0,
  MRT_ERR_NULL = 1,        /* a required pointer is NULL                               */
  MRT_ERR_SHAPE = 2,       /* batch/heads/head_dim/grid/stride values out of range      */
  MRT_ERR_BLOCK = 3,       /* (b1,b2) do not tile the grids as required                 */
  MRT_ERR_UNSUPPORTED = 4, /* valid in the paper, not built here (see each entry point) */
  MRT_ERR_WORKSPACE = 5,   /* workspace smaller than monarch_attn_workspace_min_bytes   */
  MRT_ERR_HIP = 6          /* a HIP call or kernel launch reported an error             */
} mrt_status;

typedef enum { MRT_F32 = 0, MRT_BF16 = 1 } mrt_dtype;

/* Arithmetic used inside the kernels.
 *   MRT_COMPUTE_DEFAULT : f32 storage -> fp32 arithmetic throughout;
 *                         bf16 storage -> bf16 MFMA operands, fp32 accumulation and softmax.
 *   MRT_COMPUTE_F32     : fp32 arithmetic and fp32 intermediates whatever the storage type
 *                         (slow; a device-side cross-check). */
typedef enum { MRT_COMPUTE_DEFAULT = 0, MRT_COMPUTE_F32 = 1 } mrt_compute;

/* Aligned block assignments (Sec. 4.1).  The axes before the underscore index the b1 side, those
 * after it the b2 side, the first-named axis slowest: e.g. MRT_ASSIGN_FW_H has row index
 * x = frame*w + column-of-the-frame and column index y = height.  rows x cols per grid of f frames:
 * FH_W f*h x w, W_FH w x f*h, FW_H f*w x h, H_FW h x f*w, F_HW f x h*w, HW_F h*w x f. */
typedef enum {
  MRT_ASSIGN_FH_W = 0, MRT_ASSIGN_W_FH = 1, MRT_ASSIGN_FW_H = 2,
  MRT_ASSIGN_H_FW = 3, MRT_ASSIGN_F_HW = 4, MRT_ASSIGN_HW_F = 5
} mrt_assignment;

/* Element strides of one [batch, heads, tokens, head_dim] tensor; head_dim is contiguous. */
typedef struct {
  long long batch, head, token;
} mrt_strides;

typedef struct {
  int batch, heads;
  int head_dim;        /* multiple of 32, 32..128                                          */
  int f_q, f_kv;       /* frames of the query grid and of the key/value grid               */
  int h, w;            /* height and width of both grids; N_q = f_q*h*w, N_kv = f_kv*h*w    */
  int q_frame_offset;  /* absolute frame of query frame 0 inside the kv grid (mask only)    */
  mrt_strides q, k, v, o;
  mrt_dtype dtype;     /* storage type of Q, K, V and O                                     */
  mrt_compute compute;
  float scale;         /* multiplies both logit contractions (beta_R and beta_L);
                          1.0 is the paper's softmax(Q K^T) (Sec. 2.2)                      */
  mrt_assignment assignment; /* which axes index the b1 and the b2 side; 0 = (fh, w)        */
  int tile_h;          /* 0: a tile is b1 consecutive block-grid rows.  n_h > 0 (tiled calls with
                          the (fh, w) assignment only): a tile is the neighbourhood of Sec. 4.2,
                          n_h grid rows of each of n_f = b1 / n_h consecutive frames          */
  int head_groups;     /* head groups this call runs concurrently (1..4); 0 = the process-wide
                          default of mrt_set_head_groups, which itself defaults to automatic   */
} mrt_problem;

/* Checks a MonarchRT call without touching the GPU (same rules monarch_attn_fwd applies).
 * With rows_q x cols and rows_kv x cols the block grids of the query and key side under
 * p->assignment (the column counts must agree: assignments with the frame axis on the column
 * side need f_q == f_kv):
 *   tile = 0  regular Monarch: needs f_q == f_kv, b1 == rows, b2 == cols.
 *   tile = 1  tiled: (b1,b2) are tile-local; needs rows_q % b1 == 0, rows_kv % b1 == 0,
 *             cols % b2 == 0.  A tile may be any contiguous row range, e.g. several frames or,
 *             with n_f = 1, n_h = b1 rows of one frame (the neighbourhood tiles of Sec. 4.2).
 *   iters >= 1 (R is undefined before the first update, App. A.1).
 *   causal_chunk = 0: no mask.  > 0: frames per autoregressive chunk; needs an assignment whose
 *             slowest row axis is the frame (FH_W, FW_H, F_HW).
 *             tile = 1: a key tile is visible to a query tile iff its chunk is not later than the
 *             query tile's chunk, hidden tile pairs take no part at all; tiles must not straddle
 *             a chunk: b1 divides (rows per frame)*causal_chunk and (rows per frame)*q_frame_offset.
 *             tile = 0: the one tile straddles every chunk; the mask depends on the block rows
 *             (l, k) alone, so it is a support constraint on L: L's softmax over k runs over the
 *             key rows whose frame's chunk is not later than the chunk of query row l's frame
 *             (+ q_frame_offset), and the iteration is otherwise unchanged.
 *   p->tile_h = n_h > 0 selects neighbourhood tiles (n_f, n_h, n_w) = (b1 / n_h, n_h, b2) of
 *             Sec. 4.2: needs tile = 1, assignment (fh, w), n_h | h, n_h | b1, n_f | f_q, n_f | f_kv,
 *             b2 | w, and for a mask n_f | causal_chunk and n_f | q_frame_offset.  Tile rows are
 *             ordered (frame group, row band); with n_h = h or n_f = 1 this is the same tiling as
 *             tile_h = 0.
 *   Limits of this build: b1 <= 192, b2 <= 96 (else MRT_ERR_UNSUPPORTED). */
mrt_status monarch_attn_check(const mrt_problem* p, int b1, int b2, int tile, int iters,
                              int causal_chunk);

/* Smallest workspace (bytes) monarch_attn_fwd accepts: room for the alpha_L, c_L, Y and
 * alpha_R intermediates of ONE row of query tiles of one (batch, head) (App. A; Sec. 4.3 explains
 * why these, unlike L and R, have to live in device memory, and that query chunks can be finished
 * one after the other to cap it: the "mini-sequence" strategy).  Returns 0 if the arguments are
 * invalid. */
size_t monarch_attn_workspace_min_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters);

/* Recommended workspace: one slab per (batch, head), capped at 8 GiB.  Any size from the
 * minimum up is accepted; the library processes as many heads per pass as fit (or, below one
 * head, as many query tile rows of one head), and less per pass means fewer workgroups per launch. */
size_t monarch_attn_workspace_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters);

/* MonarchRT attention forward (Alg. 1 for tile = 0, Alg. 2 for tile = 1).
 *   Q [batch, heads, N_q, head_dim], K, V [batch, heads, N_kv, head_dim], O like Q; device
 *   memory, element strides in p.  O is fully overwritten.  workspace: device memory, 256-byte
 *   aligned, contents undefined on entry and exit.  hip_stream: a hipStream_t (NULL = the
 *   default stream).  Calls sharing a workspace must be ordered on one stream.
 *   Accuracy.  MRT_F32 storage (and MRT_COMPUTE_F32): O differs from the exact result of App. A's
 *   iteration by at most 1e-4 (max-abs) for inputs of unit scale.  MRT_BF16 storage with
 *   MRT_COMPUTE_DEFAULT: the matrix operands (Q, K, V, the probabilities of R and L, alpha_L, Y,
 *   alpha_R / c_R) and O are rounded to bf16, 2^-9 relative each; the roundings of alpha_L and
 *   alpha_R enter the next logits, whose softmaxes amplify them.  For outputs of magnitude <= 1
 *   the error stays within 2e-2 max-abs; it grows with the output's magnitude and with the
 *   sharpness of the softmaxes (logits of standard deviation 3, |O| up to 3.5, three iterations:
 *   up to 6e-2, the error a CPU emulation of exactly these rounding points also shows).  A caller
 *   who needs the plain 2e-2 there selects MRT_COMPUTE_F32.
 *   Thread safety: the call may be issued from several host threads and on several streams at
 *   once (each call with its own workspace).  Calls that run more than one head group share the
 *   device's helper streams; the library serialises their enqueue, so such calls still complete
 *   correctly but their head groups queue behind each other on those streams. */
mrt_status monarch_attn_fwd(const void* Q, const void* K, const void* V, void* O,
                            const mrt_problem* p, int b1, int b2, int tile, int iters,
                            int causal_chunk, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/* For callers that cannot allocate (code under HIP graph capture, serving loops, harnesses that
 * forbid hipMalloc): monarch_attn_fwd with the library's own scratch memory in place of the
 * workspace argument.  The scratch is a 128 MiB array in the library's device image, one copy per
 * GPU, held until the process ends.  The call allocates nothing, creates no stream or event, runs
 * every kernel on hip_stream (one head group) and is otherwise identical to monarch_attn_fwd with
 * a 128 MiB workspace: as many heads, or query tile rows of one head, per pass as fit.  It returns
 * MRT_ERR_WORKSPACE if one query tile row of one (batch, head) needs more than that
 * (monarch_attn_workspace_min_bytes > 134217728).  Nothing has to be cleared between calls: every
 * kernel reads only what an earlier kernel of the same call wrote.  All calls on one GPU share the
 * array, so calls that overlap in time on one GPU (different streams or threads) race; order them
 * on one stream.  The first call on a device looks up the array's address; make that call
 * outside a graph capture. */
mrt_status monarch_attn_fwd_noalloc(const void* Q, const void* K, const void* V, void* O,
                                    const mrt_problem* p, int b1, int b2, int tile, int iters,
                                    int causal_chunk, void* hip_stream);

/* Backward pass: gradients of  sum(O * dO)  with respect to Q, K and V for the O of
 * monarch_attn_fwd with the same arguments, differentiating through every refinement iteration
 * (this is what Monarch finetuning trains through, Sec. 4.3).
 *   dO: device memory, storage type and element strides of O (p->o).  dQ [batch, heads, N_q,
 *   head_dim], dK and dV [batch, heads, N_kv, head_dim]: device memory, fp32, contiguous, fully
 *   overwritten.  Arithmetic: with p->dtype = MRT_BF16 and p->compute = MRT_COMPUTE_DEFAULT the
 *   contractions run on the bf16 matrix unit with fp32 accumulation wherever the blocks fit its
 *   kernels (stage L backward: b1 <= 144 and head_dim 64 or 128, key ranges beyond 96 rows are
 *   streamed; stage R backward: b2 <= 96; if both hold the forward intermediates are recomputed
 *   by the bf16 forward kernels too) and Q, dO must be 16-byte aligned; everything
 *   else, and every call with MRT_FP32 storage or MRT_COMPUTE_F32, runs in fp32.  Gradients of
 *   the bf16 kernels differ from exact ones by up to about 2e-2 of the largest gradient entry
 *   (typically 5e-3; ill-conditioned inputs, where several iterations pass through nearly tied
 *   softmaxes, amplify the rounding of the intermediates beyond that), of the fp32 kernels by
 *   1e-4 of it.  The forward intermediates of every iteration are recomputed
 *   into the workspace first, so nothing has to be kept from the forward call; the workspace
 *   holds whole (batch, head) entries and the library runs as many of them per pass as fit
 *   (workspace rules as for monarch_attn_fwd).
 *   Limits of this build: b1, b2 and head_dim such that the per-workgroup buffers of the fp32
 *   kernels fit the 160 KB of on-chip memory (e.g. b1 <= 96 and b2 <= 80 at head_dim 128), or
 *   such that every stage runs on the bf16 matrix unit (b1 <= 144, b2 <= 96); iters <= 16;
 *   otherwise MRT_ERR_UNSUPPORTED. */
size_t monarch_attn_bwd_workspace_min_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters);
size_t monarch_attn_bwd_workspace_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters);
mrt_status monarch_attn_bwd(const void* Q, const void* K, const void* V, const void* dO, float* dQ,
                            float* dK, float* dV, const mrt_problem* p, int b1, int b2, int tile,
                            int iters, int causal_chunk, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/* The same training step in two calls that hand the intermediates over instead of forming them
 * twice (Sec. 4.3: finetuning runs the operator forward and backward on the same inputs):
 * monarch_attn_fwd_save computes O as monarch_attn_fwd does, with the arithmetic the backward pass
 * uses (bf16 matrix unit where monarch_attn_bwd would use it, fp32 otherwise), and leaves the
 * intermediates of every iteration in `workspace`; monarch_attn_bwd_saved, given the same Q, K, V,
 * arguments and workspace, runs only the reverse sweep and returns the gradients
 * monarch_attn_bwd returns: the same bits, except where the forward call's last stage L ran the
 * streamed bf16 kernel (more than 192 key rows per query tile, or b1 > 128 with more than 96): that
 * kernel also leaves every query row's log-sum-exp and an fp32 copy of O, from which the sweep takes
 * the row statistics of the last iteration (sum_k L dL = dO . O) instead of a pass of its own over
 * the key range, and the gradients then agree to the bf16 rounding of the sweep's operands
 * (within 1e-2 of the largest gradient; the bar against the oracle is the same for both).
 * Arguments, layouts, limits and error behaviour as for
 * monarch_attn_fwd and monarch_attn_bwd, except that the workspace holds every (batch, head) at
 * once: at least monarch_attn_bwd_saved_workspace_bytes() bytes (0: unsupported problem), else
 * MRT_ERR_WORKSPACE.  The caller keeps the workspace untouched between the two calls and orders
 * them (same stream, or an event); monarch_attn_bwd_saved leaves the saved intermediates intact,
 * so it may be called again (another dO) without a new forward call. */
size_t monarch_attn_bwd_saved_workspace_bytes(const mrt_problem* p, int b1, int b2, int tile, int iters);
mrt_status monarch_attn_fwd_save(const void* Q, const void* K, const void* V, void* O, const mrt_problem* p,
                                 int b1, int b2, int tile, int iters, int causal_chunk, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);
mrt_status monarch_attn_bwd_saved(const void* Q, const void* K, const void* V, const void* dO, float* dQ,
                                  float* dK, float* dV, const mrt_problem* p, int b1, int b2, int tile,
                                  int iters, int causal_chunk, void* workspace, size_t workspace_bytes,
                                  void* hip_stream);

/* Dense baseline  O = softmax(scale * Q K^T + mask) V  (Sec. 2.2), flash-style, no workspace.
 * causal_chunk > 0 masks, per token, keys whose frame's chunk is later than the query frame's
 * chunk (query frames offset by q_frame_offset). */
mrt_status dense_attn_check(const mrt_problem* p, int causal_chunk);
mrt_status dense_attn_fwd(const void* Q, const void* K, const void* V, void* O,
                          const mrt_problem* p, int causal_chunk, void* hip_stream);

/* Number of head groups monarch_attn_fwd and monarch_attn_bwd run concurrently: 1..4, or 0 (default) to let the library
 * choose per call (one group unless the launches are long and their grids small).  With more than one
 * group the library forks helper HIP streams from hip_stream and joins them back before it
 * returns, so the call is still ordered like a single operation on hip_stream (and can be
 * captured into a HIP graph from it).  The helper streams and their events are created once per
 * device on first use, at the default priority, and live until the process ends.  This sets the
 * process-wide default; mrt_problem.head_groups > 0 overrides it for one call.  Multi-group calls
 * on one device take turns enqueueing (a mutex held from the fork to the join). */
void mrt_set_head_groups(int n);

/* Per-kernel timing for benchmarks.  mrt_profile_enable(r) with r >= 1 (at most 64) makes the two
 * entry points above issue every kernel launch r times in a row between a pair of HIP events
 * recorded on the launch's stream; r = 0 switches this off.  Every kernel reads only buffers it
 * does not write, so the repeated launches leave the same result; r > 1 spreads the cost of the
 * event pair and of the first dispatch over r launches.  This is the only mode in which the
 * library creates HIP objects, and while it is on head groups run one after the other.
 * mrt_profile_read waits for the recorded events, writes up to `capacity` (elapsed milliseconds
 * per launch, kernel kind) pairs in launch order, forgets them and returns how many it wrote.
 * Kernel kind = one of MRT_KERNEL_STAGE_R / MRT_KERNEL_STAGE_L / MRT_KERNEL_DENSE, or-ed with
 * MRT_KERNEL_FIRST (first iteration: alpha_R is Q itself) and MRT_KERNEL_LAST (last iteration:
 * stage R also forms Y, stage L forms O). */
enum { MRT_KERNEL_STAGE_R = 1, MRT_KERNEL_STAGE_L = 2, MRT_KERNEL_DENSE = 4,
       MRT_KERNEL_FIRST = 16, MRT_KERNEL_LAST = 32 };
void mrt_profile_enable(int repeats);
int mrt_profile_read(float* ms, int* kind, int capacity);

const char* mrt_status_string(mrt_status s);

/* Text of the last error detail recorded on the calling thread ("" if none). */
const char* mrt_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MONARCHRT_H */
