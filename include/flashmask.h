/*
 * flashmask.h -- C ABI of the MI355X (gfx950) FlashMask attention library.
 *
 * FlashMask (arXiv 2410.01359) describes an attention mask by four int32
 * vectors over the key columns: query row i may NOT attend to key column j iff
 *     LTS[j] <= i < LTE[j]   or   UTS[j] <= i < UTE[j]
 * (Section 4.1; rows and columns 0-based, intervals half-open, an interval with
 * start >= end is empty, any int32 value is accepted).  The library computes
 * exactly the dense-mask attention of Equations 1-2 and its gradients
 * (Algorithms 1 and 2, Section 4.4), skipping tiles that the per-block min/max
 * tables of Section 4.2 prove fully masked.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller and must stay
 *     valid until the stream has run past the call.  The library allocates and
 *     frees nothing, creates no streams and never synchronises the host: work
 *     is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns at once.
 *   - q, k, v, out, dout, dq, dk, dv: bf16, contiguous [B, H, N, d], d innermost.
 *   - lts, lte, uts, ute: int32, contiguous [B, N]; one mask per batch row,
 *     shared by all heads.
 *   - lse, and the library's own D vector: fp32 [B, H, N].
 *   - d must be 64 or 128; N is any positive length (a length that is not a
 *     multiple of 128 costs one small extra launch that pads the bound
 *     vectors inside the workspace); tensor pointers must be 16-byte aligned.
 *   - Outputs are overwritten in full.
 *   - Return value: FM_OK (0) or a negative FM_ERR_* code.  Only conditions the
 *     host can see are checked; bound VALUES live on the device and are not
 *     validated (the comparison above is defined for every int32).
 *   - Calls on different streams need different workspaces.
 *   - Calls may be recorded into a HIP graph (no allocation, no host synchronisation, and the only
 *     clears of global memory are kernels).  The first call of a kernel variant on a device raises
 *     that kernel's dynamic-LDS limit (hipFuncSetAttribute): issue one call of the same shape class
 *     (d, aligned or ragged N, contiguous or _ex) outside the capture first.
 */
#ifndef FLASHMASK_H
#define FLASHMASK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  FM_OK = 0,
  FM_ERR_NULL = -1,      /* a required pointer is NULL */
  FM_ERR_SHAPE = -2,     /* B, H, N <= 0, d not in {64,128}, sizes beyond 32-bit indexing, bad block size */
  FM_ERR_ALIGN = -3,     /* a tensor pointer is not 16-byte aligned */
  FM_ERR_WORKSPACE = -4, /* workspace is NULL or smaller than flashmask_workspace_bytes() */
  FM_ERR_HIP = -5,       /* a kernel launch failed; see flashmask_last_hip_error() */
  FM_ERR_ARG = -6,       /* unknown pass id, scale <= 0 or not finite */
  FM_ERR_STATIC_LIMIT = -7 /* flashmask_fwd_noalloc: the problem does not fit the library's static scratch */
};

/* Pass ids for flashmask_workspace_bytes / flashmask_tile_shape. */
enum {
  FM_PASS_FWD = 0,      /* forward tile loop (Algorithm 1) */
  FM_PASS_BWD_DKDV = 1, /* backward, column-parallel dK/dV loop (Algorithm 2) */
  FM_PASS_BWD_DQ = 2,   /* backward, row-parallel dQ loop (Algorithm 2's dQ update, run per query block) */
  FM_PASS_BWD = 3       /* whole backward call (workspace query only) */
};

/* Tile-class byte written by flashmask_classify (Equation 4).
 * Low two bits: kind.  Bits 4 / 5: a partially masked tile needs the element
 * mask of the lower-triangle pair / of the upper-triangle pair. */
enum {
  FM_TILE_UNMASKED = 0,
  FM_TILE_PARTIAL = 1,
  FM_TILE_FULLY = 2,
  FM_TILE_NEED_LT = 1 << 4,
  FM_TILE_NEED_UT = 1 << 5
};

/*
 * Forward pass: Algorithm 1 (its outputs O and L), i.e. Equations 1-2 with
 * S = scale * Q K^T, masked scores = -inf, out = softmax(S) V and
 * lse_i = log sum_j exp(S_ij) (natural log, of the scaled scores).
 * A query row whose keys are all masked gets out = 0 and lse = -inf.
 *
 *   q, k, v        in   bf16 [B,H,N,d]
 *   lts..ute       in   int32 [B,N]
 *   scale          in   multiplies Q K^T (1/sqrt(d) in the paper's Equation 1); must be
 *                       positive and finite (FM_ERR_ARG otherwise)
 *   out            out  bf16 [B,H,N,d]
 *   lse            out  fp32 [B,H,N]
 *   workspace      scratch of at least flashmask_workspace_bytes(FM_PASS_FWD, ...)
 *                  bytes, 256-byte aligned; contents undefined afterwards.
 */
int flashmask_fwd(const void* q, const void* k, const void* v,
                  const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                  float scale, void* out, float* lse,
                  int B, int H, int N, int d,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward pass: Algorithm 2.  Given the forward's out and lse and the upstream
 * gradient dout, writes dq, dk, dv (bf16 [B,H,N,d]):
 *   P = exp(S - lse), dV = P^T dO, dP = dO V^T, D_i = sum_c dO_ic O_ic,
 *   dS = P o (dP - D), dQ = scale dS K, dK = scale dS^T Q.
 * Rows with lse = -inf contribute nothing and get dq = 0.
 * The dQ accumulation runs per query block in a fixed order, so results are
 * bit-reproducible run to run (the paper's kernel needs a switch for that,
 * Section 5.2).
 *   workspace: at least flashmask_workspace_bytes(FM_PASS_BWD, ...) bytes.
 */
int flashmask_bwd(const void* q, const void* k, const void* v,
                  const void* out, const float* lse, const void* dout,
                  const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                  float scale, void* dq, void* dk, void* dv,
                  int B, int H, int N, int d,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * flashmask_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic,
 * kernels and results as flashmask_fwd, but the scratch (min/max tables, work counts, unit queues,
 * padded bound vectors) lives in a static device array inside the library instead of a caller's
 * workspace.  The call allocates and frees nothing.
 *   - Limit: flashmask_workspace_bytes(FM_PASS_FWD, B, H, N, d) must not exceed
 *     FLASHMASK_NOALLOC_SCRATCH_BYTES (4 MiB: about 250 000 row blocks of 128 queries over all batch
 *     rows and heads, e.g. B*H = 512 at N = 65536); larger problems return FM_ERR_STATIC_LIMIT and
 *     launch nothing.  Each GPU the library runs on holds its own copy of the array until the process
 *     ends.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress) and, like
 *     flashmask_fwd, raises the tile loop's dynamic-LDS limit: issue one call outside a capture first.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU
 *     (different streams or threads) race.  Calls on one stream, or otherwise ordered, are fine; the
 *     array's contents carry nothing from one call to the next.
 */
#define FLASHMASK_NOALLOC_SCRATCH_BYTES (4u << 20)
int flashmask_fwd_noalloc(const void* q, const void* k, const void* v,
                          const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                          float scale, void* out, float* lse,
                          int B, int H, int N, int d, void* hip_stream);

/*
 * Layout of a bf16 tensor indexed [batch][head][row][d] for the *_ex entry points: distances, in
 * ELEMENTS, between consecutive batches, heads and rows; d itself is contiguous.  A tensor stored
 * [B,N,H,d] has {N*H*d, d, H*d}; a slice of a packed [B,N,3,H,d] projection has {N*3*H*d, d, 3*H*d}.
 * Every stride must be a multiple of 8 (16-byte vectors along d), row >= d and < 2^24
 * (FM_ERR_ALIGN / FM_ERR_SHAPE otherwise).
 */
typedef struct {
  int64_t batch, head, row;
} flashmask_strides;

/*
 * The forward and backward passes above for tensors that are not contiguous [B,H,N,d], and for
 * grouped K/V heads (the inference shape of the paper's Appendix, 32 query heads on 8 K/V heads):
 * k, v (and dk, dv) have H_kv heads, H % H_kv == 0, and query head h attends to K/V head
 * h / (H / H_kv); dk, dv are summed over the query heads of a group.  Same arithmetic, same
 * workspace size (flashmask_workspace_bytes with H), same error behaviour; lse stays fp32
 * contiguous [B,H,N].  Outputs must not overlap inputs or each other.
 *   forward : sq, sk, sv, so describe q, k, v, out
 *   backward: strides[8] describe q, k, v, out, dout, dq, dk, dv in this order
 */
int flashmask_fwd_ex(const void* q, const void* k, const void* v,
                     const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                     float scale, void* out, float* lse,
                     int B, int H, int H_kv, int N, int d,
                     const flashmask_strides* sq, const flashmask_strides* sk,
                     const flashmask_strides* sv, const flashmask_strides* so,
                     void* workspace, size_t workspace_bytes, void* hip_stream);
int flashmask_bwd_ex(const void* q, const void* k, const void* v,
                     const void* out, const float* lse, const void* dout,
                     const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                     float scale, void* dq, void* dk, void* dv,
                     int B, int H, int H_kv, int N, int d,
                     const flashmask_strides* strides,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of scratch a call of the given pass needs (FM_PASS_FWD or FM_PASS_BWD).
 * Returns 0 for an invalid shape or pass.  Host-only, no device work. */
size_t flashmask_workspace_bytes(int pass, int B, int H, int N, int d);

/*
 * Preprocessing step of Section 4.2 (Algorithm 1 "precompute the min and max
 * row index"): for every block of block_c key columns, the max and min of each
 * bound vector.
 *   minmax  out  int32 [B, 8, T_c], T_c = ceil(N / block_c), rows in the order
 *                LTStart^max, LTStart^min, LTEnd^max, LTEnd^min,
 *                UTStart^max, UTStart^min, UTEnd^max, UTEnd^min.
 * block_c must be a positive multiple of 32; any N > 0 is accepted here (a
 * ragged last block covers the columns that exist).
 */
int flashmask_preprocess(const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                         int B, int N, int block_c, int32_t* minmax, void* hip_stream);

/*
 * Tile classification of Equation 4, as the skip tests and element-mask tests
 * of Algorithm 1 apply it, for every tile of block_r rows x block_c columns:
 * with r0 = i*block_r, r1 = min(r0 + block_r, N),
 *   fully(X)   = r0 >= XStart^max_j and r1 <= XEnd^min_j
 *   partial(X) = r1 >  XStart^min_j and r0 <  XEnd^max_j      X in {LT, UT}
 *   class = FULLY if fully(LT) or fully(UT); else PARTIAL | NEED_X bits if any
 *   partial(X); else UNMASKED.
 *   minmax  in   int32 [B, 8, T_c] as written by flashmask_preprocess
 *   cls     out  uint8 [B, T_r, T_c]
 * The attention kernels evaluate the same predicate on the fly; this entry
 * point exists so the tables can be checked bit for bit.
 */
int flashmask_classify(const int32_t* minmax, int B, int N, int block_r, int block_c,
                       uint8_t* cls, void* hip_stream);

/*
 * The tile scheduler's output for one pass (not in the paper; it is what balances skewed masks over
 * the chip), exported so that it can be checked like the tables above.  Work units are row blocks
 * (FM_PASS_FWD, FM_PASS_BWD_DQ) or key blocks (FM_PASS_BWD_DKDV) of the pass's tile shape, numbered
 * (b * H + h) * T + block.  They are dealt to 8 queues; slot s belongs to queue s % 8 and holds the
 * (s / 8)-th unit that queue hands out:
 *   records  out  int32 [slots, 4] = {unit or -1 (no unit), first block of the unit's live range,
 *                 one past its last (0, 0 if every tile of the unit is fully masked), 0}
 *   slots    out  HOST int: number of slots (a multiple of 8, >= B * H * T); with records == NULL
 *                 the call only reports it.
 * Every unit appears exactly once; tiles outside a unit's live range are fully masked (Equation 4).
 * Slices (b, h) go to queues whole, slice b * H + h to queue (b * H + h) % 8, while they fill rounds
 * of 8; the slices left over are shared block by block between 2, 4 or 8 queues.  A queue holds its
 * whole slices in groups of two, one group after the other, then its part of the shared slices;
 * within a group the units holding at least an eighth of the largest possible work come first, by
 * falling work, then the lighter ones by falling octave of work.  workspace as for the pass
 * (FM_PASS_FWD for the forward, FM_PASS_BWD otherwise); the records are copied out of it on the
 * stream.  N here is rounded up to a multiple of 128 (T counts blocks of the padded length).
 */
int flashmask_unit_queues(int pass, const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                          int B, int H, int N, int d, int32_t* records, int* slots,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Tile shape (rows x key columns) at which the given pass classifies and skips
 * tiles.  Host-only. */
int flashmask_tile_shape(int pass, int d, int* block_r, int* block_c);

/* Static, human-readable text for an FM_* code. */
const char* flashmask_strerror(int code);

/* Text of the last HIP error behind an FM_ERR_HIP on this thread ("" if none). */
const char* flashmask_last_hip_error(void);

/*
 * Measurement aid (not part of the paper's method): register `count` HOST
 * handles of already-created hipEvent_t objects.  While registered, every
 * flashmask_fwd / flashmask_bwd call records them on its stream between its
 * internal launches, so a benchmark can time one kernel inside the call:
 *   forward : [0] entry, [1] after preprocessing + unit queues, [2] after the tile loop
 *   backward: [0] entry, [1] after preprocessing + unit queues, [2] after the dQ loop (whose
 *             prologue is the D pre-pass), [3] after the dK/dV loop
 * The array must stay valid until cleared with (NULL, 0).  Process-global and
 * not thread-safe; entries that are NULL or beyond `count` are skipped.
 */
int flashmask_profile_events(void** events, int count);

/*
 * Measurement aid (not part of the paper's method): the matrix-core rate this chip reaches on its own.
 * Launches `workgroups` workgroups of 4 waves that do nothing but bf16 matrix-core instructions (the
 * 32x32x16 one the tile loops use, four independent accumulation chains per wave) on the operands given,
 * so a benchmark can time it with events on `hip_stream` and put the tile loops' rate next to what the
 * matrix cores deliver at the clock and power they hold by themselves (Section 5.4 of the paper quotes
 * its kernels against a theoretical peak; this is the measured counterpart).
 *   operands  in   device, 16 KiB of bf16 values, 16-byte aligned.  What they hold matters: the chip's
 *                  sustained clock depends on switching activity (zeros run at the nominal clock, random
 *                  values do not)
 *   sink      out  device, fp32 [workgroups * 256]
 *   iters     in   loop trips; each trip is 32 instruction slots per wave
 *   shape     in   0: the 32x32x16 instruction the tile loops use; 1: the 16x16x32 one (two per slot,
 *                  same floating-point operations), for comparison; 2: shape 0 with, per instruction,
 *                  the side work the forward loop has per matrix instruction (one 128-bit LDS operand
 *                  read, four fp32 multiply-adds, one exponential, all independent): the rate of the
 *                  loop's instruction mix under perfect scheduling
 *   flop      out  HOST double: floating-point operations of the launch
 */
int flashmask_mfma_ceiling(const void* operands, float* sink, int workgroups, int iters, int shape, double* flop,
                           void* hip_stream);

/*
 * Measurement aid (not part of the paper's method): the rate at which this chip takes the dQ update of
 * Algorithm 2 as the paper's column-parallel loop issues it -- every tile of the loop adds a 64 x 128
 * fp32 block into dQ in HBM.  `workgroups` workgroups each add `tiles` such blocks into
 *   acc  in/out  device fp32 [heads][n_tiles][64][128] (zero it first if the sums matter)
 * with no-return fp32 atomic adds, a head's adds all coming from one XCD.  A benchmark times the launch
 * with events; `bytes` (HOST double) receives the bytes of fp32 updates issued.  The backward here
 * computes dQ in a second, row-parallel loop instead, because this rate caps a fused loop far below
 * the matrix-core rate.
 */
int flashmask_atomic_ceiling(float* acc, int heads, int n_tiles, int tiles, int workgroups, double* bytes,
                              void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHMASK_H */
