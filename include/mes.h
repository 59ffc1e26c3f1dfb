/*
 * mes.h -- C ABI of the MI355X (gfx950) mixed-precision delta linear layer.
 *
 * The operation is the serving hot path of ME-Switch (arXiv 2406.09041): every
 * expert's weight is the shared pre-trained W_base plus a delta (Section 3,
 * "delta = W_FT - W").  The delta's non-salient input channels are quantised to
 * b = 1..4 bits with one step size per output channel (Eq. 1, Section 4.1), its k
 * salient input channels stay in fp16 (Section 4.1, "Salient-aware delta
 * selection", Eq. 2), and inference is decoupled as y = x W + x Delta~ (Eq. 4),
 * batched across experts.
 *
 * Orientation: nn.Linear style.  W[d_out, d_in], y = x W^T.  A "step per output
 * channel" is one float per ROW of the delta, a "salient input channel" is one
 * COLUMN.  (The paper writes W[m, n] with m input channels.)
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer unless its comment says HOST.
 *  - The library never allocates or frees device memory.  The hot call
 *    (mes_delta_linear) never synchronises; the offline calls that must report a
 *    device-side check (mes_pack_delta) synchronise `stream` once before returning.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - All calls return a mes_status; mes_last_error() gives a thread-local message
 *    for the last non-OK status.  All argument checks run on the host before any
 *    HIP call.
 *  - Shapes: d_in % 8 == 0 and d_out % 4 == 0 (row starts of x / y stay 16-byte /
 *    8-byte aligned).  Stored matrices are zero padded to d_out_pad = ceil64(d_out),
 *    d_in_pad = ceil128(d_in), k_pad = ceil32(k).
 *
 * Storage layouts (tile-major, so that one 64-lane wavefront reads contiguous
 * memory and holds a matrix-core operand without any shuffle).  A "lane slot" is
 * lane = 16 g + r: r = row inside a 16-row tile, g = one of four column groups.
 *  - base:    uint16 (bf16 bits) [d_in_pad/128][d_out_pad/16][4][64 lanes][8], chunk-major:
 *             all row tiles of one 128-column chunk are contiguous;
 *             slot (c, jt, kb, lane, e) holds W[16 jt + r][128 c + 32 kb + 8 g + e].
 *  - salient: uint16 (fp16 bits) [d_out_pad/16][k_pad/32][64][8];
 *             slot (jt, sb, lane, e) holds fp16(Delta[16 jt + r][S[32 sb + 8 g + e]]).
 *  - codes:   blocks of 16 rows x 128 columns, [d_in_pad/128][d_out_pad/16] (chunk-major
 *             like the base), 256 b bytes each.  Inside block (c, jt) the lane 16 g + r owns
 *             row 16 jt + r and the 32 columns 128 c + 32 g + e, e = 8 q + p (q < 4, p < 8).
 *             Codes sit in 4-bit fields (field p of a 32-bit word = bits [4 p, 4 p + 4)) so
 *             that one AND turns a word into eight fp4 (E2M1) matrix-core inputs:
 *               b = 1: uint32 [64 lanes]; code of element (q, p) at bit 4 p + q.
 *               b = 2: uint32 [64 lanes][2 w]; code of element (q, p) in word w = q / 2 at
 *                      bits [4 p + 2 (q % 2), + 2).
 *               b = 3: the b = 2 block holding the low two code bits (512 bytes), followed
 *                      by a b = 1 block holding the high code bit (256 bytes).
 *               b = 4: the b = 2 block holding the low two code bits (512 bytes), followed
 *                      by a b = 2 block holding the high two code bits (512 bytes).
 *             Codes of salient columns, padding columns and padding rows are 0.
 *    The code u is unsigned; the weight it stands for is (u - z) * step[row] with
 *    z = 2^(b-1) - 1/2 (MES_GRID_SYM) or 2^(b-1) (MES_GRID_EQ1, Eq. 1's levels).
 */
#ifndef MES_H
#define MES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MES_OK = 0,
  MES_ERR_NULL = 1,      /* a required pointer is NULL                               */
  MES_ERR_SHAPE = 2,     /* non-positive / unsupported / mismatching dimensions      */
  MES_ERR_BITS = 3,      /* bits not in {1,2,3,4}, or a grid/step policy it excludes   */
  MES_ERR_SALIENT = 4,   /* k out of range, or salient_idx not ascending / in range  */
  MES_ERR_SEGMENTS = 5,  /* seg_offsets not 0 = o[0] <= ... <= o[E] = T              */
  MES_ERR_ALIGN = 6,     /* a pointer is not 16-byte aligned                         */
  MES_ERR_WORKSPACE = 7, /* workspace missing or too small                           */
  MES_ERR_DEVICE = 8     /* a HIP call failed (message carries the HIP error string) */
} mes_status;

/* Quantisation grid (Eq. 1 and its symmetric variant). */
enum { MES_GRID_SYM = 0, MES_GRID_EQ1 = 1 };
/* Where the per-output-channel step comes from.  GIVEN: the caller's (e.g. learned by the
 * distillation of Eq. 3); MAXABS: Eq. 1's initialisation max|X| / D over the non-salient
 * columns of the row, D = 2^(b-1) - 1/2 (SYM) or 2^(b-1) - 1 (EQ1); MEANABS: b = 1 only,
 * step = 2 * mean|X| (XNOR-Net scale). */
enum { MES_STEP_GIVEN = 0, MES_STEP_MAXABS = 1, MES_STEP_MEANABS = 2 };

#define MES_MAX_EXPERTS 64
#define MES_MAX_FUSED 3        /* linear layers one mes_delta_linear_multi call may serve */
#define MES_LAYOUT_VERSION 3

/* One expert's compressed delta for one linear layer (all pointers DEVICE, caller-owned). */
typedef struct {
  int32_t d_in, d_out, k, bits, grid, layout_version;
  const void* codes;          /* mes_codes_bytes(d_in, d_out, bits) bytes, 16-byte aligned      */
  const float* step;          /* [d_out], 16-byte aligned                                       */
  const void* salient;        /* mes_salient_bytes(d_out, k) bytes of fp16, 16-byte aligned     */
  const int32_t* salient_idx; /* [k] strictly ascending, 0 <= idx < d_in (may be NULL if k = 0) */
} mes_delta;

/* One linear layer of a mes_delta_linear_multi call (HOST struct; pointers as commented). */
typedef struct {
  const void* w_base_tiled;   /* DEVICE: output of mes_pack_base for this layer's [d_out, d_in]        */
  const mes_delta* experts;   /* HOST array [n_experts]; descriptor pointers are DEVICE                */
  void* y;                    /* DEVICE: bf16 [T, d_out] row-major, fully overwritten                  */
} mes_linear;

/* ---- sizes (pure host arithmetic; 0 on invalid arguments) ------------------------------------ */
size_t mes_base_bytes(int d_in, int d_out);              /* tiled bf16 base                     */
size_t mes_codes_bytes(int d_in, int d_out, int bits);   /* packed low-bit codes of one expert  */
size_t mes_salient_bytes(int d_out, int k);              /* tiled fp16 salient columns          */
size_t mes_pack_workspace_bytes(void);
size_t mes_select_workspace_bytes(int n, int d_in, int d_out);
/* Workspace of mes_delta_linear / _multi.  Tokens are streamed in groups of 64 and one launch serves as many groups
 * as the workspace has slices for: one slice for max_tokens <= 64, two for <= 128, four above that (a slice: the
 * group's prepared activations, gathered salient activations and split-column partial sums).  A larger workspace
 * than a call needs is fine; a smaller one (at least one slice) is accepted and costs launches, not correctness.
 * Asked for with max_tokens >= 192 it also includes room for the long-segment
 * path (the segment's activations re-tiled, about 4 d_in bytes per token, and up to 64 MiB of partial sums): an
 * expert segment of 192 tokens or more is then computed as one dense product x (W + Delta~)^T (Eq. 4 before
 * decoupling; the expert's effective weight is formed in registers, block by block, as a matrix-core operand),
 * which for long segments is several times faster than streaming the weights once per 64 tokens.  A workspace
 * sized with a smaller max_tokens is accepted by every call and keeps it on the streaming path. */
size_t mes_linear_workspace_bytes(int d_in, int d_out, int max_tokens);
int mes_long_segment_tokens(void);   /* the segment length from which the one-product path is taken (192) */
size_t mes_linear_multi_workspace_bytes(int d_in, const int32_t* d_out /*HOST [n_linears]*/, int n_linears, int max_tokens);
const char* mes_last_error(void);
int mes_layout_version(void);

/* Re-tile the shared base weight (Eq. 4's W) for the kernels.  Offline.
 * w: bf16 [d_out, d_in] row-major.  w_tiled_out: mes_base_bytes() bytes, fully overwritten. */
mes_status mes_pack_base(const void* w, int d_in, int d_out, void* w_tiled_out, void* stream);
/* Inverse of mes_pack_base (test / debug). */
mes_status mes_unpack_base(const void* w_tiled, int d_in, int d_out, void* w_out, void* stream);

/* Salient input-channel selection (Section 4.1, Eq. 2).  Offline.
 * score_i = sum_t sum_j (x_ti D_ji - x_ti Dhat_ji)^2 with Dhat the b-bit quantisation of the
 * whole delta (no salient set, step policy `step_policy`, never GIVEN); the k channels with
 * the largest score are returned ascending (ties: the lower index wins).  fp64 arithmetic.
 * delta: fp32 [d_out, d_in]; x_calib: fp32 [n, d_in]; idx_out: int32 [k];
 * score_out: double [d_in] or NULL; workspace >= mes_select_workspace_bytes(n, d_in, d_out). */
mes_status mes_select_salient(const float* delta, const float* x_calib, int n, int d_in, int d_out,
                              int bits, int grid, int step_policy, int k, int32_t* idx_out,
                              double* score_out, void* workspace, size_t workspace_bytes, void* stream);

/* Compress one expert's delta (Eq. 1 per output channel; salient columns kept in fp16).  Offline.
 * delta: fp32 [d_out, d_in].  salient_idx: int32 [k] ascending (NULL if k = 0); checked on the
 * device, MES_ERR_SALIENT if not strictly ascending or out of range (outputs then undefined).
 * step_in: [d_out] for MES_STEP_GIVEN (entries that are not > 0 become 0), else ignored.
 * Outputs, fully overwritten: codes_out (mes_codes_bytes), step_out [d_out] fp32,
 * salient_out (mes_salient_bytes).  A row whose step is 0 stores code 2^(b-1) everywhere.
 * Quantisation arithmetic is fp64: t = delta / step; SYM: u = clamp(floor(t) + 2^(b-1));
 * EQ1: u = clamp(rint(t), -2^(b-1), 2^(b-1) - 1) + 2^(b-1).
 * workspace >= mes_pack_workspace_bytes().  Synchronises `stream` once before returning. */
mes_status mes_pack_delta(const float* delta, int d_in, int d_out, const int32_t* salient_idx, int k,
                          int bits, int grid, int step_policy, const float* step_in, void* codes_out,
                          float* step_out, void* salient_out, void* workspace, size_t workspace_bytes,
                          void* stream);

/* Expand a compressed delta (test / debug).  delta_hat_out: fp32 [d_out, d_in] = Delta~ of Eq. 4
 * ((u - z) * step rounded once to fp32; fp16 values at salient columns) or NULL.
 * codes_out: uint8 [d_out, d_in] (0xFF at salient columns) or NULL. */
mes_status mes_unpack_delta(const mes_delta* d, float* delta_hat_out, uint8_t* codes_out, void* stream);

/* The hot path (Eq. 4, batched across experts):
 *   y[t] = x[t] W_base^T + step_e .* (x_ns[t] (U_e - z)^T) + x_s[t] D_e^T,   e = expert of row t.
 * w_base_tiled: output of mes_pack_base for [d_out, d_in].
 * experts: HOST array [n_experts] (1 <= n_experts <= MES_MAX_EXPERTS) of descriptors whose
 *          pointers are DEVICE; all must share d_in, d_out, k, bits, grid.  Read during the call only.
 * x: bf16 [T, d_in] row-major, rows sorted by expert.  seg_offsets: HOST int32 [n_experts + 1],
 *    0 = o[0] <= o[1] <= ... <= o[E] = T; rows o[e]..o[e+1] use expert e; an expert with an
 *    empty segment costs no memory traffic.
 * y: bf16 [T, d_out] row-major, fully overwritten (round-to-nearest-even from fp32 accumulators).
 * workspace: >= mes_linear_workspace_bytes(d_in, d_out, T), 16-byte aligned, contents irrelevant (scratch: nothing
 *    is kept in it between calls); calls sharing a workspace must be stream-ordered.
 * T = 0 returns MES_OK without touching anything.  Enqueues on `stream`, never synchronises. */
mes_status mes_delta_linear(const void* w_base_tiled, const mes_delta* experts, int n_experts,
                            const void* x, int T, const int32_t* seg_offsets, void* y,
                            void* workspace, size_t workspace_bytes, void* stream);

/* The same hot path for several linear layers that read the SAME activations and routing (Eq. 4 applied to
 * each layer; e.g. the query / key / value projections, or the gate / up projections, of one block): one
 * preparation of x and one streaming launch serve all of them, y_l[t] = x[t] (W_l + Delta~_{l,e})^T.
 * linears: HOST array [n_linears], 1 <= n_linears <= MES_MAX_FUSED.  Every layer has its own base, its own
 * n_experts expert deltas (with their own salient channels) and its own output; d_out may differ between
 * layers, d_in, k, bits and grid must be the same for all layers and experts.
 * x, T, seg_offsets, stream, T = 0: as for mes_delta_linear.
 * workspace: >= mes_linear_multi_workspace_bytes(d_in, d_out[], n_linears, T), as for mes_delta_linear.
 * With n_linears = 1 this is mes_delta_linear. */
mes_status mes_delta_linear_multi(const mes_linear* linears, int n_linears, int n_experts, const void* x, int T,
                                  const int32_t* seg_offsets, void* workspace, size_t workspace_bytes, void* stream);

/* mes_delta_linear for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * mes_delta_linear, except that the per-call scratch lives in a device-resident static array of
 * mes_noalloc_scratch_bytes() bytes (64 MiB; every GPU the library runs on holds its own copy until the process
 * ends) instead of a caller-owned workspace.  The call works on the device that is current when it is made
 * (`stream` must belong to it), allocates and frees nothing, never synchronises, and returns MES_ERR_WORKSPACE
 * if a layer of this shape needs more scratch than the array holds (mes_linear_workspace_bytes(d_in, d_out, 1)
 * > mes_noalloc_scratch_bytes(); every Mistral-7B shape fits).  All calls on one GPU share that GPU's array:
 * they must be stream-ordered, calls that overlap on one GPU race. */
size_t mes_noalloc_scratch_bytes(void);
mes_status mes_delta_linear_noalloc(const void* w_base_tiled, const mes_delta* experts, int n_experts,
                                    const void* x, int T, const int32_t* seg_offsets, void* y, void* stream);

/* ---- gated MLP input: h = SiLU(y_gate) * y_up, element by element --------------------------------------------
 * The models the method is evaluated on (Section 5: Mistral-7B, LLaMA-2-13B) use a gated MLP: its down projection
 * reads SiLU(gate_proj(x)) * up_proj(x), SiLU(v) = v / (1 + exp(-v)).  y_gate and y_up are two mes_delta_linear
 * results (Eq. 4) over the same x and routing; this call computes both in one pass (like mes_delta_linear_multi)
 * and writes only h: bf16 [T, d_out], DEVICE, 16-byte aligned, rows in the order of x.  y_gate and y_up are NOT
 * rounded to bf16 on the way: SiLU and the product are taken in fp32 on the fp32 sums, h is rounded once.
 * The two layers must agree in d_in, d_out, k, bits and grid; each has its own base, experts and salient sets.
 * All tokens take the streaming path (there is no long-segment route here).  Arguments otherwise as for
 * mes_delta_linear; workspace >= mes_gated_workspace_bytes(d_in, d_out, max_tokens) (max_tokens as for
 * mes_linear_workspace_bytes: <= 64, <= 128 or more decide how many 64-token groups one launch may hold). */
size_t mes_gated_workspace_bytes(int d_in, int d_out, int max_tokens);
mes_status mes_delta_linear_gated(const void* w_gate_tiled, const mes_delta* gate_experts, const void* w_up_tiled,
                                  const mes_delta* up_experts, int n_experts, const void* x, int T,
                                  const int32_t* seg_offsets, void* h, void* workspace, size_t workspace_bytes,
                                  void* stream);

/* ---- on-demand swapping (Section 4.1, "On-demand swapping": the base model stays on the GPU, the compressed
 * deltas of the experts a batch needs are loaded when they are needed) ----------------------------------------
 * A pool serves one linear layer (mes_pool_create) or several, up to MES_POOL_MAX_LINEARS -- e.g. the seven of a
 * transformer block (mes_pool_create_multi: arrays d_in, d_out, k of n_linears entries; bits and grid are common).
 * It owns nothing but its bookkeeping: the caller gives it a DEVICE arena of n_slots * slot bytes (256-byte
 * aligned).  A slot holds one expert's packed deltas of all the pool's linears, one after the other
 * (mes_pool_multi_slot_bytes = sum of the linears' mes_pool_slot_bytes; linear l starts mes_pool_linear_offset
 * bytes into the slot); inside a linear's part the codes, steps, salient tile and salient indices sit at the
 * offsets mes_pool_slot_layout reports (offsets_out[4], in that order; its return value is mes_pool_slot_bytes).
 * Up to n_experts experts are registered, their packed data in PINNED HOST memory that stays valid and
 * unchanged while registered:
 *   mes_pool_register_blob: ONE host buffer of slot bytes, 16-byte aligned, laid out exactly like a slot (the
 *     buffers mes_pack_delta writes, copied to the offsets above).  A miss is then one host-to-device copy.
 *   mes_pool_register (single-linear pools only): the four buffers separately; a miss is four copies.
 * Not thread-safe: one thread drives a pool, always with the same copy stream.
 *
 * mes_pool_acquire_multi(pool, experts[n], out, ...): makes the n distinct experts resident and writes their
 * descriptors to out (HOST array [n_linears][n]: linear-major, within a linear in the order asked).  An expert
 * already in a slot is a hit.  A miss overwrites the least recently used slot that holds none of this request's
 * experts (never-used slots first, lowest slot index among equals; "used" = handed out by an acquire or filled
 * by a prefetch) with asynchronous copies on `copy_stream`; these copies start only after everything enqueued on
 * `compute_stream` so far (a kernel may still read the slot), and `compute_stream` is made to wait for them --
 * and for any prefetch into a slot it hands out -- so work enqueued on it after the call sees the new contents.
 * The descriptors are valid until the next acquire.  n > n_slots is MES_ERR_SHAPE.  If a copy cannot be issued
 * the call fails with MES_ERR_DEVICE and nothing it loaded counts as resident.
 * mes_pool_acquire: the same for a single-linear pool (out[n]).
 *
 * mes_pool_prefetch(pool, experts[n], n_loaded, copy_stream): starts loading those of the n experts that are not
 * resident, WITHOUT making any stream wait for the copies: a later acquire of them is a hit (and does the
 * waiting).  Only slots the latest acquire did not hand out, and no prefetch since has filled, are overwritten,
 * least recently used first; the copies start after the compute stream's position at that latest acquire, i.e.
 * they run under the kernels of the current batch.  Experts for which no such slot is left are skipped (they
 * will be misses of their acquire); *n_loaded (may be NULL) = how many copies were started.
 *
 * A pool created with dry_run != 0 does the bookkeeping only (no GPU call): for tests of the policy.
 * mes_pool_stats: hits and misses of the acquires, and payload bytes copied (prefetches included) since
 * creation (any pointer may be NULL); mes_pool_prefetched: experts loaded by prefetches. */
#define MES_POOL_MAX_LINEARS 8
typedef struct mes_pool mes_pool;
size_t mes_pool_slot_bytes(int d_in, int d_out, int k, int bits);
size_t mes_pool_slot_layout(int d_in, int d_out, int k, int bits, size_t offsets_out[4]);
size_t mes_pool_multi_slot_bytes(int n_linears, const int32_t* d_in, const int32_t* d_out, const int32_t* k, int bits);
mes_status mes_pool_create(int d_in, int d_out, int k, int bits, int grid, int n_slots, int n_experts, void* arena,
                           size_t arena_bytes, int dry_run, mes_pool** out);
mes_status mes_pool_create_multi(int n_linears, const int32_t* d_in, const int32_t* d_out, const int32_t* k, int bits,
                                 int grid, int n_slots, int n_experts, void* arena, size_t arena_bytes, int dry_run,
                                 mes_pool** out);
void mes_pool_destroy(mes_pool* pool);
size_t mes_pool_linear_offset(const mes_pool* pool, int linear);
mes_status mes_pool_register(mes_pool* pool, int expert, const void* codes, const float* step, const void* salient,
                             const int32_t* salient_idx);
mes_status mes_pool_register_blob(mes_pool* pool, int expert, const void* host_blob);
mes_status mes_pool_acquire(mes_pool* pool, const int32_t* experts, int n, mes_delta* out, void* copy_stream,
                            void* compute_stream);
mes_status mes_pool_acquire_multi(mes_pool* pool, const int32_t* experts, int n, mes_delta* out, void* copy_stream,
                                  void* compute_stream);
mes_status mes_pool_prefetch(mes_pool* pool, const int32_t* experts, int n, int* n_loaded, void* copy_stream);
int mes_pool_slot_of(const mes_pool* pool, int expert);   /* slot the expert is resident in, or -1 */
mes_status mes_pool_stats(const mes_pool* pool, uint64_t* hits, uint64_t* misses, uint64_t* bytes_copied);
uint64_t mes_pool_prefetched(const mes_pool* pool);

/* ---- learning the step sizes (Section 4.1, "Efficient distillation", taken layer by layer; straight-through
 * estimator of Section 3 for Eq. 1).  Offline. -----------------------------------------------------------------
 * The delta weights are frozen and only the step s_j of every output channel is learned, by pulling the
 * compressed layer towards the full-precision fine-tuned one on calibration activations x [n_tokens, d_in]
 * (bf16).  The base product is common to both and cancels; per output channel j
 *     r_tj = sum_i x_ti (Dtilde_ji(s_j) - delta_ji)      Dtilde of Eq. 4: b-bit columns at step s_j, fp16 salient
 *     loss_j = 1/2 sum_t r_tj^2
 *     grad_j = sum_t r_tj sum_{i not salient} x_ti ((u_ji - z) - [delta_ji / s_j inside the grid] delta_ji / s_j)
 * (for bits = 1 the code does not depend on s_j: the bracket is always 0).  The codes u are decided exactly as
 * mes_pack_delta decides them (floor / round-half-even of the exact quotient).  Arithmetic: the two operand
 * matrices are formed in fp32 and rounded to bf16, products accumulate in fp32 on the matrix cores, the sums over
 * tokens are fp32 in a fixed order (results are reproducible run to run).
 * delta: fp32 [d_out, d_in], 16-byte aligned.  salient_idx: int32 [k] ascending as for mes_pack_delta (entries
 * outside [0, d_in) are ignored), NULL if k = 0.  step: fp32 [d_out], 16-byte aligned; rows whose step is not > 0
 * report loss 0 and grad 0.  loss_out, grad_out: fp32 [d_out], fully overwritten.  n_tokens >= 0.
 * workspace >= mes_step_grad_workspace_bytes(d_in, d_out, n_tokens), 16-byte aligned.  Never synchronises. */
size_t mes_step_grad_workspace_bytes(int d_in, int d_out, int n_tokens);
mes_status mes_step_grad(const float* delta, int d_in, int d_out, const int32_t* salient_idx, int k, int bits, int grid,
                         const float* step, const void* x, int n_tokens, float* loss_out, float* grad_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/* One AdamW update (decoupled weight decay; the optimiser Section 5 names for this training) of n step sizes, in
 * place, fp32: m = beta1 m + (1 - beta1) g; v = beta2 v + (1 - beta2) g^2;
 * step = step (1 - lr weight_decay) - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).  t >= 1 is the
 * number of this update.  step, grad, m, v: DEVICE fp32 [n]; m and v start at 0. */
mes_status mes_step_adamw(float* step, const float* grad, float* m, float* v, int n, int t, float lr, float beta1,
                          float beta2, float eps, float weight_decay, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MES_H */
