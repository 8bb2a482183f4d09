/*
 * occult.h - C ABI of the MI355X (gfx950) library for the hot path of a collaboration-aware
 * expert-parallel mixture-of-experts layer (Occult, arXiv 2505.13345): the forward pass and the
 * backward pass (data movement, experts' input and weight gradients, routing weights).
 *
 * One GPU's share of the layer: the D devices of expert parallelism are simulated as
 * groups of G = E / D experts on one GPU, the rows they would exchange are packed into
 * per-device segments and counted, nothing crosses GPUs.
 *
 * Conventions for every call
 *  - returns OCCULT_OK (0) or a negative OCCULT_E* code; never throws or aborts;
 *    occult_last_error() gives a thread-local message for the last failure;
 *  - "device ptr" = memory of the current HIP device, "host ptr" = ordinary host memory;
 *  - data calls are asynchronous on the HIP stream passed as `stream` (a hipStream_t cast to
 *    void*; NULL = the default stream), allocate nothing and never synchronise;
 *    the caller owns every buffer and keeps it alive until the stream has passed the call;
 *  - arguments are checked on the host before anything is launched (shape limits below);
 *    NOT checked: `ids` are in range and distinct per token, `expert_pos` is a permutation of
 *    0..E-1.  Router scores should be finite: occult_route reads NaN and -inf as the lowest finite
 *    value and +inf as the highest, so its ids stay distinct and below E and its gates finite;
 *  - rows of x / sfd / epd / y must start 16-byte aligned: (d * element size) % 16 == 0 and
 *    (f * element size) % 16 == 0, base pointers 16-byte aligned.
 *
 * Notation (the paper's): T = tokens in ORI state, SFD = one replica of a token per distinct
 * destination device (the all-to-all payload), EPD = one replica per (token, selected expert).
 * N_sfd = number of SFD rows, N_epd = T * k.  Placement position P of an expert = device * G + slot.
 */
#ifndef OCCULT_H
#define OCCULT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OCCULT_VERSION 100

enum {
  OCCULT_OK = 0,
  OCCULT_EINVAL = -1,     /* an argument value is outside the documented range          */
  OCCULT_ESHAPE = -2,     /* shapes are inconsistent (E % D, n_d * G < k, ...)           */
  OCCULT_EALIGN = -3,     /* a row or pointer is not 16-byte aligned                     */
  OCCULT_ENULLPTR = -4,   /* a required pointer is NULL                                  */
  OCCULT_EWORKSPACE = -5, /* plan memory or workspace is smaller than occult_plan_sizes  */
  OCCULT_EHIP = -6        /* a HIP runtime call or kernel launch reported an error       */
};

enum { OCCULT_F32 = 0, OCCULT_BF16 = 1 };

/* Limits checked by every call. */
#define OCCULT_MAX_E 256
#define OCCULT_MAX_D 64
#define OCCULT_MAX_K 32

typedef void* occult_stream_t; /* a hipStream_t */

/* Layer description.  Plain data; copied by value inside each call. */
typedef struct occult_cfg {
  int32_t T;          /* tokens (ORI rows), >= 0; T * k < 2^31 and T * S < 2^31              */
  int32_t d;          /* hidden size                                                        */
  int32_t f;          /* expert intermediate size                                           */
  int32_t E;          /* routed experts, 1..OCCULT_MAX_E, E % D == 0                        */
  int32_t S;          /* shared experts applied to every token with weight 1 (0 = none)     */
  int32_t k;          /* experts per token, 1..min(E, OCCULT_MAX_K)                          */
  int32_t D;          /* simulated devices, 1..OCCULT_MAX_D                                  */
  int32_t n_d;        /* collaboration pruning (paper Sec. 3.3): 0 = off, else each token may
                         use at most n_d devices, 1..D, and n_d * (E/D) >= k                */
  int32_t prune_mode; /* 1 = keep the n_d devices of highest summed gate score over the
                         token's unpruned top-k; 2 = keep the first n_d distinct devices met
                         walking the unpruned top-k in descending score (Sec. 3.3 wording);
                         3 = expert-similarity-based pruning (Sec. 3.3): devices as in mode 2,
                         then every routed expert outside them is replaced, walking the top-k
                         in descending score, by the first expert of its row of sim_table that
                         sits on a kept device and is neither a routed expert that stays nor an
                         earlier replacement; slots keep the walk order                      */
  int32_t renorm;     /* 1 = gates divided by their sum over the selected k                 */
  int32_t dtype;      /* OCCULT_F32 or OCCULT_BF16: element type of x, weights, sfd, epd, y  */
  int32_t ffn_phase;  /* occult_expert_ffn only: 0 = both products; 1 = only the first (gate/up
                         projections + SwiGLU -> epd_h, h_shared); 2 = only the second (down
                         projection -> epd_y, y_shared).  For pipelining and per-kernel timing.  */
  const int32_t* expert_pos; /* device ptr [E]: placement position of each expert
                                (device = pos / G, slot = pos % G); NULL = contiguous, pos[e] = e */
  const int32_t* sim_table;  /* device ptr [E][E-1], read by occult_route when n_d > 0 and
                                prune_mode == 3: row i = the other experts by descending
                                similarity to i (occult_similarity_table); else may be NULL     */
} occult_cfg_t;

/* Dispatch plan: device tables, caller-allocated (one block of occult_plan_sizes() bytes carved
 * by occult_plan_bind()).  Relation to the paper's re-index matrices (Sec. 3.1, App. A.2):
 *   BRIM_0[j][t]            = tok_sfd_row[t * D + j]                  (global SFD row, -1 absent)
 *   BRIM_1 of device j      : for SFD row r in [dev_offset[j], dev_offset[j+1]) and slot s,
 *                             entry = (EPD row of (r, expert at P = j*G+s)) - exp_offset[j*G], or -1
 *   brim_w                  = epd_gate[EPD row]
 * Orders: SFD rows are device-major and token-ascending inside a device; EPD rows are
 * position-major (device, slot) and SFD-row-ascending inside an expert.                     */
typedef struct occult_plan {
  uint64_t* tok_devmask;  /* [T]        bit j set = token has an expert on device j          */
  int32_t*  dev_count;    /* [D]        SFD rows per device                                  */
  int32_t*  dev_offset;   /* [D+1]      exclusive scan of dev_count; [D] = N_sfd             */
  int32_t*  tok_sfd_row;  /* [T][D]     SFD row of token t on device j, -1 if absent         */
  int32_t*  sfd_token;    /* [T*min(k,D)] token of each SFD row (first N_sfd entries valid)  */
  int32_t*  exp_count;    /* [E]        EPD rows per placement position                      */
  int32_t*  exp_offset;   /* [E+1]      exclusive scan of exp_count; [E] = T*k               */
  int32_t*  pos_expert;   /* [E]        expert id sitting at each placement position         */
  int32_t*  epd_sfd_row;  /* [T*k]      SFD row that feeds each EPD row (replication index)  */
  float*    epd_gate;     /* [T*k]      routing weight of each EPD row                       */
  int32_t*  sfd_epd_rows; /* [T*min(k,D)][min(k,G)] EPD rows of each SFD row, slot-ascending,
                             -1 padded (the merge list of combine stage 1)                   */
  uint64_t* counters;     /* [8]        0: N_sfd, 1: N_epd, 2: T*k (standard replica rows),
                                        3: max dev_count, 4: max exp_count, 5..7: 0          */
} occult_plan_t;

/* Expert weights, device ptrs, element type cfg.dtype, K-contiguous ("out-major"):
 *   w_gate [E+S][f][d], w_up [E+S][f][d], w_down [E+S][d][f]; experts E..E+S-1 are shared. */
typedef struct occult_weights {
  const void* w_gate;
  const void* w_up;
  const void* w_down;
} occult_weights_t;

/* Host-side statistics of one plan (paper Sec. 2.2: C_T = N_sfd / T, the mean replicas per
 * token; byte counts are hidden rows over both trips: dispatch + return). */
typedef struct occult_stats {
  uint64_t n_sfd, n_epd, rows_std;
  uint64_t max_dev_count, max_exp_count;
  uint64_t bytes_occ;   /* 2 * N_sfd * d * element size                                    */
  uint64_t bytes_std;   /* 2 * T * k * d * element size (k replicas per token)             */
  uint64_t bytes_meta;  /* N_sfd * k * 8: ids and gates carried on the first trip          */
  double   c_t;         /* N_sfd / T                                                        */
} occult_stats_t;

int occult_version(void);
const char* occult_last_error(void);

/* Sizes in bytes of the plan block and of the planner's scratch workspace for cfg. Host, pure. */
int occult_plan_sizes(const occult_cfg_t* cfg, size_t* plan_bytes, size_t* workspace_bytes);

/* Carve `plan_mem` (device ptr, 256-byte aligned, >= plan_bytes) into the tables of `out`
 * (host struct).  Host, pure: touches no device memory. */
int occult_plan_bind(const occult_cfg_t* cfg, void* plan_mem, size_t plan_bytes, occult_plan_t* out);

/* Router (paper Eq. 1; Sec. 3.3 routing-score-based pruning).
 * logits [T][E] f32 device ptr (router scores g(x)); outputs ids [T][k] i32 (slot 0 = highest
 * score; equal scores -> lower expert index first) and w [T][k] f32 (softmax over all E experts
 * at the selected ones, divided by their sum if cfg.renorm).  With cfg.n_d > 0 the selection is
 * restricted to n_d devices as described at occult_cfg.  cfg.expert_pos is read when n_d > 0. */
int occult_route(const occult_cfg_t* cfg, const float* logits, int32_t* ids, float* w,
                 occult_stream_t stream);

/* Expert similarity for prune_mode 3 (paper App. "Similarity Table Construction"): the table is
 * built from profiled router scores H [N][E] through their Gram matrix H^T H.
 * occult_similarity_gram adds (accumulate != 0) or writes the Gram matrix of logits [T][E] f32
 * into gram [E][E] f64 (device ptrs), so that batches accumulate; sums run in double precision
 * with atomic adds, so the last bits depend on the order the blocks finish in.
 * occult_similarity_table (host, pure) turns a Gram matrix (host ptr [E][E] f64) into the integer
 * table (host ptr [E][E-1] i32): row i lists the experts j != i by descending
 * (g[i][j]*g[i][j]) / (g[i][i]*g[j][j]), equal values -> lower j first.  Copy it to the device
 * and pass it as cfg.sim_table.  Needs E >= 2 and a positive diagonal. */
int occult_similarity_gram(const occult_cfg_t* cfg, const float* logits, double* gram, int accumulate,
                           occult_stream_t stream);
int occult_similarity_table(const double* gram_host, int32_t E, int32_t* table_host);

/* Router projection, then routing, in one call (paper Eq. 1: g(x) is a single linear projection of the
 * hidden state, followed by Softmax and top-k as in occult_route).  x [T][d] and w_router [E][d]
 * in cfg.dtype (device ptrs, 16-byte aligned; bf16 needs d % 128 == 0); writes the scores
 * logits [T][E] f32 = x w_router^T (f32 accumulation; the summation order is fixed, so the scores
 * are reproducible run to run, but they differ in the last bits from a product summed in
 * another order) and routes them exactly as occult_route would: ids [T][k], w [T][k]. */
int occult_router(const occult_cfg_t* cfg, const void* x, const void* w_router, float* logits,
                  int32_t* ids, float* w, occult_stream_t stream);

/* Planner (paper App. A.2 "Building BRIM_0" / "Building BRIM_1" for all D simulated devices at
 * once; Sec. 2.2 replica count).  ids [T][k] i32, w [T][k] f32 device ptrs; fills every table of
 * `plan`.  `ws` device ptr of >= workspace_bytes.  Bit-reproducible (no atomics). */
int occult_plan(const occult_cfg_t* cfg, const int32_t* ids, const float* w,
                const occult_plan_t* plan, void* ws, size_t ws_bytes, occult_stream_t stream);

/* occult_plan for callers that cannot allocate device memory or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same three kernels with their
 * scratch (the per-block counts) in a device array built into the library, OCCULT_PLAN_STATIC_MAX_BYTES
 * on every GPU the library runs on, held until the process ends.  Allocates nothing and calls no
 * allocating routine; the array's device address is looked up on the first call on each device (make
 * that call outside a capture).  Results are bit-identical to occult_plan.  Layers whose workspace_bytes
 * (occult_plan_sizes) exceed the limit are refused with OCCULT_EWORKSPACE before anything is launched.
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (two
 * streams, two threads) race; the buffer's old contents never matter (each call overwrites what it reads). */
#define OCCULT_PLAN_STATIC_MAX_BYTES (4u << 20)
int occult_plan_static(const occult_cfg_t* cfg, const int32_t* ids, const float* w,
                       const occult_plan_t* plan, occult_stream_t stream);

/* Dispatch ORI -> SFD (paper App. A.2 "Dispatch"): sfd_x[tok_sfd_row[t][j]] = x[t] for every
 * device j of token t.  x [T][d], sfd_x [>= N_sfd][d] (allocate T*min(k,D) rows), device ptrs. */
int occult_dispatch(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* x, void* sfd_x,
                    occult_stream_t stream);

/* Routing metadata of the dispatched rows (paper App. A.2, pipeline: ids and w travel with the
 * hidden rows on the first exchange, and the receiving device builds BRIM_1 from them):
 * sfd_ids[r][:] = ids[t][:] and sfd_w[r][:] = w[t][:] for every SFD row r of token t.
 * ids [T][k] i32, w [T][k] f32, sfd_ids [>= N_sfd][k] i32, sfd_w [>= N_sfd][k] f32, device ptrs
 * (allocate T*min(k,D) rows).  Rows beyond N_sfd are not written. */
int occult_dispatch_meta(const occult_cfg_t* cfg, const occult_plan_t* plan, const int32_t* ids,
                         const float* w, int32_t* sfd_ids, float* sfd_w, occult_stream_t stream);

/* Expert computing (paper App. A.2 "SMM with Scattering" and the GEMM of "SMM with Merging"),
 * SwiGLU experts: for EPD row r of the expert at position P with SFD source row s = epd_sfd_row[r]:
 *   epd_h[r] = silu(W_gate sfd_x[s]) * (W_up sfd_x[s])      [N_epd][f]
 *   epd_y[r] = W_down epd_h[r]                               [N_epd][d]
 * (the SFD -> EPD replication happens in the first product's row gather; the reduction over
 * a device's experts is occult_combine's first stage).  Shared experts, if S > 0:
 *   h_shared[t] = concat_s silu(W_gate,s x[t]) * (W_up,s x[t])   [T][S*f]
 *   y_shared[t] = sum_s W_down,s h_shared[t][s]                   [T][d]
 * x, h_shared, y_shared may be NULL when S == 0.  bf16: MFMA with f32 accumulation, epd_h
 * rounded to bf16; f32: plain f32 arithmetic.  All device ptrs. */
int occult_expert_ffn(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                      const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                      void* h_shared, void* y_shared, occult_stream_t stream);

/* occult_expert_ffn with a scratch buffer, for small batches with shared experts whose down
 * projection alone (few output tiles, K = S*f) leaves most of the chip idle: 24 <= T < 192, unless
 * the batch is one whose shared experts are computed inside the routed experts' two launches
 * anyway (bf16, T <= 128 and fewer than 24 rows per routed expert on average: no scratch, ws_bytes
 * = 0).  Given `ws` (device ptr, 16-byte aligned, >= occult_expert_ffn_ws_bytes() bytes) that
 * product is split over K into f32 partial sums in ws, which a second kernel adds in slice order and
 * rounds once: y_shared then differs from occult_expert_ffn's only by the order of f32 additions;
 * epd_h and epd_y are the same bits.  With ws == NULL, too few bytes, or a layer that does not need
 * it (ws_bytes == 0), identical to occult_expert_ffn.  The contents of ws are not kept between
 * calls and need no initialisation. */
int occult_expert_ffn_ws_bytes(const occult_cfg_t* cfg, size_t* ws_bytes);
int occult_expert_ffn_ws(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                         const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                         void* h_shared, void* y_shared, void* ws, size_t ws_bytes,
                         occult_stream_t stream);

/* Optional repacked weights for decode-shaped batches (paper Sec. 4, decoding: few rows per expert, the
 * expert computation is streaming every active expert's weights once).  Below 24 rows per expert
 * on average the bf16 products run a kernel in which a wave streams its 32 output columns' weights;
 * in the layout of occult_weights_t that is 32 or 64 rows 4 KiB apart, 128 bytes at a time.
 * occult_pack_weights writes the same numbers once (again after every weight update) in the order
 * that kernel reads them, one contiguous stream per wave: `packed` is a device ptr of
 * occult_pack_weights_bytes() bytes (3*(E+S)*d*f elements; 0 for f32, where the call does nothing),
 * 16-byte aligned.  Layout: all gate|up pairs, then all down matrices; per pair, units of 32 output
 * columns; per unit, stages of 64 K elements = 8 blocks of 1 KiB ordered (K step of 32, gate or up,
 * column block of 16); a block is 64 pieces of 16 bytes, piece l = row l%16 of the column block at K
 * offset (l/16)*8; the down matrices likewise with 4 blocks per stage.
 * occult_expert_ffn_packed is occult_expert_ffn_ws reading `packed` wherever that kernel is chosen
 * and `weights` elsewhere (both must hold the same numbers); results are bit-identical to
 * occult_expert_ffn_ws.  packed == NULL: the same call. */
int occult_pack_weights_bytes(const occult_cfg_t* cfg, size_t* bytes);
int occult_pack_weights(const occult_cfg_t* cfg, const occult_weights_t* weights, void* packed,
                        size_t packed_size, occult_stream_t stream);
int occult_expert_ffn_packed(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                             const void* x, const occult_weights_t* weights, const void* packed,
                             void* epd_h, void* epd_y, void* h_shared, void* y_shared, void* ws,
                             size_t ws_bytes, occult_stream_t stream);

/* Two-stage combine (paper Sec. 3.1 two-stage aggregation of Eq. 0; App. A.2 "Weight
 * Modulation", the accumulation of "SMM with Merging", and "Combine").
 * Stage 1 (on the device, before the return trip): sfd_y[r] = sum over the EPD rows q of SFD
 *   row r, in slot order, of epd_gate[q] * epd_y[q] (f32 accumulation, stored in cfg.dtype:
 *   this is the return payload).
 * Stage 2 (after the return trip): y[t] = sum over devices j ascending of
 *   sfd_y[tok_sfd_row[t][j]]  (+ y_shared[t] if not NULL), f32 accumulation.
 * epd_y [N_epd][d], sfd_y [>= N_sfd][d], y [T][d]; device ptrs.  Order-fixed, no atomics. */
int occult_combine(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* epd_y,
                   void* sfd_y, const void* y_shared, void* y, occult_stream_t stream);

/* occult_combine with the paper's own first stage, an atomic merge (paper Sec. 3.1, first-stage merging: thread
 * blocks that write the same SFD rows add with atomic_add into a float32 output tensor that is converted to the
 * target type afterwards; App. A.2 "SMM with Merging").  Opt-in, for measuring it beside the order-fixed default:
 *   mode 0: every EPD row q adds epd_gate[q] * epd_y[q] into sfd_acc[epd_sfd_row[q]] with float32 atomic adds
 *           (sfd_acc: device ptr f32 [>= N_sfd][d], allocate T*min(k,D) rows; its first N_sfd rows are cleared by
 *           the call); then sfd_y[r] = sfd_acc[r] rounded to cfg.dtype and stage 2 exactly as occult_combine;
 *   mode 1: (bf16 layers) the same additions as packed bf16 atomic adds straight into sfd_y (cleared by the call;
 *           one bf16 rounding per addition; sfd_acc may be NULL); stage 2 as occult_combine.
 * The order of the additions into a row is not fixed: results are not bit-reproducible and agree with
 * occult_combine up to float reassociation (bit for bit when every partial sum is exactly representable). */
int occult_combine_atomic(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* epd_y, float* sfd_acc,
                          void* sfd_y, const void* y_shared, void* y, int mode, occult_stream_t stream);

/* Backward pass of the data movement (the paper trains through the layer: Introduction, Sec. 4
 * Training; it prints no backward algorithm, and every forward step here is linear in the hidden
 * rows, so the gradient is the transposed map on the same plan, Sec. 3.1).  Both calls leave the
 * plan untouched and are order-fixed like the forward calls.
 *
 * occult_combine_backward: given dy [T][d] (gradient of occult_combine's y),
 *   sfd_dy[r] = dy[token of SFD row r]                     [>= N_sfd][d]  (transposed stage 2: the
 *               payload of the first backward exchange; exactly occult_dispatch of dy)
 *   epd_dy[q] = epd_gate[q] * dy[token of EPD row q]       [N_epd][d]     rounded to cfg.dtype
 *   dw[t][s]  = < dy[t], epd_y[EPD row of (t, ids[t][s])] >  [T][k] f32    (f32 accumulation)
 * sfd_dy, epd_dy and dw are each optional (NULL = not produced); dw needs epd_y, the expert
 * outputs of the forward pass; ids [T][k] is the routing the plan was built from.  The gradient of
 * y_shared is dy itself.
 *
 * occult_dispatch_backward: given epd_dx [N_epd][d] (gradient of every expert's input row, i.e. of
 * sfd_x[epd_sfd_row[q]] as read by the first product),
 *   sfd_dx[r] = sum over the EPD rows q of SFD row r, slot order, of epd_dx[q]   [>= N_sfd][d]
 *               (f32 accumulation, stored in cfg.dtype: the payload of the backward return trip)
 *   dx[t]     = sum over devices j ascending of sfd_dx[tok_sfd_row[t][j]] (+ dx_shared[t] if not NULL)
 * i.e. the two-stage sum of occult_combine with unit weights. */
int occult_combine_backward(const occult_cfg_t* cfg, const occult_plan_t* plan, const int32_t* ids,
                            const void* dy, const void* epd_y, void* sfd_dy, void* epd_dy, float* dw,
                            occult_stream_t stream);
int occult_dispatch_backward(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* epd_dx,
                             void* sfd_dx, const void* dx_shared, void* dx, occult_stream_t stream);

/* Backward of occult_expert_ffn with respect to the expert inputs (same sources as above; the chain
 * rule through the SwiGLU expert on the same plan).
 *
 * occult_transpose_weights writes the two transposed weight copies the backward products read,
 * device ptrs in cfg.dtype: w_down_t [E+S][f][d] = w_down^T and w_gu_t [E+S][d][2f] = [w_gate^T | w_up^T]
 * side by side.  Call it again whenever the weights change.
 *
 * occult_expert_ffn_backward: for EPD row q of the expert at position P, x_q = sfd_x[epd_sfd_row[q]]:
 *   g = W_gate x_q, u = W_up x_q (recomputed, or as kept by occult_expert_ffn_train when gu_saved = 1;
 *   rounded to cfg.dtype), dh = W_down^T epd_dy[q],
 *   dg = dh * u * silu'(g), du = dh * silu(g), epd_dx[q] = W_gate^T dg + W_up^T du.
 * epd_dy [N_epd][d] is occult_combine_backward's (gate-scaled) output.  Outputs: epd_dx [N_epd][d], and
 * epd_gu [N_epd][2f] = [dg | du] (the operand a weight-gradient product needs); epd_dh [N_epd][f] is
 * scratch.  Shared experts (S > 0; x [T][d], dy [T][d] = gradient of y_shared):
 * gu_shared [T][S*2f] = per shared expert [dg | du], dh_shared [T][S*f] scratch,
 * dx_shared [T][d] = sum over the shared experts of their input gradients (pass it to
 * occult_dispatch_backward); all three may be NULL when S == 0.  Arithmetic as in the forward
 * call: bf16 on MFMA with f32 accumulation, intermediates rounded to bf16; or plain f32. */
int occult_transpose_weights(const occult_cfg_t* cfg, const occult_weights_t* weights, void* w_down_t,
                             void* w_gu_t, occult_stream_t stream);
int occult_expert_ffn_backward(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                               const void* x, const occult_weights_t* weights, const void* w_down_t,
                               const void* w_gu_t, const void* epd_dy, const void* dy, void* epd_gu,
                               void* epd_dh, void* epd_dx, void* gu_shared, void* dh_shared,
                               void* dx_shared, int gu_saved, occult_stream_t stream);

/* Forward pass of a training step: occult_expert_ffn_ws that also keeps the pre-activations, so that
 * the backward pass need not recompute them: epd_gu [N_epd][2f] = [g | u] per EPD row and, with shared
 * experts, gu_shared [T][S*2f] = per shared expert [g | u] (rounded to cfg.dtype).  On 256-row tiles
 * the first product stores them from the same accumulators; the other kernels add two products.
 * Pass gu_saved = 1 to occult_expert_ffn_backward afterwards (it overwrites both with [dg | du]);
 * gu_saved = 0 recomputes g and u there (0.5 GB less memory held between the passes at the prefill
 * size, for about a fifth more backward time). */
int occult_expert_ffn_train(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                            const void* x, const occult_weights_t* weights, void* epd_h, void* epd_y,
                            void* h_shared, void* y_shared, void* epd_gu, void* gu_shared, void* ws,
                            size_t ws_bytes, occult_stream_t stream);

/* Weight gradients of occult_expert_ffn (same sources; f32 outputs in the layout of the weights:
 * dw_gate, dw_up [E+S][f][d], dw_down [E+S][d][f], device ptrs).  For the expert at position P with
 * EPD rows q in [exp_offset[P], exp_offset[P+1]) and x_q = sfd_x[epd_sfd_row[q]]:
 *   dw_down = sum_q epd_dy[q] (x) epd_h[q],  dw_gate = sum_q dg[q] (x) x_q,  dw_up = sum_q du[q] (x) x_q,
 * rows summed in f32 (bf16: MFMA, rows in blocks of 64 in ascending order; order-fixed, no atomics).
 * Inputs: epd_h (and h_shared) as left by occult_expert_ffn, epd_dy by occult_combine_backward,
 * epd_gu = [dg | du] (and gu_shared) by occult_expert_ffn_backward; dy [T][d] serves the shared
 * experts.  accumulate = 0 overwrites the three outputs (experts without rows get zeros), 1 adds to
 * them (gradient accumulation over micro-batches).  A plan built for T == 0 writes zeros / adds nothing. */
int occult_expert_ffn_backward_weights(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                       const void* x, const void* epd_h, const void* h_shared,
                                       const void* epd_dy, const void* dy, const void* epd_gu,
                                       const void* gu_shared, float* dw_gate, float* dw_up, float* dw_down,
                                       int accumulate, occult_stream_t stream);

/* occult_expert_ffn_backward_weights with a scratch buffer.  Shared experts are fewer than 8 groups that each take all
 * T rows: at large T their products have far fewer workgroups (groups x 256 x 256 output tiles) than the chip has
 * compute units.  Given `ws` (device ptr, 16-byte aligned, >= occult_expert_ffn_backward_weights_ws_bytes() bytes) the
 * rows of such a product are cut into up to 8 slices of at least 2048 rows, every slice a workgroup of its own writing
 * an f32 partial product to ws; a second kernel adds the slices in slice order (order-fixed, no atomics) and writes or,
 * with accumulate = 1, adds the sum.  The sums then run in another order than without ws (same bars, other last bits).
 * ws == NULL, too few bytes, or a layer that does not need it (ws_bytes == 0): identical to the call above.  The
 * contents of ws are not kept between calls. */
int occult_expert_ffn_backward_weights_ws_bytes(const occult_cfg_t* cfg, size_t* ws_bytes);
int occult_expert_ffn_backward_weights_ws(const occult_cfg_t* cfg, const occult_plan_t* plan, const void* sfd_x,
                                          const void* x, const void* epd_h, const void* h_shared, const void* epd_dy,
                                          const void* dy, const void* epd_gu, const void* gu_shared, float* dw_gate,
                                          float* dw_up, float* dw_down, int accumulate, void* ws, size_t ws_bytes,
                                          occult_stream_t stream);

/* Gradient of the routing weights with respect to the router scores (paper Eq. 1: Softmax over
 * all E experts, the values at the selected experts, divided by their sum if cfg.renorm; the
 * selection is piecewise constant and has no gradient).  logits [T][E] f32, ids [T][k] as returned
 * by occult_route, dw [T][k] f32 -> dlogits [T][E] f32, all device ptrs; f32 arithmetic. */
int occult_route_backward(const occult_cfg_t* cfg, const float* logits, const int32_t* ids, const float* dw,
                          float* dlogits, occult_stream_t stream);

/* Co-activation counts (paper Preliminary, co-activation graph): C[i][j] = number of tokens
 * whose selected experts include both i and j (diagonal = expert load).  ids [T][k], C [E][E]
 * i32 device ptrs; accumulate = 0 overwrites C, 1 adds to it (profiling over batches). */
int occult_coactivation(const occult_cfg_t* cfg, const int32_t* ids, int32_t* C, int accumulate,
                        occult_stream_t stream);

/* Greedy collaboration-aware placement (paper Sec. 3.2, Algorithm 1) on the host, in integer
 * arithmetic.  C_host [E][E] i32 host ptr (diagonal ignored); needs E % D == 0 and E / D >= 2.
 * Outputs, host ptrs: L_host [D][G] (experts of each device in slot order) and
 * expert_pos_host [E].  Device 0 starts from the most co-activated pair (ties -> smallest (i, j));
 * every later device starts from the unused expert with the smallest summed count to the placed
 * experts; a device grows by the unused expert with the largest summed count to its own
 * experts (ties -> lowest expert index). */
int occult_placement_greedy(const int32_t* C_host, int32_t E, int32_t D, int32_t* L_host,
                            int32_t* expert_pos_host);

/* Collaboration statistics of a placement (paper Sec. 3.2; the "Intra / Inter" row of Table 1), host,
 * pure.  C_host [E][E] i32 co-activation counts (diagonal ignored), expert_pos_host [E] placement
 * positions (NULL = contiguous), host ptrs; needs E % D == 0.  With P = C / (largest off-diagonal
 * count), L_a = the G experts of device a:
 *   c_intra_host[a]        = mean of P[i][j] over the G*(G-1) ordered pairs i != j inside L_a (0 if G == 1)
 *   c_inter_host[a*D + b]  = mean of P[i][j] over the G*G pairs i in L_a, j in L_b, a != b (diagonal = 0)
 *   *intra_fraction_host   = share of the off-diagonal mass of C whose two experts sit on one device
 *                            (the "Intra" figure; "Inter" = 1 - it); 0 when C has no off-diagonal mass. */
int occult_collaboration_stats(const int32_t* C_host, int32_t E, int32_t D, const int32_t* expert_pos_host,
                               double* c_intra_host, double* c_inter_host, double* intra_fraction_host);

/* Copy the plan counters to the host and derive the statistics.  Synchronises `stream`
 * (the only call that does). */
int occult_plan_stats(const occult_cfg_t* cfg, const occult_plan_t* plan, occult_stats_t* out_host,
                      occult_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* OCCULT_H */
