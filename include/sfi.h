/*
 * libsfi — decode-attention hot path of Slow-Fast Inference for AMD MI355X (gfx950).
 *
 * One attention layer, single-query (decode) GQA attention over a bf16 KV cache, done two ways:
 *
 *   slow step  dense attention over the whole prefix, plus the Selector that turns the dense
 *              logits into a refreshed per-KV-head index set (paper Sec. 3.1 "Slow step",
 *              Sec. 3.2-3.3, Algorithm 2);
 *   fast step  sparse attention over  I = I_sink U I_sel U I_recent  only
 *              (paper Eq. index_set, Eq. index_set_head, Sec. 3.1 "Fast step").
 *
 * Conventions used by every call
 * -------------------------------
 *   B sequences, Hq query heads, Hkv KV heads, G = Hq / Hkv, head_dim d = 128.
 *   Positions are 0-based.  ctx_len[b] = number of rows of sequence b in the cache, the current
 *   token's row included.
 *   I_sink   = [0, min(n_sink, ctx_len))
 *   I_recent = [recent_start, ctx_len),  normally recent_start = max(n_sink, ctx_len - recent)
 *   J        = [n_sink, ctx_len - recent)   the allowed candidate set (paper Eq. allowed_set)
 *   I_sel    = sel_idx[b, h, 0 : n_sel[b, h]]   a subset of J, shared by the G query heads of KV
 *              head h (paper Sec. 3.1, "maintained per KV head").
 *
 *   q        bf16  [B, Hq, 128] contiguous.
 *   K, V     bf16, element (b, h, t, c) at  base + b*stride_b + h*stride_h + t*stride_t + c
 *            (strides in elements, given in sfi_config; a row of 128 elements is contiguous;
 *            row starts must be 16-byte aligned: stride_* multiples of 8, base 16-byte aligned).
 *   out      fp32  [B, Hq, 128] contiguous, or with cfg.out_bf16 = 1 bf16 [B, Hq, 128] (hence void*);
 *            16-byte aligned.
 *   sel_idx  int32 [B, Hkv, sel_stride]; n_sel int32 [B, Hkv].
 *   ctx_len, recent_start int32 [B].
 *
 * Every pointer named q, K, V, out, sel_idx, n_sel, ctx_len, recent_start, is_slow and the
 * workspace is a DEVICE pointer.  sfi_config, sfi_ctx** and the float array of
 * sfi_stage_times are HOST pointers.
 *
 * Ownership: the caller owns every buffer, including the workspace, which must stay alive and
 * untouched by others until sfi_destroy.  The library allocates no device memory and never
 * synchronises the device in a hot call: calls enqueue kernels on the given HIP stream
 * (hipStream_t passed as void*; NULL = the default stream) and return.  Results are valid once
 * the caller has synchronised that stream.  One context serves one stream at a time: two calls
 * on the same context must not overlap on the GPU (they share the workspace).
 *
 * Errors: every function returning int gives SFI_OK (0) or a negative sfi_status.  Host-checkable
 * argument errors are reported before anything is launched.  Values the host cannot see -- the
 * contents of ctx_len, n_sel, sel_idx, the block table -- are brought into range by the kernels
 * before they address memory, and what had to be changed is reported by sfi_device_status.
 *
 * ctx_len[b] = 0 is a legal input (an unused slot of a batch): out[b] = 0, n_sel[b] = 0, nothing of
 * K / V of that sequence is used, the other sequences are computed as if the slot were not there.
 */
#ifndef SFI_H_
#define SFI_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sfi_status {
  SFI_OK = 0,
  SFI_EINVAL = -1,      /* bad argument: null pointer, value out of range */
  SFI_EUNSUPPORTED = -2,/* a shape or mode this build does not implement */
  SFI_EWORKSPACE = -3,  /* workspace too small or misaligned */
  SFI_EALIGN = -4,      /* pointer or stride alignment violated */
  SFI_ELAUNCH = -5,     /* the HIP runtime rejected a launch or an event call */
  SFI_ENOMEM = -6       /* host allocation of the context failed */
} sfi_status;

typedef struct sfi_config {
  int32_t batch;        /* B >= 1 */
  int32_t n_q_heads;    /* Hq, multiple of n_kv_heads, Hq / Hkv <= 16 */
  int32_t n_kv_heads;   /* Hkv >= 1 */
  int32_t head_dim;     /* must be 128 */
  int32_t max_ctx;      /* upper bound of every ctx_len[b] this context will see */
  int32_t max_budget;   /* upper bound of the Selector budget K */
  int32_t n_sink;       /* |I_sink|; paper default 4 (Sec. 5 "Default SFI configuration") */
  int32_t recent;       /* recent window length; paper default 256 */
  float scale;          /* logit scale; 0 selects 1/sqrt(head_dim) */
  int32_t selector_mode;/* 0: rank by the evidence f alone (Eqs. selector_pt - selector_f, z_base);
                           1: Algorithm 2 in full: cache-aware prior, reverse-KL fusion with lambda*,
                              Soft-NMS and cross-head exclusivity before the Top-K */
  int64_t k_stride_b, k_stride_h, k_stride_t; /* elements */
  int64_t v_stride_b, v_stride_h, v_stride_t; /* elements */
  /* Selector mode 1 only (ignored in mode 0). */
  float gamma;          /* key-norm exponent, >= 0 (Eq. selector_prior_kn) */
  float beta, p, eta;   /* position prior: beta >= 0, p >= 1, eta >= 0 (Eq. selector_prior_pos) */
  float lambda_clip;    /* upper clip of lambda*, in [0, 1] (Eq. selector_lambda_closed) */
  float alpha_soft;     /* Soft-NMS strength, >= 0 (Eq. nms) */
  float alpha_cross;    /* cross-head exclusivity strength, >= 0 (Eq. head_mutex) */
  float temp;           /* T > 0 of Eq. head_softmax */
  float eps;            /* epsilon of Eqs. selector_prior_kn, selector_u, selector_prior_pos, z_base and
                           head_mutex; 0 selects 1e-8.  (1 + alpha_soft + alpha_cross) * log2(1/eps) must
                           stay below 120: the ranking key is exp(z) held in fp32 */
  int32_t nms_radius;   /* N(j) = { i in J : |i - j| <= nms_radius }, 0 .. 64 (Eq. nms_pool) */
  /* Both modes: power-mean exponent of Eq. selector_mu over the G query heads of a KV head, in (0, 1];
   * 0 selects 1 (f = the arithmetic mean of the heads' softmaxes over J). */
  float alpha;
  /* Paged cache: 0 = K and V are flat strided tensors (above); a power of two in [16, 65536] = K and V are
   * pools of blocks of page_size consecutive rows, row r of block p of KV head h at element offset
   * p * k_stride_page + r * k_stride_t + h * k_stride_h from the pool base; k_stride_b and v_stride_b must
   * be 0.  Sequences find their blocks through the block table set with
   * sfi_set_block_table.  max_ctx still bounds every ctx_len[b]. */
  int32_t page_size;
  /* Paged cache: element offset between consecutive blocks of the K / V pool; 0 selects
   * page_size * k_stride_t (blocks back to back in one run of rows, as in [blocks][page_size][Hkv][128]).
   * A [blocks][Hkv][page_size][128] pool, which keeps each head's rows of a block contiguous (the faster
   * layout for the dense kernel), has k_stride_t = 128, k_stride_h = page_size * 128 and
   * k_stride_page = Hkv * page_size * 128.  Must be a multiple of the row stride, with the same ratio for
   * K and V. */
  int64_t k_stride_page, v_stride_page;
  /* Output type of every `out` argument: 0 = fp32 [B, Hq, 128] (what the error bound of this library is
   * stated for); 1 = bf16 [B, Hq, 128], the fp32 result rounded to nearest even as it is stored (what a model
   * that keeps its activations in bf16 hands to the next projection; saves it a conversion pass). */
  int32_t out_bf16;
} sfi_config;

/*
 * Packed per-step descriptor (paper Sec. "Memory-coalesced Kernel Design and Selector Maintenance": the small control
 * state of a decoding step, built once per step and read from device memory by every kernel of every layer): one
 * 16-byte record per sequence in a DEVICE array [B] the caller owns.  sfi_step_begin fills it for the next step;
 * sfi_mixed_step_desc runs a layer's step from it.  The caller may also write it directly (it is plain data).
 * The block table of a paged cache is the context's (sfi_set_block_table); row b of it belongs to desc[b].
 */
typedef struct sfi_step_desc {
  int32_t ctx_len;      /* rows of the sequence in the cache, the current token's included */
  int32_t recent_start; /* first row of the recent window */
  int32_t is_slow;      /* 1: the step is a slow step for this sequence, 0: a fast step */
  int32_t since_slow;   /* fast steps in a row behind the sequence (state of the trigger policy) */
} sfi_step_desc;

typedef struct sfi_ctx sfi_ctx; /* opaque; host memory owned by the library */

/* Bytes of device workspace a context of this shape needs (256-byte aligned base expected).
 * Pure host arithmetic.  Returns 0 if the configuration is invalid. */
size_t sfi_workspace_bytes(const sfi_config* cfg);

/* Validate cfg, bind the caller's workspace, return a context in *out.
 * Touches the device to read its properties and to clear a few hundred bytes of the workspace (the
 * arrival counters of the fast step's in-kernel merge and the status word of sfi_device_status; a blocking
 * memset followed by a device synchronisation, so not to be called while a stream of the device is
 * capturing).  SFI_ELAUNCH if the workspace is memory the runtime knows (device, managed or pinned host
 * memory) and could not be cleared. */
int sfi_create(const sfi_config* cfg, void* workspace, size_t workspace_bytes, sfi_ctx** out);

/*
 * Paged cache (cfg.page_size > 0; paper Sec. 4.2: recent tokens "remain in paged KV", and the packed
 * per-step descriptor carries block-table pointers): block_table is a DEVICE int32 array
 * [batch][table_stride]; entry [b][i] is the block of the pools that holds rows
 * [i * page_size, (i + 1) * page_size) of sequence b.  Entries that cover rows [0, ctx_len[b]) must be valid
 * at every hot call (later ones are never read); block ids lie in [0, n_blocks), and
 * n_blocks * (block stride / row stride) must stay below 2^31 (row numbers are 32-bit; byte offsets into the
 * pools are 64-bit).  The pointer is kept until the next call of this function; the table's contents may change
 * between hot calls.  With a paged cache the K and V arguments of the hot calls are the pool bases and the
 * kernels never read rows before ctx_len[b] is known.  Passing NULL detaches the table.
 */
int sfi_set_block_table(sfi_ctx* ctx, const int32_t* block_table, int32_t table_stride, int32_t n_blocks);

/* Frees the host-side context (and its profiling events).  The workspace stays the caller's. */
int sfi_destroy(sfi_ctx* ctx);

/* Static, human-readable text for a status code. */
const char* sfi_strerror(int status);

/*
 * Slow step (paper Algorithm 1 "Slow Step" + Algorithm 2):
 *   out[b, g, :]     = softmax_j(scale * <q[b,g], K[b,h,j]>) V[b,h,:]  over j in [0, ctx_len[b])
 *   sel_idx[b, h, :] = the n_sel[b,h] = min(budget, |J|) positions of J with the largest evidence
 *                      f_h(j) = (1/G) sum_{g in group h} softmax over J of the logits of head g
 *                      (cfg.alpha = 1; in general the power mean of Eqs. selector_mu, selector_f)
 *                      (ranking score z = log(f + 1e-8) is monotone in f); equal scores: the lower
 *                      position wins; written ascending, entries [n_sel, budget) set to -1.
 * sel_idx is addressed with row stride `budget`.  max_len: host-side upper bound of ctx_len[]
 * (0 = cfg.max_ctx); it sizes the launch, and rows [0, max_len) of every (b, h) of K and V must be
 * readable memory (their contents beyond ctx_len[b] are never used): the kernel issues a tile's
 * row loads before ctx_len[b] has arrived.  0 <= ctx_len[b] <= max_len.
 */
int sfi_slow_step(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                  int32_t max_len, int32_t budget, void* out, int32_t* sel_idx, int32_t* n_sel,
                  void* stream);

/*
 * The two halves of a slow step, for layer-wise asynchronous execution (paper Sec. "Hiding Slow-step
 * Overhead via Layer-wise Asynchronous Execution": Attn_i -> Sel_i, Attn_{i+1} independent of Sel_i):
 *   sfi_slow_attn    dense attention -> out; the evidence (logits over J and their softmax statistics)
 *                    stays in this context's workspace;
 *   sfi_slow_select  the Selector on that evidence -> sel_idx, n_sel.  ctx_len, max_len must be the ones
 *                    given to the sfi_slow_attn call it follows.  It may be called again on the same evidence
 *                    (another budget): a repeat starts with one more small launch that resets the Selector's
 *                    counters.
 * sfi_slow_step is the two in a row on one stream.  To overlap Sel_i with Attn_{i+1}, give the layers
 * in flight a context (and workspace) each -- a ring of a few -- run sfi_slow_attn on the main stream and
 * sfi_slow_select on a second stream that waits for an event recorded after it; before a context is
 * reused, the main stream must wait for the event recorded after that context's last sfi_slow_select.
 * The library creates no stream and no cross-stream dependency of its own.
 */
int sfi_slow_attn(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                  int32_t max_len, void* out, void* stream);
int sfi_slow_select(sfi_ctx* ctx, const int32_t* ctx_len, int32_t max_len, int32_t budget, int32_t* sel_idx,
                    int32_t* n_sel, void* stream);

/*
 * Windowed evidence (paper Eq. window_logits and Eq. selector_mu with a window of W > 1 queries, e.g. the last
 * W queries of a prefill block; Sec. 5 "Default SFI configuration" uses W = 1 in decode):
 *   sfi_evidence_add     dense attention of one window query (-> out, as sfi_slow_attn) and its head-mean
 *                        evidence (1/G) sum_g p_g^alpha over J added to this context's accumulator
 *                        (first != 0 starts the accumulator);
 *   sfi_evidence_select  the Selector on the accumulated evidence mu = (1/W) * sum over the n_added queries:
 *                        mode 0 ranks mu, mode 1 takes f = mu^(1/alpha) through prior, fusion and refinements
 *                        (key norms from the last sfi_evidence_add).  -> sel_idx, n_sel.
 * Every added query must see the same allowed set J, i.e. the same ctx_len[] / max_len in every call; for window
 * queries that sit before the end of the context and are masked inside J, see sfi_evidence_add_causal.
 * sfi_evidence_add with out == NULL is the evidence-only pass: V is not read (and may be NULL), no attention
 * output is written -- half the cache traffic, for callers whose prefill kernel has the outputs already.
 */
int sfi_evidence_add(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                     int32_t max_len, void* out, int32_t first, void* stream);
/*
 * The same for a window query under the causal mask ("masked attention logit" of Eq. window_logits): the window's last
 * W queries of a prefill block sit at rows L - W .. L - 1 of a context of L = ctx_len[b] rows, and query tau sees rows
 * [0, q_len[b]) only, q_len[b] = L - W + tau + 1 (its own row included).  q_len: DEVICE int32 [B], 0 <= q_len[b] <= ctx_len[b]
 * (values outside are brought into that range).  ctx_len[] is the same in every call of the window and defines J; this
 * query's softmax (Eq. selector_pt) runs over the part of J it sees, it adds p = 0 elsewhere, and out (if given) is its
 * attention over the rows it sees.  The mean of Eq. selector_mu still divides by the n_added given to sfi_evidence_select.
 * With recent >= W every query sees all of J and the call equals sfi_evidence_add.  In mode 1 the key norms are those
 * exposed by the last call, so the window's last query (q_len = ctx_len) must be added last.
 */
int sfi_evidence_add_causal(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                            const int32_t* q_len, int32_t max_len, void* out, int32_t first, void* stream);
int sfi_evidence_select(sfi_ctx* ctx, int32_t n_added, const int32_t* ctx_len, int32_t max_len, int32_t budget,
                        int32_t* sel_idx, int32_t* n_sel, void* stream);

/* Dense attention only (the `out` of a slow step, no Selector).  Same arguments and meaning. */
int sfi_dense_attn(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                   int32_t max_len, void* out, void* stream);

/*
 * Fast step (paper Algorithm 1 "Fast Step"):
 *   out[b, g, :] = attention of q[b,g] over rows
 *                  [0, min(n_sink, ctx_len)) U sel_idx[b,h,0:n_sel[b,h]] U [recent_start[b], ctx_len[b]).
 * Preconditions: the three parts are disjoint; sel entries lie in [n_sink, recent_start[b]);
 * n_sink <= recent_start[b] <= ctx_len[b]; while ctx_len[b] < n_sink any recent_start[b] >= ctx_len[b] is
 * read as ctx_len[b] (an empty window: sfi_advance leaves n_sink there);
 * n_sel[b,h] <= sel_stride <= cfg.max_budget.  sel_idx / n_sel are read-only here.  With sel_stride = 0
 * (sink and recent window only) sel_idx is not read and may be NULL.
 */
int sfi_fast_step(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* sel_idx,
                  const int32_t* n_sel, int32_t sel_stride, const int32_t* recent_start,
                  const int32_t* ctx_len, void* out, void* stream);

/*
 * The fast step for callers that cannot allocate device memory or hold a workspace: code under HIP graph
 * capture that owns no buffers of its own, tight serving loops, harnesses that forbid hipMalloc.  Same result
 * as sfi_fast_step on a context created from *cfg (HOST pointer; read during the call only), same argument
 * meaning and preconditions; no sfi_ctx and no workspace are involved.  The split records and arrival counters
 * of the in-kernel merge live in a file-scope device array of the library instead (4.2 MiB, held by every GPU
 * the library runs on until the process ends), which sets the limits:
 *   batch * n_q_heads <= 8192  and  batch * n_kv_heads <= 4096, else SFI_EUNSUPPORTED;
 *   at most 8192 / (batch * n_q_heads) workgroups per (sequence, KV head): larger shapes run with a coarser split
 *   than sfi_fast_step would pick (same result up to the rounding of the split merge);
 *   flat caches only (cfg->page_size != 0: SFI_EUNSUPPORTED).
 * Calls no allocating routine.  Every call on one GPU uses that GPU's one array: calls that overlap on a GPU
 * (two streams, two threads' launches in flight together) race and give undefined outputs; calls on one stream,
 * or otherwise ordered, are fine.  The counters are zeroed by a small kernel on `stream` in a device's first call
 * and after a call whose launch failed; every completed launch leaves them at zero.  Device-side inputs out of
 * range are clamped as everywhere, but not reported (there is no context whose status word could take the bits).
 */
int sfi_fast_step_static(const sfi_config* cfg, const void* q, const void* K, const void* V, const int32_t* sel_idx,
                         const int32_t* n_sel, int32_t sel_stride, const int32_t* recent_start,
                         const int32_t* ctx_len, void* out, void* stream);

/*
 * Reorg (paper Sec. "Hiding Slow-step Overhead via Layer-wise Asynchronous Execution", Reorg_i, and
 * Sec. "Memory-coalesced Kernel Design and Selector Maintenance", two-segment KV layout): after a
 * slow step, copy the sink rows and the selected rows of every (b, h) into caller-owned compact
 * buffers, rows of 128 bf16 back to back:
 *   Kc[b, h, i, :]          = K[b, h, i, :]              i <  min(n_sink, ctx_len[b])
 *   Kc[b, h, n_sink + i, :] = K[b, h, sel_idx[b,h,i], :] i <  n_sel[b,h]
 * and the same for Vc from V.  Other rows of the buffers are left as they are.
 * Kc / Vc: device, bf16, addressed as base + b * c_stride_b + h * c_stride_h + i * 128 (strides in
 * elements, multiples of 8); every (b, h) slice holds c_rows >= n_sink + sel_stride rows, all of them
 * readable memory.  is_slow: nullptr, or device uint8 [B]: only sequences with is_slow[b] != 0 are
 * reorganised (the companion of sfi_mixed_step).  Other arguments as in sfi_fast_step.
 */
int sfi_reorg(sfi_ctx* ctx, const void* K, const void* V, const int32_t* sel_idx, const int32_t* n_sel,
              int32_t sel_stride, const int32_t* ctx_len, const uint8_t* is_slow, void* Kc, void* Vc,
              int64_t c_stride_b, int64_t c_stride_h, int32_t c_rows, void* stream);

/*
 * Fast step over the two-segment layout (same sections): the sink and selected rows are read as one
 * run of consecutive rows from the compact buffers sfi_reorg filled, the recent window
 * [recent_start[b], ctx_len[b]) in place from K / V.  Same result as sfi_fast_step on the sel_idx
 * the buffers were built from.  Preconditions as for sfi_fast_step; n_sel[b,h] <= sel_stride and
 * c_rows >= n_sink + sel_stride; n_sel[b,h] > 0 only where ctx_len[b] > n_sink.
 * While ctx_len[b] <= n_sink the whole context is read in place from K / V (nothing is selected, and
 * rows appended since sfi_reorg are sink rows the buffers do not hold).  A sequence reorganised at
 * ctx_len[b] < n_sink must be reorganised again before a compact fast step at ctx_len[b] > n_sink:
 * the sink rows that did not exist yet are not in the buffers.
 */
int sfi_fast_step_compact(sfi_ctx* ctx, const void* q, const void* Kc, const void* Vc, int64_t c_stride_b,
                          int64_t c_stride_h, int32_t c_rows, const int32_t* n_sel, int32_t sel_stride,
                          const void* K, const void* V, const int32_t* recent_start, const int32_t* ctx_len,
                          void* out, void* stream);

/*
 * Ragged mix: sequence b takes a slow step if is_slow[b] != 0 (uint8, device) and a fast step
 * otherwise; slow sequences refresh their rows of sel_idx / n_sel in place (row stride `budget`),
 * fast sequences read theirs.  No host synchronisation decides the mode.
 */
int sfi_mixed_step(sfi_ctx* ctx, const void* q, const void* K, const void* V, const uint8_t* is_slow,
                   const int32_t* ctx_len, const int32_t* recent_start, int32_t max_len, int32_t budget,
                   void* out, int32_t* sel_idx, int32_t* n_sel, void* stream);

/*
 * The ragged mix over the two-segment layout (paper Sec. "Memory-coalesced Kernel Design and Selector Maintenance" under
 * per-sequence modes): fast sequences read their sink and selected rows from the compact buffers (as
 * sfi_fast_step_compact), slow sequences take a slow step and have their buffer rows refilled from the refreshed index
 * set afterwards (Sel_i -> Reorg_i, as sfi_reorg with is_slow).  Arguments as in sfi_mixed_step and sfi_reorg;
 * c_rows >= n_sink + budget.  Every sequence's buffers must have been filled for its current index set before its first
 * fast step here (a step that is slow for it does that).
 */
int sfi_mixed_step_compact(sfi_ctx* ctx, const void* q, const void* K, const void* V, const uint8_t* is_slow,
                           const int32_t* ctx_len, const int32_t* recent_start, int32_t max_len, int32_t budget,
                           void* out, int32_t* sel_idx, int32_t* n_sel, void* Kc, void* Vc, int64_t c_stride_b,
                           int64_t c_stride_h, int32_t c_rows, void* stream);

/*
 * Trigger policy on the device (paper Sec. "Training-free trigger policy", Eq. trigger, and the last lines
 * of Algorithm 1), so that a decode loop needs no host decision between steps:
 *   is_slow[b]    = 1 if last_token[b] is in the trigger set, or since_slow[b] >= t_max; else 0
 *   since_slow[b] = 0 if is_slow[b], else since_slow[b] + 1
 * i.e. the step after a trigger token is slow, and so is the step after t_max fast steps in a row.
 * last_token: device int32 [B], the token generated by the previous step; ids outside [0, vocab_size)
 * never trigger.  trigger_bitmap: device uint32 [(vocab_size + 31) / 32], bit (id % 32) of word id / 32 set
 * iff id is in the trigger set (built once, offline, from the tokenizer).  since_slow: device int32 [B],
 * read and updated; initialise it to t_max to make the first step slow (Algorithm 1: g_0 = 1).
 * is_slow: device uint8 [B], written; the flags sfi_mixed_step and sfi_reorg take.
 */
int sfi_trigger(sfi_ctx* ctx, const int32_t* last_token, const uint32_t* trigger_bitmap, int32_t vocab_size,
                int32_t t_max, int32_t* since_slow, uint8_t* is_slow, void* stream);

/*
 * One launch per decoding step that prepares the packed descriptor for it (the state update and the trigger policy
 * together, Algorithm 1 "Update I_recent and compute g_{t+1}"): for every sequence b
 *   advance != 0:  desc[b].ctx_len += 1   (the token generated by the last step has joined the cache)
 *   desc[b].recent_start = max(n_sink, ctx_len - recent)
 *   desc[b].is_slow      = 1 if last_token[b] is in the trigger set or desc[b].since_slow >= t_max, else 0
 *   desc[b].since_slow   = 0 if is_slow, else since_slow + 1
 * last_token / trigger_bitmap / vocab_size as in sfi_trigger; either may be NULL (no trigger tokens: only the forced
 * refresh after t_max fast steps).  Before the first step: ctx_len = the prompt's rows, since_slow = t_max (g_0 = 1),
 * advance = 0.
 */
int sfi_step_begin(sfi_ctx* ctx, sfi_step_desc* desc, const int32_t* last_token, const uint32_t* trigger_bitmap,
                   int32_t vocab_size, int32_t t_max, int32_t advance, void* stream);

/* sfi_mixed_step with the per-sequence state read from the packed descriptor: ctx_len, recent_start and is_slow of
 * sequence b are desc[b]'s.  Everything else as in sfi_mixed_step. */
int sfi_mixed_step_desc(sfi_ctx* ctx, const void* q, const void* K, const void* V, const sfi_step_desc* desc,
                        int32_t max_len, int32_t budget, void* out, int32_t* sel_idx, int32_t* n_sel, void* stream);

/* State update between decode steps, on the device (paper Algorithm 1, "update I_recent"):
 * ctx_len[b] += 1;  recent_start[b] = max(n_sink, ctx_len[b] - recent). */
int sfi_advance(sfi_ctx* ctx, int32_t* ctx_len, int32_t* recent_start, void* stream);

/*
 * Per-kernel timing for benchmarks.  sfi_set_profiling(ctx, max_calls) with max_calls > 0 makes each
 * of the next max_calls hot calls bracket every kernel it launches with a pair of HIP events on the
 * caller's stream (no host synchronisation in between); max_calls = 0 switches it off.
 * sfi_stage_times waits for the recorded events and returns, per stage, the sum of elapsed
 * milliseconds and the number of launches over the calls recorded since profiling was switched on.
 * Not for production loops: event records add a gap of a few microseconds around every kernel.
 */
enum {
  SFI_STAGE_ATTN = 0,     /* split attention kernel (dense; gather or compact in a fast step) */
  SFI_STAGE_MERGE = 1,    /* split merge */
  SFI_STAGE_SCORE = 2,    /* evidence + first radix histogram (mode 1: the three scoring kernels together) */
  SFI_STAGE_CAND = 3,     /* threshold-bin candidates */
  SFI_STAGE_COUNT = 4,    /* exact threshold + per-segment counts */
  SFI_STAGE_WRITE = 5,    /* ordered index write */
  SFI_STAGE_ATTN2 = 6,    /* the gather attention kernel of a mixed step */
  SFI_STAGE_REORG = 7,    /* compact-buffer gather */
  SFI_N_STAGES = 8
};
int sfi_set_profiling(sfi_ctx* ctx, int max_calls);
int sfi_stage_times(sfi_ctx* ctx, float* ms_sum /* host, [SFI_N_STAGES] */, int32_t* count /* host, [SFI_N_STAGES] */);

/* Launch knobs for sweeps (0 keeps the current setting, a negative value restores the default):
 * dense_target_wgs     workgroups a dense launch aims for in total.  Default: decided per launch -- the
 *                      number of workgroups per (sequence, KV head) that loads the compute units most
 *                      evenly (one workgroup per compute unit, all resident at once, where the pairs
 *                      divide the compute units);
 * fast_tiles_per_wave  32-row tiles each wave of the gather launch gets.  Default: decided per launch by
 *                      the same rule -- one tile per wave (one-tile kernel) or several (pipelined loop);
 * fast_merge           how the split records of a fast step become the output: 1 (default) inside the
 *                      attention kernel, by the last workgroup of each (sequence, KV head) to finish;
 *                      2 in a merge launch of its own.  Other values > 2: SFI_EINVAL. */
int sfi_set_tuning(sfi_ctx* ctx, int32_t dense_target_wgs, int32_t fast_tiles_per_wave, int32_t fast_merge);

/* A/B knob of the dense kernel's K loads: 0 (default) = a K row leaves the compute unit as four 64-byte requests, the
 * shape the matrix instruction's operand layout asks for; 1 = as two requests for whole 128-byte lines (the gather
 * kernels' layout: a row of the product is half a K row, the halves are joined by lane exchanges).  Same results;
 * applies to flat caches, query groups of at most 8 heads, Selector mode 0 (ignored elsewhere).  The default is the
 * faster one on MI355X. */
int sfi_set_dense_k_layout(sfi_ctx* ctx, int32_t whole_lines);

/* A/B knob of the dense launch inside sfi_mixed_step, sfi_mixed_step_compact and sfi_mixed_step_desc (the ragged step of
 * Sec. 4.2, where which sequences take a slow step is only known on the device).  on = 1 (default): the launch is one
 * workgroup per compute unit; every workgroup derives the same plan from the flags and lengths -- the slow sequences
 * and, for each, a number of splits in proportion to its length -- and takes its share of the cells, so the shares are
 * equal whatever the mix (batches of up to 1024 sequences, and only where the fast step's merge runs inside its kernel;
 * otherwise as with on = 0).  on = 0: one workgroup per (split, KV head, sequence) cell of the whole batch with the
 * finest split; workgroups of fast sequences exit at once.  Same results.  Other values: SFI_EINVAL. */
int sfi_set_mixed_plan(sfi_ctx* ctx, int32_t on);

/* Launch geometry the library would choose, without launching anything (host arithmetic only): split
 * workgroups per (sequence, KV head) of a dense launch bounded by max_len rows (0 = cfg.max_ctx) and
 * of a fast step whose index lists are sel_stride wide.  Either output may be NULL.  SFI_EINVAL for a
 * max_len or sel_stride outside the configuration. */
int sfi_plan_splits(const sfi_ctx* ctx, int32_t max_len, int32_t sel_stride, int32_t* dense_splits,
                    int32_t* fast_splits);

/*
 * Device-side inputs that were out of range.  ctx_len, recent_start, n_sel, sel_idx and the block table live
 * in device memory, so no host check can vet them before a launch.  Every kernel therefore brings them into
 * range before they address memory, so that a launch stays inside the caller's buffers whatever these arrays
 * hold:
 *   ctx_len[b]       to [0, max_len] (cfg.max_ctx for calls without a max_len);
 *   recent_start[b]  to [min(n_sink, ctx_len[b]), ctx_len[b]] (silently: any value is allowed and read this way);
 *   n_sel[b, h]      to [0, sel_stride];
 *   a stored index   outside [0, ctx_len[b]) reads as row ctx_len[b] - 1;
 *   a block id       to [0, n_blocks).
 * A kernel that changed a value it used ORs the matching bit below into a word of the workspace (padding
 * entries of sel_idx and table entries past ctx_len[b] are never looked at).  The outputs of a call that raised
 * a bit are unspecified.
 *
 * This call waits for `stream`, copies the word to *flags (HOST int32) and, with clear != 0, zeroes it.
 * It blocks the host and is not part of the hot path: poll it when debugging, or once in a while.  Not to be
 * called while a stream of the device is capturing.  The word is also zeroed by sfi_create.
 */
#define SFI_GUARD_CTX_LEN 1 /* a ctx_len[b] was negative or above the call's bound */
#define SFI_GUARD_N_SEL 2   /* an n_sel[b, h] was negative or above sel_stride */
#define SFI_GUARD_SEL_IDX 4 /* an index among sel_idx[b, h, 0:n_sel] was outside [0, ctx_len[b]) */
#define SFI_GUARD_BLOCK 8   /* a block-table entry covering rows [0, ctx_len[b]) was outside [0, n_blocks) */
int sfi_device_status(sfi_ctx* ctx, int32_t* flags, int32_t clear, void* stream);

/*
 * Memory skeleton of the fast step -- a measurement aid for benchmarks, not part of the path.  Takes the arguments of
 * sfi_fast_step and launches its grid with its loads but none of its arithmetic; `out` receives no meaningful values.
 * variant:
 *   bit 0      also run the record hand-over of the real launch (LDS combine, device-scope record stores, arrival
 *              counter, merge by the pair's last workgroup);
 *   bit 1      every wave requests the rows of all its tiles at once, straight into LDS, instead of walking them through
 *              one register buffer (at most nine tiles per workgroup: the split is made finer if need be, SFI_EUNSUPPORTED
 *              if that is not enough; not together with bit 0);
 *   bits 2-3   how far down the chain of dependent loads the launch goes: 0 = all of it (the three per-step scalars and the
 *              indices, then the K and V rows); 1 = scalars and indices only; 2 = nothing (an empty grid of the same shape).
 * Flat caches only.  The time of this launch is the floor the fast-step kernel of the same shape is held against.
 */
int sfi_fast_step_floor(sfi_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* sel_idx,
                        const int32_t* n_sel, int32_t sel_stride, const int32_t* recent_start,
                        const int32_t* ctx_len, void* out, int32_t variant, void* stream);

/*
 * Memory skeleton of the dense launch -- a measurement aid like sfi_fast_step_floor: the grid and tile dealing of
 * sfi_dense_attn over rows [0, ctx_len[b]) of K and V (two tile buffers per wave, nontemporal 16-byte loads), nothing
 * computed, no logits written.  variant bits 0-3: 0 = K rows requested in the dense kernel's own layout (four 64-byte
 * pieces per row), 1 = as whole 128-byte lines.  Bits 4-10: idle units u (0 .. 64): every wave sleeps u x 64 cycles
 * after each half of each tile, where the kernel has its arithmetic.  Bits 11 and up: 1 = every workgroup gets a fifth
 * wave that stores what the slow step would expose (G x 128 bytes per tile, into the workspace's logits buffer, junk
 * values) at about the readers' pace; 2 = the same stores, all to the same 2 KB per (sequence, KV head).  Other values:
 * SFI_EUNSUPPORTED.  Flat caches only.  Its time is the streaming ceiling the dense kernel is held against; the writer
 * variants show what store instructions cost a compute unit that is streaming rows.  Overwrites the logits a slow step
 * left in the workspace.
 */
int sfi_dense_attn_floor(sfi_ctx* ctx, const void* K, const void* V, const int32_t* ctx_len, int32_t max_len,
                         int32_t variant, void* stream);

/* Launch geometry of the last call (for reports): split workgroups per (sequence, KV head). */
int sfi_query_splits(const sfi_ctx* ctx, int32_t* dense_splits, int32_t* fast_splits);

#ifdef __cplusplus
}
#endif
#endif /* SFI_H_ */
