/*
 * slicemoe.h -- C ABI of the MI355X (gfx950) SliceMoE expert-FFN library.
 *
 * The calls follow the paper's statement of the problem (SliceMoE, arXiv 2512.12990):
 *   quantize/slice   AMAT: group-wise asymmetric b_high-bit codes whose upper b_low bits are the
 *                    low-bit model (Section 4.2 and its equation, Table 1 note 1); 8/4, 6/3, 4/2
 *   route            cache-aware top-k: resident experts get a score boost (Section 2.1)
 *   expert_ffn(mask) per selected expert a SwiGLU FFN run from the MSB slice alone or from
 *                    MSB+LSB, decided by slice residency (Section 4.1)
 *   prefill_histogram  token-parallel high-bit prefill that also counts expert accesses, the
 *                    statistic Predictive Cache Warmup ranks slices by (Section 4.3)
 * plus host-only bookkeeping (slice LRU, top-N) that produces the mask and never touches the GPU.
 *
 * Conventions
 *   - Every function returns 0 (SMOE_OK) or a negative smoe_status; nothing throws.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *     All device pointers must be 16-byte aligned.  The caller owns every buffer it passes; a
 *     bank only borrows its store and must be destroyed before that memory is freed.
 *   - All device work is enqueued on the stream given to smoe_ctx_create and is asynchronous
 *     unless a function says it synchronises.  One ctx per host thread.
 *   - Matrices are row-major W[out, in]; quantisation groups are `group` consecutive elements
 *     along `in` of one output row; a last shorter group is allowed.
 *   - dtype codes: SMOE_F32 = 0, SMOE_BF16 = 1 (bf16 = upper 16 bits of an IEEE fp32).
 *   - slice_mask[e]: bit0 = MSB slice of expert e resident, bit1 = LSB slice resident.
 */
#ifndef SLICEMOE_H
#define SLICEMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SMOE_OK = 0,
  SMOE_EINVAL = -1,   /* null or invalid argument */
  SMOE_ESHAPE = -2,   /* inconsistent or unsupported dimensions */
  SMOE_EALIGN = -3,   /* device pointer not 16-byte aligned */
  SMOE_ESIZE = -4,    /* a caller buffer or the ctx workspace is too small */
  SMOE_EHIP = -5,     /* a HIP call failed; see smoe_last_hip_error */
  SMOE_ENOTIMPL = -6  /* valid request this build does not implement (e.g. a 5/2-bit nest) */
} smoe_status;

enum { SMOE_F32 = 0, SMOE_BF16 = 1 };

typedef struct smoe_ctx smoe_ctx;     /* host object: device id, stream, borrowed device workspace */
typedef struct smoe_bank smoe_bank;   /* host object describing one sliced expert store in HBM */
typedef struct smoe_cache smoe_cache; /* host-only slice LRU */

/* One set of equally shaped SwiGLU experts: gate, up are [d_ff, d_model], down is [d_model, d_ff].
 * d_model, d_ff and group must be multiples of 32 (a K that is not a multiple of `group` gets a
 * short last group).  b_high/b_low: the three nests of Table 1 are implemented -- 8/4 (8-bit codes,
 * two nibble planes), 6/3 (6-bit codes, two 3-bit planes: 3/4 of the plane bytes) and 4/2 (4-bit
 * codes, two 2-bit planes: half of them); the low-bit model is always the upper b_low bits with the
 * zero-point shifted by the same amount.  Any other pair returns SMOE_ENOTIMPL. */
typedef struct {
  int32_t n_experts, d_model, d_ff, group;
  int32_t b_high, b_low;
  int32_t w_dtype;      /* dtype of the source weights handed to smoe_quantize_slice */
  int32_t scale_dtype;  /* dtype the per-group scales are stored in (and rounded to) */
  int32_t symmetric;    /* 0: asymmetric min-max quantiser (the experts, Table 1 note 1).  1: symmetric
                         * quantiser (Section 6.1 item 1: the non-expert weights are symmetric INT8) in the same
                         * store: zero-point fixed at 2^(b_high-1); see smoe_quantize_slice.  Other
                         * values: SMOE_EINVAL. */
} smoe_bank_desc;

typedef struct {
  uint64_t msb_hit, msb_miss, lsb_hit, lsb_miss;
} smoe_cache_stats;

/* ---- context ---------------------------------------------------------------------------- */
/* Bytes of device workspace a context needs for decode calls of up to `tokens` tokens (1..16) through
 * layers of at most k routed slots of d_ff and n_shared shared experts of shared_d_ff: the routing
 * records (64 KiB reserved) plus the fp32 SwiGLU vectors of every token. */
int smoe_workspace_bytes(int tokens, int k, int d_ff, int n_shared, int shared_d_ff, size_t* bytes);
/* Creates a context bound to `device`, to `hip_stream` (a hipStream_t, NULL = default stream) and
 * to `workspace_dev`, caller-owned device memory of workspace_bytes (256-byte aligned, at least
 * smoe_workspace_bytes of the largest layer it will see; SMOE_ESIZE below 64 KiB, and later from a
 * decode call whose intermediates do not fit).  The library itself never allocates or frees device
 * memory; the workspace is borrowed until smoe_ctx_destroy and is shared by all calls of the context,
 * which therefore must not overlap in time (one stream).  workspace_dev may be NULL with
 * workspace_bytes 0: such a context serves every call that needs no workspace (quantise, route,
 * prefill, smoe_decode_layer_static); the other decode calls return SMOE_ESIZE. */
int smoe_ctx_create(int device, void* hip_stream, void* workspace_dev, size_t workspace_bytes, smoe_ctx** out);
int smoe_ctx_destroy(smoe_ctx* ctx);
const char* smoe_strerror(int status);
int smoe_last_hip_error(const smoe_ctx* ctx); /* hipError_t of the last failing HIP call, else 0 */
/* Measurement aid, no part of the method.  While enabled, smoe_expert_ffn / smoe_decode_layer record
 * a start and a stop HIP event with each of their two kernel dispatches (gate/up, down) on the ctx stream.
 * smoe_ctx_timing_read synchronises the stream, returns the summed durations in microseconds and the
 * number of calls recorded since the last read, and releases the events. */
int smoe_ctx_timing(smoe_ctx* ctx, int enable);
int smoe_ctx_timing_read(smoe_ctx* ctx, double* gateup_us, double* down_us, int* n_calls);
/* Single-launch decode (Section 6.1 item 1: the fused decode step; an option of this implementation,
 * off by default).  With the mode on, smoe_expert_ffn / smoe_decode_layer run one token's routing,
 * gate/up projections, the hand-over of the SwiGLU vector and the down projection in ONE kernel launch
 * instead of two, when the case fits: d_model <= 2048, d_model / 8 no larger than the number of gate/up
 * work-groups (at most 512), timing off, and all work-groups of the launch resident on the device
 * together (checked from the occupancy the runtime reports).  Cases that do not fit,
 * smoe_decode_layer_multi and smoe_decode_layer_static keep the two launches.  Results are
 * bit-identical in both modes.  On MI355X the two launches are the faster form (15 against 21 us per
 * token on the DeepSeek-V2-Lite-shaped layer), which is why the mode is an option.
 *   The work-groups of the single launch wait for each other inside the kernel.  The wait is bounded:
 * after spin_limit polls (0: the default, 2^20, of the order of a second) a work-group goes on with
 * whatever it finds and counts itself in n_timeouts, so a launch always ends; a call whose work-groups
 * cannot all run together (a device shared with another busy process) therefore shows up as a non-zero
 * n_timeouts and a wrong result, never as a hang.  Enabling enqueues a small kernel on the ctx stream
 * that clears the hand-over words in the first 64 KiB of the workspace (SMOE_ESIZE for a context
 * without one); calling it again clears them again.  smoe_ctx_single_launch_status synchronises the
 * stream and returns the number of decode calls that took the single launch so far and the
 * work-groups that gave up waiting since the words were last cleared. */
int smoe_ctx_single_launch(smoe_ctx* ctx, int enable, int spin_limit);
int smoe_ctx_single_launch_status(smoe_ctx* ctx, long long* n_calls, unsigned* n_timeouts);
/* Measurement aid, no part of the method.  Enqueues a kernel of n_workgroups x 512 threads that reads
 * bytes (a multiple of 16 is used) from buf_dev with 16-byte loads and does nothing else: what the same
 * bytes cost when they are only streamed, as a practical roof beside the decode kernels.  sink_dev: 16
 * bytes of device memory (never written in practice). */
int smoe_stream_read(smoe_ctx* ctx, const void* buf_dev, size_t bytes, int n_workgroups, void* sink_dev);

/* ---- quantize / slice (Section 4.2; Table 1 note 1) ------------------------------------- */
/* Bytes of device memory a bank's store needs. */
int smoe_bank_bytes(const smoe_bank_desc* desc, size_t* store_bytes);
/* Wraps caller-owned device memory `store_dev` (>= store_bytes, 256-byte aligned) as a bank.
 * No device work. */
int smoe_bank_create(smoe_ctx* ctx, const smoe_bank_desc* desc, void* store_dev, size_t store_bytes,
                     smoe_bank** out);
int smoe_bank_destroy(smoe_bank* bank);
/* Quantises experts [e0, e0+n) from dense device weights w_gate[n, d_ff, d_model],
 * w_up[n, d_ff, d_model], w_down[n, d_model, d_ff] (dtype desc.w_dtype, finite values) into the
 * bank: per group lo = min(0, min w), hi = max(0, max w), s = round_to_scale_dtype((hi-lo)/255)
 * (1 if that is not positive), zp = clamp(rint(-lo/s)), q = clamp(rint(w/s) + zp), all fp32
 * round-to-nearest-even; then the code is split into its upper nibble (MSB slice, = the 4-bit
 * model's code floor(q/16)) and lower nibble (LSB slice), stored in separate planes.
 * With desc.symmetric the first three steps are instead s = round_to_scale_dtype(max|w| /
 * (2^(b_high-1) - 1)) (1 if not positive), zp = 2^(b_high-1), q = clamp(rint(w/s) + zp); every
 * consumer reads such a bank like any other. */
int smoe_quantize_slice(smoe_ctx* ctx, smoe_bank* bank, int e0, int n, const void* w_gate_dev,
                        const void* w_up_dev, const void* w_down_dev);
/* Copies one matrix of one expert back in canonical form (matrix: 0 gate, 1 up, 2 down; N x K its
 * shape, ng = ceil(K/group)).  Host outputs, any may be NULL: q[N*K] 8-bit codes, msb[N*K] and
 * lsb[N*K] nibble values 0..15, zp[N*ng], scale[N*ng] widened to fp32.  Synchronises. */
int smoe_export_codes(smoe_ctx* ctx, const smoe_bank* bank, int expert, int matrix, uint8_t* q_host,
                      uint8_t* msb_host, uint8_t* lsb_host, uint8_t* zp_host, float* scale_host);

/* ---- route (Section 2.1) ------------------------------------------------------------------ */
/* For each of T tokens: z = logits_dev[t] (fp32 [T,E]) or, if logits_dev is NULL,
 * z_e = sum_i w_router_dev[e,i] * x_dev[t,i] (w_router fp32 [E,d_model], x of act_dtype, fp32
 * accumulation); score = z + bias (bias_dev fp32 [E] or NULL = 0); idx_dev[t,0..k) = the k largest
 * scores from the highest down, equal scores to the lower index; w_dev[t,j] = softmax(z)[idx]
 * (unbiased logits), divided by their sum if norm_topk, times routed_scale.  logits_out_dev
 * (fp32 [T,E], may be NULL) receives z.  E <= 256, k <= 16.  With the mat-vec a work-group keeps the
 * activations of eight (bf16) or four (fp32) tokens in LDS: SMOE_ESIZE if they exceed 160 KB (bf16
 * d_model above about 9000, fp32 above about 8000). */
int smoe_route(smoe_ctx* ctx, int T, int E, int k, int d_model, const float* logits_dev,
               const void* x_dev, int act_dtype, const float* w_router_dev, const float* bias_dev,
               int norm_topk, float routed_scale, float* logits_out_dev, int32_t* idx_dev,
               float* w_dev);

/* ---- expert_ffn(mask) (Section 4.1) ------------------------------------------------------- */
/* One token.  y = sum_j w[j] * FFN_{idx[j]}^{prec[j]}(x) + sum_{shared e} gamma * FFN_e^{HIGH}(x)
 * (+ x if add_residual), FFN(x) = Wd (silu(Wg x) * (Wu x)).
 * prec[j] = HIGH iff (slice_mask[idx[j]] & 3) == 3 and (tau_head <= 0 or w[j] >= tau_head):
 * HIGH uses s*(16*msb + lsb - zp), LOW uses 16*s*(msb - floor(zp/16)) and never reads the LSB
 * plane.  gamma = 1, or sigmoid(shared_gate_w . x) when shared_gate_w_dev (act_dtype [d_model]) is
 * given.  `routed` may be NULL with k = 0 (dense FFN through `shared`); `shared` may be NULL.
 * x_dev, y_dev: act_dtype [d_model]; idx_dev int32 [k]; w_dev fp32 [k]; slice_mask_dev uint8 [E];
 * prec_out_dev uint8 [k] or NULL.  y_dev may not alias x_dev.
 * idx_dev lives in device memory, so the host cannot validate it: an index outside [0, n_experts)
 * is clamped to the nearest valid expert by the kernel (no error, no access outside the bank).
 * Limits of the decode entry points: d_model <= 8192 (SMOE_ENOTIMPL beyond) and a multiple of 8,
 * group = 32 * 2^n, k <= 16, at most 8 shared experts, one scale dtype and one nest per layer, and
 * k * d_ff + n_shared * shared_d_ff floats of intermediates within the ctx workspace (SMOE_ESIZE). */
int smoe_expert_ffn(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared,
                    const void* x_dev, int act_dtype, int k, const int32_t* idx_dev,
                    const float* w_dev, const uint8_t* slice_mask_dev, float tau_head,
                    const void* shared_gate_w_dev, int add_residual, void* y_dev,
                    uint8_t* prec_out_dev);

/* route + expert_ffn for one token without a host round trip between them; same results as the
 * two calls.  logits_dev fp32 [E] or NULL (then w_router_dev is used); idx_out_dev / w_out_dev /
 * prec_out_dev ([k], may be NULL) receive the routing decision for the host's cache bookkeeping. */
int smoe_decode_layer(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared,
                      const void* x_dev, int act_dtype, int k, const float* logits_dev,
                      const float* w_router_dev, const float* bias_dev, int norm_topk,
                      float routed_scale, const uint8_t* slice_mask_dev, float tau_head,
                      const void* shared_gate_w_dev, int add_residual, void* y_dev,
                      int32_t* idx_out_dev, float* w_out_dev, uint8_t* prec_out_dev);

/* smoe_decode_layer for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, bit-identical
 * results; the workspace (routing record, router logits, fp32 SwiGLU vectors) is a file-scope device
 * array of smoe_static_scratch_bytes() = 512 KiB inside the library instead of the context's buffer,
 * so the context may have been created without one.  Every GPU the library has run this call on holds
 * its own copy of that array until the process ends.  The call makes no hipMalloc / hipFree and no
 * allocating library call.  Limit: 64 KiB + 4 * (k * d_ff + n_shared * shared_d_ff) bytes must fit the
 * array (114,688 floats of intermediates); SMOE_ESIZE beyond, before any device work.  All calls on one
 * GPU share the array and it keeps the last call's contents (nothing in it needs clearing: every word
 * read by a call was written by that call first); calls that overlap in time on one GPU -- two
 * streams, two contexts, two threads -- race on it and must be serialised by the caller. */
int smoe_static_scratch_bytes(size_t* bytes);
int smoe_decode_layer_static(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared,
                             const void* x_dev, int act_dtype, int k, const float* logits_dev,
                             const float* w_router_dev, const float* bias_dev, int norm_topk,
                             float routed_scale, const uint8_t* slice_mask_dev, float tau_head,
                             const void* shared_gate_w_dev, int add_residual, void* y_dev,
                             int32_t* idx_out_dev, float* w_out_dev, uint8_t* prec_out_dev);

/* smoe_decode_layer for T tokens (1 <= T <= 16) that pass the same layer in one pair of launches,
 * e.g. the draft tokens of a speculative step or a small batch: token t uses row t of x_dev
 * [T, d_model], logits_dev [T, E] (required: no router mat-vec here), y_dev [T, d_model] and of the
 * optional outputs idx_out_dev / w_out_dev / prec_out_dev [T, k]; bias and slice mask are shared.
 * Every token is computed exactly as by smoe_decode_layer.  The work-groups that need the same
 * weight rows for different tokens run side by side on one XCD, so the weights they share (shared
 * experts, coinciding routed experts) come from HBM once and from L2 afterwards.  T > 1 needs
 * d_model a multiple of 64 (SMOE_ESHAPE otherwise). */
int smoe_decode_layer_multi(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int T,
                            const void* x_dev, int act_dtype, int k, const float* logits_dev,
                            const float* bias_dev, int norm_topk, float routed_scale,
                            const uint8_t* slice_mask_dev, float tau_head, const void* shared_gate_w_dev,
                            int add_residual, void* y_dev, int32_t* idx_out_dev, float* w_out_dev,
                            uint8_t* prec_out_dev);

/* ---- prefill_histogram (Section 4.3) ------------------------------------------------------ */
/* Bytes of device scratch smoe_prefill_histogram needs for T tokens; shared_d_ff = d_ff of the shared
 * experts (0 without a shared bank). */
int smoe_prefill_bytes(int T, int E, int k, int d_model, int d_ff, int shared_d_ff, size_t* scratch_bytes);
/* T tokens through one layer, every expert HIGH: routes each token (as smoe_route), counts
 * hist_dev[e] = number of (token, slot) pairs sent to expert e (uint32 [E], overwritten), runs the
 * experts as a grouped GEMM over the tokens of each expert, and writes
 * y_dev[t] = sum_j w[t,j] * FFN_{idx[t,j]}(x[t]) + gamma[t] * sum_shared FFN_s(x[t]) (+ x[t] if
 * add_residual), gamma[t] = sigmoid(shared_gate_w . x[t]) or 1 without a gate vector (act dtype
 * [d_model]); the shared experts see every token and run as dense GEMMs.
 * x_dev, y_dev: act_dtype [T, d_model] (bf16 only); idx_dev int32 [T,k]; w_dev fp32 [T,k].
 * d_model and every d_ff must be multiples of 64, groups powers of two >= 32. */
int smoe_prefill_histogram(smoe_ctx* ctx, const smoe_bank* routed, const smoe_bank* shared, int T,
                           const void* x_dev, int act_dtype, int k, const float* logits_dev,
                           const float* w_router_dev, int norm_topk, float routed_scale,
                           const void* shared_gate_w_dev, int add_residual, void* scratch_dev,
                           size_t scratch_bytes, void* y_dev, int32_t* idx_dev, float* w_dev,
                           uint32_t* hist_dev);

/* Host only.  Retention order after prefill, hottest first: slice id = ((layer*E + expert) << 1)
 * | is_lsb; every MSB slice before any LSB slice, within a plane by descending count, equal counts
 * by ascending layer then expert.  Writes min(N, 2*L*E) ids, returns that number in *n_out. */
int smoe_topn_slices(const uint32_t* hist_host, int L, int E, int N, uint32_t* slice_ids_host,
                     int* n_out);

/* ---- host bookkeeping that produces the mask (Section 4.1; Section 6.1 item 3); no device work -------- */
/* One LRU over the slices of all layers; capacity in slices (>= 2). */
int smoe_cache_create(int L, int E, int capacity_slices, smoe_cache** out);
int smoe_cache_destroy(smoe_cache* c);
/* Replaces the contents by slice_ids[0..n) (most recently used first), truncated to capacity. */
int smoe_cache_init_order(smoe_cache* c, const uint32_t* slice_ids, int n);
/* slice_mask[e] and bias[e] = beta if the MSB slice of (layer, e) is resident else 0. */
int smoe_cache_snapshot(const smoe_cache* c, int layer, float beta, uint8_t* slice_mask_host,
                        float* bias_host);
/* Applies one token's accesses in slot order.  MSB: hit -> most recent; miss -> fetched, most
 * recent.  LSB (only if want_high[j]): hit -> position unchanged; miss -> fetched, placed as the
 * next eviction victim.  A fetch into a full cache first evicts the least recent slice. */
int smoe_cache_access(smoe_cache* c, int layer, int k, const int32_t* idx_host,
                      const uint8_t* want_high_host);
/* The same for one token's pass through all L layers, in layer order: the snapshot fills
 * slice_mask_host[L*E] (and bias_host[L*E] unless NULL); the access takes the selections of layer l
 * at idx_host[l*idx_stride .. l*idx_stride + k) (idx_stride >= k, so rows padded for alignment can be
 * passed as they are) and want_high_host[l*k .. ) (NULL = no LSB requests).  Either all layers are
 * applied or, on an invalid index, none. */
int smoe_cache_snapshot_all(const smoe_cache* c, float beta, uint8_t* slice_mask_host, float* bias_host);
int smoe_cache_access_all(smoe_cache* c, int k, const int32_t* idx_host, int idx_stride,
                          const uint8_t* want_high_host);
int smoe_cache_stats_get(const smoe_cache* c, smoe_cache_stats* out);
/* Copies the resident slice ids, most recent first; returns their number in *n_out. */
int smoe_cache_order(const smoe_cache* c, uint32_t* slice_ids_host, int max_n, int* n_out);

/* ---- modeled cost of a decode trace on the paper's target system (Section 5; Figs. 9, 10) --- */
/* The paper evaluates energy and latency on a modeled device: an 8-bit PE array fed from LPDDR4
 * DRAM that holds the slice cache, with UFS Flash behind it holding every slice.  Host only. */
typedef struct {
  double flash_gbit_s;      /* Flash -> DRAM bandwidth, Gbit/s */
  double dram_gbit_s;       /* DRAM bandwidth, Gbit/s */
  double xpu_tops;          /* PE array throughput, tera-operations/s */
  double flash_pj_bit;      /* Flash access energy, pJ/bit */
  double dram_pj_bit;       /* DRAM read or write energy, pJ/bit */
  double xpu_tops_w;        /* PE array efficiency, tera-operations/s per watt */
} smoe_system_spec;

typedef struct {
  double flash_bits;        /* every missed slice is read from Flash once */
  double dram_bits;         /* every requested slice is read from DRAM; a missed one is written there first */
  double ops;               /* as passed in */
  double energy_j;          /* flash_bits*flash_pj + dram_bits*dram_pj + ops / (xpu_tops_w * 1e12) */
  double latency_s;         /* flash_bits/flash rate + dram_bits/dram rate + ops/xpu rate: the three served one
                               after the other (a missed slice is loaded before it is used) */
  double miss_rate_high;    /* high-bit-normalised miss rate: Flash bytes / (MSB requests * bytes of a
                               whole high-bit expert), i.e. relative to a cache of whole high-bit experts
                               that misses on every request */
} smoe_cost;

/* The system of Section 5: 10 Gbit/s and 103 pJ/bit Flash, 104 Gbit/s and 1.5 pJ/bit DRAM,
 * 16.4 TOPS at 3.18 TOPS/W. */
int smoe_system_spec_paper(smoe_system_spec* out);
/* Cost of the accesses counted in `stats`: msb_slice_bytes / lsb_slice_bytes are the bytes of one
 * MSB / LSB slice of one expert (planes of its three matrices + metadata with the MSB slice);
 * ops = operations of the expert FFNs of the trace (2 per multiply-accumulate).  SMOE_EINVAL for
 * null pointers or a non-positive rate. */
int smoe_cost_model(const smoe_system_spec* spec, const smoe_cache_stats* stats, uint64_t msb_slice_bytes,
                    uint64_t lsb_slice_bytes, double ops, smoe_cost* out);

#ifdef __cplusplus
}
#endif
#endif /* SLICEMOE_H */
