/*
 * hot.h - C ABI of the MI355X (gfx950) implementation of the HOT linear-layer
 * backward pass (arxiv 2503.21261, "HOT: Hadamard-based Optimized Training").
 *
 * Notation (Sec. 4.1, Eq. 7-8): x [L x I] input activation, w [O x I] weight,
 * y = x.w^T [L x O], g_y [L x O] output gradient,
 *     g_x = g_y . w   [L x I]      g_w = g_y^T . x   [O x I].
 * L is the flattened token index (batch x sequence), tiled consecutively in
 * blocks of n for the token-direction transform.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers to row-major, contiguous buffers,
 *     16-byte aligned, fp32 unless stated.  Pointers marked "host" are host
 *     memory.  The caller owns every buffer; the library never allocates, frees
 *     or keeps device memory between calls.
 *   - `ws` is caller-provided device scratch of at least hot_workspace_bytes()
 *     bytes, 256-byte aligned (checked: HOT_ERR_ARG otherwise).  Its first
 *     HOT_WS_PREFIX_BYTES hold scalars, exchange slots and flags; the packed
 *     operands of the call follow, and the hot_debug_* calls decode them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return without synchronising, except
 *     hot_select_quantizer, which waits for its own result.
 *   - Errors are return codes; arguments are checked on the host before any
 *     launch, so a failing call has launched nothing.  Inputs must be finite.
 *   - Two calls that share a workspace or an output must be ordered by the
 *     caller (same stream, or events).
 *   - HIP graphs: the kernels whose workgroups exchange values through the
 *     workspace (single-pass transforms, split-K GEMM) tell a launch's values
 *     from stale ones by a tag.  By default the host chooses it per call, and a
 *     replayed graph would repeat it: such calls must not be recorded.  With
 *     hot_config.replayable set, every call first advances a 64-bit epoch in the
 *     workspace (one more one-thread kernel) and the kernels derive their tags
 *     from it on the device, so that the call may be recorded and replayed (with
 *     the buffers it was recorded with; call it once with the same shapes before
 *     recording: launch plans are made on first use).  hot_select_quantizer waits
 *     for its result and cannot be recorded either way.
 */
#ifndef HOT_H
#define HOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HOT_OK = 0,
  HOT_ERR_ARG = 1,        /* null pointer, bad enum, bad config field            */
  HOT_ERR_SHAPE = 2,      /* a size the method or the int32 accumulators forbid  */
  HOT_ERR_WORKSPACE = 3,  /* ws_bytes smaller than hot_workspace_bytes()         */
  HOT_ERR_DEVICE = 4,     /* a HIP runtime call failed                           */
  HOT_ERR_UNIMPLEMENTED = 5,
  HOT_ERR_SCRATCH_LIMIT = 6 /* hot_linear_backward_gx_noalloc: the shape needs more than
                               HOT_NOALLOC_SCRATCH_BYTES of scratch                      */
} hot_status;

/* Sec. 5.2.2: granularity of the scale of the rotated g_y. */
typedef enum { HOT_Q_PER_TENSOR = 0, HOT_Q_PER_TOKEN = 1 } hot_quantizer;

/* Sec. 5.1: the paper's quantiser rounds pseudo-stochastically; nearest-even is
 * offered so the half-step round-trip bound can be checked. */
typedef enum { HOT_ROUND_NEAREST_EVEN = 0, HOT_ROUND_PSEUDO_STOCHASTIC = 1 } hot_rounding;

typedef struct {
  int32_t block;           /* n: WHT tile, 16 (paper, Supp. D) | 32 | 64                */
  int32_t keep;            /* r: rows of each n-block kept by HLA on the g_w path,
                              1..n (paper: 8 of 16, Supp. B)                          */
  const int32_t* keep_idx; /* host, r distinct natural-order row indices in [0,n), or
                              NULL = the r rows of lowest sequency, by increasing
                              sequency (Sec. 3.3)                                     */
  int32_t gx_bits;         /* 4 (paper, Sec. 5.1) | 8 (INT8 warm-up, Supp. B)         */
  int32_t gw_bits;         /* 8 (Sec. 5.2) | 16: bfloat16 operands, fp32 accumulation   */
  int32_t rounding;        /* hot_rounding                                            */
  float lqs_threshold;     /* 0.5 (Sec. 5.2.2)                                        */
  int32_t sample_tokens;   /* 0: the L tokens are one run, tiled in blocks of n (needs
                              L % n == 0).  S > 0: L = B x S tokens of B samples; the
                              token-direction transform (ABC, g_w path) tiles every sample
                              separately and pads its last block with zero tokens, so
                              S need not be a multiple of n (ViT: S = 197); then
                              L*r/n below reads B * ceil(S/n) * r                       */
  int32_t replayable;      /* 0: launch tags from the host (default).  1: from an epoch in
                              the workspace that every call advances with one more
                              launch; calls may then be recorded into a HIP graph        */
} hot_config;

/* Fills *cfg with the paper's defaults: n = 16, r = 8, low-sequency rows, INT4 /
 * INT8, pseudo-stochastic rounding, threshold 0.5, one run of tokens, host tags. */
void hot_default_config(hot_config* cfg);

const char* hot_status_string(hot_status s);

/* Bytes of the compressed activation buffer for x [L x I] (Sec. 5.2.1): a
 * 256-byte header holding the scale, then L*r/n x I INT8 codes stored with the
 * reduced token index contiguous (row pitch rounded up to 128 bytes).  Returns 0
 * for an invalid config or shape. */
size_t hot_act_buffer_bytes(const hot_config* cfg, int64_t L, int64_t I);

/* Bytes every workspace starts with (scales, abs-max exchange slots, split-K flags); the
 * whole workspace of hot_compress_activation and hot_quantize_weight. */
#define HOT_WS_PREFIX_BYTES 24832

/* Scratch bytes sufficient for every call below at this (L, O, I); 0 = invalid.  A function
 * of the configuration and the shape only: launch plans, and with them the scratch of the
 * split-K GEMMs, are made for the 256 compute units of the MI355X whatever device is
 * current. */
size_t hot_workspace_bytes(const hot_config* cfg, int64_t L, int64_t O, int64_t I);

/*
 * Activation Buffer Compression, Sec. 5.2.1, run right after the forward pass:
 *   x_hat = rows keep_idx of (H_n applied to every block of n consecutive tokens
 *   of x), INT8 with one abs-max scale for the tensor.
 * x: device [L x I] (in).  act_buf: device, hot_act_buffer_bytes() bytes (out).
 * ws: at least HOT_WS_PREFIX_BYTES (nothing beyond them is touched).
 * Requires L % n == 0, L*r/n <= 133144.
 */
hot_status hot_compress_activation(const hot_config* cfg, const float* x, int64_t L, int64_t I,
                                   void* act_buf, void* ws, size_t ws_bytes, void* stream);

/*
 * Activation-gradient path, Sec. 5.1 (Eq. 3-4 with Q = INT4):
 *   g_x = dequant( Q(g_y.H^T) . Q(H.w) ),  H block-diagonal along O.
 * g_y: device [L x O] (in); w: device [O x I] (in); g_x: device [L x I] (out).
 * gy_quantizer: scale of the rotated g_y per token or per tensor (Sec. 4.3,
 * 5.2.2); the rotated w always has one scale.  Requires O % n == 0.
 */
hot_status hot_linear_backward_gx(const hot_config* cfg, const float* g_y, const float* w,
                                  int64_t L, int64_t O, int64_t I, hot_quantizer gy_quantizer,
                                  float* g_x, void* ws, size_t ws_bytes, void* stream);

/*
 * hot_linear_backward_gx for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture set-up, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same g_x bit for bit, but the scratch is
 * an array inside the library's code object (HOT_NOALLOC_SCRATCH_BYTES, 64 MiB, held on
 * every GPU the library runs on until the process ends) instead of `ws`.  The call
 * allocates and frees nothing, on the device or through any library.
 *   - A shape whose hot_linear_backward_gx workspace layout exceeds the array returns
 *     HOT_ERR_SCRATCH_LIMIT before anything is launched (ViT-B fc1 at 12608 tokens needs
 *     59.5 MB and fits; 50432 tokens do not).
 *   - The array belongs to the device that is current at the call; `stream` must be a
 *     stream of that device.
 *   - All calls on one GPU share the array, which keeps the last call's contents.  Nothing
 *     in it has to be cleared between calls, but two calls that overlap in time on one GPU
 *     (different streams, different threads) race on it: order them.
 */
#define HOT_NOALLOC_SCRATCH_BYTES (64u << 20)
hot_status hot_linear_backward_gx_noalloc(const hot_config* cfg, const float* g_y, const float* w,
                                          int64_t L, int64_t O, int64_t I,
                                          hot_quantizer gy_quantizer, float* g_x, void* stream);

/*
 * Frozen weights (Sec. 5.3: with LoRA-style fine-tuning the base weights stay fixed and
 * only g_x is needed): quantise H.w once, reuse it every step.
 * hot_weight_buffer_bytes: a 256-byte header holding the scale, then I rows of O codes
 * (gx_bits each, row pitch rounded up to 128 bytes); 0 for an invalid config or shape.
 * hot_quantize_weight: w device [O x I] (in) -> wq_buf device (out); ws: at least
 * HOT_WS_PREFIX_BYTES.
 * hot_linear_backward_gx_cached: hot_linear_backward_gx with the weight operand taken
 * from wq_buf (same cfg, O, I); same g_x bit for bit.  Its ws holds no weight codes:
 * hot_gx_cached_workspace_bytes() (never more than hot_workspace_bytes()) is enough, and a
 * smaller one is HOT_ERR_WORKSPACE.
 */
size_t hot_weight_buffer_bytes(const hot_config* cfg, int64_t O, int64_t I);
size_t hot_gx_cached_workspace_bytes(const hot_config* cfg, int64_t L, int64_t O, int64_t I);
hot_status hot_quantize_weight(const hot_config* cfg, const float* w, int64_t O, int64_t I,
                               void* wq_buf, void* ws, size_t ws_bytes, void* stream);
hot_status hot_linear_backward_gx_cached(const hot_config* cfg, const float* g_y,
                                         const void* wq_buf, int64_t L, int64_t O, int64_t I,
                                         hot_quantizer gy_quantizer, float* g_x, void* ws,
                                         size_t ws_bytes, void* stream);

/*
 * Weight-gradient path, Sec. 5.2 (Eq. 5 with INT8 operands):
 *   g_w = dequant( Q(HLA(g_y))^T . x_hat ),  HLA along the token index L.
 * With gw_bits = 16 (g_w is the gradient Sec. 4.2 finds sensitive to quantisation) the two
 * low-rank operands are rounded to bfloat16 instead (nearest even, no scales; the
 * activation buffer is then 25 % of fp32), multiplied on the bf16 matrix cores with fp32
 * accumulation and divided by n; no limit on L*r/n.
 * g_y: device [L x O] (in); act_buf: what hot_compress_activation wrote for the
 * same cfg, L, I (in); g_w: device [O x I] (out).  Requires L % n == 0.
 */
hot_status hot_linear_backward_gw(const hot_config* cfg, const float* g_y, const void* act_buf,
                                  int64_t L, int64_t O, int64_t I, float* g_w, void* ws,
                                  size_t ws_bytes, void* stream);

/*
 * Both gradients of one layer in one call (Sec. 5.1 and 5.2 on the same g_y): the same
 * g_x and g_w, bit for bit, as hot_linear_backward_gx followed by
 * hot_linear_backward_gw.  Where it is faster (16-row blocks and a g_y too large for the
 * single-pass token-direction kernel) the two quantised views of g_y (rotated along O,
 * and HLA-compressed along L) come out of shared reads of g_y: two passes over it instead
 * of three; otherwise the two separate paths run one after the other.
 * Arguments as for the two separate calls.  Requires O % n == 0 and L % n == 0
 * (or whole samples with sample_tokens).
 */
hot_status hot_linear_backward(const hot_config* cfg, const float* g_y, const float* w,
                               const void* act_buf, int64_t L, int64_t O, int64_t I,
                               hot_quantizer gy_quantizer, float* g_x, float* g_w, void* ws,
                               size_t ws_bytes, void* stream);

/*
 * Layer-wise Quantizer Selection, Sec. 5.2.2, for one layer's calibration g_y:
 * mean squared error between g_y and its rotated, gx_bits-quantised,
 * de-rotated version with per-token and with per-tensor scales; per-token is
 * chosen iff mse_tensor > 0 and (mse_tensor - mse_token) >= lqs_threshold *
 * mse_tensor.  choice / mse_token / mse_tensor are HOST pointers (the two MSE
 * pointers may be NULL).  Synchronises the stream.
 */
hot_status hot_select_quantizer(const hot_config* cfg, const float* g_y, int64_t L, int64_t O,
                                hot_quantizer* choice, double* mse_token, double* mse_tensor,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * Low-pass rows by the LP_L1 criterion (Supp. B, "Hyper-parameter of HLA": the paper keeps
 * the top 8 of 16 vectors by the LP_L1 criterion of the 2-D transform it builds on).  Host
 * only.  Reading taken (the criterion is defined in that earlier work, not in the paper):
 * the n tokens of a block are a grid in raster order (4 x 4 for n = 16, 8 x 8 for n = 64,
 * 4 rows of 8 for n = 32); H_n = H_rows (x) H_cols, so natural row k = a * cols + b has
 * vertical sequency seq(a) and horizontal sequency seq(b); rows are listed by increasing
 * seq(a) + seq(b), ties by increasing max of the two, then by increasing seq(a).
 * keep_idx: host, `keep` entries (out), to be passed as hot_config.keep_idx.
 */
hot_status hot_lowpass_l1_rows(int32_t block, int32_t keep, int32_t* keep_idx);

/* ---- parity views (not on the timed path): logical forms of packed data ---- */

/* Compressed activation as row-major codes [L*r/n x I] and its scale [1].  With
 * gw_bits = 16 `codes` receives bfloat16 bit patterns, two bytes each (pass an int16
 * buffer), and the scale is 1. */
hot_status hot_debug_unpack_activation(const hot_config* cfg, const void* act_buf, int64_t L,
                                       int64_t I, int8_t* codes, float* scale, void* stream);

/* Quantised weights as row-major codes [O x I] (one code per byte) and their scale [1]. */
hot_status hot_debug_unpack_weight(const hot_config* cfg, const void* wq_buf, int64_t O, int64_t I,
                                   int8_t* codes, float* scale, void* stream);

/* Operands left in `ws` by the last hot_linear_backward_gx with these arguments:
 * codes of the rotated g_y [L x O] and w [O x I] (row-major, one code per byte),
 * scales of g_y ([L] per token, [1] per tensor) and of w [1], and the int32
 * integer product [L x I] recomputed from those operands by the GEMM the call itself
 * used (the GEMM scratch at the end of `ws` is overwritten).  Any output may be NULL. */
hot_status hot_debug_gx_operands(const hot_config* cfg, void* ws, int64_t L, int64_t O,
                                 int64_t I, hot_quantizer gy_quantizer, int8_t* gy_codes,
                                 float* gy_scales, int8_t* w_codes, float* w_scale, int32_t* acc,
                                 void* stream);

/* Operands left in `ws` by the last hot_linear_backward_gw: codes of HLA(g_y)
 * [L*r/n x O] row-major, its scale [1], and the int32 product [O x I] recomputed
 * from those codes and act_buf.  Any output may be NULL.  With gw_bits = 16 the codes are
 * bfloat16 bit patterns (two bytes each) and `acc` receives the fp32 accumulators' bit
 * patterns. */
hot_status hot_debug_gw_operands(const hot_config* cfg, void* ws, const void* act_buf,
                                 int64_t L, int64_t O, int64_t I, int8_t* gy_codes,
                                 float* gy_scale, int32_t* acc, void* stream);

/* Operands left in `ws` by the last hot_linear_backward (block size 16 or 32): the
 * outputs of both views above.  Any output may be NULL. */
hot_status hot_debug_fused_operands(const hot_config* cfg, void* ws, const void* act_buf,
                                    int64_t L, int64_t O, int64_t I, hot_quantizer gy_quantizer,
                                    int8_t* gy_codes, float* gy_scales, int8_t* w_codes,
                                    float* w_scale, int32_t* acc_gx, int8_t* gyT_codes,
                                    float* gyT_scale, int32_t* acc_gw, void* stream);

/* Strategy of hot_linear_backward: 0 = chosen by the library (default), 1 = always the two
 * separate paths, 2 = the shared passes over g_y whenever they exist (block sizes 16 and
 * 32, INT8 g_w operands, one run of tokens), 3 = the separate paths with every kernel in a
 * launch of its own (by default the g_x path quantises small weights and the per-token g_y
 * operand in one combined launch; the setting also applies to hot_linear_backward_gx).
 * Results do not depend on it.  Process-wide. */
hot_status hot_debug_set_backward_strategy(int strategy);

/* Tensors small enough to stay in the register files of the resident workgroups (x and
 * w of the ViT-sized layers) are transformed and quantised by a single-pass kernel whose
 * workgroups exchange their abs-max through the workspace and wait for each other at most
 * `us` microseconds (default 200) before computing what is missing themselves; results
 * do not depend on the value.  us = 0: never wait (exercises the self-computed path);
 * us < 0: always use the two-pass kernels.  The same bound (us <= 0: never wait) applies
 * to a split-K GEMM's wait for another workgroup's partial sums.  Process-wide setting. */
hot_status hot_debug_set_exchange_wait_us(int us);

/* Work distribution of the GEMMs: 0 = chosen by the library (default: K is split for
 * outputs with no more tiles than compute units), 1 = one workgroup per output tile,
 * s = 2..8: the K range cut into s slices, one workgroup each, wherever a split of the
 * 128x128 tile applies (integer operands, at least 4 K stages per slice); the slices'
 * partial sums are handed to the last one through the workspace; 10 / 11 / 12 / 13: every
 * GEMM on 128x128 / 192x256 / 256x256 / 128x256 tiles, one workgroup per tile (11 and 13
 * exist for INT4 operands only; INT8 and bfloat16 GEMMs then take 256x256).  Integer results, and therefore all outputs, do not depend on it.
 * Process-wide. */
hot_status hot_debug_set_gemm_mode(int mode);

/* ---- stage timing for benchmarks (off by default) ---- */

/* Kernel roles timed separately; hot_debug_stage_name() gives their names. */
#define HOT_NUM_STAGES 15

/* From this call on, every kernel the library launches is bracketed by two HIP
 * events recorded on its stream.  Host-side state only; not thread-safe against
 * concurrent hot_* calls from other threads' streams being interleaved. */
hot_status hot_debug_profile_begin(void);

/* Stops recording, waits for the recorded events, and returns per stage the
 * summed elapsed milliseconds and the number of launches (host arrays of
 * HOT_NUM_STAGES entries). */
hot_status hot_debug_profile_end(float* stage_ms, int64_t* stage_launches);

/* The stages of the recording that the last hot_debug_profile_end closed, in launch order:
 * writes up to `capacity` stage ids to `stages` (host; may be NULL) and returns how many
 * launches there were. */
int64_t hot_debug_profile_sequence(int32_t* stages, int64_t capacity);

const char* hot_debug_stage_name(int stage);

/* Machine-peak probes (context for the roofline figures, not the method): one launch of
 * kind 0 = read `bytes` of buf, 1 = write them (4 = with the streaming, non-temporal, hint the
 * GEMM epilogue uses), 2 / 3 = `iters` x 16 int8 32x32x32 matrix
 * instructions per wave on all SIMDs with constant / pseudo-random register operands
 * (buf, >= 1 MiB, receives a checksum).  The caller times the launch. */
hot_status hot_debug_probe(int kind, void* buf, size_t bytes, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HOT_H */
