/*
 * fade.h — C ABI of libfade: FADE's batched probability step and per-stream arithmetic coder on one
 * AMD MI355X (gfx950), hand-written HIP.
 *
 * For B independent byte streams advancing in lock-step the library computes, per step,
 *   context window -> embedding -> Dual-Stream Multi-Scale Decoupler (rolling-cache global stream,
 *   causal-conv local stream, content-adaptive router) -> Hierarchical Gated Refiner -> 256-way softmax
 *   -> integer frequency table summing to 2^16 -> arithmetic encode / decode of the next byte,
 * and, in online mode, the matching backward pass and Adam update.
 * (Paper: Method section — Preliminaries, Eq. 1-10; appendix Algorithm 1; loss Eq. 12.)
 *
 * Conventions
 *   - `*_dev` arguments are HIP device pointers on the context's device; `*_host` are host pointers.
 *     The caller owns every buffer it passes; the library copies what it keeps.
 *   - All tensors are dense, row-major, without padding unless a stride argument says otherwise.
 *   - Every call returns FADE_OK (0) or a negative FADE_E_* code; fade_last_error() gives a message.
 *     Nothing throws or aborts across this boundary. After an error the context stays destroyable;
 *     output buffers are unspecified.
 *   - Calls on one context must not overlap in time. All device work of a call is enqueued on the
 *     context's stream (`hip_stream`, or a stream the library creates); calls that return results to the
 *     host synchronise that stream before returning, device-only calls (fade_step_*) do not.
 *   - Without a GPU or without the compiled kernels every compute call fails with FADE_E_HIP: there is
 *     no CPU fallback.
 */
#ifndef FADE_H
#define FADE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

#define FADE_ABI_VERSION 2u

typedef struct fade_ctx fade_ctx; /* opaque; owns all device state */

enum { FADE_F32 = 0, FADE_BF16 = 1 };            /* operand type of the matrix products (accumulation is fp32) */
enum { FADE_FROZEN = 0, FADE_ONLINE_ADAM = 1 };  /* weights fixed | updated after every coded symbol */

typedef struct {
  uint32_t struct_size;  /* sizeof(fade_config) */
  uint32_t abi_version;  /* FADE_ABI_VERSION */
  uint32_t B;            /* streams coded in lock-step (batch axis; stream k owns slice k of W_U) */
  uint32_t T;            /* context window in bytes ("time steps") */
  uint32_t D;            /* embedding dimension; D_h = T * D */
  uint32_t H;            /* hidden width: rolling-cache width D_cache and refiner width D_e unless given below */
  uint32_t d_low;        /* d_h of Eq. 7 (low-rank width of the per-stream memory); 0 => 64 */
  uint32_t cache_chunk;  /* c: width of one rolling-cache slot (GeGLU output of Eq. 1); 0 => D_cache / T */
  uint32_t conv_k;       /* taps of the causal Conv1d of Eq. 4; 0 => 3 */
  uint32_t d_cache;      /* D_cache, width of the rolling cache M (T slots of c); 0 => H */
  uint32_t d_e;          /* D_e, expansion width of the fine refiner (Eq. 9-10); 0 => H */
  uint32_t ablation;     /* which prefix of the model feeds the output head (the paper's progressive ablation):
                          * 0 or 5 the full model; 1 the global stream alone (H_global, Eq. 3); 2 the decoupler (H_mix,
                          * Eq. 6); 3 channel interaction without its gate (H_a + lambda_c H_mix); 4 with the gate
                          * (H_coarse, Eq. 8). With FADE_ONLINE_ADAM the stages behind the cut get no gradient and stay as
                          * loaded. The weight blob is the same. */
  uint32_t dtype;        /* FADE_F32 | FADE_BF16 */
  uint32_t update_mode;  /* FADE_FROZEN | FADE_ONLINE_ADAM */
  float lr, beta1, beta2, eps; /* Adam; 0 => 1e-3, 0.9, 0.999, 1e-8 */
  int32_t device;        /* HIP device ordinal */
  void *hip_stream;      /* hipStream_t to enqueue on; NULL => the library creates one */
} fade_config;

enum {
  FADE_OK = 0,
  FADE_E_INVALID_ARG = -1,      /* NULL pointer, wrong struct_size / abi_version, size mismatch */
  FADE_E_BAD_CONFIG = -2,       /* dimensions the model or the kernels do not support (see fade_create) */
  FADE_E_NO_WEIGHTS = -3,       /* compute call before fade_load_weights */
  FADE_E_WEIGHTS_MISMATCH = -4, /* blob size wrong, or container written with other weights */
  FADE_E_BUFFER_TOO_SMALL = -5, /* *dst_len is set to the size needed */
  FADE_E_CORRUPT_STREAM = -6,   /* container fails validation or the coder leaves its interval */
  FADE_E_HIP = -7,              /* a HIP call failed, no device, or kernels not built */
  FADE_E_OOM = -8,              /* host or device allocation failed */
  FADE_E_NUMERIC = -9           /* non-finite weights or probabilities */
};

/* Bytes of the canonical weight blob for a configuration (0 if the configuration is invalid). The blob is
 * fp32, tensors back to back in this order, every matrix row-major [in][out] so that y = x W:
 *   E[256][D]; gamma_e[D]; beta_e[D]; gamma_l[D]; beta_l[D]; W_g[D][c]; W_v[D][c]; W_m[D_cache][D_h]; lambda_m[1];
 *   W_conv[k][D][D]; b_conv[D]; W_r[D_h][D_h]; gamma_c[D_h]; beta_c[D_h]; W_down[D_h][d_low];
 *   W_U[B][d_low][d_low]; W_up[d_low][D_h]; W_c[D_h][D_h]; lambda_c[1]; gamma_f[D_h]; beta_f[D_h];
 *   W_fg[D_h][D_e]; W_fv[D_h][D_e]; W_f[D_e][D_h]; gamma_o[D_h]; beta_o[D_h]; lambda_o[1]; W_o[D_h][256]; b_o[256].
 * (E, W_g/W_v: Eq. 1; W_m, lambda_m: Eq. 3; W_conv: Eq. 4; W_r: Eq. 5; W_down/W_U/W_up: Eq. 7; W_c, lambda_c:
 * Eq. 8; W_fg/W_fv: Eq. 9; W_f, lambda_o: Eq. 10; W_o/b_o: the 256-way output head the problem statement
 * implies. gamma_e/beta_e normalise X per token; gamma_l/beta_l are Eq. 4's LN; gamma_c, gamma_f, gamma_o are
 * the LNs of Eq. 7, 9, 10.) */
size_t fade_weights_nbytes(const fade_config *cfg);

/* Create a context: validates the configuration and allocates all device state (compute weights, rolling
 * caches M [B][D_cache], per-stream memories W_U, activations, coder state; optimiser state in online mode).
 * Supported shapes: D % 32 == 0 (FADE_BF16) or D % 16 == 0 (FADE_F32), (T*D) % 128 == 0, D_cache % 64 == 0 and
 * D_cache <= 4096, D_e % 64 == 0 and D_e <= 8192, d_low == 64, conv_k <= 4, D_cache % cache_chunk == 0,
 * cache_chunk <= 256; with FADE_ONLINE_ADAM also T*D <= 2048, D <= 32, T a divisor of 128 and D a divisor of 256;
 * anything else is FADE_E_BAD_CONFIG. No device, or a device ordinal out of range: FADE_E_HIP. *out is NULL on failure. */
int fade_create(const fade_config *cfg, fade_ctx **out);

/* Load the canonical fp32 blob from host memory (copied; rounded to bf16 for FADE_BF16 matrix operands) and
 * reset the context. nbytes must equal fade_weights_nbytes(). Non-finite values: FADE_E_NUMERIC. */
int fade_load_weights(fade_ctx *ctx, const void *blob_host, size_t nbytes);

/* Zero the rolling caches and coder state, restore the loaded weights and zero the optimiser state. */
int fade_reset(fade_ctx *ctx);

/* One model step for all B streams (Eq. 1-10, head, softmax, quantiser). STATEFUL: rolls each active
 * stream's cache (Eq. 2), so calls must follow stream order.
 *   windows_dev [B][T] bytes, oldest first: the T symbols preceding the one to be coded.
 *   active_dev  [B] bytes or NULL (all active); inactive streams are skipped (no cache roll, outputs untouched).
 *   freq_dev    [B][256] uint16 or NULL: f >= 1, each row summing to 65536.
 *   probs_dev   [B][256] float or NULL: the softmax output the table was quantised from.
 * Enqueues on the context's stream and returns without synchronising. */
int fade_step_probs(fade_ctx *ctx, const uint8_t *windows_dev, const uint8_t *active_dev, uint16_t *freq_dev,
                    float *probs_dev);

/* Online mode only: mean NLL (Eq. 12) of targets_dev[B] over the active streams under the probabilities of
 * the preceding fade_step_probs, backward through the step, one Adam update of every parameter (shared
 * weights and each active stream's W_U slice). The library keeps its own copy of that call's windows, so the caller's
 * window buffer need not outlive fade_step_probs. Asynchronous like fade_step_probs. */
int fade_step_update(fade_ctx *ctx, const uint8_t *targets_dev, const uint8_t *active_dev);

/* Upper bound of the container size for n input bytes. */
size_t fade_encode_bound(const fade_ctx *ctx, size_t n);

/* Compress n bytes (Algorithm 1): split into B contiguous streams of L = ceil(n / B) bytes (stream k =
 * bytes [kL, min(n, (k+1)L))); the first T symbols of each stream are coded with the uniform table, every
 * later symbol with the model's table, followed in online mode by the update. Resets the context first.
 * Container (little-endian): 64-byte header {magic "FADE", version u16, dtype u8, update_mode u8, T u16, D u16,
 * D_e u32, d_low u16, c u16, k u16, pad u16, B u32, lr, beta1, beta2, eps (f32 bits), D_cache u32 (0 when it equals
 * D_e), n u64, FNV-1a-64 of the weight blob}, then B x u32 payload lengths, then the B payloads. Weights are not stored.
 * Frozen bf16 contexts take several consecutive steps of every stream per pass here and in fade_encode_device (the
 * model's steps are independent once the input is known); the container is byte for byte the one single steps write.
 * The steps per pass are fixed at fade_create (about 16384 / B, at most 256; environment variable
 * FADE_STEPS_PER_PASS overrides, 1 = single steps only) and size the context's activation buffers.
 * The host-buffer calls (fade_encode, fade_decode, fade_payloads, fade_decode_device's payload upload) stage the job and
 * the flat payloads in device buffers that belong to the context: allocated at the first call, grown when a later job is
 * larger, released by fade_destroy; a context that codes job after job of one size allocates once. */
int fade_encode(fade_ctx *ctx, const uint8_t *src_host, size_t n, uint8_t *dst_host, size_t dst_cap, size_t *dst_len);

/* Inverse of fade_encode with the same configuration and weights (checked against the header). */
int fade_decode(fade_ctx *ctx, const uint8_t *src_host, size_t src_len, uint8_t *dst_host, size_t dst_cap,
                size_t *dst_len);

/* Device-resident form of the two loops above, for callers that keep data in HBM (and for timing without
 * PCIe): src_dev / dst_dev hold the n bytes on the device. A job may be run in pieces: each call codes steps
 * [first_step, first_step + n_steps) of every stream (n_steps = 0 => up to the last step L); first_step = 0
 * resets the context and starts a job, any other first_step must continue the job in progress exactly where
 * the previous call stopped (else FADE_E_INVALID_ARG).
 *   fade_encode_device: leaves the per-stream payloads in the context; they are terminated when step L is reached.
 *   fade_payloads: after a complete encode, copies the payload lengths [B] and the concatenated payloads to host
 *     (bytes_host may be NULL with cap 0 to query *total: returns FADE_E_BUFFER_TOO_SMALL then).
 *   fade_decode_device: lengths_host / bytes_host / total as produced by fade_payloads (read when first_step = 0
 *     only, may be NULL afterwards); decoded bytes appear in dst_dev [n].
 * All three synchronise before returning. */
int fade_encode_device(fade_ctx *ctx, const uint8_t *src_dev, size_t n, size_t first_step, size_t n_steps);
int fade_payloads(fade_ctx *ctx, uint32_t *lengths_host /*[B]*/, uint8_t *bytes_host, size_t cap, size_t *total);
int fade_decode_device(fade_ctx *ctx, const uint32_t *lengths_host, const uint8_t *bytes_host, size_t total,
                       uint8_t *dst_dev, size_t n, size_t first_step, size_t n_steps);

/* Stand-alone kernels (parity gates for the integer parts).
 *   fade_quantize: probs_dev [rows][256] float -> freq_dev [rows][256] uint16 by the quantiser rule
 *     f_i = 1 + trunc(fp32(p_i * 65280)), remainder 65536 - sum f added at the lowest index of the maximum.
 *   fade_coder_encode_tables: code n_steps symbols for each of n_streams streams under given tables.
 *     freq_dev [n_steps][n_streams][256], sym_dev [n_steps][n_streams]; out_dev [n_streams][cap] receives each
 *     stream's bytes, len_dev [n_streams] their count (32-bit interval coder after Witten, Neal & Cleary,
 *     totals 2^16, bits MSB first, terminated and zero-padded to a byte).
 *   fade_coder_decode_tables: the inverse; in_dev [n_streams][cap] with len_dev [n_streams].
 * All synchronise before returning. */
int fade_quantize(fade_ctx *ctx, const float *probs_dev, size_t rows, uint16_t *freq_dev);
int fade_coder_encode_tables(fade_ctx *ctx, const uint16_t *freq_dev, const uint8_t *sym_dev, size_t n_steps,
                             size_t n_streams, uint8_t *out_dev, size_t cap, uint32_t *len_dev);
int fade_coder_decode_tables(fade_ctx *ctx, const uint16_t *freq_dev, size_t n_steps, size_t n_streams,
                             const uint8_t *in_dev, size_t cap, const uint32_t *len_dev, uint8_t *sym_dev);

/* fade_coder_encode_tables for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same output bit for bit, but the per-stream coder state lives
 * in a fixed array inside the library's device image (8 x uint32 per stream, FADE_NOALLOC_MAX_STREAMS streams, 2 MiB per
 * GPU, held until the process ends) instead of a temporary allocation. The call allocates and frees nothing.
 * n_streams > FADE_NOALLOC_MAX_STREAMS => FADE_E_INVALID_ARG. Every call on a GPU shares that GPU's array (also across
 * contexts): calls that overlap in time on one GPU race; one after the other they are independent, each call
 * re-initialises the state it uses. Synchronises before returning. */
#define FADE_NOALLOC_MAX_STREAMS 65536
int fade_coder_encode_tables_noalloc(fade_ctx *ctx, const uint16_t *freq_dev, const uint8_t *sym_dev, size_t n_steps,
                                     size_t n_streams, uint8_t *out_dev, size_t cap, uint32_t *len_dev);

/* Debug/test taps: copy an intermediate activation of the most recent step to host as fp32, [B][width].
 * `which` uses FADE_TAP_*; returns the width (0 if unknown); out_host may be NULL to query the width. */
enum {
  FADE_TAP_X = 0, FADE_TAP_CACHE, FADE_TAP_H_GLOBAL, FADE_TAP_H_LOCAL, FADE_TAP_ALPHA, FADE_TAP_H_MIX,
  FADE_TAP_Y_DOWN, FADE_TAP_Z_BMM, FADE_TAP_H_A, FADE_TAP_H_COARSE, FADE_TAP_H_EXPAND, FADE_TAP_H_OUT,
  FADE_TAP_LOGITS, FADE_TAP_PROBS, FADE_TAP_COUNT
};
size_t fade_tap(fade_ctx *ctx, int which, float *out_host, size_t cap_floats);

/* Current master weights as a canonical fp32 blob (after online updates). */
int fade_get_weights(fade_ctx *ctx, void *blob_host, size_t nbytes);

/* Debug/test: the gradient of the mean NLL computed by the most recent fade_step_update, in blob layout (fp32).
 * Complete only in contexts created with FADE_DEBUG_WU_GRAD=1 in the environment: normally the W_U gradients, and from
 * 2048 streams on the sums of the weight gradients that are formed in ranges of the batch, are consumed inside the kernel
 * that applies them and never reach memory (those ranges of the blob then hold zeros or an older step's values). */
int fade_debug_grad(fade_ctx *ctx, void *blob_host, size_t nbytes);

/* Per-kernel device time of the most recent fade_encode_device / fade_decode_device, measured with HIP
 * events on the context's stream when enabled by fade_profile(ctx, 1): names[i] / ms[i] / launches[i] for
 * i < returned count (at most cap). Profiling serialises launches and is off by default. */
int fade_profile(fade_ctx *ctx, int enable);
int fade_profile_read(fade_ctx *ctx, const char **names, double *ms, uint64_t *launches, int cap);

const char *fade_last_error(const fade_ctx *ctx);
void fade_destroy(fade_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif
