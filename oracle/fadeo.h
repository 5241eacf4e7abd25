/*
 * fadeo.h — C ABI of the CPU oracle for FADE's batched probability step and coder.
 *
 * TEST INFRASTRUCTURE ONLY. This library is a plain, slow, single-threaded restatement of what the
 * method computes, written from the paper (Method section, Eq. 1-10; Algorithm 1 of the appendix).
 * It shares no source with the HIP library and must never be on a product code path: only tests,
 * the smoke check and the bench's cpu_baseline leg may load it.
 *
 * Numerics: weights are held as fp32 (for the bf16 configuration: rounded to bf16, then widened);
 * every activation and every accumulation is fp64; psi is the exact erf GeLU; LayerNorm uses the
 * biased variance and eps = 1e-5; the softmax output is rounded once to fp32 before quantisation.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py (closed forms, invariants,
 * special cases, finite differences, brute force); compression ratio against the paper's tables is
 * "parity unpinned" (its datasets are not available).
 */
#ifndef FADEO_H
#define FADEO_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct fadeo_ctx fadeo_ctx;

enum { FADEO_F32 = 0, FADEO_BF16 = 1 };
enum { FADEO_FROZEN = 0, FADEO_ONLINE_ADAM = 1 };

/* Same field order as the product library's config: the harness fills one and hands it to both. */
typedef struct {
  uint32_t struct_size, abi_version;
  uint32_t B, T, D, H;     /* streams, context window, embedding dim, hidden width (D_cache = D_e = H unless given below) */
  uint32_t d_low;          /* d_h of Eq. 7; 0 => 64 */
  uint32_t cache_chunk;    /* c: width of one rolling-cache slot; 0 => D_cache / T */
  uint32_t conv_k;         /* taps of the causal Conv1d of Eq. 4; 0 => 3 */
  uint32_t d_cache;        /* D_cache (rolling cache width, Eq. 2-3); 0 => H */
  uint32_t d_e;            /* D_e (expansion width of Eq. 9-10); 0 => H */
  uint32_t ablation;       /* 0 or 5: full model; 1: head on H_global; 2: on H_mix; 3: on H_a + lambda_c H_mix; 4: on H_coarse
                            * (frozen weights only) */
  uint32_t dtype;          /* FADEO_F32 | FADEO_BF16 */
  uint32_t update_mode;    /* FADEO_FROZEN | FADEO_ONLINE_ADAM */
  float lr, beta1, beta2, eps; /* 0 => 1e-3, 0.9, 0.999, 1e-8 */
  int32_t device;          /* ignored */
  void *hip_stream;        /* ignored */
} fadeo_config;

enum {
  FADEO_OK = 0, FADEO_E_INVALID_ARG = -1, FADEO_E_BAD_CONFIG = -2, FADEO_E_NO_WEIGHTS = -3,
  FADEO_E_WEIGHTS_MISMATCH = -4, FADEO_E_BUFFER_TOO_SMALL = -5, FADEO_E_CORRUPT_STREAM = -6,
  FADEO_E_NUMERIC = -9
};

/* Intermediate activations of the most recent model step, per stream (fp64). */
enum {
  FADEO_TAP_X = 0, FADEO_TAP_CACHE, FADEO_TAP_H_GLOBAL, FADEO_TAP_H_LOCAL, FADEO_TAP_ALPHA,
  FADEO_TAP_H_MIX, FADEO_TAP_Y_DOWN, FADEO_TAP_Z_BMM, FADEO_TAP_H_A, FADEO_TAP_H_COARSE,
  FADEO_TAP_H_EXPAND, FADEO_TAP_H_OUT, FADEO_TAP_LOGITS, FADEO_TAP_PROBS, FADEO_TAP_COUNT
};

size_t fadeo_weights_nbytes(const fadeo_config *cfg);
int  fadeo_create(const fadeo_config *cfg, fadeo_ctx **out);
int  fadeo_load_weights(fadeo_ctx *, const void *blob, size_t nbytes);
int  fadeo_reset(fadeo_ctx *);
/* One model step (Eq. 1-10 + head + softmax + quantiser) for B streams; advances the rolling cache of
 * every active stream. windows: [B][T] bytes, oldest first. freq: [B][256] or NULL; probs: [B][256] or NULL. */
int  fadeo_step_probs(fadeo_ctx *, const uint8_t *windows, const uint8_t *active, uint16_t *freq, float *probs);
/* Mean NLL (nats, fp64) of targets under the probabilities of the last step. */
int  fadeo_loss(fadeo_ctx *, const uint8_t *targets, const uint8_t *active, double *loss);
/* Gradient of that mean NLL w.r.t. every parameter, laid out like the weight blob (fp64). No update. */
int  fadeo_backward(fadeo_ctx *, const uint8_t *targets, const uint8_t *active, double *grad_blob);
/* backward + one Adam step (only in FADEO_ONLINE_ADAM). */
int  fadeo_step_update(fadeo_ctx *, const uint8_t *targets, const uint8_t *active);
/* Current master weights (fp32 blob layout). */
int  fadeo_get_weights(fadeo_ctx *, float *blob, size_t nbytes);
size_t fadeo_tap(fadeo_ctx *, int which, uint32_t stream, double *out, size_t cap);

size_t fadeo_encode_bound(const fadeo_ctx *, size_t n);
int  fadeo_encode(fadeo_ctx *, const uint8_t *src, size_t n, uint8_t *dst, size_t dst_cap, size_t *dst_len);
int  fadeo_decode(fadeo_ctx *, const uint8_t *src, size_t src_len, uint8_t *dst, size_t dst_cap, size_t *dst_len);
/* Sum over coded symbols of -log2(f[x]/65536) and of -log2(p[x]) during the last encode (bits). */
int  fadeo_last_code_stats(fadeo_ctx *, double *bits_from_freq, double *bits_from_probs, uint64_t *model_steps);

/* Stand-alone pieces (no context). */
int  fadeo_quantize(const float *p /*[rows][256]*/, size_t rows, uint16_t *freq /*[rows][256]*/);
/* Code `n` symbols of ONE stream, symbol i under table freq[i][256] (each summing to 65536). */
int  fadeo_coder_encode(const uint16_t *freq, const uint8_t *sym, size_t n, uint8_t *out, size_t cap, size_t *len);
int  fadeo_coder_decode(const uint16_t *freq, size_t n, const uint8_t *in, size_t in_len, uint8_t *sym);
uint64_t fadeo_fnv1a64(const void *p, size_t n);
/* Test hook: overwrite one stream's rolling cache (Dc values). */
int  fadeo_test_set_cache(fadeo_ctx *, uint32_t stream, const double *m, size_t n);
const char *fadeo_last_error(const fadeo_ctx *);
void fadeo_destroy(fadeo_ctx *);

#ifdef __cplusplus
}
#endif
#endif
