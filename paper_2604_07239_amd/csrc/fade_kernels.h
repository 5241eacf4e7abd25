// fade_kernels.h — host-side launchers of libfade's kernels (internal to the library).
#pragma once
#include "fade_dev.h"

enum {
  GEMM_CONV = 0, GEMM_GLOBAL, GEMM_ROUTER, GEMM_DOWN, GEMM_UP, GEMM_GATE, GEMM_FNR_IN, GEMM_FNR_OUT, GEMM_HEAD,
  GEMM_PARTIAL,  // bf16 only: split-K product leaving fp32 partials [splits][M][N]
  GEMM_OP_COUNT
};
// Launch one of the model step's products (see fade_gemm.hip). bf16 selects the MFMA path (activations
// bf16, W in fragment order) or the fp32 path (activations fp32, W plain [K][N]).
hipError_t fade_gemm(int op, bool bf16, const GemmArgs &g, hipStream_t s);

enum { CODE_NONE = 0, CODE_ENCODE = 1, CODE_DECODE = 2 };

// Per-stream coder state (structure of arrays, all of length B) and the payload buffers.
struct CoderBufs {
  uint32_t *low, *high, *pending, *bitbuf, *nbits, *pos;  // encoder (low/high shared with the decoder)
  uint32_t *value, *bitpos;                               // decoder
  uint8_t *out;            // [B][cap] payload bytes written by the encoder
  const uint8_t *in;       // [B][cap] payload bytes read by the decoder
  const uint32_t *in_len;  // [B]
  size_t cap;
  int *err;                // device flag: 1 payload overflow, 2 decoder left its interval, 3 non-finite probabilities
};

struct EmbedArgs {
  WinSrc ws;
  int T, D, Dh, Dc, c;
  const void *tabXe, *tabXl;  // [256][D] activation type
  const float *tabXe32;       // [256][D]
  const float *Wg, *Wv;       // [D][c]
  void *X, *XL;               // [B][Dh]
  void *M;                    // [B][Dc]
  float *GG, *GV;             // optional [B][c]: pre-activations of Eq. 1 for the backward pass
};

// arguments of the kernels that finish a split-K product with a folded LayerNorm (bf16 path)
struct CciArgs {
  int B, Dh, splits, stats_n;
  const float *part;     // [splits][B][64] partials of H_mix W'_down
  const float *stats;    // [B][stats_n][2] row sums of H_mix
  const float *s_fold, *t_fold;  // [64]
  const bf16_t *WU;      // [B][64][64]
  float *y;              // [B][64] Down(LN(H_mix))
  bf16_t *z;             // [B][64] y W_U
};
struct GegluArgs {
  int B, Dh, De, splits, stats_n;
  const float *part;     // [splits][B][2 De] partials, gate | value interleaved per 128 columns
  const float *stats;    // row sums of H_coarse
  const float *s_fold, *t_fold;  // [2 De] in the same interleaved order
  bf16_t *Hexp;          // [B][De]
  bf16_t *eg, *ev;       // optional [B][De]: pre-activations for the backward pass
};
struct HoutArgs {
  int B, Dh, stats_n;
  const bf16_t *V, *Hc;
  const float *stats, *gamma, *beta, *lam;
  bf16_t *Hout;
};

struct SqcArgs {
  WinSrc ws;
  int B;
  int splits;           // 0: logits are final; > 0: [splits][B][256] partials to be summed, plus bias
  const float *bias;    // [256] when splits > 0
  float *logits_out;    // optional [B][256]: the reduced logits
  const float *logits;  // [B][256] or [splits][B][256]
  float *probs;         // optional [B][256]
  uint16_t *freq;       // optional [B][256]
  uint8_t *sym_base;    // symbol of stream b at step i lives at sym_base + b * ws.stride + i
  CoderBufs cb;
};

hipError_t fade_preshuffle(const float *W0, const float *W1, int k_real, int K, int N, int interleave, const float *rowscale, void *out,
                           hipStream_t s);
hipError_t fade_fold_vectors(const float *W0, const float *W1, int K, int N, int interleave, const float *gamma, const float *beta,
                             float *s_out, float *t_out, hipStream_t s);
hipError_t fade_cci(const CciArgs &a, hipStream_t s);
hipError_t fade_geglu(const GegluArgs &a, hipStream_t s);
hipError_t fade_hout(const HoutArgs &a, hipStream_t s);
hipError_t fade_virtual_copy(const float *W0, const float *W1, int k_real, int K, int N, int interleave, float *out, hipStream_t s);
hipError_t fade_convert(const float *src, void *dst, size_t n, bool bf16, hipStream_t s);
hipError_t fade_round_bf16(const float *src, float *dst, size_t n, hipStream_t s);
hipError_t fade_tables(const float *E, const float *ge, const float *be, const float *gl, const float *bl, int D, void *tabXe,
                       void *tabXl, float *tabXe32, bool bf16, hipStream_t s);
hipError_t fade_embed_cache(const EmbedArgs &a, int B, bool bf16, hipStream_t s);
hipError_t fade_bmm(const float *y, const void *WU, void *z, int B, bool bf16, hipStream_t s);
hipError_t fade_softmax_quant_code(const SqcArgs &a, int mode, hipStream_t s);
hipError_t fade_quantize_rows(const float *probs, size_t rows, uint16_t *freq, int *err, hipStream_t s);
hipError_t fade_code_tables(const uint16_t *freq, uint8_t *sym, int n_streams, const CoderBufs &cb, int mode, hipStream_t s);
hipError_t fade_code_uniform(const WinSrc &ws, uint8_t *sym_base, int B, const CoderBufs &cb, int mode, hipStream_t s);
hipError_t fade_coder_init(const CoderBufs &cb, int B, int decode, hipStream_t s);
hipError_t fade_coder_finish(const CoderBufs &cb, int B, long long stride, long long n, hipStream_t s);
hipError_t fade_payload_move(uint8_t *strided, size_t cap, uint8_t *flat, const unsigned long long *offsets, const uint32_t *lens, int B,
                             int gather, hipStream_t s);
