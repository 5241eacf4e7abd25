// fade_kernels.h — host-side launchers of libfade's kernels (internal to the library).
#pragma once
#include "fade_dev.h"

enum {
  GEMM_CONV = 0, GEMM_GLOBAL, GEMM_ROUTER, GEMM_DOWN, GEMM_UP, GEMM_GATE, GEMM_FNR_IN, GEMM_FNR_OUT, GEMM_HEAD,
  GEMM_PARTIAL,  // product leaving fp32 partials [splits][M][N] (fp32 path: one split)
  GEMM_X_STORE,  // backward: dX = dY W^T, stored as activations
  GEMM_W,        // backward: dW = L^T R, reduction over the batch, fp32 gradient out
  GEMM_W_TN,     // the same from row-major operands (bf16 path): A = L [a_rows][lda], W = R [K][ldb], K = padded batch
  GEMM_CONVT,    // backward of Eq. 4 w.r.t. its input
  GEMM_HEAD_PLAIN,  // fp32 path, ablation levels below 5: logits = A W_o + b_o on the stage the head reads (no Eq. 10 tail)
  GEMM_OP_COUNT
};
// Launch one of the model step's products (see fade_gemm.hip). bf16 selects the MFMA path (activations
// bf16, W in fragment order) or the fp32 path (activations fp32, W plain [K][N]).
hipError_t fade_gemm(int op, bool bf16, const GemmArgs &g, hipStream_t s);
bool fade_gemm_tn2_ok(int M, int N, int K);  // dW[M][N] over a batch of K rows runs on 256 x 256 tiles as a launch of its own
int fade_gemm_tn_tiles(int M, int N);  // workgroups per batch range of a grouped weight-gradient product dW[M][N]; 0: shape not supported
hipError_t fade_gemm_group_add(GemmGroup &gg, int op, const GemmArgs &g);
hipError_t fade_gemm_group_launch(const GemmGroup &gg, hipStream_t s);
hipError_t fade_gemm_tn2_group_add(Tn2Group &tg, const GemmArgs &g);  // g as for GEMM_W_TN with fade_gemm_tn2_ok(g.M, g.N, g.K)
hipError_t fade_gemm_tn2_group_launch(const Tn2Group &tg, hipStream_t s);

enum { CODE_NONE = 0, CODE_ENCODE = 1, CODE_DECODE = 2, CODE_RANGES = 3 };  // CODE_RANGES: leave each row's coding interval for a later pass

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
  const void *slot_tab;       // optional [256][c] activation type: Eq. 1's slot of every symbol (frozen weights only)
  const float *gg_tab, *gv_tab;  // optional [256][c]: Eq. 1's two pre-activations of every symbol (adapting weights)
  int B, S;                   // several steps per launch (slot_tab required): row s * B + b is stream b at step ws.i + s
  // Eq. 4 in the same launch (bf16, D = 32; conv_W == NULL: a separate product does it): W_conv as MFMA fragments
  // [K_c / 16][64][8], bias [D], outputs H_local [rows][T][D] and, optionally, the pre-activations for the backward pass.
  // XL may then be NULL when nothing else reads it.
  const void *conv_W;
  const float *conv_b;
  void *Hl, *cv;
  int taps, Kc;
};

// arguments of the kernels that finish a split-K product with a folded LayerNorm (bf16 path)
struct CciArgs {
  int B, Dh, splits, stats_n;
  int streams;           // row r uses W_U[r % streams] (rows beyond the first `streams` are later steps of the same streams)
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
  const void *V, *Hc;
  const float *stats, *gamma, *beta, *lam;
  void *Hout;
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
  int streams;          // CODE_RANGES: B = streams * steps rows, row s * streams + b is stream b at step ws.i + s
  uint2 *ranges;        // CODE_RANGES: [B] (cum, cum + freq) of the symbol each row has to code
};

hipError_t fade_preshuffle(const float *W0, const float *W1, int k_real, int K, int N, int interleave, const float *rowscale, void *out,
                           hipStream_t s);
// fragments of the TRANSPOSE of the (possibly interleaved) matrix [K][N]: the result multiplies from the right as [N][K]
hipError_t fade_preshuffle_t(const float *W0, const float *W1, int K, int N, int interleave, void *out, hipStream_t s);
// weight preparation in one launch: every descriptor is an element-wise map master -> compute copy
enum { PREP_FRAG = 0, PREP_FRAG_T = 1, PREP_ROUND = 2, PREP_FRAG_CONVT = 3 };
struct PrepDesc {
  int kind;
  const float *W0, *W1;   // source(s) in the fp32 blob
  int k_real, K, N;       // PREP_FRAG: virtual [K][N] with rows >= k_real zero; PREP_FRAG_T: source [K][N], result for [N][K]; PREP_ROUND: N values
  int interleave;         // gate | value interleave per 128 columns over the pair (W0, W1)
  const float *rowscale;  // PREP_FRAG: folded LayerNorm gain or NULL
  void *out;
  int taps, D;            // PREP_FRAG_CONVT: W0 = W_conv [taps][D][D]; virtual [K][D] with row (r*D+o), column i = W_conv[r][i][o]
};
// the per-symbol tables in the same launch (has_tables): they read the master embedding and round it themselves
struct TablesArgs {
  const float *E, *ge, *be, *gl, *bl;
  int D, round_bf16;       // round_bf16: E counts as its bf16 rounding (what the bf16 path's embedding copy holds)
  void *tabXe, *tabXl;     // bf16
  float *tabXe32, *tabXhat, *tabRstd;
  // optional, same launch: Eq. 1 per symbol from the masters W_g, W_v [D][c] (rounded to bf16 as their compute copies are):
  // slot_tab [256][c] bf16 entries (frozen weights) and / or gg_tab, gv_tab [256][c] fp32 pre-activations (adapting weights)
  const float *Wg, *Wv;
  int c;
  void *slot_tab;
  float *gg_tab, *gv_tab;
};
struct PrepBatch {
  PrepDesc d[20];
  int count;
  int has_tables;
  TablesArgs tab;
};
hipError_t fade_prep_batch(const PrepBatch &pb, hipStream_t s);
hipError_t fade_convt_build(const float *Wconv, int taps, int D, int Kc, float *V, hipStream_t s);
hipError_t fade_cci(const CciArgs &a, hipStream_t s);
hipError_t fade_residual_add(const void *x, const void *y, const float *lam, void *out, size_t n, bool bf16, hipStream_t s);  // out = x + lam[0] * y
hipError_t fade_geglu(const GegluArgs &a, hipStream_t s);
hipError_t fade_hout(const HoutArgs &a, bool bf16, hipStream_t s);
hipError_t fade_virtual_copy(const float *W0, const float *W1, int k_real, int K, int N, int interleave, float *out, hipStream_t s);
hipError_t fade_convert(const float *src, void *dst, size_t n, bool bf16, hipStream_t s);
hipError_t fade_round_bf16(const float *src, float *dst, size_t n, hipStream_t s);
hipError_t fade_tables(const float *E, const float *ge, const float *be, const float *gl, const float *bl, int D, void *tabXe,
                       void *tabXl, float *tabXe32, float *tabXhat, float *tabRstd, bool bf16, hipStream_t s);
hipError_t fade_embed_cache(const EmbedArgs &a, int B, bool bf16, hipStream_t s);
hipError_t fade_embed_steps(const EmbedArgs &a, hipStream_t s);  // bf16, a.B * a.S rows, cache rebuilt from the window
hipError_t fade_encode_ranges(const WinSrc &ws, const uint2 *ranges, int B, int S, const CoderBufs &cb, hipStream_t s);
hipError_t fade_bmm(const float *y, const void *WU, void *z, int B, bool bf16, hipStream_t s);
hipError_t fade_softmax_quant_code(const SqcArgs &a, int mode, hipStream_t s);
hipError_t fade_quantize_rows(const float *probs, size_t rows, uint16_t *freq, int *err, hipStream_t s);
hipError_t fade_code_tables(const uint16_t *freq, uint8_t *sym, int n_streams, const CoderBufs &cb, int mode, hipStream_t s);
hipError_t fade_code_uniform(const WinSrc &ws, uint8_t *sym_base, int B, const CoderBufs &cb, int mode, hipStream_t s);
hipError_t fade_coder_init(const CoderBufs &cb, int B, int decode, hipStream_t s);
hipError_t fade_fill_u32(uint32_t *dst, uint32_t value, size_t n, hipStream_t s);  // a fill as a kernel (safe to capture in a graph, unlike a memset node)
hipError_t fade_coder_finish(const CoderBufs &cb, int B, long long stride, long long n, hipStream_t s);
hipError_t fade_payload_move(uint8_t *strided, size_t cap, uint8_t *flat, const unsigned long long *offsets, const uint32_t *lens, int B,
                             int gather, hipStream_t s);

// ---------------------------------------------------------------------------------------------------
// online update (fade_bwd.hip)
// ---------------------------------------------------------------------------------------------------
struct UpdateState {
  int na;         // active streams of this step
  int t;          // Adam step count
  float c1, c2;   // 1 - beta^t
  float inv_na;
};
struct TransposeArgs {
  const void *src; int ld;     // [B][ld]
  void *dst; int Bp;           // [N][Bp]
  int B;
  const float *stats; int stats_n, width;  // optional LayerNorm on the way (stats == NULL: plain copy)
  const float *gamma, *beta;
};
// u = LN(h) written out row-major (the forward pass folds these LayerNorms into the following product and never stores u;
// the weight gradients of Eq. 7's Down and Eq. 9's pair need it as their left operand)
struct LnApplyArgs { const void *src; void *dst; const float *stats, *gamma, *beta; };
// The loss gradient (fade_loss_grad's work) can ride in the same launch: it needs nothing the copies produce.
struct LossGradArgs {
  WinSrc ws;
  const uint8_t *targets; long long tstride;
  const float *probs;
  UpdateState *u;
  float beta1, beta2;
  void *dl;
  float *col_part;
};
struct LnApplyBatch { LnApplyArgs a[2]; int count, B, Dh, stats_n; int with_loss; LossGradArgs loss; };
hipError_t fade_ln_apply(const LnApplyBatch &lb, bool bf16, hipStream_t s);
// several transposes in one launch (blockIdx.z picks one)
struct TransposeBatch {
  TransposeArgs t[8];
  int N[8];
  int count;
};
struct BwdOutArgs {
  int B, Dh, stats_n;
  int groups;  // row groups per workgroup (set by the launcher)
  float *ln_part;  // [blocks][2][Dh] partial sums of d gamma, d beta over this workgroup's rows
  const void *dH, *V, *Hc;
  const float *stats, *gamma, *beta, *lam;
  void *dV, *dHc;
  float *row_dlam;
};
struct BwdGateArgs {
  int B, Dh, stats_n;
  int groups;  // row groups per workgroup (set by the launcher)
  float *ln_part;
  const void *du, *Hc, *dHc, *sg, *Ha, *Hmix;
  const float *stats, *gamma, *lam;
  void *dHa, *dac, *dHmix;
  float *row_dlam;
  const float *du_part;  // instead of du: split-K partials [du_splits][B][Dh] of the product that forms it, added here in range order
  int du_splits;
};
struct BwdMixArgs {
  int B, Dh, stats_n;
  int groups;  // row groups per workgroup (set by the launcher)
  float *ln_part;
  const void *dnc, *Hmix, *dHmix1, *dHmix2, *alpha, *hm, *cv, *X;  // hm, cv: pre-activations of the global / local stream
  const float *stats, *gamma, *lam;
  void *dar, *dhm, *dcv, *dX;
  float *row_dlam;
};
struct BwdCciArgs {
  int B, splits;
  const float *dz_part;   // [splits][B][64]
  const float *y;         // [B][64]
  void *WU_c;             // [B][64][64] compute copy (read, then rewritten by Adam)
  float *master, *m, *v;  // W_U's slice of the fp32 blob and of the two moment blobs
  float *dy; void *dy_at; // [B][64]
  const UpdateState *u;
  float lr, beta1, beta2, eps;
  float *g_dbg;           // optional [B][64][64]: the gradient y dz^T written out (debug: it is otherwise consumed in registers)
};
struct BwdSlotArgs {
  WinSrc ws;
  int B, T;
  int Dh, Dc, c, D, round_bf16;
  const void *dhm;        // [B][Dh]
  const void *dg;         // optional [B][c] (activation type): d(hm) W_m[Dc-c..Dc)^T already formed by a product; else
                          // the kernel forms it from Wm itself
  const float *Wm;        // fp32 master W_m [Dc][Dh]
  const float *GG, *GV;   // [B][c]
  const float *Wg, *Wv;   // [D][c] compute values
  float *dgg, *dgv;       // [B][c]
  float *dxt;             // [B][D]
  const float *tabXe32;   // [256][D] normalised embedding rows (x_t of the newest symbol)
  float *part;            // [ceil(B / 4)][2][D][c] first stage of dW_g, dW_v
};
struct ConvGradArgs {
  int B, T, D, taps;
  const void *XL, *dcv;   // [B*T][D]
  float *part;            // [ceil(B*T/128)][taps*D + 1][D]
  // bf16, D = 32 only: Eq. 4 backward w.r.t. its input in the same launch (WT == NULL: a separate product does it).
  // WT: fragments of the virtual [Kc][D] matrix with row (r * D + o), column i = W_conv[r][i][o]; dxl [B*T][D].
  const void *WT;
  void *dxl;
  int Kc;
};
struct BwdTokenArgs {
  WinSrc ws;
  int B, T, D;
  const void *dX1, *dX2, *dxl;   // [B*T][D]
  const float *dxt;               // [B][D], added at the newest token
  const float *tabXhat, *tabRstd; // [256][D], [256]
  const float *gamma_e, *gamma_l;
  float *part;                    // [blocks][2][256][D] per-symbol partial sums
};

hipError_t fade_transpose(const TransposeArgs &a, int N, bool bf16, hipStream_t s);
hipError_t fade_transpose_batch(const TransposeBatch &tb, bool bf16, hipStream_t s);
hipError_t fade_embed_t(const WinSrc &ws, int B, int Bp, int T, int D, const void *tab, void *XT, bool bf16, hipStream_t s);
hipError_t fade_bwd_out(const BwdOutArgs &a, bool bf16, hipStream_t s);
hipError_t fade_bwd_geglu(int B, int De, const void *dHexp, const void *eg, const void *ev, void *dE, bool bf16, hipStream_t s);
hipError_t fade_bwd_gate(const BwdGateArgs &a, bool bf16, hipStream_t s);
hipError_t fade_bwd_mix(const BwdMixArgs &a, bool bf16, hipStream_t s);
int fade_rows_per_block(int B);  // rows per workgroup of the backward row kernels at batch size B
// Second stages (out[n] = sum over p < P of part[p][n], rows added in a fixed order) that nothing inside the backward pass
// waits for are queued here and run as ONE launch just before Adam. The stage-1 launchers below take the queue.
// Adam's hyper-parameters and state arrays (device layout; gradient, master weights and both moments share the offsets)
struct AdamArrays {
  const float *grad_base;  // gradients in blob order (the Adam pass over the matrices stores sums of partial gradients here: see AdamMat)
  float *master, *m, *v;
  const UpdateState *u;
  float lr, beta1, beta2, eps;
};
struct ReduceBatch {
  int count;
  int adam[16];          // item's output is a parameter gradient: apply Adam to the parameter right after the sum
  AdamArrays opt;        // used when any adam[] is set
  int P[16], N[16];
  const float *part[16];
  float *out[16];
  bool push(int p, int n, const float *src, float *dst) {
    if (count >= 16) return false;
    P[count] = p; N[count] = n; part[count] = src; out[count] = dst; adam[count] = 1; ++count;
    return true;
  }
  bool push_plain(int p, int n, const float *src, float *dst) {  // a sum that is not a parameter gradient
    if (!push(p, n, src, dst)) return false;
    adam[count - 1] = 0;
    return true;
  }
};
hipError_t fade_reduce_batch(const ReduceBatch &rb, hipStream_t s);
hipError_t fade_loss_grad(const WinSrc &ws, const uint8_t *targets, long long tstride, int B, const float *probs, UpdateState *u, float beta1,
                          float beta2, void *dl, float *col_part, float *dbo, bool bf16, ReduceBatch &rb, hipStream_t s);
// Adam on a [K][N] matrix of the blob in 64 x 64 blocks, writing the refreshed bf16 operand copies in the same pass: the
// forward fragments (optionally with a LayerNorm gain folded in, plus the partial column sums of its fix-up vectors) and the
// fragments of the transpose. A matrix may be one half of the interleaved GeGLU pair (virtual column mapping).
struct AdamMat {
  unsigned long long off;  // offset in the blob
  int K, N;
  int vcol0, vstride, VN;  // virtual column of column n: (n / 64) * vstride + (n % 64) + vcol0; VN = width of the virtual matrix
  void *frag, *fragT;      // may be NULL
  const float *gamma, *beta;
  float *fold_part;        // [K / 64][2][VN] when gamma is set
  int first_block;
  // gradient left as gsplits partial sums [gsplits][K][N] over ranges of the batch (NULL: complete in the gradient array);
  // the Adam pass adds them in range order and stores the sum in the gradient array
  const float *gpart;
  int gsplits;
};
struct AdamRefreshBatch {
  int count, total_blocks;
  int refresh_only;        // no Adam step: rebuild the copies from the master weights as they are (load / reset)
  int keep_sum;            // a gradient that arrives as slices over ranges of the batch: also store the sum in the gradient array (debug contexts)
  AdamMat m[10];
  AdamArrays opt;
};
hipError_t fade_adam_refresh(const AdamRefreshBatch &ab, hipStream_t s);
hipError_t fade_bwd_cci(const BwdCciArgs &a, bool bf16, hipStream_t s);
hipError_t fade_bwd_slot(const BwdSlotArgs &a, float *dWgv, bool bf16, ReduceBatch &rb, hipStream_t s);
hipError_t fade_bwd_slot_conv(const BwdSlotArgs &sa, float *dWgv, const ConvGradArgs &ca, float *dWb, ReduceBatch &rb, hipStream_t s);
hipError_t fade_conv_grad(const ConvGradArgs &a, float *dWb, bool bf16, ReduceBatch &rb, hipStream_t s);
hipError_t fade_bwd_embed(const BwdTokenArgs &a, int nblocks, float *contrib, float *dE, float *dparams, bool bf16, ReduceBatch &rb,
                          hipStream_t s);
