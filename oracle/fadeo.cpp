/*
 * fadeo.cpp — CPU oracle for FADE's batched probability step, quantiser, arithmetic coder and online
 * update. TEST INFRASTRUCTURE ONLY (see fadeo.h): plain loops, single thread, fp64 arithmetic, no
 * blocking or fusion, so that each function can be checked against the paper by eye.
 *
 * Paper passages restated here:
 *   - embedding X_emb, flattened normalised input X, D_h = T*D      : "Dual-Stream Multi-Scale Decoupler", Design
 *   - GeGLU of the newest symbol and the rolling cache               : Eq. 1, Eq. 2
 *   - global projection with learnable residual scale lambda_m       : Eq. 3
 *   - local stream Flatten(psi(Conv(LN(X_emb))))                     : Eq. 4
 *   - content-adaptive router and the mix                            : Eq. 5, Eq. 6
 *   - coarse channel interaction Up(BMM(Down(LN(.)), W_U))           : Eq. 7
 *   - self gate with lambda_c residual                               : Eq. 8
 *   - fine refinement: GeGLU(LN(.)), W_f, LN, psi, lambda_o residual : Eq. 9, Eq. 10
 *   - uniform coding of the first T symbols, predict/code/update loop: Algorithm 1 (appendix)
 *   - NLL loss                                                       : Eq. 12 (ablation section)
 * Where the paper is silent (output head, quantiser, coder details, optimiser, conv hyper-parameters,
 * cache slot width) the readings are the fixed rules documented next to each function below.
 */
#include "fadeo.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

namespace {

typedef std::vector<double> dvec;

// ----------------------------------------------------------------------------------------------
// scalar functions
// ----------------------------------------------------------------------------------------------
const double kInvSqrt2 = 0.70710678118654752440;
const double kInvSqrt2Pi = 0.39894228040143267794;

// psi: exact GeLU, x * Phi(x) (Eq. 1 names psi as the GeLU).
double gelu(double x) { return 0.5 * x * (1.0 + std::erf(x * kInvSqrt2)); }
double gelu_grad(double x) {
  return 0.5 * (1.0 + std::erf(x * kInvSqrt2)) + x * kInvSqrt2Pi * std::exp(-0.5 * x * x);
}
double sigmoid(double x) { return 1.0 / (1.0 + std::exp(-x)); }

// round-to-nearest-even fp32 -> bf16 -> fp32 (weights of the bf16 configuration).
float bf16_round(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return f;  // inf / nan unchanged
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  float r;
  std::memcpy(&r, &u, 4);
  return r;
}

// ----------------------------------------------------------------------------------------------
// parameter blob layout (canonical order; every matrix is [in][out], row-major, so y = x * W)
// ----------------------------------------------------------------------------------------------
enum ParamId {
  P_E, P_GAMMA_E, P_BETA_E, P_GAMMA_L, P_BETA_L, P_WG, P_WV, P_WM, P_LAMBDA_M, P_WCONV, P_BCONV,
  P_WR, P_GAMMA_C, P_BETA_C, P_WDOWN, P_WU, P_WUP, P_WC, P_LAMBDA_C, P_GAMMA_F, P_BETA_F, P_WFG,
  P_WFV, P_WF, P_GAMMA_O, P_BETA_O, P_LAMBDA_O, P_WO, P_BO, P_COUNT
};

struct Dims {
  size_t B, T, D, H, Dh, Dc, De, dl, c, k;
};

struct Layout {
  size_t off[P_COUNT + 1];
  bool is_matrix[P_COUNT];  // rounded to bf16 in the bf16 configuration
};

Layout make_layout(const Dims &d) {
  Layout L;
  size_t n[P_COUNT];
  bool m[P_COUNT];
  for (int i = 0; i < P_COUNT; ++i) m[i] = false;
  n[P_E] = 256 * d.D;            m[P_E] = true;
  n[P_GAMMA_E] = d.D;  n[P_BETA_E] = d.D;  n[P_GAMMA_L] = d.D;  n[P_BETA_L] = d.D;
  n[P_WG] = d.D * d.c;           m[P_WG] = true;
  n[P_WV] = d.D * d.c;           m[P_WV] = true;
  n[P_WM] = d.Dc * d.Dh;         m[P_WM] = true;
  n[P_LAMBDA_M] = 1;
  n[P_WCONV] = d.k * d.D * d.D;  m[P_WCONV] = true;
  n[P_BCONV] = d.D;
  n[P_WR] = d.Dh * d.Dh;         m[P_WR] = true;
  n[P_GAMMA_C] = d.Dh; n[P_BETA_C] = d.Dh;
  n[P_WDOWN] = d.Dh * d.dl;      m[P_WDOWN] = true;
  n[P_WU] = d.B * d.dl * d.dl;   m[P_WU] = true;
  n[P_WUP] = d.dl * d.Dh;        m[P_WUP] = true;
  n[P_WC] = d.Dh * d.Dh;         m[P_WC] = true;
  n[P_LAMBDA_C] = 1;
  n[P_GAMMA_F] = d.Dh; n[P_BETA_F] = d.Dh;
  n[P_WFG] = d.Dh * d.De;        m[P_WFG] = true;
  n[P_WFV] = d.Dh * d.De;        m[P_WFV] = true;
  n[P_WF] = d.De * d.Dh;         m[P_WF] = true;
  n[P_GAMMA_O] = d.Dh; n[P_BETA_O] = d.Dh;
  n[P_LAMBDA_O] = 1;
  n[P_WO] = d.Dh * 256;          m[P_WO] = true;
  n[P_BO] = 256;
  size_t o = 0;
  for (int i = 0; i < P_COUNT; ++i) { L.off[i] = o; o += n[i]; L.is_matrix[i] = m[i]; }
  L.off[P_COUNT] = o;
  return L;
}

// ----------------------------------------------------------------------------------------------
// small dense helpers (definitions written out)
// ----------------------------------------------------------------------------------------------
// y[n] = sum_k x[k] * W[k][n]   (W is [K][N] row-major, fp32 values, fp64 accumulation in k order)
void vec_mat(const double *x, const float *W, size_t K, size_t N, double *y) {
  for (size_t n = 0; n < N; ++n) y[n] = 0.0;
  for (size_t k = 0; k < K; ++k) {
    const double xk = x[k];
    const float *w = W + k * N;
    for (size_t n = 0; n < N; ++n) y[n] += xk * (double)w[n];
  }
}
// dx[k] = sum_n W[k][n] * dy[n]
void mat_vec_t(const float *W, const double *dy, size_t K, size_t N, double *dx) {
  for (size_t k = 0; k < K; ++k) {
    const float *w = W + k * N;
    double a = 0.0;
    for (size_t n = 0; n < N; ++n) a += (double)w[n] * dy[n];
    dx[k] = a;
  }
}
// dW[k][n] += x[k] * dy[n]
void outer_acc(const double *x, const double *dy, size_t K, size_t N, double *dW) {
  for (size_t k = 0; k < K; ++k) {
    const double xk = x[k];
    double *w = dW + k * N;
    for (size_t n = 0; n < N; ++n) w[n] += xk * dy[n];
  }
}

const double kLnEps = 1e-5;

// LayerNorm over n values: xhat = (x - mean) / sqrt(biased var + eps); y = xhat * gamma + beta.
void layer_norm(const double *x, size_t n, const float *gamma, const float *beta, double *y, double *xhat,
                double *rstd_out) {
  double mean = 0.0;
  for (size_t i = 0; i < n; ++i) mean += x[i];
  mean /= (double)n;
  double var = 0.0;
  for (size_t i = 0; i < n; ++i) var += (x[i] - mean) * (x[i] - mean);
  var /= (double)n;
  const double rstd = 1.0 / std::sqrt(var + kLnEps);
  for (size_t i = 0; i < n; ++i) {
    const double h = (x[i] - mean) * rstd;
    if (xhat) xhat[i] = h;
    y[i] = h * (double)gamma[i] + (double)beta[i];
  }
  if (rstd_out) *rstd_out = rstd;
}
// Backward of layer_norm: accumulates dgamma, dbeta; adds into dx.
void layer_norm_bwd(const double *dy, const double *xhat, double rstd, size_t n, const float *gamma,
                    double *dgamma, double *dbeta, double *dx_acc) {
  double m1 = 0.0, m2 = 0.0;
  for (size_t i = 0; i < n; ++i) {
    const double dh = dy[i] * (double)gamma[i];
    m1 += dh;
    m2 += dh * xhat[i];
    dgamma[i] += dy[i] * xhat[i];
    dbeta[i] += dy[i];
  }
  m1 /= (double)n;
  m2 /= (double)n;
  for (size_t i = 0; i < n; ++i) {
    const double dh = dy[i] * (double)gamma[i];
    dx_acc[i] += rstd * (dh - m1 - xhat[i] * m2);
  }
}

// ----------------------------------------------------------------------------------------------
// quantiser: probabilities -> integer frequencies summing to 2^16, every entry >= 1.
// Rule (the paper does not give one): f_i = 1 + trunc(p_i * 65280) with the product formed as ONE
// fp32 round-to-nearest multiplication; the remainder 65536 - sum(f) is added to the lowest index
// holding the maximum f. An exact integer function of the fp32 vector p.
// ----------------------------------------------------------------------------------------------
int quantize_row(const float *p, uint16_t *f) {
  uint32_t q[256];
  int64_t sum = 0;
  for (int i = 0; i < 256; ++i) {
    if (!(p[i] >= 0.0f) || !(p[i] <= 1.0f)) return FADEO_E_NUMERIC;  // also rejects NaN
    volatile float prod = p[i] * 65280.0f;  // volatile: one rounded fp32 product, no contraction
    q[i] = 1u + (uint32_t)prod;
    sum += q[i];
  }
  int m = 0;
  for (int i = 1; i < 256; ++i)
    if (q[i] > q[m]) m = i;
  int64_t fm = (int64_t)q[m] + (65536 - sum);
  if (fm < 1 || fm > 65535) return FADEO_E_NUMERIC;
  q[m] = (uint32_t)fm;
  for (int i = 0; i < 256; ++i) f[i] = (uint16_t)q[i];
  return FADEO_OK;
}

// ----------------------------------------------------------------------------------------------
// arithmetic coder (the paper cites Witten, Neal & Cleary 1987 and gives no parameters).
// Fixed rule: 32-bit interval [low, high], totals 2^16, bit-plus-follow carry handling, bits packed
// MSB first. One independent coder per stream.
// ----------------------------------------------------------------------------------------------
const uint32_t kHalf = 0x80000000u, kQuarter = 0x40000000u, kThreeQ = 0xC0000000u;

struct BitSink {
  std::vector<uint8_t> bytes;
  uint8_t cur = 0;
  int nb = 0;
  void put(int bit) {
    cur = (uint8_t)((cur << 1) | (bit & 1));
    if (++nb == 8) { bytes.push_back(cur); cur = 0; nb = 0; }
  }
  void pad() {
    while (nb != 0) put(0);
  }
};

struct Encoder {
  uint32_t low = 0, high = 0xFFFFFFFFu;
  uint64_t pending = 0;
  BitSink sink;
  void emit(int bit) {
    sink.put(bit);
    for (; pending > 0; --pending) sink.put(!bit);
  }
  void encode(uint32_t cum_lo, uint32_t cum_hi) {  // C[s], C[s+1], totals 65536
    const uint64_t range = (uint64_t)high - low + 1;
    high = low + (uint32_t)((range * cum_hi) >> 16) - 1;
    low = low + (uint32_t)((range * cum_lo) >> 16);
    for (;;) {
      if (high < kHalf) {
        emit(0);
      } else if (low >= kHalf) {
        emit(1);
      } else if (low >= kQuarter && high < kThreeQ) {
        ++pending;
        low -= kQuarter;
        high -= kQuarter;
      } else {
        break;
      }
      low <<= 1;
      high = (high << 1) | 1u;
    }
  }
  void finish() {
    ++pending;
    emit(low < kQuarter ? 0 : 1);
    sink.pad();
  }
};

struct Decoder {
  uint32_t low = 0, high = 0xFFFFFFFFu, value = 0;
  const uint8_t *in = nullptr;
  size_t in_len = 0, bitpos = 0;
  int next_bit() {
    int b = 0;
    const size_t byte = bitpos >> 3;
    if (byte < in_len) b = (in[byte] >> (7 - (bitpos & 7))) & 1;
    ++bitpos;  // zeros past the end
    return b;
  }
  void start(const uint8_t *p, size_t n) {
    in = p; in_len = n; bitpos = 0; value = 0;
    for (int i = 0; i < 32; ++i) value = (value << 1) | (uint32_t)next_bit();
  }
  // cum: C[0..256], C[0] = 0, C[256] = 65536
  int decode(const uint32_t *cum) {
    const uint64_t range = (uint64_t)high - low + 1;
    const uint64_t target = ((((uint64_t)(value - low) + 1) << 16) - 1) / range;
    if (target >= 65536) return -1;
    int s = 0;
    while (!(cum[s] <= target && target < cum[s + 1])) ++s;  // f >= 1 makes s unique
    high = low + (uint32_t)((range * cum[s + 1]) >> 16) - 1;
    low = low + (uint32_t)((range * cum[s]) >> 16);
    for (;;) {
      if (high < kHalf) {
      } else if (low >= kHalf) {
        value -= kHalf; low -= kHalf; high -= kHalf;
      } else if (low >= kQuarter && high < kThreeQ) {
        value -= kQuarter; low -= kQuarter; high -= kQuarter;
      } else {
        break;
      }
      low <<= 1;
      high = (high << 1) | 1u;
      value = (value << 1) | (uint32_t)next_bit();
    }
    return s;
  }
};

void cumulate(const uint16_t *f, uint32_t *cum) {
  cum[0] = 0;
  for (int i = 0; i < 256; ++i) cum[i + 1] = cum[i] + f[i];
}

// ----------------------------------------------------------------------------------------------
// per-stream activations of one model step (everything the backward pass needs)
// ----------------------------------------------------------------------------------------------
struct Act {
  std::vector<uint8_t> win;                       // [T]
  dvec xe_hat, xl_hat, xe, xl;                    // [T*D] LN_e / LN_l of the embedded window
  dvec rstd_e, rstd_l;                            // [T]
  dvec gg, gv, g;                                 // [c]
  dvec M;                                         // [Dc] cache after the roll
  dvec hm, Hg;                                    // [Dh]
  dvec cv, Hl;                                    // [Dh]
  dvec ar, alpha, Hmix;                           // [Dh]
  dvec nc_hat, nc; double rstd_c;                 // [Dh]
  dvec y, z;                                      // [dl]
  dvec Ha, ac, sg, Hc;                            // [Dh]
  dvec u_hat, u; double rstd_f;                   // [Dh]
  dvec eg, ev, Hexp;                              // [De]
  dvec v, nv_hat, nv; double rstd_o;              // [Dh]
  dvec Hout;                                      // [Dh]
  dvec logits, p;                                 // [256]
  bool valid = false;
  void size(const Dims &d) {
    win.assign(d.T, 0);
    for (dvec *a : {&xe_hat, &xl_hat, &xe, &xl}) a->assign(d.Dh, 0.0);
    rstd_e.assign(d.T, 0.0); rstd_l.assign(d.T, 0.0);
    for (dvec *a : {&gg, &gv, &g}) a->assign(d.c, 0.0);
    M.assign(d.Dc, 0.0);
    for (dvec *a : {&hm, &Hg, &cv, &Hl, &ar, &alpha, &Hmix, &nc_hat, &nc, &Ha, &ac, &sg, &Hc, &u_hat, &u, &v,
                    &nv_hat, &nv, &Hout})
      a->assign(d.Dh, 0.0);
    y.assign(d.dl, 0.0); z.assign(d.dl, 0.0);
    for (dvec *a : {&eg, &ev, &Hexp}) a->assign(d.De, 0.0);
    logits.assign(256, 0.0); p.assign(256, 0.0);
  }
};

}  // namespace

// ----------------------------------------------------------------------------------------------
// context
// ----------------------------------------------------------------------------------------------
struct fadeo_ctx {
  fadeo_config cfg;
  Dims d;
  Layout lay;
  bool have_weights = false;
  std::vector<float> loaded;   // blob as loaded (restored by reset)
  std::vector<float> master;   // fp32 master weights
  std::vector<float> w;        // compute copy (matrices rounded to bf16 when dtype == BF16)
  dvec adam_m, adam_v;
  uint64_t adam_t = 0;
  uint64_t weights_hash = 0;
  std::vector<dvec> cache;     // [B][Dc] rolling cache M
  std::vector<Act> act;        // [B]
  std::string err;
  double bits_freq = 0.0, bits_prob = 0.0;
  uint64_t model_steps = 0;

  const float *P(int id) const { return w.data() + lay.off[id]; }
  void refresh_compute() {
    w = master;
    if (cfg.dtype == FADEO_BF16)
      for (int id = 0; id < P_COUNT; ++id)
        if (lay.is_matrix[id])
          for (size_t i = lay.off[id]; i < lay.off[id + 1]; ++i) w[i] = bf16_round(w[i]);
  }
};

namespace {

int fail(fadeo_ctx *c, int code, const char *msg) {
  if (c) c->err = msg;
  return code;
}

bool resolve_dims(const fadeo_config &cfg, Dims &d) {
  d.B = cfg.B; d.T = cfg.T; d.D = cfg.D; d.H = cfg.H;
  d.Dh = d.T * d.D; d.Dc = cfg.d_cache ? cfg.d_cache : d.H; d.De = cfg.d_e ? cfg.d_e : d.H;
  d.dl = cfg.d_low ? cfg.d_low : 64;
  d.k = cfg.conv_k ? cfg.conv_k : 3;
  if (d.B == 0 || d.T == 0 || d.D == 0 || d.H == 0) return false;
  if (cfg.cache_chunk) d.c = cfg.cache_chunk;
  else { if (d.Dc % d.T) return false; d.c = d.Dc / d.T; }
  if (d.c == 0 || d.Dc % d.c) return false;
  if (cfg.dtype > FADEO_BF16 || cfg.update_mode > FADEO_ONLINE_ADAM) return false;
  if (cfg.ablation > 5) return false;
  return true;
}

// ----------------------------------------------------------------------------------------------
// one model step for one stream: window -> probabilities (steps in the order of the paper's Method)
// ----------------------------------------------------------------------------------------------
void forward_stream(fadeo_ctx *C, size_t b, const uint8_t *win) {
  const Dims &d = C->d;
  Act &a = C->act[b];
  const size_t T = d.T, D = d.D, Dh = d.Dh;
  for (size_t j = 0; j < T; ++j) a.win[j] = win[j];

  // X_emb[j] = E[w_j]; X = Flatten_j(LN_D(X_emb[j])) with its own affine pair; the local stream
  // normalises the same embeddings with a second affine pair (Eq. 4's LN). Time-major: the newest
  // symbol occupies the last D channels.
  dvec e(D);
  for (size_t j = 0; j < T; ++j) {
    const float *row = C->P(P_E) + (size_t)win[j] * D;
    for (size_t i = 0; i < D; ++i) e[i] = (double)row[i];
    layer_norm(e.data(), D, C->P(P_GAMMA_E), C->P(P_BETA_E), &a.xe[j * D], &a.xe_hat[j * D], &a.rstd_e[j]);
    layer_norm(e.data(), D, C->P(P_GAMMA_L), C->P(P_BETA_L), &a.xl[j * D], &a.xl_hat[j * D], &a.rstd_l[j]);
  }
  const double *X = a.xe.data();

  // Eq. 1: GeGLU(X_t) = psi(X_t W_g) (.) (X_t W_v), X_t = last D channels of X.
  const double *Xt = X + (T - 1) * D;
  vec_mat(Xt, C->P(P_WG), D, d.c, a.gg.data());
  vec_mat(Xt, C->P(P_WV), D, d.c, a.gv.data());
  for (size_t i = 0; i < d.c; ++i) a.g[i] = gelu(a.gg[i]) * a.gv[i];

  // Eq. 2: roll — drop the oldest slot, append the new one at the end.
  dvec &M = C->cache[b];
  for (size_t i = 0; i + d.c < d.Dc; ++i) M[i] = M[i + d.c];
  for (size_t i = 0; i < d.c; ++i) M[d.Dc - d.c + i] = a.g[i];
  a.M = M;

  // Eq. 3: H_global = psi(M W_m) + lambda_m X
  vec_mat(M.data(), C->P(P_WM), d.Dc, Dh, a.hm.data());
  const double lam_m = (double)C->P(P_LAMBDA_M)[0];
  for (size_t i = 0; i < Dh; ++i) a.Hg[i] = gelu(a.hm[i]) + lam_m * X[i];

  // Progressive ablation (the paper's component table): the output head reads the feature vector of the last stage
  // that is switched on. 1: the global stream alone; 2: + local stream and router; 3: + channel interaction without
  // its gate; 4: with the gate; 0 / 5: the full model.
  const unsigned level = C->cfg.ablation == 0 ? 5u : C->cfg.ablation;
  const double *feat = a.Hg.data();
  if (level >= 2) {
  // Eq. 4: causal Conv1d over time (k taps, channels D -> D, left zero padding, bias), psi, flatten.
  const float *Wc = C->P(P_WCONV);
  for (size_t j = 0; j < T; ++j) {
    double *out = &a.cv[j * D];
    for (size_t o = 0; o < D; ++o) out[o] = (double)C->P(P_BCONV)[o];
    for (size_t r = 0; r < d.k; ++r) {
      const long src = (long)j - (long)(d.k - 1) + (long)r;
      if (src < 0) continue;  // zero padding
      const double *xin = &a.xl[(size_t)src * D];
      const float *Wr = Wc + r * D * D;
      for (size_t i = 0; i < D; ++i)
        for (size_t o = 0; o < D; ++o) out[o] += xin[i] * (double)Wr[i * D + o];
    }
    for (size_t o = 0; o < D; ++o) a.Hl[j * D + o] = gelu(out[o]);
  }

  // Eq. 5-6: alpha = sigma(X W_r); H_mix = alpha (.) H_global + (1 - alpha) (.) H_local
  vec_mat(X, C->P(P_WR), Dh, Dh, a.ar.data());
  for (size_t i = 0; i < Dh; ++i) {
    a.alpha[i] = sigmoid(a.ar[i]);
    a.Hmix[i] = a.alpha[i] * a.Hg[i] + (1.0 - a.alpha[i]) * a.Hl[i];
  }
  feat = a.Hmix.data();
  }
  if (level >= 3) {

  // Eq. 7: H_a = Up(BMM(Down(LN(H_mix)), W_U)); slice b of W_U belongs to stream b; purely linear chain.
  layer_norm(a.Hmix.data(), Dh, C->P(P_GAMMA_C), C->P(P_BETA_C), a.nc.data(), a.nc_hat.data(), &a.rstd_c);
  vec_mat(a.nc.data(), C->P(P_WDOWN), Dh, d.dl, a.y.data());
  vec_mat(a.y.data(), C->P(P_WU) + b * d.dl * d.dl, d.dl, d.dl, a.z.data());
  vec_mat(a.z.data(), C->P(P_WUP), d.dl, Dh, a.Ha.data());

  // Eq. 8: H_coarse = H_a (.) sigma(H_mix W_c) + lambda_c H_mix; without the gate (level 3) the sigmoid factor is dropped
  const double lam_c = (double)C->P(P_LAMBDA_C)[0];
  if (level >= 4) {
    vec_mat(a.Hmix.data(), C->P(P_WC), Dh, Dh, a.ac.data());
    for (size_t i = 0; i < Dh; ++i) {
      a.sg[i] = sigmoid(a.ac[i]);
      a.Hc[i] = a.Ha[i] * a.sg[i] + lam_c * a.Hmix[i];
    }
  } else {
    for (size_t i = 0; i < Dh; ++i) a.Hc[i] = a.Ha[i] + lam_c * a.Hmix[i];
  }
  feat = a.Hc.data();
  }
  if (level >= 5) {

  // Eq. 9: H_expand = psi(u W_fg) (.) (u W_fv), u = LN(H_coarse)
  layer_norm(a.Hc.data(), Dh, C->P(P_GAMMA_F), C->P(P_BETA_F), a.u.data(), a.u_hat.data(), &a.rstd_f);
  vec_mat(a.u.data(), C->P(P_WFG), Dh, d.De, a.eg.data());
  vec_mat(a.u.data(), C->P(P_WFV), Dh, d.De, a.ev.data());
  for (size_t i = 0; i < d.De; ++i) a.Hexp[i] = gelu(a.eg[i]) * a.ev[i];

  // Eq. 10: H = psi(LN(H_expand W_f)) + lambda_o H_coarse
  vec_mat(a.Hexp.data(), C->P(P_WF), d.De, Dh, a.v.data());
  layer_norm(a.v.data(), Dh, C->P(P_GAMMA_O), C->P(P_BETA_O), a.nv.data(), a.nv_hat.data(), &a.rstd_o);
  const double lam_o = (double)C->P(P_LAMBDA_O)[0];
  for (size_t i = 0; i < Dh; ++i) a.Hout[i] = gelu(a.nv[i]) + lam_o * a.Hc[i];
  feat = a.Hout.data();
  }

  // head (implied by the problem statement: a distribution over the 256 byte values): one linear
  // layer with bias, then a max-subtracted softmax.
  vec_mat(feat, C->P(P_WO), Dh, 256, a.logits.data());
  double mx = -INFINITY;
  for (int i = 0; i < 256; ++i) {
    a.logits[i] += (double)C->P(P_BO)[i];
    if (a.logits[i] > mx) mx = a.logits[i];
  }
  double s = 0.0;
  for (int i = 0; i < 256; ++i) { a.p[i] = std::exp(a.logits[i] - mx); s += a.p[i]; }
  for (int i = 0; i < 256; ++i) a.p[i] /= s;
  a.valid = true;
}

// ----------------------------------------------------------------------------------------------
// backward of one stream: dlogits = scale * (p - onehot(target)); accumulates into grad (blob layout).
// The gradient reaches the cache only through its newest slot (older slots are kept as computed).
// ----------------------------------------------------------------------------------------------
void backward_stream(fadeo_ctx *C, size_t b, uint8_t target, double scale, double *grad) {
  const Dims &d = C->d;
  const Layout &L = C->lay;
  const Act &a = C->act[b];
  const size_t T = d.T, D = d.D, Dh = d.Dh;
  auto G = [&](int id) { return grad + L.off[id]; };

  dvec dlog(256);
  for (int i = 0; i < 256; ++i) dlog[i] = scale * (a.p[i] - (i == (int)target ? 1.0 : 0.0));

  // head: its input is the feature vector of the ablation level (forward_stream), and the gradient enters the chain there;
  // parameters of the stages that are switched off get no gradient
  const unsigned level = C->cfg.ablation == 0 ? 5u : C->cfg.ablation;
  const dvec &feat = level >= 5 ? a.Hout : level >= 3 ? a.Hc : level == 2 ? a.Hmix : a.Hg;
  outer_acc(feat.data(), dlog.data(), Dh, 256, G(P_WO));
  for (int i = 0; i < 256; ++i) G(P_BO)[i] += dlog[i];
  dvec dHout(Dh);
  mat_vec_t(C->P(P_WO), dlog.data(), Dh, 256, dHout.data());

  dvec dHc(Dh, 0.0), dHmix(Dh, 0.0), dHg(Dh, 0.0), dHl(Dh, 0.0), dX(Dh, 0.0), tmp(Dh);
  if (level == 4 || level == 3) dHc = dHout;
  if (level == 2) dHmix = dHout;
  if (level == 1) dHg = dHout;

  if (level >= 5) {
  // Eq. 10
  dvec dnv(Dh), dv(Dh, 0.0);
  const double lam_o = (double)C->P(P_LAMBDA_O)[0];
  for (size_t i = 0; i < Dh; ++i) {
    dnv[i] = dHout[i] * gelu_grad(a.nv[i]);
    G(P_LAMBDA_O)[0] += dHout[i] * a.Hc[i];
    dHc[i] += lam_o * dHout[i];
  }
  layer_norm_bwd(dnv.data(), a.nv_hat.data(), a.rstd_o, Dh, C->P(P_GAMMA_O), G(P_GAMMA_O), G(P_BETA_O), dv.data());
  outer_acc(a.Hexp.data(), dv.data(), d.De, Dh, G(P_WF));
  dvec dHexp(d.De);
  mat_vec_t(C->P(P_WF), dv.data(), d.De, Dh, dHexp.data());

  // Eq. 9
  dvec deg(d.De), dev(d.De), du(Dh);
  for (size_t i = 0; i < d.De; ++i) {
    deg[i] = dHexp[i] * a.ev[i] * gelu_grad(a.eg[i]);
    dev[i] = dHexp[i] * gelu(a.eg[i]);
  }
  outer_acc(a.u.data(), deg.data(), Dh, d.De, G(P_WFG));
  outer_acc(a.u.data(), dev.data(), Dh, d.De, G(P_WFV));
  mat_vec_t(C->P(P_WFG), deg.data(), Dh, d.De, du.data());
  mat_vec_t(C->P(P_WFV), dev.data(), Dh, d.De, tmp.data());
  for (size_t i = 0; i < Dh; ++i) du[i] += tmp[i];
  layer_norm_bwd(du.data(), a.u_hat.data(), a.rstd_f, Dh, C->P(P_GAMMA_F), G(P_GAMMA_F), G(P_BETA_F), dHc.data());
  }

  if (level >= 3) {
  // Eq. 8 (level 3: without the gate, H_coarse = H_a + lambda_c H_mix)
  dvec dHa(Dh), dac(Dh);
  const double lam_c = (double)C->P(P_LAMBDA_C)[0];
  for (size_t i = 0; i < Dh; ++i) {
    dHa[i] = level >= 4 ? dHc[i] * a.sg[i] : dHc[i];
    dac[i] = level >= 4 ? dHc[i] * a.Ha[i] * a.sg[i] * (1.0 - a.sg[i]) : 0.0;
    G(P_LAMBDA_C)[0] += dHc[i] * a.Hmix[i];
    dHmix[i] += lam_c * dHc[i];
  }
  if (level >= 4) {
    outer_acc(a.Hmix.data(), dac.data(), Dh, Dh, G(P_WC));
    mat_vec_t(C->P(P_WC), dac.data(), Dh, Dh, tmp.data());
    for (size_t i = 0; i < Dh; ++i) dHmix[i] += tmp[i];
  }

  // Eq. 7
  dvec dz(d.dl), dy(d.dl), dnc(Dh);
  outer_acc(a.z.data(), dHa.data(), d.dl, Dh, G(P_WUP));
  mat_vec_t(C->P(P_WUP), dHa.data(), d.dl, Dh, dz.data());
  outer_acc(a.y.data(), dz.data(), d.dl, d.dl, G(P_WU) + b * d.dl * d.dl);
  mat_vec_t(C->P(P_WU) + b * d.dl * d.dl, dz.data(), d.dl, d.dl, dy.data());
  outer_acc(a.nc.data(), dy.data(), Dh, d.dl, G(P_WDOWN));
  mat_vec_t(C->P(P_WDOWN), dy.data(), Dh, d.dl, dnc.data());
  layer_norm_bwd(dnc.data(), a.nc_hat.data(), a.rstd_c, Dh, C->P(P_GAMMA_C), G(P_GAMMA_C), G(P_BETA_C), dHmix.data());
  }

  dvec dxl(Dh, 0.0);
  if (level >= 2) {
  // Eq. 5-6
  dvec dar(Dh);
  for (size_t i = 0; i < Dh; ++i) {
    dHg[i] = dHmix[i] * a.alpha[i];
    dHl[i] = dHmix[i] * (1.0 - a.alpha[i]);
    dar[i] = dHmix[i] * (a.Hg[i] - a.Hl[i]) * a.alpha[i] * (1.0 - a.alpha[i]);
  }
  outer_acc(a.xe.data(), dar.data(), Dh, Dh, G(P_WR));
  mat_vec_t(C->P(P_WR), dar.data(), Dh, Dh, dX.data());

  // Eq. 4
  dvec dcv(D);
  for (size_t j = 0; j < T; ++j) {
    for (size_t o = 0; o < D; ++o) {
      dcv[o] = dHl[j * D + o] * gelu_grad(a.cv[j * D + o]);
      G(P_BCONV)[o] += dcv[o];
    }
    for (size_t r = 0; r < d.k; ++r) {
      const long src = (long)j - (long)(d.k - 1) + (long)r;
      if (src < 0) continue;
      const double *xin = &a.xl[(size_t)src * D];
      const float *Wr = C->P(P_WCONV) + r * D * D;
      double *dWr = G(P_WCONV) + r * D * D;
      for (size_t i = 0; i < D; ++i) {
        double acc = 0.0;
        for (size_t o = 0; o < D; ++o) {
          dWr[i * D + o] += xin[i] * dcv[o];
          acc += (double)Wr[i * D + o] * dcv[o];
        }
        dxl[(size_t)src * D + i] += acc;
      }
    }
  }
  }

  // Eq. 3
  dvec dhm(Dh), dM(d.Dc);
  const double lam_m = (double)C->P(P_LAMBDA_M)[0];
  for (size_t i = 0; i < Dh; ++i) {
    dhm[i] = dHg[i] * gelu_grad(a.hm[i]);
    G(P_LAMBDA_M)[0] += dHg[i] * a.xe[i];
    dX[i] += lam_m * dHg[i];
  }
  outer_acc(a.M.data(), dhm.data(), d.Dc, Dh, G(P_WM));
  mat_vec_t(C->P(P_WM), dhm.data(), d.Dc, Dh, dM.data());

  // Eq. 1-2: only the newest slot carries gradient.
  dvec dgg(d.c), dgv(d.c), dxt(D), tmpD(D);
  for (size_t i = 0; i < d.c; ++i) {
    const double dg = dM[d.Dc - d.c + i];
    dgg[i] = dg * a.gv[i] * gelu_grad(a.gg[i]);
    dgv[i] = dg * gelu(a.gg[i]);
  }
  const double *Xt = a.xe.data() + (T - 1) * D;
  outer_acc(Xt, dgg.data(), D, d.c, G(P_WG));
  outer_acc(Xt, dgv.data(), D, d.c, G(P_WV));
  mat_vec_t(C->P(P_WG), dgg.data(), D, d.c, dxt.data());
  mat_vec_t(C->P(P_WV), dgv.data(), D, d.c, tmpD.data());
  for (size_t i = 0; i < D; ++i) dX[(T - 1) * D + i] += dxt[i] + tmpD[i];

  // the two per-token LayerNorms and the embedding rows
  dvec de(D);
  for (size_t j = 0; j < T; ++j) {
    for (size_t i = 0; i < D; ++i) de[i] = 0.0;
    layer_norm_bwd(&dX[j * D], &a.xe_hat[j * D], a.rstd_e[j], D, C->P(P_GAMMA_E), G(P_GAMMA_E), G(P_BETA_E), de.data());
    layer_norm_bwd(&dxl[j * D], &a.xl_hat[j * D], a.rstd_l[j], D, C->P(P_GAMMA_L), G(P_GAMMA_L), G(P_BETA_L), de.data());
    double *dErow = G(P_E) + (size_t)a.win[j] * D;
    for (size_t i = 0; i < D; ++i) dErow[i] += de[i];
  }
}

size_t count_active(const fadeo_ctx *C, const uint8_t *active) {
  size_t n = 0;
  for (size_t b = 0; b < C->d.B; ++b) n += (!active || active[b]) ? 1 : 0;
  return n;
}

int compute_grad(fadeo_ctx *C, const uint8_t *targets, const uint8_t *active, dvec &grad) {
  const size_t na = count_active(C, active);
  grad.assign(C->lay.off[P_COUNT], 0.0);
  if (na == 0) return FADEO_OK;
  for (size_t b = 0; b < C->d.B; ++b) {
    if (active && !active[b]) continue;
    if (!C->act[b].valid) return fail(C, FADEO_E_INVALID_ARG, "backward before a model step");
    backward_stream(C, b, targets[b], 1.0 / (double)na, grad.data());
  }
  return FADEO_OK;
}

// Adam (Kingma & Ba), bias-corrected, no weight decay; master weights are fp32, moments fp64.
void adam_step(fadeo_ctx *C, const dvec &grad) {
  const double lr = C->cfg.lr, b1 = C->cfg.beta1, b2 = C->cfg.beta2, eps = C->cfg.eps;
  C->adam_t += 1;
  const double c1 = 1.0 - std::pow(b1, (double)C->adam_t), c2 = 1.0 - std::pow(b2, (double)C->adam_t);
  for (size_t i = 0; i < grad.size(); ++i) {
    const double g = grad[i];
    C->adam_m[i] = b1 * C->adam_m[i] + (1.0 - b1) * g;
    C->adam_v[i] = b2 * C->adam_v[i] + (1.0 - b2) * g * g;
    const double mh = C->adam_m[i] / c1, vh = C->adam_v[i] / c2;
    C->master[i] = (float)((double)C->master[i] - lr * mh / (std::sqrt(vh) + eps));
  }
  C->refresh_compute();
}

// ----------------------------------------------------------------------------------------------
// container: 64-byte little-endian header, B payload lengths (u32), B payloads back to back
// ----------------------------------------------------------------------------------------------
const size_t kHeader = 64;
void put_u16(uint8_t *p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
void put_u32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
void put_u64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
uint32_t get_u16(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
uint32_t get_u32(const uint8_t *p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
uint64_t get_u64(const uint8_t *p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }
uint32_t f32_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }

void write_header(const fadeo_ctx *C, uint64_t n, uint8_t *h) {
  std::memset(h, 0, kHeader);
  h[0] = 'F'; h[1] = 'A'; h[2] = 'D'; h[3] = 'E';
  put_u16(h + 4, 1);
  h[6] = (uint8_t)C->cfg.dtype; h[7] = (uint8_t)C->cfg.update_mode;
  put_u16(h + 8, (uint32_t)C->d.T); put_u16(h + 10, (uint32_t)C->d.D); put_u32(h + 12, (uint32_t)C->d.De);
  if (C->d.Dc != C->d.De) put_u32(h + 44, (uint32_t)C->d.Dc);  // 0: the cache is as wide as the refiner
  put_u16(h + 16, (uint32_t)C->d.dl); put_u16(h + 18, (uint32_t)C->d.c); put_u16(h + 20, (uint32_t)C->d.k);
  h[22] = (uint8_t)(C->cfg.ablation == 0 ? 5u : C->cfg.ablation);  // which stage feeds the head: part of the model's definition
  put_u32(h + 24, (uint32_t)C->d.B);
  put_u32(h + 28, f32_bits(C->cfg.lr)); put_u32(h + 32, f32_bits(C->cfg.beta1));
  put_u32(h + 36, f32_bits(C->cfg.beta2)); put_u32(h + 40, f32_bits(C->cfg.eps));
  put_u64(h + 48, n); put_u64(h + 56, C->weights_hash);
}

int check_header(fadeo_ctx *C, const uint8_t *h, uint64_t *n) {
  if (!(h[0] == 'F' && h[1] == 'A' && h[2] == 'D' && h[3] == 'E') || get_u16(h + 4) != 1)
    return fail(C, FADEO_E_CORRUPT_STREAM, "bad magic or version");
  const bool same = h[6] == C->cfg.dtype && h[7] == C->cfg.update_mode && get_u16(h + 8) == C->d.T &&
                    get_u16(h + 10) == C->d.D && get_u32(h + 12) == C->d.De && get_u32(h + 44) == (C->d.Dc != C->d.De ? C->d.Dc : 0) &&
                    get_u16(h + 16) == C->d.dl &&
                    get_u16(h + 18) == C->d.c && get_u16(h + 20) == C->d.k && get_u32(h + 24) == C->d.B &&
                    h[22] == (C->cfg.ablation == 0 ? 5u : C->cfg.ablation) &&
                    get_u32(h + 28) == f32_bits(C->cfg.lr) && get_u32(h + 32) == f32_bits(C->cfg.beta1) &&
                    get_u32(h + 36) == f32_bits(C->cfg.beta2) && get_u32(h + 40) == f32_bits(C->cfg.eps);
  if (!same) return fail(C, FADEO_E_BAD_CONFIG, "container was written with a different configuration");
  if (get_u64(h + 56) != C->weights_hash) return fail(C, FADEO_E_WEIGHTS_MISMATCH, "weight hash differs");
  *n = get_u64(h + 48);
  return FADEO_OK;
}

void do_reset(fadeo_ctx *C) {
  for (auto &m : C->cache) m.assign(C->d.Dc, 0.0);
  for (auto &a : C->act) a.valid = false;
  if (C->have_weights) {
    C->master = C->loaded;
    C->refresh_compute();
  }
  C->adam_m.assign(C->lay.off[P_COUNT], 0.0);
  C->adam_v.assign(C->lay.off[P_COUNT], 0.0);
  C->adam_t = 0;
  C->bits_freq = C->bits_prob = 0.0;
  C->model_steps = 0;
}

// Length of stream k when n bytes are split into B contiguous streams of L = ceil(n / B) bytes.
size_t stream_len(size_t n, size_t L, size_t k) {
  const size_t start = k * L;
  if (start >= n) return 0;
  return (n - start < L) ? (n - start) : L;
}

}  // namespace

// ----------------------------------------------------------------------------------------------
// C ABI
// ----------------------------------------------------------------------------------------------
extern "C" {

size_t fadeo_weights_nbytes(const fadeo_config *cfg) {
  Dims d;
  if (!cfg || !resolve_dims(*cfg, d)) return 0;
  return make_layout(d).off[P_COUNT] * sizeof(float);
}

int fadeo_create(const fadeo_config *cfg, fadeo_ctx **out) {
  if (!cfg || !out) return FADEO_E_INVALID_ARG;
  *out = nullptr;
  if (cfg->struct_size != sizeof(fadeo_config)) return FADEO_E_INVALID_ARG;
  Dims d;
  if (!resolve_dims(*cfg, d)) return FADEO_E_BAD_CONFIG;
  fadeo_ctx *C = new fadeo_ctx();
  C->cfg = *cfg;
  if (C->cfg.lr == 0.0f) C->cfg.lr = 1e-3f;
  if (C->cfg.beta1 == 0.0f) C->cfg.beta1 = 0.9f;
  if (C->cfg.beta2 == 0.0f) C->cfg.beta2 = 0.999f;
  if (C->cfg.eps == 0.0f) C->cfg.eps = 1e-8f;
  C->d = d;
  C->lay = make_layout(d);
  C->cache.assign(d.B, dvec(d.Dc, 0.0));
  C->act.resize(d.B);
  for (auto &a : C->act) a.size(d);
  do_reset(C);
  *out = C;
  return FADEO_OK;
}

int fadeo_load_weights(fadeo_ctx *C, const void *blob, size_t nbytes) {
  if (!C || !blob) return FADEO_E_INVALID_ARG;
  if (nbytes != C->lay.off[P_COUNT] * sizeof(float)) return fail(C, FADEO_E_WEIGHTS_MISMATCH, "blob size");
  C->loaded.resize(C->lay.off[P_COUNT]);
  std::memcpy(C->loaded.data(), blob, nbytes);
  for (float f : C->loaded)
    if (!std::isfinite(f)) return fail(C, FADEO_E_NUMERIC, "non-finite weight");
  C->weights_hash = fadeo_fnv1a64(blob, nbytes);
  C->have_weights = true;
  do_reset(C);
  return FADEO_OK;
}

int fadeo_reset(fadeo_ctx *C) {
  if (!C) return FADEO_E_INVALID_ARG;
  do_reset(C);
  return FADEO_OK;
}

int fadeo_step_probs(fadeo_ctx *C, const uint8_t *windows, const uint8_t *active, uint16_t *freq, float *probs) {
  if (!C || !windows) return FADEO_E_INVALID_ARG;
  if (!C->have_weights) return fail(C, FADEO_E_NO_WEIGHTS, "no weights loaded");
  for (size_t b = 0; b < C->d.B; ++b) {
    if (active && !active[b]) { C->act[b].valid = false; continue; }
    forward_stream(C, b, windows + b * C->d.T);
    float pf[256];
    for (int i = 0; i < 256; ++i) pf[i] = (float)C->act[b].p[i];
    if (probs) std::memcpy(probs + b * 256, pf, sizeof(pf));
    if (freq) {
      int rc = quantize_row(pf, freq + b * 256);
      if (rc) return fail(C, rc, "probabilities are not finite");
    }
  }
  return FADEO_OK;
}

int fadeo_loss(fadeo_ctx *C, const uint8_t *targets, const uint8_t *active, double *loss) {
  if (!C || !targets || !loss) return FADEO_E_INVALID_ARG;
  const size_t na = count_active(C, active);
  double s = 0.0;
  for (size_t b = 0; b < C->d.B; ++b) {
    if (active && !active[b]) continue;
    if (!C->act[b].valid) return fail(C, FADEO_E_INVALID_ARG, "loss before a model step");
    s += -std::log(C->act[b].p[targets[b]]);
  }
  *loss = na ? s / (double)na : 0.0;
  return FADEO_OK;
}

int fadeo_backward(fadeo_ctx *C, const uint8_t *targets, const uint8_t *active, double *grad_blob) {
  if (!C || !targets || !grad_blob) return FADEO_E_INVALID_ARG;
  dvec g;
  int rc = compute_grad(C, targets, active, g);
  if (rc) return rc;
  std::memcpy(grad_blob, g.data(), g.size() * sizeof(double));
  return FADEO_OK;
}

int fadeo_step_update(fadeo_ctx *C, const uint8_t *targets, const uint8_t *active) {
  if (!C || !targets) return FADEO_E_INVALID_ARG;
  if (C->cfg.update_mode != FADEO_ONLINE_ADAM) return fail(C, FADEO_E_BAD_CONFIG, "context is frozen");
  if (count_active(C, active) == 0) return FADEO_OK;  // nothing coded, nothing learned, no Adam tick
  dvec g;
  int rc = compute_grad(C, targets, active, g);
  if (rc) return rc;
  adam_step(C, g);
  return FADEO_OK;
}

int fadeo_get_weights(fadeo_ctx *C, float *blob, size_t nbytes) {
  if (!C || !blob || nbytes != C->master.size() * sizeof(float)) return FADEO_E_INVALID_ARG;
  std::memcpy(blob, C->master.data(), nbytes);
  return FADEO_OK;
}

size_t fadeo_tap(fadeo_ctx *C, int which, uint32_t stream, double *out, size_t cap) {
  if (!C || stream >= C->d.B) return 0;
  const Act &a = C->act[stream];
  const dvec *v = nullptr;
  switch (which) {
    case FADEO_TAP_X: v = &a.xe; break;
    case FADEO_TAP_CACHE: v = &a.M; break;
    case FADEO_TAP_H_GLOBAL: v = &a.Hg; break;
    case FADEO_TAP_H_LOCAL: v = &a.Hl; break;
    case FADEO_TAP_ALPHA: v = &a.alpha; break;
    case FADEO_TAP_H_MIX: v = &a.Hmix; break;
    case FADEO_TAP_Y_DOWN: v = &a.y; break;
    case FADEO_TAP_Z_BMM: v = &a.z; break;
    case FADEO_TAP_H_A: v = &a.Ha; break;
    case FADEO_TAP_H_COARSE: v = &a.Hc; break;
    case FADEO_TAP_H_EXPAND: v = &a.Hexp; break;
    case FADEO_TAP_H_OUT: v = &a.Hout; break;
    case FADEO_TAP_LOGITS: v = &a.logits; break;
    case FADEO_TAP_PROBS: v = &a.p; break;
    default: return 0;
  }
  if (out && cap >= v->size()) std::memcpy(out, v->data(), v->size() * sizeof(double));
  return v->size();
}

size_t fadeo_encode_bound(const fadeo_ctx *C, size_t n) {
  if (!C) return 0;
  const size_t B = C->d.B, L = (n + B - 1) / B;
  // a symbol costs at most 16 bits (f >= 1 of 2^16) plus termination and padding per stream
  return kHeader + 4 * B + B * (2 * L + 8);
}

int fadeo_encode(fadeo_ctx *C, const uint8_t *src, size_t n, uint8_t *dst, size_t dst_cap, size_t *dst_len) {
  if (!C || (!src && n) || !dst || !dst_len) return FADEO_E_INVALID_ARG;
  if (!C->have_weights) return fail(C, FADEO_E_NO_WEIGHTS, "no weights loaded");
  do_reset(C);
  const Dims &d = C->d;
  const size_t B = d.B, T = d.T, L = (n + B - 1) / B;
  std::vector<Encoder> enc(B);
  std::vector<uint8_t> active(B), targets(B), windows(B * T);
  std::vector<uint16_t> freq(B * 256);
  std::vector<float> probs(B * 256);
  uint32_t cum[257];
  // Algorithm 1: the first T symbols of every stream are coded with p = 1/256 (f = 256 each); from
  // then on predict from the previous T symbols, code, and (online mode) update after coding.
  for (size_t i = 0; i < L; ++i) {
    size_t na = 0;
    for (size_t k = 0; k < B; ++k) {
      active[k] = i < stream_len(n, L, k) ? 1 : 0;
      na += active[k];
      if (active[k]) targets[k] = src[k * L + i];
    }
    if (na == 0) break;
    if (i < T) {
      for (size_t k = 0; k < B; ++k)
        if (active[k]) enc[k].encode((uint32_t)targets[k] * 256u, ((uint32_t)targets[k] + 1u) * 256u);
      continue;
    }
    for (size_t k = 0; k < B; ++k)
      if (active[k]) std::memcpy(&windows[k * T], src + k * L + i - T, T);
    int rc = fadeo_step_probs(C, windows.data(), active.data(), freq.data(), probs.data());
    if (rc) return rc;
    for (size_t k = 0; k < B; ++k) {
      if (!active[k]) continue;
      cumulate(&freq[k * 256], cum);
      enc[k].encode(cum[targets[k]], cum[targets[k] + 1]);
      C->bits_freq += -std::log2((double)freq[k * 256 + targets[k]] / 65536.0);
      C->bits_prob += -std::log2(C->act[k].p[targets[k]]);
      C->model_steps += 1;
    }
    if (C->cfg.update_mode == FADEO_ONLINE_ADAM) {
      rc = fadeo_step_update(C, targets.data(), active.data());
      if (rc) return rc;
    }
  }
  size_t total = kHeader + 4 * B;
  for (size_t k = 0; k < B; ++k) {
    if (stream_len(n, L, k) > 0) enc[k].finish();
    total += enc[k].sink.bytes.size();
  }
  *dst_len = total;
  if (total > dst_cap) return fail(C, FADEO_E_BUFFER_TOO_SMALL, "dst_cap too small");
  write_header(C, n, dst);
  size_t pos = kHeader + 4 * B;
  for (size_t k = 0; k < B; ++k) {
    const auto &by = enc[k].sink.bytes;
    put_u32(dst + kHeader + 4 * k, (uint32_t)by.size());
    if (!by.empty()) std::memcpy(dst + pos, by.data(), by.size());
    pos += by.size();
  }
  return FADEO_OK;
}

int fadeo_decode(fadeo_ctx *C, const uint8_t *src, size_t src_len, uint8_t *dst, size_t dst_cap, size_t *dst_len) {
  if (!C || !src || !dst_len) return FADEO_E_INVALID_ARG;
  if (!C->have_weights) return fail(C, FADEO_E_NO_WEIGHTS, "no weights loaded");
  const Dims &d = C->d;
  const size_t B = d.B, T = d.T;
  if (src_len < kHeader + 4 * B) return fail(C, FADEO_E_CORRUPT_STREAM, "truncated header");
  uint64_t n64 = 0;
  int rc = check_header(C, src, &n64);
  if (rc) return rc;
  const size_t n = (size_t)n64, L = (n + B - 1) / B;
  *dst_len = n;
  if (n > dst_cap || (!dst && n)) return fail(C, FADEO_E_BUFFER_TOO_SMALL, "dst_cap too small");
  std::vector<Decoder> dec(B);
  size_t pos = kHeader + 4 * B;
  for (size_t k = 0; k < B; ++k) {
    const size_t len = get_u32(src + kHeader + 4 * k);
    if (len > src_len - pos) return fail(C, FADEO_E_CORRUPT_STREAM, "payload runs past the end");
    if ((stream_len(n, L, k) == 0) != (len == 0)) return fail(C, FADEO_E_CORRUPT_STREAM, "payload length");
    dec[k].start(src + pos, len);
    pos += len;
  }
  if (pos != src_len) return fail(C, FADEO_E_CORRUPT_STREAM, "trailing bytes");
  do_reset(C);
  std::vector<uint8_t> active(B), targets(B), windows(B * T);
  std::vector<uint16_t> freq(B * 256);
  uint32_t cum[257];
  for (size_t i = 0; i < L; ++i) {
    size_t na = 0;
    for (size_t k = 0; k < B; ++k) { active[k] = i < stream_len(n, L, k) ? 1 : 0; na += active[k]; }
    if (na == 0) break;
    if (i < T) {
      for (int s = 0; s <= 256; ++s) cum[s] = (uint32_t)s * 256u;
      for (size_t k = 0; k < B; ++k)
        if (active[k]) {
          int s = dec[k].decode(cum);
          if (s < 0) return fail(C, FADEO_E_CORRUPT_STREAM, "coder target out of range");
          dst[k * L + i] = (uint8_t)s;
        }
      continue;
    }
    for (size_t k = 0; k < B; ++k)
      if (active[k]) std::memcpy(&windows[k * T], dst + k * L + i - T, T);
    rc = fadeo_step_probs(C, windows.data(), active.data(), freq.data(), nullptr);
    if (rc) return rc;
    for (size_t k = 0; k < B; ++k) {
      if (!active[k]) continue;
      cumulate(&freq[k * 256], cum);
      int s = dec[k].decode(cum);
      if (s < 0) return fail(C, FADEO_E_CORRUPT_STREAM, "coder target out of range");
      dst[k * L + i] = (uint8_t)s;
      targets[k] = (uint8_t)s;
    }
    if (C->cfg.update_mode == FADEO_ONLINE_ADAM) {
      rc = fadeo_step_update(C, targets.data(), active.data());
      if (rc) return rc;
    }
  }
  return FADEO_OK;
}

int fadeo_last_code_stats(fadeo_ctx *C, double *bf, double *bp, uint64_t *steps) {
  if (!C) return FADEO_E_INVALID_ARG;
  if (bf) *bf = C->bits_freq;
  if (bp) *bp = C->bits_prob;
  if (steps) *steps = C->model_steps;
  return FADEO_OK;
}

int fadeo_quantize(const float *p, size_t rows, uint16_t *freq) {
  if (!p || !freq) return FADEO_E_INVALID_ARG;
  for (size_t r = 0; r < rows; ++r) {
    int rc = quantize_row(p + r * 256, freq + r * 256);
    if (rc) return rc;
  }
  return FADEO_OK;
}

int fadeo_coder_encode(const uint16_t *freq, const uint8_t *sym, size_t n, uint8_t *out, size_t cap, size_t *len) {
  if ((!freq && n) || (!sym && n) || !len) return FADEO_E_INVALID_ARG;
  Encoder e;
  uint32_t cum[257];
  for (size_t i = 0; i < n; ++i) {
    cumulate(freq + i * 256, cum);
    if (cum[256] != 65536) return FADEO_E_INVALID_ARG;
    if (freq[i * 256 + sym[i]] == 0) return FADEO_E_INVALID_ARG;
    e.encode(cum[sym[i]], cum[sym[i] + 1]);
  }
  if (n) e.finish();
  *len = e.sink.bytes.size();
  if (*len > cap || (!out && *len)) return FADEO_E_BUFFER_TOO_SMALL;
  if (*len) std::memcpy(out, e.sink.bytes.data(), *len);
  return FADEO_OK;
}

int fadeo_coder_decode(const uint16_t *freq, size_t n, const uint8_t *in, size_t in_len, uint8_t *sym) {
  if ((!freq && n) || (!sym && n) || (!in && in_len)) return FADEO_E_INVALID_ARG;
  Decoder dcd;
  dcd.start(in, in_len);
  uint32_t cum[257];
  for (size_t i = 0; i < n; ++i) {
    cumulate(freq + i * 256, cum);
    if (cum[256] != 65536) return FADEO_E_INVALID_ARG;
    int s = dcd.decode(cum);
    if (s < 0) return FADEO_E_CORRUPT_STREAM;
    sym[i] = (uint8_t)s;
  }
  return FADEO_OK;
}

/* Test hook: overwrite the rolling cache of one stream (used by the finite-difference test, which must
 * hold stored slots constant while perturbing weights). */
int fadeo_test_set_cache(fadeo_ctx *C, uint32_t stream, const double *m, size_t n) {
  if (!C || stream >= C->d.B || !m || n != C->d.Dc) return FADEO_E_INVALID_ARG;
  C->cache[stream].assign(m, m + n);
  return FADEO_OK;
}

uint64_t fadeo_fnv1a64(const void *p, size_t n) {
  const uint8_t *b = (const uint8_t *)p;
  uint64_t h = 0xcbf29ce484222325ull;
  for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 0x100000001b3ull; }
  return h;
}

const char *fadeo_last_error(const fadeo_ctx *C) { return C ? C->err.c_str() : "null context"; }

void fadeo_destroy(fadeo_ctx *C) { delete C; }

}  // extern "C"
