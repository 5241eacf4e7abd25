// fade_bwd.hip — the online update's non-GEMM kernels: loss gradient, LayerNorm / activation backward passes,
// batch-transposed operand copies for the weight-gradient products, per-stream memory backward + its Adam,
// conv / embedding gradients, parameter reductions and Adam (Algorithm 1's "backpropagate to update P"; loss Eq. 12).
// All reductions run in a fixed order (no atomics): encoder and decoder must reproduce the same weights bit for bit.
#include "fade_dev.h"
#include "fade_kernels.h"

namespace {

__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float x) {
  return 0.5f * (1.0f + erff(x * 0.70710678118654752f)) + x * 0.3989422804014327f * expf(-0.5f * x * x);
}

template <typename AT> __device__ __forceinline__ void ld8(const AT *p, float v[8]);
template <> __device__ __forceinline__ void ld8<bf16_t>(const bf16_t *p, float v[8]) {
  const bf16x8 r = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)r[i];
}
template <> __device__ __forceinline__ void ld8<float>(const float *p, float v[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
}
template <typename AT> __device__ __forceinline__ void st8(AT *p, const float v[8]);
template <> __device__ __forceinline__ void st8<bf16_t>(bf16_t *p, const float v[8]) {
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (bf16_t)v[i];
  *reinterpret_cast<bf16x8 *>(p) = r;
}
template <> __device__ __forceinline__ void st8<float>(float *p, const float v[8]) {
  f32x4 a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
  *reinterpret_cast<f32x4 *>(p) = a;
  *reinterpret_cast<f32x4 *>(p + 4) = b;
}

__device__ __forceinline__ void moments(const float *stats, int stats_n, int width, float &mean, float &rstd) {
  float s = 0.0f, q = 0.0f;
  for (int j = 0; j < stats_n; ++j) { s += stats[2 * j]; q += stats[2 * j + 1]; }
  const float inv = 1.0f / (float)width;
  mean = s * inv;
  rstd = 1.0f / sqrtf(fmaxf(q * inv - mean * mean, 0.0f) + 1e-5f);
}

// Sum of one value per thread over a 256-thread workgroup, same order every time: butterfly inside each
// wavefront, then the four wavefront sums added in index order. Every thread gets the result.
__device__ __forceinline__ float block_sum(float v, float *red /*[4]*/) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();  // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// ---------------------------------------------------------------------------------------------------
// step bookkeeping: number of active streams, Adam's step count and bias corrections (one thread)
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void update_prep_kernel(WinSrc ws, int B, UpdateState *u, float beta1, float beta2) {
  __shared__ int cnt[256];
  int mine = 0;
  for (int b = threadIdx.x; b < B; b += 256) mine += stream_active(ws, b) ? 1 : 0;
  cnt[threadIdx.x] = mine;
  __syncthreads();
  if (threadIdx.x != 0) return;
  int na = 0;
  for (int k = 0; k < 256; ++k) na += cnt[k];
  u->na = na;
  if (na > 0) {
    u->t += 1;
    u->c1 = 1.0f - powf(beta1, (float)u->t);
    u->c2 = 1.0f - powf(beta2, (float)u->t);
    u->inv_na = 1.0f / (float)na;
  }
}

// dlogits = (p - onehot(target)) / n_active for active streams, 0 otherwise (gradient of the mean NLL, Eq. 12)
template <typename AT>
__global__ __launch_bounds__(256) void dlogits_kernel(WinSrc ws, const uint8_t *targets, long long tstride, int B, const float *probs,
                                                      const UpdateState *u, AT *dl) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= B) return;
  const bool act = stream_active(ws, b);
  const f32x4 p = *reinterpret_cast<const f32x4 *>(probs + (size_t)b * 256 + 4 * lane);
  const int x = act ? targets[(long long)b * tstride] : -1;
  const float sc = u->inv_na;
  AT *o = dl + (size_t)b * 256 + 4 * lane;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (AT)(act ? sc * (p[i] - ((4 * lane + i) == x ? 1.0f : 0.0f)) : 0.0f);
}

// ---------------------------------------------------------------------------------------------------
// batch-major -> feature-major copies: dst[n][b] = f(src[b][n]) for the weight-gradient products, which reduce over
// the batch and therefore need batch-contiguous operands. Optional LayerNorm on the way (u = LN(H_coarse), LN(H_mix)).
// 64 x 64 tiles through LDS; dst has leading dimension Bp (batch rounded up to 64, padding stays zero).
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void transpose_kernel(TransposeArgs a) {
  __shared__ float tile[64][65];
  const AT *src = static_cast<const AT *>(a.src);
  AT *dst = static_cast<AT *>(a.dst);
  const int b0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4) {
    const int b = b0 + r;
    float v = 0.0f;
    if (b < a.B) {
      v = (float)src[(size_t)b * a.ld + n0 + tx];
      if (a.stats) {
        float mean, rstd;
        moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.width, mean, rstd);
        v = (v - mean) * rstd * a.gamma[n0 + tx] + a.beta[n0 + tx];
      }
    }
    tile[r][tx] = v;
  }
  __syncthreads();
  for (int r = ty; r < 64; r += 4) {
    const int b = b0 + tx;
    if (b < a.B) dst[(size_t)(n0 + r) * a.Bp + b] = (AT)tile[tx][r];
  }
}

// X_T[j*D+i][b] = LN_e(E[w_{b,j}])[i] straight from the per-symbol table (X is a gather, so is its transpose)
template <typename AT>
__global__ __launch_bounds__(256) void embed_t_kernel(WinSrc ws, int B, int Bp, int T, int D, const AT *tab, AT *XT) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int bchunks = Bp / 8;
  if (t >= (size_t)T * D * bchunks) return;
  const int row = (int)(t / bchunks), b8 = (int)(t % bchunks) * 8;
  const int j = row / D, i = row - j * D;
  float v[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int b = b8 + q;
    v[q] = (b < B && stream_active(ws, b)) ? (float)tab[(size_t)stream_window(ws, b, T)[j] * D + i] : 0.0f;
  }
  st8<AT>(XT + (size_t)row * Bp + b8, v);
}

// ---------------------------------------------------------------------------------------------------
// row-wise backward passes (one workgroup per stream; a thread owns 8-wide chunks tid, tid+256, ...)
// ---------------------------------------------------------------------------------------------------
constexpr int kMaxChunks = 4;  // D_h <= 8192

// Eq. 10 backward: dnv = dH * psi'(nv), LN backward -> dV; dH_coarse = lambda_o dH; row part of d lambda_o.
template <typename AT>
__global__ __launch_bounds__(256) void bwd_out_kernel(BwdOutArgs a) {
  __shared__ float red[4];
  const int b = blockIdx.x, tid = threadIdx.x, nch = a.Dh / 8;
  float mean, rstd;
  moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd);
  const float lam = a.lam[0];
  const size_t base = (size_t)b * a.Dh;
  float dh[kMaxChunks][8], xh[kMaxChunks][8];
  float s1 = 0.0f, s2 = 0.0f, sl = 0.0f;
#pragma unroll
  for (int q = 0; q < kMaxChunks; ++q) {
    const int ch = q * 256 + tid;
    if (ch < nch) {
      float dH[8], v[8], hc[8], ga[8], be[8], dnv[8], dhc[8];
      ld8<AT>(static_cast<const AT *>(a.dH) + base + ch * 8, dH);
      ld8<AT>(static_cast<const AT *>(a.V) + base + ch * 8, v);
      ld8<AT>(static_cast<const AT *>(a.Hc) + base + ch * 8, hc);
      ld8<float>(a.gamma + ch * 8, ga);
      ld8<float>(a.beta + ch * 8, be);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xh[q][i] = (v[i] - mean) * rstd;
        const float nv = xh[q][i] * ga[i] + be[i];
        dnv[i] = dH[i] * gelu_grad_f(nv);
        dh[q][i] = dnv[i] * ga[i];
        s1 += dh[q][i];
        s2 += dh[q][i] * xh[q][i];
        sl += dH[i] * hc[i];
        dhc[i] = lam * dH[i];
      }
      st8<AT>(static_cast<AT *>(a.dnv) + base + ch * 8, dnv);
      st8<AT>(static_cast<AT *>(a.dHc) + base + ch * 8, dhc);
    }
  }
  const float m1 = block_sum(s1, red) / (float)a.Dh, m2 = block_sum(s2, red) / (float)a.Dh;
  const float sumlam = block_sum(sl, red);
  if (tid == 0) a.row_dlam[b] = sumlam;
#pragma unroll
  for (int q = 0; q < kMaxChunks; ++q) {
    const int ch = q * 256 + tid;
    if (ch < nch) {
      float dv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) dv[i] = rstd * (dh[q][i] - m1 - xh[q][i] * m2);
      st8<AT>(static_cast<AT *>(a.dV) + base + ch * 8, dv);
    }
  }
}

// Eq. 9 backward (element-wise): d gate = dH_exp * value * psi'(gate), d value = dH_exp * psi(gate); written in the
// gate | value layout interleaved per 128 columns that the GeGLU weight pair uses as one operand.
template <typename AT>
__global__ __launch_bounds__(256) void bwd_geglu_kernel(int B, int De, const AT *dHexp, const AT *eg, const AT *ev, AT *dE) {
  const int chunks = De / 8;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)B * chunks) return;
  const int b = (int)(t / chunks), j8 = (int)(t % chunks) * 8;
  const int vg = (j8 / 64) * 128 + (j8 & 63), vv = vg + 64;
  float d[8], g[8], v[8], dg[8], dv[8];
  ld8<AT>(dHexp + (size_t)b * De + j8, d);
  ld8<AT>(eg + (size_t)b * De + j8, g);
  ld8<AT>(ev + (size_t)b * De + j8, v);
#pragma unroll
  for (int i = 0; i < 8; ++i) { dg[i] = d[i] * v[i] * gelu_grad_f(g[i]); dv[i] = d[i] * gelu_f(g[i]); }
  st8<AT>(dE + (size_t)b * 2 * De + vg, dg);
  st8<AT>(dE + (size_t)b * 2 * De + vv, dv);
}

// LN (Eq. 9) backward into dH_coarse, then Eq. 8 backward element-wise:
// dH_a = dHc * s, d(gate logits) = dHc * H_a * s (1 - s), dH_mix = lambda_c dHc, row part of d lambda_c.
template <typename AT>
__global__ __launch_bounds__(256) void bwd_gate_kernel(BwdGateArgs a) {
  __shared__ float red[4];
  const int b = blockIdx.x, tid = threadIdx.x, nch = a.Dh / 8;
  float mean, rstd;
  moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd);
  const float lam = a.lam[0];
  const size_t base = (size_t)b * a.Dh;
  float dh[kMaxChunks][8], xh[kMaxChunks][8];
  float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
  for (int q = 0; q < kMaxChunks; ++q) {
    const int ch = q * 256 + tid;
    if (ch < nch) {
      float du[8], hc[8], ga[8];
      ld8<AT>(static_cast<const AT *>(a.du) + base + ch * 8, du);
      ld8<AT>(static_cast<const AT *>(a.Hc) + base + ch * 8, hc);
      ld8<float>(a.gamma + ch * 8, ga);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xh[q][i] = (hc[i] - mean) * rstd;
        dh[q][i] = du[i] * ga[i];
        s1 += dh[q][i];
        s2 += dh[q][i] * xh[q][i];
      }
    }
  }
  const float m1 = block_sum(s1, red) / (float)a.Dh, m2 = block_sum(s2, red) / (float)a.Dh;
  float sl = 0.0f;
#pragma unroll
  for (int q = 0; q < kMaxChunks; ++q) {
    const int ch = q * 256 + tid;
    if (ch < nch) {
      float dhc[8], sg[8], ha[8], hm[8], dHa[8], dac[8], dmix[8];
      ld8<AT>(static_cast<const AT *>(a.dHc) + base + ch * 8, dhc);
      ld8<AT>(static_cast<const AT *>(a.sg) + base + ch * 8, sg);
      ld8<AT>(static_cast<const AT *>(a.Ha) + base + ch * 8, ha);
      ld8<AT>(static_cast<const AT *>(a.Hmix) + base + ch * 8, hm);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = dhc[i] + rstd * (dh[q][i] - m1 - xh[q][i] * m2);
        dHa[i] = d * sg[i];
        dac[i] = d * ha[i] * sg[i] * (1.0f - sg[i]);
        dmix[i] = lam * d;
        sl += d * hm[i];
      }
      st8<AT>(static_cast<AT *>(a.dHa) + base + ch * 8, dHa);
      st8<AT>(static_cast<AT *>(a.dac) + base + ch * 8, dac);
      st8<AT>(static_cast<AT *>(a.dHmix) + base + ch * 8, dmix);
    }
  }
  const float sumlam = block_sum(sl, red);
  if (tid == 0) a.row_dlam[b] = sumlam;
}

// LN (Eq. 7) backward into dH_mix (+ the gate path's contribution), then Eq. 5-6 and the branch activations:
// dHg = dmix a, dHl = dmix (1-a), d(router logits) = dmix (Hg - Hl) a (1-a), d(global pre-act) = dHg psi'(hm),
// d(conv pre-act) = dHl psi'(cv), dX = lambda_m dHg, row part of d lambda_m.
template <typename AT>
__global__ __launch_bounds__(256) void bwd_mix_kernel(BwdMixArgs a) {
  __shared__ float red[4];
  const int b = blockIdx.x, tid = threadIdx.x, nch = a.Dh / 8;
  float mean, rstd;
  moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd);
  const float lam = a.lam[0];
  const size_t base = (size_t)b * a.Dh;
  float dh[kMaxChunks][8], xh[kMaxChunks][8];
  float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
  for (int q = 0; q < kMaxChunks; ++q) {
    const int ch = q * 256 + tid;
    if (ch < nch) {
      float dn[8], hm[8], ga[8];
      ld8<AT>(static_cast<const AT *>(a.dnc) + base + ch * 8, dn);
      ld8<AT>(static_cast<const AT *>(a.Hmix) + base + ch * 8, hm);
      ld8<float>(a.gamma + ch * 8, ga);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xh[q][i] = (hm[i] - mean) * rstd;
        dh[q][i] = dn[i] * ga[i];
        s1 += dh[q][i];
        s2 += dh[q][i] * xh[q][i];
      }
    }
  }
  const float m1 = block_sum(s1, red) / (float)a.Dh, m2 = block_sum(s2, red) / (float)a.Dh;
  float sl = 0.0f;
#pragma unroll
  for (int q = 0; q < kMaxChunks; ++q) {
    const int ch = q * 256 + tid;
    if (ch < nch) {
      float d1[8], d2[8], al[8], hg[8], hl[8], pre_g[8], pre_c[8], x[8], dar[8], dhm[8], dcv[8], dX[8];
      ld8<AT>(static_cast<const AT *>(a.dHmix1) + base + ch * 8, d1);
      ld8<AT>(static_cast<const AT *>(a.dHmix2) + base + ch * 8, d2);
      ld8<AT>(static_cast<const AT *>(a.alpha) + base + ch * 8, al);
      ld8<AT>(static_cast<const AT *>(a.Hg) + base + ch * 8, hg);
      ld8<AT>(static_cast<const AT *>(a.Hl) + base + ch * 8, hl);
      ld8<AT>(static_cast<const AT *>(a.hm) + base + ch * 8, pre_g);
      ld8<AT>(static_cast<const AT *>(a.cv) + base + ch * 8, pre_c);
      ld8<AT>(static_cast<const AT *>(a.X) + base + ch * 8, x);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = d1[i] + d2[i] + rstd * (dh[q][i] - m1 - xh[q][i] * m2);
        const float dHg = d * al[i], dHl = d * (1.0f - al[i]);
        dar[i] = d * (hg[i] - hl[i]) * al[i] * (1.0f - al[i]);
        dhm[i] = dHg * gelu_grad_f(pre_g[i]);
        dcv[i] = dHl * gelu_grad_f(pre_c[i]);
        dX[i] = lam * dHg;
        sl += dHg * x[i];
      }
      st8<AT>(static_cast<AT *>(a.dar) + base + ch * 8, dar);
      st8<AT>(static_cast<AT *>(a.dhm) + base + ch * 8, dhm);
      st8<AT>(static_cast<AT *>(a.dcv) + base + ch * 8, dcv);
      st8<AT>(static_cast<AT *>(a.dX) + base + ch * 8, dX);
    }
  }
  const float sumlam = block_sum(sl, red);
  if (tid == 0) a.row_dlam[b] = sumlam;
}

// d gamma[n] = sum_b dn[b][n] * xhat[b][n], d beta[n] = sum_b dn[b][n] for a row LayerNorm over `width` columns.
// One workgroup per 64 columns; four row phases, each summing its rows in increasing order, combined in phase order.
template <typename AT>
__global__ __launch_bounds__(256) void ln_param_grad_kernel(int B, int width, int stats_n, const AT *dn, const AT *x, const float *stats,
                                                            float *dgamma, float *dbeta) {
  __shared__ float pg[4][64], pb[4][64];
  const int n = blockIdx.x * 64 + (threadIdx.x & 63), ph = threadIdx.x >> 6;
  float sg = 0.0f, sb = 0.0f;
  for (int b = ph; b < B; b += 4) {
    float mean, rstd;
    moments(stats + (size_t)b * stats_n * 2, stats_n, width, mean, rstd);
    const float d = (float)dn[(size_t)b * width + n];
    sg += d * ((float)x[(size_t)b * width + n] - mean) * rstd;
    sb += d;
  }
  pg[ph][threadIdx.x & 63] = sg;
  pb[ph][threadIdx.x & 63] = sb;
  __syncthreads();
  if (ph == 0) {
    const int c = threadIdx.x;
    dgamma[n] = (pg[0][c] + pg[1][c]) + (pg[2][c] + pg[3][c]);
    dbeta[n] = (pb[0][c] + pb[1][c]) + (pb[2][c] + pb[3][c]);
  }
}

// out[n] = sum_b src[b][n] (bias gradients). Same structure as above.
template <typename AT>
__global__ __launch_bounds__(256) void colsum_kernel(int B, int N, const AT *src, float *out) {
  __shared__ float ps[4][64];
  const int n = blockIdx.x * 64 + (threadIdx.x & 63), ph = threadIdx.x >> 6;
  float s = 0.0f;
  for (int b = ph; b < B; b += 4) s += (float)src[(size_t)b * N + n];
  ps[ph][threadIdx.x & 63] = s;
  __syncthreads();
  if (ph == 0) out[n] = (ps[0][threadIdx.x] + ps[1][threadIdx.x]) + (ps[2][threadIdx.x] + ps[3][threadIdx.x]);
}

// Sum per-row partials [B] into one scalar each (the three residual scales). One workgroup, fixed order.
__global__ __launch_bounds__(256) void scalar_sums_kernel(int B, const float *r0, const float *r1, const float *r2, float *o0, float *o1,
                                                          float *o2) {
  __shared__ float red[4];
  const float *rs[3] = {r0, r1, r2};
  float *os[3] = {o0, o1, o2};
  for (int k = 0; k < 3; ++k) {
    float s = 0.0f;
    for (int b = threadIdx.x; b < B; b += 256) s += rs[k][b];
    const float tot = block_sum(s, red);
    if (threadIdx.x == 0) os[k][0] = tot;
  }
}

// ---------------------------------------------------------------------------------------------------
// Eq. 7's per-stream memory, backward + its own Adam step (one wavefront per stream, d_low = 64):
//   dz = sum of split partials; dy[k] = sum_n W_U[b][k][n] dz[n]; grad W_U[b][k][n] = y[k] dz[n].
// The gradient is consumed on the spot by Adam (master, moments, compute copy), so it never goes to memory.
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void bwd_cci_kernel(BwdCciArgs a) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= a.B) return;
  float dz = 0.0f;
  for (int s = 0; s < a.splits; ++s) dz += a.dz_part[((size_t)s * a.B + b) * 64 + lane];
  const float yv = a.y[(size_t)b * 64 + lane];
  const AT *Wc = static_cast<const AT *>(a.WU_c) + (size_t)b * 4096;
  // dy[lane] = row `lane` of W_U[b] dot dz: walk the columns, broadcasting dz
  float dy = 0.0f;
  for (int n = 0; n < 64; ++n) dy = fmaf((float)Wc[lane * 64 + n], __shfl(dz, n, 64), dy);
  a.dy[(size_t)b * 64 + lane] = dy;
  static_cast<AT *>(a.dy_at)[(size_t)b * 64 + lane] = (AT)dy;
  const UpdateState u = *a.u;
  if (u.na == 0) return;
  // Adam on slice b: lane owns column `lane`, rows k = 0..63
  float *master = a.master + (size_t)b * 4096, *m = a.m + (size_t)b * 4096, *v = a.v + (size_t)b * 4096;
  AT *Wo = static_cast<AT *>(a.WU_c) + (size_t)b * 4096;
  for (int k = 0; k < 64; ++k) {
    const int idx = k * 64 + lane;
    const float g = __shfl(yv, k, 64) * dz;
    const float mk = a.beta1 * m[idx] + (1.0f - a.beta1) * g;
    const float vk = a.beta2 * v[idx] + (1.0f - a.beta2) * g * g;
    m[idx] = mk;
    v[idx] = vk;
    const float w = master[idx] - a.lr * (mk / u.c1) / (sqrtf(vk / u.c2) + a.eps);
    master[idx] = w;
    Wo[idx] = (AT)w;
  }
}

// ---------------------------------------------------------------------------------------------------
// Eq. 1-3 backward through the newest cache slot (one workgroup per stream):
//   dg[q] = sum_n d(hm)[n] W_m[Dc-c+q][n];  d gg = dg gv psi'(gg);  d gv = dg psi(gg);  dxt = W_g d gg + W_v d gv
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void bwd_slot_kernel(BwdSlotArgs a) {
  __shared__ float red[4];
  __shared__ float dgg_s[64], dgv_s[64];
  const int b = blockIdx.x, tid = threadIdx.x;
  const AT *dhm = static_cast<const AT *>(a.dhm) + (size_t)b * a.Dh;
  for (int q = 0; q < a.c; ++q) {
    const float *wrow = a.Wm + (size_t)(a.Dc - a.c + q) * a.Dh;
    float s = 0.0f;
    for (int n = tid; n < a.Dh; n += 256) {
      float w = wrow[n];
      if (a.round_bf16) w = (float)(bf16_t)w;
      s = fmaf((float)dhm[n], w, s);
    }
    const float dg = block_sum(s, red);
    if (tid == 0) {
      const float gg = a.GG[(size_t)b * a.c + q], gv = a.GV[(size_t)b * a.c + q];
      dgg_s[q] = dg * gv * gelu_grad_f(gg);
      dgv_s[q] = dg * gelu_f(gg);
      a.dgg[(size_t)b * a.c + q] = dgg_s[q];
      a.dgv[(size_t)b * a.c + q] = dgv_s[q];
    }
  }
  __syncthreads();
  if (tid < a.D) {
    float s = 0.0f;
    for (int q = 0; q < a.c; ++q) s += a.Wg[tid * a.c + q] * dgg_s[q] + a.Wv[tid * a.c + q] * dgv_s[q];
    a.dxt[(size_t)b * a.D + tid] = s;
  }
}

// dW_g[i][q] = sum_b xt[b][i] d gg[b][q] (same for W_v): one thread per output, batch in increasing order.
__global__ void slot_weight_grad_kernel(WinSrc ws, int B, int T, int D, int c, const float *tabXe32, const float *dgg, const float *dgv,
                                        float *dWg, float *dWv) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= D * c) return;
  const int i = t / c, q = t - i * c;
  float sg = 0.0f, sv = 0.0f;
  for (int b = 0; b < B; ++b) {
    if (!stream_active(ws, b)) continue;
    const float xt = tabXe32[(size_t)stream_window(ws, b, T)[T - 1] * D + i];
    sg = fmaf(xt, dgg[(size_t)b * c + q], sg);
    sv = fmaf(xt, dgv[(size_t)b * c + q], sv);
  }
  dWg[t] = sg;
  dWv[t] = sv;
}

// ---------------------------------------------------------------------------------------------------
// Eq. 4's weight gradient: dW_conv[r][i][o] = sum over tokens (b, j) of xl[b][j-(k-1)+r][i] * dcv[b][j][o] and
// db_conv[o] = sum dcv. Stage 1: each workgroup reduces its slice of tokens into a partial [taps*D + 1][D];
// stage 2 adds the partials in workgroup order.
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void conv_grad_partial_kernel(ConvGradArgs a) {
  const int tid = threadIdx.x;
  const int rows = a.taps * a.D;                  // (tap, i) pairs
  const int o = tid % a.D, grp = tid / a.D, ngrp = 256 / a.D;
  const int per = (rows + ngrp - 1) / ngrp;       // (tap, i) rows owned by this thread's group (<= 16)
  float acc[16], bsum = 0.0f;
#pragma unroll
  for (int q = 0; q < 16; ++q) acc[q] = 0.0f;
  const long long tokens = (long long)a.B * a.T;
  const long long per_blk = (tokens + gridDim.x - 1) / gridDim.x;
  const long long t0 = (long long)blockIdx.x * per_blk, t1 = (t0 + per_blk < tokens) ? t0 + per_blk : tokens;
  const AT *XL = static_cast<const AT *>(a.XL), *dcv = static_cast<const AT *>(a.dcv);
  for (long long t = t0; t < t1; ++t) {
    const int b = (int)(t / a.T), j = (int)(t - (long long)b * a.T);
    const float d = (float)dcv[(size_t)t * a.D + o];
    if (grp == 0) bsum += d;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int r = grp * per + q;
      if (q < per && r < rows) {
        const int tap = r / a.D, i = r - tap * a.D, tok = j - (a.taps - 1) + tap;
        if (tok >= 0) acc[q] = fmaf((float)XL[((size_t)b * a.T + tok) * a.D + i], d, acc[q]);
      }
    }
  }
  float *part = a.part + (size_t)blockIdx.x * (rows + 1) * a.D;
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int r = grp * per + q;
    if (q < per && r < rows) part[(size_t)r * a.D + o] = acc[q];
  }
  if (grp == 0) part[(size_t)rows * a.D + o] = bsum;
}
__global__ void conv_grad_reduce_kernel(int nblk, int rows, int D, const float *part, float *dW, float *db) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (rows + 1) * D) return;
  float s = 0.0f;
  for (int k = 0; k < nblk; ++k) s += part[(size_t)k * (rows + 1) * D + t];
  if (t < rows * D) dW[t] = s;
  else db[t - rows * D] = s;
}

// ---------------------------------------------------------------------------------------------------
// the two per-token LayerNorms backward -> d(embedding row) per token, plus their gain / shift gradients
// de[t][:] (fp32) for token t = (b, j); per-workgroup partial sums of d gamma / d beta, reduced afterwards.
// One thread per token; a wavefront handles 64 tokens.
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void bwd_token_kernel(BwdTokenArgs a) {
  __shared__ float red[4];
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x, tokens = (long long)a.B * a.T;
  const int D = a.D;
  float pge = 0.0f, pbe = 0.0f, pgl = 0.0f, pbl = 0.0f;  // this thread's contribution for the column handled below
  // pass 1: de rows
  if (t < tokens) {
    const int b = (int)(t / a.T), j = (int)(t - (long long)b * a.T);
    const bool act = stream_active(a.ws, b);
    const int s = act ? stream_window(a.ws, b, a.T)[j] : 0;
    const float *xh = a.tabXhat + (size_t)s * D;
    const float rstd = a.tabRstd[s];
    const AT *dX1 = static_cast<const AT *>(a.dX1) + (size_t)t * D, *dX2 = static_cast<const AT *>(a.dX2) + (size_t)t * D;
    const AT *dxl = static_cast<const AT *>(a.dxl) + (size_t)t * D;
    float m1e = 0.0f, m2e = 0.0f, m1l = 0.0f, m2l = 0.0f;
    for (int i = 0; i < D; ++i) {
      float de = (float)dX1[i] + (float)dX2[i];
      if (j == a.T - 1) de += a.dxt[(size_t)b * D + i];
      const float dhe = de * a.gamma_e[i], dhl = (float)dxl[i] * a.gamma_l[i];
      m1e += dhe; m2e += dhe * xh[i];
      m1l += dhl; m2l += dhl * xh[i];
    }
    m1e /= (float)D; m2e /= (float)D; m1l /= (float)D; m2l /= (float)D;
    float *out = a.de + (size_t)t * D;
    for (int i = 0; i < D; ++i) {
      float de = (float)dX1[i] + (float)dX2[i];
      if (j == a.T - 1) de += a.dxt[(size_t)b * D + i];
      const float dhe = de * a.gamma_e[i], dhl = (float)dxl[i] * a.gamma_l[i];
      out[i] = act ? rstd * ((dhe - m1e - xh[i] * m2e) + (dhl - m1l - xh[i] * m2l)) : 0.0f;
    }
  }
  // pass 2: column sums over this workgroup's 256 tokens for d gamma_e, d beta_e, d gamma_l, d beta_l
  for (int i = 0; i < D; ++i) {
    pge = pbe = pgl = pbl = 0.0f;
    if (t < tokens) {
      const int b = (int)(t / a.T), j = (int)(t - (long long)b * a.T);
      if (stream_active(a.ws, b)) {
        const int s = stream_window(a.ws, b, a.T)[j];
        const float xh = a.tabXhat[(size_t)s * D + i];
        float de = (float)static_cast<const AT *>(a.dX1)[(size_t)t * D + i] + (float)static_cast<const AT *>(a.dX2)[(size_t)t * D + i];
        if (j == a.T - 1) de += a.dxt[(size_t)b * D + i];
        const float dl = (float)static_cast<const AT *>(a.dxl)[(size_t)t * D + i];
        pge = de * xh; pbe = de; pgl = dl * xh; pbl = dl;
      }
    }
    const float s0 = block_sum(pge, red), s1 = block_sum(pbe, red), s2 = block_sum(pgl, red), s3 = block_sum(pbl, red);
    if (threadIdx.x == 0) {
      float *p = a.part + ((size_t)blockIdx.x * 4) * D;
      p[i] = s0; p[D + i] = s1; p[2 * D + i] = s2; p[3 * D + i] = s3;
    }
  }
}
__global__ void token_param_reduce_kernel(int nblk, int D, const float *part, float *dge, float *dbe, float *dgl, float *dbl) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= 4 * D) return;
  float s = 0.0f;
  for (int k = 0; k < nblk; ++k) s += part[(size_t)k * 4 * D + t];
  float *outs[4] = {dge, dbe, dgl, dbl};
  outs[t / D][t % D] = s;
}

// dE[s][:] = sum of de over the tokens whose symbol is s. One workgroup per symbol; eight token phases of D lanes,
// each phase walking its tokens in increasing order; phases combined in index order.
__global__ __launch_bounds__(256) void embed_grad_kernel(WinSrc ws, int B, int T, int D, const float *de, float *dE) {
  __shared__ float ps[256];
  const int s = blockIdx.x, i = threadIdx.x % D, ph = threadIdx.x / D, nph = 256 / D;
  float acc = 0.0f;
  for (int b = 0; b < B; ++b) {
    if (!stream_active(ws, b)) continue;
    const uint8_t *win = stream_window(ws, b, T);
    for (int j = ph; j < T; j += nph)
      if (win[j] == s) acc += de[((size_t)b * T + j) * D + i];
  }
  ps[threadIdx.x] = acc;
  __syncthreads();
  if (ph == 0) {
    float tot = 0.0f;
    for (int k = 0; k < nph; ++k) tot += ps[k * D + i];
    dE[(size_t)s * D + i] = tot;
  }
}

// ---------------------------------------------------------------------------------------------------
// Adam (bias-corrected, no weight decay) on a range of the blob
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void adam_kernel(size_t n, const float *grad, float *master, float *m, float *v, const UpdateState *u,
                                                   float lr, float beta1, float beta2, float eps) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= n) return;
  const UpdateState us = *u;
  if (us.na == 0) return;
  const float g = grad[t];
  const float mk = beta1 * m[t] + (1.0f - beta1) * g;
  const float vk = beta2 * v[t] + (1.0f - beta2) * g * g;
  m[t] = mk;
  v[t] = vk;
  master[t] = master[t] - lr * (mk / us.c1) / (sqrtf(vk / us.c2) + eps);
}

inline unsigned nblk(size_t n, unsigned per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

#define DISPATCH_AT(bf16, KERNEL, grid, block, stream, ...)                                       \
  do {                                                                                            \
    if (bf16) hipLaunchKernelGGL((KERNEL<bf16_t>), grid, block, 0, stream, __VA_ARGS__);          \
    else hipLaunchKernelGGL((KERNEL<float>), grid, block, 0, stream, __VA_ARGS__);                \
    return hipGetLastError();                                                                     \
  } while (0)

hipError_t fade_update_prep(const WinSrc &ws, int B, UpdateState *u, float beta1, float beta2, hipStream_t s) {
  hipLaunchKernelGGL(update_prep_kernel, dim3(1), dim3(256), 0, s, ws, B, u, beta1, beta2);
  return hipGetLastError();
}
hipError_t fade_dlogits(const WinSrc &ws, const uint8_t *targets, long long tstride, int B, const float *probs, const UpdateState *u,
                        void *dl, bool bf16, hipStream_t s) {
  if (bf16) hipLaunchKernelGGL(dlogits_kernel<bf16_t>, dim3((B + 3) / 4), dim3(256), 0, s, ws, targets, tstride, B, probs, u, static_cast<bf16_t *>(dl));
  else hipLaunchKernelGGL(dlogits_kernel<float>, dim3((B + 3) / 4), dim3(256), 0, s, ws, targets, tstride, B, probs, u, static_cast<float *>(dl));
  return hipGetLastError();
}
hipError_t fade_transpose(const TransposeArgs &a, int N, bool bf16, hipStream_t s) {
  if (N % 64) return hipErrorInvalidValue;
  DISPATCH_AT(bf16, transpose_kernel, dim3((a.B + 63) / 64, N / 64), dim3(256), s, a);
}
hipError_t fade_embed_t(const WinSrc &ws, int B, int Bp, int T, int D, const void *tab, void *XT, bool bf16, hipStream_t s) {
  const size_t n = (size_t)T * D * (Bp / 8);
  if (bf16) hipLaunchKernelGGL(embed_t_kernel<bf16_t>, dim3(nblk(n, 256)), dim3(256), 0, s, ws, B, Bp, T, D, static_cast<const bf16_t *>(tab), static_cast<bf16_t *>(XT));
  else hipLaunchKernelGGL(embed_t_kernel<float>, dim3(nblk(n, 256)), dim3(256), 0, s, ws, B, Bp, T, D, static_cast<const float *>(tab), static_cast<float *>(XT));
  return hipGetLastError();
}
hipError_t fade_bwd_out(const BwdOutArgs &a, int B, bool bf16, hipStream_t s) { DISPATCH_AT(bf16, bwd_out_kernel, dim3(B), dim3(256), s, a); }
hipError_t fade_bwd_geglu(int B, int De, const void *dHexp, const void *eg, const void *ev, void *dE, bool bf16, hipStream_t s) {
  const size_t n = (size_t)B * (De / 8);
  if (bf16) hipLaunchKernelGGL(bwd_geglu_kernel<bf16_t>, dim3(nblk(n, 256)), dim3(256), 0, s, B, De, static_cast<const bf16_t *>(dHexp), static_cast<const bf16_t *>(eg), static_cast<const bf16_t *>(ev), static_cast<bf16_t *>(dE));
  else hipLaunchKernelGGL(bwd_geglu_kernel<float>, dim3(nblk(n, 256)), dim3(256), 0, s, B, De, static_cast<const float *>(dHexp), static_cast<const float *>(eg), static_cast<const float *>(ev), static_cast<float *>(dE));
  return hipGetLastError();
}
hipError_t fade_bwd_gate(const BwdGateArgs &a, int B, bool bf16, hipStream_t s) { DISPATCH_AT(bf16, bwd_gate_kernel, dim3(B), dim3(256), s, a); }
hipError_t fade_bwd_mix(const BwdMixArgs &a, int B, bool bf16, hipStream_t s) { DISPATCH_AT(bf16, bwd_mix_kernel, dim3(B), dim3(256), s, a); }
hipError_t fade_ln_param_grad(int B, int width, int stats_n, const void *dn, const void *x, const float *stats, float *dgamma, float *dbeta,
                              bool bf16, hipStream_t s) {
  if (width % 64) return hipErrorInvalidValue;
  if (bf16) hipLaunchKernelGGL(ln_param_grad_kernel<bf16_t>, dim3(width / 64), dim3(256), 0, s, B, width, stats_n, static_cast<const bf16_t *>(dn), static_cast<const bf16_t *>(x), stats, dgamma, dbeta);
  else hipLaunchKernelGGL(ln_param_grad_kernel<float>, dim3(width / 64), dim3(256), 0, s, B, width, stats_n, static_cast<const float *>(dn), static_cast<const float *>(x), stats, dgamma, dbeta);
  return hipGetLastError();
}
hipError_t fade_colsum(int B, int N, const void *src, float *out, bool bf16, hipStream_t s) {
  if (N % 64) return hipErrorInvalidValue;
  if (bf16) hipLaunchKernelGGL(colsum_kernel<bf16_t>, dim3(N / 64), dim3(256), 0, s, B, N, static_cast<const bf16_t *>(src), out);
  else hipLaunchKernelGGL(colsum_kernel<float>, dim3(N / 64), dim3(256), 0, s, B, N, static_cast<const float *>(src), out);
  return hipGetLastError();
}
hipError_t fade_scalar_sums(int B, const float *r0, const float *r1, const float *r2, float *o0, float *o1, float *o2, hipStream_t s) {
  hipLaunchKernelGGL(scalar_sums_kernel, dim3(1), dim3(256), 0, s, B, r0, r1, r2, o0, o1, o2);
  return hipGetLastError();
}
hipError_t fade_bwd_cci(const BwdCciArgs &a, bool bf16, hipStream_t s) { DISPATCH_AT(bf16, bwd_cci_kernel, dim3((a.B + 3) / 4), dim3(256), s, a); }
hipError_t fade_bwd_slot(const BwdSlotArgs &a, int B, bool bf16, hipStream_t s) { DISPATCH_AT(bf16, bwd_slot_kernel, dim3(B), dim3(256), s, a); }
hipError_t fade_slot_weight_grad(const WinSrc &ws, int B, int T, int D, int c, const float *tabXe32, const float *dgg, const float *dgv,
                                 float *dWg, float *dWv, hipStream_t s) {
  hipLaunchKernelGGL(slot_weight_grad_kernel, dim3(nblk((size_t)D * c, 64)), dim3(64), 0, s, ws, B, T, D, c, tabXe32, dgg, dgv, dWg, dWv);
  return hipGetLastError();
}
hipError_t fade_conv_grad(const ConvGradArgs &a, int nblocks, float *dW, float *db, bool bf16, hipStream_t s) {
  if (256 % a.D || (a.taps * a.D + 256 / a.D - 1) / (256 / a.D) > 16) return hipErrorInvalidValue;
  if (bf16) hipLaunchKernelGGL(conv_grad_partial_kernel<bf16_t>, dim3(nblocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(conv_grad_partial_kernel<float>, dim3(nblocks), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rows = a.taps * a.D;
  hipLaunchKernelGGL(conv_grad_reduce_kernel, dim3(nblk((size_t)(rows + 1) * a.D, 256)), dim3(256), 0, s, nblocks, rows, a.D, a.part, dW, db);
  return hipGetLastError();
}
hipError_t fade_bwd_token(const BwdTokenArgs &a, float *dge, float *dbe, float *dgl, float *dbl, bool bf16, hipStream_t s) {
  const int blocks = (int)(((long long)a.B * a.T + 255) / 256);
  if (bf16) hipLaunchKernelGGL(bwd_token_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(bwd_token_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(token_param_reduce_kernel, dim3(nblk((size_t)4 * a.D, 64)), dim3(64), 0, s, blocks, a.D, a.part, dge, dbe, dgl, dbl);
  return hipGetLastError();
}
hipError_t fade_embed_grad(const WinSrc &ws, int B, int T, int D, const float *de, float *dE, hipStream_t s) {
  if (256 % D) return hipErrorInvalidValue;
  hipLaunchKernelGGL(embed_grad_kernel, dim3(256), dim3(256), 0, s, ws, B, T, D, de, dE);
  return hipGetLastError();
}
hipError_t fade_adam(size_t n, const float *grad, float *master, float *m, float *v, const UpdateState *u, float lr, float beta1, float beta2,
                     float eps, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(adam_kernel, dim3(nblk(n, 256)), dim3(256), 0, s, n, grad, master, m, v, u, lr, beta1, beta2, eps);
  return hipGetLastError();
}
