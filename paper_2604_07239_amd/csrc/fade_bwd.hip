// fade_bwd.hip — the online update's non-GEMM kernels: loss gradient, LayerNorm / activation backward passes,
// batch-transposed operand copies for the weight-gradient products, per-stream memory backward + its Adam,
// conv / embedding gradients, parameter reductions and Adam (Algorithm 1's "backpropagate to update P"; loss Eq. 12).
// All reductions run in a fixed order (no atomics): encoder and decoder must reproduce the same weights bit for bit.
#include "fade_dev.h"
#include "fade_kernels.h"
#include <cstdlib>

namespace {

__device__ __forceinline__ float gelu_f(float x) { return fade_gelu(x); }
__device__ __forceinline__ float gelu_grad_f(float x) { return fade_gelu_grad(x); }

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

// 8 values as loaded (no conversion: nothing waits for the load until cvt() is called)
template <typename AT> struct Raw8B;
template <> struct Raw8B<bf16_t> {
  bf16x8 r;
  __device__ __forceinline__ void load(const bf16_t *p) { r = *reinterpret_cast<const bf16x8 *>(p); }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (bf16_t)0.0f;
  }
  __device__ __forceinline__ void cvt(float v[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)r[i];
  }
};
template <> struct Raw8B<float> {
  f32x4 a, b;
  __device__ __forceinline__ void load(const float *p) { a = *reinterpret_cast<const f32x4 *>(p); b = *reinterpret_cast<const f32x4 *>(p + 4); }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = 0.0f; b[i] = 0.0f; }
  }
  __device__ __forceinline__ void cvt(float v[8]) const {
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
};

__device__ __forceinline__ void moments(const float *stats, int stats_n, int width, float &mean, float &rstd) {
  fade_row_moments(stats, stats_n, width, mean, rstd);
}

// One Adam step (bias-corrected, no weight decay) on element idx of the blob, given its gradient; returns the new weight.
__device__ __forceinline__ float adam_element(const AdamArrays &o, size_t idx, float g) {
  const UpdateState us = *o.u;
  if (us.na == 0) return o.master[idx];  // no active stream: no update
  const float mk = o.beta1 * o.m[idx] + (1.0f - o.beta1) * g;
  const float vk = o.beta2 * o.v[idx] + (1.0f - o.beta2) * g * g;
  o.m[idx] = mk;
  o.v[idx] = vk;
  const float w = o.master[idx] - o.lr * (mk / us.c1) / (sqrtf(vk / us.c2) + o.eps);
  o.master[idx] = w;
  return w;
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
// Start of the update, one launch: the number of active streams (every workgroup counts for itself), Adam's step count
// and bias corrections (workgroup 0 records them for the kernels that follow), the loss gradient
//   dlogits = (p - onehot(target)) / n_active for active streams, 0 otherwise   (gradient of the mean NLL, Eq. 12)
// and the first stage of db_o (column sums over this workgroup's 8 streams). Thread = one of the 256 symbols.
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__device__ __forceinline__ void loss_grad_body(int block, const WinSrc &ws, const uint8_t *targets, long long tstride, int B, const float *probs,
                                               UpdateState *u, float beta1, float beta2, AT *dl, float *col_part) {
  __shared__ int cnt[4];
  const int tid = threadIdx.x;
  int mine = 0;
  for (int b = tid; b < B; b += 256) mine += stream_active(ws, b) ? 1 : 0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
  if ((tid & 63) == 0) cnt[tid >> 6] = mine;
  __syncthreads();
  const int na = cnt[0] + cnt[1] + cnt[2] + cnt[3];
  const float sc = na > 0 ? 1.0f / (float)na : 0.0f;
  if (block == 0 && tid == 0) {
    u->na = na;
    if (na > 0) {
      u->t += 1;
      u->c1 = 1.0f - powf(beta1, (float)u->t);
      u->c2 = 1.0f - powf(beta2, (float)u->t);
      u->inv_na = sc;
    }
  }
  const int b0 = block * 8;
  float colsum = 0.0f;
  // targets and flags of the 8 streams first, then the probabilities (all loads in flight together)
  float p[8];
  int x[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int b = b0 + r;
    const bool act = b < B && stream_active(ws, b);
    x[r] = act ? (int)targets[(long long)b * tstride] : -1;
    p[r] = b < B ? probs[(size_t)b * 256 + tid] : 0.0f;
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int b = b0 + r;
    if (b >= B) break;
    const float g = x[r] >= 0 ? sc * (p[r] - (tid == x[r] ? 1.0f : 0.0f)) : 0.0f;
    const AT gq = (AT)g;
    dl[(size_t)b * 256 + tid] = gq;
    colsum += (float)gq;  // db_o is the column sum of the gradient the products see
  }
  col_part[(size_t)block * 256 + tid] = colsum;
}

template <typename AT>
__global__ __launch_bounds__(256) void loss_grad_kernel(WinSrc ws, const uint8_t *targets, long long tstride, int B, const float *probs,
                                                        UpdateState *u, float beta1, float beta2, AT *dl, float *col_part) {
  loss_grad_body<AT>(blockIdx.x, ws, targets, tstride, B, probs, u, beta1, beta2, dl, col_part);
}

// ---------------------------------------------------------------------------------------------------
// batch-major -> feature-major copies: dst[n][b] = f(src[b][n]) for the weight-gradient products, which reduce over
// the batch and therefore need batch-contiguous operands. Optional LayerNorm on the way (u = LN(H_coarse), LN(H_mix)).
// 64 x 64 tiles through LDS; dst has leading dimension Bp (batch rounded up to 64, padding stays zero).
// ---------------------------------------------------------------------------------------------------
// One 64 x 64 tile: 16-byte (bf16) / 32-byte (fp32) pieces on both the read and the write side, the turn happens in LDS
// (pitch 65 floats: the piece-wise row writes and the column reads both touch all 64 banks).
template <typename AT>
__device__ __forceinline__ void transpose_tile(const TransposeArgs &a, int b0, int n0, float (*tile)[65], float *mr /*[2][64]*/) {
  const AT *src = static_cast<const AT *>(a.src);
  AT *dst = static_cast<AT *>(a.dst);
  const int tid = threadIdx.x;
  if (a.stats) {
    if (tid < 64) {
      float mean = 0.0f, rstd = 0.0f;
      if (b0 + tid < a.B) moments(a.stats + (size_t)(b0 + tid) * a.stats_n * 2, a.stats_n, a.width, mean, rstd);
      mr[tid] = mean; mr[64 + tid] = rstd;
    }
    __syncthreads();
  }
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int q = tid + 256 * p, r = q >> 3, c8 = (q & 7) * 8, b = b0 + r;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = 0.0f;
    if (b < a.B) {
      ld8<AT>(src + (size_t)b * a.ld + n0 + c8, v);
      if (a.stats) {
        const float mean = mr[r], rstd = mr[64 + r];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (v[i] - mean) * rstd * a.gamma[n0 + c8 + i] + a.beta[n0 + c8 + i];  // blob vectors: dword-aligned only
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) tile[r][c8 + i] = v[i];
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int q = tid + 256 * p, n = q >> 3, bc = (q & 7) * 8;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = tile[bc + i][n];
    st8<AT>(dst + (size_t)(n0 + n) * a.Bp + b0 + bc, v);  // rows past B were staged as zeros: the padding stays zero
  }
}

template <typename AT>
__global__ __launch_bounds__(256) void transpose_kernel(TransposeArgs a) {
  __shared__ float tile[64][65];
  __shared__ float mr[128];
  transpose_tile<AT>(a, blockIdx.x * 64, blockIdx.y * 64, tile, mr);
}

template <typename AT>
__global__ __launch_bounds__(256) void transpose_batch_kernel(TransposeBatch tb) {
  __shared__ float tile[64][65];
  __shared__ float mr[128];
  const TransposeArgs &a = tb.t[blockIdx.z];
  const int b0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  if (b0 >= a.B || n0 >= tb.N[blockIdx.z]) return;  // uniform over the workgroup
  transpose_tile<AT>(a, b0, n0, tile, mr);
}

template <typename AT, int RPT>
__global__ __launch_bounds__(256) void ln_apply_kernel(LnApplyBatch lb) {
  if ((int)blockIdx.y == lb.count) {  // the loss gradient's workgroups (with_loss)
    const LossGradArgs &l = lb.loss;
    if ((int)blockIdx.x < (lb.B + 7) / 8)
      loss_grad_body<AT>(blockIdx.x, l.ws, l.targets, l.tstride, lb.B, l.probs, l.u, l.beta1, l.beta2, static_cast<AT *>(l.dl), l.col_part);
    return;
  }
  __shared__ float mom[FADE_GROUP_ROWS_MAX][2];
  const LnApplyArgs &a = lb.a[blockIdx.y];
  const int chunks = lb.Dh / 8;
  const int r0 = fade_group_moments<RPT>(a.stats, lb.stats_n, lb.Dh, chunks, lb.B, mom);
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)((lb.B + RPT - 1) / RPT) * chunks) return;
  const int b0 = (int)(t / chunks) * RPT, c8 = (int)(t % chunks) * 8;
  float v[RPT][8], ga[8], be[8];
#pragma unroll
  for (int i = 0; i < RPT; ++i)
    if (b0 + i < lb.B) ld8<AT>(static_cast<const AT *>(a.src) + (size_t)(b0 + i) * lb.Dh + c8, v[i]);
  ld8<float>(a.gamma + c8, ga);
  ld8<float>(a.beta + c8, be);
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    if (b0 + i >= lb.B) continue;
    const float mean = mom[b0 + i - r0][0], rstd = mom[b0 + i - r0][1];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[i][j] = (v[i][j] - mean) * rstd * ga[j] + be[j];
    st8<AT>(static_cast<AT *>(a.dst) + (size_t)(b0 + i) * lb.Dh + c8, v[i]);
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
// a thread of the row kernels owns one 8-wide chunk: D_h <= 2048
// Rows handled by one workgroup of the row kernels; its LayerNorm gain / shift partial sums cover those rows. Few rows per
// workgroup while the batch is small (more workgroups to hide the two dependent rounds of loads), four for large batches
// (fewer partial sums to write and add up). B = 1024: the three kernels 15.5 / 20.0 / 26.7 us with four rows, 13.7 / 14.8 /
// 21.3 with two (one row: 13.3 / 14.4 / 20.1, but 8 us more in the reduction of twice as many partial sums).
inline int env_int(const char *name) { const char *e = getenv(name); return e ? atoi(e) : 0; }
// Rows a workgroup of a row kernel takes through each phase together. Small batches: 2 (few workgroups, latency-bound);
// below 4096 rows: 4; from 4096 on: 1, where the lower register count (two more wavefronts per SIMD) is worth more than
// the shared reductions (B = 16384, with 16 row groups per workgroup: Eq. 10 / Eq. 8 / Eq. 5-6 backward 116 / 178 / 244 us
// with 4 rows, 95 / 136 / 213 with 1; B = 4096, 4 groups of 1 row against 1 group of 4: 26 / 44 / 78 against 30 / 47 / 82).
inline int rows_per_block(int B) {
  static const int r = env_int("FADE_ROWS_R");  // tuning override: 1, 2 or 4
  return (r == 1 || r == 2 || r == 4) ? r : (B <= 2048 ? 2 : B < 4096 ? 4 : 1);
}
// Row groups one workgroup of a row kernel walks through, adding the LayerNorm-gain partials of all of them in registers:
// at large batches this keeps the first-stage partial buffers (one row of 2 D_h floats per workgroup) small.
inline int row_groups(int B) {
  static const int g = env_int("FADE_ROWS_G");  // tuning override
  return g > 0 ? g : (B >= 8192 ? 16 : B >= 4096 ? 4 : 1);
}

// Several row sums at once over a 256-thread workgroup (same fixed order as block_sum); red holds 4 * N floats.
template <int N>
__device__ __forceinline__ void block_sum_n(float (&v)[N], float *red) {
#pragma unroll
  for (int k = 0; k < N; ++k) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v[k] += __shfl_xor(v[k], off, 64);
  }
  __syncthreads();  // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int k = 0; k < N; ++k) red[(threadIdx.x >> 6) * N + k] = v[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < N; ++k) v[k] = (red[k] + red[N + k]) + (red[2 * N + k] + red[3 * N + k]);
}

// The row kernels below take their R rows through each phase together (all loads of a phase in flight at once,
// one workgroup reduction per phase for all rows), not row after row: they are bound by memory latency, not by arithmetic.

// Eq. 10 backward: dnv = dH * psi'(nv), LN backward -> dV; dH_coarse = lambda_o dH; row part of d lambda_o.
template <typename AT, int R>
__global__ __launch_bounds__(256) void bwd_out_kernel(BwdOutArgs a) {
  __shared__ float red[4 * 3 * R];
  const int tid = threadIdx.x, nch = a.Dh / 8;
  const bool mine = tid < nch;
  const float lam = a.lam[0];
  float ga[8], be[8], pg[8], pb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { ga[i] = be[i] = pg[i] = pb[i] = 0.0f; }
  if (mine) { ld8<float>(a.gamma + tid * 8, ga); ld8<float>(a.beta + tid * 8, be); }
  float dh[R][8], xh[R][8], rstd[R], sums[3 * R];
  const int G = a.groups;
  for (int rb = blockIdx.x * G; rb < (int)blockIdx.x * G + G; ++rb) {
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int b = rb * R + r;
    float s1 = 0.0f, s2 = 0.0f, sl = 0.0f, mean = 0.0f;
    rstd[r] = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { dh[r][i] = 0.0f; xh[r][i] = 0.0f; }
    if (b < a.B && mine) {  // b < B is uniform over the workgroup
      // the row pieces are requested before the row's statistics are summed: one round trip, not two
      const size_t base = (size_t)b * a.Dh + tid * 8;
      float dH[8], v[8], hc[8], dhc[8];
      ld8<AT>(static_cast<const AT *>(a.dH) + base, dH);
      ld8<AT>(static_cast<const AT *>(a.V) + base, v);
      ld8<AT>(static_cast<const AT *>(a.Hc) + base, hc);
      moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd[r]);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xh[r][i] = (v[i] - mean) * rstd[r];
        const float nv = xh[r][i] * ga[i] + be[i];
        const float dnv = dH[i] * gelu_grad_f(nv);
        dh[r][i] = dnv * ga[i];
        s1 += dh[r][i];
        s2 += dh[r][i] * xh[r][i];
        sl += dH[i] * hc[i];
        dhc[i] = lam * dH[i];
        pg[i] += dnv * xh[r][i];
        pb[i] += dnv;
      }
      st8<AT>(static_cast<AT *>(a.dHc) + base, dhc);
    }
    sums[r] = s1; sums[R + r] = s2; sums[2 * R + r] = sl;
  }
  block_sum_n<3 * R>(sums, red);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int b = rb * R + r;
    if (b >= a.B) break;
    if (tid == 0) a.row_dlam[b] = sums[2 * R + r];
    if (mine) {
      const float m1 = sums[r] / (float)a.Dh, m2 = sums[R + r] / (float)a.Dh;
      float dv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) dv[i] = rstd[r] * (dh[r][i] - m1 - xh[r][i] * m2);
      st8<AT>(static_cast<AT *>(a.dV) + (size_t)b * a.Dh + tid * 8, dv);
    }
  }
  }
  if (mine) {
    float *p = a.ln_part + (size_t)blockIdx.x * 2 * a.Dh;
    st8<float>(p + tid * 8, pg);
    st8<float>(p + a.Dh + tid * 8, pb);
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
// Ablation levels: a.du == NULL: no refiner behind H_coarse, dHc arrives complete; a.sg == NULL: Eq. 8 without its gate.
template <typename AT, int R>
__global__ __launch_bounds__(256) void bwd_gate_kernel(BwdGateArgs a) {
  __shared__ float red[4 * 2 * R];
  const int tid = threadIdx.x, nch = a.Dh / 8;
  const bool mine = tid < nch;
  const float lam = a.lam[0];
  float ga[8], pg[8], pb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { ga[i] = pg[i] = pb[i] = 0.0f; }
  if (mine) ld8<float>(a.gamma + tid * 8, ga);
  float dh[R][8], xh[R][8], rstd[R], sums[2 * R], sl[R];
  const int G = a.groups;
  for (int rb = blockIdx.x * G; rb < (int)blockIdx.x * G + G; ++rb) {
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int b = rb * R + r;
    float s1 = 0.0f, s2 = 0.0f, mean = 0.0f;
    rstd[r] = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { dh[r][i] = 0.0f; xh[r][i] = 0.0f; }
    if (b < a.B && mine) {
      const size_t base = (size_t)b * a.Dh + tid * 8;
      float du[8], hc[8];
      ld8<AT>(static_cast<const AT *>(a.Hc) + base, hc);  // requested before the statistics are summed
      if (!a.du_part && a.du) ld8<AT>(static_cast<const AT *>(a.du) + base, du);
      moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd[r]);
      if (a.du_part || !a.du) {
#pragma unroll
        for (int i = 0; i < 8; ++i) du[i] = 0.0f;
      }
      if (a.du_part) {
        for (int sp = 0; sp < a.du_splits; ++sp) {
          float pv[8];
          ld8<float>(a.du_part + (size_t)sp * a.B * a.Dh + base, pv);
#pragma unroll
          for (int i = 0; i < 8; ++i) du[i] += pv[i];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) du[i] = (float)(AT)du[i];  // the value the unsplit product would have stored
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xh[r][i] = (hc[i] - mean) * rstd[r];
        dh[r][i] = du[i] * ga[i];
        s1 += dh[r][i];
        s2 += dh[r][i] * xh[r][i];
        pg[i] += du[i] * xh[r][i];
        pb[i] += du[i];
      }
    }
    sums[r] = s1; sums[R + r] = s2;
  }
  block_sum_n<2 * R>(sums, red);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int b = rb * R + r;
    sl[r] = 0.0f;
    if (b < a.B && mine) {
      const size_t base = (size_t)b * a.Dh + tid * 8;
      const float m1 = sums[r] / (float)a.Dh, m2 = sums[R + r] / (float)a.Dh;
      float dhc[8], sg[8], ha[8], hm[8], dHa[8], dac[8], dmix[8];
      ld8<AT>(static_cast<const AT *>(a.dHc) + base, dhc);
#pragma unroll
      for (int i = 0; i < 8; ++i) sg[i] = 1.0f;
      if (a.sg) ld8<AT>(static_cast<const AT *>(a.sg) + base, sg);
      ld8<AT>(static_cast<const AT *>(a.Ha) + base, ha);
      ld8<AT>(static_cast<const AT *>(a.Hmix) + base, hm);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = dhc[i] + rstd[r] * (dh[r][i] - m1 - xh[r][i] * m2);
        dHa[i] = d * sg[i];
        dac[i] = d * ha[i] * sg[i] * (1.0f - sg[i]);
        dmix[i] = lam * d;
        sl[r] += d * hm[i];
      }
      st8<AT>(static_cast<AT *>(a.dHa) + base, dHa);
      if (a.sg) st8<AT>(static_cast<AT *>(a.dac) + base, dac);
      st8<AT>(static_cast<AT *>(a.dHmix) + base, dmix);
    }
  }
  block_sum_n<R>(sl, red);
  if (tid == 0) {
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (rb * R + r < a.B) a.row_dlam[rb * R + r] = sl[r];
  }
  }
  if (mine) {
    float *p = a.ln_part + (size_t)blockIdx.x * 2 * a.Dh;
    st8<float>(p + tid * 8, pg);
    st8<float>(p + a.Dh + tid * 8, pb);
  }
}

// The two branch outputs are not read back: H_g = psi(hm) + lambda_m X and H_l = psi(cv) follow from the pre-activations
// and X, which the kernel reads anyway, and psi shares Phi and the Gaussian with psi' (two of ten row reads less).
// LN (Eq. 7) backward into dH_mix (+ the gate path's contribution), then Eq. 5-6 and the branch activations:
// dHg = dmix a, dHl = dmix (1-a), d(router logits) = dmix (Hg - Hl) a (1-a), d(global pre-act) = dHg psi'(hm),
// d(conv pre-act) = dHl psi'(cv), dX = lambda_m dHg, row part of d lambda_m.
// Ablation levels: a.dnc == NULL: nothing behind H_mix but what dHmix1 (+ dHmix2) carry; a.dHmix2 == NULL: no gate product;
// a.alpha == NULL: the global stream alone (alpha = 1: no local stream, no router), dar / dcv are not written.
template <typename AT, int R>
__global__ __launch_bounds__(256) void bwd_mix_kernel(BwdMixArgs a) {
  __shared__ float red[4 * 2 * R];
  const int tid = threadIdx.x, nch = a.Dh / 8;
  const bool mine = tid < nch;
  const float lam = a.lam[0];
  float ga[8], pg[8], pb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { ga[i] = pg[i] = pb[i] = 0.0f; }
  if (mine) ld8<float>(a.gamma + tid * 8, ga);
  float dh[R][8], xh[R][8], rstd[R], sums[2 * R], sl[R];
  const int G = a.groups;
  for (int rb = blockIdx.x * G; rb < (int)blockIdx.x * G + G; ++rb) {
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int b = rb * R + r;
    float s1 = 0.0f, s2 = 0.0f, mean = 0.0f;
    rstd[r] = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { dh[r][i] = 0.0f; xh[r][i] = 0.0f; }
    if (b < a.B && mine) {
      const size_t base = (size_t)b * a.Dh + tid * 8;
      float dn[8], hm[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { dn[i] = 0.0f; hm[i] = 0.0f; }
      if (a.dnc) {  // requested before the statistics are summed
        ld8<AT>(static_cast<const AT *>(a.dnc) + base, dn);
        ld8<AT>(static_cast<const AT *>(a.Hmix) + base, hm);
      }
      moments(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd[r]);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xh[r][i] = (hm[i] - mean) * rstd[r];
        dh[r][i] = dn[i] * ga[i];
        s1 += dh[r][i];
        s2 += dh[r][i] * xh[r][i];
        pg[i] += dn[i] * xh[r][i];
        pb[i] += dn[i];
      }
    }
    sums[r] = s1; sums[R + r] = s2;
  }
  block_sum_n<2 * R>(sums, red);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int b = rb * R + r;
    sl[r] = 0.0f;
    if (b < a.B && mine) {
      const size_t base = (size_t)b * a.Dh + tid * 8;
      const float m1 = sums[r] / (float)a.Dh, m2 = sums[R + r] / (float)a.Dh;
      float d1[8], d2[8], al[8], pre_g[8], pre_c[8], x[8], dar[8], dhm[8], dcv[8], dX[8];
      ld8<AT>(static_cast<const AT *>(a.dHmix1) + base, d1);
#pragma unroll
      for (int i = 0; i < 8; ++i) { d2[i] = 0.0f; al[i] = 1.0f; pre_c[i] = 0.0f; }
      if (a.dHmix2) ld8<AT>(static_cast<const AT *>(a.dHmix2) + base, d2);
      if (a.alpha) {
        ld8<AT>(static_cast<const AT *>(a.alpha) + base, al);
        ld8<AT>(static_cast<const AT *>(a.cv) + base, pre_c);
      }
      ld8<AT>(static_cast<const AT *>(a.hm) + base, pre_g);
      ld8<AT>(static_cast<const AT *>(a.X) + base, x);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = d1[i] + d2[i] + rstd[r] * (dh[r][i] - m1 - xh[r][i] * m2);
        const float dHg = d * al[i], dHl = d * (1.0f - al[i]);
        float grad_g, grad_c;
        const float hg = fmaf(lam, x[i], fade_gelu_both(pre_g[i], grad_g)), hl = fade_gelu_both(pre_c[i], grad_c);
        dar[i] = d * (hg - hl) * al[i] * (1.0f - al[i]);
        dhm[i] = dHg * grad_g;
        dcv[i] = dHl * grad_c;
        dX[i] = lam * dHg;
        sl[r] += dHg * x[i];
      }
      if (a.alpha) {
        st8<AT>(static_cast<AT *>(a.dar) + base, dar);
        st8<AT>(static_cast<AT *>(a.dcv) + base, dcv);
      }
      st8<AT>(static_cast<AT *>(a.dhm) + base, dhm);
      st8<AT>(static_cast<AT *>(a.dX) + base, dX);
    }
  }
  block_sum_n<R>(sl, red);
  if (tid == 0) {
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (rb * R + r < a.B) a.row_dlam[rb * R + r] = sl[r];
  }
  }
  if (mine) {
    float *p = a.ln_part + (size_t)blockIdx.x * 2 * a.Dh;
    st8<float>(p + tid * 8, pg);
    st8<float>(p + a.Dh + tid * 8, pb);
  }
}

// Column sums in two deterministic stages. Stage 1 (inside a producer kernel) leaves partial sums per row block as
// part[P][N]; stage 2 adds the P partials of each column in a fixed order.
// Several queued column sums in one launch (blockIdx.y picks the item). 1024 threads = cw columns x (1024 / cw) row
// phases, cw = 32 or, for an item narrower than that, the next power of two >= N (a [B][1] column of per-stream terms
// then has all 1024 threads on its rows). Phase h adds rows h, h + phases, ... in increasing order; the phase sums are
// folded pairwise in a fixed tree: the result does not depend on timing.
__global__ __launch_bounds__(1024) void reduce_batch_kernel(ReduceBatch rb) {
  // The sums run in fp64 (rounded to fp32 once at the end): some of them, the residual-scale gradients above all, are small
  // differences of many large terms, and fp64 adds cost nothing here.
  __shared__ double ps[1024];
  const int k = blockIdx.y, P = rb.P[k], N = rb.N[k], tid = threadIdx.x;
  int lg = 5;
  while (lg > 0 && (1 << (lg - 1)) >= N) --lg;
  const int cw = 1 << lg, phases = 1024 >> lg;
  if ((int)blockIdx.x * cw >= N) return;  // uniform over the workgroup
  const float *part = rb.part[k];
  const int c = tid & (cw - 1), h = tid >> lg, n = blockIdx.x * cw + c;
  double s = 0.0;
  if (n < N) {
#pragma unroll 8
    for (int p = h; p < P; p += phases) s += (double)part[(size_t)p * N + n];
  }
  ps[tid] = s;  // [phase][column]
  __syncthreads();
  for (int st = phases >> 1; st > 0; st >>= 1) {
    if (h < st) ps[tid] += ps[tid + (st << lg)];
    __syncthreads();
  }
  if (h == 0 && n < N) {
    const float t = (float)ps[tid];
    rb.out[k][n] = t;
    if (rb.adam[k]) adam_element(rb.opt, (size_t)(rb.out[k] - rb.opt.grad_base) + n, t);
  }
}
// ---------------------------------------------------------------------------------------------------
// Eq. 7's per-stream memory, backward + its own Adam step (one wavefront per stream, d_low = 64):
//   dz = sum of split partials; dy[k] = sum_n W_U[b][k][n] dz[n]; grad W_U[b][k][n] = y[k] dz[n].
// The gradient is consumed on the spot by Adam (master, moments, compute copy), so it never goes to memory.
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void bwd_cci_kernel(BwdCciArgs a) {
  __shared__ float dz_s[64], y_s[64];
  const int b = blockIdx.x, tid = threadIdx.x;
  // the Adam operands of this stream (4 x 4 consecutive elements per thread and array) are requested first: nothing
  // below depends on them until the update, so their latency runs under the dz / dy part
  float *master = a.master + (size_t)b * 4096, *m = a.m + (size_t)b * 4096, *v = a.v + (size_t)b * 4096;
  f32x4 w4[4], m4[4], v4[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int idx = (e * 256 + tid) * 4;
    w4[e] = *reinterpret_cast<const f32x4 *>(master + idx);
    m4[e] = *reinterpret_cast<const f32x4 *>(m + idx);
    v4[e] = *reinterpret_cast<const f32x4 *>(v + idx);
  }
  if (tid < 64) {
    float dz = 0.0f;
    for (int s0 = 0; s0 < a.splits; s0 += 8) {  // 8 partials in flight, added in split order
      float pv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) pv[j] = a.dz_part[((size_t)(s0 + j < a.splits ? s0 + j : a.splits - 1) * a.B + b) * 64 + tid];
#pragma unroll
      for (int j = 0; j < 8; ++j) dz += (s0 + j < a.splits) ? pv[j] : 0.0f;
    }
    dz_s[tid] = dz;
    y_s[tid] = a.y[(size_t)b * 64 + tid];
  }
  __syncthreads();
  AT *Wc = static_cast<AT *>(a.WU_c) + (size_t)b * 4096;
  {  // dy[k] = row k of W_U[b] dot dz. The compute copy W_U[b] is the master rounded to the activation type, and the master
     // is in registers already (thread: rows 16 e + tid / 16, columns 4 (tid % 16) .. + 3): no second read of the matrix.
     // 16 threads share a row: their partial sums are combined in a fixed butterfly.
    const int n0 = (tid & 15) * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float s = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) s = fmaf((float)(AT)w4[e][i], dz_s[n0 + i], s);
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      s += __shfl_xor(s, 4, 64);
      s += __shfl_xor(s, 8, 64);
      if ((tid & 15) == 0) {
        const int k = e * 16 + (tid >> 4);
        a.dy[(size_t)b * 64 + k] = s;
        static_cast<AT *>(a.dy_at)[(size_t)b * 64 + k] = (AT)s;
      }
    }
  }
  const UpdateState u = *a.u;
  if (u.na == 0) return;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int idx = (e * 256 + tid) * 4, k = idx >> 6, n = idx & 63;
    float wn[4];
    if (a.g_dbg) {  // debug: the gradient itself, which otherwise only exists in registers
      f32x4 g4;
#pragma unroll
      for (int i = 0; i < 4; ++i) g4[i] = y_s[k] * dz_s[n + i];
      *reinterpret_cast<f32x4 *>(a.g_dbg + (size_t)b * 4096 + idx) = g4;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float g = y_s[k] * dz_s[n + i];
      const float mk = a.beta1 * m4[e][i] + (1.0f - a.beta1) * g;
      const float vk = a.beta2 * v4[e][i] + (1.0f - a.beta2) * g * g;
      m4[e][i] = mk;
      v4[e][i] = vk;
      wn[i] = w4[e][i] - a.lr * (mk / u.c1) / (sqrtf(vk / u.c2) + a.eps);
      w4[e][i] = wn[i];
    }
    *reinterpret_cast<f32x4 *>(m + idx) = m4[e];
    *reinterpret_cast<f32x4 *>(v + idx) = v4[e];
    *reinterpret_cast<f32x4 *>(master + idx) = w4[e];
#pragma unroll
    for (int i = 0; i < 4; ++i) Wc[idx + i] = (AT)wn[i];
  }
}

// ---------------------------------------------------------------------------------------------------
// Eq. 1-3 backward through the newest cache slot. A wavefront owns SPW streams (4 * SPW per workgroup):
//   dg[q] = sum_n d(hm)[n] W_m[Dc-c+q][n];  d gg = dg gv psi'(gg);  d gv = dg psi(gg);  dxt = W_g d gg + W_v d gv
// and the first stage of dW_g[i][q] = sum_b xt[b][i] d gg[b][q] (same for W_v): the workgroup's streams, in order,
// as part[workgroup][2][D][c] (blob order); the second stage adds the workgroups in index order.
// Without a.dg every wavefront walks all c rows of W_m's last slot itself, which is fine for the narrow slots of the
// benchmark shapes (c = 4..8) and far too much L2 traffic for wide ones: there dg comes from a product (a.dg) and this
// kernel only does the element-wise part. Narrow rows (D_h <= 512: one 8-wide chunk per lane, KCH = 1) put 4 streams on a
// wavefront.
// ---------------------------------------------------------------------------------------------------
template <typename AT, int SPW, int KCH>
__device__ __forceinline__ void bwd_slot_body(const BwdSlotArgs &a, int block) {
  constexpr int NS = 4 * SPW;  // streams per workgroup
  __shared__ float dg_s[NS][2][256];  // cache_chunk <= 256
  __shared__ float xt_s[NS][64];      // D <= 64
  __shared__ int sym_s[NS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = block * NS + wave * SPW;  // this wavefront's first stream
  const int nch = a.Dh / 8;  // 8-wide chunks of a row: lane owns chunks lane, lane + 64, ... (KCH of them)
  float dh[SPW][KCH][8];
#pragma unroll
  for (int u = 0; u < SPW; ++u)
#pragma unroll
    for (int k = 0; k < KCH; ++k) {
      // no branch around the loads (a branch makes the compiler wait for each load before it issues the next): addresses
      // are clamped into the array, values of streams / chunks that do not exist are zeroed afterwards
      const int ch = lane + 64 * k, bc = b0 + u < a.B ? b0 + u : a.B - 1, cc = ch < nch ? ch : nch - 1;
      ld8<AT>(static_cast<const AT *>(a.dhm) + (size_t)bc * a.Dh + cc * 8, dh[u][k]);
    }
#pragma unroll
  for (int u = 0; u < SPW; ++u)
#pragma unroll
    for (int k = 0; k < KCH; ++k)
      if (!(b0 + u < a.B && lane + 64 * k < nch)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) dh[u][k][i] = 0.0f;
      }
  for (int q0 = 0; q0 < a.c; q0 += 64) {  // 64 slot columns at a time: lane ql ends up with dg[q0 + ql] of each stream
    const int qn = a.c - q0 < 64 ? a.c - q0 : 64;
    float mine[SPW];
#pragma unroll
    for (int u = 0; u < SPW; ++u) {
      mine[u] = 0.0f;
      if (a.dg && lane < qn && b0 + u < a.B) mine[u] = (float)static_cast<const AT *>(a.dg)[(size_t)(b0 + u) * a.c + q0 + lane];
    }
    for (int ql = 0; ql < (a.dg ? 0 : qn); ++ql) {
      const float *wrow = a.Wm + (size_t)(a.Dc - a.c + q0 + ql) * a.Dh;
      float sacc[SPW];
#pragma unroll
      for (int u = 0; u < SPW; ++u) sacc[u] = 0.0f;
      float w[KCH][8];
#pragma unroll
      for (int k = 0; k < KCH; ++k) {  // all of the row's pieces requested together; a chunk past the row meets dh = 0
        const int ch = lane + 64 * k;
        ld8<float>(wrow + (ch < nch ? ch : nch - 1) * 8, w[k]);
      }
#pragma unroll
      for (int k = 0; k < KCH; ++k) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float wi = a.round_bf16 ? (float)(bf16_t)w[k][i] : w[k][i];
#pragma unroll
          for (int u = 0; u < SPW; ++u) sacc[u] = fmaf(dh[u][k][i], wi, sacc[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < SPW; ++u) {
        float sv = sacc[u];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sv += __shfl_xor(sv, off, 64);
        if (lane == ql) mine[u] = sv;
      }
    }
    if (lane < qn) {
      const int q = q0 + lane;
#pragma unroll
      for (int u = 0; u < SPW; ++u) {
        const int b = b0 + u;
        float dgg = 0.0f, dgv = 0.0f;
        if (b < a.B) {
          const float gg = a.GG[(size_t)b * a.c + q], gv = a.GV[(size_t)b * a.c + q];
          dgg = mine[u] * gv * gelu_grad_f(gg);
          dgv = mine[u] * gelu_f(gg);
          a.dgg[(size_t)b * a.c + q] = dgg;
          a.dgv[(size_t)b * a.c + q] = dgv;
        }
        dg_s[wave * SPW + u][0][q] = dgg;
        dg_s[wave * SPW + u][1][q] = dgv;
      }
    }
  }
  if (lane < SPW) {
    const int b = b0 + lane;
    sym_s[wave * SPW + lane] = (b < a.B && stream_active(a.ws, b)) ? (int)stream_window(a.ws, b, a.T)[a.T - 1] : -1;
  }
  __syncthreads();
  // one thread per (stream, channel): the stream's x_t row goes to LDS (zero for an inactive stream: it then adds
  // nothing below), and dxt[channel] = sum_q W_g[channel][q] d gg[q] + W_v[channel][q] d gv[q]
  const bool wide = a.c >= 64;
  for (int t = tid; t < NS * a.D; t += 256) {
    const int k = t / a.D, i = t - k * a.D, b = block * NS + k;
    xt_s[k][i] = sym_s[k] >= 0 ? a.tabXe32[(size_t)sym_s[k] * a.D + i] : 0.0f;
    if (b < a.B && !wide) {
      float sv = 0.0f;
      for (int q = 0; q < a.c; ++q) sv += a.Wg[i * a.c + q] * dg_s[k][0][q] + a.Wv[i * a.c + q] * dg_s[k][1][q];
      a.dxt[(size_t)b * a.D + i] = sv;
    }
  }
  if (wide) {
    // wide slots: a thread walking all c columns of its channel's rows of W_g, W_v reads them with a stride of a whole row
    // between neighbouring threads. Here a wavefront takes channels wave, wave + 4, ... and its lanes run along the slot
    // columns (coalesced rows, read once for all of the workgroup's streams); each stream's sum is folded over the lanes in
    // a fixed butterfly and lane k keeps stream k's.
    for (int i = wave; i < a.D; i += 4) {
      float acc[NS];
#pragma unroll
      for (int k = 0; k < NS; ++k) acc[k] = 0.0f;
      for (int q = lane; q < a.c; q += 64) {
        const float wg = a.Wg[i * a.c + q], wv = a.Wv[i * a.c + q];
#pragma unroll
        for (int k = 0; k < NS; ++k) acc[k] = fmaf(wg, dg_s[k][0][q], fmaf(wv, dg_s[k][1][q], acc[k]));
      }
      float keep = 0.0f;
#pragma unroll
      for (int k = 0; k < NS; ++k) {
        float sv = acc[k];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sv += __shfl_xor(sv, off, 64);
        if (lane == k) keep = sv;
      }
      if (lane < NS && block * NS + lane < a.B) a.dxt[(size_t)(block * NS + lane) * a.D + i] = keep;
    }
  }
  __syncthreads();
  const int nout = 2 * a.D * a.c;
  for (int t = tid; t < nout; t += 256) {
    const int which = t / (a.D * a.c), r = t - which * a.D * a.c, i = r / a.c, q = r - i * a.c;
    float sv = 0.0f;
#pragma unroll
    for (int k = 0; k < NS; ++k) sv = fmaf(xt_s[k][i], dg_s[k][which][q], sv);
    a.part[(size_t)block * nout + t] = sv;
  }
}
template <typename AT, int SPW, int KCH>
__global__ __launch_bounds__(256) void bwd_slot_kernel(BwdSlotArgs a) {
  bwd_slot_body<AT, SPW, KCH>(a, (int)blockIdx.x);
}

// ---------------------------------------------------------------------------------------------------
// Eq. 4's weight gradient: dW_conv[r][i][o] = sum over tokens (b, j) of xl[b][j-(k-1)+r][i] * dcv[b][j][o] and
// db_conv[o] = sum dcv. Stage 1: each workgroup reduces its slice of tokens into a partial [taps*D + 1][D];
// stage 2 adds the partials in workgroup order.
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void conv_grad_partial_kernel(ConvGradArgs a) {
  // One workgroup = 128 consecutive tokens = whole streams (T divides 128), both tiles staged in LDS as fp32. The input
  // tile carries taps-1 zero rows in front of every stream: tap r of token j is then row j + r of the padded stream, no
  // boundary test is left in the loop, and the (tap, i) rows a thread owns are contiguous floats.
  constexpr int kXs = (128 + 3 * 32) * 32 + 32;  // taps <= 4, T >= 4, 16 <= D <= 32; 32 floats of slack for the over-read below
  __shared__ __attribute__((aligned(16))) float xs[kXs];
  __shared__ __attribute__((aligned(16))) float ds[128 * 32];
  const int tid = threadIdx.x, D = a.D, pad = a.taps - 1;
  const int lgD = 31 - __builtin_clz(D), lgT = 31 - __builtin_clz(a.T), Tm = a.T - 1, Tp = a.T + pad;  // D, T: powers of two
  const long long tokens = (long long)a.B * a.T, nchunks = (tokens + 127) / 128;
  const int used = (((128 >> lgT) * Tp) << lgD) + 32;
  for (int e = tid; e < used; e += 256) xs[e] = 0.0f;  // the zero rows stay zero: the tiles below never touch them
  const int rows = a.taps * D;                    // (tap, i) pairs
  const int o = tid & (D - 1), grp = tid >> lgD, ngrp = 256 >> lgD;
  const int per = (rows + ngrp - 1) / ngrp;       // (tap, i) rows owned by this thread's group (<= 16)
  const float *xp = xs + grp * per;
  float acc[16], bsum = 0.0f;
#pragma unroll
  for (int q = 0; q < 16; ++q) acc[q] = 0.0f;
  // a workgroup takes chunks blockIdx.x, blockIdx.x + gridDim.x, ... and keeps adding into the same registers
  for (long long chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x) {
  const long long t0 = chunk * 128;
  const AT *XL = static_cast<const AT *>(a.XL) + (size_t)t0 * D, *dcv = static_cast<const AT *>(a.dcv) + (size_t)t0 * D;
  __syncthreads();  // the zero fill, or the previous chunk's reads, are done
  const int left = (int)((tokens - t0 < 128 ? tokens - t0 : 128)) << lgD;  // elements of this tile that exist
  for (int e = tid * 8; e < (128 << lgD); e += 2048) {
    float x[8], d[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { x[q] = 0.0f; d[q] = 0.0f; }
    if (e < left) { ld8<AT>(XL + e, x); ld8<AT>(dcv + e, d); }
    const int tl = e >> lgD, at = ((((tl >> lgT) * Tp) + pad + (tl & Tm)) << lgD) + (e & (D - 1));
#pragma unroll
    for (int q = 0; q < 8; ++q) { xs[at + q] = x[q]; ds[e + q] = d[q]; }
  }
  __syncthreads();
  // rows past `per` (or past `rows`) are read and accumulated too (in bounds thanks to the slack) and dropped at the end
  if ((per & 3) == 0) {
    for (int tl = 0; tl < 128; ++tl) {
      const float d = ds[(tl << lgD) + o];
      bsum += d;
      const f32x4 *x4 = reinterpret_cast<const f32x4 *>(xp + ((((tl >> lgT) * Tp) + (tl & Tm)) << lgD));
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 x = x4[q4];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[4 * q4 + i] = fmaf(x[i], d, acc[4 * q4 + i]);
      }
    }
  } else {
    for (int tl = 0; tl < 128; ++tl) {
      const float d = ds[(tl << lgD) + o];
      bsum += d;
      const float *x = xp + ((((tl >> lgT) * Tp) + (tl & Tm)) << lgD);
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[q] = fmaf(x[q], d, acc[q]);
    }
  }
  }
  float *part = a.part + (size_t)blockIdx.x * (rows + 1) * D;
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int r = grp * per + q;
    if (q < per && r < rows) part[(size_t)r * D + o] = acc[q];
  }
  if (grp == 0) part[(size_t)rows * D + o] = bsum;
}

// The same on the matrix cores (bf16 activations, D = 32): per 128-token chunk, dW_conv[r] (32 x 32) = X_r^T dcv with X_r the
// input tile shifted by tap r, a contraction over the tokens. Both operands sit in LDS row-major as they are in memory
// (bf16, 64 bytes per token, the input tile with its zero rows in front of every stream) and are read with the transposing
// LDS load (see the weight-gradient kernel in fade_gemm.hip: a lane supplies the address of 4 consecutive values of ITS
// row, so the rows of one fragment need not be equidistant, which is what the per-stream zero rows require). Wavefront r
// owns tap r; wavefront 0 also forms the bias gradient as a product with a fragment of ones. bf16 x bf16 products are exact in
// fp32, so this differs from the scalar kernel in summation order only.
__device__ __forceinline__ void conv_grad_mfma_body(const ConvGradArgs &a, int block, int nblocks) {
  typedef __attribute__((ext_vector_type(4))) short i16x4;
  typedef __attribute__((ext_vector_type(8))) short i16x8;
  constexpr int D = 32, PITCH = 64, XROWS = 128 + 3 * 32;  // taps <= 4, T >= 4: at most 32 streams x 3 zero rows
  __shared__ __attribute__((aligned(16))) unsigned char xs[XROWS * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char ds[128 * PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, pad = a.taps - 1;
  const int lgT = 31 - __builtin_clz(a.T), Tm = a.T - 1, Tp = a.T + pad;
  const long long tokens = (long long)a.B * a.T, nchunks = (tokens + 127) / 128;
  for (int e = tid; e < XROWS * PITCH / 16; e += 256) reinterpret_cast<f32x4 *>(xs)[e] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  f32x16 acc, accb;
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc[e] = 0.0f; accb[e] = 0.0f; }
  bf16x8 ones;
#pragma unroll
  for (int q = 0; q < 8; ++q) ones[q] = (bf16_t)1.0f;
  // this lane's part of a fragment: rows (tokens) 8 (lane / 32) + (lane % 16) / 4 and 4 further, 4 columns from byte colb on
  const int s16 = lane & 15, tk = (lane >> 5) * 8 + (s16 >> 2), mh = (lane >> 4) & 1;
  const int colb = ((2 * mh + ((s16 & 3) >> 1)) << 4) + (s16 & 1) * 8;
  auto prow = [&](int tl) { return (tl >> lgT) * Tp + (tl & Tm); };  // row of token tl's tap 0 in the padded tile
  auto tr_load = [](const unsigned char *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)p); };
  const bf16_t *XL = static_cast<const bf16_t *>(a.XL), *dcv = static_cast<const bf16_t *>(a.dcv);
  // d(input) = the anti-causal convolution of dcv with the taps turned round: token j gets sum_r dcv[j + (taps-1) - r] W[r]^T,
  // as far as that token is still in the window. Wavefront w owns tokens 32 w .. 32 w + 31 of the chunk; its operand piece
  // (8 consecutive channels of one token) is one 16-byte read of the dcv tile as it lies.
  const int xsteps = a.WT ? a.Kc / 16 : 0;  // <= 8
  bf16x8 wt[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
    for (int q = 0; q < 8; ++q) wt[ks][q] = (bf16_t)0.0f;
    if (ks < xsteps) wt[ks] = static_cast<const bf16x8 *>(a.WT)[(size_t)ks * 64 + lane];
  }
  // The pieces of chunk c + 1 are requested before the matrix work on chunk c and waited for after it, BEFORE chunk c's
  // stores: the counter of outstanding memory operations is in order and covers stores, and behind stores that sit in a
  // branch the compiler's count for an older load is the pessimistic one, so a wait placed after the stores would also
  // wait for them to be acknowledged. No branch around the loads: addresses clamped, tokens past the end zeroed at use.
  f32x4 pxv[2], pdv[2];
  auto request = [&](long long t0) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {  // 128 tokens x 4 pieces of 16 bytes, for each operand
      const int e = tid + 256 * it, tl = e >> 2, pc = e & 3;
      const long long t = t0 + tl < tokens ? t0 + tl : tokens - 1;
      pxv[it] = *reinterpret_cast<const f32x4 *>(XL + (size_t)t * D + pc * 8);
      pdv[it] = *reinterpret_cast<const f32x4 *>(dcv + (size_t)t * D + pc * 8);
    }
  };
  if (block < nchunks) request((long long)block * 128);
  for (long long chunk = block; chunk < nchunks; chunk += nblocks) {
    const long long t0 = chunk * 128;
    __syncthreads();  // the zero fill, or the previous chunk's reads, are done
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int e = tid + 256 * it, tl = e >> 2, pc = e & 3;
      const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
      const bool live = t0 + tl < tokens;
      *reinterpret_cast<f32x4 *>(xs + (prow(tl) + pad) * PITCH + pc * 16) = live ? pxv[it] : zero4;
      *reinterpret_cast<f32x4 *>(ds + tl * PITCH + pc * 16) = live ? pdv[it] : zero4;
    }
    __syncthreads();
    request(chunk + nblocks < nchunks ? (chunk + nblocks) * 128 : t0);  // the last turn asks for its own chunk again
    if (wave < a.taps) {
#pragma unroll 2
      for (int ks = 0; ks < 8; ++ks) {
        const int tl = ks * 16 + tk;
        const i16x4 al = tr_load(xs + (prow(tl) + wave) * PITCH + colb), ah = tr_load(xs + (prow(tl + 4) + wave) * PITCH + colb);
        const i16x4 bl = tr_load(ds + tl * PITCH + colb), bh = tr_load(ds + (tl + 4) * PITCH + colb);
        const bf16x8 af = __builtin_bit_cast(bf16x8, (i16x8)__builtin_shufflevector(al, ah, 0, 1, 2, 3, 4, 5, 6, 7));
        const bf16x8 bf = __builtin_bit_cast(bf16x8, (i16x8)__builtin_shufflevector(bl, bh, 0, 1, 2, 3, 4, 5, 6, 7));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf, acc, 0, 0, 0);
        if (wave == 0) accb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, bf, accb, 0, 0, 0);
      }
    }
    if (a.WT) {
      const int tl = wave * 32 + (lane & 31), jj = tl & Tm;
      f32x16 accx;
#pragma unroll
      for (int e = 0; e < 16; ++e) accx[e] = 0.0f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        if (ks < xsteps) {
          const int k = ks * 16 + (lane >> 5) * 8, tap = k >> 5, o = k & 31, ahead = pad - tap;  // D = 32
          bf16x8 af;
#pragma unroll
          for (int q = 0; q < 8; ++q) af[q] = (bf16_t)0.0f;
          if (tap < a.taps && jj + ahead <= Tm) af = *reinterpret_cast<const bf16x8 *>(ds + (tl + ahead) * PITCH + o * 2);
          accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, wt[ks], accx, 0, 0, 0);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" : "+v"(pxv[0]), "+v"(pxv[1]), "+v"(pdv[0]), "+v"(pdv[1]), "+v"(accx) : : "memory");  // see above
      bf16_t *dxl = static_cast<bf16_t *>(a.dxl);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const long long t = t0 + wave * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (t < tokens) dxl[(size_t)t * D + (lane & 31)] = (bf16_t)accx[e];
      }
    }
  }
  const int rows = a.taps * D;
  float *part = a.part + (size_t)block * (rows + 1) * D;
  if (wave < a.taps) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int i = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
      part[(size_t)(wave * D + i) * D + (lane & 31)] = acc[e];
    }
  }
  if (wave == 0 && lane < 32) part[(size_t)rows * D + lane] = accb[0];
}
__global__ __launch_bounds__(256) void conv_grad_mfma_kernel(ConvGradArgs a) {
  conv_grad_mfma_body(a, (int)blockIdx.x, (int)gridDim.x);
}
// The newest-slot backward and the conv backward both start from what the mix backward left and feed the embedding
// backward: independent, so one launch carries both. The first pconv workgroups take the conv part: each of them walks
// many 128-token chunks, so they start first and the short slot workgroups fill in around them.
// Three wavefronts per SIMD: the slot half's streams are one wavefront each and need the occupancy; without the bound the
// conv half's prefetch registers take the kernel to two (136 us against 101-107; a bound of four spills and gives 108).
template <int SPW, int KCH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void slot_conv_kernel(BwdSlotArgs sa, ConvGradArgs ca, int pconv) {
  if ((int)blockIdx.x < pconv) conv_grad_mfma_body(ca, (int)blockIdx.x, pconv);
  else bwd_slot_body<bf16_t, SPW, KCH>(sa, (int)blockIdx.x - pconv);
}

// ---------------------------------------------------------------------------------------------------
// the two per-token LayerNorms and the embedding, backward. For a fixed symbol s the LayerNorm backward is a LINEAR map of
// the incoming gradient (mean, 1/sigma and x-hat depend on E[s] only), so tokens are first summed per symbol:
//   SX[s] = sum over tokens with symbol s of dX (router + global residual + newest-slot paths),  SL[s] likewise of dX_l,
// and everything else happens on the 256 x D tables:
//   dE[s] = rstd_s * ( P_s(gamma_e * SX[s]) + P_s(gamma_l * SL[s]) ),  P_s(v) = v - mean(v) - xhat_s * mean(v * xhat_s)
//   d gamma_e = sum_s xhat_s * SX[s], d beta_e = sum_s SX[s]  (same with SL for the pair of Eq. 4's LayerNorm).
// ---------------------------------------------------------------------------------------------------
// Stage 1 of the per-symbol sums, on the matrix cores: S[s][n] = sum over tokens t of onehot[t][s] * V[t][n], with V = [dX paths | dX_l]
// (2 D columns). The one-hot operand is exact in bf16; V is split into bf16 terms (hi + mid + lo carries 24 mantissa bits; two
// terms are enough for bf16 inputs), so the result is an fp32-accurate sum in a fixed order. One workgroup owns a contiguous token range and leaves a
// partial table [2][256][D]; wavefront w owns symbols 64 w .. 64 w + 63. V is staged row-major (16-byte pieces, permuted as
// in the weight-gradient kernel) and read with the transposing LDS load.
// NTH threads: wavefront w owns the 256 / (NTH / 64) symbols from 256 w / (NTH / 64) on (RT = 1 or 2 row tiles of 32).
template <typename AT, int D, int NTH>
__global__ __launch_bounds__(NTH) void symbol_sums_mfma_kernel(BwdTokenArgs a, int per_block) {
  typedef __attribute__((ext_vector_type(4))) short i16x4;
  typedef __attribute__((ext_vector_type(8))) short i16x8;
  typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;
  constexpr int W2 = 2 * D, PITCH = W2 * 2, NT = W2 / 32, PPR = W2 / 8, CH = 128;
  // bf16 inputs: a sum of two bf16 values (plus, for one token in T, an fp32 term) is carried by two terms to 2^-17
  constexpr int NS = sizeof(AT) == 2 ? 2 : 3;
  constexpr int RT = 8 / (NTH / 64);  // 32-symbol row tiles per wavefront
  static_assert(NTH == 256 || NTH == 512, "threads");
  __shared__ __attribute__((aligned(16))) unsigned char vs[NS][CH * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned short sym[CH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lgT = 31 - __builtin_clz(a.T), Tm1 = a.T - 1;
  const long long tokens = (long long)a.B * a.T, t_begin = (long long)blockIdx.x * per_block;
  long long t_end = t_begin + per_block;
  if (t_end > tokens) t_end = tokens;
  auto swz = [](int r) { return PITCH == 128 ? (((r >> 1) & 1) << 2) : 0; };
  f32x16 acc[RT][NT];
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  // addresses this lane supplies to the transposing loads (k-step 0, first of the two loads), per column tile
  const int s16 = lane & 15, r0 = (lane >> 5) * 8 + (s16 >> 2), mh = (lane >> 4) & 1;
  int b_off[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) b_off[j] = r0 * PITCH + (((j * 4 + 2 * mh + ((s16 & 3) >> 1)) ^ swz(r0)) << 4) + (s16 & 1) * 8;
  const bf16_t one = (bf16_t)1.0f, zero = (bf16_t)0.0f;

  // global loads of chunk c + 1 are issued before the matrix work on chunk c (values wait in registers). The two big loads
  // of an item are issued without a branch (addresses clamped into the arrays, values masked when they are used): with the
  // loads inside `if (t < t_end)` the compiler waits for each item's loads before it issues the next item's.
  constexpr int ITEMS = CH * PPR / NTH;
  Raw8B<AT> ra[ITEMS], rb[ITEMS];
  Raw8B<float> rc[ITEMS];
  unsigned short psym = 0xFFFF;
  auto fetch = [&](long long c0) {
    // the symbol first: its address depends on loaded values (active flag, window position), and waiting for that chain
    // must not wait for the big loads behind it
    psym = 0xFFFF;  // matches no symbol: tokens past the range and inactive streams contribute nothing
    if (tid < CH) {
      const long long t = c0 + tid;
      if (t < t_end) {
        const int b = (int)(t >> lgT), j = (int)(t & Tm1);
        if (stream_active(a.ws, b)) psym = stream_window(a.ws, b, a.T)[j];
      }
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int item = tid + NTH * it, tl = item / PPR, col = (item % PPR) * 8;
      const long long t = c0 + tl < tokens ? c0 + tl : tokens - 1;
      const bool first = col < D;  // columns [0, D): dX1 + dX2 (+ dxt at the newest token); [D, 2 D): dxl
      const size_t g = (size_t)t * D + (first ? col : col - D);
      ra[it].load(first ? static_cast<const AT *>(a.dX1) + g : static_cast<const AT *>(a.dxl) + g);
      rb[it].load(static_cast<const AT *>(a.dX2) + g);  // used by the first half only
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int item = tid + NTH * it, tl = item / PPR, col = (item % PPR) * 8;
      const long long t = c0 + tl;
      rc[it].zero();
      // newest token of its stream: the cache-slot path ends here too
      if (t < t_end && col < D && (int)(t & Tm1) == Tm1) rc[it].load(a.dxt + (size_t)(t >> lgT) * D + col);
    }
  };
  if (t_begin < t_end) fetch(t_begin);
  for (long long c0 = t_begin; c0 < t_end; c0 += CH) {
    __syncthreads();  // the previous chunk has been consumed
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int item = tid + NTH * it, tl = item / PPR, pc = item % PPR;
      float v[8], w[8], x[8];
      ra[it].cvt(v); rb[it].cvt(w); rc[it].cvt(x);
      const bool live = c0 + tl < t_end, both = live && pc * 8 < D;
      bf16x8 hi, mid, lo;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float val = ((live ? v[q] : 0.0f) + (both ? w[q] : 0.0f)) + x[q];
        hi[q] = (bf16_t)val;
        const float r1 = val - (float)hi[q];
        mid[q] = (bf16_t)r1;
        lo[q] = (bf16_t)(r1 - (float)mid[q]);
      }
      const int pos = tl * PITCH + ((pc ^ swz(tl)) << 4);
      *reinterpret_cast<bf16x8 *>(&vs[0][pos]) = hi;
      *reinterpret_cast<bf16x8 *>(&vs[1][pos]) = mid;
      if (NS == 3) *reinterpret_cast<bf16x8 *>(&vs[NS - 1][pos]) = lo;
    }
    if (tid < CH) sym[tid] = psym;
    __syncthreads();
    if (c0 + CH < t_end) fetch(c0 + CH);
#pragma unroll 2
    for (int ks = 0; ks < CH / 16; ++ks) {
      const u16x8 sy = *reinterpret_cast<const u16x8 *>(sym + ks * 16 + (lane >> 5) * 8);
      bf16x8 af[RT];
#pragma unroll
      for (int i = 0; i < RT; ++i) {
        const unsigned short s = (unsigned short)((wave * RT + i) * 32 + (lane & 31));
#pragma unroll
        for (int q = 0; q < 8; ++q) af[i][q] = sy[q] == s ? one : zero;
      }
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int sp = 0; sp < NS; ++sp) {
          const unsigned char *p = &vs[sp][0] + b_off[j] + ks * 16 * PITCH;
          const i16x4 l4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)p);
          const i16x4 h4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(p + 4 * PITCH));
          const bf16x8 bfr = __builtin_bit_cast(bf16x8, (i16x8)__builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
          for (int i = 0; i < RT; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr, acc[i][j], 0, 0, 0);
        }
    }
  }
  float *out = a.part + (size_t)blockIdx.x * 2 * 256 * D;
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int s = (wave * RT + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3), n = j * 32 + (lane & 31);
        out[((size_t)(n / D) * 256 + s) * D + (n % D)] = acc[i][j][e];
      }
}

// Finish on the tables: one workgroup per symbol. First the symbol's two rows of the per-symbol sums (SX then SL) from the
// P partial tables part[P][2][256][D] (64 columns x 4 phases; phase h adds partials h, h + 4, ... in increasing order, the
// phase sums are added in phase order), then, lane = channel, dE[s] and this symbol's contribution to (d gamma_e, d beta_e,
// d gamma_l, d beta_l) as contrib[s][4][D]. D <= 32.
__global__ __launch_bounds__(256) void embed_finish_kernel(int D, int P, const float *part, const float *tabXhat, const float *tabRstd,
                                                           const float *gamma_e, const float *gamma_l, float *dE, float *contrib) {
  __shared__ float ps[4][64];
  __shared__ float red[4][64];
  const int s = blockIdx.x, tid = threadIdx.x, c = tid & 63, h = tid >> 6;
  float acc = 0.0f;
  if (c < 2 * D) {
    const int tab = c / D, ch = c - tab * D;
    const float *src = part + ((size_t)tab * 256 + s) * D + ch;
    const size_t stride = (size_t)2 * 256 * D;
#pragma unroll 8
    for (int p = h; p < P; p += 4) acc += src[(size_t)p * stride];
  }
  ps[h][c] = acc;
  __syncthreads();
  const int i = tid;
  const bool on = i < D;
  float sx = 0.0f, sl = 0.0f;
  if (on) {
    sx = ((ps[0][i] + ps[1][i]) + ps[2][i]) + ps[3][i];
    sl = ((ps[0][D + i] + ps[1][D + i]) + ps[2][D + i]) + ps[3][D + i];
  }
  const float xh = on ? tabXhat[(size_t)s * D + i] : 0.0f;
  const float he = on ? sx * gamma_e[i] : 0.0f, hl = on ? sl * gamma_l[i] : 0.0f;
  if (i < 64) { red[0][i] = he; red[1][i] = he * xh; red[2][i] = hl; red[3][i] = hl * xh; }
  __syncthreads();
  if (on) {
    float m[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int k = 0; k < D; ++k) { m[0] += red[0][k]; m[1] += red[1][k]; m[2] += red[2][k]; m[3] += red[3][k]; }
    const float inv = 1.0f / (float)D;
    dE[(size_t)s * D + i] = tabRstd[s] * ((he - m[0] * inv - xh * m[1] * inv) + (hl - m[2] * inv - xh * m[3] * inv));
    float *cb = contrib + (size_t)s * 4 * D;
    cb[i] = xh * sx; cb[D + i] = sx; cb[2 * D + i] = xh * sl; cb[3 * D + i] = sl;
  }
}

// ---------------------------------------------------------------------------------------------------
// Adam on the big matrices + refresh of their bf16 operand copies, one 64 x 64 block per workgroup
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void adam_refresh_kernel(AdamRefreshBatch ab) {
  __shared__ float tile[64][65];
  __shared__ float gb[2][64];
  UpdateState us{};
  if (!ab.refresh_only) {
    us = *ab.opt.u;
    if (us.na == 0) return;  // nothing was updated, every copy is still valid
  }
  int p = 0;
  while (p + 1 < ab.count && (int)blockIdx.x >= ab.m[p + 1].first_block) ++p;
  const AdamMat &M = ab.m[p];
  const int local = (int)blockIdx.x - M.first_block, nbn = M.N / 64;
  const int kb = local / nbn, nb = local - kb * nbn, k0 = kb * 64, n0 = nb * 64;
  const int tid = threadIdx.x;
  const float b1 = ab.opt.beta1, b2 = ab.opt.beta2, lr = ab.opt.lr, eps = ab.opt.eps;
  {  // Adam: thread = 4 consecutive columns of rows r, r + 16, r + 32, r + 48
    const int c4 = (tid & 15) * 4;
    f32x4 g[4], mm[4], vv[4], w[4];
    size_t idx[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) idx[q] = M.off + (size_t)(k0 + (tid >> 4) + 16 * q) * M.N + n0 + c4;
    // a gradient that arrives as partial sums over ranges of the batch: add them in range order (done before the other
    // operands are fetched, so that it needs no registers of its own); the sum itself only goes to memory in a debug
    // context, nothing but this step uses it
    const bool parts = !ab.refresh_only && M.gpart != nullptr;
    if (parts) {
      const size_t mat = (size_t)M.K * M.N;
#pragma unroll
      for (int q = 0; q < 4; ++q) g[q] = *reinterpret_cast<const f32x4 *>(M.gpart + (idx[q] - M.off));
#pragma unroll 2
      for (int sp = 1; sp < M.gsplits; ++sp)
#pragma unroll
        for (int q = 0; q < 4; ++q) g[q] += *reinterpret_cast<const f32x4 *>(M.gpart + sp * mat + (idx[q] - M.off));
      if (ab.keep_sum) {
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<f32x4 *>(const_cast<float *>(ab.opt.grad_base) + idx[q]) = g[q];
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      w[q] = *reinterpret_cast<const f32x4 *>(ab.opt.master + idx[q]);
      if (!ab.refresh_only) {
        if (!parts) g[q] = *reinterpret_cast<const f32x4 *>(ab.opt.grad_base + idx[q]);
        mm[q] = *reinterpret_cast<const f32x4 *>(ab.opt.m + idx[q]);
        vv[q] = *reinterpret_cast<const f32x4 *>(ab.opt.v + idx[q]);
      }
    }
    if (ab.refresh_only) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[(tid >> 4) + 16 * q][c4 + i] = w[q][i];
    } else
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float mk = b1 * mm[q][i] + (1.0f - b1) * g[q][i];
        const float vk = b2 * vv[q][i] + (1.0f - b2) * g[q][i] * g[q][i];
        mm[q][i] = mk;
        vv[q][i] = vk;
        w[q][i] = w[q][i] - lr * (mk / us.c1) / (sqrtf(vk / us.c2) + eps);
        tile[(tid >> 4) + 16 * q][c4 + i] = w[q][i];
      }
      *reinterpret_cast<f32x4 *>(ab.opt.m + idx[q]) = mm[q];
      *reinterpret_cast<f32x4 *>(ab.opt.v + idx[q]) = vv[q];
      *reinterpret_cast<f32x4 *>(ab.opt.master + idx[q]) = w[q];
    }
  }
  if (M.gamma && tid < 64) { gb[0][tid] = M.gamma[k0 + tid]; gb[1][tid] = M.beta[k0 + tid]; }
  __syncthreads();
  const int vbase = (n0 >> 6) * M.vstride + M.vcol0;  // virtual column of this block's first column (64 columns stay together)
  // 8 fragments of each kind per block, 64 lanes each: two (fragment, lane) pairs per thread
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int id = tid + 256 * q, fl = id >> 6, lane = id & 63, t2 = fl >> 2, s4 = fl & 3;
    if (M.frag) {  // forward operand: lane = column, 8 consecutive rows
      const int n = t2 * 32 + (lane & 31), kk = s4 * 16 + (lane >> 5) * 8;
      bf16x8 r;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float x = tile[kk + i][n];
        if (M.gamma) x = gb[0][kk + i] * (float)(bf16_t)x;
        r[i] = (bf16_t)x;
      }
      const size_t f = (size_t)(vbase / 32 + t2) * (M.K / 16) + (k0 / 16 + s4);
      reinterpret_cast<bf16x8 *>(M.frag)[f * 64 + lane] = r;
    }
    if (M.fragT) {  // operand of dX = dY W^T: lane = row of W, 8 consecutive (virtual) columns
      const int k = t2 * 32 + (lane & 31), nn = s4 * 16 + (lane >> 5) * 8;
      bf16x8 r;
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = (bf16_t)tile[k][nn + i];
      const size_t f = (size_t)(k0 / 32 + t2) * (M.VN / 16) + (vbase / 16 + s4);
      reinterpret_cast<bf16x8 *>(M.fragT)[f * 64 + lane] = r;
    }
  }
  if (M.gamma && tid < 64) {  // this block's part of the folded-LayerNorm vectors: s = column sums of W', t = beta^T W
    float sa = 0.0f, ta = 0.0f;
    for (int k = 0; k < 64; ++k) {
      const float w = (float)(bf16_t)tile[k][tid];
      sa += (float)(bf16_t)(gb[0][k] * w);
      ta = fmaf(gb[1][k], w, ta);
    }
    float *pp = M.fold_part + (size_t)kb * 2 * M.VN;
    pp[vbase + tid] = sa;
    pp[M.VN + vbase + tid] = ta;
  }
}

inline unsigned nblk(size_t n, unsigned per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

#define DISPATCH_AT(bf16, KERNEL, grid, block, stream, ...)                                       \
  do {                                                                                            \
    if (bf16) hipLaunchKernelGGL((KERNEL<bf16_t>), grid, block, 0, stream, __VA_ARGS__);          \
    else hipLaunchKernelGGL((KERNEL<float>), grid, block, 0, stream, __VA_ARGS__);                \
    return hipGetLastError();                                                                     \
  } while (0)

// col_part must hold ceil(B / 8) * 256 floats; db_o's second stage is queued in rb
hipError_t fade_loss_grad(const WinSrc &ws, const uint8_t *targets, long long tstride, int B, const float *probs, UpdateState *u, float beta1,
                          float beta2, void *dl, float *col_part, float *dbo, bool bf16, ReduceBatch &rb, hipStream_t s) {
  const int P = (B + 7) / 8;
  if (bf16) hipLaunchKernelGGL(loss_grad_kernel<bf16_t>, dim3(P), dim3(256), 0, s, ws, targets, tstride, B, probs, u, beta1, beta2, static_cast<bf16_t *>(dl), col_part);
  else hipLaunchKernelGGL(loss_grad_kernel<float>, dim3(P), dim3(256), 0, s, ws, targets, tstride, B, probs, u, beta1, beta2, static_cast<float *>(dl), col_part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return rb.push(P, 256, col_part, dbo) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t fade_transpose(const TransposeArgs &a, int N, bool bf16, hipStream_t s) {
  if (N % 64) return hipErrorInvalidValue;
  DISPATCH_AT(bf16, transpose_kernel, dim3((a.B + 63) / 64, N / 64), dim3(256), s, a);
}
hipError_t fade_ln_apply(const LnApplyBatch &lb, bool bf16, hipStream_t s) {
  if (lb.count < 0 || lb.count > 2 || (lb.count == 0 && !lb.with_loss) || lb.Dh % 8 || lb.Dh < 64) return hipErrorInvalidValue;
  const int rpt = fade_rows_per_thread((long long)lb.B * (lb.count ? lb.count : 1), lb.Dh / 8);
  unsigned gx = lb.count ? nblk((size_t)((lb.B + rpt - 1) / rpt) * (lb.Dh / 8), 256) : 1;
  if (lb.with_loss && gx < (unsigned)((lb.B + 7) / 8)) gx = (unsigned)((lb.B + 7) / 8);
  const dim3 grid(gx, lb.count + (lb.with_loss ? 1 : 0));
  if (rpt == 4) {
    if (bf16) hipLaunchKernelGGL((ln_apply_kernel<bf16_t, 4>), grid, dim3(256), 0, s, lb);
    else hipLaunchKernelGGL((ln_apply_kernel<float, 4>), grid, dim3(256), 0, s, lb);
  } else {
    if (bf16) hipLaunchKernelGGL((ln_apply_kernel<bf16_t, 1>), grid, dim3(256), 0, s, lb);
    else hipLaunchKernelGGL((ln_apply_kernel<float, 1>), grid, dim3(256), 0, s, lb);
  }
  return hipGetLastError();
}
hipError_t fade_transpose_batch(const TransposeBatch &tb, bool bf16, hipStream_t s) {
  if (tb.count <= 0 || tb.count > 8) return hipErrorInvalidValue;
  int maxB = 0, maxN = 0;
  for (int i = 0; i < tb.count; ++i) {
    if (tb.N[i] % 64) return hipErrorInvalidValue;
    if (tb.t[i].B > maxB) maxB = tb.t[i].B;
    if (tb.N[i] > maxN) maxN = tb.N[i];
  }
  const dim3 grid((maxB + 63) / 64, maxN / 64, tb.count);
  if (bf16) hipLaunchKernelGGL(transpose_batch_kernel<bf16_t>, grid, dim3(256), 0, s, tb);
  else hipLaunchKernelGGL(transpose_batch_kernel<float>, grid, dim3(256), 0, s, tb);
  return hipGetLastError();
}
hipError_t fade_embed_t(const WinSrc &ws, int B, int Bp, int T, int D, const void *tab, void *XT, bool bf16, hipStream_t s) {
  const size_t n = (size_t)T * D * (Bp / 8);
  if (bf16) hipLaunchKernelGGL(embed_t_kernel<bf16_t>, dim3(nblk(n, 256)), dim3(256), 0, s, ws, B, Bp, T, D, static_cast<const bf16_t *>(tab), static_cast<bf16_t *>(XT));
  else hipLaunchKernelGGL(embed_t_kernel<float>, dim3(nblk(n, 256)), dim3(256), 0, s, ws, B, Bp, T, D, static_cast<const float *>(tab), static_cast<float *>(XT));
  return hipGetLastError();
}
#define DISPATCH_ROWS(bf16, KERNEL, B, stream, args)                                                                             \
  do {                                                                                                                            \
    const int R_ = rows_per_block(B), RG_ = R_ * row_groups(B);                                                                   \
    auto args_ = args;                                                                                                            \
    args_.groups = row_groups(B);                                                                                                 \
    const dim3 grid_((B + RG_ - 1) / RG_);                                                                                        \
    if (bf16) {                                                                                                                   \
      if (R_ == 1) hipLaunchKernelGGL((KERNEL<bf16_t, 1>), grid_, dim3(256), 0, stream, args_);                                    \
      else if (R_ == 2) hipLaunchKernelGGL((KERNEL<bf16_t, 2>), grid_, dim3(256), 0, stream, args_);                               \
      else hipLaunchKernelGGL((KERNEL<bf16_t, 4>), grid_, dim3(256), 0, stream, args_);                                            \
    } else {                                                                                                                      \
      if (R_ == 1) hipLaunchKernelGGL((KERNEL<float, 1>), grid_, dim3(256), 0, stream, args_);                                     \
      else if (R_ == 2) hipLaunchKernelGGL((KERNEL<float, 2>), grid_, dim3(256), 0, stream, args_);                                \
      else hipLaunchKernelGGL((KERNEL<float, 4>), grid_, dim3(256), 0, stream, args_);                                             \
    }                                                                                                                             \
    return hipGetLastError();                                                                                                     \
  } while (0)
hipError_t fade_bwd_out(const BwdOutArgs &a, bool bf16, hipStream_t s) { DISPATCH_ROWS(bf16, bwd_out_kernel, a.B, s, a); }
hipError_t fade_bwd_geglu(int B, int De, const void *dHexp, const void *eg, const void *ev, void *dE, bool bf16, hipStream_t s) {
  const size_t n = (size_t)B * (De / 8);
  if (bf16) hipLaunchKernelGGL(bwd_geglu_kernel<bf16_t>, dim3(nblk(n, 256)), dim3(256), 0, s, B, De, static_cast<const bf16_t *>(dHexp), static_cast<const bf16_t *>(eg), static_cast<const bf16_t *>(ev), static_cast<bf16_t *>(dE));
  else hipLaunchKernelGGL(bwd_geglu_kernel<float>, dim3(nblk(n, 256)), dim3(256), 0, s, B, De, static_cast<const float *>(dHexp), static_cast<const float *>(eg), static_cast<const float *>(ev), static_cast<float *>(dE));
  return hipGetLastError();
}
hipError_t fade_bwd_gate(const BwdGateArgs &a, bool bf16, hipStream_t s) { DISPATCH_ROWS(bf16, bwd_gate_kernel, a.B, s, a); }
hipError_t fade_bwd_mix(const BwdMixArgs &a, bool bf16, hipStream_t s) { DISPATCH_ROWS(bf16, bwd_mix_kernel, a.B, s, a); }
int fade_rows_per_block(int B) { return rows_per_block(B) * row_groups(B); }
hipError_t fade_reduce_batch(const ReduceBatch &rb, hipStream_t s) {
  if (rb.count <= 0) return hipSuccess;
  int maxN = 0;
  for (int i = 0; i < rb.count; ++i) maxN = rb.N[i] > maxN ? rb.N[i] : maxN;
  hipLaunchKernelGGL(reduce_batch_kernel, dim3(nblk((size_t)maxN, 32), rb.count), dim3(1024), 0, s, rb);
  return hipGetLastError();
}
hipError_t fade_bwd_cci(const BwdCciArgs &a, bool bf16, hipStream_t s) { DISPATCH_AT(bf16, bwd_cci_kernel, dim3(a.B), dim3(256), s, a); }
// a.part must hold ceil(B / 4) * 2 * D * c floats; dWgv points at W_g's gradient (W_v's follows it in the blob)
hipError_t fade_bwd_slot(const BwdSlotArgs &a, float *dWgv, bool bf16, ReduceBatch &rb, hipStream_t s) {
  if (a.Dh > 2048 || a.Dh % 8 || a.c > 256 || a.D > 64) return hipErrorInvalidValue;
  const bool narrow = a.Dh <= 512;  // one chunk per lane: room for 4 streams per wavefront
  const int P = narrow ? (a.B + 15) / 16 : (a.B + 3) / 4;
  if (narrow) {
    if (bf16) hipLaunchKernelGGL((bwd_slot_kernel<bf16_t, 4, 1>), dim3(P), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((bwd_slot_kernel<float, 4, 1>), dim3(P), dim3(256), 0, s, a);
  } else {
    if (bf16) hipLaunchKernelGGL((bwd_slot_kernel<bf16_t, 1, 4>), dim3(P), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((bwd_slot_kernel<float, 1, 4>), dim3(P), dim3(256), 0, s, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return rb.push(P, 2 * a.D * a.c, a.part, dWgv) ? hipSuccess : hipErrorInvalidValue;
}
// Both of the above in one launch (bf16, D = 32, the matrix-core conv kernel with its input gradient).
hipError_t fade_bwd_slot_conv(const BwdSlotArgs &sa, float *dWgv, const ConvGradArgs &ca, float *dWb, ReduceBatch &rb, hipStream_t s) {
  if (sa.Dh > 2048 || sa.Dh % 8 || sa.c > 256 || sa.D > 64) return hipErrorInvalidValue;
  if (ca.D != 32 || 128 % ca.T || ca.T < 4 || ca.taps > 4 || !ca.WT || !ca.dxl || ca.Kc % 16 || ca.Kc > 128 || ca.taps * 32 > ca.Kc) return hipErrorInvalidValue;
  const bool narrow = sa.Dh <= 512;
  // narrow rows with wide slots (the paper-default shape: D_h = 512, c = 256): a stream's element-wise part and its share of
  // the partial sums are long, so two streams per wavefront instead of four (twice the workgroups)
  static const int spw_env = env_int("FADE_SLOT_SPW");
  const int spw = narrow ? ((spw_env == 2 || spw_env == 4) ? spw_env : (sa.c >= 64 ? 2 : 4)) : 1;
  const int Ps = (sa.B + 4 * spw - 1) / (4 * spw);
  const long long nchunks = ((long long)ca.B * ca.T + 127) / 128;
  const int Pc = (int)(nchunks < 512 ? nchunks : 512);
  if (spw == 4) hipLaunchKernelGGL((slot_conv_kernel<4, 1>), dim3(Ps + Pc), dim3(256), 0, s, sa, ca, Pc);
  else if (spw == 2) hipLaunchKernelGGL((slot_conv_kernel<2, 1>), dim3(Ps + Pc), dim3(256), 0, s, sa, ca, Pc);
  else hipLaunchKernelGGL((slot_conv_kernel<1, 4>), dim3(Ps + Pc), dim3(256), 0, s, sa, ca, Pc);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!rb.push(Ps, 2 * sa.D * sa.c, sa.part, dWgv) || !rb.push(Pc, (ca.taps * ca.D + 1) * ca.D, ca.part, dWb)) return hipErrorInvalidValue;
  return hipSuccess;
}
// a.part must hold ceil(B * T / 128) * (taps * D + 1) * D floats; dWb points at W_conv's gradient (b_conv's follows it)
hipError_t fade_conv_grad(const ConvGradArgs &a, float *dWb, bool bf16, ReduceBatch &rb, hipStream_t s) {
  if (256 % a.D || a.D > 32 || a.D < 16 || 128 % a.T || a.T < 4 || a.taps > 4 || (a.taps * a.D + 256 / a.D - 1) / (256 / a.D) > 16) return hipErrorInvalidValue;
  const long long nchunks = ((long long)a.B * a.T + 127) / 128;
  const int P = (int)(nchunks < 512 ? nchunks : 512);  // 128-token chunks are dealt round-robin to at most 512 workgroups
  if (a.WT && (!bf16 || a.D != 32 || !a.dxl || a.Kc % 16 || a.Kc > 128 || a.taps * 32 > a.Kc)) return hipErrorInvalidValue;
  if (bf16 && a.D == 32) hipLaunchKernelGGL(conv_grad_mfma_kernel, dim3(P), dim3(256), 0, s, a);
  else if (bf16) hipLaunchKernelGGL(conv_grad_partial_kernel<bf16_t>, dim3(P), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(conv_grad_partial_kernel<float>, dim3(P), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return rb.push(P, (a.taps * a.D + 1) * a.D, a.part, dWb) ? hipSuccess : hipErrorInvalidValue;
}
// a.part: nblocks * 2 * 256 * D floats; contrib: 256 * 4 * D.
// dE: gradient of the embedding; dparams: gradient of gamma_e (beta_e, gamma_l, beta_l follow it in the blob).
hipError_t fade_bwd_embed(const BwdTokenArgs &a, int nblocks, float *contrib, float *dE, float *dparams, bool bf16, ReduceBatch &rb,
                          hipStream_t s) {
  if (256 % a.D || a.D > 32 || a.D % 8) return hipErrorInvalidValue;
  if (a.D != 16 && a.D != 32) return hipErrorInvalidValue;
  const long long tokens = (long long)a.B * a.T;
  const int per = (int)(((tokens + nblocks - 1) / nblocks + 127) / 128 * 128);  // whole 128-token chunks per workgroup
  // D = 32 in bf16: eight wavefronts of one 32-symbol row tile each (twice the wavefronts per compute unit for the same
  // number of partial tables; B = 16384: 96 -> 89 us)
  if (bf16) {
    if (a.D == 32) hipLaunchKernelGGL((symbol_sums_mfma_kernel<bf16_t, 32, 512>), dim3(nblocks), dim3(512), 0, s, a, per);
    else hipLaunchKernelGGL((symbol_sums_mfma_kernel<bf16_t, 16, 256>), dim3(nblocks), dim3(256), 0, s, a, per);
  } else {
    if (a.D == 32) hipLaunchKernelGGL((symbol_sums_mfma_kernel<float, 32, 256>), dim3(nblocks), dim3(256), 0, s, a, per);
    else hipLaunchKernelGGL((symbol_sums_mfma_kernel<float, 16, 256>), dim3(nblocks), dim3(256), 0, s, a, per);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the second stage of the per-symbol sums happens inside the finishing kernel
  hipLaunchKernelGGL(embed_finish_kernel, dim3(256), dim3(256), 0, s, a.D, nblocks, a.part, a.tabXhat, a.tabRstd, a.gamma_e, a.gamma_l, dE, contrib);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return rb.push(256, 4 * a.D, contrib, dparams) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t fade_adam_refresh(const AdamRefreshBatch &ab, hipStream_t s) {
  if (ab.count <= 0 || ab.count > 10) return hipErrorInvalidValue;
  for (int i = 0; i < ab.count; ++i)
    if (ab.m[i].K % 64 || ab.m[i].N % 64 || ab.m[i].off % 4 || ab.m[i].vstride % 64 || ab.m[i].vcol0 % 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(adam_refresh_kernel, dim3(ab.total_blocks), dim3(256), 0, s, ab);
  return hipGetLastError();
}
