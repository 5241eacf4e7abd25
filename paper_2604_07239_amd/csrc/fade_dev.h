// fade_dev.h — types shared by the HIP translation units of libfade (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Where the context windows come from: stream b's window is the T bytes ending just before symbol i,
// i.e. base + b * stride + (i - T). n is the total byte count (streams past the end are inactive).
struct WinSrc {
  const uint8_t *base;
  long long stride;        // bytes between consecutive streams
  long long n;             // total bytes (stream b is active at step i iff b * stride + i < n and i < stride)
  const uint8_t *active;   // optional explicit mask [B]; overrides the rule above when non-NULL
  long long i;             // index of the symbol being coded in every stream
};

__device__ __forceinline__ bool stream_active(const WinSrc &w, int b) {
  if (w.active) return w.active[b] != 0;
  const long long i = w.i;
  return i < w.stride && (long long)b * w.stride + i < w.n;
}
__device__ __forceinline__ const uint8_t *stream_window(const WinSrc &w, int b, int T) {
  return w.base + (long long)b * w.stride + (w.i - T);
}

// ---------------------------------------------------------------------------------------------------
// prologue (how the A operand of a product is formed) and epilogue (what happens to the accumulator)
// ---------------------------------------------------------------------------------------------------
enum {
  PRO_PLAIN = 0,   // A[m][k]
  PRO_LN,          // (A[m][k] - mean_m) * rstd_m * gamma[k] + beta[k]          (LN of Eq. 7 / Eq. 9)
  PRO_FINAL,       // psi(LN(A)[m][k]) + lam * A2[m][k]                          (Eq. 10, feeding the head)
  PRO_CONV,        // row (b, j): concat over taps r of XL[b][j-(k-1)+r][:], zero where the index is negative (Eq. 4)
  PRO_CONVT,       // backward of Eq. 4 w.r.t. its input: row (b, j): concat over taps r of dY[b][j+(k-1)-r][:], zero past T-1
};
enum {
  EPI_STORE = 0,   // C = acc                                   (+ optional row statistics for a following LN)
  EPI_STORE_F32,   // C (fp32) = acc + bias
  EPI_GLOBAL,      // C = psi(acc) + lam * S1                   (Eq. 3; S1 = X)
  EPI_MIX,         // a = sigma(acc); C = a*S1 + (1-a)*S2       (Eq. 5-6; S1 = H_global, S2 = H_local)
  EPI_GATE,        // s = sigma(acc); C = S1*s + lam*S2         (Eq. 8; S1 = H_a, S2 = H_mix)
  EPI_GEGLU,       // C = psi(acc_gate) * acc_value             (Eq. 9; gate/value interleaved per 128 columns)
  EPI_CONV,        // C = psi(acc + bias[n])                    (Eq. 4)
  EPI_PARTIAL,     // C (fp32)[split][M][N] = acc of this block's K range (summed later in split order)
  EPI_GRAD,        // C (fp32) = acc: a weight gradient; with C3 set, columns interleaved per 128 go to the pair (C, C3)
  EPI_GEGLU_FOLD,  // EPI_GEGLU on a product of raw activations: the LayerNorm folded into W is finished here, per row
                   // (statistics of A) and per column (fold_s, fold_t), then C = psi(gate) * value; C2 / C3 = gate / value
};

// LN(h) W = rstd * (h W' - mean * s) + t for one output element (raw = h W'); one spelling for every kernel that finishes
// a folded LayerNorm, so that they agree to the bit.
__device__ __forceinline__ float fade_fold_ln(float raw, float mean, float rstd, float s, float t) {
  return fmaf(rstd, fmaf(-mean, s, raw), t);
}

struct GemmArgs {
  int M, N, K;            // C[M][N] = A'[M][K] * W[K][N]
  int splits;             // EPI_PARTIAL: number of K ranges (grid.y); 0 or 1 otherwise
  int sum_splits;         // EPI_PARTIAL, pipelined kernel: one workgroup takes all ranges in turn and writes the sum of their
                          // sums (added in range order) as the only partial
  // A operand
  const void *A;  int lda;
  int a_rows;             // row-major weight-gradient product: rows of A that exist (rows up to K are clamped to the last one)
  const void *A2;         // PRO_FINAL: residual source (same leading dimension)
  const float *stats;     // PRO_LN / PRO_FINAL: [M][stats_n][2] partial (sum, sum of squares) of A's rows
  int stats_n;
  const float *gamma, *beta;
  const float *lam;       // device scalar used by PRO_FINAL / EPI_GLOBAL / EPI_GATE
  int T, D, taps;         // PRO_CONV geometry
  // B operand: bf16 fragments in MFMA order (bf16 path) or plain fp32 [K][N] (fp32 path)
  const void *W;
  int ldb;                // pipelined kernel with a row-major B operand ([N][ldb], K contiguous); fp32 kernel with wt != 0
  int wt;                 // fp32 kernel: W is given transposed ([N][ldb]) instead of [K][N]
  // output
  void *C;  int ldc;
  void *C2, *C3;          // optional copies of pre-activation values for the backward pass
  const void *S1, *S2;    // side inputs [M][N] (leading dimension ldc)
  const float *bias;
  float *stats_out;       // optional [M][N / BN][2]
  const float *fold_s, *fold_t;  // EPI_GEGLU_FOLD: the folded LayerNorm's column vectors [N] (stats / stats_n: rows of A)
  int rows16;             // fp32 path: the small-batch kernel (16 x 16 tiles; row statistics per 16 columns instead of per 128)
  int col_groups;         // pipelined kernel: column ranges of the XCD split of the tile grid (1, 2, 4, 8; 0 = chosen by the launcher)
};

// A grouped launch: up to 4 independent products, each with the kernel body named by kind[]; blocks [first_block[p],
// first_block[p + 1]) work on problem p (tiles[p] output tiles x splits[p] ranges of K).
enum { GK_STORE_64x128 = 0, GK_STORE_64x64, GK_STORE_128x128, GK_PARTIAL_64x64, GK_PARTIAL_128x128, GK_TN_64x128, GK_TN_128x128, GK_TN_64x64 };
struct GemmGroup {
  int count;
  int kind[4], tiles[4], splits[4], first_block[5];
  GemmArgs g[4];
};

// Weight gradients on 256 x 256 tiles (gemm_tn2_kernel's body) of several matrices in ONE launch: blocks [first_block[p],
// first_block[p + 1]) are the tiles[p] x splits[p] workgroups of product p. A weight gradient feeds nothing but the
// optimiser, so the products of a whole backward pass can wait for its end; with one range count for all of them the
// workgroups are equally long and fill whole rounds of the chip.
struct Tn2Group {
  int count;
  int near;  // an XCD's units are consecutive ones (see tn2_block)
  int splits[8], first_block[9];
  GemmArgs g[8];
};

// Row statistics are accumulated per block tile of BN columns; consumers add the partials in index order.
#define FADE_STATS_BN 128

// (sum, sum of squares) partials of one row -> mean and 1 / sigma (biased variance, eps 1e-5). The pairs are fetched 16 at
// a time with no add between the loads (a loop of load-add-load-add would pay the memory latency once per pair); the adds
// run in index order, slots past stats_n add an exact zero.
__device__ __forceinline__ void fade_row_moments(const float *stats, int stats_n, int width, float &mean, float &rstd) {
  const float2 *p = reinterpret_cast<const float2 *>(stats);
  float s = 0.0f, q = 0.0f;
  for (int j0 = 0; j0 < stats_n; j0 += 16) {
    float2 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int idx = j0 + j;
      v[j] = p[idx < stats_n ? idx : stats_n - 1];
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const bool in = j0 + j < stats_n;
      s += in ? v[j].x : 0.0f;
      q += in ? v[j].y : 0.0f;
    }
  }
  const float inv = 1.0f / (float)width;
  mean = s * inv;
  // explicit product and fused multiply-add: this function is inlined into many kernels whose results must agree bit for
  // bit, which must not depend on which of the two products the compiler fuses with the subtraction
  rstd = 1.0f / sqrtf(fmaxf(fmaf(q, inv, -__fmul_rn(mean, mean)), 0.0f) + 1e-5f);
}

// Row-wise element kernels: thread t = blockIdx.x * 256 + tid owns the 8-wide chunk t % chunks of the RPT rows of row
// group t / chunks (RPT = 4 for tall inputs: one fetch of the per-column vectors serves 4 rows, whose loads are in flight
// together; RPT = 1 when there are too few rows to fill the chip that way). The moments of the rows a workgroup covers
// are formed once per row and shared through LDS instead of once per thread. mom must hold RPT * (256 / chunks + 2)
// rows (chunks >= 8: at most FADE_GROUP_ROWS_MAX). Returns the workgroup's first row; ends with a barrier.
#define FADE_GROUP_ROWS_MAX 136
template <int RPT>
__device__ __forceinline__ int fade_group_moments(const float *stats, int stats_n, int width, int chunks, int rows, float (*mom)[2]) {
  const long long t0 = (long long)blockIdx.x * 256;
  const int g0 = (int)(t0 / chunks), g1 = (int)((t0 + 255) / chunks);
  const int r0 = g0 * RPT, nr = (g1 - g0 + 1) * RPT;
  for (int r = threadIdx.x; r < nr; r += 256)
    if (r0 + r < rows) fade_row_moments(stats + (size_t)(r0 + r) * stats_n * 2, stats_n, width, mom[r][0], mom[r][1]);
  __syncthreads();
  return r0;
}
// rows per thread for `rows` rows of `chunks` chunks: 4 once that still leaves four workgroups for every compute unit
inline int fade_rows_per_thread(long long rows, int chunks) { return (rows / 4) * chunks / 256 >= 1024 ? 4 : 1; }

// ---------------------------------------------------------------------------------------------------
// activation arithmetic shared by every kernel (encoder and decoder run the same code, so they agree bit for bit)
// ---------------------------------------------------------------------------------------------------
// erf by the rational-times-Gaussian formula 7.1.26 of Abramowitz & Stegun (|error| <= 1.5e-7 absolute): the row kernels
// run one wavefront per SIMD and were bound by the library erff + expf (over a hundred instructions per element).
// The Gaussian e = exp(-x^2) is passed in because GeLU's derivative needs the same exponential.
__device__ __forceinline__ float fade_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }
__device__ __forceinline__ float fade_erf_pos(float ax, float e) {  // ax >= 0, e = exp(-ax^2)
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  return fmaf(-p * t, e, 1.0f);
}
// Phi(x) = (1 + erf(x / sqrt 2)) / 2 and the Gaussian g = exp(-x^2 / 2)
__device__ __forceinline__ float fade_norm_cdf(float x, float &g) {
  const float ax = fabsf(x) * 0.70710678118654752f;
  g = fade_exp(-ax * ax);
  const float er = fade_erf_pos(ax, g);
  return 0.5f * (1.0f + copysignf(er, x));
}
__device__ __forceinline__ float fade_gelu(float x) {  // psi(x) = x Phi(x) (exact-erf GeLU)
  float g;
  return x * fade_norm_cdf(x, g);
}
__device__ __forceinline__ float fade_gelu_grad(float x) {  // psi'(x) = Phi(x) + x phi(x)
  float g;
  const float cdf = fade_norm_cdf(x, g);
  return fmaf(x * 0.3989422804014327f, g, cdf);
}
// psi(x) and psi'(x) from one evaluation of Phi and the Gaussian
__device__ __forceinline__ float fade_gelu_both(float x, float &grad) {
  float g;
  const float cdf = fade_norm_cdf(x, g);
  grad = fmaf(x * 0.3989422804014327f, g, cdf);
  return x * cdf;
}
__device__ __forceinline__ float fade_sigmoid(float x) { return __builtin_amdgcn_rcpf(1.0f + fade_exp(-x)); }
