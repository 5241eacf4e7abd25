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
};

struct GemmArgs {
  int M, N, K;            // C[M][N] = A'[M][K] * W[K][N]
  int splits;             // EPI_PARTIAL: number of K ranges (grid.y); 0 or 1 otherwise
  // A operand
  const void *A;  int lda;
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
};

// Row statistics are accumulated per block tile of BN columns; consumers add the partials in index order.
#define FADE_STATS_BN 128
