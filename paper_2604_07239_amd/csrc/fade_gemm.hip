// fade_gemm.hip — the dense products of the model step with fused prologues and epilogues (gfx950).
//
// bf16 path: C[M][N] = A[M][K] * W[K][N] on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//   * Both operands stream global -> LDS by LDS-DMA (global_load_lds_dwordx4) through a ring of stages synchronised by
//     hand (s_waitcnt vmcnt + a bare s_barrier); A is row-major with its 16-byte pieces XOR-permuted in LDS, W was
//     rearranged at load time into MFMA fragment order (1 KiB per 32 columns x 16 k, contiguous along K).
//     pipe_body: 4 wavefronts, tiles of 64 / 128 rows x 64 / 128 columns, stages of 64 along K (small and medium batches,
//     grouped launches, split-K partials). pipe2_body: 8 wavefronts on a 256 x 256 tile, ring of four 32-wide stages with
//     the stage hand-over between the two k-steps of a stage (large batches). Fragment reads go through inline assembly
//     with hand-placed lgkmcnt waits, so that the next k-step's reads stay in flight under the matrix instructions.
//   * gemm_bf16_kernel forms A on the fly instead (the causal-conv row gather; Eq. 10's tail for the head product) and
//     stages it through LDS from registers; its W fragments go straight from L2 into registers.
//   * Weight gradients dW = L^T R contract over the batch: tn_body stages both row-major operands as they lie in memory
//     and turns them on the way out of LDS with the transposing read (ds_read_b64_tr_b16); 4 wavefronts on up to
//     128 x 128 inside grouped launches, 8 wavefronts on 256 x 256 as a launch of its own at large batches.
//   * The accumulators are parked in LDS (fp32; 64-row slabs for the 256-row tiles) and re-read row-wise, so that every
//     side input and every output moves in 16-byte pieces and per-row statistics for the next LayerNorm fall out of a
//     16-lane butterfly. Partial statistics are stored per 128-column tile and summed by the consumer in index order: no
//     atomics, so the result is reproducible bit for bit, and the same for every tile shape.
//   * blockIdx -> tile: the chip dispatches consecutive workgroups round-robin over its 8 XCDs, each with a private L2;
//     tile_of_block gives an XCD a range of column tiles (its share of W stays in its L2) and walks its tiles row by row.
// fp32 path: the same prologues / epilogues around a plain FMA core (gemm_f32_kernel), and 16 x 16 tiles with the
// contraction split over the workgroup's threads for batches of up to 256 rows (gemm_f32_rows_kernel).
#include <cstdlib>
#include <type_traits>

#include "fade_dev.h"
#include "fade_kernels.h"

int fade_gemm_tune();

namespace {

__device__ __forceinline__ float gelu_f(float x) { return fade_gelu(x); }
__device__ __forceinline__ float sigmoid_f(float x) { return fade_sigmoid(x); }

// 8 consecutive activations <-> registers
__device__ __forceinline__ void load8(const bf16_t *p, float v[8]) {
  const bf16x8 r = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)r[i];
}
__device__ __forceinline__ void load8(const float *p, float v[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
}
__device__ __forceinline__ void store8(bf16_t *p, const float v[8]) {
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (bf16_t)v[i];
  *reinterpret_cast<bf16x8 *>(p) = r;
}
__device__ __forceinline__ void store8(float *p, const float v[8]) {
  f32x4 a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
  *reinterpret_cast<f32x4 *>(p) = a;
  *reinterpret_cast<f32x4 *>(p + 4) = b;
}

// ---------------------------------------------------------------------------------------------------
// A-operand staging: one thread owns one 8-wide chunk of one row per pass.
// ---------------------------------------------------------------------------------------------------
template <typename AT> struct Raw8 { float v[8]; };
template <> struct Raw8<bf16_t> { bf16x8 v; };

template <typename AT> __device__ __forceinline__ void raw_zero(Raw8<AT> &r);
template <> __device__ __forceinline__ void raw_zero<bf16_t>(Raw8<bf16_t> &r) {
#pragma unroll
  for (int i = 0; i < 8; ++i) r.v[i] = (bf16_t)0.0f;
}
template <> __device__ __forceinline__ void raw_zero<float>(Raw8<float> &r) {
#pragma unroll
  for (int i = 0; i < 8; ++i) r.v[i] = 0.0f;
}
__device__ __forceinline__ void raw_load(Raw8<bf16_t> &r, const bf16_t *p) { r.v = *reinterpret_cast<const bf16x8 *>(p); }
__device__ __forceinline__ void raw_load(Raw8<float> &r, const float *p) { load8(p, r.v); }
__device__ __forceinline__ void raw_to_float(const Raw8<bf16_t> &r, float v[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)r.v[i];
}
__device__ __forceinline__ void raw_to_float(const Raw8<float> &r, float v[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = r.v[i];
}

// Issue the global loads for chunk (row m, columns k..k+7) of the A operand.
template <int PRO, typename AT>
__device__ __forceinline__ void stage_load(const GemmArgs &g, int m, int k, Raw8<AT> &a, Raw8<AT> &a2) {
  const AT *A = static_cast<const AT *>(g.A);
  if (m >= g.M) { raw_zero(a); if (PRO == PRO_FINAL) raw_zero(a2); return; }
  if (PRO == PRO_CONV) {
    const int b = m / g.T, j = m - b * g.T;
    const int tap = k / g.D, i = k - tap * g.D;
    const int tok = j - (g.taps - 1) + tap;
    if (tap < g.taps && tok >= 0) raw_load(a, A + ((size_t)b * g.T + tok) * g.D + i);
    else raw_zero(a);
  } else if (PRO == PRO_CONVT) {
    const int b = m / g.T, j = m - b * g.T;
    const int tap = k / g.D, i = k - tap * g.D;
    const int tok = j + (g.taps - 1) - tap;
    if (tap < g.taps && tok < g.T) raw_load(a, A + ((size_t)b * g.T + tok) * g.D + i);
    else raw_zero(a);
  } else {
    raw_load(a, A + (size_t)m * g.lda + k);
    if (PRO == PRO_FINAL) raw_load(a2, static_cast<const AT *>(g.A2) + (size_t)m * g.lda + k);
  }
}

// Turn the loaded chunk into operand values.
template <int PRO, typename AT>
__device__ __forceinline__ void stage_transform(const GemmArgs &g, int k, const Raw8<AT> &a, const Raw8<AT> &a2,
                                                float mean, float rstd, float lam, float v[8]) {
  raw_to_float(a, v);
  if (PRO == PRO_LN || PRO == PRO_FINAL) {
    float ga[8], be[8];
    load8(g.gamma + k, ga);
    load8(g.beta + k, be);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = fmaf(__fmul_rn(v[i] - mean, rstd), ga[i], be[i]);
    if (PRO == PRO_FINAL) {
      float r[8];
      raw_to_float(a2, r);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = fmaf(lam, r[i], gelu_f(v[i]));
    }
  }
}

// The same with the LayerNorm gain / shift of the chunk already in registers (requested together with the chunk itself).
template <int PRO, typename AT>
__device__ __forceinline__ void stage_transform_gb(const Raw8<AT> &a, const Raw8<AT> &a2, float mean, float rstd, float lam,
                                                   const float ga[8], const float be[8], float v[8]) {
  raw_to_float(a, v);
  if (PRO == PRO_LN || PRO == PRO_FINAL) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = fmaf(__fmul_rn(v[i] - mean, rstd), ga[i], be[i]);
    if (PRO == PRO_FINAL) {
      float r[8];
      raw_to_float(a2, r);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = fmaf(lam, r[i], gelu_f(v[i]));
    }
  }
}

// mean / rstd of row m from the partial sums its producer left behind (fixed summation order).
__device__ __forceinline__ void row_moments(const GemmArgs &g, int m, float &mean, float &rstd) {
  mean = 0.0f; rstd = 1.0f;
  if (m >= g.M) return;
  fade_row_moments(g.stats + (size_t)m * g.stats_n * 2, g.stats_n, g.K, mean, rstd);
}

// ---------------------------------------------------------------------------------------------------
// epilogue: the accumulator tile sits in LDS as fp32 [BM][BN + 4]; threads walk it in 8-wide row chunks
// ---------------------------------------------------------------------------------------------------
// Side inputs an epilogue reads beside the accumulator: 2 for the mix and gate forms, 1 for the global projection.
template <int EPI> struct EpiSides { static constexpr int n = (EPI == EPI_MIX || EPI == EPI_GATE) ? 2 : (EPI == EPI_GLOBAL ? 1 : 0); };

// Issue the global loads of one 8-wide chunk of the side inputs (element offset o); the values stay raw until used.
template <int EPI, typename AT>
__device__ __forceinline__ void epi_side_load(const GemmArgs &g, size_t o, bool live, Raw8<AT> *sd) {
  if (!live) return;
  if (EpiSides<EPI>::n >= 1) raw_load(sd[0], static_cast<const AT *>(g.S1) + o);
  if (EpiSides<EPI>::n >= 2) raw_load(sd[1], static_cast<const AT *>(g.S2) + o);
}

// The arithmetic below is written with explicit fused multiply-adds and unfusable products (fmaf, __fmul_rn): instances of
// this function for different tile shapes must give the same bits (a pass over many steps and a single step use different
// ones), which must not depend on where the compiler chooses to contract a * b + c.
// A thread walks rows r0, r0 + RP, ... of its 8-wide column chunk. The side inputs (and the row moments of the folded
// form) of U consecutive passes are requested together before the first of them is used, so that one memory latency
// covers U rows; with PRE the caller has requested them even earlier (`pre`: [pass][input], all BM / RP passes).
// ALL: every row of the tile exists (M is a multiple of the tile height): the stores then sit behind no branch. The counter
// of outstanding memory operations is in order and covers stores; for a load older than stores that sit in branches the
// compiler's wait count assumes the branches not taken, so the wait for the next slab's side inputs would also wait for
// this slab's stores to be acknowledged.
template <int EPI, typename AT, int BM, int BN, int LDC = BN + 4, int NT = 256, bool PRE = false, bool ALL = false>
__device__ __forceinline__ void epilogue(const GemmArgs &g, const float *Cs, int m0, int n0, int nt, int tid, int split = 0,
                                         const Raw8<AT> (*pre)[2] = nullptr) {
  constexpr bool kGeglu = EPI == EPI_GEGLU || EPI == EPI_GEGLU_FOLD;
  constexpr int BNO = kGeglu ? BN / 2 : BN;  // output columns of this tile
  constexpr int CH = BNO / 8;                            // chunks (threads) per row
  constexpr int RP = NT / CH;                            // rows per pass
  constexpr int PASSES = (BM + RP - 1) / RP;
  constexpr int NS = EpiSides<EPI>::n;
  constexpr bool kAhead = NS > 0 || EPI == EPI_GEGLU_FOLD;
  constexpr int U = PRE ? PASSES : (kAhead ? (PASSES < 4 ? PASSES : 4) : 1);
  constexpr bool kRagged = BM % (RP * U) != 0;  // a tile shorter than one round of passes: some threads own no row
  static_assert(PASSES % U == 0 && !(PRE && kRagged), "row passes");
  const int c8 = (tid % CH) * 8, r0 = tid / CH;
  const int nout0 = kGeglu ? nt * BNO : n0;  // first output column of the tile
  float lam = 0.0f;
  if (EPI == EPI_GLOBAL || EPI == EPI_GATE) lam = g.lam[0];
  float sg[8], tg[8], sv[8], tv[8];
  if (EPI == EPI_GEGLU_FOLD) {
    load8(g.fold_s + n0 + c8, sg); load8(g.fold_t + n0 + c8, tg);
    load8(g.fold_s + n0 + BNO + c8, sv); load8(g.fold_t + n0 + BNO + c8, tv);
  }
#pragma unroll 1
  for (int rb = r0; rb < BM; rb += RP * U) {
    Raw8<AT> own[PRE ? 1 : U][2];
    float mean[U], rstd[U];
    if (!PRE) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int m = m0 + rb + u * RP;
        if (kRagged && rb + u * RP >= BM) continue;
        // past the last row: any row (dropped below); a branch around the loads would cost the exact vmcnt waits
        epi_side_load<EPI, AT>(g, (size_t)(m < g.M ? m : g.M - 1) * g.ldc + nout0 + c8, true, own[u]);
        if (EPI == EPI_GEGLU_FOLD) row_moments(g, m, mean[u], rstd[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
    const Raw8<AT> *sd = PRE ? pre[u] : own[u];
    const int r = rb + u * RP;
    if (kRagged && r >= BM) continue;
    const int m = m0 + r;
    const bool live = ALL || m < g.M;
    float x[8], out[8];
    load8(Cs + r * LDC + c8, x);
    const size_t o = (size_t)m * g.ldc + nout0 + c8;
    if (live) {
      if (EPI == EPI_STORE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = x[i];
        store8(static_cast<AT *>(g.C) + o, out);
      } else if (EPI == EPI_STORE_F32) {
        float bi[8];
        if (g.bias) load8(g.bias + n0 + c8, bi);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = g.bias ? x[i] + bi[i] : x[i];
        store8(static_cast<float *>(g.C) + o, out);
      } else if (EPI == EPI_GLOBAL) {
        float s1[8];
        raw_to_float(sd[0], s1);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = fmaf(lam, s1[i], gelu_f(x[i]));
        store8(static_cast<AT *>(g.C) + o, out);
        if (g.C2) store8(static_cast<AT *>(g.C2) + o, x);
      } else if (EPI == EPI_MIX) {
        float s1[8], s2[8], al[8];
        raw_to_float(sd[0], s1);
        raw_to_float(sd[1], s2);
#pragma unroll
        for (int i = 0; i < 8; ++i) { al[i] = sigmoid_f(x[i]); out[i] = fmaf(al[i], s1[i], __fmul_rn(1.0f - al[i], s2[i])); }
        store8(static_cast<AT *>(g.C) + o, out);
        if (g.C2) store8(static_cast<AT *>(g.C2) + o, al);
      } else if (EPI == EPI_GATE) {
        float s1[8], s2[8], sgm[8];
        raw_to_float(sd[0], s1);
        raw_to_float(sd[1], s2);
#pragma unroll
        for (int i = 0; i < 8; ++i) { sgm[i] = sigmoid_f(x[i]); out[i] = fmaf(lam, s2[i], __fmul_rn(s1[i], sgm[i])); }
        store8(static_cast<AT *>(g.C) + o, out);
        if (g.C2) store8(static_cast<AT *>(g.C2) + o, sgm);
      } else if (EPI == EPI_GEGLU) {
        float xv[8];
        load8(Cs + r * LDC + BNO + c8, xv);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = gelu_f(x[i]) * xv[i];
        store8(static_cast<AT *>(g.C) + o, out);
        if (g.C2) store8(static_cast<AT *>(g.C2) + o, x);
        if (g.C3) store8(static_cast<AT *>(g.C3) + o, xv);
      } else if (EPI == EPI_GEGLU_FOLD) {
        float xv[8], eg[8], ev[8];
        load8(Cs + r * LDC + BNO + c8, xv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          eg[i] = fade_fold_ln(x[i], mean[u], rstd[u], sg[i], tg[i]);
          ev[i] = fade_fold_ln(xv[i], mean[u], rstd[u], sv[i], tv[i]);
          out[i] = gelu_f(eg[i]) * ev[i];
        }
        store8(static_cast<AT *>(g.C) + o, out);
        if (g.C2) store8(static_cast<AT *>(g.C2) + o, eg);
        if (g.C3) store8(static_cast<AT *>(g.C3) + o, ev);
      } else if (EPI == EPI_GRAD) {  // split: partial sum over one range of the batch, slices [split][M][width] behind each other
        if (g.C3) {
          const int v = n0 + c8;
          float *dstp = ((v & 127) < 64) ? static_cast<float *>(g.C) : static_cast<float *>(g.C3);
          store8(dstp + ((size_t)split * g.M + m) * (g.N / 2) + (v / 128) * 64 + (v & 63), x);
        } else {
          store8(static_cast<float *>(g.C) + (size_t)split * g.M * g.ldc + o, x);
        }
      } else if (EPI == EPI_PARTIAL) {
        store8(static_cast<float *>(g.C) + ((size_t)split * g.M + m) * g.ldc + n0 + c8, x);
      } else if (EPI == EPI_CONV) {
        float bi[8], pre_act[8];
        load8(g.bias + n0 + c8, bi);
#pragma unroll
        for (int i = 0; i < 8; ++i) { pre_act[i] = x[i] + bi[i]; out[i] = gelu_f(pre_act[i]); }
        store8(static_cast<AT *>(g.C) + o, out);
        if (g.C2) store8(static_cast<AT *>(g.C2) + o, pre_act);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] = 0.0f;
    }
    if (g.stats_out && (EPI == EPI_STORE || EPI == EPI_MIX || EPI == EPI_GATE)) {
      float s = 0.0f, q = 0.0f;
#pragma unroll
      for (int i = 0; i < 8; ++i) { s += out[i]; q = fmaf(out[i], out[i], q); }
#pragma unroll
      for (int off = CH / 2; off > 0; off >>= 1) { s += __shfl_xor(s, off, 64); q += __shfl_xor(q, off, 64); }
      if (ALL) {  // every lane of the row's group holds the sums: all store them (same value, same address), no branch
        float *p = g.stats_out + ((size_t)m * (g.N / BN) + nt) * 2;
        *reinterpret_cast<float2 *>(p) = make_float2(s, q);
      } else if (live && (tid % CH) == 0) {
        float *p = g.stats_out + ((size_t)m * (g.N / BN) + nt) * 2;
        p[0] = s; p[1] = q;
      }
    }
    }
  }
}

// Block -> tile. Workgroups are dealt to the 8 XCDs round-robin (bid % 8), and each XCD has its own L2: the XCDs split
// the tile grid into cg column ranges x (8 / cg) interleaved row sets, and one XCD walks its tiles row by row, so the
// tiles that run together share their A rows and the XCD's slice of W stays in its L2. cg = 8 suits a small A (every
// XCD streams all of A past its own eighth of W); a tall A wants fewer column ranges so that it is fetched cg times
// instead of 8. Returns false for the padding blocks of a grid rounded up to whole row sets.
__device__ __forceinline__ bool tile_of_block(int bid, int ntm, int ntn, int cg, int &mt, int &nt) {
  if (cg <= 0) cg = 8;
  if (ntn % cg == 0) {
    const int rg = 8 / cg, x = bid & 7, r = bid >> 3, per = ntn / cg;
    nt = (x % cg) * per + r % per;
    mt = (r / per) * rg + x / cg;
  } else {
    nt = bid % ntn;
    mt = bid / ntn;
  }
  return mt < ntm;
}

// ---------------------------------------------------------------------------------------------------
// bf16 MFMA core
// ---------------------------------------------------------------------------------------------------
// KEEP (PRO_FINAL, M a multiple of the tile height): the operand formed on the fly, H of Eq. 10, is also written to C2
// ([M][lda], the update needs it for the head's weight gradient). Its stores are unconditional and sit behind the request
// for the block after next, so that no load ever waits for them (the memory counter is in order and covers stores).
template <int WM, int WN, int TM, int TN, int PRO, int EPI, bool KEEP = false>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
  typedef bf16_t AT;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64, LDA = BK + 8, PASSES = BM / 32, LDC = BN + 4;
  static_assert(WM * WN == 4, "four wavefronts per workgroup");
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t *As = reinterpret_cast<bf16_t *>(smem);  // [2][BM][LDA]
  float *Cs = reinterpret_cast<float *>(smem);    // [BM][LDC], reuses the space after the K loop

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = g.N / BN, ntm = (g.M + BM - 1) / BM;
  int mt, nt;
  if (!tile_of_block(blockIdx.x, ntm, ntn, 8, mt, nt)) return;
  const int m0 = mt * BM, n0 = nt * BN;

  const int srow = tid >> 3, skc = (tid & 7) * 8;
  float mean[PASSES], rstd[PASSES];
  float lam = 0.0f;
  if (PRO == PRO_LN || PRO == PRO_FINAL) {
#pragma unroll
    for (int p = 0; p < PASSES; ++p) row_moments(g, m0 + p * 32 + srow, mean[p], rstd[p]);
    if (PRO == PRO_FINAL) lam = g.lam[0];
  }

  // EPI_PARTIAL: the contraction in ranges (grid.y), each leaving its own partial, or, with sum_splits, every range in
  // turn inside this workgroup with their sums added in range order: the same bits as separate partials added later
  const bool fuse = EPI == EPI_PARTIAL && g.sum_splits != 0;
  const int nsplit = EPI == EPI_PARTIAL ? (fuse ? g.splits : (int)gridDim.y) : 1;
  const int sp_first = fuse ? 0 : (int)blockIdx.y, sp_end = fuse ? nsplit : (int)blockIdx.y + 1;
  const int nkb = g.K / BK / nsplit, ksteps = g.K / 16;
  // fragment stream of this wavefront's first column tile
  const bf16x8 *Wf = static_cast<const bf16x8 *>(g.W) + ((size_t)((n0 + wn * TN * 32) / 32) * ksteps) * 64 + lane;

  f32x16 acc[TM][TN], tot[EPI == EPI_PARTIAL ? TM : 1][EPI == EPI_PARTIAL ? TN : 1];
  for (int sp = sp_first; sp < sp_end; ++sp) {
  const int kb0 = sp * nkb;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  Raw8<AT> ra[PASSES], ra2[PASSES];
  bf16x8 bcur[4][TN], bnext[4][TN];
  bf16x8 hkeep[KEEP ? PASSES : 1];  // KEEP: the block's transformed values as they went to LDS
  // LayerNorm gain / shift of this thread's 8 columns of the block: requested with the block's rows, not when they are used
  constexpr bool kGB = PRO == PRO_LN || PRO == PRO_FINAL;
  float ga[kGB ? 8 : 1], be[kGB ? 8 : 1];
  auto load_gb = [&](int k) {
    if constexpr (kGB) { load8(g.gamma + k, ga); load8(g.beta + k, be); }
  };

  // preamble: the range's first K block
#pragma unroll
  for (int p = 0; p < PASSES; ++p) stage_load<PRO, AT>(g, m0 + p * 32 + srow, kb0 * BK + skc, ra[p], ra2[p]);
  load_gb(kb0 * BK + skc);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int j = 0; j < TN; ++j) bcur[ks][j] = Wf[((size_t)j * ksteps + kb0 * 4 + ks) * 64];
  if (sp != sp_first) __syncthreads();  // the previous range's last block has been read
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    bf16_t *dst = As + (p * 32 + srow) * LDA + skc;
    if (PRO == PRO_PLAIN || PRO == PRO_CONV || PRO == PRO_CONVT) {
      *reinterpret_cast<bf16x8 *>(dst) = ra[p].v;
    } else {
      float v[8];
      if constexpr (kGB) stage_transform_gb<PRO, AT>(ra[p], ra2[p], mean[p], rstd[p], lam, ga, be, v);
      else stage_transform<PRO, AT>(g, kb0 * BK + skc, ra[p], ra2[p], mean[p], rstd[p], lam, v);
      store8(dst, v);
      if constexpr (KEEP) {
#pragma unroll
        for (int q = 0; q < 8; ++q) hkeep[p][q] = (bf16_t)v[q];
      }
    }
  }
  auto request = [&](int kb_abs) {  // rows, gain / shift and W fragments of K block kb_abs
    const int k1 = kb_abs * BK;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) stage_load<PRO, AT>(g, m0 + p * 32 + srow, k1 + skc, ra[p], ra2[p]);
    load_gb(k1 + skc);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int j = 0; j < TN; ++j) bnext[ks][j] = Wf[((size_t)j * ksteps + kb_abs * 4 + ks) * 64];
  };
  auto keep_store = [&](int kb_abs) {
    if constexpr (KEEP) {
#pragma unroll
      for (int p = 0; p < PASSES; ++p)
        *reinterpret_cast<bf16x8 *>(static_cast<AT *>(g.C2) + (size_t)(m0 + p * 32 + srow) * g.lda + kb_abs * BK + skc) = hkeep[p];
    }
  };
  if constexpr (KEEP) {
    if (nkb > 1) request(kb0 + 1);
    keep_store(kb0);
  }

  for (int kb = 0; kb < nkb; ++kb) {
    const bool more = kb + 1 < nkb;
    if (more && !KEEP) {
      const int k1 = (kb0 + kb + 1) * BK;
#pragma unroll
      for (int p = 0; p < PASSES; ++p) stage_load<PRO, AT>(g, m0 + p * 32 + srow, k1 + skc, ra[p], ra2[p]);
      load_gb(k1 + skc);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int j = 0; j < TN; ++j) bnext[ks][j] = Wf[((size_t)j * ksteps + (kb0 + kb + 1) * 4 + ks) * 64];
    }
    __syncthreads();
    const bf16_t *Ab = As + (kb & 1) * BM * LDA;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8 *>(Ab + ((wm * TM + i) * 32 + (lane & 31)) * LDA + ks * 16 + (lane >> 5) * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bcur[ks][j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      bf16_t *An = As + ((kb + 1) & 1) * BM * LDA;
      const int k1 = (kb0 + kb + 1) * BK;
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        bf16_t *dst = An + (p * 32 + srow) * LDA + skc;
        if (PRO == PRO_PLAIN || PRO == PRO_CONV || PRO == PRO_CONVT) {
          *reinterpret_cast<bf16x8 *>(dst) = ra[p].v;
        } else {
          float v[8];
          if constexpr (kGB) stage_transform_gb<PRO, AT>(ra[p], ra2[p], mean[p], rstd[p], lam, ga, be, v);
          else stage_transform<PRO, AT>(g, k1 + skc, ra[p], ra2[p], mean[p], rstd[p], lam, v);
          store8(dst, v);
          if constexpr (KEEP) {
#pragma unroll
        for (int q = 0; q < 8; ++q) hkeep[p][q] = (bf16_t)v[q];
      }
        }
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int j = 0; j < TN; ++j) bcur[ks][j] = bnext[ks][j];
      if constexpr (KEEP) {
        if (kb + 2 < nkb) request(kb0 + kb + 2);
        keep_store(kb0 + kb + 1);
      }
    }
  }
  if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (sp == sp_first) tot[i][j] = acc[i][j];
        else tot[i][j] += acc[i][j];
      }
  }
  }

  // park the accumulators: lane l of a 32x32 tile holds column l % 32, rows (e / 4) * 8 + (l / 32) * 4 + e % 4
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = (wm * TM + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        const int col = (wn * TN + j) * 32 + (lane & 31);
        if constexpr (EPI == EPI_PARTIAL) Cs[row * LDC + col] = tot[i][j][e];
        else Cs[row * LDC + col] = acc[i][j][e];
      }
  __syncthreads();
  epilogue<EPI, AT, BM, BN>(g, Cs, m0, n0, nt, tid, fuse ? 0 : (int)blockIdx.y);
}

// ---------------------------------------------------------------------------------------------------
// bf16 MFMA core, pipelined: both operands stream global -> LDS with the asynchronous LDS-DMA loads
// (global_load_lds_dwordx4: 16 bytes per lane land at M0-base + lane * 16, no registers involved), STAGES
// K blocks deep. Each 1 KiB DMA is one MFMA fragment (32 rows x 16 k): the lanes gather 16-byte row pieces
// of the row-major A (two lanes per 32-byte run) or read a ready-made fragment of W, so that the later
// ds_read_b128 of a fragment is one contiguous, conflict-free 1 KiB read. Synchronisation is by hand:
// s_waitcnt vmcnt(n) for this wavefront's own DMAs, then a bare s_barrier (a __syncthreads() would drain
// every outstanding load and with it the pipeline).
//   A: plain row-major bf16 [M][lda] (rows past M are clamped to row M-1 and never stored)
//   W: bf16 fragments as written by the weight preparation
//   grid.y > 1: split K, each block leaves an fp32 partial tile (EPI_PARTIAL)
// ---------------------------------------------------------------------------------------------------
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
__device__ __forceinline__ void bare_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void dma16(const bf16_t *src, unsigned char *lds_chunk) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                   (__attribute__((address_space(3))) void *)lds_chunk, 16, 0, 0);
}

// LDS fragment reads whose completion is waited for by hand: the compiler would wait for every outstanding read before the
// first matrix instruction of a group (s_waitcnt lgkmcnt(0)), also for the reads just issued for the next group. Reads issued
// through lds_read16 are invisible to it; lds_wait<N> lets the N youngest stay in flight (LDS returns in order) and
// lds_landed ties the value to the wait, so that no use can move above it.
template <int OFF> __device__ __forceinline__ bf16x8 lds_read16(uint32_t addr) {
  typedef __attribute__((ext_vector_type(4))) int i32x4;
  i32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return __builtin_bit_cast(bf16x8, v);
}
template <int N> __device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void lds_landed(bf16x8 &v) {
  typedef __attribute__((ext_vector_type(4))) int i32x4;
  i32x4 t = __builtin_bit_cast(i32x4, v);
  asm volatile("" : "+v"(t));
  v = __builtin_bit_cast(bf16x8, t);
}
// The same for gfx950's transposing read of four 16-bit values per lane (ds_read_b64_tr_b16); two of them make one operand.
typedef __attribute__((ext_vector_type(2))) int i32x2;
template <int OFF> __device__ __forceinline__ i32x2 tr_read8(uint32_t addr) {
  i32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
__device__ __forceinline__ void tr_landed(i32x2 &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ bf16x8 tr_pair(i32x2 lo, i32x2 hi) {
  typedef __attribute__((ext_vector_type(4))) int i32x4;
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
}

template <int BM, int BN, int STAGES, int EPI, bool BROW, int NW = 4>
__device__ __forceinline__ void pipe_body(const GemmArgs &g, int bid, int split, int nsplit) {
  typedef bf16_t AT;
  constexpr int BK = 64, KS = 4;
  constexpr int WN = NW / 2;                         // wavefronts 2 (rows) x WN (columns)
  constexpr int TM = BM / 64, TN = BN / (32 * WN);   // 32x32 tiles per wavefront
  constexpr int BFR = BN / 32;
  constexpr int A_BYTES = BM * 128;                  // A stage: BM rows of 64 k (128 bytes), 16-byte pieces XOR-swizzled
  constexpr int ACH = BM / 8 / NW;                   // A DMAs per wavefront and stage (one DMA = 8 rows x 128 bytes)
  constexpr int BCH = BROW ? BN / 8 / NW : BFR * KS / NW;  // W DMAs per wavefront and stage (one fragment, or 8 rows x 128 bytes)
  constexpr int LPW = ACH + BCH;
  constexpr int STAGE_BYTES = A_BYTES + BFR * KS * 1024, LDC = BN + 4;
  static_assert((BM / 8) % NW == 0 && (BFR * KS) % NW == 0 && (BN / 8) % NW == 0, "chunk split");
  static_assert((STAGES - 2) * LPW <= 63, "vmcnt range");
  extern __shared__ __align__(16) unsigned char smem[];
  float *Cs = reinterpret_cast<float *>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = g.N / BN, ntm = (g.M + BM - 1) / BM;
  int mt, nt;
  if (!tile_of_block(bid, ntm, ntn, g.col_groups, mt, nt)) return;
  const int m0 = mt * BM, n0 = nt * BN;
  const int ksplit = g.K / nsplit, nkb = ksplit / BK;
  const int ksteps = g.K / 16;

  // DMA sources of this wavefront for one stage.
  // A: DMA c covers rows 8c .. 8c+7; lane i fetches row r = 8c + i/8, 16-byte piece (i % 8) ^ ((r / 2) % 8): eight lanes
  //    read one 128-byte run of a row, and the XOR spreads the pieces that a later fragment read touches (16 rows
  //    x one piece per quarter-wavefront) over all 64 LDS banks.
  // W: DMA c is fragment c / 4 (32 columns), k-step c % 4, already contiguous.
  const bf16_t *src[LPW];
#pragma unroll
  for (int q = 0; q < ACH; ++q) {
    const int c = wave + NW * q;
    int row = m0 + c * 8 + (lane >> 3);
    row = row < g.M ? row : g.M - 1;
    const int sw = ((c * 8 + (lane >> 3)) >> 1) & 7;
    src[q] = static_cast<const bf16_t *>(g.A) + (size_t)row * g.lda + (((lane & 7) ^ sw) << 3);
  }
#pragma unroll
  for (int q = 0; q < BCH; ++q) {
    const int c = wave + NW * q;
    if (BROW) {  // row-major [N][ldb]: same 8-rows-per-DMA, XOR-swizzled scheme as A
      const int row = n0 + c * 8 + (lane >> 3);
      const int sw = ((c * 8 + (lane >> 3)) >> 1) & 7;
      src[ACH + q] = static_cast<const bf16_t *>(g.W) + (size_t)row * g.ldb + (((lane & 7) ^ sw) << 3);
    } else {
      const int fr = c / KS, ks = c % KS;
      src[ACH + q] = static_cast<const bf16_t *>(g.W) + (((size_t)(n0 / 32 + fr) * ksteps + ks) * 64 + lane) * 8;
    }
  }
  auto issue = [&](int slot, int kb) {  // kb: 64-wide k block counted from the start of K
    unsigned char *base = smem + slot * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < ACH; ++q) dma16(src[q] + (size_t)kb * BK, base + (wave + NW * q) * 1024);
#pragma unroll
    for (int q = 0; q < BCH; ++q) dma16(src[ACH + q] + (BROW ? (size_t)kb * BK : (size_t)kb * KS * 512), base + A_BYTES + (wave + NW * q) * 1024);
  };


  // fragment read offsets inside a stage: row r, k-step ks, half h -> r * 128 + (((2 ks + h) ^ ((r / 2) & 7)) * 16)
  // as LDS addresses of this lane per k-step (A tile i of the wavefront 4096 bytes = 32 rows further on; W fragment j
  // KS KiB further on, or 32 rows for a row-major W)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
  const int a_sw = (lane >> 1) & 7, a_half = lane >> 5;  // tile rows start at multiples of 32, so (r / 2) & 7 == (lane / 2) & 7
  uint32_t a_ks[KS], b_ks[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    a_ks[ks] = lds0 + (wm * TM * 32 + (lane & 31)) * 128 + (((2 * ks + a_half) ^ a_sw) << 4);
    b_ks[ks] = BROW ? lds0 + A_BYTES + (wn * TN * 32 + (lane & 31)) * 128 + (((2 * ks + a_half) ^ a_sw) << 4)
                    : lds0 + A_BYTES + (((wn * TN * KS) * 64 + lane) << 4);
  }

  // EPI_PARTIAL with sum_splits: this workgroup walks all K ranges itself and adds their sums in range order, which is
  // bit for bit what the reducing kernels make of separate partials; otherwise it owns the one range `split`.
  const bool fuse = EPI == EPI_PARTIAL && g.sum_splits != 0;
  const int sp_first = fuse ? 0 : split, sp_end = fuse ? nsplit : split + 1;
  f32x16 acc[TM][TN], tot[EPI == EPI_PARTIAL ? TM : 1][EPI == EPI_PARTIAL ? TN : 1];
  for (int sp = sp_first; sp < sp_end; ++sp) {
  const int kb0 = sp * nkb;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  if (sp != sp_first) bare_barrier();  // every wavefront has read the last stages of the previous range
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nkb) issue(s, kb0 + s);

  for (int kb = 0; kb < nkb; ++kb) {
    // stage kb must have landed; up to STAGES-2 younger stages may stay in flight
    if (kb + STAGES - 2 < nkb) wait_vmcnt<(STAGES - 2) * LPW>();
    else wait_vmcnt<0>();
    bare_barrier();  // everyone's part of stage kb is in LDS, and everyone is done reading stage kb-1
    if (kb + STAGES - 1 < nkb) issue((kb + STAGES - 1) % STAGES, kb0 + kb + STAGES - 1);
    // fragments of k-step ks+1 are fetched from LDS while the matrix cores work on k-step ks: reads through lds_read16 with
    // hand-placed waits (the compiler's own wait in front of a group of matrix instructions also covers the reads just issued
    // for the next group)
    const uint32_t st = (kb % STAGES) * STAGE_BYTES;
    bf16x8 af[2][TM], bf[2][TN];
    auto fetch = [&](auto buf_c, auto ks_c) {
      constexpr int buf = decltype(buf_c)::value, ks = decltype(ks_c)::value;
      static_assert(TM <= 4 && TN <= 4, "tiles per wavefront");
      const uint32_t sa = a_ks[ks] + st, sb = BROW ? b_ks[ks] + st : b_ks[0] + st;
      constexpr int BO = BROW ? 0 : ks * 1024, BS = BROW ? 4096 : KS * 1024;
      af[buf][0] = lds_read16<0>(sa);
      if constexpr (TM > 1) af[buf][1] = lds_read16<4096>(sa);
      if constexpr (TM > 2) af[buf][2] = lds_read16<8192>(sa);
      if constexpr (TM > 3) af[buf][3] = lds_read16<12288>(sa);
      bf[buf][0] = lds_read16<BO>(sb);
      if constexpr (TN > 1) bf[buf][1] = lds_read16<BO + BS>(sb);
      if constexpr (TN > 2) bf[buf][2] = lds_read16<BO + 2 * BS>(sb);
      if constexpr (TN > 3) bf[buf][3] = lds_read16<BO + 3 * BS>(sb);
    };
    auto mfma = [&](auto buf_c, auto newer_c) {  // newer: reads issued after this buffer's, allowed to stay in flight
      constexpr int buf = decltype(buf_c)::value;
      lds_wait<decltype(newer_c)::value>();
#pragma unroll
      for (int i = 0; i < TM; ++i) lds_landed(af[buf][i]);
#pragma unroll
      for (int j = 0; j < TN; ++j) lds_landed(bf[buf][j]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bf[buf][j], acc[i][j], 0, 0, 0);
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, 2> I2;
    typedef std::integral_constant<int, 3> I3;
    typedef std::integral_constant<int, TM + TN> INext;
    static_assert(KS == 4, "k-steps per stage");
    fetch(I0{}, I0{});
    fetch(I1{}, I1{});
    mfma(I0{}, INext{});
    fetch(I0{}, I2{});
    mfma(I1{}, INext{});
    fetch(I1{}, I3{});
    mfma(I0{}, INext{});
    mfma(I1{}, I0{});
  }
  if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (sp == sp_first) tot[i][j] = acc[i][j];
        else tot[i][j] += acc[i][j];
      }
  }
  }

  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = (wm * TM + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        const int col = (wn * TN + j) * 32 + (lane & 31);
        if constexpr (EPI == EPI_PARTIAL) Cs[row * LDC + col] = tot[i][j][e];
        else Cs[row * LDC + col] = acc[i][j][e];
      }
  __syncthreads();
  epilogue<EPI, AT, BM, BN>(g, Cs, m0, n0, nt, tid, fuse ? 0 : split);
}
template <int BM, int BN, int STAGES, int EPI, bool BROW>
__global__ __launch_bounds__(256, (STAGES == 2 && BM * BN <= 128 * 128) ? 2 : 1) void gemm_pipe_kernel(GemmArgs g) {
  pipe_body<BM, BN, STAGES, EPI, BROW>(g, (int)blockIdx.x, (int)blockIdx.y, g.sum_splits ? g.splits : (int)gridDim.y);
}


// ---------------------------------------------------------------------------------------------------
// The same product with stages of 32 along K (two k-steps) in a ring of STAGES: half the bytes per stage, so that the ring
// is deep enough (three stages ahead) for the LDS-DMA of all compute units together, which the L2 fabric serves at about
// 50 bytes per clock and unit, and so that the fragments of a stage's first k-step can be fetched from LDS while the matrix
// cores still work on the last k-step of the stage before: the wait for a stage's DMA and the workgroup barrier sit in
// the middle of a stage, between its two k-steps, and no fragment read is ever waited for with idle matrix cores.
//   iteration h:  fetch (h, k-step 1) | MFMA (h, 0) | wait DMA of h+1, barrier, issue DMA of h+STAGES-1 | fetch (h+1, 0) | MFMA (h, 1)
// A stage: A as BM rows of 64 bytes (one DMA = 16 rows; the four 16-byte pieces of row r XOR-permuted by (r / 4) % 4, so
// that the 16 rows a quarter-wavefront reads one piece of cover all 64 banks), then W as ready-made 1 KiB fragments.
// The slot that iteration h refills is the one stage h-1 lived in: its last fragment read was waited for before
// MFMA (h-1, 1) was issued, which every wavefront has done when it arrives at iteration h's barrier.
// Every output element sees the same sequence of k-steps as in pipe_body, so both give the same bits.
// ---------------------------------------------------------------------------------------------------
template <int BM, int BN, int STAGES, int EPI, int NW = 4>
__device__ __forceinline__ void pipe2_body(const GemmArgs &g, int bid, int split, int nsplit) {
  typedef bf16_t AT;
  constexpr int BK = 32, KS = 2;
  constexpr int WN = NW / 2;                         // wavefronts 2 (rows) x WN (columns)
  constexpr int TM = BM / 64, TN = BN / (32 * WN);   // 32x32 tiles per wavefront
  constexpr int BFR = BN / 32;
  constexpr int A_BYTES = BM * 64;                   // A stage: BM rows of 32 k (64 bytes)
  constexpr int ACH = BM / 16 / NW;                  // A DMAs per wavefront and stage (one DMA = 16 rows x 64 bytes)
  constexpr int BCH = BFR * KS / NW;                 // W DMAs per wavefront and stage (one fragment each)
  constexpr int LPW = ACH + BCH;
  constexpr int STAGE_BYTES = A_BYTES + BFR * KS * 1024, LDC = BN + 4;
  constexpr bool SLAB = BM > 128;                    // the fp32 tile leaves through LDS in slabs of 64 rows
  static_assert((BM / 16) % NW == 0 && (BFR * KS) % NW == 0 && STAGES >= 3, "chunk split");
  static_assert((STAGES - 3) * LPW <= 63, "vmcnt range");
  extern __shared__ __align__(16) unsigned char smem[];
  float *Cs = reinterpret_cast<float *>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = g.N / BN, ntm = (g.M + BM - 1) / BM;
  int mt, nt;
  if (!tile_of_block(bid, ntm, ntn, g.col_groups, mt, nt)) return;
  const int m0 = mt * BM, n0 = nt * BN;
  const int ksplit = g.K / nsplit, nkh = ksplit / BK;
  const int ksteps = g.K / 16;

  const bf16_t *src[LPW];
#pragma unroll
  for (int q = 0; q < ACH; ++q) {
    const int c = wave + NW * q, r = c * 16 + (lane >> 2);
    int row = m0 + r;
    row = row < g.M ? row : g.M - 1;
    src[q] = static_cast<const bf16_t *>(g.A) + (size_t)row * g.lda + (((lane & 3) ^ ((r >> 2) & 3)) << 3);
  }
#pragma unroll
  for (int q = 0; q < BCH; ++q) {
    const int c = wave + NW * q, fr = c / KS, ks = c % KS;
    src[ACH + q] = static_cast<const bf16_t *>(g.W) + (((size_t)(n0 / 32 + fr) * ksteps + ks) * 64 + lane) * 8;
  }
  auto issue = [&](int slot, int kh) {  // kh: 32-wide stage counted from the start of K
    unsigned char *base = smem + slot * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < ACH; ++q) dma16(src[q] + (size_t)kh * BK, base + (wave + NW * q) * 1024);
#pragma unroll
    for (int q = 0; q < BCH; ++q) dma16(src[ACH + q] + (size_t)kh * KS * 512, base + A_BYTES + (wave + NW * q) * 1024);
  };

  // fragment read addresses inside a stage (bytes from the stage's start): A tile i of this wavefront at a_base[k-step] +
  // i * 2048 (32 rows of 64 bytes), W tile j at b_base + k-step * 1024 + j * 2048
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
  const int a_sw = (lane >> 2) & 3, a_half = lane >> 5;  // tile rows start at multiples of 32: (r / 4) % 4 == (lane / 4) % 4
  uint32_t a_base[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) a_base[ks] = lds0 + (wm * TM * 32 + (lane & 31)) * 64 + (((2 * ks + a_half) ^ a_sw) << 4);
  const uint32_t b_base = lds0 + A_BYTES + (((wn * TN * KS) * 64 + lane) << 4);

  const bool fuse = EPI == EPI_PARTIAL && g.sum_splits != 0;
  const int sp_first = fuse ? 0 : split, sp_end = fuse ? nsplit : split + 1;
  f32x16 acc[TM][TN], tot[EPI == EPI_PARTIAL ? TM : 1][EPI == EPI_PARTIAL ? TN : 1];
  for (int sp = sp_first; sp < sp_end; ++sp) {
    const int kh0 = sp * nkh;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    if (sp != sp_first) bare_barrier();  // every wavefront has read the last stages of the previous range
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
      if (s < nkh) issue(s, kh0 + s);

    bf16x8 af[2][TM], bf[2][TN];
    auto fetch = [&](auto buf_c, int slot, auto ks_c) {  // TM + TN reads, left in flight
      constexpr int buf = decltype(buf_c)::value, ks = decltype(ks_c)::value;
      const uint32_t sa = a_base[ks] + slot * STAGE_BYTES, sb = b_base + slot * STAGE_BYTES;
      static_assert(TM <= 4 && TN <= 4, "tiles per wavefront");
      af[buf][0] = lds_read16<0>(sa);
      if constexpr (TM > 1) af[buf][1] = lds_read16<2048>(sa);
      if constexpr (TM > 2) af[buf][2] = lds_read16<4096>(sa);
      if constexpr (TM > 3) af[buf][3] = lds_read16<6144>(sa);
      bf[buf][0] = lds_read16<ks * 1024>(sb);
      if constexpr (TN > 1) bf[buf][1] = lds_read16<ks * 1024 + 2048>(sb);
      if constexpr (TN > 2) bf[buf][2] = lds_read16<ks * 1024 + 4096>(sb);
      if constexpr (TN > 3) bf[buf][3] = lds_read16<ks * 1024 + 6144>(sb);
    };
    auto mfma = [&](auto buf_c, auto newer_c) {  // newer: reads issued after this buffer's, allowed to stay in flight
      constexpr int buf = decltype(buf_c)::value;
      lds_wait<decltype(newer_c)::value>();
#pragma unroll
      for (int i = 0; i < TM; ++i) lds_landed(af[buf][i]);
#pragma unroll
      for (int j = 0; j < TN; ++j) lds_landed(bf[buf][j]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bf[buf][j], acc[i][j], 0, 0, 0);
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, TM + TN> INext;
    // stage 0 has landed once at most the younger stages of the preamble are in flight
    if (nkh >= STAGES - 1) wait_vmcnt<(STAGES - 2) * LPW>();
    else wait_vmcnt<0>();
    bare_barrier();
    fetch(I0{}, 0, I0{});
    int slot = 0, fill = STAGES - 1;  // slot of stage h; slot the next DMA goes to
    // One iteration: the two k-steps of stage h around the hand-over to stage h + 1. STEADY: a further stage is requested;
    // else the ring only drains.
    auto step = [&](int h, auto steady) {
      fetch(I1{}, slot, I1{});
      mfma(I0{}, INext{});
      if constexpr (decltype(steady)::value) wait_vmcnt<(STAGES - 3) * LPW>();
      else wait_vmcnt<0>();
      bare_barrier();  // stage h+1 is in LDS for everyone, and everyone is done reading stage h-1
      if constexpr (decltype(steady)::value) {
        issue(fill, kh0 + h + STAGES - 1);
        fill = fill + 1 == STAGES ? 0 : fill + 1;
      }
      slot = slot + 1 == STAGES ? 0 : slot + 1;
      fetch(I0{}, slot, I0{});
      mfma(I1{}, INext{});
    };
    int h = 0;
    for (; h + STAGES - 1 < nkh; ++h) step(h, std::true_type{});
    for (; h + 1 < nkh; ++h) step(h, std::false_type{});
    fetch(I1{}, slot, I1{});  // last stage: nothing follows
    mfma(I0{}, INext{});
    mfma(I1{}, I0{});
    if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (sp == sp_first) tot[i][j] = acc[i][j];
          else tot[i][j] += acc[i][j];
        }
    }
  }

  wait_vmcnt<0>();
  if constexpr (SLAB) {
    // The fp32 tile does not fit LDS at once: it leaves in slabs of 64 rows, each handed to the epilogue as 128-column
    // pieces (the width the row statistics are kept at), so every output is formed exactly as by the smaller tiles.
    // (a GeGLU tile is gate | value per 128 columns, so each 128-column piece is a complete pair)
    static_assert(EPI != EPI_PARTIAL && TM % 2 == 0 && BN % 128 == 0, "slab epilogue");
    constexpr int NT = NW * 64, SP = 64 / (NT / 16);     // passes of a thread over a 64-row, 128-column slab piece
    // With one workgroup on the unit (eight wavefronts) the side inputs of slab p + 1 are requested before slab p is worked
    // on; with two workgroups per unit the other one's matrix work covers that latency and the registers are not spent.
    constexpr bool PRE = NW == 8 && EpiSides<EPI>::n != 0;
    Raw8<AT> sd[PRE ? 2 : 1][BN / 128][SP][2];
    auto side = [&](int buf, int p) {
      if constexpr (PRE) {
#pragma unroll
        for (int h = 0; h < BN / 128; ++h)
#pragma unroll
          for (int u = 0; u < SP; ++u) {
            int m = m0 + p * 64 + u * (NT / 16) + tid / 16;
            m = m < g.M ? m : g.M - 1;  // past the last row: any row (the epilogue drops it); no branch around the loads
            epi_side_load<EPI, AT>(g, (size_t)m * g.ldc + n0 + h * 128 + (tid % 16) * 8, true, sd[buf][h][u]);
          }
      }
    };
    side(0, 0);
#pragma unroll
    for (int p = 0; p < BM / 64; ++p) {
      constexpr int ROWS_PER_WAVE = 32 * TM;
      const int owner = (p * 64) / ROWS_PER_WAVE, i0 = ((p * 64) % ROWS_PER_WAVE) / 32;
      if (p + 1 < BM / 64) side((p + 1) & 1, p + 1);
      __syncthreads();  // the ring, or the previous slab, is no longer being read
      if (wm == owner) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int row = ii * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
              const int col = (wn * TN + j) * 32 + (lane & 31);
              Cs[row * LDC + col] = acc[i0 + ii][j][e];
            }
      }
      __syncthreads();
#pragma unroll
      for (int h = 0; h < BN / 128; ++h)
        epilogue<EPI, AT, 64, 128, LDC, NT, PRE, NW == 8>(g, Cs + h * 128, m0 + p * 64, n0 + h * 128, nt * (BN / 128) + h, tid, 0, sd[PRE ? (p & 1) : 0][h]);
    }
  } else {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = (wm * TM + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
          const int col = (wn * TN + j) * 32 + (lane & 31);
          if constexpr (EPI == EPI_PARTIAL) Cs[row * LDC + col] = tot[i][j][e];
          else Cs[row * LDC + col] = acc[i][j][e];
        }
    __syncthreads();
    epilogue<EPI, AT, BM, BN>(g, Cs, m0, n0, nt, tid, fuse ? 0 : split);
  }
}
// WPU: workgroups the launch bounds leave room for on one compute unit
template <int BM, int BN, int STAGES, int EPI, int NW, int WPU>
__global__ __launch_bounds__(NW * 64, WPU) void gemm_pipe2_kernel(GemmArgs g) {
  pipe2_body<BM, BN, STAGES, EPI, NW>(g, (int)blockIdx.x, (int)blockIdx.y, g.sum_splits ? g.splits : (int)gridDim.y);
}

// ---------------------------------------------------------------------------------------------------
// Weight gradients from ROW-MAJOR operands: C[M][N] = sum over rows b < K of A[b][m] * W[b][n]  (dW = L^T R over the batch;
// A = a forward activation [a_rows][lda], W = a gradient [K][ldb] whose rows past the batch are zero).
// The contraction index is the row index, which the matrix cores want contiguous per lane; instead of keeping transposed
// copies of all sixteen operands in HBM, the turn happens on the way out of LDS. A stage holds 64 rows of BM (BN) columns
// as they are in memory (LDS-DMA, 1 KiB = 8 rows x 128 bytes or 4 rows x 256 bytes per instruction), and fragments are
// read with gfx950's transposing LDS load (ds_read_b64_tr_b16): within each group of 16 lanes, lane s supplies the
// address of 4 consecutive 16-bit values, and lane i receives value (i % 4) of the lanes i / 4, i / 4 + 4, i / 4 + 8,
// i / 4 + 12 (layout checked on the hardware). Pointing lane s at row s / 4, columns 4 (s % 4) .. + 3 of a 4 x 16 block
// therefore hands lane i column i of the block with its 4 rows in order: two such loads give a lane the 8 contraction
// rows of its column, which is the operand layout of v_mfma_f32_32x32x16_bf16.
// Bank conflicts: one load touches 4 rows x 64 contiguous bytes per 32 lanes; with a row pitch of 128 (256) bytes those
// rows would share banks, so the 16-byte pieces of a row are XOR-permuted by a function of the row (below) such that
// 4 consecutive rows land in 4 different quarter-ranges of the 64 banks.
// ---------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
// piece permutation of row r in a stage whose rows are PITCH bytes long
template <int PITCH> __device__ __forceinline__ int tn_swizzle(int r) {
  static_assert(PITCH == 128 || PITCH == 256 || PITCH == 512, "row pitch");
  return PITCH >= 256 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2);  // 512: the permutation stays inside a row's 256-byte half
}

// NW wavefronts as 2 (rows) x NW / 2 (columns); a 256 x 256 tile on eight of them hands its fp32 result to the epilogue in
// slabs of 64 rows (as pipe2_body does), half the operand bytes and three quarters of the LDS reads per flop of 128 x 128.
template <int BM, int BN, int STAGES, int NW = 4>
__device__ __forceinline__ void tn_body(const GemmArgs &g, int bid, int split = 0, int nsplit = 1, int mt_in = -1, int nt_in = -1) {
  typedef bf16_t AT;
  constexpr int BK = 64, KS = 4;
  constexpr int WN = NW / 2;
  constexpr int TM = BM / 64, TN = BN / (32 * WN);
  constexpr int PA = BM / 8, PB = BN / 8;          // 16-byte pieces per row
  constexpr int RA = 64 / PA, RB = 64 / PB;        // rows per DMA
  constexpr int A_BYTES = BK * BM * 2, B_BYTES = BK * BN * 2;
  constexpr int ACH = BK / RA / NW, BCH = BK / RB / NW;  // DMAs per wavefront and stage
  constexpr int LPW = ACH + BCH, STAGE_BYTES = A_BYTES + B_BYTES, LDC = BN + 4;
  static_assert(PA >= 8 && PB >= 8 && (BK / RA) % NW == 0 && (BK / RB) % NW == 0 && BN % (32 * WN) == 0, "tile shape");
  static_assert((STAGES - 2) * LPW <= 63, "vmcnt range");
  extern __shared__ __align__(16) unsigned char smem[];
  float *Cs = reinterpret_cast<float *>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = g.N / BN, ntm = g.M / BM;
  int mt = mt_in, nt = nt_in;
  if (mt_in < 0 && !tile_of_block(bid, ntm, ntn, 8, mt, nt)) return;
  const int m0 = mt * BM, n0 = nt * BN;
  const int nkb = g.K / BK / nsplit, kb0 = split * nkb;  // this workgroup's range of the contraction (the batch)

  // DMA c of an operand covers rows c * R .. c * R + R - 1 of the stage; lane i lands at byte 16 i of that KiB, i.e. at
  // (row, piece) = (c * R + i / P, i % P), and fetches the piece whose index is XORed as described above.
  int a_row[ACH], b_row[BCH];
  const bf16_t *a_col[ACH], *b_src[BCH];
#pragma unroll
  for (int q = 0; q < ACH; ++q) {
    const int row = (wave + NW * q) * RA + lane / PA, piece = (lane % PA) ^ tn_swizzle<BM * 2>(row);
    a_row[q] = row;
    a_col[q] = static_cast<const bf16_t *>(g.A) + m0 + piece * 8;
  }
#pragma unroll
  for (int q = 0; q < BCH; ++q) {
    const int row = (wave + NW * q) * RB + lane / PB, piece = (lane % PB) ^ tn_swizzle<BN * 2>(row);
    b_row[q] = row;
    b_src[q] = static_cast<const bf16_t *>(g.W) + (size_t)row * g.ldb + n0 + piece * 8;
  }
  const int last_a = g.a_rows - 1;
  auto issue = [&](int slot, int kb) {
    unsigned char *base = smem + slot * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < ACH; ++q) {
      int r = kb * BK + a_row[q];
      r = r < last_a ? r : last_a;  // past the batch: any finite row, its partner row of W is zero
      dma16(a_col[q] + (size_t)r * g.lda, base + (wave + NW * q) * 1024);
    }
#pragma unroll
    for (int q = 0; q < BCH; ++q) dma16(b_src[q] + (size_t)kb * BK * g.ldb, base + A_BYTES + (wave + NW * q) * 1024);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nkb) issue(s, kb0 + s);

  // address this lane supplies to the transposing loads of k-step 0 (first of the two loads; the second is 4 rows on):
  // row 8 * (lane / 32) + (lane % 16) / 4, columns tile * 32 + 16 * ((lane / 16) % 2) + 4 * (lane % 4) .. + 3
  const int s16 = lane & 15, r0 = (lane >> 5) * 8 + (s16 >> 2), mh = (lane >> 4) & 1;
  int a_off[TM], b_off[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
    a_off[i] = r0 * (BM * 2) + ((((wm * TM + i) * 4 + 2 * mh + ((s16 & 3) >> 1)) ^ tn_swizzle<BM * 2>(r0)) << 4) + (s16 & 1) * 8;
#pragma unroll
  for (int j = 0; j < TN; ++j)
    b_off[j] = A_BYTES + r0 * (BN * 2) + ((((wn * TN + j) * 4 + 2 * mh + ((s16 & 3) >> 1)) ^ tn_swizzle<BN * 2>(r0)) << 4) + (s16 & 1) * 8;
  // rows 4 and 16 further on have the same (r & 3) and the same ((r >> 1) & 1): the permutation term does not change

  // The transposing reads go through inline assembly with hand-placed waits (tr_read8 / lds_wait / tr_landed): issued through
  // the builtin, the compiler orders every one of them behind the LDS-DMA just requested for the next stage
  // (s_waitcnt vmcnt(0) in front of the first read), which exposes a full memory latency per stage.
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
  for (int kb = 0; kb < nkb; ++kb) {
    if (kb + STAGES - 2 < nkb) wait_vmcnt<(STAGES - 2) * LPW>();
    else wait_vmcnt<0>();
    bare_barrier();
    if (kb + STAGES - 1 < nkb) issue((kb + STAGES - 1) % STAGES, kb0 + kb + STAGES - 1);
    const uint32_t st = lds0 + (kb % STAGES) * STAGE_BYTES;
    i32x2 alo[2][TM], ahi[2][TM], blo[2][TN], bhi[2][TN];
    auto fetch = [&](auto buf_c, auto ks_c) {
      constexpr int buf = decltype(buf_c)::value, ks = decltype(ks_c)::value;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        alo[buf][i] = tr_read8<ks * 16 * (BM * 2)>(st + a_off[i]);
        ahi[buf][i] = tr_read8<ks * 16 * (BM * 2) + 4 * (BM * 2)>(st + a_off[i]);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        blo[buf][j] = tr_read8<ks * 16 * (BN * 2)>(st + b_off[j]);
        bhi[buf][j] = tr_read8<ks * 16 * (BN * 2) + 4 * (BN * 2)>(st + b_off[j]);
      }
    };
    auto mfma = [&](auto buf_c, auto newer_c) {  // newer: reads issued after this buffer's, allowed to stay in flight
      constexpr int buf = decltype(buf_c)::value;
      lds_wait<decltype(newer_c)::value>();
      bf16x8 af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) { tr_landed(alo[buf][i]); tr_landed(ahi[buf][i]); af[i] = tr_pair(alo[buf][i], ahi[buf][i]); }
#pragma unroll
      for (int j = 0; j < TN; ++j) { tr_landed(blo[buf][j]); tr_landed(bhi[buf][j]); bf[j] = tr_pair(blo[buf][j], bhi[buf][j]); }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, 2> I2;
    typedef std::integral_constant<int, 3> I3;
    typedef std::integral_constant<int, 2 * (TM + TN)> INext;
    static_assert(KS == 4 && 2 * (TM + TN) <= 15, "k-steps per stage; lgkmcnt range");
    fetch(I0{}, I0{});
    fetch(I1{}, I1{});
    mfma(I0{}, INext{});
    fetch(I0{}, I2{});
    mfma(I1{}, INext{});
    fetch(I1{}, I3{});
    mfma(I0{}, INext{});
    mfma(I1{}, I0{});
  }

  wait_vmcnt<0>();
  if constexpr (BM > 128) {
    static_assert(TM % 2 == 0 && BN % 128 == 0, "slab epilogue");
#pragma unroll
    for (int p = 0; p < BM / 64; ++p) {
      constexpr int ROWS_PER_WAVE = 32 * TM;
      const int owner = (p * 64) / ROWS_PER_WAVE, i0 = ((p * 64) % ROWS_PER_WAVE) / 32;
      __syncthreads();  // the ring, or the previous slab, is no longer being read
      if (wm == owner) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int row = ii * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
              const int col = (wn * TN + j) * 32 + (lane & 31);
              Cs[row * LDC + col] = acc[i0 + ii][j][e];
            }
      }
      __syncthreads();
#pragma unroll
      for (int h = 0; h < BN / 128; ++h)
        epilogue<EPI_GRAD, AT, 64, 128, LDC, NW * 64>(g, Cs + h * 128, m0 + p * 64, n0 + h * 128, nt * (BN / 128) + h, tid, split);
    }
  } else {
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = (wm * TM + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        const int col = (wn * TN + j) * 32 + (lane & 31);
        Cs[row * LDC + col] = acc[i][j][e];
      }
  __syncthreads();
  epilogue<EPI_GRAD, AT, BM, BN>(g, Cs, m0, n0, nt, tid, split);
  }
}
template <int BM, int BN, int STAGES>
__global__ __launch_bounds__(256) void gemm_tn_kernel(GemmArgs g) {
  tn_body<BM, BN, STAGES>(g, (int)blockIdx.x);
}
// 256 x 256 tiles on eight wavefronts, one workgroup per compute unit; blockIdx.y is the range of the batch.
// Workgroups go to the eight XCDs round-robin and each XCD has its own L2: an XCD takes whole units of eight workgroups,
// a unit being a block of 2 x 4 tiles of one range of the batch (2 + 4 operand panels for 8 tiles; one row or column of
// tiles would need 1 + 8).
// near: an XCD's units are consecutive ones (unit = tile block within a range, ranges outermost), so the units it runs
// side by side are neighbouring tile blocks of one range and share operand panels in its L2 (D_h x D_h over four ranges:
// an XCD's four units are 4 x 8 tiles of one range, 4 + 8 panels for 32 tiles instead of 4 x (2 + 4)).
__device__ __forceinline__ void tn2_block(const GemmArgs &g, int bid, int nsplit, bool near) {
  const int ntm = g.M / 256, ntn = g.N / 256, tiles = ntm * ntn;
  if (ntm % 2 == 0 && ntn % 4 == 0 && (tiles / 8 * nsplit) % 8 == 0) {
    const int x = bid & 7, r = bid >> 3, w = r & 7, U = tiles / 8;
    const int u = near ? x * (U * nsplit / 8) + (r >> 3) : x + 8 * (r >> 3), b = u % U, split = u / U;
    tn_body<256, 256, 2, 8>(g, 0, split, nsplit, (b / (ntn / 4)) * 2 + (w >> 2), (b % (ntn / 4)) * 4 + (w & 3));
  } else {
    tn_body<256, 256, 2, 8>(g, bid % tiles, bid / tiles, nsplit);
  }
}
__global__ __launch_bounds__(512, 1) void gemm_tn2_kernel(GemmArgs g, int nsplit) { tn2_block(g, (int)blockIdx.x, nsplit, false); }
// The same for several matrices in one launch (Tn2Group). Where every product's block count is a multiple of 8 (all the
// shapes of the benchmark configurations), a block's position within its product goes to the same XCD as in a launch of
// its own; otherwise only the L2 reuse of the later products suffers.
__global__ __launch_bounds__(512, 1) void gemm_tn2_group_kernel(Tn2Group tg) {
  int p = 0;
  while (p + 1 < tg.count && (int)blockIdx.x >= tg.first_block[p + 1]) ++p;
  tn2_block(tg.g[p], (int)blockIdx.x - tg.first_block[p], tg.splits[p], tg.near != 0);
}

// Several independent products in ONE launch (a block-uniform switch picks the problem and its kernel body): the products
// of one backward phase (dX = dY W^T, dW = L^T dY, ...) consume the same gradient and do not depend on each other, and at
// B = 1024 none of them fills the chip alone.
template <int STAGES>
__device__ __forceinline__ void group_body(const GemmGroup &gg) {
  int p = 0;
  while (p + 1 < gg.count && (int)blockIdx.x >= gg.first_block[p + 1]) ++p;
  const int local = (int)blockIdx.x - gg.first_block[p], tiles = gg.tiles[p];
  const GemmArgs &g = gg.g[p];
  switch (gg.kind[p]) {
    case GK_STORE_64x128:   pipe_body<64, 128, STAGES, EPI_STORE, false>(g, local, 0, 1); break;
    case GK_STORE_128x128:  pipe_body<128, 128, STAGES, EPI_STORE, false>(g, local, 0, 1); break;
    case GK_STORE_64x64:    pipe_body<64, 64, STAGES, EPI_STORE, false>(g, local, 0, 1); break;
    case GK_PARTIAL_64x64:  pipe_body<64, 64, STAGES, EPI_PARTIAL, false>(g, local % tiles, local / tiles, gg.splits[p]); break;
    case GK_PARTIAL_128x128: pipe_body<128, 128, STAGES, EPI_PARTIAL, false>(g, local % tiles, local / tiles, gg.splits[p]); break;
    case GK_TN_64x128:      tn_body<64, 128, STAGES>(g, local % tiles, local / tiles, gg.splits[p]); break;
    case GK_TN_128x128:     tn_body<128, 128, STAGES>(g, local % tiles, local / tiles, gg.splits[p]); break;
    case GK_TN_64x64:       tn_body<64, 64, STAGES>(g, local % tiles, local / tiles, gg.splits[p]); break;
    default: break;
  }
}
__global__ __launch_bounds__(256) void gemm_group_kernel(GemmGroup gg) { group_body<4>(gg); }
// The same with two-stage rings and at most 256 registers: two workgroups share a compute unit, so one's pipeline fill and
// epilogue run under the other's products. For groups with workgroups enough to use that (large batches).
__global__ __launch_bounds__(256, 2) void gemm_group2_kernel(GemmGroup gg) { group_body<2>(gg); }


// ---------------------------------------------------------------------------------------------------
// fp32 FMA core: 256 threads, each owning 8 consecutive columns of one row; tile (2048 / BN) x BN,
// K blocks of 32; W is plain [K][N] fp32
// ---------------------------------------------------------------------------------------------------
template <int BN, int PRO, int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  typedef float AT;
  constexpr int CHN = BN / 8, BM = 256 / CHN, BK = 32, LDC = BN + 4;
  constexpr int NCH = (BM * 4 + 255) / 256;  // A chunks staged per thread
  __shared__ __align__(16) float As[BM][BK + 4];
  __shared__ __align__(16) float Ws[BK][BN];
  __shared__ __align__(16) float Cs[BM * LDC];
  const int tid = threadIdx.x;
  const int ntn = g.N / BN;
  const int nt = blockIdx.x % ntn, mt = blockIdx.x / ntn;
  const int m0 = mt * BM, n0 = nt * BN;
  const int r = tid / CHN, cg = (tid % CHN) * 8;  // this thread's output row and first column
  float mean[NCH], rstd[NCH], lam = 0.0f;
#pragma unroll
  for (int q = 0; q < NCH; ++q) {
    mean[q] = 0.0f; rstd[q] = 1.0f;
    const int c = q * 256 + tid;
    if ((PRO == PRO_LN || PRO == PRO_FINAL) && c < BM * 4) row_moments(g, m0 + (c >> 2), mean[q], rstd[q]);
  }
  if (PRO == PRO_FINAL) lam = g.lam[0];
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
  const float *W = static_cast<const float *>(g.W);
  for (int k0 = 0; k0 < g.K; k0 += BK) {
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
      const int c = q * 256 + tid;
      if (c < BM * 4) {
        const int srow = c >> 2, skc = (c & 3) * 8;
        Raw8<AT> a, a2;
        stage_load<PRO, AT>(g, m0 + srow, k0 + skc, a, a2);
        float v[8];
        stage_transform<PRO, AT>(g, k0 + skc, a, a2, mean[q], rstd[q], lam, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) As[srow][skc + i] = v[i];
      }
    }
    if (g.wt) {  // W given as [N][ldb]: rows are output columns, K contiguous
      for (int idx = tid; idx < BK * BN; idx += 256) {
        const int c = idx / BK, kk = idx % BK;
        Ws[kk][c] = W[(size_t)(n0 + c) * g.ldb + k0 + kk];
      }
    } else {
      for (int idx = tid; idx < BK * BN / 4; idx += 256) {
        const int kk = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
        *reinterpret_cast<f32x4 *>(&Ws[kk][c4]) = *reinterpret_cast<const f32x4 *>(W + (size_t)(k0 + kk) * g.N + n0 + c4);
      }
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < BK; ++kk) {
      const float a = As[r][kk];
      const f32x4 w0 = *reinterpret_cast<const f32x4 *>(&Ws[kk][cg]), w1 = *reinterpret_cast<const f32x4 *>(&Ws[kk][cg + 4]);
#pragma unroll
      for (int i = 0; i < 4; ++i) { acc[i] = fmaf(a, w0[i], acc[i]); acc[4 + i] = fmaf(a, w1[i], acc[4 + i]); }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) Cs[r * LDC + cg + i] = acc[i];
  __syncthreads();
  epilogue<EPI, AT, BM, BN>(g, Cs, m0, n0, nt, tid);
}

// ---------------------------------------------------------------------------------------------------
// fp32 products of very small batches (the 16-stream configuration): 16 rows x 16 columns per workgroup, the whole
// contraction inside it. With 16 rows a 128-column tile leaves four workgroups on a 256-unit chip walking K in lock step
// (50 us for a 16 x 512 x 512 product); here N / 16 workgroups each keep the 16 operand rows in LDS (prologue applied
// once) and split K 64 ways: thread (q, cg) owns the terms k = q, q + 64, ... of all 16 rows for 4 of the tile's columns,
// so every weight element is loaded once per workgroup (a lane's row pieces are requested up front, before the operand
// rows are staged: one round trip for K <= 512), the operand values come from LDS (a wavefront reads 16 consecutive k of
// one row: conflict-free, each value broadcast to the 4 column groups). The 64 K slices are added in a fixed tree: inside
// a wavefront a butterfly over the slice bits of the lane index that halves the rows a lane keeps at every level (lane
// bit 5 decides rows 0-7 / 8-15, bit 4 the half of those, ...: 32 + 16 + 8 + 4 exchanges instead of 4 x 64), then the four
// wavefronts' sums in wavefront order through LDS. A step streams the weights (4 MB for that configuration) once.
// GeGLU tiles take 8 gate and the matching 8 value columns of a 128-column group (columns c and c + 64).
// Row statistics are left per 16-column tile: consumers must be told stats_n = N / 16.
// ---------------------------------------------------------------------------------------------------
template <int PRO, int EPI>
__global__ __launch_bounds__(256) void gemm_f32_rows_kernel(GemmArgs g) {
  typedef float AT;
  constexpr int BM = 16, BN = 16, LDC = BN + 4;
  constexpr bool kGeglu = EPI == EPI_GEGLU;
  extern __shared__ __align__(16) unsigned char smem[];
  const int LDA = g.K + 16;  // rows 16 banks apart
  float *As = reinterpret_cast<float *>(smem);   // [16][LDA]
  float *Cs = As + BM * LDA;                     // [16][LDC]
  float *mom = Cs + BM * LDC;                    // [16][2]
  float *red = mom + 2 * BM;                     // [4 wavefronts][16][16]
  const int tid = threadIdx.x, nt = blockIdx.x, m0 = blockIdx.y * BM;
  const int n0 = kGeglu ? (nt / 8) * 128 + (nt % 8) * 8 : nt * BN;   // first (gate) column of the tile in W
  const int q = tid >> 2, cg = tid & 3, lane = tid & 63, wave = tid >> 6;
  // this thread's 4 columns of W: gate columns 0-7 then value columns 64-71 for a GeGLU tile
  const float *W = static_cast<const float *>(g.W) + n0 + (kGeglu ? (cg >> 1) * 64 + (cg & 1) * 4 : cg * 4);
  constexpr int U = 8;  // k values of a lane per batch (K <= 512: all of them)
  f32x4 w[U];
  // W given transposed ([N][ldb], K contiguous: the activation gradients of the update): the 16 slices of a wavefront
  // read 64 contiguous bytes of each of the tile's columns
  const float *Wt = static_cast<const float *>(g.W) + (size_t)(n0 + cg * 4) * g.ldb;
  auto load_w = [&](int k0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = k0 + 64 * u, kk = k < g.K ? k : 0;  // past K: any row, its term is dropped
      if (g.wt) {
#pragma unroll
        for (int j = 0; j < 4; ++j) w[u][j] = Wt[(size_t)j * g.ldb + kk];
      } else {
        w[u] = *reinterpret_cast<const f32x4 *>(W + (size_t)kk * g.N);
      }
    }
  };
  load_w(q);
  float lam = 0.0f;
  if (PRO == PRO_FINAL) lam = g.lam[0];
  if (PRO == PRO_LN || PRO == PRO_FINAL) {
    if (tid < BM) {
      float mean, rstd;
      row_moments(g, m0 + tid, mean, rstd);
      mom[tid * 2] = mean; mom[tid * 2 + 1] = rstd;
    }
    __syncthreads();
  }
  const int kch = g.K / 8;
  for (int c = tid; c < BM * kch; c += 256) {
    const int row = c / kch, kc = (c - row * kch) * 8;
    Raw8<AT> a, a2;
    stage_load<PRO, AT>(g, m0 + row, kc, a, a2);
    float v[8];
    stage_transform<PRO, AT>(g, kc, a, a2, (PRO == PRO_LN || PRO == PRO_FINAL) ? mom[row * 2] : 0.0f,
                             (PRO == PRO_LN || PRO == PRO_FINAL) ? mom[row * 2 + 1] : 1.0f, lam, v);
    store8(As + row * LDA + kc, v);
  }
  __syncthreads();
  float acc[16][4];
#pragma unroll
  for (int r = 0; r < 16; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[r][j] = 0.0f;
  for (int k0 = q; k0 < g.K; k0 += 64 * U) {
    if (k0 != q) load_w(k0);
#pragma unroll
    for (int u = 0; u < U; ++u) {  // in k order
      const int k = k0 + 64 * u;
      if (k < g.K) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float a = As[r * LDA + k];
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[r][j] = fmaf(a, w[u][j], acc[r][j]);
        }
      }
    }
  }
  // butterfly over the 16 K slices of a wavefront (lane bits 2-5), keeping half of the rows at every level
  float h8[8][4], h4[4][4], h2[2][4], h1[4];
  {
    const bool up = lane & 32;
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float keep = up ? acc[8 + r][j] : acc[r][j], send = up ? acc[r][j] : acc[8 + r][j];
        h8[r][j] = keep + __shfl_xor(send, 32, 64);
      }
  }
  {
    const bool up = lane & 16;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float keep = up ? h8[4 + r][j] : h8[r][j], send = up ? h8[r][j] : h8[4 + r][j];
        h4[r][j] = keep + __shfl_xor(send, 16, 64);
      }
  }
  {
    const bool up = lane & 8;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float keep = up ? h4[2 + r][j] : h4[r][j], send = up ? h4[r][j] : h4[2 + r][j];
        h2[r][j] = keep + __shfl_xor(send, 8, 64);
      }
  }
  {
    const bool up = lane & 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float keep = up ? h2[1][j] : h2[0][j], send = up ? h2[0][j] : h2[1][j];
      h1[j] = keep + __shfl_xor(send, 4, 64);
    }
  }
  {  // the lane now holds row (bits 5, 4, 3, 2 of the lane index), its 4 columns, summed over the wavefront's 16 slices
    const int row = ((lane >> 5) & 1) * 8 + ((lane >> 4) & 1) * 4 + ((lane >> 3) & 1) * 2 + ((lane >> 2) & 1);
#pragma unroll
    for (int j = 0; j < 4; ++j) red[(wave * 16 + row) * 16 + cg * 4 + j] = h1[j];
  }
  __syncthreads();
  Cs[(tid >> 4) * LDC + (tid & 15)] = (red[tid] + red[256 + tid]) + (red[512 + tid] + red[768 + tid]);
  __syncthreads();
  epilogue<EPI, AT, BM, BN>(g, Cs, m0, kGeglu ? 0 : n0, nt, tid);
}

template <int PRO, int EPI>
hipError_t launch_f32_rows(const GemmArgs &g, hipStream_t s) {
  constexpr bool kGeglu = EPI == EPI_GEGLU;
  if (g.M <= 0 || g.K % 16 || g.K > 2048 || g.N % (kGeglu ? 128 : 16) || (g.wt && (kGeglu || g.ldb < g.K))) return hipErrorInvalidValue;
  const size_t lds = ((size_t)16 * (g.K + 16) + 16 * 20 + 32 + 4 * 256) * sizeof(float);
  static size_t attr = 0;
  auto kern = gemm_f32_rows_kernel<PRO, EPI>;
  if (lds > attr) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr = lds;
  }
  hipLaunchKernelGGL(kern, dim3(g.N / 16, (g.M + 15) / 16), dim3(256), lds, s, g);
  return hipGetLastError();
}

template <int WM, int WN, int TM, int TN, int PRO, int EPI, bool KEEP = false>
hipError_t launch_bf16(const GemmArgs &g, hipStream_t s) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr size_t lds_a = 2 * BM * (64 + 8) * sizeof(bf16_t), lds_c = (size_t)BM * (BN + 4) * sizeof(float);
  constexpr size_t lds = lds_a > lds_c ? lds_a : lds_c;
  static bool attr_done = false;
  auto kern = gemm_bf16_kernel<WM, WN, TM, TN, PRO, EPI, KEEP>;
  if (KEEP && (g.M % BM || !g.C2)) return hipErrorInvalidValue;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int splits = (EPI == EPI_PARTIAL && g.splits > 1) ? g.splits : 1;
  if (g.N % BN || g.K % (64 * splits) || g.M <= 0 || (EPI != EPI_PARTIAL && (g.splits > 1 || g.sum_splits))) return hipErrorInvalidValue;
  const int grid = ((g.M + BM - 1) / BM) * (g.N / BN);
  hipLaunchKernelGGL(kern, dim3(grid, g.sum_splits ? 1 : splits), dim3(256), lds, s, g);
  return hipGetLastError();
}

// Column ranges of the XCD split (see tile_of_block) by the size of the A operand; FADE_GEMM_XCD overrides for sweeps.
int fade_gemm_col_groups(int M, int K, int N, size_t w_slice = (size_t)2 << 20) {
  static int v = -1;
  if (v < 0) { const char *e = getenv("FADE_GEMM_XCD"); v = e ? atoi(e) : 0; }
  if (v > 0) return v;
  // Router product, M = 16384, N = K = 2048 (A 64 MiB, 200 MiB algorithmic reads): 8 ranges fetch 678 MiB from memory,
  // 4 fetch 467, 2 fetch 433, 1 (rows only; W then streams through every L2) 453, at equal run time within 3 %.
  // Tall A: as few ranges as keep an XCD's slice of W (K x N / ranges, bf16) within 2 MiB, half of its L2.
  if ((size_t)M * K < ((size_t)4 << 20)) return 8;
  int cg = 1;
  while (cg < 8 && (size_t)K * N * 2 / cg > w_slice) cg *= 2;
  return cg;
}

template <int BM, int BN, int STAGES, int EPI, bool BROW = false>
hipError_t launch_pipe(const GemmArgs &g, hipStream_t s) {
  constexpr int BK = 64;
  constexpr size_t lds_ring = (size_t)STAGES * (BM * 128 + (BN / 32) * 4 * 1024), lds_c = (size_t)BM * (BN + 4) * sizeof(float);
  constexpr size_t lds = lds_ring > lds_c ? lds_ring : lds_c;
  static bool attr_done = false;
  auto kern = gemm_pipe_kernel<BM, BN, STAGES, EPI, BROW>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int splits = g.splits > 1 ? g.splits : 1;
  if (g.N % BN || g.M <= 0 || g.K % (splits * BK) || (EPI != EPI_PARTIAL && splits != 1) || g.lda % 8 || (BROW && g.ldb % 8)) return hipErrorInvalidValue;
  GemmArgs ga = g;
  const int ntm = (g.M + BM - 1) / BM, ntn = g.N / BN;
  if (ga.col_groups == 0) ga.col_groups = fade_gemm_col_groups(g.M, g.K, g.N);
  if ((ga.col_groups != 1 && ga.col_groups != 2 && ga.col_groups != 4) || ntn % ga.col_groups) ga.col_groups = 8;
  const int rg = 8 / ga.col_groups;
  if (ga.sum_splits && EPI != EPI_PARTIAL) return hipErrorInvalidValue;
  const dim3 grid((ntn % ga.col_groups == 0 ? (ntm + rg - 1) / rg * rg : ntm) * ntn, ga.sum_splits ? 1 : splits);
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, ga);
  return hipGetLastError();
}

template <int BM, int BN, int STAGES>
hipError_t launch_tn(const GemmArgs &g, hipStream_t s) {
  constexpr size_t lds_ring = (size_t)STAGES * 64 * (BM + BN) * 2, lds_c = (size_t)BM * (BN + 4) * sizeof(float);
  constexpr size_t lds = lds_ring > lds_c ? lds_ring : lds_c;
  static bool attr_done = false;
  auto kern = gemm_tn_kernel<BM, BN, STAGES>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if (g.M % BM || g.N % BN || g.K % 64 || g.K <= 0 || g.a_rows <= 0 || g.a_rows > g.K || g.lda % 8 || g.ldb % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((g.M / BM) * (g.N / BN)), dim3(256), lds, s, g);
  return hipGetLastError();
}

hipError_t launch_tn2(const GemmArgs &g, hipStream_t s) {
  constexpr size_t lds = (size_t)2 * 64 * (256 + 256) * 2;
  static_assert(lds >= (size_t)64 * 260 * sizeof(float) && lds <= 160 * 1024, "LDS per compute unit");
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_tn2_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int splits = g.splits > 1 ? g.splits : 1;
  if (g.M % 256 || g.N % 256 || g.K <= 0 || g.K % (splits * 64) || g.a_rows <= 0 || g.a_rows > g.K || g.lda % 8 || g.ldb % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gemm_tn2_kernel, dim3((g.M / 256) * (g.N / 256) * splits), dim3(512), lds, s, g, splits);
  return hipGetLastError();
}

}  // namespace
hipError_t fade_gemm_tn2_group_add(Tn2Group &tg, const GemmArgs &g) {
  const int splits = g.splits > 1 ? g.splits : 1;
  if (tg.count >= 8 || !fade_gemm_tn2_ok(g.M, g.N, g.K) || g.K % (splits * 64) || g.a_rows <= 0 || g.a_rows > g.K || g.lda % 8 || g.ldb % 8)
    return hipErrorInvalidValue;
  const int p = tg.count, blocks = (g.M / 256) * (g.N / 256) * splits;
  if (p == 0) tg.first_block[0] = 0;
  tg.g[p] = g; tg.splits[p] = splits; tg.first_block[p + 1] = tg.first_block[p] + blocks;
  tg.count = p + 1;
  return hipSuccess;
}
hipError_t fade_gemm_tn2_group_launch(const Tn2Group &tg, hipStream_t s) {
  if (tg.count <= 0) return hipSuccess;
  constexpr size_t lds = (size_t)2 * 64 * (256 + 256) * 2;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_tn2_group_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  // the products with the most workgroups first: their blocks then start on a multiple of 256, and the units an XCD runs
  // side by side belong to one product
  Tn2Group o{};
  o.count = tg.count;
  int idx[8];
  for (int p = 0; p < tg.count; ++p) idx[p] = p;
  for (int i = 1; i < tg.count; ++i)
    for (int j = i; j > 0; --j) {
      const int a = idx[j - 1], b = idx[j];
      if (tg.first_block[b + 1] - tg.first_block[b] <= tg.first_block[a + 1] - tg.first_block[a]) break;
      idx[j - 1] = b; idx[j] = a;
    }
  o.first_block[0] = 0;
  for (int p = 0; p < tg.count; ++p) {
    const int q = idx[p];
    o.g[p] = tg.g[q]; o.splits[p] = tg.splits[q];
    o.first_block[p + 1] = o.first_block[p] + (tg.first_block[q + 1] - tg.first_block[q]);
  }
  static int near = -1;
  if (near < 0) { const char *e = getenv("FADE_TN2_NEAR"); near = (e && e[0] == '0') ? 0 : 1; }
  o.near = near;
  hipLaunchKernelGGL(gemm_tn2_group_kernel, dim3(o.first_block[o.count]), dim3(512), lds, s, o);
  return hipGetLastError();
}
namespace {

template <int BM, int BN, int STAGES, int EPI, int NW, int WPU>
hipError_t launch_pipe2(const GemmArgs &g, hipStream_t s) {
  constexpr size_t lds_ring = (size_t)STAGES * (BM * 64 + (BN / 32) * 2 * 1024);
  constexpr size_t lds_c = BM > 128 ? (size_t)64 * (BN + 4) * sizeof(float) : (size_t)BM * (BN + 4) * sizeof(float);
  constexpr size_t lds = lds_ring > lds_c ? lds_ring : lds_c;
  static_assert(lds * WPU <= 160 * 1024, "LDS per compute unit");
  static bool attr_done = false;
  auto kern = gemm_pipe2_kernel<BM, BN, STAGES, EPI, NW, WPU>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int splits = g.splits > 1 ? g.splits : 1;
  if (g.N % BN || g.M <= 0 || g.K % (splits * 32) || (EPI != EPI_PARTIAL && splits != 1) || g.lda % 8) return hipErrorInvalidValue;
  if (g.sum_splits && EPI != EPI_PARTIAL) return hipErrorInvalidValue;
  if (BM > 128 && NW == 8 && g.M % BM) return hipErrorInvalidValue;  // the slab epilogue of the eight-wavefront tile assumes whole tiles
  GemmArgs ga = g;
  const int ntm = (g.M + BM - 1) / BM, ntn = g.N / BN;
  if (ga.col_groups == 0) ga.col_groups = fade_gemm_col_groups(g.M, g.K, g.N, BN >= 256 ? (size_t)4 << 20 : (size_t)2 << 20);
  if ((ga.col_groups != 1 && ga.col_groups != 2 && ga.col_groups != 4) || ntn % ga.col_groups) ga.col_groups = 8;
  const int rg = 8 / ga.col_groups;
  const dim3 grid((ntn % ga.col_groups == 0 ? (ntm + rg - 1) / rg * rg : ntm) * ntn, ga.sum_splits ? 1 : splits);
  hipLaunchKernelGGL(kern, grid, dim3(NW * 64), lds, s, ga);
  return hipGetLastError();
}

// Tile shape by problem size. Small batches: 64 x 128 tiles, four stages, so that every compute unit gets a tile. From
// 512 tiles of 128 x 128 on: that tile with a two-stage ring (64 KiB of LDS), two workgroups per compute unit: one's
// epilogue (side inputs from HBM, stores) and pipeline fill run under the other's products, which measured faster than
// either a deeper ring or a 256 x 128 tile with one workgroup per unit (router product, M = 4096: 43 us against 54).
// Once every compute unit gets a 256 x 256 tile (M >= 8192 at N = 2048): that tile on eight wavefronts with the ring of
// four 32-wide stages (pipe2_body): half the operand bytes per flop of 128 x 128 and two wavefronts per SIMD. On random
// operands at M = 16384, N = 2048: K = 2048 188 us against 207 for the same tile on a two-stage ring of 64-wide stages,
// 230 for 128 x 128; K = 512 88 against 104; mix epilogue in both. With a contraction of 64 the two shapes tie.
template <int EPI>
hipError_t launch_pipe_auto(const GemmArgs &g, hipStream_t s) {
  const int tiles128 = ((g.M + 127) / 128) * (g.N / 128);
  const int tune = fade_gemm_tune();
  if constexpr (EPI != EPI_PARTIAL) {
    const int tiles256 = ((g.M + 255) / 256) * (g.N / 256);
    if (g.N % 256 == 0 && g.M % 256 == 0 && (tune == 20 || (tune == 0 && tiles256 >= 256 && g.K >= 256))) return launch_pipe2<256, 256, 4, EPI, 8, 1>(g, s);
    if (tune == 21) return launch_pipe2<256, 128, 3, EPI, 4, 2>(g, s);
  }
  if (tune == 23) return launch_pipe2<128, 128, 4, EPI, 4, 2>(g, s);
  if (tune == 11 || (tune == 0 && tiles128 >= 512)) return launch_pipe<128, 128, 2, EPI>(g, s);
  if (tune == 10) return launch_pipe<256, 128, 3, EPI>(g, s);
  if (tune == 1 || (tune == 0 && tiles128 >= 256)) return launch_pipe<128, 128, 4, EPI>(g, s);
  return launch_pipe<64, 128, 4, EPI>(g, s);
}

template <int BN, int PRO, int EPI>
hipError_t launch_f32_bn(const GemmArgs &g, hipStream_t s) {
  constexpr int BM = 256 / (BN / 8);
  const int grid = ((g.M + BM - 1) / BM) * (g.N / BN);
  hipLaunchKernelGGL((gemm_f32_kernel<BN, PRO, EPI>), dim3(grid), dim3(256), 0, s, g);
  return hipGetLastError();
}
// wide == true: N is a multiple of 128 (required by the statistics and GeGLU layouts); otherwise N in {64, 32, 16}.
template <int PRO, int EPI, bool WIDE>
hipError_t launch_f32(const GemmArgs &g, hipStream_t s) {
  if (g.K % 32 || g.M <= 0) return hipErrorInvalidValue;
  if constexpr (WIDE) {
    if (g.N % 128) return hipErrorInvalidValue;
    return launch_f32_bn<128, PRO, EPI>(g, s);
  } else {
  if (g.N % 64 == 0) return launch_f32_bn<64, PRO, EPI>(g, s);
  if (g.N % 32 == 0) return launch_f32_bn<32, PRO, EPI>(g, s);
  if (g.N % 16 == 0) return launch_f32_bn<16, PRO, EPI>(g, s);
  return hipErrorInvalidValue;
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
// grouped launches (bf16 path)
// ---------------------------------------------------------------------------------------------------
namespace {
size_t group_kind_lds(int kind, int stages) {  // the larger of the operand ring and the fp32 tile parked for the epilogue
  size_t ring, tile;
  switch (kind) {
    case GK_STORE_64x128: case GK_TN_64x128: ring = 8192 + 16384; tile = 64 * 132 * 4; break;
    case GK_TN_128x128: case GK_STORE_128x128: case GK_PARTIAL_128x128: ring = 16384 + 16384; tile = 128 * 132 * 4; break;
    default: ring = 8192 + 8192; tile = 64 * 68 * 4; break;  // the 64 x 64 kinds
  }
  ring *= (size_t)stages;
  return ring > tile ? ring : tile;
}
}  // namespace

// Tile shape of a weight-gradient product dW[M][N] in a grouped launch.
static bool tn_shape(int M, int N, int &kind, int &bm, int &bn) {
  if (N % 128 == 0) {
    const bool big = M % 128 == 0 && (M / 128) * (N / 128) >= 256 && fade_gemm_tune() != 8;
    kind = big ? GK_TN_128x128 : GK_TN_64x128; bm = big ? 128 : 64; bn = 128;
    return true;
  }
  if (N % 64 == 0) { kind = GK_TN_64x64; bm = 64; bn = 64; return true; }
  return false;
}
// A weight gradient that gets the 256 x 256 tiles of gemm_tn2_kernel, as a launch of its own: large batches, 16 tiles or
// more (fewer would need ranges of the batch shorter than the pipeline is worth). At B = 4096 the grouped 128 x 128 tiles
// are faster (gate and router phases 104 / 106 us against 138 / 138, and 31 us less in the Adam pass).
bool fade_gemm_tn2_ok(int M, int N, int K) {
  static int mink = -1;  // rows of the batch from which the 256 x 256 weight-gradient tiles are used (sweeps: FADE_TN2_MINK)
  if (mink < 0) { const char *e = getenv("FADE_TN2_MINK"); mink = e ? atoi(e) : 8192; }
  return M > 0 && M % 256 == 0 && N % 256 == 0 && K >= mink && (M / 256) * (N / 256) >= 16 && fade_gemm_tune() != 26;
}
int fade_gemm_tn_tiles(int M, int N) {
  int kind, bm, bn;
  if (M <= 0 || M % 64 || !tn_shape(M, N, kind, bm, bn)) return 0;
  return (M / bm) * (N / bn);
}

// Append one product to a group; the kernel body is chosen from the operation and the shape. op is one of GEMM_X_STORE
// (C = A W, W as fragments), GEMM_PARTIAL (split-K partials [splits][M][N], fp32) and GEMM_W_TN (dW from row-major operands).
hipError_t fade_gemm_group_add(GemmGroup &gg, int op, const GemmArgs &g) {
  if (gg.count >= 4 || g.M <= 0 || g.K <= 0 || g.K % 64 || g.lda % 8) return hipErrorInvalidValue;
  int kind, bm, bn, splits = 1;
  if (op == GEMM_X_STORE) {
    bm = 64;
    const int t128 = g.N % 128 == 0 ? ((g.M + 127) / 128) * (g.N / 128) : 0;
    // 128 x 128 tiles from 256 of them on, or from 128 when the contraction is long (then the bytes per flop matter more than
    // the number of workgroups: B = 1024, K = D_h = 2048: 43 us against 48 with 64 x 128; K = 64: 12.6 against 9.0)
    // a very long contraction with few output tiles (du = dE [W_fg W_fv]^T at D_e = 8192: K = 16384, 4096 x 512 outputs) is a
    // chain of hundreds of K blocks per workgroup: small tiles, many workgroups (D_e = 8192, B = 4096: that phase 327 -> 2xx us)
    if (g.K >= 4096 && g.N % 64 == 0 && t128 < 256) { kind = GK_STORE_64x64; bn = 64; }
    else if ((t128 >= 256 || (t128 >= 128 && g.K >= 1024)) && fade_gemm_tune() != 9) { kind = GK_STORE_128x128; bm = 128; bn = 128; }
    else if (g.N % 128 == 0 && ((g.M + 63) / 64) * (g.N / 128) >= 128) { kind = GK_STORE_64x128; bn = 128; }
    else if (g.N % 64 == 0) { kind = GK_STORE_64x64; bn = 64; }
    else return hipErrorInvalidValue;
  } else if (op == GEMM_PARTIAL) {
    if (g.N % 64 || g.sum_splits) return hipErrorInvalidValue;
    if (g.N % 128 == 0) { kind = GK_PARTIAL_128x128; bm = 128; bn = 128; }
    else { kind = GK_PARTIAL_64x64; bm = 64; bn = 64; }
    splits = g.splits > 1 ? g.splits : 1;
    if (g.K % (splits * 64)) return hipErrorInvalidValue;
  } else if (op == GEMM_W_TN) {
    if (g.a_rows <= 0 || g.a_rows > g.K || g.ldb % 8 || g.M % 64) return hipErrorInvalidValue;
    splits = g.splits > 1 ? g.splits : 1;  // ranges of the batch, each leaving its own slice of C (and C3)
    if (g.K % (splits * 64)) return hipErrorInvalidValue;
    if (!tn_shape(g.M, g.N, kind, bm, bn)) return hipErrorInvalidValue;
  } else {
    return hipErrorInvalidValue;
  }
  const int p = gg.count;
  if (p == 0) gg.first_block[0] = 0;
  gg.kind[p] = kind;
  gg.tiles[p] = ((g.M + bm - 1) / bm) * (g.N / bn);
  gg.splits[p] = splits;
  gg.first_block[p + 1] = gg.first_block[p] + gg.tiles[p] * splits;
  gg.g[p] = g;
  gg.count = p + 1;
  return hipSuccess;
}
hipError_t fade_gemm_group_launch(const GemmGroup &gg, hipStream_t s) {
  if (gg.count <= 0) return hipSuccess;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_group_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * (16384 + 16384));
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_group2_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 132 * 4);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  // two workgroups per compute unit pay off once the group has about two workgroups for every unit (400 of them; B = 1024: the gate / router
  // groups 52 -> 44 us, the small refiner group 18 -> 24 us if forced; B = 4096: 177 -> 139 us)
  const int tune = fade_gemm_tune();
  const int stages = (tune == 14 || (tune != 13 && gg.first_block[gg.count] >= 400)) ? 2 : 4;
  size_t lds = 0;
  for (int p = 0; p < gg.count; ++p) lds = group_kind_lds(gg.kind[p], stages) > lds ? group_kind_lds(gg.kind[p], stages) : lds;
  if (stages == 2) hipLaunchKernelGGL(gemm_group2_kernel, dim3(gg.first_block[gg.count]), dim3(256), lds, s, gg);
  else hipLaunchKernelGGL(gemm_group_kernel, dim3(gg.first_block[gg.count]), dim3(256), lds, s, gg);
  return hipGetLastError();
}

// Tuning override for experiments (FADE_GEMM_TUNE: 0 automatic, 1 force 128x128x4 stages, 2 force 64x128, 10 force 256x128x3,
// 11 force 128x128x2 with two workgroups per compute unit; rings of 32-wide stages: 20 force 256x256 on eight wavefronts,
// 21 256x128 with two workgroups per unit, 23 128x128 with two workgroups per unit; grouped launches: 13 force the
// four-stage kernel, 14 force the two-stage one).
int fade_gemm_tune() {
  static int v = -1;
  if (v < 0) { const char *e = getenv("FADE_GEMM_TUNE"); v = e ? atoi(e) : 0; }
  return v;
}

// One entry per (shape class, prologue, epilogue) the model step uses.
hipError_t fade_gemm(int op, bool bf16, const GemmArgs &g, hipStream_t s) {
  if (bf16) {
    switch (op) {
      case GEMM_CONV:     return launch_bf16<4, 1, 1, 1, PRO_CONV, EPI_CONV>(g, s);       // 128 x 32 tiles
      case GEMM_GLOBAL:   return launch_pipe_auto<EPI_GLOBAL>(g, s);
      case GEMM_ROUTER:   return launch_pipe_auto<EPI_MIX>(g, s);
      case GEMM_UP:       return launch_pipe_auto<EPI_STORE>(g, s);
      case GEMM_GATE:     return launch_pipe_auto<EPI_GATE>(g, s);
      case GEMM_FNR_OUT:  return launch_pipe_auto<EPI_STORE>(g, s);
      case GEMM_FNR_IN:   // Eq. 9 in one piece (no split-K): folded LayerNorm and GeGLU in the epilogue
        if (!g.stats || !g.fold_s || !g.fold_t) return hipErrorInvalidValue;
        return launch_pipe_auto<EPI_GEGLU_FOLD>(g, s);
      case GEMM_PARTIAL:  // split-K products whose LayerNorm / bias / non-linearity follow in the reducing kernel
        if (g.N % 128 == 0) return launch_pipe<128, 128, 4, EPI_PARTIAL>(g, s);
        return launch_pipe<64, 64, 4, EPI_PARTIAL>(g, s);
      case GEMM_X_STORE:  // backward dX = dY W^T: W^T is kept as a second set of fragments
        if (g.N % 128) return launch_pipe<64, 64, 4, EPI_STORE>(g, s);
        return launch_pipe_auto<EPI_STORE>(g, s);
      case GEMM_W:        // backward dW = L^T R over the batch: both operands are feature-major copies [*][Bp]
        if (g.N % 128 == 0) return launch_pipe<64, 128, 4, EPI_GRAD, true>(g, s);
        return launch_pipe<64, 64, 4, EPI_GRAD, true>(g, s);
      case GEMM_W_TN:     // the same from row-major operands (no copies): A = L [a_rows][lda], W = R [K][ldb]
        if (fade_gemm_tn2_ok(g.M, g.N, g.K)) return launch_tn2(g, s);
        if (g.N % 128 == 0) {
          if (fade_gemm_tune() == 7 && g.M % 128 == 0) return launch_tn<128, 128, 4>(g, s);
          return launch_tn<64, 128, 4>(g, s);
        }
        return launch_tn<64, 64, 4>(g, s);
      case GEMM_CONVT:    return launch_bf16<4, 1, 1, 1, PRO_CONVT, EPI_STORE>(g, s);
      case GEMM_HEAD:     // head on H = psi(LN(V)) + lam * H_coarse formed in the operand load (Eq. 10's tail never goes to memory):
        // 32 rows x all 256 columns per workgroup (two workgroups per unit), so every row is transformed once; split-K partials as GEMM_PARTIAL leaves them
        if (!g.stats || !g.A2 || !g.gamma || !g.beta || !g.lam || g.N != 256) return hipErrorInvalidValue;
        if (g.C2) return launch_bf16<1, 4, 1, 2, PRO_FINAL, EPI_PARTIAL, true>(g, s);  // H itself kept for the update
        return launch_bf16<1, 4, 1, 2, PRO_FINAL, EPI_PARTIAL>(g, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (g.rows16) {  // very small batches: 16 x 16 tiles, statistics per 16 columns (see gemm_f32_rows_kernel)
    switch (op) {
      case GEMM_CONV:     return launch_f32_rows<PRO_CONV, EPI_CONV>(g, s);
      case GEMM_GLOBAL:   return launch_f32_rows<PRO_PLAIN, EPI_GLOBAL>(g, s);
      case GEMM_ROUTER:   return launch_f32_rows<PRO_PLAIN, EPI_MIX>(g, s);
      case GEMM_DOWN:     return launch_f32_rows<PRO_LN, EPI_STORE_F32>(g, s);
      case GEMM_UP:       return launch_f32_rows<PRO_PLAIN, EPI_STORE>(g, s);
      case GEMM_GATE:     return launch_f32_rows<PRO_PLAIN, EPI_GATE>(g, s);
      case GEMM_FNR_IN:   return launch_f32_rows<PRO_LN, EPI_GEGLU>(g, s);
      case GEMM_FNR_OUT:  return launch_f32_rows<PRO_PLAIN, EPI_STORE>(g, s);
      case GEMM_HEAD:     return launch_f32_rows<PRO_FINAL, EPI_STORE_F32>(g, s);
      case GEMM_HEAD_PLAIN: return launch_f32_rows<PRO_PLAIN, EPI_STORE_F32>(g, s);
      case GEMM_X_STORE:  return launch_f32_rows<PRO_PLAIN, EPI_STORE>(g, s);  // W passed transposed (wt = 1)
      case GEMM_PARTIAL:  // one range only: a plain fp32 store
        if (g.splits > 1 || g.sum_splits) return hipErrorInvalidValue;
        return launch_f32_rows<PRO_PLAIN, EPI_PARTIAL>(g, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (op) {
    case GEMM_CONV:     return launch_f32<PRO_CONV, EPI_CONV, false>(g, s);
    case GEMM_GLOBAL:   return launch_f32<PRO_PLAIN, EPI_GLOBAL, true>(g, s);
    case GEMM_ROUTER:   return launch_f32<PRO_PLAIN, EPI_MIX, true>(g, s);
    case GEMM_DOWN:     return launch_f32<PRO_LN, EPI_STORE_F32, false>(g, s);
    case GEMM_UP:       return launch_f32<PRO_PLAIN, EPI_STORE, true>(g, s);
    case GEMM_GATE:     return launch_f32<PRO_PLAIN, EPI_GATE, true>(g, s);
    case GEMM_FNR_IN:   return launch_f32<PRO_LN, EPI_GEGLU, true>(g, s);
    case GEMM_FNR_OUT:  return launch_f32<PRO_PLAIN, EPI_STORE, true>(g, s);
    case GEMM_HEAD:     return launch_f32<PRO_FINAL, EPI_STORE_F32, true>(g, s);
    case GEMM_HEAD_PLAIN: return launch_f32<PRO_PLAIN, EPI_STORE_F32, true>(g, s);
    case GEMM_X_STORE:  // W passed transposed (wt = 1)
      if (g.N % 128 == 0) return launch_f32<PRO_PLAIN, EPI_STORE, true>(g, s);
      return launch_f32<PRO_PLAIN, EPI_STORE, false>(g, s);
    case GEMM_PARTIAL:  return launch_f32<PRO_PLAIN, EPI_PARTIAL, false>(g, s);  // one "split": the full sum
    case GEMM_W:
      if (g.N % 128 == 0) return launch_f32<PRO_PLAIN, EPI_GRAD, true>(g, s);
      return launch_f32<PRO_PLAIN, EPI_GRAD, false>(g, s);
    case GEMM_CONVT:    return launch_f32<PRO_CONVT, EPI_STORE, false>(g, s);
    default: return hipErrorInvalidValue;
  }
}
