// fade_misc.hip — everything of the step that is not a dense product: weight preparation, the embedding /
// window gather with the rolling-cache update (Eq. 1-2), the per-stream memory product of Eq. 7, and the
// fused softmax -> frequency table -> arithmetic coder kernel (one wavefront per stream).
#include <cstdlib>

#include "fade_dev.h"
#include "fade_kernels.h"

namespace {

__device__ __forceinline__ float gelu_f(float x) { return fade_gelu(x); }

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// ---------------------------------------------------------------------------------------------------
// weight preparation
// ---------------------------------------------------------------------------------------------------
// fp32 [k_real][N] (row-major) -> bf16 fragments for v_mfma_f32_32x32x16_bf16's B operand:
// fragment (nt, ks) is 64 lanes x 8 values, lane l holding W[ks*16 + (l/32)*8 + i][nt*32 + l%32], i = 0..7;
// fragments of one 32-column tile are contiguous along K. Rows >= k_real are zero (padding of K).
// interleave = 1: the source is the pair (W0, W1) of [k_real][N/2] matrices and virtual column v maps to
// column (v/128)*64 + v%64 of W0 when v%128 < 64, else of W1 (gate and value of Eq. 9 side by side in one tile).
// rowscale (optional, [k_real]): the stored value is bf16(rowscale[k] * bf16(W[k][n])): a LayerNorm gain folded into
// the weights of the product that consumes the normalised activations.
__global__ void preshuffle_kernel(const float *W0, const float *W1, int k_real, int K, int N, int interleave, const float *rowscale,
                                  bf16_t *out) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one thread per (fragment, lane)
  const size_t total = (size_t)(N / 32) * (K / 16) * 64;
  if (t >= total) return;
  const int lane = (int)(t & 63);
  const size_t frag = t >> 6;
  const int ks = (int)(frag % (size_t)(K / 16)), nt = (int)(frag / (size_t)(K / 16));
  const int v = nt * 32 + (lane & 31);
  const float *src = W0;
  int col = v, ld = N;
  if (interleave) {
    ld = N / 2;
    col = (v / 128) * 64 + (v & 63);
    if ((v & 127) >= 64) src = W1;
  }
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = ks * 16 + (lane >> 5) * 8 + i;
    float w = k < k_real ? src[(size_t)k * ld + col] : 0.0f;
    if (rowscale && k < k_real) w = rowscale[k] * (float)(bf16_t)w;
    r[i] = (bf16_t)w;
  }
  reinterpret_cast<bf16x8 *>(out)[t] = r;
}

// fp32 path: the same virtual matrix, plain [K][N] fp32.
__global__ void virtual_copy_kernel(const float *W0, const float *W1, int k_real, int K, int N, int interleave, float *out) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (size_t)K * N) return;
  const int k = (int)(t / N), v = (int)(t % N);
  const float *src = W0;
  int col = v, ld = N;
  if (interleave) {
    ld = N / 2;
    col = (v / 128) * 64 + (v & 63);
    if ((v & 127) >= 64) src = W1;
  }
  out[t] = k < k_real ? src[(size_t)k * ld + col] : 0.0f;
}

template <typename AT> __global__ void convert_kernel(const float *src, AT *dst, size_t n) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) dst[t] = (AT)src[t];
}
// fp32 -> value rounded to bf16 and widened again (small fp32-resident operands of the bf16 configuration)
__global__ void round_bf16_kernel(const float *src, float *dst, size_t n) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) dst[t] = (float)(bf16_t)src[t];
}

// Per-symbol tables: LN_D(E[s]) with the two affine pairs (X of the Design paragraph; LN of Eq. 4), and, for the
// update, the normalised row x-hat and 1/sigma. One workgroup per symbol, lane = channel (D <= 256).
template <typename AT>
__device__ __forceinline__ void tables_body(int s, const float *E, bool round_bf16, const float *ge, const float *be, const float *gl, const float *bl, int D,
                                            AT *tabXe, AT *tabXl, float *tabXe32, float *tabXhat, float *tabRstd) {
  __shared__ float red[256];
  const int i = threadIdx.x;
  float e = i < D ? E[(size_t)s * D + i] : 0.0f;
  if (round_bf16) e = (float)(bf16_t)e;
  red[i] = e;
  __syncthreads();
  float mean = 0.0f;
  for (int k = 0; k < D; ++k) mean += red[k];
  mean /= (float)D;
  __syncthreads();
  const float dlt = e - mean;
  red[i] = i < D ? dlt * dlt : 0.0f;
  __syncthreads();
  float var = 0.0f;
  for (int k = 0; k < D; ++k) var += red[k];
  var /= (float)D;
  const float rstd = 1.0f / sqrtf(var + 1e-5f);
  if (i < D) {
    const float h = dlt * rstd, xe = h * ge[i] + be[i];
    tabXe32[(size_t)s * D + i] = xe;
    tabXe[(size_t)s * D + i] = (AT)xe;
    tabXl[(size_t)s * D + i] = (AT)(h * gl[i] + bl[i]);
    if (tabXhat) tabXhat[(size_t)s * D + i] = h;
  }
  if (i == 0 && tabRstd) tabRstd[s] = rstd;
}
// Eq. 1 for symbol s in the same workgroup: x = the row just formed (fp32, as tabXe32 holds it), W_g / W_v rounded to bf16 as
// their compute copies are; slot_pair's order of operations, so the values are those that function gives from the copies.
__device__ __forceinline__ void tables_slot_body(int s, const TablesArgs &t) {
  __shared__ float xrow[256];
  const int i = threadIdx.x;
  __syncthreads();  // tabXe32's row of this symbol was written by this workgroup just above
  if (i < t.D) xrow[i] = t.tabXe32[(size_t)s * t.D + i];
  __syncthreads();
  for (int q = i; q < t.c; q += 256) {
    float gg = 0.0f, gv = 0.0f;
    for (int k = 0; k < t.D; ++k) {
      gg = fmaf(xrow[k], (float)(bf16_t)t.Wg[k * t.c + q], gg);
      gv = fmaf(xrow[k], (float)(bf16_t)t.Wv[k * t.c + q], gv);
    }
    if (t.slot_tab) static_cast<bf16_t *>(t.slot_tab)[(size_t)s * t.c + q] = (bf16_t)(gelu_f(gg) * gv);
    if (t.gg_tab) { t.gg_tab[(size_t)s * t.c + q] = gg; t.gv_tab[(size_t)s * t.c + q] = gv; }
  }
}
template <typename AT>
__global__ __launch_bounds__(256) void tables_kernel(const float *E, const float *ge, const float *be, const float *gl, const float *bl, int D,
                                                     AT *tabXe, AT *tabXl, float *tabXe32, float *tabXhat, float *tabRstd) {
  tables_body<AT>(blockIdx.x, E, false, ge, be, gl, bl, D, tabXe, tabXl, tabXe32, tabXhat, tabRstd);
}

// ---------------------------------------------------------------------------------------------------
// window gather + rolling cache (one workgroup per stream)
// ---------------------------------------------------------------------------------------------------
// Eq. 1's two pre-activations for column q: x W_g and x W_v (x: one embedded row of D channels)
__device__ __forceinline__ void slot_pair(const float *xt, const float *Wg, const float *Wv, int D, int c, int q, float &gg, float &gv) {
  gg = 0.0f; gv = 0.0f;
  for (int i = 0; i < D; ++i) {
    gg = fmaf(xt[i], Wg[i * c + q], gg);
    gv = fmaf(xt[i], Wv[i * c + q], gv);
  }
}
// Eq. 4 for one window on the matrix cores (bf16, D = 32): H_local[j][o] = psi(b[o] + sum_{r,i} xl[j - (taps-1) + r][i] W[r][i][o]).
// A wavefront takes the 32 tokens of one tile (T <= 128). A lane's operand piece, 8 consecutive channels of one tap of one
// token, is one 16-byte read of the per-symbol table; the W fragments are read as they lie. One accumulator takes the K
// steps in order and the tail is the product kernel's conv epilogue, so the result is bit for bit that kernel's.
// Three stages, so that the caller can put its own loads of the same depth beside each: the window's symbols, the operand
// pieces they address, then the arithmetic. No load sits behind a branch (the compiler ends such a branch by waiting for
// every load in flight): indices are clamped into the arrays and pieces that do not exist are zeroed afterwards.
// K steps of Eq. 4 that carry data: two per tap (D = 32); K_c may be padded beyond that with zero rows, whose steps every
// kernel here skips alike (they would add exact zeros)
__device__ __forceinline__ int conv_ksteps(const EmbedArgs &a) { return a.Kc / 16 < 2 * a.taps ? a.Kc / 16 : 2 * a.taps; }
// tile: which 32 tokens; af / bf: the K steps' operand pieces (ok[tap]: that tap's token exists); the 32 x 32 result passes
// through the wavefront's own LDS patch (no workgroup barrier) so that a lane ends up with 16 consecutive channels of one
// token (h: psi of the pre-activations p), 2 x 16 bytes per output, instead of 16 scattered 2-byte values
template <int KS>
__device__ __forceinline__ void conv_tile_compute(const EmbedArgs &a, const bf16x8 *af, const bool *ok, const bf16x8 *bf, float bias, bf16x8 *h, bf16x8 *p) {
  const int lane = threadIdx.x & 63, ksteps = conv_ksteps(a);
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    bf16x8 av = af[ks];
    if (!ok[ks >> 1]) {
#pragma unroll
      for (int q = 0; q < 8; ++q) av[q] = (bf16_t)0.0f;
    }
    if (ks < ksteps) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bf[ks], acc, 0, 0, 0);
  }
  __shared__ float patch[4][32][33];
  float (*pt)[33] = patch[(threadIdx.x >> 6) & 3];
  const int o = lane & 31;
#pragma unroll
  for (int e = 0; e < 16; ++e) pt[(e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)][o] = acc[e] + bias;
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the wavefront's LDS writes have landed before its lanes read each other's
  const int tr = lane >> 1, c0 = (lane & 1) * 16;
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const float pre = pt[tr][c0 + q];
    h[q >> 3][q & 7] = (bf16_t)gelu_f(pre);
    p[q >> 3][q & 7] = (bf16_t)pre;
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // ... and read before a later tile of this wavefront overwrites the patch
}
__device__ __forceinline__ void conv_tile_store(const EmbedArgs &a, size_t row, int tile, const bf16x8 *h, const bf16x8 *p) {
  const int lane = threadIdx.x & 63, tr = lane >> 1, c0 = (lane & 1) * 16, t = tile * 32 + tr;
  if (t < a.T) {
    bf16_t *Hl = static_cast<bf16_t *>(a.Hl) + row * a.Dh + t * 32 + c0;
    *reinterpret_cast<bf16x8 *>(Hl) = h[0];
    *reinterpret_cast<bf16x8 *>(Hl + 8) = h[1];
    if (a.cv) {
      bf16_t *cv = static_cast<bf16_t *>(a.cv) + row * a.Dh + t * 32 + c0;
      *reinterpret_cast<bf16x8 *>(cv) = p[0];
      *reinterpret_cast<bf16x8 *>(cv + 8) = p[1];
    }
  }
}
template <int KS>
__device__ __forceinline__ void conv_tile_finish(const EmbedArgs &a, const bf16x8 *af, const bool *ok, const bf16x8 *bf, float bias, size_t row, int tile) {
  bf16x8 h[2], p[2];
  conv_tile_compute<KS>(a, af, ok, bf, bias, h, p);
  conv_tile_store(a, row, tile, h, p);
}
template <int KS>  // K steps held in registers: K_c / 16 <= KS <= 8
struct ConvWindow {
  int sym[4];
  bool ok[4];
  bf16x8 af[KS], bf[KS];
  float bias;
  __device__ __forceinline__ void symbols(const EmbedArgs &a, const uint8_t *win, int tile) {
    const int j = tile * 32 + (threadIdx.x & 31);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int tok = j - (a.taps - 1) + r;
      ok[r] = r < a.taps && tok >= 0 && j < a.T;
      sym[r] = win[ok[r] ? tok : 0];
    }
  }
  __device__ __forceinline__ void operands(const EmbedArgs &a, const bf16_t *tabXl) {
    const int lane = threadIdx.x & 63, ksteps = conv_ksteps(a);  // K_c <= 128: at most 8 K steps, 2 per tap
    const bf16x8 *Wf = static_cast<const bf16x8 *>(a.conv_W) + lane;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int i = (ks & 1) * 16 + (lane >> 5) * 8;  // k = 16 ks + 8 (lane / 32) = 32 tap + i
      af[ks] = *reinterpret_cast<const bf16x8 *>(tabXl + (size_t)sym[ks >> 1] * 32 + i);
      bf[ks] = Wf[(size_t)(ks < ksteps ? ks : 0) * 64];
    }
    bias = a.conv_b[lane & 31];
  }
  __device__ __forceinline__ void finish(const EmbedArgs &a, size_t row, int tile) { conv_tile_finish<KS>(a, af, ok, bf, bias, row, tile); }
};
__device__ __forceinline__ void conv_window_mfma(const EmbedArgs &a, const uint8_t *win, const bf16_t *tabXl, size_t row, int tile) {
  if (tile * 32 >= a.T) return;
  ConvWindow<8> cw;
  cw.symbols(a, win, tile);
  cw.operands(a, tabXl);
  cw.finish(a, row, tile);
}

// One workgroup per stream, in rounds of loads of equal depth: first what depends on nothing (the window's symbols, the
// cache row), then what a symbol addresses (table pieces for X, X_l and Eq. 4, the newest symbol's slot), then stores and
// arithmetic. nt threads: 256, or 64 per 32-token tile of Eq. 4 (see the launcher). KS: K steps of Eq. 4 held in registers
// (>= K_c / 16); NKP: 16-byte pieces of the cache row per thread (>= D_cache / (nt V), wide slots).
template <typename AT, int KS, int NKP>
__global__ __launch_bounds__(256) void embed_cache_kernel(EmbedArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  if (!stream_active(a.ws, b)) return;
  const uint8_t *win = stream_window(a.ws, b, a.T);
  const AT *tabXe = static_cast<const AT *>(a.tabXe), *tabXl = static_cast<const AT *>(a.tabXl);
  AT *X = static_cast<AT *>(a.X) + (size_t)b * a.Dh, *XL = a.XL ? static_cast<AT *>(a.XL) + (size_t)b * a.Dh : nullptr;
  AT *M = static_cast<AT *>(a.M) + (size_t)b * a.Dc;
  constexpr int V = 16 / sizeof(AT);  // elements per 16-byte piece
  typedef f32x4 piece_t;              // 16 bytes, whatever the element type
  const bool wide = a.c % V == 0;     // wide slots: the shift of Eq. 2 is a whole number of 16-byte pieces
  const int np = a.Dc / V, sh = a.c / V, nx = a.Dh / V;
  const bool conv_live = sizeof(AT) == 2 && a.conv_W && (tid >> 6) * 32 < a.T;
  const int tile = conv_live ? tid >> 6 : 0;
  // first batch of loads: window symbols and the cache row
  const bool two = tid + nt < nx;  // the first two pieces of X of this thread (all of them when D_h <= 2 nt V)
  const int e0 = (tid < nx ? tid : 0) * V, j0 = e0 / a.D, i0 = e0 - j0 * a.D;
  const int e1 = (two ? tid + nt : 0) * V, j1 = e1 / a.D, i1 = e1 - j1 * a.D;
  const int s0 = win[j0], s1 = win[j1], slast = win[a.T - 1];
  piece_t kp[NKP];
  if (wide) {
#pragma unroll
    for (int q = 0; q < NKP; ++q) {
      const int idx = q * nt + tid;
      kp[q] = reinterpret_cast<const piece_t *>(M)[idx < np ? idx : np - 1];
    }
  }
  ConvWindow<KS> cw;
  if constexpr (sizeof(AT) == 2) {
    if (a.conv_W) cw.symbols(a, win, tile);
  }
  // second batch of loads: the table pieces the symbols address
  const piece_t xe0 = *reinterpret_cast<const piece_t *>(tabXe + (size_t)s0 * a.D + i0);
  const piece_t xe1 = *reinterpret_cast<const piece_t *>(tabXe + (size_t)s1 * a.D + i1);
  const piece_t xl0 = *reinterpret_cast<const piece_t *>(tabXl + (size_t)s0 * a.D + i0);
  const piece_t xl1 = *reinterpret_cast<const piece_t *>(tabXl + (size_t)s1 * a.D + i1);
  // frozen weights: the slot depends on the symbol alone (without the table: a read of X's table that nothing uses)
  const AT slot = static_cast<const AT *>(a.slot_tab ? a.slot_tab : a.tabXe)[a.slot_tab ? (size_t)slast * a.c + (tid < a.c ? tid : 0) : 0];
  if constexpr (sizeof(AT) == 2) {
    if (a.conv_W) cw.operands(a, reinterpret_cast<const bf16_t *>(tabXl));
  }
  float gg = 0.0f, gv = 0.0f;  // adapting weights: Eq. 1's two pre-activations of the newest symbol, in the same round
  if (!a.slot_tab && tid < a.c) {
    // per symbol they are a table too where the refresh builds it (same operations in the same order, so the same bits)
    if (a.gg_tab) { gg = a.gg_tab[(size_t)slast * a.c + tid]; gv = a.gv_tab[(size_t)slast * a.c + tid]; }
    else slot_pair(a.tabXe32 + (size_t)slast * a.D, a.Wg, a.Wv, a.D, a.c, tid, gg, gv);
  }
  // stores and arithmetic
  if (tid < nx) {
    *reinterpret_cast<piece_t *>(X + e0) = xe0;
    if (a.XL) *reinterpret_cast<piece_t *>(XL + e0) = xl0;
  }
  if (two) {
    *reinterpret_cast<piece_t *>(X + e1) = xe1;
    if (a.XL) *reinterpret_cast<piece_t *>(XL + e1) = xl1;
  }
  for (int ch = tid + 2 * nt; ch < nx; ch += nt) {  // rows of more than 2 nt pieces
    const int e = ch * V, j = e / a.D, i = e - j * a.D;
    const int s = win[j];
    *reinterpret_cast<piece_t *>(X + e) = *reinterpret_cast<const piece_t *>(tabXe + (size_t)s * a.D + i);
    if (a.XL) *reinterpret_cast<piece_t *>(XL + e) = *reinterpret_cast<const piece_t *>(tabXl + (size_t)s * a.D + i);
  }
  if constexpr (sizeof(AT) == 2) {
    if (conv_live) cw.finish(a, (size_t)b, tile);
  }
  // Eq. 2: shift the cache left by one slot (through registers, so the move is safe in place) ...
  if (wide) {
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NKP; ++q) {
      const int idx = q * nt + tid;
      if (idx < np && idx >= sh) reinterpret_cast<piece_t *>(M)[idx - sh] = kp[q];
    }
  } else {
    AT keep[16];  // D_cache <= 16 nt
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int idx = q * nt + tid;
      if (idx < a.Dc) keep[q] = M[idx];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int idx = q * nt + tid;
      if (idx < a.Dc && idx >= a.c) M[idx - a.c] = keep[q];
    }
  }
  // ... and append Eq. 1's GeGLU of the newest symbol: psi(x_t W_g) * (x_t W_v)
  if (tid < a.c) {
    if (a.slot_tab) {
      M[a.Dc - a.c + tid] = slot;
    } else {
      M[a.Dc - a.c + tid] = (AT)(gelu_f(gg) * gv);
      if (a.GG) { a.GG[(size_t)b * a.c + tid] = gg; a.GV[(size_t)b * a.c + tid] = gv; }
    }
  }
}

// The same step with the two per-symbol tables in LDS (bf16, Eq. 4 in the launch, T = 32, 64 or 128, a cache row of at
// most 64 pieces). In the kernel above every wavefront issues some 25 gathering loads per stream (symbols, table pieces,
// the weights of Eq. 4), and the vector memory path of the compute unit, not HBM, sets its pace. Here a workgroup of
// four wavefronts copies both tables to LDS once (32 KiB), keeps the weights of Eq. 4 in registers, and then walks over
// streams: T / 32 wavefronts per stream, 4 / (T / 32) streams side by side. Per stream a wavefront reads the window once
// from memory (lane l: bytes l and 64 + l, parked in its own LDS row); everything a symbol addresses comes from LDS
// except Eq. 1's entry of the newest symbol (its table: `slot_tab`, or with adapting weights the two pre-activations
// `gg_tab` / `gv_tab`).
// One wait for memory per turn, placed after the arithmetic and before the turn's stores: the counter of outstanding
// memory operations is in order and covers stores, and behind stores that sit in branches the compiler's count for an
// older load is the pessimistic one, so a wait anywhere after the stores would expose their whole round trip. The loads it
// covers (window and cache row two streams ahead, the slot entry one stream ahead) and the stores before them are then
// a turn's arithmetic old. Streams past the end or inactive are read at clamped addresses and store nothing.
// UPD: the weights adapt (X_l, the pre-activations of Eq. 4 and of Eq. 1 are kept for the update).
// HALF: cache slots of four elements (Eq. 2 shifts the row by half a 16-byte piece); a template argument so that the
// kernel for whole-piece shifts keeps its instruction schedule.
template <int KS, bool UPD, bool HALF = false>
__global__ __launch_bounds__(256) void embed_cache_lds_kernel(EmbedArgs a) {
  __shared__ __align__(16) bf16_t sXe[256 * 32], sXl[256 * 32];
  __shared__ uint8_t sWin[4][128];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, B = a.B;
  const int wps = a.T / 32, grp = wave / wps, tile = wave - grp * wps, ngrp = 4 / wps;  // wavefronts per stream, streams per workgroup
  const int nt = wps * 64, vt = tid - grp * nt;                                          // threads per stream, this one's index
  const int np = a.Dc / 8, sh = a.c / 8, ksteps = conv_ksteps(a);
  for (int i = tid; i < 1024; i += 256) {
    reinterpret_cast<f32x4 *>(sXe)[i] = static_cast<const f32x4 *>(a.tabXe)[i];
    reinterpret_cast<f32x4 *>(sXl)[i] = static_cast<const f32x4 *>(a.tabXl)[i];
  }
  bf16x8 bf[KS];
  {
    const bf16x8 *Wf = static_cast<const bf16x8 *>(a.conv_W) + lane;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bf[ks] = Wf[(size_t)(ks < ksteps ? ks : 0) * 64];
  }
  const float bias = a.conv_b[lane & 31];
  int toff[4];
  bool ok[4];
  {
    const int j = tile * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int tok = j - (a.taps - 1) + r;
      ok[r] = r < a.taps && tok >= 0 && j < a.T;
      toff[r] = ok[r] ? tok : 0;
    }
  }
  const int j0 = vt >> 2, j1 = (vt + nt) >> 2, i0 = (vt & 3) * 8;  // D = 32: four pieces per token, 2 nt pieces per row
  const int pk = vt < np ? vt : np - 1, l1 = 64 + lane < a.T ? 64 + lane : a.T - 1, vc = vt < a.c ? vt : 0;
  uint8_t *myWin = sWin[wave];
  struct Ahead { int w0, w1, act; f32x4 kp; };  // the window (lane l: bytes l and 64 + l), the mask byte, this thread's piece of the cache row
  struct Slot { uint32_t tab; float gg, gv; };  // tab: the bf16 entry's bits
  auto request = [&](int b, Ahead &y) {
    const int bc = b < B ? b : B - 1;
    long long off = (long long)bc * a.ws.stride + (a.ws.i - a.T);
    if (!a.ws.active) { const long long hi = a.ws.n - a.T; off = off < hi ? off : hi; }
    const uint8_t *win = a.ws.base + off;
    y.w0 = win[lane < a.T ? lane : a.T - 1];
    y.w1 = win[l1];
    y.act = *(a.ws.active ? a.ws.active + bc : win);
    y.kp = reinterpret_cast<const f32x4 *>(static_cast<const bf16_t *>(a.M) + (size_t)bc * a.Dc)[pk];
  };
  auto request_slot = [&](const Ahead &y, Slot &e) {  // the newest symbol: byte T - 1 of the window
    const int slast = __builtin_amdgcn_readlane(a.T > 64 ? y.w1 : y.w0, (a.T - 1) & 63);
    if constexpr (UPD) {
      e.gg = a.gg_tab[(size_t)slast * a.c + vc];
      e.gv = a.gv_tab[(size_t)slast * a.c + vc];
    } else {
      e.tab = static_cast<const uint16_t *>(a.slot_tab)[(size_t)slast * a.c + vc];
    }
  };
  const int step = gridDim.x * ngrp;
  int b = blockIdx.x * ngrp + grp;
  Ahead cur, nx, n2;
  Slot cs{0u, 0.0f, 0.0f}, ns{0u, 0.0f, 0.0f};
  request(b, cur);
  request(b + step, nx);
  request_slot(cur, cs);
  __syncthreads();  // the tables are in LDS
  for (; b < B; b += step) {  // a wavefront's trip count depends on its group only: no workgroup barrier inside
    myWin[lane] = (uint8_t)cur.w0;
    myWin[64 + lane] = (uint8_t)cur.w1;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the wavefront's own window row is written before its lanes read it
    const int s0 = myWin[j0], s1 = myWin[j1];
    int sym[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) sym[r] = myWin[toff[r]];
    const f32x4 xe0 = *reinterpret_cast<const f32x4 *>(sXe + s0 * 32 + i0), xe1 = *reinterpret_cast<const f32x4 *>(sXe + s1 * 32 + i0);
    f32x4 xl0 = xe0, xl1 = xe1;
    if constexpr (UPD) {
      xl0 = *reinterpret_cast<const f32x4 *>(sXl + s0 * 32 + i0);
      xl1 = *reinterpret_cast<const f32x4 *>(sXl + s1 * 32 + i0);
    }
    bf16x8 af[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) af[ks] = *reinterpret_cast<const bf16x8 *>(sXl + sym[ks >> 1] * 32 + (ks & 1) * 16 + (lane >> 5) * 8);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // every read of the window row is done before the next turn overwrites it
    bf16x8 h[2], p[2];
    conv_tile_compute<KS>(a, af, ok, bf, bias, h, p);
    // the turn's one wait for memory (see above). Its operands tie the arithmetic above to this side of it and tell the
    // compiler that the loaded values used below are in their registers from here on.
    {
      f32x4 h0 = __builtin_bit_cast(f32x4, h[0]), h1 = __builtin_bit_cast(f32x4, h[1]), p0 = __builtin_bit_cast(f32x4, p[0]), p1 = __builtin_bit_cast(f32x4, p[1]);
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(h0), "+v"(h1), "+v"(p0), "+v"(p1), "+v"(cur.kp), "+v"(cs.tab), "+v"(cs.gg), "+v"(cs.gv), "+v"(nx.w0), "+v"(nx.w1), "+v"(cur.act)
                   :
                   : "memory");
      h[0] = __builtin_bit_cast(bf16x8, h0); h[1] = __builtin_bit_cast(bf16x8, h1);
      p[0] = __builtin_bit_cast(bf16x8, p0); p[1] = __builtin_bit_cast(bf16x8, p1);
    }
    request(b + 2 * step, n2);
    request_slot(nx, ns);
    const bool alive = a.ws.active ? cur.act != 0 : (a.ws.i < a.ws.stride && (long long)b * a.ws.stride + a.ws.i < a.ws.n);
    if (alive) {
      bf16_t *X = static_cast<bf16_t *>(a.X) + (size_t)b * a.Dh;
      *reinterpret_cast<f32x4 *>(X + vt * 8) = xe0;
      *reinterpret_cast<f32x4 *>(X + (vt + nt) * 8) = xe1;
      if constexpr (UPD) {
        if (a.XL) {
          bf16_t *XL = static_cast<bf16_t *>(a.XL) + (size_t)b * a.Dh;
          *reinterpret_cast<f32x4 *>(XL + vt * 8) = xl0;
          *reinterpret_cast<f32x4 *>(XL + (vt + nt) * 8) = xl1;
        }
      }
      conv_tile_store(a, (size_t)b, tile, h, p);
      // Eq. 2: the row shifted left by one slot; all of its pieces sit in one wavefront, read two turns ago
      bf16_t *M = static_cast<bf16_t *>(a.M) + (size_t)b * a.Dc;
      if constexpr (HALF) {
        // new piece q = upper half of old piece q, lower half of old piece q + 1 (the row's pieces sit in consecutive lanes
        // of one wavefront); the last piece keeps its lower half for the slot appended below
        const float n0 = __shfl_down(cur.kp[0], 1, 64), n1 = __shfl_down(cur.kp[1], 1, 64);
        if (vt < np - 1) {
          f32x4 v;
          v[0] = cur.kp[2]; v[1] = cur.kp[3]; v[2] = n0; v[3] = n1;
          reinterpret_cast<f32x4 *>(M)[vt] = v;
        } else if (vt == np - 1) {
          float2 v;
          v.x = cur.kp[2]; v.y = cur.kp[3];
          *reinterpret_cast<float2 *>(M + a.Dc - 8) = v;
        }
      } else {
        if (vt < np && vt >= sh) reinterpret_cast<f32x4 *>(M)[vt - sh] = cur.kp;
      }
      if (vt < a.c) {  // ... and Eq. 1's GeGLU of the newest symbol appended
        if constexpr (UPD) {
          M[a.Dc - a.c + vt] = (bf16_t)(gelu_f(cs.gg) * cs.gv);
          if (a.GG) { a.GG[(size_t)b * a.c + vt] = cs.gg; a.GV[(size_t)b * a.c + vt] = cs.gv; }
        } else {
          reinterpret_cast<uint16_t *>(M)[a.Dc - a.c + vt] = (uint16_t)cs.tab;
        }
      }
    }
    cur = nx; nx = n2; cs = ns;
  }
}

// Several steps of every stream in one launch (frozen weights, coding a known input): row r = s * B + b is stream b at
// step i + s. The cache of Eq. 2 is rebuilt from the window instead of rolled: after step i, slot j holds the symbol
// window[j]'s entry of Eq. 1, provided the model already ran at the step that appended it (steps before T code under the
// uniform table and append nothing, so those slots are still the zeros of the reset).
__global__ __launch_bounds__(256) void embed_steps_kernel(EmbedArgs a, int rpb) {
  // rpb rows per workgroup (4, 2 or 1: as many as give every wavefront one 32-token tile of Eq. 4)
  const int tid = threadIdx.x, rows = a.B * a.S;
  const bf16_t *tabXe = static_cast<const bf16_t *>(a.tabXe), *tabXl = static_cast<const bf16_t *>(a.tabXl);
  const bf16_t *tab = static_cast<const bf16_t *>(a.slot_tab);
  for (int q = 0; q < rpb; ++q) {
    const int r = blockIdx.x * rpb + q;
    if (r >= rows) break;
    const int s = r / a.B, b = r - s * a.B;
    WinSrc w = a.ws;
    w.i += s;
    if (!stream_active(w, b)) continue;
    const uint8_t *win = stream_window(w, b, a.T);
    bf16_t *X = static_cast<bf16_t *>(a.X) + (size_t)r * a.Dh, *XL = a.XL ? static_cast<bf16_t *>(a.XL) + (size_t)r * a.Dh : nullptr;
    for (int ch = tid; ch < a.Dh / 8; ch += 256) {
      const int e0 = ch * 8, j = e0 / a.D, i = e0 - j * a.D;
      const int sy = win[j];
      *reinterpret_cast<f32x4 *>(X + e0) = *reinterpret_cast<const f32x4 *>(tabXe + (size_t)sy * a.D + i);
      if (XL) *reinterpret_cast<f32x4 *>(XL + e0) = *reinterpret_cast<const f32x4 *>(tabXl + (size_t)sy * a.D + i);
    }
    bf16_t *M = static_cast<bf16_t *>(a.M) + (size_t)r * a.Dc;
    // The cache holds Dc / c slots, oldest first. Slot j was appended at step i - (slots - 1 - j), a model step iff that is
    // >= T, and holds Eq. 1's entry of the symbol that was newest then, x[i - slots + j] = win[T - slots + j]: inside the
    // window when there are at most T slots, otherwise further back in the stream's own bytes (never before its start:
    // a model step's newest symbol has index >= T - 1).
    const int slots = a.Dc / a.c;
    const long long first_slot = (long long)slots - 1 + a.T - w.i;
    const uint8_t *newest = win + (a.T - slots);
    for (int idx = tid; idx < a.Dc; idx += 256) {
      const int j = idx / a.c, qq = idx - j * a.c;
      M[idx] = j >= first_slot ? tab[(size_t)newest[j] * a.c + qq] : (bf16_t)0.0f;
    }
  }
  if (a.conv_W) {  // wavefront w: row w / tiles-per-row of this workgroup, tokens 32 (w % tiles-per-row) ..
    const int wave = tid >> 6, tpr = 4 / rpb, q = wave / tpr, r = blockIdx.x * rpb + q;
    if (r < rows) {
      const int s = r / a.B, b = r - s * a.B;
      WinSrc w = a.ws;
      w.i += s;
      if (stream_active(w, b)) conv_window_mfma(a, stream_window(w, b, a.T), tabXl, (size_t)r, wave % tpr);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Eq. 7's batched product: z[b] = y[b] * W_U[b], one wavefront per stream, lane = output column (d_low = 64)
// ---------------------------------------------------------------------------------------------------
template <typename AT>
__global__ __launch_bounds__(256) void bmm_kernel(const float *y, const AT *WU, AT *z, int B) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= B) return;
  const float yv = y[(size_t)b * 64 + lane];
  const AT *W = WU + (size_t)b * 4096;
  float acc = 0.0f;
#pragma unroll 8
  for (int k = 0; k < 64; ++k) acc = fmaf(__shfl(yv, k, 64), (float)W[k * 64 + lane], acc);
  z[(size_t)b * 64 + lane] = (AT)acc;
}

// ---------------------------------------------------------------------------------------------------
// LayerNorm folded through a product. For u = LN(h) = (h - mean) * rstd * gamma + beta,
//   u W = rstd * (h W' - mean * s) + t,  W' = diag(gamma) W,  s[n] = sum_k W'[k][n],  t[n] = sum_k beta[k] W[k][n],
// so the product runs on the raw activations h and the normalisation becomes a per-row / per-column fix-up in
// the kernel that reduces the split-K partials. s is summed from the bf16 values the matrix cores multiply.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void moments_from_partials(const float *stats, int stats_n, int width, float &mean, float &rstd) {
  fade_row_moments(stats, stats_n, width, mean, rstd);
}

// Eq. 7 between Down and Up (bf16 path): reduce the split-K partials of H_mix W'_down, apply the folded LayerNorm,
// then the per-stream memory: z[b] = y[b] W_U[b]. One wavefront per stream, lane = column (d_low = 64).
__global__ __launch_bounds__(256) void cci_kernel(CciArgs a) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= a.B) return;
  // the stream's W_U (8 KiB, contiguous) as eight 16-byte pieces per lane, requested before anything else: piece
  // lane + 64 i holds row k = lane / 8 + 8 i, columns 8 (lane % 8) .. + 7
  const bf16x8 *Wp = reinterpret_cast<const bf16x8 *>(a.WU + (size_t)(b % a.streams) * 4096) + lane;
  bf16x8 w[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) w[i] = Wp[64 * i];
  float raw = 0.0f;
  for (int s0 = 0; s0 < a.splits; s0 += 8) {  // 8 partials in flight, added in split order
    float pv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) pv[j] = a.part[((size_t)(s0 + j < a.splits ? s0 + j : a.splits - 1) * a.B + b) * 64 + lane];
#pragma unroll
    for (int j = 0; j < 8; ++j) raw += (s0 + j < a.splits) ? pv[j] : 0.0f;
  }
  float mean, rstd;
  moments_from_partials(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd);
  const float yv = rstd * (raw - mean * a.s_fold[lane]) + a.t_fold[lane];
  a.y[(size_t)b * 64 + lane] = yv;
  // z[n] = sum_k y[k] W_U[k][n]: a lane adds its eight rows for its eight columns (k = lane / 8, + 8, ... in order), then the
  // eight lanes that share the columns are added in a fixed tree; lanes 0..7 store 16 bytes each
  const int m = lane >> 3;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float yk = __shfl(yv, m + 8 * i, 64);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = fmaf(yk, (float)w[i][j], acc[j]);
  }
#pragma unroll
  for (int off = 8; off < 64; off <<= 1)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += __shfl_xor(acc[j], off, 64);
  if (m == 0) {
    bf16x8 zv;
#pragma unroll
    for (int j = 0; j < 8; ++j) zv[j] = (bf16_t)acc[j];
    *reinterpret_cast<bf16x8 *>(a.z + (size_t)b * 64 + lane * 8) = zv;
  }
}

// Eq. 9 (bf16 path): reduce the split-K partials of H_coarse [W'_fg | W'_fv] (gate and value interleaved per 128
// columns), apply the folded LayerNorm, H_expand = psi(gate) * value. One thread per 8 output columns.
__global__ __launch_bounds__(256) void geglu_kernel(GegluArgs a) {
  const int chunks = a.De / 8;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)a.B * chunks) return;
  const int b = (int)(t / chunks), j8 = (int)(t % chunks) * 8;
  const int vg = (j8 / 64) * 128 + (j8 & 63), vv = vg + 64, N2 = 2 * a.De;
  float g[8], v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { g[i] = 0.0f; v[i] = 0.0f; }
  for (int s0 = 0; s0 < a.splits; s0 += 4) {  // 4 partials in flight, added in split order
    f32x4 g0[4], g1[4], v0[4], v1[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float *row = a.part + ((size_t)(s0 + j < a.splits ? s0 + j : a.splits - 1) * a.B + b) * N2;
      g0[j] = *reinterpret_cast<const f32x4 *>(row + vg); g1[j] = *reinterpret_cast<const f32x4 *>(row + vg + 4);
      v0[j] = *reinterpret_cast<const f32x4 *>(row + vv); v1[j] = *reinterpret_cast<const f32x4 *>(row + vv + 4);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (s0 + j < a.splits) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { g[i] += g0[j][i]; g[4 + i] += g1[j][i]; v[i] += v0[j][i]; v[4 + i] += v1[j][i]; }
      }
    }
  }
  float mean, rstd;
  moments_from_partials(a.stats + (size_t)b * a.stats_n * 2, a.stats_n, a.Dh, mean, rstd);
  bf16x8 out, eg, ev;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float gi = fade_fold_ln(g[i], mean, rstd, a.s_fold[vg + i], a.t_fold[vg + i]);
    const float vi = fade_fold_ln(v[i], mean, rstd, a.s_fold[vv + i], a.t_fold[vv + i]);
    out[i] = (bf16_t)(gelu_f(gi) * vi);
    eg[i] = (bf16_t)gi;
    ev[i] = (bf16_t)vi;
  }
  const size_t o = (size_t)b * a.De + j8;
  *reinterpret_cast<bf16x8 *>(a.Hexp + o) = out;
  if (a.eg) { *reinterpret_cast<bf16x8 *>(a.eg + o) = eg; *reinterpret_cast<bf16x8 *>(a.ev + o) = ev; }
}

// Eq. 10's tail: H = psi(LN(V)) + lambda_o * H_coarse. One thread per 8 columns.
template <typename AT> __device__ __forceinline__ void ldv8(const AT *p, float v[8]);
template <> __device__ __forceinline__ void ldv8<bf16_t>(const bf16_t *p, float v[8]) {
  const bf16x8 r = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)r[i];
}
template <> __device__ __forceinline__ void ldv8<float>(const float *p, float v[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
}
template <typename AT> __device__ __forceinline__ void stv8(AT *p, const float v[8]);
template <> __device__ __forceinline__ void stv8<bf16_t>(bf16_t *p, const float v[8]) {
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (bf16_t)v[i];
  *reinterpret_cast<bf16x8 *>(p) = r;
}
template <> __device__ __forceinline__ void stv8<float>(float *p, const float v[8]) {
  f32x4 a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
  *reinterpret_cast<f32x4 *>(p) = a;
  *reinterpret_cast<f32x4 *>(p + 4) = b;
}
template <typename AT, int RPT>
__global__ __launch_bounds__(256) void hout_kernel(HoutArgs a) {
  __shared__ float mom[FADE_GROUP_ROWS_MAX][2];
  const int chunks = a.Dh / 8;
  const int r0 = fade_group_moments<RPT>(a.stats, a.stats_n, a.Dh, chunks, a.B, mom);
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)((a.B + RPT - 1) / RPT) * chunks) return;
  const int b0 = (int)(t / chunks) * RPT, c8 = (int)(t % chunks) * 8;
  float v[RPT][8], hc[RPT][8], ga[8], be[8];
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    if (b0 + i >= a.B) continue;
    const size_t o = (size_t)(b0 + i) * a.Dh + c8;
    ldv8<AT>(static_cast<const AT *>(a.V) + o, v[i]);
    ldv8<AT>(static_cast<const AT *>(a.Hc) + o, hc[i]);
  }
  ldv8<float>(a.gamma + c8, ga);
  ldv8<float>(a.beta + c8, be);
  const float lam = a.lam[0];
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    if (b0 + i >= a.B) continue;
    const float mean = mom[b0 + i - r0][0], rstd = mom[b0 + i - r0][1];
    float out[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = gelu_f((v[i][j] - mean) * rstd * ga[j] + be[j]) + lam * hc[i][j];
    stv8<AT>(static_cast<AT *>(a.Hout) + (size_t)(b0 + i) * a.Dh + c8, out);
  }
}

// The same in fp32, 4 elements per thread.
__global__ __launch_bounds__(256) void residual_add_f32_kernel(const float *x, const float *y, const float *lam, float *out, size_t n4) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= n4) return;
  const f32x4 xv = reinterpret_cast<const f32x4 *>(x)[t], yv = reinterpret_cast<const f32x4 *>(y)[t];
  const float l = lam[0];
  f32x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = fmaf(l, yv[i], xv[i]);
  reinterpret_cast<f32x4 *>(out)[t] = o;
}

// Eq. 8 with its gate switched off (ablation level 3): out = x + lam * y, 8 bf16 per thread.
__global__ __launch_bounds__(256) void residual_add_kernel(const bf16_t *x, const bf16_t *y, const float *lam, bf16_t *out, size_t n8) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= n8) return;
  const bf16x8 xv = reinterpret_cast<const bf16x8 *>(x)[t], yv = reinterpret_cast<const bf16x8 *>(y)[t];
  const float l = lam[0];
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (bf16_t)fmaf(l, (float)yv[i], (float)xv[i]);
  reinterpret_cast<bf16x8 *>(out)[t] = o;
}

// All element-wise weight preparation of one refresh in a single launch: blockIdx.y picks the descriptor.
__global__ __launch_bounds__(256) void prep_batch_kernel(PrepBatch pb) {
  if ((int)blockIdx.y == pb.count) {  // the per-symbol tables: workgroup x = symbol x
    const TablesArgs &t = pb.tab;
    if (blockIdx.x < 256) {
      tables_body<bf16_t>(blockIdx.x, t.E, t.round_bf16 != 0, t.ge, t.be, t.gl, t.bl, t.D, static_cast<bf16_t *>(t.tabXe), static_cast<bf16_t *>(t.tabXl),
                          t.tabXe32, t.tabXhat, t.tabRstd);
      if (t.Wg) tables_slot_body(blockIdx.x, t);
    }
    return;
  }
  const PrepDesc &d = pb.d[blockIdx.y];
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (d.kind == PREP_ROUND) {
    if (t < (size_t)d.N) static_cast<float *>(d.out)[t] = (float)(bf16_t)d.W0[t];
    return;
  }
  const bool tr = d.kind == PREP_FRAG_T;
  const int Kv = tr ? d.N : d.K, Nv = tr ? d.K : d.N;  // shape of the matrix whose fragments are written
  const size_t total = (size_t)(Nv / 32) * (Kv / 16) * 64;
  if (t >= total) return;
  const int lane = (int)(t & 63);
  const size_t frag = t >> 6;
  const int ks = (int)(frag % (size_t)(Kv / 16)), nt = (int)(frag / (size_t)(Kv / 16));
  const int n = nt * 32 + (lane & 31);
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = ks * 16 + (lane >> 5) * 8 + i;
    float w;
    if (d.kind == PREP_FRAG_CONVT) {
      const int rr = k / d.D, o = k - rr * d.D;
      w = rr < d.taps ? d.W0[((size_t)rr * d.D + n) * d.D + o] : 0.0f;
    } else {
      const int row = tr ? n : k, v = tr ? k : n;  // position in the (virtual) source [K][N]
      const float *src = d.W0;
      int col = v, ld = d.N;
      if (d.interleave) {
        ld = d.N / 2;
        col = (v / 128) * 64 + (v & 63);
        if ((v & 127) >= 64) src = d.W1;
      }
      w = (tr || row < d.k_real) ? src[(size_t)row * ld + col] : 0.0f;
      if (!tr && d.rowscale && row < d.k_real) w = d.rowscale[row] * (float)(bf16_t)w;
    }
    r[i] = (bf16_t)w;
  }
  reinterpret_cast<bf16x8 *>(d.out)[t] = r;
}

// Eq. 4 backward w.r.t. its input is again a (anti-causal) convolution; its weight as a product operand:
// V[(r * D + o)][i] = W_conv[r][i][o], rows past taps * D are zero. fp32 [Kc][D].
__global__ void convt_build_kernel(const float *Wconv, int taps, int D, int Kc, float *V) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= Kc * D) return;
  const int row = t / D, i = t - row * D;
  const int r = row / D, o = row - r * D;
  V[t] = (r < taps) ? Wconv[((size_t)r * D + i) * D + o] : 0.0f;
}

// Fragments of the transpose: virtual V[k'][n'] = W[n'][k'] with W the (possibly interleaved) [K][N] matrix, so V is [N][K]:
// reduction index k' runs over W's columns, output column n' over W's rows.
__global__ void preshuffle_t_kernel(const float *W0, const float *W1, int K, int N, int interleave, bf16_t *out) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one thread per (fragment, lane)
  const int Kv = N, Nv = K;
  const size_t total = (size_t)(Nv / 32) * (Kv / 16) * 64;
  if (t >= total) return;
  const int lane = (int)(t & 63);
  const size_t frag = t >> 6;
  const int ks = (int)(frag % (size_t)(Kv / 16)), nt = (int)(frag / (size_t)(Kv / 16));
  const int row = nt * 32 + (lane & 31);  // row of W
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int v = ks * 16 + (lane >> 5) * 8 + i;  // column of the virtual W
    const float *src = W0;
    int col = v, ld = N;
    if (interleave) {
      ld = N / 2;
      col = (v / 128) * 64 + (v & 63);
      if ((v & 127) >= 64) src = W1;
    }
    r[i] = (bf16_t)src[(size_t)row * ld + col];
  }
  reinterpret_cast<bf16x8 *>(out)[t] = r;
}

// ---------------------------------------------------------------------------------------------------
// probabilities -> frequencies (wavefront-wide, lane l owns symbols 4l .. 4l+3)
// f_i = 1 + trunc(fp32(p_i * 65280)); the remainder 65536 - sum f goes to the lowest index of the maximum.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ bool quantize_wave(const float p[4], int lane, uint32_t q[4]) {
  bool ok = true;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ok = ok && (p[i] >= 0.0f) && (p[i] <= 1.0f);
    q[i] = 1u + (uint32_t)__fmul_rn(p[i], 65280.0f);
  }
  const uint32_t total = wave_sum<uint32_t>(q[0] + q[1] + q[2] + q[3]);
  uint32_t best = q[0], bi = 0;
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (q[i] > best) { best = q[i]; bi = i; }
  // order by (value, then smaller index): key = value << 10 | (1023 - index)
  uint32_t key = (best << 10) | (1023u - (uint32_t)(4 * lane + bi));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = __shfl_xor(key, off, 64);
    key = o > key ? o : key;
  }
  const int arg = 1023 - (int)(key & 1023u);
  if ((arg >> 2) == lane) q[arg & 3] += 65536u - total;  // wraps correctly when total > 65536
  return __all(ok);
}

// Exclusive prefix of the lane totals; cum[i] = sum of every frequency before symbol 4*lane + i.
__device__ __forceinline__ void cumulate_wave(const uint32_t q[4], int lane, uint32_t cum[4]) {
  const uint32_t tot = q[0] + q[1] + q[2] + q[3];
  uint32_t inc = tot;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(inc, off, 64);
    if (lane >= off) inc += o;
  }
  const uint32_t base = inc - tot;
  cum[0] = base; cum[1] = base + q[0]; cum[2] = cum[1] + q[1]; cum[3] = cum[2] + q[2];
}

// ---------------------------------------------------------------------------------------------------
// arithmetic coder: 32-bit interval, totals 2^16, bit-plus-follow carries, bits MSB first
// ---------------------------------------------------------------------------------------------------
constexpr uint32_t kQuarter = 0x40000000u;

struct EncState {
  uint32_t low, high, pending, bitbuf, nbits, pos;
};
__device__ __forceinline__ void enc_load(const CoderBufs &c, int b, EncState &e) {
  e.low = c.low[b]; e.high = c.high[b]; e.pending = c.pending[b]; e.bitbuf = c.bitbuf[b]; e.nbits = c.nbits[b]; e.pos = c.pos[b];
}
__device__ __forceinline__ void enc_store(const CoderBufs &c, int b, const EncState &e) {
  c.low[b] = e.low; c.high[b] = e.high; c.pending[b] = e.pending; c.bitbuf[b] = e.bitbuf; c.nbits[b] = e.nbits; c.pos[b] = e.pos;
}
__device__ __forceinline__ void put_bit(const CoderBufs &c, int b, EncState &e, uint32_t bit) {
  e.bitbuf = (e.bitbuf << 1) | bit;
  if (++e.nbits == 8) {
    if (e.pos < c.cap) c.out[(size_t)b * c.cap + e.pos] = (uint8_t)e.bitbuf;
    else *c.err = 1;  // payload buffer exhausted: flagged, never written out of bounds
    ++e.pos; e.bitbuf = 0; e.nbits = 0;
  }
}
__device__ __forceinline__ void emit(const CoderBufs &c, int b, EncState &e, uint32_t bit) {
  put_bit(c, b, e, bit);
  for (; e.pending > 0; --e.pending) put_bit(c, b, e, bit ^ 1u);
}
// Append the low `count` (<= 32) bits of `value`, most significant first.
__device__ __forceinline__ void put_bits(const CoderBufs &c, int b, EncState &e, uint32_t value, uint32_t count) {
  uint64_t acc = ((uint64_t)e.bitbuf << count) | value;
  uint32_t total = e.nbits + count;  // < 40
  while (total >= 8) {
    total -= 8;
    if (e.pos < c.cap) c.out[(size_t)b * c.cap + e.pos] = (uint8_t)(acc >> total);
    else *c.err = 1;  // payload buffer exhausted: flagged, never written out of bounds
    ++e.pos;
  }
  e.bitbuf = (uint32_t)acc & ((1u << total) - 1u);
  e.nbits = total;
}
// One symbol. The renormalisation loop of the classic coder (shift out a settled top bit, or drop the second bit while the
// interval straddles the middle) always runs as n shifts of the first kind followed by m of the second: once the top bits of
// low and high differ they stay different. Both counts are leading-bit counts, so the loop is done in closed form:
//   n = leading bits in which low and high agree; they are the output: the first of them, then the `pending` opposite
//       bits owed from earlier straddles, then the other n - 1;
//   m = after those shifts, the length of the run 0111.. / 1000.. below the top bit; pending becomes m (plus the old
//       count when n = 0), and the run is cut out of both bounds.
// The interval is wider than 2^30 before and at least 2^14 - 1 after the update, so n <= 18 and m <= 30.
__device__ __forceinline__ void enc_symbol(const CoderBufs &c, int b, EncState &e, uint32_t cum_lo, uint32_t cum_hi) {
  const uint64_t range = (uint64_t)e.high - e.low + 1;
  uint32_t high = e.low + (uint32_t)((range * cum_hi) >> 16) - 1;
  uint32_t low = e.low + (uint32_t)((range * cum_lo) >> 16);
  const uint32_t n = (uint32_t)__clz((int)(low ^ high));
  if (n > 0) {
    const uint32_t b0 = low >> 31;
    put_bits(c, b, e, b0, 1);
    for (uint32_t left = e.pending; left > 0;) {
      const uint32_t k = left < 32u ? left : 32u;
      put_bits(c, b, e, b0 ? 0u : (k == 32u ? 0xFFFFFFFFu : (1u << k) - 1u), k);
      left -= k;
    }
    e.pending = 0;
    if (n > 1) put_bits(c, b, e, (low >> (32 - n)) & ((1u << (n - 1)) - 1u), n - 1);
    low <<= n;
    high = (high << n) | ((1u << n) - 1u);
  }
  const uint32_t m = (uint32_t)__clz((int)~((low & ~high) << 1));
  if (m > 0) {
    e.pending += m;
    low = (low << m) & 0x7FFFFFFFu;
    high = (high << m) | ((1u << m) - 1u) | 0x80000000u;
  }
  e.low = low; e.high = high;
}
__device__ __forceinline__ void enc_finish(const CoderBufs &c, int b, EncState &e) {
  ++e.pending;
  emit(c, b, e, e.low < kQuarter ? 0u : 1u);
  while (e.nbits != 0) put_bit(c, b, e, 0);
}

struct DecState {
  uint32_t low, high, value, bitpos;
};
__device__ __forceinline__ uint32_t dec_bit(const CoderBufs &c, int b, DecState &d) {
  const uint32_t byte = d.bitpos >> 3;
  uint32_t bit = 0;
  if (byte < c.in_len[b]) bit = (c.in[(size_t)b * c.cap + byte] >> (7 - (d.bitpos & 7))) & 1u;
  ++d.bitpos;  // zeros past the end
  return bit;
}
__device__ __forceinline__ uint32_t dec_target(const DecState &d) {
  const uint64_t range = (uint64_t)d.high - d.low + 1;
  return (uint32_t)((((((uint64_t)(d.value - d.low)) + 1) << 16) - 1) / range);
}
// The next `count` (<= 25) payload bits of stream b, zeros past the end.
__device__ __forceinline__ uint32_t dec_bits(const CoderBufs &c, int b, DecState &d, uint32_t count) {
  const uint32_t byte0 = d.bitpos >> 3, off = d.bitpos & 7u, len = c.in_len[b];
  const uint8_t *in = c.in + (size_t)b * c.cap;
  uint32_t w = 0;
#pragma unroll
  for (uint32_t k = 0; k < 4; ++k) w = (w << 8) | (byte0 + k < len ? (uint32_t)in[byte0 + k] : 0u);
  d.bitpos += count;
  return count ? (w << off) >> (32 - count) : 0u;
}
// The decoder's side of enc_symbol's closed form: the same n and m (the bounds do not depend on the payload), `value`
// shifted along with them; a straddle step removes the bit below the top one.
__device__ __forceinline__ void dec_update(const CoderBufs &c, int b, DecState &d, uint32_t cum_lo, uint32_t cum_hi) {
  const uint64_t range = (uint64_t)d.high - d.low + 1;
  uint32_t high = d.low + (uint32_t)((range * cum_hi) >> 16) - 1;
  uint32_t low = d.low + (uint32_t)((range * cum_lo) >> 16);
  uint32_t value = d.value;
  const uint32_t n = (uint32_t)__clz((int)(low ^ high));
  if (n > 0) {
    low <<= n;
    high = (high << n) | ((1u << n) - 1u);
    value = (value << n) | dec_bits(c, b, d, n);
  }
  uint32_t m = (uint32_t)__clz((int)~((low & ~high) << 1));
  if (m > 0) {
    low = (low << m) & 0x7FFFFFFFu;
    high = (high << m) | ((1u << m) - 1u) | 0x80000000u;
    while (m > 0) {
      const uint32_t k = m < 24u ? m : 24u;
      value = (value & 0x80000000u) | ((value << k) & 0x7FFFFFFFu) | dec_bits(c, b, d, k);
      m -= k;
    }
  }
  d.low = low; d.high = high; d.value = value;
}

// Code one symbol of stream b under the table q (lane-distributed). mode: CODE_NONE / CODE_ENCODE / CODE_DECODE.
template <int MODE>
__device__ __forceinline__ void code_wave(const CoderBufs &c, int b, int lane, const uint32_t q[4], uint8_t *sym_ptr) {
  if (MODE == CODE_NONE) return;
  uint32_t cum[4];
  cumulate_wave(q, lane, cum);
  if (MODE == CODE_ENCODE) {
    const int s = *sym_ptr;
    const uint32_t mylo = cum[s & 3], myhi = mylo + q[s & 3];
    const uint32_t lo = __shfl(mylo, s >> 2, 64), hi = __shfl(myhi, s >> 2, 64);
    if (lane == 0) {
      EncState e;
      enc_load(c, b, e);
      enc_symbol(c, b, e, lo, hi);
      enc_store(c, b, e);
    }
  } else {
    DecState d;
    d.low = c.low[b]; d.high = c.high[b]; d.value = c.value[b]; d.bitpos = c.bitpos[b];
    const uint32_t target = dec_target(d);
    int found = -1;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (cum[i] <= target && target < cum[i] + q[i]) found = i;
    const unsigned long long vote = __ballot(found >= 0);
    if (vote == 0ull) {  // target outside [0, 2^16): the payload does not belong to this model
      if (lane == 0) *c.err = 2;
      return;
    }
    const int owner = __ffsll((long long)vote) - 1;
    const int fi = found < 0 ? 0 : found;
    const uint32_t lo = __shfl(cum[fi], owner, 64), hi = __shfl(cum[fi] + q[fi], owner, 64);
    const int s = __shfl(4 * lane + fi, owner, 64);
    if (lane == 0) {
      dec_update(c, b, d, lo, hi);
      c.low[b] = d.low; c.high[b] = d.high; c.value[b] = d.value; c.bitpos[b] = d.bitpos;
      *sym_ptr = (uint8_t)s;
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// softmax over the 256 logits of a stream, quantise, code: one wavefront per stream
// ---------------------------------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void softmax_quant_code_kernel(SqcArgs a) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;  // row
  if (b >= a.B) return;
  WinSrc w = a.ws;
  int sb = b;  // stream of this row
  if (MODE == CODE_RANGES) {
    const int st = b / a.streams;
    sb = b - st * a.streams;
    w.i += st;
  }
  if (!stream_active(w, sb)) return;
  f32x4 z = *reinterpret_cast<const f32x4 *>(a.logits + (size_t)b * 256 + 4 * lane);
  if (a.splits > 0) {  // logits arrive as split-K partials; the head's bias is added here
    for (int s0 = 1; s0 < a.splits; s0 += 8) {  // up to 8 partials in flight, added in split order
      f32x4 zp[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        zp[j] = *reinterpret_cast<const f32x4 *>(a.logits + ((size_t)(s0 + j < a.splits ? s0 + j : a.splits - 1) * a.B + b) * 256 + 4 * lane);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (s0 + j < a.splits) z += zp[j];
    }
    z += *reinterpret_cast<const f32x4 *>(a.bias + 4 * lane);
    if (a.logits_out) *reinterpret_cast<f32x4 *>(a.logits_out + (size_t)b * 256 + 4 * lane) = z;
  }
  const float mx = wave_max(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])));
  float p[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) p[i] = expf(z[i] - mx);
  const float sum = wave_sum<float>((p[0] + p[1]) + (p[2] + p[3]));
#pragma unroll
  for (int i = 0; i < 4; ++i) p[i] = p[i] / sum;
  if (a.probs) {
    f32x4 o = {p[0], p[1], p[2], p[3]};
    *reinterpret_cast<f32x4 *>(a.probs + (size_t)b * 256 + 4 * lane) = o;
  }
  uint32_t q[4];
  if (!quantize_wave(p, lane, q)) {
    if (lane == 0) *a.cb.err = 3;  // non-finite probabilities
    return;
  }
  if (a.freq) {
    ushort4 f = make_ushort4((unsigned short)q[0], (unsigned short)q[1], (unsigned short)q[2], (unsigned short)q[3]);
    *reinterpret_cast<ushort4 *>(a.freq + (size_t)b * 256 + 4 * lane) = f;
  }
  if (MODE == CODE_RANGES) {
    uint32_t cum[4];
    cumulate_wave(q, lane, cum);
    const int sy = a.sym_base[(long long)sb * w.stride + w.i];
    const uint32_t mylo = cum[sy & 3], myhi = mylo + q[sy & 3];
    const uint32_t lo = __shfl(mylo, sy >> 2, 64), hi = __shfl(myhi, sy >> 2, 64);
    if (lane == 0) a.ranges[b] = make_uint2(lo, hi);
  } else if (MODE != CODE_NONE) {
    uint8_t *sym = a.sym_base + (long long)b * a.ws.stride + a.ws.i;
    code_wave<MODE>(a.cb, b, lane, q, sym);
  }
}

// Second half of a multi-step encode: feed each stream's S intervals, in step order, to its coder. One thread per stream;
// the intervals come through LDS in slabs of 16 steps so that the coder's dependent chain never waits on HBM.
__global__ __launch_bounds__(64) void encode_ranges_kernel(WinSrc ws, const uint2 *ranges, int B, int S, CoderBufs cb) {
  __shared__ uint2 slab[16][64];
  const int b = blockIdx.x * 64 + threadIdx.x;
  const bool mine = b < B;
  EncState e;
  if (mine) enc_load(cb, b, e);
  bool live = mine;
  for (int s0 = 0; s0 < S; s0 += 16) {
    __syncthreads();
    if (mine) {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (s0 + j < S) slab[j][threadIdx.x] = ranges[(size_t)(s0 + j) * B + b];
    }
    __syncthreads();
    for (int j = 0; j < 16 && s0 + j < S && live; ++j) {
      WinSrc w = ws;
      w.i += s0 + j;
      live = stream_active(w, b);  // a stream that has ended stays ended
      if (live) enc_symbol(cb, b, e, slab[j][threadIdx.x].x, slab[j][threadIdx.x].y);
    }
  }
  if (mine) enc_store(cb, b, e);
}

__global__ __launch_bounds__(256) void quantize_kernel(const float *probs, size_t rows, uint16_t *freq, int *err) {
  const size_t r = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= rows) return;
  const f32x4 pv = *reinterpret_cast<const f32x4 *>(probs + r * 256 + 4 * lane);
  const float p[4] = {pv[0], pv[1], pv[2], pv[3]};
  uint32_t q[4];
  if (!quantize_wave(p, lane, q)) {
    if (lane == 0) *err = 3;
    return;
  }
  ushort4 f = make_ushort4((unsigned short)q[0], (unsigned short)q[1], (unsigned short)q[2], (unsigned short)q[3]);
  *reinterpret_cast<ushort4 *>(freq + r * 256 + 4 * lane) = f;
}

// Code one symbol per stream under explicit tables freq[stream][256] (the stand-alone coder entry points).
template <int MODE>
__global__ __launch_bounds__(256) void code_tables_kernel(const uint16_t *freq, uint8_t *sym, int n_streams, CoderBufs cb) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= n_streams) return;
  const ushort4 f = *reinterpret_cast<const ushort4 *>(freq + (size_t)b * 256 + 4 * lane);
  const uint32_t q[4] = {f.x, f.y, f.z, f.w};
  code_wave<MODE>(cb, b, lane, q, sym + b);
}

// Algorithm 1's first T symbols: every symbol has frequency 256 (p = 1/256). One thread per stream.
template <int MODE>
__global__ void code_uniform_kernel(WinSrc ws, uint8_t *sym_base, int B, CoderBufs cb) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B || !stream_active(ws, b)) return;
  uint8_t *sym = sym_base + (long long)b * ws.stride + ws.i;
  if (MODE == CODE_ENCODE) {
    const uint32_t s = *sym;
    EncState e;
    enc_load(cb, b, e);
    enc_symbol(cb, b, e, s * 256u, (s + 1u) * 256u);
    enc_store(cb, b, e);
  } else {
    DecState d;
    d.low = cb.low[b]; d.high = cb.high[b]; d.value = cb.value[b]; d.bitpos = cb.bitpos[b];
    const uint32_t target = dec_target(d);
    if (target >= 65536u) { *cb.err = 2; return; }
    const uint32_t s = target >> 8;
    dec_update(cb, b, d, s * 256u, (s + 1u) * 256u);
    cb.low[b] = d.low; cb.high[b] = d.high; cb.value[b] = d.value; cb.bitpos[b] = d.bitpos;
    *sym = (uint8_t)s;
  }
}

// Reset coder state; for decoding also prime `value` with the first 32 payload bits.
__global__ void coder_init_kernel(CoderBufs cb, int B, int decode) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  cb.low[b] = 0; cb.high[b] = 0xFFFFFFFFu; cb.pending[b] = 0; cb.bitbuf[b] = 0; cb.nbits[b] = 0; cb.pos[b] = 0;
  cb.value[b] = 0; cb.bitpos[b] = 0;
  if (decode) {
    DecState d = {0u, 0xFFFFFFFFu, 0u, 0u};
    for (int i = 0; i < 32; ++i) d.value = (d.value << 1) | dec_bit(cb, b, d);
    cb.value[b] = d.value; cb.bitpos[b] = d.bitpos;
  }
}

// Terminate every non-empty stream's payload; pos[b] becomes its byte length.
__global__ void coder_finish_kernel(CoderBufs cb, int B, long long stride, long long n) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  if ((long long)b * stride >= n) return;  // empty stream: zero-length payload
  EncState e;
  enc_load(cb, b, e);
  enc_finish(cb, b, e);
  enc_store(cb, b, e);
}

// Move per-stream payloads between the strided working buffer [B][cap] and one contiguous run (offsets[b], lens[b]).
// gather != 0: strided -> contiguous (after encoding); else contiguous -> strided (before decoding).
__global__ __launch_bounds__(256) void payload_move_kernel(uint8_t *strided, size_t cap, uint8_t *flat, const unsigned long long *offsets,
                                                           const uint32_t *lens, int gather) {
  const int b = blockIdx.x;
  const uint32_t len = lens[b];
  uint8_t *s = strided + (size_t)b * cap, *f = flat + offsets[b];
  for (uint32_t i = threadIdx.x; i < len; i += 256) {
    if (gather) f[i] = s[i];
    else s[i] = f[i];
  }
}

inline unsigned blocks_for(size_t n, unsigned per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

// ---------------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------------
hipError_t fade_preshuffle(const float *W0, const float *W1, int k_real, int K, int N, int interleave, const float *rowscale, void *out,
                           hipStream_t s) {
  const size_t total = (size_t)(N / 32) * (K / 16) * 64;
  hipLaunchKernelGGL(preshuffle_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, W0, W1, k_real, K, N, interleave, rowscale,
                     static_cast<bf16_t *>(out));
  return hipGetLastError();
}
hipError_t fade_virtual_copy(const float *W0, const float *W1, int k_real, int K, int N, int interleave, float *out, hipStream_t s) {
  hipLaunchKernelGGL(virtual_copy_kernel, dim3(blocks_for((size_t)K * N, 256)), dim3(256), 0, s, W0, W1, k_real, K, N,
                     interleave, out);
  return hipGetLastError();
}
hipError_t fade_convert(const float *src, void *dst, size_t n, bool bf16, hipStream_t s) {
  if (bf16) hipLaunchKernelGGL(convert_kernel<bf16_t>, dim3(blocks_for(n, 256)), dim3(256), 0, s, src, static_cast<bf16_t *>(dst), n);
  else hipLaunchKernelGGL(convert_kernel<float>, dim3(blocks_for(n, 256)), dim3(256), 0, s, src, static_cast<float *>(dst), n);
  return hipGetLastError();
}
hipError_t fade_round_bf16(const float *src, float *dst, size_t n, hipStream_t s) {
  hipLaunchKernelGGL(round_bf16_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, src, dst, n);
  return hipGetLastError();
}
hipError_t fade_tables(const float *E, const float *ge, const float *be, const float *gl, const float *bl, int D, void *tabXe,
                       void *tabXl, float *tabXe32, float *tabXhat, float *tabRstd, bool bf16, hipStream_t s) {
  if (D > 256) return hipErrorInvalidValue;
  if (bf16)
    hipLaunchKernelGGL(tables_kernel<bf16_t>, dim3(256), dim3(256), 0, s, E, ge, be, gl, bl, D, static_cast<bf16_t *>(tabXe),
                       static_cast<bf16_t *>(tabXl), tabXe32, tabXhat, tabRstd);
  else
    hipLaunchKernelGGL(tables_kernel<float>, dim3(256), dim3(256), 0, s, E, ge, be, gl, bl, D, static_cast<float *>(tabXe),
                       static_cast<float *>(tabXl), tabXe32, tabXhat, tabRstd);
  return hipGetLastError();
}
hipError_t fade_embed_cache(const EmbedArgs &a, int B, bool bf16, hipStream_t s) {
  if (a.Dc > 4096 || a.c > 256 || a.c <= 0) return hipErrorInvalidValue;  // the kernel's register file holds one cache row
  if (a.conv_W && (!bf16 || a.D != 32 || a.T > 128 || a.Kc % 16 || a.Kc > 128 || a.taps * 32 > a.Kc || !a.Hl || !a.conv_b)) return hipErrorInvalidValue;
  // One wavefront per 32-token tile of Eq. 4 when that is fewer than four: every wavefront then carries the same work (on
  // 256 threads the tiles' matrix work and activations sit on T / 32 of the four SIMDs), and a compute unit holds twice as
  // many streams, each a chain of dependent round trips (window byte -> table piece -> store).
  int nt = 256;
  if (a.conv_W && a.T % 32 == 0 && a.T < 128 && a.c % 8 == 0 && a.Dc / 8 <= 4 * 2 * a.T && a.c <= 2 * a.T) nt = 2 * a.T;
  const bool frozen_shape = a.slot_tab && !a.XL && !a.cv, adapting_shape = !a.slot_tab && a.gg_tab && a.gv_tab;
  if (bf16 && a.conv_W && (a.T == 32 || a.T == 64 || a.T == 128) && (a.c % 8 == 0 || a.c == 4) && a.Dc % 8 == 0 && a.Dc / 8 <= 64 && a.c <= 64 && a.Dh == a.T * 32 && a.ws.i >= a.T &&
      (a.ws.active || a.ws.n >= a.T) && (frozen_shape || adapting_shape) && B >= 1) {
    static const int per_cu = getenv("FADE_EMBED_WGS") ? atoi(getenv("FADE_EMBED_WGS")) : 3;
    EmbedArgs p = a;
    p.B = B;
    const int ngrp = 4 / (a.T / 32), want = (B + ngrp - 1) / ngrp;
    const int G = want < 256 * per_cu ? want : 256 * per_cu;
    if (per_cu > 0) {
      const bool half = a.c == 4;
      if (a.Kc <= 96 || a.taps <= 3) {
        if (half && frozen_shape) hipLaunchKernelGGL((embed_cache_lds_kernel<6, false, true>), dim3(G), dim3(256), 0, s, p);
        else if (half) hipLaunchKernelGGL((embed_cache_lds_kernel<6, true, true>), dim3(G), dim3(256), 0, s, p);
        else if (frozen_shape) hipLaunchKernelGGL((embed_cache_lds_kernel<6, false>), dim3(G), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((embed_cache_lds_kernel<6, true>), dim3(G), dim3(256), 0, s, p);
      } else {
        if (half && frozen_shape) hipLaunchKernelGGL((embed_cache_lds_kernel<8, false, true>), dim3(G), dim3(256), 0, s, p);
        else if (half) hipLaunchKernelGGL((embed_cache_lds_kernel<8, true, true>), dim3(G), dim3(256), 0, s, p);
        else if (frozen_shape) hipLaunchKernelGGL((embed_cache_lds_kernel<8, false>), dim3(G), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((embed_cache_lds_kernel<8, true>), dim3(G), dim3(256), 0, s, p);
      }
      return hipGetLastError();
    }
  }
  if (!bf16) hipLaunchKernelGGL((embed_cache_kernel<float, 8, 4>), dim3(B), dim3(nt), 0, s, a);
  else if (a.conv_W && (a.Kc <= 96 || a.taps <= 3) && a.c % 8 == 0 && a.Dc / 8 <= nt) hipLaunchKernelGGL((embed_cache_kernel<bf16_t, 6, 1>), dim3(B), dim3(nt), 0, s, a);
  else hipLaunchKernelGGL((embed_cache_kernel<bf16_t, 8, 4>), dim3(B), dim3(nt), 0, s, a);
  return hipGetLastError();
}
hipError_t fade_embed_steps(const EmbedArgs &a, hipStream_t s) {
  if (!a.slot_tab || a.B <= 0 || a.S <= 0 || a.Dh % 8) return hipErrorInvalidValue;
  if (a.conv_W && (a.D != 32 || a.T > 128 || a.Kc % 16 || a.Kc > 128 || a.taps * 32 > a.Kc || !a.Hl || !a.conv_b)) return hipErrorInvalidValue;
  const int tiles = (a.T + 31) / 32, rpb = (a.conv_W && tiles <= 2) ? 4 / tiles : 1;  // tiles = 3 or 4: one row, idle wavefronts
  hipLaunchKernelGGL(embed_steps_kernel, dim3((a.B * a.S + rpb - 1) / rpb), dim3(256), 0, s, a, rpb);
  return hipGetLastError();
}
__global__ void fill_u32_kernel(uint32_t *dst, uint32_t value, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = value;
}
hipError_t fade_fill_u32(uint32_t *dst, uint32_t value, size_t n, hipStream_t s) {
  if (!n) return hipSuccess;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, value, n);
  return hipGetLastError();
}
hipError_t fade_encode_ranges(const WinSrc &ws, const uint2 *ranges, int B, int S, const CoderBufs &cb, hipStream_t s) {
  hipLaunchKernelGGL(encode_ranges_kernel, dim3((B + 63) / 64), dim3(64), 0, s, ws, ranges, B, S, cb);
  return hipGetLastError();
}
hipError_t fade_bmm(const float *y, const void *WU, void *z, int B, bool bf16, hipStream_t s) {
  if (bf16)
    hipLaunchKernelGGL(bmm_kernel<bf16_t>, dim3((B + 3) / 4), dim3(256), 0, s, y, static_cast<const bf16_t *>(WU), static_cast<bf16_t *>(z), B);
  else
    hipLaunchKernelGGL(bmm_kernel<float>, dim3((B + 3) / 4), dim3(256), 0, s, y, static_cast<const float *>(WU), static_cast<float *>(z), B);
  return hipGetLastError();
}
// st_out: [2][N] (s then t); part: scratch of 16 * 2 * N floats
hipError_t fade_cci(const CciArgs &a, hipStream_t s) {
  hipLaunchKernelGGL(cci_kernel, dim3((a.B + 3) / 4), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t fade_geglu(const GegluArgs &a, hipStream_t s) {
  hipLaunchKernelGGL(geglu_kernel, dim3(blocks_for((size_t)a.B * (a.De / 8), 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t fade_residual_add(const void *x, const void *y, const float *lam, void *out, size_t n, bool bf16, hipStream_t s) {
  if (n % 8) return hipErrorInvalidValue;
  if (!bf16) {
    hipLaunchKernelGGL(residual_add_f32_kernel, dim3(blocks_for(n / 4, 256)), dim3(256), 0, s, static_cast<const float *>(x), static_cast<const float *>(y),
                       lam, static_cast<float *>(out), n / 4);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(residual_add_kernel, dim3(blocks_for(n / 8, 256)), dim3(256), 0, s, static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(y),
                     lam, static_cast<bf16_t *>(out), n / 8);
  return hipGetLastError();
}
hipError_t fade_hout(const HoutArgs &a, bool bf16, hipStream_t s) {
  if (a.Dh % 8 || a.Dh < 64 || a.B <= 0) return hipErrorInvalidValue;
  const int rpt = fade_rows_per_thread(a.B, a.Dh / 8);
  const dim3 grid(blocks_for((size_t)((a.B + rpt - 1) / rpt) * (a.Dh / 8), 256));
  if (rpt == 4) {
    if (bf16) hipLaunchKernelGGL((hout_kernel<bf16_t, 4>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((hout_kernel<float, 4>), grid, dim3(256), 0, s, a);
  } else {
    if (bf16) hipLaunchKernelGGL((hout_kernel<bf16_t, 1>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((hout_kernel<float, 1>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}
hipError_t fade_preshuffle_t(const float *W0, const float *W1, int K, int N, int interleave, void *out, hipStream_t s) {
  const size_t total = (size_t)(K / 32) * (N / 16) * 64;
  hipLaunchKernelGGL(preshuffle_t_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, W0, W1, K, N, interleave, static_cast<bf16_t *>(out));
  return hipGetLastError();
}
hipError_t fade_prep_batch(const PrepBatch &pb, hipStream_t s) {
  if (pb.count <= 0 || pb.count > 20) return hipErrorInvalidValue;
  size_t most = 0;
  for (int i = 0; i < pb.count; ++i) {
    const PrepDesc &d = pb.d[i];
    size_t n;
    if (d.kind == PREP_ROUND) n = (size_t)d.N;
    else if (d.kind == PREP_FRAG_T) n = (size_t)(d.K / 32) * (d.N / 16) * 64;
    else n = (size_t)(d.N / 32) * (d.K / 16) * 64;
    if (n > most) most = n;
  }
  if (pb.has_tables) {
    if (pb.tab.D > 256) return hipErrorInvalidValue;
    if (most < 256 * 256) most = 256 * 256;  // 256 workgroups for the tables
  }
  hipLaunchKernelGGL(prep_batch_kernel, dim3(blocks_for(most, 256), pb.count + (pb.has_tables ? 1 : 0)), dim3(256), 0, s, pb);
  return hipGetLastError();
}
hipError_t fade_convt_build(const float *Wconv, int taps, int D, int Kc, float *V, hipStream_t s) {
  hipLaunchKernelGGL(convt_build_kernel, dim3(blocks_for((size_t)Kc * D, 256)), dim3(256), 0, s, Wconv, taps, D, Kc, V);
  return hipGetLastError();
}
hipError_t fade_softmax_quant_code(const SqcArgs &a, int mode, hipStream_t s) {
  const dim3 grid((a.B + 3) / 4), block(256);
  if (mode == CODE_ENCODE) hipLaunchKernelGGL(softmax_quant_code_kernel<CODE_ENCODE>, grid, block, 0, s, a);
  else if (mode == CODE_DECODE) hipLaunchKernelGGL(softmax_quant_code_kernel<CODE_DECODE>, grid, block, 0, s, a);
  else if (mode == CODE_RANGES) {
    if (!a.ranges || a.streams <= 0 || a.B % a.streams) return hipErrorInvalidValue;
    hipLaunchKernelGGL(softmax_quant_code_kernel<CODE_RANGES>, grid, block, 0, s, a);
  }
  else hipLaunchKernelGGL(softmax_quant_code_kernel<CODE_NONE>, grid, block, 0, s, a);
  return hipGetLastError();
}
hipError_t fade_quantize_rows(const float *probs, size_t rows, uint16_t *freq, int *err, hipStream_t s) {
  hipLaunchKernelGGL(quantize_kernel, dim3(blocks_for(rows, 4)), dim3(256), 0, s, probs, rows, freq, err);
  return hipGetLastError();
}
hipError_t fade_code_tables(const uint16_t *freq, uint8_t *sym, int n_streams, const CoderBufs &cb, int mode, hipStream_t s) {
  const dim3 grid((n_streams + 3) / 4), block(256);
  if (mode == CODE_ENCODE) hipLaunchKernelGGL(code_tables_kernel<CODE_ENCODE>, grid, block, 0, s, freq, sym, n_streams, cb);
  else hipLaunchKernelGGL(code_tables_kernel<CODE_DECODE>, grid, block, 0, s, freq, sym, n_streams, cb);
  return hipGetLastError();
}
hipError_t fade_code_uniform(const WinSrc &ws, uint8_t *sym_base, int B, const CoderBufs &cb, int mode, hipStream_t s) {
  const dim3 grid((B + 63) / 64), block(64);
  if (mode == CODE_ENCODE) hipLaunchKernelGGL(code_uniform_kernel<CODE_ENCODE>, grid, block, 0, s, ws, sym_base, B, cb);
  else hipLaunchKernelGGL(code_uniform_kernel<CODE_DECODE>, grid, block, 0, s, ws, sym_base, B, cb);
  return hipGetLastError();
}
hipError_t fade_coder_init(const CoderBufs &cb, int B, int decode, hipStream_t s) {
  hipLaunchKernelGGL(coder_init_kernel, dim3((B + 63) / 64), dim3(64), 0, s, cb, B, decode);
  return hipGetLastError();
}
hipError_t fade_coder_finish(const CoderBufs &cb, int B, long long stride, long long n, hipStream_t s) {
  hipLaunchKernelGGL(coder_finish_kernel, dim3((B + 63) / 64), dim3(64), 0, s, cb, B, stride, n);
  return hipGetLastError();
}
hipError_t fade_payload_move(uint8_t *strided, size_t cap, uint8_t *flat, const unsigned long long *offsets, const uint32_t *lens, int B,
                             int gather, hipStream_t s) {
  hipLaunchKernelGGL(payload_move_kernel, dim3(B), dim3(256), 0, s, strided, cap, flat, offsets, lens, gather);
  return hipGetLastError();
}
