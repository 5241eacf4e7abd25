// fade_api.hip — libfade's C ABI: context, device state, the step sequence and the compress / decompress loops.
#include <algorithm>
#include <initializer_list>
#include <utility>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/fade.h"
#include "fade_kernels.h"

namespace {

struct Dims {
  size_t B, T, D, H, Dh, Dc, De, dl, c, k, Kc;  // Kc: K of the conv product (k * D rounded up to 64)
};

// canonical blob order (see fade.h)
enum ParamId {
  P_E, P_GAMMA_E, P_BETA_E, P_GAMMA_L, P_BETA_L, P_WG, P_WV, P_WM, P_LAMBDA_M, P_WCONV, P_BCONV, P_WR, P_GAMMA_C,
  P_BETA_C, P_WDOWN, P_WU, P_WUP, P_WC, P_LAMBDA_C, P_GAMMA_F, P_BETA_F, P_WFG, P_WFV, P_WF, P_GAMMA_O, P_BETA_O,
  P_LAMBDA_O, P_WO, P_BO, P_COUNT
};

struct Layout {
  size_t off[P_COUNT + 1];
  size_t len[P_COUNT];
};

// canonical: the blob of the C ABI, tensors back to back. Device arrays (master, gradient, Adam moments) start every tensor on
// a 16-byte boundary instead (only the three scalar residual scales get padding), so that kernels can use 16-byte accesses,
// and the big matrices on a 128-byte boundary: the Adam pass walks them in 64 x 64 blocks whose 256-byte row pieces then
// cover two whole cache lines instead of parts of three. Padding comes in front of a matrix only, so the neighbours that
// some kernels write as one run (a LayerNorm's gain and shift, W_g and W_v, W_conv and b_conv) stay adjacent.
Layout make_layout(const Dims &d, bool canonical) {
  const size_t n[P_COUNT] = {
      256 * d.D, d.D, d.D, d.D, d.D, d.D * d.c, d.D * d.c, d.Dc * d.Dh, 1, d.k * d.D * d.D, d.D, d.Dh * d.Dh, d.Dh, d.Dh,
      d.Dh * d.dl, d.B * d.dl * d.dl, d.dl * d.Dh, d.Dh * d.Dh, 1, d.Dh, d.Dh, d.Dh * d.De, d.Dh * d.De, d.De * d.Dh,
      d.Dh, d.Dh, 1, d.Dh * 256, 256};
  Layout L;
  size_t o = 0;
  for (int i = 0; i < P_COUNT; ++i) {
    const bool big = i == P_WM || i == P_WR || i == P_WDOWN || i == P_WU || i == P_WUP || i == P_WC || i == P_WFG || i == P_WFV || i == P_WF || i == P_WO;
    if (!canonical && big) o = (o + 31) / 32 * 32;
    L.off[i] = o; o += canonical ? n[i] : (n[i] + 3) / 4 * 4; L.len[i] = n[i];
  }
  L.off[P_COUNT] = o;
  return L;
}

int resolve_dims(const fade_config &cfg, Dims &d, std::string *why) {
  auto bad = [&](const char *m) { if (why) *why = m; return FADE_E_BAD_CONFIG; };
  d.B = cfg.B; d.T = cfg.T; d.D = cfg.D; d.H = cfg.H;
  d.Dh = d.T * d.D; d.Dc = cfg.d_cache ? cfg.d_cache : d.H; d.De = cfg.d_e ? cfg.d_e : d.H;
  d.dl = cfg.d_low ? cfg.d_low : 64;
  d.k = cfg.conv_k ? cfg.conv_k : 3;
  if (!d.B || !d.T || !d.D || !d.H) return bad("B, T, D, H must be positive");
  if (cfg.cache_chunk) d.c = cfg.cache_chunk;
  else { if (d.Dc % d.T) return bad("D_cache is not a multiple of T and cache_chunk is 0"); d.c = d.Dc / d.T; }
  if (!d.c || d.Dc % d.c) return bad("D_cache is not a multiple of cache_chunk");
  if (cfg.dtype > FADE_BF16 || cfg.update_mode > FADE_ONLINE_ADAM) return bad("unknown dtype or update_mode");
  if (cfg.ablation > 5) return bad("ablation level must be 0..5");
  d.Kc = (d.k * d.D + 63) / 64 * 64;
  return FADE_OK;
}

// what the kernels support on top of what the model needs
int check_kernel_limits(const fade_config &cfg, const Dims &d, std::string *why) {
  auto bad = [&](const char *m) { if (why) *why = m; return FADE_E_BAD_CONFIG; };
  if (d.dl != 64) return bad("kernels need d_low == 64");
  if (d.Dh % 128) return bad("kernels need T*D to be a multiple of 128");
  if (d.Dc % 64 || d.Dc > 4096) return bad("kernels need D_cache to be a multiple of 64, at most 4096");
  if (d.De % 64 || d.De > 8192) return bad("kernels need D_e to be a multiple of 64, at most 8192");
  if (d.c > 256) return bad("kernels need cache_chunk <= 256");
  if (d.k > 4) return bad("kernels need conv_k <= 4");
  if (cfg.dtype == FADE_BF16 ? (d.D % 32 != 0) : (d.D % 16 != 0)) return bad("kernels need D % 32 == 0 (bf16) or D % 16 == 0 (fp32)");
  if (d.B * d.T > 0x7fffffffull / 4 || d.B > (1u << 20)) return bad("B too large");
  if (cfg.update_mode == FADE_ONLINE_ADAM && (d.Dh > 2048 || d.D > 32 || 128 % d.T || 256 % d.D))
    return bad("the update kernels need T*D <= 2048, D in {16, 32} and T a power of two up to 128");
  return FADE_OK;
}

uint64_t fnv1a64(const void *p, size_t n) {
  const unsigned char *b = static_cast<const unsigned char *>(p);
  uint64_t h = 14695981039346656037ull;
  for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
  return h;
}

constexpr size_t kHeaderBytes = 64;
void wr16(uint8_t *p, uint32_t v) { p[0] = v & 0xff; p[1] = (v >> 8) & 0xff; }
void wr32(uint8_t *p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (v >> (8 * i)) & 0xff; }
void wr64(uint8_t *p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (v >> (8 * i)) & 0xff; }
uint32_t rd16(const uint8_t *p) { return p[0] | (uint32_t)p[1] << 8; }
uint32_t rd32(const uint8_t *p) { uint32_t v = 0; for (int i = 3; i >= 0; --i) v = (v << 8) | p[i]; return v; }
uint64_t rd64(const uint8_t *p) { uint64_t v = 0; for (int i = 7; i >= 0; --i) v = (v << 8) | p[i]; return v; }
uint32_t fbits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }

}  // namespace

// Coder state of fade_coder_encode_tables_noalloc: device memory that lives in the library's image instead of coming from
// hipMalloc (eight uint32 per stream: low, high, pending, bit buffer, bit count, position, value, bit position). Every GPU
// the library runs on holds its own copy until the process ends. The name below is a host-side stand-in, not a device
// address: host code only ever uses the pointer hipGetSymbolAddress returns for the current device (scratch_for_device).
static __device__ __align__(256) uint32_t scratch[8 * FADE_NOALLOC_MAX_STREAMS];

namespace {
constexpr int kMaxDevices = 64;
uint32_t *g_scratch_ptr[kMaxDevices] = {};
// Address of `scratch` on `device`, looked up once per device with that device current.
hipError_t scratch_for_device(int device, uint32_t **out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device && (e = hipSetDevice(device)) != hipSuccess) return e;
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (cur != device) (void)hipSetDevice(cur);
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = static_cast<uint32_t *>(p);
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}
}  // namespace

struct fade_ctx {
  fade_config cfg;
  Dims d;
  Layout lay;
  bool bf16 = false, online = false;
  size_t esz = 4;  // bytes per activation element
  hipStream_t stream = nullptr;
  bool own_stream = false;
  std::string err;
  std::vector<void *> allocs;
  // staging of the host-buffer entry points (job bytes, flat payloads, payload offsets): grown on demand, kept until
  // fade_destroy, so a context that codes job after job allocates once
  void *stage[3] = {nullptr, nullptr, nullptr};
  size_t stage_cap[3] = {0, 0, 0};

  bool have_weights = false;
  std::vector<float> loaded;
  uint64_t weights_hash = 0;

  // parameters
  float *master = nullptr;                                   // fp32 blob on the device
  float *E_c = nullptr, *Wg_c = nullptr, *Wv_c = nullptr;     // fp32-resident operands (bf16-rounded in the bf16 configuration)
  void *tabXe = nullptr, *tabXl = nullptr;
  float *tabXe32 = nullptr;
  void *Wm_c = nullptr, *Wconv_c = nullptr, *Wr_c = nullptr, *Wdown_c = nullptr, *WU_c = nullptr, *Wup_c = nullptr,
       *Wc_c = nullptr, *Wfgv_c = nullptr, *Wf_c = nullptr, *Wo_c = nullptr;

  // activations of the current step
  void *X = nullptr, *XL = nullptr, *M = nullptr, *Hg = nullptr, *Hl = nullptr, *Hmix = nullptr, *Ha = nullptr,
       *Hc = nullptr, *V = nullptr, *Hexp = nullptr, *z = nullptr;
  float *y = nullptr, *logits = nullptr, *stats_c = nullptr, *stats_f = nullptr, *stats_o = nullptr;
  // bf16 path: split-K partials, folded-LayerNorm vectors, the materialised H of Eq. 10
  float *part_down = nullptr, *part_fnr = nullptr, *part_head = nullptr;
  float *s_down = nullptr, *t_down = nullptr, *s_fnr = nullptr, *t_fnr = nullptr;
  float *fold_down = nullptr, *fold_fnr = nullptr;  // per 64-row block partials of those vectors, written by the Adam + refresh kernel
  void *Hout = nullptr;
  int sp_down = 1, sp_fnr = 1, sp_head = 1;
  // frozen bf16 encode: up to `steps_max` consecutive steps share one pass (rows = B * steps); buffers hold B * steps_max rows
  int steps_max = 1;
  void *slot_tab = nullptr;   // [256][c] Eq. 1 per symbol
  float *gg_tab = nullptr, *gv_tab = nullptr;  // [256][c] its two pre-activations per symbol (adapting weights)
  uint2 *ranges = nullptr;    // [B * steps_max] coding intervals of one pass
  // kept for the backward pass (online mode only)
  void *hm = nullptr, *alpha = nullptr, *sg = nullptr, *eg = nullptr, *ev = nullptr, *cv = nullptr;
  float *GG = nullptr, *GV = nullptr;
  float *probs_buf = nullptr;
  // online update: gradients, optimiser state, backward temporaries (see backward())
  size_t Bp = 0;  // batch rounded up to 64: leading dimension of the feature-major copies and row count of GEMM_W operands
  float *grad = nullptr, *adam_m = nullptr, *adam_v = nullptr;
  UpdateState *ustate = nullptr;
  uint8_t *win_copy = nullptr;  // online mode: the windows of the last fade_step_probs, for fade_step_update
  float *tabXhat = nullptr, *tabRstd = nullptr, *convt_f32 = nullptr;
  void *WT_o = nullptr, *WT_f = nullptr, *WT_fgv = nullptr, *WT_c = nullptr, *WT_up = nullptr, *WT_down = nullptr, *WT_r = nullptr,
       *WT_conv = nullptr;
  void *WT_mslot = nullptr, *dg_slot = nullptr;  // wide cache slots (c % 64 == 0): W_m's last slot transposed (fragments [Dh][c]), dg [B][c]
  void *dl = nullptr, *dHout = nullptr, *dV = nullptr, *dHc = nullptr, *dHexp = nullptr, *dE = nullptr, *du = nullptr,
       *dHa = nullptr, *dac = nullptr, *dHmix1 = nullptr, *dHmix2 = nullptr, *dy_at = nullptr, *dnc = nullptr, *dar = nullptr,
       *dhm = nullptr, *dcv = nullptr, *dX1 = nullptr, *dX2 = nullptr, *dxl = nullptr;
  void *LT[8] = {};  // left operands of the weight gradients that need a copy: LN(H_coarse), LN(H_mix) row-major (bf16 path); feature-major copies [width][Bp] of all eight (fp32 path)
  float *dz_part = nullptr, *dy = nullptr, *dgg = nullptr, *dgv = nullptr, *dxt = nullptr, *row_dlam = nullptr,
        *conv_part = nullptr, *tok_part = nullptr;
  float *ln_part = nullptr, *col_part = nullptr, *slot_part = nullptr, *emb_part = nullptr;
  int sp_dz = 1, emb_blocks = 128;
  // weight gradients with few output tiles are left as partial sums over ranges of the batch (bf16 path): per parameter
  // tensor the number of ranges (1: none) and the slices [ranges][K][N]; the Adam pass adds them up
  int gsp[P_COUNT] = {};
  // weight gradients on 256 x 256 tiles wait here until the end of the backward pass and run as one launch (defer_tn2)
  Tn2Group tn2q{};
  bool defer_tn2 = false;
  float *gpart[P_COUNT] = {};
  int sp_du = 1;            // ranges of K = 2 D_e in du = dE [W_fg W_fv]^T (bf16 path, wide refiners)
  float *du_part = nullptr;

  // coder and step bookkeeping
  CoderBufs cb{};
  uint8_t *payload = nullptr;
  uint32_t *in_len = nullptr;
  size_t payload_cap = 0;
  uint8_t *ones = nullptr;
  WinSrc last_ws{};
  int *dev_err = nullptr;
  bool rows16 = false;               // fp32 path at very small batches: 16 x 16 product tiles, row statistics per 16 columns
  size_t stats_n = 0;                // partial (sum, sum of squares) pairs per row the statistics buffers hold
  bool debug_wu_grad = false;        // FADE_DEBUG_WU_GRAD=1 at fade_create: gradients consumed where they are formed (W_U's, the sums of sliced weight gradients) are also written to the gradient array
  uint32_t *scratch_dev = nullptr;   // this device's copy of the file-scope scratch array (see scratch_for_device)
  size_t loop_n = 0, loop_next = 0;  // job size and next step of the device-resident loop in progress
  int loop_mode = 0;
  bool enc_complete = false;

  // profiling
  bool profiling = false;
  struct Ev { hipEvent_t a, b; int name; };
  std::vector<Ev> events;
  std::vector<std::string> prof_names;
  std::vector<double> prof_ms;
  std::vector<uint64_t> prof_n;

  Layout blob;  // canonical layout of the C ABI's blob (lay: the device arrays)
  const float *P(int id) const { return master + lay.off[id]; }
};

namespace {

int fail(fade_ctx *c, int code, const std::string &msg) {
  if (c) c->err = msg;
  return code;
}
int hip_fail(fade_ctx *c, hipError_t e, const char *what) {
  return fail(c, e == hipErrorOutOfMemory ? FADE_E_OOM : FADE_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(ctx, call)                                \
  do {                                                    \
    hipError_t e_ = (call);                               \
    if (e_ != hipSuccess) return hip_fail(ctx, e_, #call); \
  } while (0)

template <typename T> int dev_alloc(fade_ctx *c, T **p, size_t count) {
  void *q = nullptr;
  hipError_t e = hipMalloc(&q, (count ? count : 1) * sizeof(T));
  if (e != hipSuccess) return hip_fail(c, e, "hipMalloc");
  c->allocs.push_back(q);
  *p = static_cast<T *>(q);
  // Every buffer starts at zero. Rows of streams that are never active (a ragged last stream, an explicit mask) are never
  // written by the window gather, yet the dense products and the backward pass run over all B rows: their contribution is
  // (zero gradient) x (activation), which must not be 0 x NaN from recycled memory.
  e = hipMemsetAsync(q, 0, (count ? count : 1) * sizeof(T), c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "hipMemsetAsync");
  return FADE_OK;
}
int dev_alloc_bytes(fade_ctx *c, void **p, size_t bytes) {
  uint8_t *q = nullptr;
  int rc = dev_alloc(c, &q, bytes);
  *p = q;
  return rc;
}

// Staging buffer `slot` of at least `bytes` bytes (STAGE_*). A buffer that is too small is replaced (the stream is idle
// between calls of the host-buffer entry points, which are the only users); contents are not kept.
enum { STAGE_JOB = 0, STAGE_FLAT = 1, STAGE_OFF = 2 };
int stage_buf(fade_ctx *c, int slot, size_t bytes, void **p) {
  if (bytes == 0) bytes = 1;
  if (c->stage_cap[slot] < bytes) {
    if (c->stage[slot]) {
      hipError_t e = hipStreamSynchronize(c->stream);
      if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
      (void)hipFree(c->stage[slot]);
      c->stage[slot] = nullptr; c->stage_cap[slot] = 0;
    }
    hipError_t e = hipMalloc(&c->stage[slot], bytes);
    if (e != hipSuccess) { c->stage[slot] = nullptr; return hip_fail(c, e, "hipMalloc(staging)"); }
    c->stage_cap[slot] = bytes;
  }
  *p = c->stage[slot];
  return FADE_OK;
}

// profiling: bracket a launch with two events on the context's stream
struct Prof {
  fade_ctx *c; int idx = -1; hipStream_t st;
  Prof(fade_ctx *ctx, const char *name, hipStream_t on = nullptr) : c(ctx), st(on ? on : ctx->stream) {
    if (!c->profiling) return;
    int id = -1;
    for (size_t i = 0; i < c->prof_names.size(); ++i) if (c->prof_names[i] == name) id = (int)i;
    if (id < 0) { id = (int)c->prof_names.size(); c->prof_names.push_back(name); c->prof_ms.push_back(0); c->prof_n.push_back(0); }
    fade_ctx::Ev ev; ev.name = id;
    if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) return;
    (void)hipEventRecord(ev.a, st);
    c->events.push_back(ev);
    idx = (int)c->events.size() - 1;
  }
  ~Prof() { if (idx >= 0) (void)hipEventRecord(c->events[idx].b, st); }
};

void prof_collect(fade_ctx *c) {
  for (auto &ev : c->events) {
    float ms = 0;
    if (hipEventElapsedTime(&ms, ev.a, ev.b) == hipSuccess) { c->prof_ms[ev.name] += ms; c->prof_n[ev.name] += 1; }
    (void)hipEventDestroy(ev.a); (void)hipEventDestroy(ev.b);
  }
  c->events.clear();
}

// ---------------------------------------------------------------------------------------------------
// master weights -> compute copies (runs on the stream; repeated after every online update)
// ---------------------------------------------------------------------------------------------------
// The nine big matrices: (online: one Adam step, then) both bf16 fragment copies and the partial sums of the folded-LayerNorm
// vectors, one pass over 64 x 64 blocks. fp32 path: the Adam step only (operands are the master weights themselves).
int refresh_matrices(fade_ctx *c, bool adam) {
  const Dims &d = c->d;
  const bool bf = c->bf16;
  AdamRefreshBatch ab{};
  ab.refresh_only = adam ? 0 : 1;
  ab.keep_sum = c->debug_wu_grad ? 1 : 0;
  ab.opt = AdamArrays{c->grad, c->master, c->adam_m, c->adam_v, c->ustate, c->cfg.lr, c->cfg.beta1, c->cfg.beta2, c->cfg.eps};
  auto add = [&](int id, size_t K, size_t N, int vcol0, int vstride, size_t VN, void *frag, void *fragT, const float *ga, const float *be, float *fp) {
    AdamMat &m = ab.m[ab.count++];
    m.off = c->lay.off[id]; m.K = (int)K; m.N = (int)N; m.vcol0 = vcol0; m.vstride = vstride; m.VN = (int)VN;
    m.frag = bf ? frag : nullptr; m.fragT = (bf && c->online) ? fragT : nullptr; m.gamma = bf ? ga : nullptr; m.beta = bf ? be : nullptr; m.fold_part = fp;
    m.first_block = ab.total_blocks;
    m.gpart = (adam && c->gsp[id] > 1) ? c->gpart[id] : nullptr; m.gsplits = c->gsp[id];
    ab.total_blocks += (int)((K / 64) * (N / 64));
  };
  // matrices whose gradient may arrive as partial sums go first: their blocks have the longer chain of loads
  add(P_WDOWN, d.Dh, d.dl, 0, 64, d.dl, c->Wdown_c, c->WT_down, c->P(P_GAMMA_C), c->P(P_BETA_C), c->fold_down);
  add(P_WO, d.Dh, 256, 0, 64, 256, c->Wo_c, c->WT_o, nullptr, nullptr, nullptr);
  add(P_WF, d.De, d.Dh, 0, 64, d.Dh, c->Wf_c, c->WT_f, nullptr, nullptr, nullptr);
  add(P_WFG, d.Dh, d.De, 0, 128, 2 * d.De, c->Wfgv_c, c->WT_fgv, c->P(P_GAMMA_F), c->P(P_BETA_F), c->fold_fnr);
  add(P_WFV, d.Dh, d.De, 64, 128, 2 * d.De, c->Wfgv_c, c->WT_fgv, c->P(P_GAMMA_F), c->P(P_BETA_F), c->fold_fnr);
  add(P_WR, d.Dh, d.Dh, 0, 64, d.Dh, c->Wr_c, c->WT_r, nullptr, nullptr, nullptr);
  add(P_WC, d.Dh, d.Dh, 0, 64, d.Dh, c->Wc_c, c->WT_c, nullptr, nullptr, nullptr);
  add(P_WM, d.Dc, d.Dh, 0, 64, d.Dh, c->Wm_c, nullptr, nullptr, nullptr, nullptr);
  add(P_WUP, d.dl, d.Dh, 0, 64, d.Dh, c->Wup_c, c->WT_up, nullptr, nullptr, nullptr);
  HIP_TRY(c, fade_adam_refresh(ab, c->stream));
  return FADE_OK;
}
// bf16 path, after the matrices: the small operands (embedding, slot pair, conv taps in both orientations), the folded-LayerNorm
// vectors from their per-block partials, the per-symbol tables
// `pending`: second-stage reductions of the update still to be launched; the two folded-LayerNorm sums join that launch.
int refresh_small(fade_ctx *c, ReduceBatch *pending = nullptr) {
  const Dims &d = c->d;
  hipStream_t s = c->stream;
  ReduceBatch local{};
  ReduceBatch &fr = pending ? *pending : local;  // s then t, adjacent
  if (!fr.push_plain((int)(d.Dh / 64), (int)(2 * d.dl), c->fold_down, c->s_down) ||
      !fr.push_plain((int)(d.Dh / 64), (int)(4 * d.De), c->fold_fnr, c->s_fnr))
    return fail(c, FADE_E_INVALID_ARG, "reduction queue full");
  HIP_TRY(c, fade_reduce_batch(fr, s));
  PrepBatch pb{};
  auto padd = [&](int kind, const float *W0, size_t k_real, size_t K, size_t N, void *out) {
    PrepDesc &q = pb.d[pb.count++];
    q.kind = kind; q.W0 = W0; q.W1 = nullptr; q.k_real = (int)k_real; q.K = (int)K; q.N = (int)N; q.interleave = 0; q.rowscale = nullptr;
    q.out = out; q.taps = (int)d.k; q.D = (int)d.D;
  };
  padd(PREP_ROUND, c->P(P_E), 0, 0, 256 * d.D, c->E_c);
  padd(PREP_ROUND, c->P(P_WG), 0, 0, d.D * d.c, c->Wg_c);
  padd(PREP_ROUND, c->P(P_WV), 0, 0, d.D * d.c, c->Wv_c);
  padd(PREP_FRAG, c->P(P_WCONV), d.k * d.D, d.Kc, d.D, c->Wconv_c);
  if (c->online) padd(PREP_FRAG_CONVT, c->P(P_WCONV), d.k * d.D, d.Kc, d.D, c->WT_conv);
  if (c->WT_mslot) padd(PREP_FRAG_T, c->P(P_WM) + (d.Dc - d.c) * d.Dh, d.c, d.c, d.Dh, c->WT_mslot);
  pb.has_tables = 1;  // same launch: the tables read the master embedding and round it as the copy above does
  pb.tab = TablesArgs{c->P(P_E), c->P(P_GAMMA_E), c->P(P_BETA_E), c->P(P_GAMMA_L), c->P(P_BETA_L), (int)d.D, 1, c->tabXe, c->tabXl, c->tabXe32,
                      c->tabXhat, c->tabRstd, nullptr, nullptr, (int)d.c, c->slot_tab, c->gg_tab, c->gv_tab};
  if (c->slot_tab || c->gg_tab) { pb.tab.Wg = c->P(P_WG); pb.tab.Wv = c->P(P_WV); }  // Eq. 1 per symbol rides along
  HIP_TRY(c, fade_prep_batch(pb, s));
  return FADE_OK;
}

int prepare_compute(fade_ctx *c, bool with_wu = true) {
  const Dims &d = c->d;
  hipStream_t s = c->stream;
  if (c->bf16) {
    int rc = refresh_matrices(c, false);
    if (rc) return rc;
    if (with_wu) HIP_TRY(c, fade_convert(c->P(P_WU), c->WU_c, d.B * d.dl * d.dl, true, s));
    return refresh_small(c);
  } else {
    HIP_TRY(c, fade_virtual_copy(c->P(P_WCONV), nullptr, (int)(d.k * d.D), (int)d.Kc, (int)d.D, 0, static_cast<float *>(c->Wconv_c), s));
    HIP_TRY(c, fade_virtual_copy(c->P(P_WFG), c->P(P_WFV), (int)d.Dh, (int)d.Dh, (int)(2 * d.De), 1, static_cast<float *>(c->Wfgv_c), s));
    if (c->online) HIP_TRY(c, fade_convt_build(c->P(P_WCONV), (int)d.k, (int)d.D, (int)d.Kc, c->convt_f32, s));
  }
  HIP_TRY(c, fade_tables(c->E_c, c->P(P_GAMMA_E), c->P(P_BETA_E), c->P(P_GAMMA_L), c->P(P_BETA_L), (int)d.D, c->tabXe,
                         c->tabXl, c->tabXe32, c->tabXhat, c->tabRstd, c->bf16, s));
  return FADE_OK;
}

int do_reset(fade_ctx *c) {
  const Dims &d = c->d;
  hipStream_t s = c->stream;
  HIP_TRY(c, hipMemsetAsync(c->M, 0, d.B * d.Dc * c->esz, s));
  HIP_TRY(c, hipMemsetAsync(c->dev_err, 0, sizeof(int), s));
  if (c->have_weights) {
    HIP_TRY(c, hipMemcpyAsync(c->master, c->loaded.data(), c->loaded.size() * sizeof(float), hipMemcpyHostToDevice, s));
    int rc = prepare_compute(c);
    if (rc) return rc;
  }
  if (c->online) {
    const size_t np = c->lay.off[P_COUNT];
    HIP_TRY(c, hipMemsetAsync(c->adam_m, 0, np * sizeof(float), s));
    HIP_TRY(c, hipMemsetAsync(c->adam_v, 0, np * sizeof(float), s));
    HIP_TRY(c, hipMemsetAsync(c->ustate, 0, sizeof(UpdateState), s));
  }
  c->enc_complete = false;
  HIP_TRY(c, hipStreamSynchronize(s));
  return FADE_OK;
}

// ---------------------------------------------------------------------------------------------------
// one model step: windows -> logits -> (probabilities, table, coded symbol)
// ---------------------------------------------------------------------------------------------------
int forward_f32(fade_ctx *c, const WinSrc &ws, int mode, uint8_t *sym_base, uint16_t *freq, float *probs) {
  const Dims &d = c->d;
  hipStream_t s = c->stream;
  const bool bf = false;
  const int B = (int)d.B, Dh = (int)d.Dh, SN = (int)c->stats_n;
  const int r16 = c->rows16 ? 1 : 0;
  // progressive ablation (the paper's component table): the head reads the last stage that is switched on
  const int level = c->cfg.ablation == 0 ? 5 : (int)c->cfg.ablation;
  const void *feat = c->Hg;
  {
    Prof p(c, "embed_cache");
    EmbedArgs a{};
    a.ws = ws; a.T = (int)d.T; a.D = (int)d.D; a.Dh = Dh; a.Dc = (int)d.Dc; a.c = (int)d.c;
    a.tabXe = c->tabXe; a.tabXl = c->tabXl; a.tabXe32 = c->tabXe32; a.Wg = c->Wg_c; a.Wv = c->Wv_c;
    a.X = c->X; a.XL = c->XL; a.M = c->M; a.GG = c->GG; a.GV = c->GV;
    HIP_TRY(c, fade_embed_cache(a, B, bf, s));
  }
  if (level >= 2) {  // Eq. 4
    Prof p(c, "gemm_conv");
    GemmArgs g{};
    g.M = (int)(d.B * d.T); g.N = (int)d.D; g.K = (int)d.Kc;
    g.A = c->XL; g.T = (int)d.T; g.D = (int)d.D; g.taps = (int)d.k;
    g.W = c->Wconv_c; g.C = c->Hl; g.ldc = (int)d.D; g.C2 = c->online ? c->cv : nullptr; g.bias = c->P(P_BCONV);
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_CONV, bf, g, s));
  }
  {  // Eq. 3
    Prof p(c, "gemm_global");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = (int)d.Dc;
    g.A = c->M; g.lda = (int)d.Dc; g.W = c->Wm_c; g.C = c->Hg; g.ldc = Dh; g.C2 = c->online ? c->hm : nullptr; g.S1 = c->X; g.lam = c->P(P_LAMBDA_M);
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_GLOBAL, bf, g, s));
  }
  if (level >= 2) {  // Eq. 5-6
    feat = c->Hmix;
    Prof p(c, "gemm_router");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = Dh;
    g.A = c->X; g.lda = Dh; g.W = c->Wr_c; g.C = c->Hmix; g.ldc = Dh; g.C2 = c->online ? c->alpha : nullptr; g.S1 = c->Hg; g.S2 = c->Hl;
    g.stats_out = c->stats_c;
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_ROUTER, bf, g, s));
  }
  if (level >= 3) {  // Eq. 7: Down(LN(H_mix))
    Prof p(c, "gemm_down");
    GemmArgs g{};
    g.M = B; g.N = (int)d.dl; g.K = Dh;
    g.A = c->Hmix; g.lda = Dh; g.stats = c->stats_c; g.stats_n = SN; g.gamma = c->P(P_GAMMA_C); g.beta = c->P(P_BETA_C);
    g.W = c->Wdown_c; g.C = c->y; g.ldc = (int)d.dl;
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_DOWN, bf, g, s));
  }
  if (level >= 3) {  // Eq. 7: the per-stream memory
    Prof p(c, "bmm_wu");
    HIP_TRY(c, fade_bmm(c->y, c->WU_c, c->z, B, bf, s));
  }
  if (level >= 3) {  // Eq. 7: Up
    feat = c->Hc;
    Prof p(c, "gemm_up");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = (int)d.dl;
    g.A = c->z; g.lda = (int)d.dl; g.W = c->Wup_c; g.C = c->Ha; g.ldc = Dh;
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_UP, bf, g, s));
  }
  if (level == 3) {  // Eq. 8 without its gate
    Prof p(c, "residual_add");
    HIP_TRY(c, fade_residual_add(c->Ha, c->Hmix, c->P(P_LAMBDA_C), c->Hc, (size_t)B * Dh, false, s));
  }
  if (level >= 4) {  // Eq. 8
    Prof p(c, "gemm_gate");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = Dh;
    g.A = c->Hmix; g.lda = Dh; g.W = c->Wc_c; g.C = c->Hc; g.ldc = Dh; g.C2 = c->online ? c->sg : nullptr; g.S1 = c->Ha; g.S2 = c->Hmix;
    g.lam = c->P(P_LAMBDA_C); g.stats_out = c->stats_f;
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_GATE, bf, g, s));
  }
  if (level >= 5) {  // Eq. 9
    Prof p(c, "gemm_fnr_in");
    GemmArgs g{};
    g.M = B; g.N = (int)(2 * d.De); g.K = Dh;
    g.A = c->Hc; g.lda = Dh; g.stats = c->stats_f; g.stats_n = SN; g.gamma = c->P(P_GAMMA_F); g.beta = c->P(P_BETA_F);
    g.W = c->Wfgv_c; g.C = c->Hexp; g.ldc = (int)d.De; if (c->online) { g.C2 = c->eg; g.C3 = c->ev; }
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_FNR_IN, bf, g, s));
  }
  if (level >= 5) {  // Eq. 10: H_expand W_f (+ statistics for its LayerNorm)
    Prof p(c, "gemm_fnr_out");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = (int)d.De;
    g.A = c->Hexp; g.lda = (int)d.De; g.W = c->Wf_c; g.C = c->V; g.ldc = Dh; g.stats_out = c->stats_o;
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_FNR_OUT, bf, g, s));
  }
  if (c->online && level >= 5) {  // the update needs H itself (for dW_o); frozen mode forms it only inside the head's operand load
    Prof p(c, "hout");
    HoutArgs a{};
    a.B = B; a.Dh = Dh; a.stats_n = SN; a.V = c->V; a.Hc = c->Hc; a.stats = c->stats_o; a.gamma = c->P(P_GAMMA_O);
    a.beta = c->P(P_BETA_O); a.lam = c->P(P_LAMBDA_O); a.Hout = c->Hout;
    HIP_TRY(c, fade_hout(a, false, s));
  }
  if (level < 5) {  // the head on the last stage that is switched on: logits = feat W_o + b_o
    Prof p(c, "gemm_head");
    GemmArgs g{};
    g.M = B; g.N = 256; g.K = Dh;
    g.A = feat; g.lda = Dh; g.W = c->Wo_c; g.C = c->logits; g.ldc = 256; g.bias = c->P(P_BO);
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_HEAD_PLAIN, bf, g, s));
  } else {  // Eq. 10's tail fused into the head's operand load; logits = H W_o + b_o
    Prof p(c, "gemm_head");
    GemmArgs g{};
    g.M = B; g.N = 256; g.K = Dh;
    g.A = c->V; g.A2 = c->Hc; g.lda = Dh; g.stats = c->stats_o; g.stats_n = SN; g.gamma = c->P(P_GAMMA_O); g.beta = c->P(P_BETA_O);
    g.lam = c->P(P_LAMBDA_O); g.W = c->Wo_c; g.C = c->logits; g.ldc = 256; g.bias = c->P(P_BO);
    g.rows16 = r16;
    HIP_TRY(c, fade_gemm(GEMM_HEAD, bf, g, s));
  }
  {
    Prof p(c, "softmax_quant_code");
    SqcArgs a{};
    a.ws = ws; a.B = B; a.logits = c->logits; a.probs = probs; a.freq = freq; a.sym_base = sym_base; a.cb = c->cb;
    HIP_TRY(c, fade_softmax_quant_code(a, mode, s));
  }
  return FADE_OK;
}

// bf16 path: every product runs on raw bf16 activations through the pipelined MFMA kernel; LayerNorms are folded
// into the weights and finished where the split-K partials are reduced.
int pick_splits(int tiles, int k_blocks, int cap) {
  int s = 1;
  while (tiles * s < 192 && s * 2 <= cap && k_blocks % (s * 2) == 0 && k_blocks / (s * 2) >= 2) s *= 2;
  return s;
}

// steps > 1 (frozen weights, CODE_ENCODE only): rows s * B + b carry stream b at step ws.i + s through one pass; every row's
// arithmetic is the one a single step performs (same split-K counts, same summation order), so the tables, and with them
// the payload, are those of `steps` single steps.
int forward_bf16(fade_ctx *c, const WinSrc &ws, int mode, uint8_t *sym_base, uint16_t *freq, float *probs, int steps = 1) {
  const Dims &d = c->d;
  hipStream_t s = c->stream;
  const int streams = (int)d.B, B = streams * steps;  // B: rows of this pass
  const int Dh = (int)d.Dh, De = (int)d.De, SN = (int)c->stats_n;
  // a multi-step pass has tiles enough without splitting K: each workgroup adds the K ranges itself, in the order the
  // reducing kernels would, and those then see one partial
  const int fuse = steps > 1 ? 1 : 0;
  const int sp_down = fuse ? 1 : c->sp_down, sp_fnr = fuse ? 1 : c->sp_fnr, sp_head = fuse ? 1 : c->sp_head;
  if (steps > 1 && (steps > c->steps_max || mode != CODE_ENCODE || c->online)) return fail(c, FADE_E_INVALID_ARG, "multi-step pass not available");
  // progressive ablation (the paper's component table): the head reads the last stage that is switched on
  const int level = c->cfg.ablation == 0 ? 5 : (int)c->cfg.ablation;
  const void *feat = c->Hg;
  const bool conv_fused = level >= 2 && d.D == 32 && d.T <= 128 && d.k * 32 <= d.Kc && d.Kc <= 128;
  {
    Prof p(c, "embed_cache");
    EmbedArgs a{};
    a.ws = ws; a.T = (int)d.T; a.D = (int)d.D; a.Dh = Dh; a.Dc = (int)d.Dc; a.c = (int)d.c;
    a.tabXe = c->tabXe; a.tabXl = c->tabXl; a.tabXe32 = c->tabXe32; a.Wg = c->Wg_c; a.Wv = c->Wv_c;
    a.X = c->X; a.XL = c->XL; a.M = c->M; a.GG = c->GG; a.GV = c->GV; a.slot_tab = c->slot_tab; a.gg_tab = c->gg_tab; a.gv_tab = c->gv_tab; a.B = streams; a.S = steps;
    if (conv_fused) {  // Eq. 4 rides along: one launch less, and the per-token rows XL only exist for the backward pass
      a.conv_W = c->Wconv_c; a.conv_b = c->P(P_BCONV); a.Hl = c->Hl; a.cv = c->online ? c->cv : nullptr; a.taps = (int)d.k; a.Kc = (int)d.Kc;
      if (!c->online) a.XL = nullptr;
    }
    if (steps > 1) HIP_TRY(c, fade_embed_steps(a, s));
    else HIP_TRY(c, fade_embed_cache(a, streams, true, s));
  }
  if (level >= 2 && !conv_fused) {  // Eq. 4
    Prof p(c, "gemm_conv");
    GemmArgs g{};
    g.M = B * (int)d.T; g.N = (int)d.D; g.K = (int)d.Kc;
    g.A = c->XL; g.T = (int)d.T; g.D = (int)d.D; g.taps = (int)d.k;
    g.W = c->Wconv_c; g.C = c->Hl; g.ldc = (int)d.D; g.C2 = c->online ? c->cv : nullptr; g.bias = c->P(P_BCONV);
    HIP_TRY(c, fade_gemm(GEMM_CONV, true, g, s));
  }
  {  // Eq. 3
    Prof p(c, "gemm_global");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = (int)d.Dc;
    g.A = c->M; g.lda = (int)d.Dc; g.W = c->Wm_c; g.C = c->Hg; g.ldc = Dh; g.C2 = c->online ? c->hm : nullptr; g.S1 = c->X; g.lam = c->P(P_LAMBDA_M);
    HIP_TRY(c, fade_gemm(GEMM_GLOBAL, true, g, s));
  }
  if (level >= 2) {  // Eq. 5-6
    feat = c->Hmix;
    Prof p(c, "gemm_router");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = Dh;
    g.A = c->X; g.lda = Dh; g.W = c->Wr_c; g.C = c->Hmix; g.ldc = Dh; g.C2 = c->online ? c->alpha : nullptr; g.S1 = c->Hg; g.S2 = c->Hl;
    g.stats_out = c->stats_c;
    HIP_TRY(c, fade_gemm(GEMM_ROUTER, true, g, s));
  }
  if (level >= 3) {  // Eq. 7: H_mix W'_down as split-K partials
    Prof p(c, "gemm_down");
    GemmArgs g{};
    g.M = B; g.N = (int)d.dl; g.K = Dh; g.splits = c->sp_down; g.sum_splits = fuse;
    g.A = c->Hmix; g.lda = Dh; g.W = c->Wdown_c; g.C = c->part_down; g.ldc = (int)d.dl;
    HIP_TRY(c, fade_gemm(GEMM_PARTIAL, true, g, s));
  }
  if (level >= 3) {  // Eq. 7: folded LN, then the per-stream memory
    Prof p(c, "cci_wu");
    CciArgs a{};
    a.B = B; a.streams = streams; a.Dh = Dh; a.splits = sp_down; a.stats_n = SN; a.part = c->part_down; a.stats = c->stats_c;
    a.s_fold = c->s_down; a.t_fold = c->t_down; a.WU = static_cast<const bf16_t *>(c->WU_c); a.y = c->y; a.z = static_cast<bf16_t *>(c->z);
    HIP_TRY(c, fade_cci(a, s));
  }
  if (level >= 3) {  // Eq. 7: Up
    feat = c->Hc;
    Prof p(c, "gemm_up");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = (int)d.dl;
    g.A = c->z; g.lda = (int)d.dl; g.W = c->Wup_c; g.C = c->Ha; g.ldc = Dh;
    HIP_TRY(c, fade_gemm(GEMM_UP, true, g, s));
  }
  if (level == 3) {  // Eq. 8 without its gate
    Prof p(c, "residual_add");
    HIP_TRY(c, fade_residual_add(c->Ha, c->Hmix, c->P(P_LAMBDA_C), c->Hc, (size_t)B * Dh, true, s));
  }
  if (level >= 4) {  // Eq. 8
    Prof p(c, "gemm_gate");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = Dh;
    g.A = c->Hmix; g.lda = Dh; g.W = c->Wc_c; g.C = c->Hc; g.ldc = Dh; g.C2 = c->online ? c->sg : nullptr; g.S1 = c->Ha; g.S2 = c->Hmix;
    g.lam = c->P(P_LAMBDA_C); g.stats_out = c->stats_f;
    HIP_TRY(c, fade_gemm(GEMM_GATE, true, g, s));
  }
  if (level < 5) {
  } else if (c->sp_fnr == 1) {  // Eq. 9, enough tiles without splitting K: folded LN and GeGLU in the product's epilogue
    Prof p(c, "gemm_fnr_in");
    GemmArgs g{};
    g.M = B; g.N = 2 * De; g.K = Dh;
    g.A = c->Hc; g.lda = Dh; g.W = c->Wfgv_c; g.C = c->Hexp; g.ldc = De; if (c->online) { g.C2 = c->eg; g.C3 = c->ev; }
    g.stats = c->stats_f; g.stats_n = SN; g.fold_s = c->s_fnr; g.fold_t = c->t_fnr;
    HIP_TRY(c, fade_gemm(GEMM_FNR_IN, true, g, s));
  } else {
  {  // Eq. 9: H_coarse [W'_fg | W'_fv] as split-K partials
    Prof p(c, "gemm_fnr_in");
    GemmArgs g{};
    g.M = B; g.N = 2 * De; g.K = Dh; g.splits = c->sp_fnr; g.sum_splits = fuse;
    g.A = c->Hc; g.lda = Dh; g.W = c->Wfgv_c; g.C = c->part_fnr; g.ldc = 2 * De;
    HIP_TRY(c, fade_gemm(GEMM_PARTIAL, true, g, s));
  }
  {
    Prof p(c, "geglu");
    GegluArgs a{};
    a.B = B; a.Dh = Dh; a.De = De; a.splits = sp_fnr; a.stats_n = SN; a.part = c->part_fnr; a.stats = c->stats_f;
    a.s_fold = c->s_fnr; a.t_fold = c->t_fnr; a.Hexp = static_cast<bf16_t *>(c->Hexp);
    if (c->online) { a.eg = static_cast<bf16_t *>(c->eg); a.ev = static_cast<bf16_t *>(c->ev); }  // only the update reads them
    HIP_TRY(c, fade_geglu(a, s));
  }
  }
  if (level >= 5) {  // Eq. 10: H_expand W_f (+ statistics for its LayerNorm)
    Prof p(c, "gemm_fnr_out");
    GemmArgs g{};
    g.M = B; g.N = Dh; g.K = De;
    g.A = c->Hexp; g.lda = De; g.W = c->Wf_c; g.C = c->V; g.ldc = Dh; g.stats_out = c->stats_o;
    HIP_TRY(c, fade_gemm(GEMM_FNR_OUT, true, g, s));
  }
  // Frozen weights: nothing but the head reads H, so Eq. 10's tail is formed in the head product's operand load
  // (FADE_FUSE_HEAD=0 keeps the separate kernel; the update needs H itself for the head's weight gradient).
  static const bool fuse_head_env = !(getenv("FADE_FUSE_HEAD") && getenv("FADE_FUSE_HEAD")[0] == '0');
  // with adapting weights the product also writes H (the head's weight gradient reads it); needs whole 32-row tiles
  const bool fuse_head = level >= 5 && fuse_head_env && (!c->online || B % 32 == 0);
  if (level >= 5 && !fuse_head) {  // Eq. 10's tail
    feat = c->Hout;
    Prof p(c, "hout");
    HoutArgs a{};
    a.B = B; a.Dh = Dh; a.stats_n = SN; a.V = c->V; a.Hc = c->Hc;
    a.stats = c->stats_o; a.gamma = c->P(P_GAMMA_O); a.beta = c->P(P_BETA_O); a.lam = c->P(P_LAMBDA_O); a.Hout = c->Hout;
    HIP_TRY(c, fade_hout(a, true, s));
  }
  {  // head: H W_o as split-K partials; bias and reduction happen in the softmax kernel
    Prof p(c, "gemm_head");
    GemmArgs g{};
    g.M = B; g.N = 256; g.K = Dh; g.splits = c->sp_head; g.sum_splits = fuse;
    g.A = feat; g.lda = Dh; g.W = c->Wo_c; g.C = c->part_head; g.ldc = 256;
    if (fuse_head) {
      g.A = c->V; g.A2 = c->Hc; g.stats = c->stats_o; g.stats_n = SN; g.gamma = c->P(P_GAMMA_O); g.beta = c->P(P_BETA_O); g.lam = c->P(P_LAMBDA_O);
      if (c->online) g.C2 = c->Hout;
      HIP_TRY(c, fade_gemm(GEMM_HEAD, true, g, s));
    } else {
      HIP_TRY(c, fade_gemm(GEMM_PARTIAL, true, g, s));
    }
  }
  {
    Prof p(c, "softmax_quant_code");
    SqcArgs a{};
    a.ws = ws; a.B = B; a.splits = sp_head; a.bias = c->P(P_BO); a.logits_out = steps > 1 ? nullptr : c->logits; a.logits = c->part_head;
    a.probs = probs; a.freq = freq; a.sym_base = sym_base; a.cb = c->cb; a.streams = streams; a.ranges = c->ranges;
    HIP_TRY(c, fade_softmax_quant_code(a, steps > 1 ? CODE_RANGES : mode, s));
  }
  if (steps > 1) {
    Prof p(c, "encode_ranges");
    HIP_TRY(c, fade_encode_ranges(ws, c->ranges, streams, steps, c->cb, s));
  }
  return FADE_OK;
}

int forward(fade_ctx *c, const WinSrc &ws, int mode, uint8_t *sym_base, uint16_t *freq, float *probs) {
  float *p = c->online ? c->probs_buf : probs;  // the update needs the probabilities: keep them in the context
  int rc = c->bf16 ? forward_bf16(c, ws, mode, sym_base, freq, p) : forward_f32(c, ws, mode, sym_base, freq, p);
  if (rc) return rc;
  if (c->online && probs)
    HIP_TRY(c, hipMemcpyAsync(probs, c->probs_buf, c->d.B * 256 * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
  return FADE_OK;
}

// ---------------------------------------------------------------------------------------------------
// the online update: gradient of the mean NLL (Eq. 12) through the step, then Adam on every parameter
// ---------------------------------------------------------------------------------------------------
// dX = dY W^T. bf16: W^T lives as a second fragment set (wt_frag); fp32: W itself, read transposed.
GemmArgs args_x(fade_ctx *c, const void *dY, int Kred, int Nout, const void *wt_frag, const float *w_f32, int ld_w, void *out) {
  GemmArgs g{};
  g.M = (int)c->d.B; g.N = Nout; g.K = Kred; g.A = dY; g.lda = Kred; g.C = out; g.ldc = Nout;
  if (c->bf16) g.W = wt_frag;
  else { g.W = w_f32; g.wt = 1; g.ldb = ld_w; g.rows16 = c->rows16 && Kred % 16 == 0 && Kred <= 2048 && Nout % 16 == 0; }
  return g;
}
// dW[Kw][N] = L^T R over the batch. bf16 path: both operands row-major as the forward / backward kernels left them
// (L [B][ldL], R [Bp][N] with zero rows past the batch), turned on the way out of LDS. fp32 path: LT is a feature-major
// copy [Kw][Bp] of L, R is read row-major.
GemmArgs args_w(fade_ctx *c, const void *L, int ldL, const void *LT, int Kw, const void *R, int N, int id, int id_pair = -1) {
  GemmArgs g{};
  float *G = c->grad;
  g.M = Kw; g.N = N; g.K = (int)c->Bp; g.ldc = N; g.W = R;
  g.C = G + c->lay.off[id];
  if (id_pair >= 0) g.C3 = G + c->lay.off[id_pair];
  if (c->bf16) {
    g.A = L; g.lda = ldL; g.a_rows = (int)c->d.B; g.ldb = N;
    if (c->gsp[id] > 1) {  // partial sums over ranges of the batch; a pair splits alike
      g.splits = c->gsp[id]; g.C = c->gpart[id];
      if (id_pair >= 0) g.C3 = c->gpart[id_pair];
    }
  } else { g.A = LT; g.lda = (int)c->Bp; }
  return g;
}
// The products of one backward phase consume the same gradient and are independent: one grouped launch (bf16 path), or
// one launch each (fp32 path).
struct PhaseGemms {
  int n = 0;
  int op[4];
  GemmArgs g[4];
  void add(int o, const GemmArgs &a) { op[n] = o; g[n++] = a; }
  // A phase's pair dX = dY W^T, dW = L^T dY: the workgroups of the first product start first. Measured: with a long
  // contraction (K >= 1024) the activation gradient first is faster (B = 4096, D_h = 2048: gate phase 140 -> 116 us,
  // FNR-out 37 -> 33), with a short one the weight gradient first (D_h = 512, D_e = 8192: FNR-out 98 against 129).
  void add_pair(const GemmArgs &x, const GemmArgs &w) {
    if (x.K >= 1024) { add(GEMM_X_STORE, x); add(GEMM_W_TN, w); }
    else { add(GEMM_W_TN, w); add(GEMM_X_STORE, x); }
  }
};
int run_phase(fade_ctx *c, const char *name, const PhaseGemms &ph) {
  Prof p(c, name);
  if (c->bf16) {
    // An activation gradient that fills the chip with 256 x 256 tiles by itself (large batches) runs as a launch of its
    // own on the eight-wavefront kernel: half the operand bytes per flop of the 128 x 128 tiles a group is made of
    // (B = 16384: gate phase 357 -> 337 us, router phase 454 -> 434). With a short contraction (the head's K = 256) the
    // overlap with the weight gradient inside a group is worth more (87 us grouped against 105).
    GemmGroup gg{};
    for (int i = 0; i < ph.n; ++i) {
      const GemmArgs &g = ph.g[i];
      const bool alone = (ph.op[i] == GEMM_X_STORE && g.N % 256 == 0 && g.K >= 1024 && ((g.M + 255) / 256) * (g.N / 256) >= 256) ||
                         (ph.op[i] == GEMM_W_TN && fade_gemm_tn2_ok(g.M, g.N, g.K));
      if (alone && ph.op[i] == GEMM_W_TN && c->defer_tn2) HIP_TRY(c, fade_gemm_tn2_group_add(c->tn2q, g));  // launched at the end of the pass
      else if (alone) HIP_TRY(c, fade_gemm(ph.op[i], true, g, c->stream));
      else HIP_TRY(c, fade_gemm_group_add(gg, ph.op[i], g));
    }
    HIP_TRY(c, fade_gemm_group_launch(gg, c->stream));
  } else {
    for (int i = 0; i < ph.n; ++i) HIP_TRY(c, fade_gemm(ph.op[i] == GEMM_W_TN ? GEMM_W : ph.op[i], false, ph.g[i], c->stream));
  }
  return FADE_OK;
}
TransposeArgs tr_desc(fade_ctx *c, const void *src, int ld, void *dst, const float *stats, const float *gamma, const float *beta) {
  TransposeArgs t{};
  t.src = src; t.ld = ld; t.dst = dst; t.Bp = (int)c->Bp; t.B = (int)c->d.B;
  t.stats = stats; t.stats_n = (int)c->stats_n; t.width = ld; t.gamma = gamma; t.beta = beta;
  return t;
}
int backward(fade_ctx *c, const WinSrc &ws, const uint8_t *targets, long long tstride) {
  const Dims &d = c->d;
  // The weight-gradient products (w) feed nothing but Adam and could overlap the chain of activation gradients (s) on a
  // second stream; that variant produced rare wrong results on this machine whose cause was not found, so both are one stream.
  hipStream_t s = c->stream, w = c->stream;
  const bool bf = c->bf16;
  const int B = (int)d.B, Dh = (int)d.Dh, De = (int)d.De, dl = (int)d.dl, SN = (int)c->stats_n;
  float *G = c->grad;
  auto Gp = [&](int id) { return G + c->lay.off[id]; };
  const int RB = (B + fade_rows_per_block(B) - 1) / fade_rows_per_block(B);
  ReduceBatch rq{};  // second-stage reductions nothing in here waits for: one launch before Adam
  c->tn2q.count = 0;
  int rc;
  // ablation level: the head's gradient enters the chain at the level's feature vector; the stages behind it do not run
  // and their parameters keep a zero gradient (their Adam step is then exactly zero)
  const int level = c->cfg.ablation == 0 ? 5 : (int)c->cfg.ablation;
  const void *feat = level >= 5 ? c->Hout : level >= 3 ? c->Hc : level == 2 ? c->Hmix : c->Hg;
  void *dfeat = level >= 5 ? c->dHout : level >= 3 ? c->dHc : c->dHmix1;
  if (bf) {  // the loss gradient, and in the same launch the two left operands the forward pass never stores: LN(H_coarse), LN(H_mix), row-major
    Prof p(c, "bwd_loss_ln_copies");
    LnApplyBatch lb{};
    lb.B = B; lb.Dh = Dh; lb.stats_n = SN;
    if (level >= 5) lb.a[lb.count++] = {c->Hc, c->LT[2], c->stats_f, c->P(P_GAMMA_F), c->P(P_BETA_F)};
    if (level >= 3) lb.a[lb.count++] = {c->Hmix, c->LT[5], c->stats_c, c->P(P_GAMMA_C), c->P(P_BETA_C)};
    lb.with_loss = 1;
    lb.loss = LossGradArgs{ws, targets, tstride, c->probs_buf, c->ustate, c->cfg.beta1, c->cfg.beta2, c->dl, c->col_part};
    HIP_TRY(c, fade_ln_apply(lb, true, s));
    if (!rq.push((B + 7) / 8, 256, c->col_part, Gp(P_BO))) return fail(c, FADE_E_INVALID_ARG, "reduction queue full");
  } else {  // fp32 path: feature-major copies of every forward activation that is the left operand of a weight gradient
    {
      Prof p(c, "bwd_prep_dlogits");
      HIP_TRY(c, fade_loss_grad(ws, targets, tstride, B, c->probs_buf, c->ustate, c->cfg.beta1, c->cfg.beta2, c->dl, c->col_part, Gp(P_BO), bf, rq, s));
    }
    Prof p(c, "transpose", w);
    TransposeBatch tb{};
    auto add = [&](const void *src, int width, void *dst, const float *st, const float *ga, const float *be) {
      tb.t[tb.count] = tr_desc(c, src, width, dst, st, ga, be);
      tb.N[tb.count++] = width;
    };
    add(feat, Dh, c->LT[0], nullptr, nullptr, nullptr);  // the stage the head reads (H of Eq. 10 with every stage on)
    add(c->Hexp, De, c->LT[1], nullptr, nullptr, nullptr);
    add(c->Hc, Dh, c->LT[2], c->stats_f, c->P(P_GAMMA_F), c->P(P_BETA_F));   // u = LN(H_coarse)
    add(c->Hmix, Dh, c->LT[3], nullptr, nullptr, nullptr);
    add(c->z, dl, c->LT[4], nullptr, nullptr, nullptr);
    add(c->Hmix, Dh, c->LT[5], c->stats_c, c->P(P_GAMMA_C), c->P(P_BETA_C)); // LN(H_mix)
    add(c->M, (int)d.Dc, c->LT[6], nullptr, nullptr, nullptr);
    HIP_TRY(c, fade_transpose_batch(tb, false, w));
    HIP_TRY(c, fade_embed_t(ws, B, (int)c->Bp, (int)d.T, (int)d.D, c->tabXe, c->LT[7], false, w));  // X^T straight from the table
  }
  // head
  {
    PhaseGemms ph;
    ph.add(GEMM_W_TN, args_w(c, feat, Dh, c->LT[0], Dh, c->dl, 256, P_WO));
    ph.add(GEMM_X_STORE, args_x(c, c->dl, 256, Dh, c->WT_o, c->P(P_WO), 256, dfeat));
    if ((rc = run_phase(c, "gemms_head", ph))) return rc;
  }
  if (level >= 5) {
  {  // Eq. 10
    Prof p(c, "bwd_out");
    BwdOutArgs a{};
    a.B = B; a.Dh = Dh; a.stats_n = SN; a.ln_part = c->ln_part; a.dH = c->dHout; a.V = c->V; a.Hc = c->Hc; a.stats = c->stats_o; a.gamma = c->P(P_GAMMA_O);
    a.beta = c->P(P_BETA_O); a.lam = c->P(P_LAMBDA_O); a.dV = c->dV; a.dHc = c->dHc; a.row_dlam = c->row_dlam;
    HIP_TRY(c, fade_bwd_out(a, bf, s));
    rq.push(RB, 2 * Dh, c->ln_part, Gp(P_GAMMA_O));  // gamma_o then beta_o, adjacent in the blob
  }
  {
    PhaseGemms ph;
    ph.add_pair(args_x(c, c->dV, Dh, De, c->WT_f, c->P(P_WF), Dh, c->dHexp), args_w(c, c->Hexp, De, c->LT[1], De, c->dV, Dh, P_WF));
    if ((rc = run_phase(c, "gemms_fnr_out", ph))) return rc;
  }
  {  // Eq. 9
    Prof p(c, "bwd_geglu");
    HIP_TRY(c, fade_bwd_geglu(B, De, c->dHexp, c->eg, c->ev, c->dE, bf, s));
  }
  {
    PhaseGemms ph;
    GemmArgs gx = args_x(c, c->dE, 2 * De, Dh, c->WT_fgv, static_cast<const float *>(c->Wfgv_c), 2 * De, c->du);
    if (c->sp_du > 1) {  // a long contraction (K = 2 D_e) over few output tiles: ranges of K as fp32 partials, summed by the next kernel
      gx.splits = c->sp_du; gx.C = c->du_part;
      ph.add(GEMM_PARTIAL, gx);
      ph.add(GEMM_W_TN, args_w(c, c->LT[2], Dh, c->LT[2], Dh, c->dE, 2 * De, P_WFG, P_WFV));
    } else {
      ph.add(GEMM_W_TN, args_w(c, c->LT[2], Dh, c->LT[2], Dh, c->dE, 2 * De, P_WFG, P_WFV));
      ph.add(GEMM_X_STORE, gx);
    }
    if ((rc = run_phase(c, "gemms_fnr_in", ph))) return rc;
  }
  }
  if (level >= 3) {
  {  // LN of Eq. 9 + Eq. 8
    Prof p(c, "bwd_gate");
    BwdGateArgs a{};
    a.B = B; a.Dh = Dh; a.stats_n = SN; a.ln_part = c->ln_part + (size_t)RB * 2 * Dh; a.du = level >= 5 ? c->du : nullptr;
    if (level >= 5 && c->sp_du > 1) { a.du_part = c->du_part; a.du_splits = c->sp_du; } a.Hc = c->Hc; a.dHc = c->dHc;
    a.sg = level >= 4 ? c->sg : nullptr; a.Ha = c->Ha; a.Hmix = c->Hmix;
    a.stats = c->stats_f; a.gamma = c->P(P_GAMMA_F); a.lam = c->P(P_LAMBDA_C); a.dHa = c->dHa; a.dac = c->dac; a.dHmix = c->dHmix1;
    a.row_dlam = c->row_dlam + B;
    HIP_TRY(c, fade_bwd_gate(a, bf, s));
    if (level >= 5) rq.push(RB, 2 * Dh, c->ln_part + (size_t)RB * 2 * Dh, Gp(P_GAMMA_F));
  }
  {  // Eq. 8's gate product and Eq. 7's Up
    PhaseGemms ph;
    if (level >= 4) ph.add_pair(args_x(c, c->dac, Dh, Dh, c->WT_c, c->P(P_WC), Dh, c->dHmix2), args_w(c, c->Hmix, Dh, c->LT[3], Dh, c->dac, Dh, P_WC));
    ph.add(GEMM_W_TN, args_w(c, c->z, dl, c->LT[4], dl, c->dHa, Dh, P_WUP));
    GemmArgs g{};
    g.M = B; g.N = dl; g.K = Dh; g.splits = c->sp_dz; g.A = c->dHa; g.lda = Dh; g.C = c->dz_part; g.ldc = dl;
    if (bf) g.W = c->WT_up;
    else { g.W = c->P(P_WUP); g.wt = 1; g.ldb = Dh; g.rows16 = c->rows16 && c->sp_dz <= 1 && dl % 16 == 0; }
    ph.add(GEMM_PARTIAL, g);
    if ((rc = run_phase(c, "gemms_gate_up", ph))) return rc;
  }
  {  // per-stream memory: dy, and Adam on W_U in place
    Prof p(c, "bwd_cci_adam");
    BwdCciArgs a{};
    a.B = B; a.splits = c->sp_dz; a.dz_part = c->dz_part; a.y = c->y; a.WU_c = c->WU_c;
    a.master = c->master + c->lay.off[P_WU]; a.m = c->adam_m + c->lay.off[P_WU]; a.v = c->adam_v + c->lay.off[P_WU];
    a.dy = c->dy; a.dy_at = c->dy_at; a.u = c->ustate;
    a.lr = c->cfg.lr; a.beta1 = c->cfg.beta1; a.beta2 = c->cfg.beta2; a.eps = c->cfg.eps;
    a.g_dbg = c->debug_wu_grad ? c->grad + c->lay.off[P_WU] : nullptr;
    HIP_TRY(c, fade_bwd_cci(a, bf, s));
  }
  {
    PhaseGemms ph;
    ph.add(GEMM_W_TN, args_w(c, c->LT[5], Dh, c->LT[5], Dh, c->dy_at, dl, P_WDOWN));
    ph.add(GEMM_X_STORE, args_x(c, c->dy_at, dl, Dh, c->WT_down, c->P(P_WDOWN), dl, c->dnc));
    if ((rc = run_phase(c, "gemms_down", ph))) return rc;
  }
  }
  {  // LN of Eq. 7 + Eq. 5-6 + branch activations
    Prof p(c, "bwd_mix");
    BwdMixArgs a{};
    a.B = B; a.Dh = Dh; a.stats_n = SN; a.ln_part = c->ln_part + (size_t)RB * 4 * Dh; a.dnc = level >= 3 ? c->dnc : nullptr; a.Hmix = c->Hmix; a.dHmix1 = c->dHmix1;
    a.dHmix2 = level >= 4 ? c->dHmix2 : nullptr; a.alpha = level >= 2 ? c->alpha : nullptr;
    a.hm = c->hm; a.cv = c->cv; a.X = c->X; a.stats = c->stats_c; a.gamma = c->P(P_GAMMA_C);
    a.lam = c->P(P_LAMBDA_M); a.dar = c->dar; a.dhm = c->dhm; a.dcv = c->dcv; a.dX = c->dX1; a.row_dlam = c->row_dlam + 2 * B;
    HIP_TRY(c, fade_bwd_mix(a, bf, s));
    if (level >= 3) rq.push(RB, 2 * Dh, c->ln_part + (size_t)RB * 4 * Dh, Gp(P_GAMMA_C));
    if (level >= 5) rq.push(B, 1, c->row_dlam, Gp(P_LAMBDA_O));  // the three residual scales: per-stream terms, one column each
    if (level >= 3) rq.push(B, 1, c->row_dlam + B, Gp(P_LAMBDA_C));
    rq.push(B, 1, c->row_dlam + 2 * B, Gp(P_LAMBDA_M));
  }
  {  // router and global stream
    PhaseGemms ph;
    if (level >= 2) ph.add_pair(args_x(c, c->dar, Dh, Dh, c->WT_r, c->P(P_WR), Dh, c->dX2), args_w(c, c->X, Dh, c->LT[7], Dh, c->dar, Dh, P_WR));
    ph.add(GEMM_W_TN, args_w(c, c->M, (int)d.Dc, c->LT[6], (int)d.Dc, c->dhm, Dh, P_WM));
    if ((rc = run_phase(c, "gemms_router_global", ph))) return rc;
  }
  {
    const bool both = bf && level >= 2 && d.D == 32 && d.Kc <= 128 && d.k * 32 <= d.Kc;  // the matrix-core conv kernel also forms d(input)
    BwdSlotArgs a{};
    a.dg = c->dg_slot;
    a.Dh = Dh; a.Dc = (int)d.Dc; a.c = (int)d.c; a.D = (int)d.D; a.round_bf16 = bf ? 1 : 0; a.dhm = c->dhm; a.Wm = c->P(P_WM);
    a.GG = c->GG; a.GV = c->GV; a.Wg = c->Wg_c; a.Wv = c->Wv_c; a.dgg = c->dgg; a.dgv = c->dgv; a.dxt = c->dxt;
    a.ws = ws; a.B = B; a.T = (int)d.T; a.tabXe32 = c->tabXe32; a.part = c->slot_part;
    ConvGradArgs cg{};  // local stream
    cg.B = B; cg.T = (int)d.T; cg.D = (int)d.D; cg.taps = (int)d.k; cg.XL = c->XL; cg.dcv = c->dcv; cg.part = c->conv_part;
    {
      Prof p(c, "bwd_slot_conv");
      if (c->dg_slot) {  // wide slots: dg = d(hm) W_m[Dc-c..Dc)^T as a product
        GemmArgs g = args_x(c, c->dhm, Dh, (int)d.c, c->WT_mslot, c->P(P_WM) + (d.Dc - d.c) * d.Dh, Dh, c->dg_slot);
        HIP_TRY(c, fade_gemm(GEMM_X_STORE, bf, g, s));
      }
      if (both) {  // newest-slot backward and conv backward are independent: one launch (W_g then W_v, W_conv then b_conv: adjacent in the blob)
        cg.WT = c->WT_conv; cg.dxl = c->dxl; cg.Kc = (int)d.Kc;
        HIP_TRY(c, fade_bwd_slot_conv(a, Gp(P_WG), cg, Gp(P_WCONV), rq, s));
      } else {
        HIP_TRY(c, fade_bwd_slot(a, Gp(P_WG), bf, rq, s));
      }
    }
    if (level >= 2 && !both) {
      Prof p(c, "bwd_conv");
      HIP_TRY(c, fade_conv_grad(cg, Gp(P_WCONV), bf, rq, s));  // W_conv then b_conv, adjacent in the blob
      GemmArgs g{};
      g.M = (int)(d.B * d.T); g.N = (int)d.D; g.K = (int)d.Kc; g.A = c->dcv; g.T = (int)d.T; g.D = (int)d.D; g.taps = (int)d.k;
      g.W = bf ? c->WT_conv : static_cast<const void *>(c->convt_f32); g.C = c->dxl; g.ldc = (int)d.D;
      HIP_TRY(c, fade_gemm(GEMM_CONVT, bf, g, s));
    }
  }
  {  // the two per-token LayerNorms and the embedding
    Prof p(c, "bwd_embed");
    BwdTokenArgs a{};
    a.ws = ws; a.B = B; a.T = (int)d.T; a.D = (int)d.D; a.dX1 = c->dX1; a.dX2 = c->dX2; a.dxl = c->dxl; a.dxt = c->dxt;
    a.tabXhat = c->tabXhat; a.tabRstd = c->tabRstd; a.gamma_e = c->P(P_GAMMA_E); a.gamma_l = c->P(P_GAMMA_L);
    a.part = c->emb_part;
    // gamma_e, beta_e, gamma_l, beta_l are adjacent in the blob
    HIP_TRY(c, fade_bwd_embed(a, c->emb_blocks, c->tok_part, Gp(P_E), Gp(P_GAMMA_E), bf, rq, s));
  }
  // Adam on everything except W_U (done in place above) and the refresh of every compute copy: the matrices first (their
  // pass leaves the partial sums of the folded-LayerNorm vectors), then one launch for every pending column sum (vectors,
  // scalars, biases and the small tensors get their Adam step right where their gradient sums are finished), then the small
  // operand copies and the per-symbol tables
  if (c->tn2q.count > 0) {  // the weight gradients that waited: their operands are activations and gradients of this pass, all still in place
    Prof p(c, "gemms_weights");
    HIP_TRY(c, fade_gemm_tn2_group_launch(c->tn2q, s));
    c->tn2q.count = 0;
  }
  {
    Prof p(c, "adam_matrices");
    if ((rc = refresh_matrices(c, true))) return rc;
  }
  {
    Prof p(c, "refresh_small");
    const AdamArrays opt{c->grad, c->master, c->adam_m, c->adam_v, c->ustate, c->cfg.lr, c->cfg.beta1, c->cfg.beta2, c->cfg.eps};
    rq.opt = opt;
    rq.push(1, (int)(256 * d.D), Gp(P_E), Gp(P_E));  // dE is complete already: a one-row "sum" that only adds the Adam step
    if (bf) {
      rc = refresh_small(c, &rq);
    } else {
      HIP_TRY(c, fade_reduce_batch(rq, s));
      rc = prepare_compute(c, false);
    }
    if (rc) return rc;
  }
  return FADE_OK;
}

int check_dev_err(fade_ctx *c) {
  int e = 0;
  HIP_TRY(c, hipMemcpy(&e, c->dev_err, sizeof(int), hipMemcpyDeviceToHost));
  if (e == 1) return fail(c, FADE_E_BUFFER_TOO_SMALL, "payload buffer exhausted");
  if (e == 2) return fail(c, FADE_E_CORRUPT_STREAM, "decoder left its interval: payload does not match the model");
  if (e == 3) return fail(c, FADE_E_NUMERIC, "non-finite probabilities");
  return FADE_OK;
}

size_t payload_cap_for(size_t L) { return 2 * L + 16; }

int ensure_payload(fade_ctx *c, size_t L) {
  const size_t cap = payload_cap_for(L);
  if (c->payload && c->payload_cap >= cap) return FADE_OK;
  // grow only: older (smaller) buffers stay owned by the context until it is destroyed
  uint8_t *p = nullptr;
  int rc = dev_alloc(c, &p, c->d.B * cap);
  if (rc) return rc;
  c->payload = p;
  c->payload_cap = cap;
  c->cb.out = p; c->cb.in = p; c->cb.cap = cap;
  return FADE_OK;
}

// Payloads live strided ([B][cap]) on the device and concatenated on the host: one staging buffer, one copy, one kernel.
// gather: device -> host after encoding (lens_host already filled); else host -> device before decoding (also uploads lengths).
int move_payloads(fade_ctx *c, uint32_t *lens_host, uint8_t *bytes_host, size_t total, int gather) {
  const size_t B = c->d.B;
  std::vector<unsigned long long> off(B);
  unsigned long long o = 0;
  for (size_t b = 0; b < B; ++b) { off[b] = o; o += lens_host[b]; }
  void *off_p = nullptr, *flat_p = nullptr;
  int rc = stage_buf(c, STAGE_OFF, B * sizeof(unsigned long long), &off_p);
  if (!rc) rc = stage_buf(c, STAGE_FLAT, total, &flat_p);
  if (rc) return rc;
  unsigned long long *off_dev = static_cast<unsigned long long *>(off_p);
  uint8_t *flat = static_cast<uint8_t *>(flat_p);
  hipStream_t s = c->stream;
  hipError_t e = hipMemcpyAsync(off_dev, off.data(), B * sizeof(unsigned long long), hipMemcpyHostToDevice, s);
  if (e == hipSuccess && !gather) {
    e = hipMemcpyAsync(c->in_len, lens_host, B * sizeof(uint32_t), hipMemcpyHostToDevice, s);
    if (e == hipSuccess && total) e = hipMemcpyAsync(flat, bytes_host, total, hipMemcpyHostToDevice, s);
  }
  if (e == hipSuccess) e = fade_payload_move(c->payload, c->payload_cap, flat, off_dev, gather ? c->cb.pos : c->in_len, (int)B, gather, s);
  if (e == hipSuccess && gather && total) e = hipMemcpyAsync(bytes_host, flat, total, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(c, e, "payload transfer");
  return FADE_OK;
}

// the loop of Algorithm 1 on device-resident bytes, steps [first, first + count); mode is CODE_ENCODE or CODE_DECODE
int run_loop(fade_ctx *c, uint8_t *bytes_dev, size_t n, size_t first, size_t count, int mode) {
  const Dims &d = c->d;
  hipStream_t s = c->stream;
  const size_t L = (n + d.B - 1) / d.B;
  const size_t last = (count == 0 || first + count > L) ? L : first + count;
  WinSrc ws{};
  ws.base = bytes_dev; ws.stride = (long long)L; ws.n = (long long)n; ws.active = nullptr;
  for (size_t i = first; i < last; ++i) {
    ws.i = (long long)i;
    if (i < d.T) {
      Prof p(c, "code_uniform");
      HIP_TRY(c, fade_code_uniform(ws, bytes_dev, (int)d.B, c->cb, mode, s));
    } else if (mode == CODE_ENCODE && c->steps_max > 1 && last - i > 1) {
      // frozen weights and the whole input at hand: the model's steps do not depend on each other, only the coder's do
      const int steps = (int)std::min<size_t>((size_t)c->steps_max, last - i);
      int rc = forward_bf16(c, ws, mode, bytes_dev, nullptr, nullptr, steps);
      if (rc) return rc;
      i += (size_t)steps - 1;
      if (last - (i + 1) < 2)  // leave the rolling cache as the last of these steps would have: single steps may follow
        HIP_TRY(c, hipMemcpyAsync(c->M, static_cast<char *>(c->M) + (size_t)(steps - 1) * d.B * d.Dc * c->esz, d.B * d.Dc * c->esz,
                                  hipMemcpyDeviceToDevice, s));
    } else {
      int rc = forward(c, ws, mode, bytes_dev, nullptr, nullptr);
      if (rc) return rc;
      if (c->online) {  // Algorithm 1: update after the symbol has been coded (the decoder has just produced it)
        rc = backward(c, ws, bytes_dev + i, (long long)L);
        if (rc) return rc;
      }
    }
  }
  c->loop_next = last;
  if (mode == CODE_ENCODE && last == L && !c->enc_complete) {
    HIP_TRY(c, fade_coder_finish(c->cb, (int)d.B, (long long)L, (long long)n, s));
    c->enc_complete = true;
  }
  HIP_TRY(c, hipStreamSynchronize(s));
  if (c->profiling) prof_collect(c);
  return check_dev_err(c);
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------------
extern "C" {

size_t fade_weights_nbytes(const fade_config *cfg) {
  Dims d;
  if (!cfg || resolve_dims(*cfg, d, nullptr)) return 0;
  return make_layout(d, true).off[P_COUNT] * sizeof(float);
}

void fade_destroy(fade_ctx *c) {
  if (!c) return;
  if (c->stream) (void)hipStreamSynchronize(c->stream);
  for (auto &ev : c->events) { (void)hipEventDestroy(ev.a); (void)hipEventDestroy(ev.b); }
  for (void *p : c->allocs) (void)hipFree(p);
  for (void *p : c->stage) if (p) (void)hipFree(p);
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
  delete c;
}

int fade_create(const fade_config *cfg, fade_ctx **out) {
  if (!cfg || !out) return FADE_E_INVALID_ARG;
  *out = nullptr;
  if (cfg->struct_size != sizeof(fade_config) || cfg->abi_version != FADE_ABI_VERSION) return FADE_E_INVALID_ARG;
  Dims d;
  std::string why;
  int rc = resolve_dims(*cfg, d, &why);
  if (rc) return rc;
  rc = check_kernel_limits(*cfg, d, &why);
  if (rc) return rc;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) return FADE_E_HIP;
  if (hipSetDevice(cfg->device) != hipSuccess) return FADE_E_HIP;
  fade_ctx *c = new (std::nothrow) fade_ctx();
  if (!c) return FADE_E_OOM;
  if (scratch_for_device(cfg->device, &c->scratch_dev) != hipSuccess) { delete c; return FADE_E_HIP; }
  c->cfg = *cfg;
  if (c->cfg.lr == 0.0f) c->cfg.lr = 1e-3f;
  if (c->cfg.beta1 == 0.0f) c->cfg.beta1 = 0.9f;
  if (c->cfg.beta2 == 0.0f) c->cfg.beta2 = 0.999f;
  if (c->cfg.eps == 0.0f) c->cfg.eps = 1e-8f;
  c->d = d;
  c->lay = make_layout(d, false);
  c->blob = make_layout(d, true);
  c->bf16 = cfg->dtype == FADE_BF16;
  c->online = cfg->update_mode == FADE_ONLINE_ADAM;
  c->esz = c->bf16 ? 2 : 4;
  if (const char *e = getenv("FADE_DEBUG_WU_GRAD")) c->debug_wu_grad = e[0] == '1';
  if (cfg->hip_stream) c->stream = static_cast<hipStream_t>(cfg->hip_stream);
  else {
    if (hipStreamCreate(&c->stream) != hipSuccess) { delete c; return FADE_E_HIP; }
    c->own_stream = true;
  }
  if (c->bf16 && !c->online) {  // rows of one multi-step encode pass: enough to fill the chip, bounded by the buffers' size
    size_t steps = std::max<size_t>(1, 16384 / d.B);
    steps = std::min(steps, std::max<size_t>(1, ((size_t)1 << 26) / (d.B * d.Dh)));
    if (const char *e = getenv("FADE_STEPS_PER_PASS")) steps = (size_t)std::max(1, atoi(e));
    c->steps_max = (int)std::min<size_t>(steps, 256);
  }
  const size_t R = d.B * (size_t)c->steps_max;  // rows of the forward buffers
  const size_t np = c->lay.off[P_COUNT], BDh = R * d.Dh;
  // fp32 contexts of up to 256 streams use the small-batch products (statistics per 16 columns); FADE_F32_ROWS16=0 keeps the general kernel
  c->rows16 = !c->bf16 && d.B <= 256 && d.Dh <= 2048 && d.Dc <= 2048 && d.De <= 2048 && d.Dh % 16 == 0 && d.Dc % 16 == 0 && d.De % 64 == 0 &&
              d.Kc % 16 == 0 && d.D % 16 == 0;
  if (const char *e = getenv("FADE_F32_ROWS16")) c->rows16 = c->rows16 && e[0] != '0';
  const size_t SN = c->rows16 ? d.Dh / 16 : d.Dh / FADE_STATS_BN;
  c->stats_n = SN;
  auto A = [&](void **p, size_t elems) { return dev_alloc_bytes(c, p, elems * c->esz); };
#define TRY_ALLOC(expr) do { rc = (expr); if (rc) { fade_destroy(c); return rc; } } while (0)
  TRY_ALLOC(dev_alloc(c, &c->master, np));
  if (c->bf16) {
    TRY_ALLOC(dev_alloc(c, &c->E_c, 256 * d.D));
    TRY_ALLOC(dev_alloc(c, &c->Wg_c, d.D * d.c));
    TRY_ALLOC(dev_alloc(c, &c->Wv_c, d.D * d.c));
    TRY_ALLOC(A(&c->Wm_c, d.Dc * d.Dh));
    TRY_ALLOC(A(&c->Wconv_c, d.Kc * d.D));
    TRY_ALLOC(A(&c->Wr_c, d.Dh * d.Dh));
    TRY_ALLOC(A(&c->Wdown_c, d.Dh * d.dl));
    TRY_ALLOC(A(&c->WU_c, d.B * d.dl * d.dl));
    TRY_ALLOC(A(&c->Wup_c, d.dl * d.Dh));
    TRY_ALLOC(A(&c->Wc_c, d.Dh * d.Dh));
    TRY_ALLOC(A(&c->Wfgv_c, d.Dh * 2 * d.De));
    TRY_ALLOC(A(&c->Wf_c, d.De * d.Dh));
    TRY_ALLOC(A(&c->Wo_c, d.Dh * 256));
    TRY_ALLOC(A(&c->Hout, BDh));
    c->sp_down = pick_splits((int)((d.B + 63) / 64), (int)(d.Dh / 64), 16);
    c->sp_fnr = pick_splits((int)((d.B + 127) / 128 * (2 * d.De / 128)), (int)(d.Dh / 64), 8);
    c->sp_head = pick_splits((int)((d.B + 127) / 128 * 2), (int)(d.Dh / 64), 8);
    // single steps leave one slice per K range, multi-step passes one slice of all their rows
    const auto part_rows = [&](int splits) { return std::max((size_t)splits * d.B, R); };
    TRY_ALLOC(dev_alloc(c, &c->part_down, part_rows(c->sp_down) * d.dl));
    if (c->sp_fnr > 1) TRY_ALLOC(dev_alloc(c, &c->part_fnr, part_rows(c->sp_fnr) * 2 * d.De));  // one K range: no partials (folded epilogue)
    TRY_ALLOC(dev_alloc(c, &c->part_head, part_rows(c->sp_head) * 256));
    if (c->steps_max > 1) TRY_ALLOC(dev_alloc(c, &c->ranges, R));
    if (!c->online) {
      TRY_ALLOC(A(&c->slot_tab, 256 * d.c));
    } else {
      TRY_ALLOC(dev_alloc(c, &c->gg_tab, 256 * d.c));
      TRY_ALLOC(dev_alloc(c, &c->gv_tab, 256 * d.c));
    }
    TRY_ALLOC(dev_alloc(c, &c->s_down, 2 * d.dl));
    c->t_down = c->s_down + d.dl;
    TRY_ALLOC(dev_alloc(c, &c->s_fnr, 4 * d.De));
    c->t_fnr = c->s_fnr + 2 * d.De;
    TRY_ALLOC(dev_alloc(c, &c->fold_down, d.Dh / 64 * 2 * d.dl));
    TRY_ALLOC(dev_alloc(c, &c->fold_fnr, d.Dh / 64 * 2 * 2 * d.De));
  } else {  // fp32: most operands are used straight from the master blob
    c->E_c = c->master + c->lay.off[P_E];
    c->Wg_c = c->master + c->lay.off[P_WG];
    c->Wv_c = c->master + c->lay.off[P_WV];
    c->Wm_c = c->master + c->lay.off[P_WM];
    c->Wr_c = c->master + c->lay.off[P_WR];
    c->Wdown_c = c->master + c->lay.off[P_WDOWN];
    c->WU_c = c->master + c->lay.off[P_WU];
    c->Wup_c = c->master + c->lay.off[P_WUP];
    c->Wc_c = c->master + c->lay.off[P_WC];
    c->Wf_c = c->master + c->lay.off[P_WF];
    c->Wo_c = c->master + c->lay.off[P_WO];
    TRY_ALLOC(A(&c->Wconv_c, d.Kc * d.D));
    TRY_ALLOC(A(&c->Wfgv_c, d.Dh * 2 * d.De));
  }
  TRY_ALLOC(A(&c->tabXe, 256 * d.D));
  TRY_ALLOC(A(&c->tabXl, 256 * d.D));
  TRY_ALLOC(dev_alloc(c, &c->tabXe32, 256 * d.D));
  for (void **p : {&c->X, &c->XL, &c->Hg, &c->Hl, &c->Hmix, &c->Ha, &c->Hc, &c->V}) TRY_ALLOC(A(p, BDh));
  TRY_ALLOC(A(&c->M, R * d.Dc));
  TRY_ALLOC(A(&c->Hexp, R * d.De));
  TRY_ALLOC(A(&c->z, R * d.dl));
  TRY_ALLOC(dev_alloc(c, &c->y, R * d.dl));
  TRY_ALLOC(dev_alloc(c, &c->logits, d.B * 256));
  TRY_ALLOC(dev_alloc(c, &c->stats_c, R * SN * 2));
  TRY_ALLOC(dev_alloc(c, &c->stats_f, R * SN * 2));
  TRY_ALLOC(dev_alloc(c, &c->stats_o, R * SN * 2));
  if (c->online) {
    const size_t Bp = (d.B + 63) / 64 * 64, BpDh = Bp * d.Dh;
    c->Bp = Bp;
    for (void **p : {&c->hm, &c->alpha, &c->sg, &c->cv}) TRY_ALLOC(A(p, BDh));
    TRY_ALLOC(A(&c->eg, d.B * d.De));
    TRY_ALLOC(A(&c->ev, d.B * d.De));
    TRY_ALLOC(dev_alloc(c, &c->GG, d.B * d.c));
    TRY_ALLOC(dev_alloc(c, &c->GV, d.B * d.c));
    TRY_ALLOC(dev_alloc(c, &c->probs_buf, d.B * 256));
    if (!c->bf16) TRY_ALLOC(A(&c->Hout, BDh));
    TRY_ALLOC(dev_alloc(c, &c->grad, np));
    TRY_ALLOC(dev_alloc(c, &c->adam_m, np));
    TRY_ALLOC(dev_alloc(c, &c->adam_v, np));
    TRY_ALLOC(dev_alloc(c, &c->ustate, 1));
    TRY_ALLOC(dev_alloc(c, &c->tabXhat, 256 * d.D));
    TRY_ALLOC(dev_alloc(c, &c->tabRstd, 256));
    TRY_ALLOC(dev_alloc(c, &c->convt_f32, d.Kc * d.D));
    if (c->bf16) {
      TRY_ALLOC(A(&c->WT_o, d.Dh * 256));
      TRY_ALLOC(A(&c->WT_f, d.De * d.Dh));
      TRY_ALLOC(A(&c->WT_fgv, d.Dh * 2 * d.De));
      TRY_ALLOC(A(&c->WT_c, d.Dh * d.Dh));
      TRY_ALLOC(A(&c->WT_up, d.dl * d.Dh));
      TRY_ALLOC(A(&c->WT_down, d.Dh * d.dl));
      TRY_ALLOC(A(&c->WT_r, d.Dh * d.Dh));
      TRY_ALLOC(A(&c->WT_conv, d.Kc * d.D));
      if (d.c % 64 == 0) TRY_ALLOC(A(&c->WT_mslot, d.Dh * d.c));
    }
    if (d.c % 64 == 0) TRY_ALLOC(A(&c->dg_slot, Bp * d.c));
    // gradients that serve as the right operand of a weight-gradient product have Bp rows (padding rows stay zero)
    struct { void **p; size_t n; } bufs[] = {
        {&c->dl, Bp * 256}, {&c->dHout, BDh}, {&c->dV, BpDh}, {&c->dHc, BDh}, {&c->dHexp, d.B * d.De},
        {&c->dE, Bp * 2 * d.De}, {&c->du, BDh}, {&c->dHa, BpDh}, {&c->dac, BpDh}, {&c->dHmix1, BDh}, {&c->dHmix2, BDh},
        {&c->dy_at, Bp * d.dl}, {&c->dnc, BDh}, {&c->dar, BpDh}, {&c->dhm, BpDh}, {&c->dcv, BDh}, {&c->dX1, BDh}, {&c->dX2, BDh},
        {&c->dxl, BDh},
        {&c->LT[2], d.Dh * Bp}, {&c->LT[5], d.Dh * Bp}};
    for (auto &b : bufs) {
      TRY_ALLOC(A(b.p, b.n));
      if (hipMemsetAsync(*b.p, 0, b.n * c->esz, c->stream) != hipSuccess) { fade_destroy(c); return FADE_E_HIP; }
    }
    if (!c->bf16) {  // fp32 path: feature-major copies [width][Bp] of the remaining left operands
      struct { void **p; size_t n; } lts[] = {{&c->LT[0], d.Dh * Bp}, {&c->LT[1], d.De * Bp}, {&c->LT[3], d.Dh * Bp}, {&c->LT[4], d.dl * Bp},
                                               {&c->LT[6], d.Dc * Bp}, {&c->LT[7], d.Dh * Bp}};
      for (auto &b : lts) TRY_ALLOC(A(b.p, b.n));
    }
    if (c->bf16) {
      // weight gradients whose tiles are few: the contraction (the batch) is cut into ranges until the product has ~256
      // workgroups; products with tiles enough keep their single pass. The Adam pass reads every range's slice, so a
      // big matrix is cut only when its chain of 64-row blocks is long (B >= 2048) and into ranges of at least 8 blocks;
      // W_down (128 K elements) is cut down to ranges of 2 blocks. B = 1024: Down phase 16 -> 13 us, the others unchanged
      // (cutting them too cost 11 us more in the Adam pass than it saved); B = 4096: head / FNR-out / FNR-in / Down
      // phases 52 / 55 / 55 / 62 -> 24 / 37 / 39 / 16 us for 12 us more in the Adam pass.
      // The two D_h x D_h gradients (256 tiles: a full product by the rule above) share their phase with an activation
      // gradient whose workgroups walk D_h / 64 blocks while theirs walk the batch; after the first round of the 512
      // workgroup slots they run on half the chip, and two ranges make that second round a full one. The Adam pass pays
      // 15 us for the two extra 16 MiB slices, which B = 4096 only just gets back (phases 114 / 123 -> 106 / 115 us) and
      // B = 16384 does (445 / 460 -> 375 / 470, step 3.74 -> 3.64 ms): from 8192 rows on, with W_up and W_m of the same phases.
      const struct { int id, pair, M, N; } gw[] = {{P_WO, -1, (int)d.Dh, 256}, {P_WF, -1, (int)d.De, (int)d.Dh}, {P_WFG, P_WFV, (int)d.Dh, (int)(2 * d.De)},
                                                    {P_WDOWN, -1, (int)d.Dh, (int)d.dl}, {P_WUP, -1, (int)d.dl, (int)d.Dh}, {P_WM, -1, (int)d.Dc, (int)d.Dh},
                                                    {P_WC, -1, (int)d.Dh, (int)d.Dh}, {P_WR, -1, (int)d.Dh, (int)d.Dh}};
      // Weight gradients on 256 x 256 tiles feed nothing but the optimiser: with two or more of them they wait for the end
      // of the backward pass and run as ONE launch with the same number of ranges of the batch for every matrix, so that
      // all workgroups are equally long; the count is the smallest that gives at least two workgroups per compute unit
      // and wastes least of the last round (D_h = 2048, D_e = D_cache = 512, B = 16384: 192 tiles x 4 ranges = 3 rounds of
      // 256, 192 MiB of slices for the Adam pass to add up; launched one by one, with 4 / 8 / 16 ranges until each launch
      // had 256 workgroups: 320 MiB). FADE_TN2_DEFER=0 keeps the launches apart.
      int tn2_total = 0, tn2_count = 0, tn2_sp = 0;
      for (const auto &w : gw)
        if (fade_gemm_tn2_ok(w.M, w.N, (int)Bp)) { tn2_total += (w.M / 256) * (w.N / 256); ++tn2_count; }
      const char *defer_env = getenv("FADE_TN2_DEFER");
      if (tn2_count >= 2 && tn2_count <= 8 && !(defer_env && defer_env[0] == '0')) {
        const int nkb = (int)(Bp / 64);
        double best = 0.0;
        for (int sp = 1; sp <= 16; sp *= 2) {
          if (nkb % sp || nkb / sp < 8 || tn2_total * sp < 512) continue;
          const int blocks = tn2_total * sp;
          const double fill = (double)blocks / (((blocks + 255) / 256) * 256);
          if (fill > best + 1e-9) { best = fill; tn2_sp = sp; }
        }
        c->defer_tn2 = tn2_sp > 0;
      }
      for (const auto &w : gw) {
        if (fade_gemm_tn2_ok(w.M, w.N, (int)Bp)) {  // 256 x 256 tiles, one workgroup per compute unit: ranges until every unit has one
          const int tiles256 = (w.M / 256) * (w.N / 256), nkb = (int)(Bp / 64);
          int sp = 1;
          if (c->defer_tn2) sp = tn2_sp;
          else while (sp < 16 && tiles256 * sp * 2 <= 256 && nkb % (sp * 2) == 0 && nkb / (sp * 2) >= 8) sp *= 2;
          if (sp > 1) {
            c->gsp[w.id] = sp;
            TRY_ALLOC(dev_alloc(c, &c->gpart[w.id], (size_t)sp * c->lay.len[w.id]));
            if (w.pair >= 0) { c->gsp[w.pair] = sp; TRY_ALLOC(dev_alloc(c, &c->gpart[w.pair], (size_t)sp * c->lay.len[w.pair])); }
          }
          continue;
        }
        const int tiles = fade_gemm_tn_tiles(w.M, w.N);
        if (tiles <= 0) continue;
        const bool small = c->lay.len[w.id] <= (256u << 10);
        const int nkb = (int)(Bp / 64);
        if ((w.id == P_WUP || w.id == P_WM || w.id == P_WC || w.id == P_WR) && nkb < 128) continue;
        int sp;
        if (tiles < 192) {
          if (!small && nkb < 32) continue;
          sp = pick_splits(tiles, small ? nkb : nkb / 4, 16);  // nkb / 4: ranges of at least 8 blocks
        } else if (tiles < 512 && nkb >= 32 && nkb % 2 == 0) {
          sp = 2;
        } else {
          continue;
        }
        if (sp <= 1 || nkb % sp) continue;
        c->gsp[w.id] = sp;
        TRY_ALLOC(dev_alloc(c, &c->gpart[w.id], (size_t)sp * c->lay.len[w.id]));
        if (w.pair >= 0) { c->gsp[w.pair] = sp; TRY_ALLOC(dev_alloc(c, &c->gpart[w.pair], (size_t)sp * c->lay.len[w.pair])); }
      }
    }
    if (c->bf16 && 2 * d.De >= 4096 && d.Dh % 128 == 0) {
      c->sp_du = pick_splits((int)((d.B + 127) / 128 * (d.Dh / 128)) / 2, (int)(2 * d.De / 64 / 4), 16);  // ~384+ workgroups, ranges of 8+ blocks
      if (c->sp_du > 1) TRY_ALLOC(dev_alloc(c, &c->du_part, (size_t)c->sp_du * d.B * d.Dh));
    }
    c->sp_dz = c->bf16 ? pick_splits((int)((d.B + 63) / 64), (int)(d.Dh / 64), 16) : 1;
    TRY_ALLOC(dev_alloc(c, &c->dz_part, (size_t)c->sp_dz * d.B * d.dl));
    TRY_ALLOC(dev_alloc(c, &c->dy, d.B * d.dl));
    TRY_ALLOC(dev_alloc(c, &c->dgg, d.B * d.c));
    TRY_ALLOC(dev_alloc(c, &c->dgv, d.B * d.c));
    TRY_ALLOC(dev_alloc(c, &c->dxt, d.B * d.D));
    TRY_ALLOC(dev_alloc(c, &c->row_dlam, 3 * d.B));
    TRY_ALLOC(dev_alloc(c, &c->win_copy, d.B * d.T));
    const size_t tokens = d.B * d.T, rb = (d.B + fade_rows_per_block((int)d.B) - 1) / fade_rows_per_block((int)d.B);
    // workgroups of the per-symbol sums: each leaves a 64 KiB partial table, so few of them, but a workgroup walks its
    // 128-token chunks one after the other: 256 up to 64 Ki tokens (B = 1024: 22.5 us against 24.8 with 512), 512 above
    // (B = 4096: 43.9 against 52.9)
    c->emb_blocks = (int)std::min<size_t>(tokens > (64u << 10) ? 512 : 256, (tokens + 127) / 128);
    TRY_ALLOC(dev_alloc(c, &c->conv_part, (tokens + 127) / 128 * (d.k * d.D + 1) * d.D));
    TRY_ALLOC(dev_alloc(c, &c->tok_part, 256 * 4 * d.D));
    TRY_ALLOC(dev_alloc(c, &c->ln_part, 3 * rb * 2 * d.Dh));
    TRY_ALLOC(dev_alloc(c, &c->col_part, (d.B + 7) / 8 * 256));
    TRY_ALLOC(dev_alloc(c, &c->slot_part, (d.B + 3) / 4 * 2 * d.D * d.c));
    TRY_ALLOC(dev_alloc(c, &c->emb_part, (size_t)c->emb_blocks * 2 * 256 * d.D));
    if (hipMemsetAsync(c->grad, 0, np * sizeof(float), c->stream) != hipSuccess) { fade_destroy(c); return FADE_E_HIP; }
  }
  for (uint32_t **p : {&c->cb.low, &c->cb.high, &c->cb.pending, &c->cb.bitbuf, &c->cb.nbits, &c->cb.pos, &c->cb.value, &c->cb.bitpos})
    TRY_ALLOC(dev_alloc(c, p, d.B));
  TRY_ALLOC(dev_alloc(c, &c->in_len, d.B));
  c->cb.in_len = c->in_len;
  TRY_ALLOC(dev_alloc(c, &c->ones, d.B));
  TRY_ALLOC(dev_alloc(c, &c->dev_err, 1));
  c->cb.err = c->dev_err;
#undef TRY_ALLOC
  if (hipMemsetAsync(c->ones, 1, d.B, c->stream) != hipSuccess || hipMemsetAsync(c->dev_err, 0, sizeof(int), c->stream) != hipSuccess ||
      hipMemsetAsync(c->M, 0, d.B * d.Dc * c->esz, c->stream) != hipSuccess || hipStreamSynchronize(c->stream) != hipSuccess) {
    fade_destroy(c);
    return FADE_E_HIP;
  }
  *out = c;
  return FADE_OK;
}

int fade_load_weights(fade_ctx *c, const void *blob_host, size_t nbytes) {
  if (!c || !blob_host) return FADE_E_INVALID_ARG;
  const size_t np = c->blob.off[P_COUNT];
  if (nbytes != np * sizeof(float)) return fail(c, FADE_E_WEIGHTS_MISMATCH, "blob size does not match the configuration");
  const float *f = static_cast<const float *>(blob_host);
  for (size_t i = 0; i < np; ++i)
    if (!std::isfinite(f[i])) return fail(c, FADE_E_NUMERIC, "non-finite weight");
  c->loaded.assign(c->lay.off[P_COUNT], 0.0f);  // kept in the device layout
  for (int t = 0; t < P_COUNT; ++t) std::memcpy(c->loaded.data() + c->lay.off[t], f + c->blob.off[t], c->blob.len[t] * sizeof(float));
  c->weights_hash = fnv1a64(blob_host, nbytes);
  c->have_weights = true;
  return do_reset(c);
}

int fade_reset(fade_ctx *c) {
  if (!c) return FADE_E_INVALID_ARG;
  return do_reset(c);
}

int fade_step_probs(fade_ctx *c, const uint8_t *windows_dev, const uint8_t *active_dev, uint16_t *freq_dev, float *probs_dev) {
  if (!c || !windows_dev) return FADE_E_INVALID_ARG;
  if (!c->have_weights) return fail(c, FADE_E_NO_WEIGHTS, "no weights loaded");
  WinSrc ws{};
  ws.base = windows_dev; ws.stride = (long long)c->d.T; ws.n = 0; ws.active = active_dev ? active_dev : c->ones; ws.i = (long long)c->d.T;
  if (c->online) {  // fade_step_update re-reads the windows (embedding and slot gradients): keep a copy, the caller's may be gone by then
    HIP_TRY(c, hipMemcpyAsync(c->win_copy, windows_dev, c->d.B * c->d.T, hipMemcpyDeviceToDevice, c->stream));
    ws.base = c->win_copy;
  }
  c->last_ws = ws;
  return forward(c, ws, CODE_NONE, nullptr, freq_dev, probs_dev);
}

int fade_step_update(fade_ctx *c, const uint8_t *targets_dev, const uint8_t *active_dev) {
  if (!c || !targets_dev) return FADE_E_INVALID_ARG;
  if (!c->online) return fail(c, FADE_E_BAD_CONFIG, "context is frozen");
  if (!c->have_weights) return fail(c, FADE_E_NO_WEIGHTS, "no weights loaded");
  WinSrc ws = c->last_ws;
  ws.active = active_dev ? active_dev : c->ones;
  return backward(c, ws, targets_dev, 1);
}

size_t fade_encode_bound(const fade_ctx *c, size_t n) {
  if (!c) return 0;
  const size_t B = c->d.B, L = (n + B - 1) / B;
  return kHeaderBytes + 4 * B + B * (2 * L + 8);
}

int fade_encode_device(fade_ctx *c, const uint8_t *src_dev, size_t n, size_t first_step, size_t n_steps) {
  if (!c || (!src_dev && n)) return FADE_E_INVALID_ARG;
  if (!c->have_weights) return fail(c, FADE_E_NO_WEIGHTS, "no weights loaded");
  if (first_step == 0) {
    int rc = do_reset(c);
    if (rc) return rc;
    rc = ensure_payload(c, (n + c->d.B - 1) / c->d.B);
    if (rc) return rc;
    HIP_TRY(c, fade_coder_init(c->cb, (int)c->d.B, 0, c->stream));
    c->loop_n = n; c->loop_next = 0; c->loop_mode = CODE_ENCODE;
  } else if (c->loop_mode != CODE_ENCODE || c->loop_n != n || c->loop_next != first_step) {
    return fail(c, FADE_E_INVALID_ARG, "first_step does not continue the encode in progress");
  }
  return run_loop(c, const_cast<uint8_t *>(src_dev), n, first_step, n_steps, CODE_ENCODE);
}

int fade_payloads(fade_ctx *c, uint32_t *lengths_host, uint8_t *bytes_host, size_t cap, size_t *total) {
  if (!c || !lengths_host || !total) return FADE_E_INVALID_ARG;
  if (!c->enc_complete) return fail(c, FADE_E_INVALID_ARG, "no completed encode to read payloads from");
  const size_t B = c->d.B;
  HIP_TRY(c, hipMemcpy(lengths_host, c->cb.pos, B * sizeof(uint32_t), hipMemcpyDeviceToHost));
  size_t sum = 0;
  for (size_t b = 0; b < B; ++b) sum += lengths_host[b];
  *total = sum;
  if (sum > cap || (!bytes_host && sum)) return fail(c, FADE_E_BUFFER_TOO_SMALL, "payload buffer too small");
  return move_payloads(c, lengths_host, bytes_host, sum, 1);
}

int fade_decode_device(fade_ctx *c, const uint32_t *lengths_host, const uint8_t *bytes_host, size_t total, uint8_t *dst_dev,
                       size_t n, size_t first_step, size_t n_steps) {
  if (!c || (!dst_dev && n)) return FADE_E_INVALID_ARG;
  if (!c->have_weights) return fail(c, FADE_E_NO_WEIGHTS, "no weights loaded");
  const size_t B = c->d.B, L = (n + B - 1) / B;
  if (first_step != 0) {
    if (c->loop_mode != CODE_DECODE || c->loop_n != n || c->loop_next != first_step)
      return fail(c, FADE_E_INVALID_ARG, "first_step does not continue the decode in progress");
    return run_loop(c, dst_dev, n, first_step, n_steps, CODE_DECODE);
  }
  if (!lengths_host || (!bytes_host && total)) return FADE_E_INVALID_ARG;
  int rc = do_reset(c);
  if (rc) return rc;
  rc = ensure_payload(c, L);
  if (rc) return rc;
  size_t pos = 0;
  for (size_t b = 0; b < B; ++b) {
    const size_t len = lengths_host[b];
    if (len > c->payload_cap || len > total - pos) return fail(c, FADE_E_CORRUPT_STREAM, "payload length out of range");
    const bool empty = b * L >= n;
    if (empty != (len == 0)) return fail(c, FADE_E_CORRUPT_STREAM, "payload length does not match the stream split");
    pos += len;
  }
  if (pos != total) return fail(c, FADE_E_CORRUPT_STREAM, "trailing payload bytes");
  rc = move_payloads(c, const_cast<uint32_t *>(lengths_host), const_cast<uint8_t *>(bytes_host), total, 0);
  if (rc) return rc;
  HIP_TRY(c, fade_coder_init(c->cb, (int)B, 1, c->stream));
  c->loop_n = n; c->loop_next = 0; c->loop_mode = CODE_DECODE;
  return run_loop(c, dst_dev, n, 0, n_steps, CODE_DECODE);
}

int fade_encode(fade_ctx *c, const uint8_t *src_host, size_t n, uint8_t *dst_host, size_t dst_cap, size_t *dst_len) {
  if (!c || (!src_host && n) || !dst_host || !dst_len) return FADE_E_INVALID_ARG;
  if (!c->have_weights) return fail(c, FADE_E_NO_WEIGHTS, "no weights loaded");
  const size_t B = c->d.B;
  void *src_p = nullptr;
  int rc = stage_buf(c, STAGE_JOB, n, &src_p);
  if (rc) return rc;
  uint8_t *src_dev = static_cast<uint8_t *>(src_p);
  hipError_t e = hipSuccess;
  std::vector<uint32_t> lens(B);
  size_t total = 0;
  do {
    if (n && (e = hipMemcpy(src_dev, src_host, n, hipMemcpyHostToDevice)) != hipSuccess) { rc = hip_fail(c, e, "upload"); break; }
    if ((rc = fade_encode_device(c, src_dev, n, 0, 0))) break;
    if ((e = hipMemcpy(lens.data(), c->cb.pos, B * sizeof(uint32_t), hipMemcpyDeviceToHost)) != hipSuccess) { rc = hip_fail(c, e, "lengths"); break; }
    for (size_t b = 0; b < B; ++b) total += lens[b];
    *dst_len = kHeaderBytes + 4 * B + total;
    if (*dst_len > dst_cap) { rc = fail(c, FADE_E_BUFFER_TOO_SMALL, "dst_cap too small"); break; }
    uint8_t *h = dst_host;
    std::memset(h, 0, kHeaderBytes);
    std::memcpy(h, "FADE", 4);
    wr16(h + 4, 1);
    h[6] = (uint8_t)c->cfg.dtype; h[7] = (uint8_t)c->cfg.update_mode;
    wr16(h + 8, (uint32_t)c->d.T); wr16(h + 10, (uint32_t)c->d.D); wr32(h + 12, (uint32_t)c->d.De);
    if (c->d.Dc != c->d.De) wr32(h + 44, (uint32_t)c->d.Dc);  // 0: the cache is as wide as the refiner
    wr16(h + 16, (uint32_t)c->d.dl); wr16(h + 18, (uint32_t)c->d.c); wr16(h + 20, (uint32_t)c->d.k);
    h[22] = (uint8_t)(c->cfg.ablation == 0 ? 5 : c->cfg.ablation);  // the stage that feeds the head (same blob, same hash, another model)
    wr32(h + 24, (uint32_t)B);
    wr32(h + 28, fbits(c->cfg.lr)); wr32(h + 32, fbits(c->cfg.beta1)); wr32(h + 36, fbits(c->cfg.beta2)); wr32(h + 40, fbits(c->cfg.eps));
    wr64(h + 48, n); wr64(h + 56, c->weights_hash);
    for (size_t b = 0; b < B; ++b) wr32(h + kHeaderBytes + 4 * b, lens[b]);
    size_t got = 0;
    rc = fade_payloads(c, lens.data(), dst_host + kHeaderBytes + 4 * B, dst_cap - kHeaderBytes - 4 * B, &got);
  } while (0);
  return rc;
}

int fade_decode(fade_ctx *c, const uint8_t *src_host, size_t src_len, uint8_t *dst_host, size_t dst_cap, size_t *dst_len) {
  if (!c || !src_host || !dst_len) return FADE_E_INVALID_ARG;
  if (!c->have_weights) return fail(c, FADE_E_NO_WEIGHTS, "no weights loaded");
  const size_t B = c->d.B;
  if (src_len < kHeaderBytes + 4 * B) return fail(c, FADE_E_CORRUPT_STREAM, "truncated header");
  const uint8_t *h = src_host;
  if (std::memcmp(h, "FADE", 4) != 0 || rd16(h + 4) != 1) return fail(c, FADE_E_CORRUPT_STREAM, "bad magic or version");
  const bool same = h[6] == c->cfg.dtype && h[7] == c->cfg.update_mode && rd16(h + 8) == c->d.T && rd16(h + 10) == c->d.D &&
                    rd32(h + 12) == c->d.De && rd32(h + 44) == (c->d.Dc != c->d.De ? c->d.Dc : 0) && rd16(h + 16) == c->d.dl && rd16(h + 18) == c->d.c && rd16(h + 20) == c->d.k &&
                    h[22] == (c->cfg.ablation == 0 ? 5u : c->cfg.ablation) &&
                    rd32(h + 24) == B && rd32(h + 28) == fbits(c->cfg.lr) && rd32(h + 32) == fbits(c->cfg.beta1) &&
                    rd32(h + 36) == fbits(c->cfg.beta2) && rd32(h + 40) == fbits(c->cfg.eps);
  if (!same) return fail(c, FADE_E_BAD_CONFIG, "container was written with a different configuration");
  if (rd64(h + 56) != c->weights_hash) return fail(c, FADE_E_WEIGHTS_MISMATCH, "container was written with different weights");
  const uint64_t n64 = rd64(h + 48);
  const size_t n = (size_t)n64;
  *dst_len = n;
  if (n > dst_cap || (!dst_host && n)) return fail(c, FADE_E_BUFFER_TOO_SMALL, "dst_cap too small");
  std::vector<uint32_t> lens(B);
  size_t total = 0;
  const size_t body = src_len - kHeaderBytes - 4 * B;
  for (size_t b = 0; b < B; ++b) {
    lens[b] = rd32(h + kHeaderBytes + 4 * b);
    if (lens[b] > body - total) return fail(c, FADE_E_CORRUPT_STREAM, "payload runs past the end");
    total += lens[b];
  }
  if (total != body) return fail(c, FADE_E_CORRUPT_STREAM, "trailing bytes");
  void *dst_p = nullptr;
  int rc = stage_buf(c, STAGE_JOB, n, &dst_p);
  if (rc) return rc;
  uint8_t *dst_dev = static_cast<uint8_t *>(dst_p);
  hipError_t e = hipSuccess;
  rc = fade_decode_device(c, lens.data(), src_host + kHeaderBytes + 4 * B, total, dst_dev, n, 0, 0);
  if (!rc && n && (e = hipMemcpy(dst_host, dst_dev, n, hipMemcpyDeviceToHost)) != hipSuccess) rc = hip_fail(c, e, "download");
  return rc;
}

int fade_quantize(fade_ctx *c, const float *probs_dev, size_t rows, uint16_t *freq_dev) {
  if (!c || !probs_dev || !freq_dev) return FADE_E_INVALID_ARG;
  HIP_TRY(c, hipMemsetAsync(c->dev_err, 0, sizeof(int), c->stream));
  if (rows) HIP_TRY(c, fade_quantize_rows(probs_dev, rows, freq_dev, c->dev_err, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return check_dev_err(c);
}

// `state`: 8 * n_streams uint32 of device memory for the coder state, or NULL: allocated here and freed on return. With a
// caller-provided state nothing in here allocates (flags are cleared by a kernel, not by a memset node).
static int coder_tables(fade_ctx *c, const uint16_t *freq_dev, uint8_t *sym_dev, size_t n_steps, size_t n_streams, uint8_t *buf_dev,
                        size_t cap, uint32_t *len_dev, int mode, uint32_t *state = nullptr) {
  if (!c || (!freq_dev && n_steps) || (!sym_dev && n_steps) || !buf_dev || !len_dev || n_streams == 0) return FADE_E_INVALID_ARG;
  hipStream_t s = c->stream;
  const bool own_state = state == nullptr;
  hipError_t e = hipSuccess;
  if (own_state) {  // private coder state for n_streams streams
    e = hipMalloc(reinterpret_cast<void **>(&state), 8 * n_streams * sizeof(uint32_t));
    if (e != hipSuccess) return hip_fail(c, e, "hipMalloc(coder state)");
  }
  CoderBufs cb{};
  cb.low = state; cb.high = state + n_streams; cb.pending = state + 2 * n_streams; cb.bitbuf = state + 3 * n_streams;
  cb.nbits = state + 4 * n_streams; cb.pos = state + 5 * n_streams; cb.value = state + 6 * n_streams; cb.bitpos = state + 7 * n_streams;
  cb.out = buf_dev; cb.in = buf_dev; cb.in_len = len_dev; cb.cap = cap; cb.err = c->dev_err;
  int rc = FADE_OK;
  do {
    if (own_state) e = hipMemsetAsync(c->dev_err, 0, sizeof(int), s);
    else e = fade_fill_u32(reinterpret_cast<uint32_t *>(c->dev_err), 0u, 1, s);
    if (e != hipSuccess) { rc = hip_fail(c, e, "clear error flag"); break; }
    if ((e = fade_coder_init(cb, (int)n_streams, mode == CODE_DECODE, s)) != hipSuccess) { rc = hip_fail(c, e, "coder_init"); break; }
    for (size_t i = 0; i < n_steps && rc == FADE_OK; ++i) {
      e = fade_code_tables(freq_dev + i * n_streams * 256, sym_dev + i * n_streams, (int)n_streams, cb, mode, s);
      if (e != hipSuccess) rc = hip_fail(c, e, "code_tables");
    }
    if (rc) break;
    if (mode == CODE_ENCODE) {
      // every stream coded n_steps symbols: terminate all of them when there was anything to code
      if (n_steps && (e = fade_coder_finish(cb, (int)n_streams, 1, (long long)n_streams, s)) != hipSuccess) { rc = hip_fail(c, e, "finish"); break; }
      if ((e = hipMemcpyAsync(len_dev, cb.pos, n_streams * sizeof(uint32_t), hipMemcpyDeviceToDevice, s)) != hipSuccess) { rc = hip_fail(c, e, "copy"); break; }
    }
    if ((e = hipStreamSynchronize(s)) != hipSuccess) { rc = hip_fail(c, e, "sync"); break; }
    rc = check_dev_err(c);
  } while (0);
  if (own_state) (void)hipFree(state);
  return rc;
}

int fade_coder_encode_tables_noalloc(fade_ctx *c, const uint16_t *freq_dev, const uint8_t *sym_dev, size_t n_steps, size_t n_streams,
                                     uint8_t *out_dev, size_t cap, uint32_t *len_dev) {
  if (!c) return FADE_E_INVALID_ARG;
  if (n_streams > FADE_NOALLOC_MAX_STREAMS)
    return fail(c, FADE_E_INVALID_ARG, "fade_coder_encode_tables_noalloc: n_streams exceeds FADE_NOALLOC_MAX_STREAMS (65536)");
  if (!c->scratch_dev) return fail(c, FADE_E_HIP, "scratch array has no device address");
  // coder_init rewrites all eight state words of every stream it will use, so what the previous call left behind in the
  // shared array is never read
  return coder_tables(c, freq_dev, const_cast<uint8_t *>(sym_dev), n_steps, n_streams, out_dev, cap, len_dev, CODE_ENCODE, c->scratch_dev);
}

int fade_coder_encode_tables(fade_ctx *c, const uint16_t *freq_dev, const uint8_t *sym_dev, size_t n_steps, size_t n_streams,
                             uint8_t *out_dev, size_t cap, uint32_t *len_dev) {
  return coder_tables(c, freq_dev, const_cast<uint8_t *>(sym_dev), n_steps, n_streams, out_dev, cap, len_dev, CODE_ENCODE);
}

int fade_coder_decode_tables(fade_ctx *c, const uint16_t *freq_dev, size_t n_steps, size_t n_streams, const uint8_t *in_dev, size_t cap,
                             const uint32_t *len_dev, uint8_t *sym_dev) {
  return coder_tables(c, freq_dev, sym_dev, n_steps, n_streams, const_cast<uint8_t *>(in_dev), cap, const_cast<uint32_t *>(len_dev),
                      CODE_DECODE);
}

size_t fade_tap(fade_ctx *c, int which, float *out_host, size_t cap_floats) {
  if (!c) return 0;
  const Dims &d = c->d;
  const void *src = nullptr;
  size_t width = 0;
  bool is_f32 = false;
  switch (which) {
    case FADE_TAP_X: src = c->X; width = d.Dh; break;
    case FADE_TAP_CACHE: src = c->M; width = d.Dc; break;
    case FADE_TAP_H_GLOBAL: src = c->Hg; width = d.Dh; break;
    case FADE_TAP_H_LOCAL: src = c->Hl; width = d.Dh; break;
    case FADE_TAP_ALPHA: src = c->alpha; width = d.Dh; break;
    case FADE_TAP_H_MIX: src = c->Hmix; width = d.Dh; break;
    case FADE_TAP_Y_DOWN: src = c->y; width = d.dl; is_f32 = true; break;
    case FADE_TAP_Z_BMM: src = c->z; width = d.dl; break;
    case FADE_TAP_H_A: src = c->Ha; width = d.Dh; break;
    case FADE_TAP_H_COARSE: src = c->Hc; width = d.Dh; break;
    case FADE_TAP_H_EXPAND: src = c->Hexp; width = d.De; break;
    case FADE_TAP_LOGITS: src = c->logits; width = 256; is_f32 = true; break;
    default: return 0;  // H_out is never materialised (it lives in the head product's operand load); probs are an output
  }
  if (!src) return 0;
  if (!out_host) return width;
  const size_t n = d.B * width;
  if (cap_floats < n) return 0;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return 0;
  if (is_f32 || !c->bf16) {
    if (hipMemcpy(out_host, src, n * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return 0;
  } else {
    std::vector<uint16_t> tmp(n);
    if (hipMemcpy(tmp.data(), src, n * 2, hipMemcpyDeviceToHost) != hipSuccess) return 0;
    for (size_t i = 0; i < n; ++i) { uint32_t u = (uint32_t)tmp[i] << 16; std::memcpy(&out_host[i], &u, 4); }
  }
  return width;
}

// device array (device layout) -> canonical blob on the host
static int read_blob(fade_ctx *c, const float *dev, void *blob_host) {
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  std::vector<float> tmp(c->lay.off[P_COUNT]);
  HIP_TRY(c, hipMemcpy(tmp.data(), dev, tmp.size() * sizeof(float), hipMemcpyDeviceToHost));
  for (int t = 0; t < P_COUNT; ++t)
    std::memcpy(static_cast<float *>(blob_host) + c->blob.off[t], tmp.data() + c->lay.off[t], c->blob.len[t] * sizeof(float));
  return FADE_OK;
}

int fade_get_weights(fade_ctx *c, void *blob_host, size_t nbytes) {
  if (!c || !blob_host || nbytes != c->blob.off[P_COUNT] * sizeof(float)) return FADE_E_INVALID_ARG;
  return read_blob(c, c->master, blob_host);
}

int fade_debug_grad(fade_ctx *c, void *blob_host, size_t nbytes) {
  if (!c || !blob_host || nbytes != c->blob.off[P_COUNT] * sizeof(float)) return FADE_E_INVALID_ARG;
  if (!c->online) return fail(c, FADE_E_BAD_CONFIG, "context is frozen");
  return read_blob(c, c->grad, blob_host);
}

int fade_profile(fade_ctx *c, int enable) {
  if (!c) return FADE_E_INVALID_ARG;
  c->profiling = enable != 0;
  c->prof_names.clear(); c->prof_ms.clear(); c->prof_n.clear();
  return FADE_OK;
}

int fade_profile_read(fade_ctx *c, const char **names, double *ms, uint64_t *launches, int cap) {
  if (!c) return 0;
  int n = 0;
  for (size_t i = 0; i < c->prof_names.size() && n < cap; ++i, ++n) {
    if (names) names[n] = c->prof_names[i].c_str();
    if (ms) ms[n] = c->prof_ms[i];
    if (launches) launches[n] = c->prof_n[i];
  }
  return n;
}

const char *fade_last_error(const fade_ctx *c) { return c ? c->err.c_str() : "null context"; }

}  // extern "C"
