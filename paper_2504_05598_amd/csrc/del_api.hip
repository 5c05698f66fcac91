// Host side of the library: context, weight loading, prefill, the round driver and the DEL
// policy (statistics + Token-per-Layer selection).  See include/del.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/del.h"
#include "del_kernels.h"

using namespace del;

namespace {

// ---- DEL policy (Sections 4.1-4.3) -----------------------------------------------------
// Decayed sums are kept as running values: S <- omega * S + a, which equals the paper's
// S(a) = sum_i omega^(r-i-1) a[i] (newest entry has weight 1).
struct Policy {
  int L = 0, d_max = 0;
  double omega = 0.95;
  std::vector<double> Sc;  // [L+1]
  double Sn = 0.0;
  std::vector<double> alpha;
  std::vector<double> St, Sf, tau;  // decayed confidence sums (matched / mismatched), thresholds
  int next_E = 1, next_gamma = 0;

  void reset(int L_, int d_max_, double omega_) {
    L = L_; d_max = d_max_; omega = omega_;
    Sc.assign(L + 1, 0.0);
    alpha.assign(L + 1, 0.0);
    St.assign(L + 1, 0.0); Sf.assign(L + 1, 0.0); tau.assign(L + 1, 0.0);
    Sn = 0.0; next_E = 1; next_gamma = 0;
  }
  // c, tcs, fcs indexed by layer number 1..L
  void update(const int* c, int n, const double* tcs, const double* fcs) {
    for (int l = 1; l <= L; ++l) {
      Sc[l] = omega * Sc[l] + (double)c[l];
      St[l] = omega * St[l] + tcs[l];
      Sf[l] = omega * Sf[l] + fcs[l];
    }
    Sn = omega * Sn + (double)n;
    select();
  }
  // Dynamic threshold (Section 4.4, Eq. 3): midpoint of the decayed mean confidence of the
  // matched and of the mismatched shadow tokens; mismatches = valid positions - matches; a ratio
  // with a zero denominator counts as 0.
  void thresholds() {
    for (int l = 1; l <= L; ++l) {
      const double sm = Sn - Sc[l];
      const double a = Sc[l] > 0.0 ? St[l] / Sc[l] : 0.0;
      const double b = sm > 0.0 ? Sf[l] / sm : 0.0;
      tau[l] = 0.5 * (a + b);
    }
  }
  // alpha_l = S(c^l)/S(n) (Eq. 2 with n_r = u_r + 1 valid positions);
  // (E, gamma) = argmax_{l in [1,L), d in [0,d_max]} TPL(l, d) (Eq. 1, Section 4.3).
  // TPL numerator as the sum of alpha^i, i = 0..d; first maximum in l-major order wins.
  void select() {
    for (int l = 1; l <= L; ++l) alpha[l] = Sn > 0.0 ? Sc[l] / Sn : 0.0;
    double best = -1.0;
    int bl = 1, bd = 0;
    for (int l = 1; l < L; ++l) {
      const double a = alpha[l];
      double num = 0.0, pw = 1.0;
      for (int d = 0; d <= d_max; ++d) {
        num += pw;
        pw *= a;
        const double v = num / (double)(d * l + L);
        if (v > best) { best = v; bl = l; bd = d; }
      }
    }
    next_E = bl; next_gamma = bd;
    thresholds();
  }
};

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace

struct del_ctx {
  del_config cfg{};
  hipStream_t stream = nullptr;
  std::string err;
  // shape
  int L = 0, d = 0, nq = 0, nkv = 0, hd = 0, f = 0, V = 0, wd = 0, esize = 0, KPL = 0, TK = 0;
  int qdim = 0, kvdim = 0, dpad = 0, qpad = 0, fpad = 0;
  int KTd = 0, KTq = 0, KTf = 0, NBqkv = 0, NBd = 0, NBgu = 0, NBv = 0;
  int maxrows = 0, Tcap = 0;
  int prows = 0;    // token rows of a wide prefill pass (0: prefill runs in 16-row passes)
  int hrows = 0;    // rows per layer of the hidden buffer and of the per-row work buffers
  float* rowscale_w = nullptr;   // [hrows] RMS scales of a wide pass
  char* vct = nullptr; int TcapT = 0; size_t vct_layer_bytes = 0;   // feature-major copy of the values for the
                                                                     // prefill's matrix-core attention (0: off)
  // device memory
  char* arena = nullptr;
  size_t off_qkv = 0, off_o = 0, off_gu = 0, off_dn = 0, layer_stride = 0, arena_bytes = 0;
  char* embed_t = nullptr; char* head_t = nullptr; size_t vocab_bytes = 0;
  float* gains = nullptr;  // [L][2][gpad], then final [gpad]
  int gpad = 0;
  char* kc = nullptr; char* vc = nullptr; size_t kv_layer_bytes = 0;
  float2* rope = nullptr;
  float* hid = nullptr; float* q = nullptr; float* attn = nullptr; float* act = nullptr;
  uint16_t* xs_layer = nullptr; uint16_t* xs_shadow = nullptr; float* rowscale = nullptr;
  uint16_t* xs_h = nullptr; uint16_t* xs_attn = nullptr; uint16_t* xs_h1 = nullptr; uint16_t* xs_act = nullptr;
  float* ssq_h = nullptr; float* ssq_h1 = nullptr;
  float* PM = nullptr; float* PL = nullptr; float* PA = nullptr; int nch_max = 0, attn_ct = 64, attn_S = 0, attn_dec_rows = 16;
  int attn_direct_rows = 0;   // passes of at least this many rows (> 1): one context split per row, no merge kernel   // attn_S > 0: register decode kernel with S splits
  bool verify_flash = true;   // passes of 2..16 rows: attention on the matrix cores, split over the context
  int verify_flash_waves = 1024;   // waves (splits x query heads) that kernel aims for
  float* pval = nullptr; int* pidx = nullptr; float* psum = nullptr;
  float* conf_dev = nullptr;   // [Rmax] shadow confidences, then [d_max+1] draft confidences (inside the result block)
  float* conf_host = nullptr;  // pinned mirror (inside the host result block)
  int* step_host = nullptr;    // pinned: (token id, confidence bits) of the last draft step; bytes 8..15: the
                               // (sequence number, confidence) word a draft step's head writes for the polling host
  unsigned note_seq = 0;
  int* state = nullptr; int* draft_ids = nullptr; int* shadow_ids = nullptr; int* result = nullptr;
  int* ids_dev = nullptr; int* result_host = nullptr;
  size_t res_ints = 0, res_words = 0;   // ints of a round's result block / all its 32-bit words (ints, then confidences)
  float* logits_dbg = nullptr; float* sink = nullptr;
  // speculative sampling: logits and fixed-point weights of the draft rows [0, d_max] and of the
  // target rows [d_max+1, 2*d_max+1], one SampRow each, and the round's uniform numbers
  float* slog = nullptr; unsigned long long* swf = nullptr; SampRow* srows = nullptr; float* unif_dev = nullptr;
  int64_t sld = 0;   // row stride of slog and swf, in elements
  void* stage = nullptr; size_t stage_bytes = 0;
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  // host state
  std::vector<uint8_t> loaded;  // [(L+1)*12]
  int phase = 0;                // 0 created, 1 prefilled
  int T = 0, pending = -1, rounds = 0;
  int last_rows = 0;            // valid rows of hid from the last pass
  Policy pol;
  int last_E = 0, last_gamma = 0, last_u = 0, last_n = 0;
  std::vector<int> last_c, last_shadow, last_draft;
  std::vector<float> last_conf, last_draft_conf;   // like last_shadow / last_draft
  int last_stopped = 0;
  float t_draft = 0, t_verify = 0, t_shadow = 0;
  int target_waves = 3072;
  int rows_form = 0;          // one-row GEMV: 1 = one row block per work-group for every matrix (DEL_ROWS_FORM)
  int wide_form = 0;          // prefill GEMMs: 1 = the two-stage form for every matrix (DEL_WIDE_FORM)
  int head_form = 4;          // shadow-head kernel: 4 = register-blocked, 1 = one row block per wave (DEL_HEAD_FORM)
  // Optional (DEL_GRAPHS=1): the segments of a round are captured once per (kind, E, gamma) into HIP
  // graphs and replayed; positions and token ids live in device memory, so a graph depends on
  // nothing else.  Off by default: on this GPU the kernels of a round already run back to back
  // from plain launches, and replaying graphs measured no faster.
  bool use_graphs = false;
  bool own_stream = false;
  std::map<std::tuple<int, int, int>, hipGraphExec_t> graphs;
  // per-kernel profiling (off by default)
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;     // pairs
  std::vector<int> prof_cls;           // class index of each recorded pair
  int prof_used = 0;                   // pairs recorded since the last collect
  std::vector<del_prof_entry> prof;

  del_status fail(hipError_t e, const char* what) {
    err = std::string(what) + ": " + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? DEL_E_NOMEM : DEL_E_DEVICE;
  }
  float* hid_row(int layer, int row) const { return hid + ((size_t)layer * hrows + row) * dpad; }
  float* gain_attn(int li) const { return gains + ((size_t)li * 2) * gpad; }
  float* gain_ffn(int li) const { return gains + ((size_t)li * 2 + 1) * gpad; }
  float* gain_final() const { return gains + (size_t)L * 2 * gpad; }
  bool all_loaded() const {
    for (int l = -1; l < L; ++l)
      for (int k = 0; k < 12; ++k) {
        const bool global = k <= DEL_T_FINAL_NORM;
        if ((l == -1) != global) continue;
        if (k == DEL_T_LM_HEAD && cfg.tied_embeddings) continue;
        if (!loaded[(size_t)(l + 1) * 12 + k]) return false;
      }
    return true;
  }
  // waves per 16-row block: the whole k range of a block is split over the waves of its
  // work-group; 16 waves for the matrices with few blocks, 8 when there are many
  int pick_waves(int NB, int KT) const {
    int w = NB * 8 >= 2 * target_waves ? 8 : 16;
    while (w > 1 && KT < 2 * w) w >>= 1;
    return w;
  }
};

#define HIPCHK(call)                                              \
  do {                                                            \
    hipError_t e_ = (call);                                       \
    if (e_ != hipSuccess) return ctx->fail(e_, #call);            \
  } while (0)

namespace {

template <typename T>
hipError_t dmalloc(T** p, size_t bytes) { return hipMalloc((void**)p, bytes ? bytes : 16); }

int prof_begin(del_ctx* ctx, int flavour, int epi, int rows, int64_t bytes) {
  if (!ctx->prof_on) return -1;
  int cls = -1;
  for (size_t i = 0; i < ctx->prof.size(); ++i)
    if (ctx->prof[i].flavour == flavour && ctx->prof[i].epilogue == epi && ctx->prof[i].rows == rows &&
        ctx->prof[i].weight_bytes == bytes)
      cls = (int)i;
  if (cls < 0) {
    del_prof_entry e{flavour, epi, rows, 0, 0.0, bytes};
    ctx->prof.push_back(e);
    cls = (int)ctx->prof.size() - 1;
  }
  ctx->prof[cls].weight_bytes = bytes;
  const int pair = ctx->prof_used;
  if ((size_t)(2 * pair + 1) >= ctx->prof_ev.size()) {
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -1;
    ctx->prof_ev.push_back(a);
    ctx->prof_ev.push_back(b);
    ctx->prof_cls.push_back(cls);
  }
  ctx->prof_cls[pair] = cls;
  return pair;
}

// the launch itself stamps the pair with the kernel's own start and stop times
void prof_end(del_ctx* ctx, int pair) {
  if (pair >= 0) ctx->prof_used = pair + 1;
}

// after a stream synchronisation: fold the recorded pairs into the class totals
void prof_collect(del_ctx* ctx) {
  for (int i = 0; i < ctx->prof_used; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]) == hipSuccess) {
      ctx->prof[ctx->prof_cls[i]].launches += 1;
      ctx->prof[ctx->prof_cls[i]].total_ms += ms;
    }
  }
  ctx->prof_used = 0;
}

// One GEMM of the path: on the matrix cores (split the fp32 rows first) or as vector-ALU
// groups of 8/4/2/1 rows.
constexpr int WIDE_S = 8;   // most context splits (partials per row and head) of a wide pass's attention

del_status gemm(del_ctx* ctx, GemmP p, int epi, int m, bool mfma) {
  const int waves = ctx->pick_waves(p.NB, p.KT);
  const int64_t wbytes = (int64_t)p.NB * p.KT * 1024;
  if (mfma) {
    // blocks of up to 16 token rows, each split into tiles and multiplied on its own
    for (int off = 0; off < m; off += 16) {
      const int mb = std::min(16, m - off);
      GemmP q = p;
      q.X = p.X + (size_t)off * p.ldx;
      if (q.Y) q.Y = p.Y + (size_t)off * p.ldy;
      HIPCHK(launch_prep_split(q.X, mb, mb, 0, q.ldx, q.K, q.KT, q.gain, q.rms, q.eps, ctx->xs_layer, ctx->rowscale,
                               ctx->stream));
      q.Xs = ctx->xs_layer;
      q.rowscale = q.rms ? ctx->rowscale : nullptr;
      q.M = mb;
      const int pr = prof_begin(ctx, gemm_mfma_rows_applies(q, epi, 1) ? 5 : 1, epi, mb, wbytes);
      if (pr >= 0) { q.ev_start = ctx->prof_ev[2 * pr]; q.ev_stop = ctx->prof_ev[2 * pr + 1]; }
      HIPCHK(launch_gemm_mfma(q, epi, waves, 1, ctx->stream));
      prof_end(ctx, pr);
    }
    return DEL_OK;
  }
  int off = 0;
  while (off < m) {
    int g = p.wdtype == DEL_DTYPE_BF16 ? 2 : 8;   // 16-bit weights unpack to twice the registers per tile: two rows at most
    while (g > m - off) g >>= 1;
    GemmP q = p;
    q.M = g;
    q.X = p.X + (size_t)off * p.ldx;
    if (q.Y) q.Y = p.Y + (size_t)off * p.ldy;
    if (q.R) q.R = p.R + (size_t)off * p.ldr;
    if (q.Q) q.Q = p.Q + (size_t)off * p.ldq;
    if (q.ACT) q.ACT = p.ACT + (size_t)off * p.ldact;
    q.row_off = p.row_off + off;
    q.prow0 = p.prow0 + off;
    const int pr = prof_begin(ctx, gemv_rows_applies(q) ? 4 : 0, epi, g, wbytes);
    if (pr >= 0) { q.ev_start = ctx->prof_ev[2 * pr]; q.ev_stop = ctx->prof_ev[2 * pr + 1]; }
    HIPCHK(launch_gemm_valu(q, epi, waves, ctx->stream));
    prof_end(ctx, pr);
    off += g;
  }
  return DEL_OK;
}

GemmP base_gemm(const del_ctx* ctx) {
  GemmP p;
  memset(&p, 0, sizeof(p));
  p.wdtype = ctx->wd;
  p.eps = ctx->cfg.rms_eps;
  p.rows_form = ctx->rows_form;
  // between rounds the host's T is the device's; not while a prompt is being absorbed, and not under graph
  // replay (a captured launch would keep the value it was captured with)
  p.ctx_len1 = (ctx->phase == 1 && !ctx->use_graphs) ? ctx->T + 1 : 0;
  return p;
}

// Matrix-core GEMM whose input split tiles are already in p.Xs.
del_status gemm_mf(del_ctx* ctx, GemmP p, int epi, int m) {
  const int waves = ctx->pick_waves(p.NB, p.KT);
  p.M = m;
  const int pr = prof_begin(ctx, gemm_mfma_rows_applies(p, epi, 1) ? 5 : 1, epi, m, (int64_t)p.NB * p.KT * 1024);
  if (pr >= 0) { p.ev_start = ctx->prof_ev[2 * pr]; p.ev_stop = ctx->prof_ev[2 * pr + 1]; }
  HIPCHK(launch_gemm_mfma(p, epi, waves, 1, ctx->stream));
  prof_end(ctx, pr);
  return DEL_OK;
}

// Transformer_l on rows [row0, row0+m) of the hidden buffer; positions T + row0 + i.
// `chained`: on the matrix-core path the previous layer of this pass has already left the
// split tiles of this layer's (gained) input in xs_h and their sums of squares in ssq_h.
del_status run_layer(del_ctx* ctx, int l, int row0, int m, bool chained) {
  const int li = l - 1;
  // more than 16 rows in a round (gamma > 15) take the wide path (see layer_pass) or, failing that, the vector path
  const bool mf = ctx->cfg.use_mfma && ctx->wd == DEL_DTYPE_BF16 && m > 1 && m <= 16;
  char* base = ctx->arena + (size_t)li * ctx->layer_stride;
  float* hin = ctx->hid_row(l - 1, row0);
  float* hout = ctx->hid_row(l, row0);
  del_status st;
  // 1. RMSNorm + fused QKV + rotary + KV append
  GemmP p = base_gemm(ctx);
  p.Wt = base + ctx->off_qkv; p.NB = ctx->NBqkv; p.KT = ctx->KTd; p.N = ctx->NBqkv * 16; p.K = ctx->d;
  p.X = hin; p.ldx = ctx->dpad; p.gain = ctx->gain_attn(li); p.rms = 1;
  p.Q = ctx->q; p.ldq = ctx->qpad;
  p.Kc = ctx->kc + (size_t)li * ctx->kv_layer_bytes; p.Vc = ctx->vc + (size_t)li * ctx->kv_layer_bytes;
  p.n_q = ctx->nq; p.n_kv = ctx->nkv; p.hd = ctx->hd; p.Tcap = ctx->Tcap;
  p.state = ctx->state; p.row_off = row0; p.rope = ctx->rope;
  void* Kc = p.Kc; void* Vc = p.Vc;
  // the feature-major copy of the values is kept by every pass, so that the matrix-core attention
  // kernels can be used at any point of a generation
  void* VcT = ctx->vct ? ctx->vct + (size_t)li * ctx->vct_layer_bytes : nullptr;
  p.VcT = VcT; p.TcapT = ctx->TcapT;
  if (mf) {
    p.Xs = ctx->xs_h;
    if (chained) {
      p.ssq_in = ctx->ssq_h; p.ssq_nb = ctx->NBd;
    } else {
      HIPCHK(launch_prep_split(hin, m, m, 0, ctx->dpad, ctx->d, ctx->KTd, p.gain, 1, p.eps, ctx->xs_h, ctx->rowscale,
                               ctx->stream));
      p.rowscale = ctx->rowscale;
    }
    st = gemm_mf(ctx, p, EPI_QKV, m);
  } else {
    st = gemm(ctx, p, EPI_QKV, m, false);
  }
  if (st != DEL_OK) return st;
  // 2. attention over the cache (split over the context) + combine
  AttnP a;
  memset(&a, 0, sizeof(a));
  a.Q = ctx->q; a.ldq = ctx->qpad; a.Kc = Kc; a.Vc = Vc; a.kvdtype = ctx->wd;
  a.n_q = ctx->nq; a.n_kv = ctx->nkv; a.hd = ctx->hd; a.Tcap = ctx->Tcap; a.m = m;
  a.state = ctx->state; a.row_off = row0;
  a.ctx_len1 = (ctx->phase == 1 && !ctx->use_graphs) ? ctx->T + 1 : 0;
  a.PM = ctx->PM; a.PL = ctx->PL; a.PA = ctx->PA; a.nch_max = ctx->nch_max; a.ct = ctx->attn_ct;
  a.O = ctx->attn; a.ldo = ctx->qpad;
  a.XsOut = mf ? ctx->xs_attn : nullptr;
  // few token rows: the register kernel, one work-group per (split, kv head, row); a single row's
  // partials are merged by the O projection itself, several rows' by the merge kernel
  const bool dec_any = ctx->attn_S > 0 && m <= ctx->attn_dec_rows;
  const bool dec = dec_any && m == 1;
  if (mf && VcT && ctx->verify_flash && row0 == 0) {
    // several rows (verify): on the matrix cores, the cache read once for all rows, split over the
    // context so that splits x query heads waves are in flight; then the merge
    // the split plan depends on the cache capacity only, never on the current length: a round's launch
    // sequence (and its rounding) is then a function of (E, gamma) alone; spans past the context are empty
    int rps = ceil_div((int64_t)ctx->Tcap * ctx->nq, ctx->verify_flash_waves);
    rps = std::max(32, ceil_div(rps, 32) * 32);
    while (ceil_div(ctx->Tcap, rps) > ctx->nch_max) rps += 32;
    const int S = ceil_div(ctx->Tcap, rps);
    a.VcT = VcT; a.TcapT = ctx->TcapT;
    HIPCHK(launch_attention_flash_split(a, S, rps, ctx->stream));
    a.nsplit = S; a.rps = rps;
    HIPCHK(launch_attention_merge(a, ctx->stream));
  } else if (dec_any && m > 1 && ctx->attn_direct_rows > 0 && m >= ctx->attn_direct_rows) {
    a.nsplit = -1;   // one split per row: the kernel writes the output rows and their tiles itself
    HIPCHK(launch_attention_decode(a, 1, ctx->stream));
  } else if (dec_any) {
    HIPCHK(launch_attention_decode(a, ctx->attn_S, ctx->stream));
    if (m > 1) {
      a.nsplit = ctx->attn_S;
      HIPCHK(launch_attention_merge(a, ctx->stream));
    }
  } else {
    HIPCHK(launch_attention(a, ctx->stream));
  }
  // 3. output projection + residual
  p = base_gemm(ctx);
  p.Wt = base + ctx->off_o; p.NB = ctx->NBd; p.KT = ctx->KTq; p.N = ctx->d; p.K = ctx->qdim;
  p.X = ctx->attn; p.ldx = ctx->qpad;
  p.R = hin; p.ldr = ctx->dpad; p.Y = hout; p.ldy = ctx->dpad;
  if (dec) {
    p.att_PM = ctx->PM; p.att_PL = ctx->PL; p.att_PA = ctx->PA;
    p.att_S = ctx->attn_S; p.att_stride = ctx->nch_max; p.att_hd = ctx->hd;
  }
  if (mf) {
    p.Xs = ctx->xs_attn;
    p.XsOut = ctx->xs_h1; p.gain_out = ctx->gain_ffn(li); p.ssq_out = ctx->ssq_h1;
    st = gemm_mf(ctx, p, EPI_RESID, m);
  } else {
    st = gemm(ctx, p, EPI_RESID, m, false);
  }
  if (st != DEL_OK) return st;
  // 4. RMSNorm + fused gate/up + SiLU(gate) * up
  p = base_gemm(ctx);
  p.Wt = base + ctx->off_gu; p.NB = ctx->NBgu; p.KT = ctx->KTd; p.N = ctx->NBgu * 16; p.K = ctx->d;
  p.X = hout; p.ldx = ctx->dpad; p.gain = ctx->gain_ffn(li); p.rms = 1;
  p.ACT = ctx->act; p.ldact = ctx->fpad; p.d_ffn = ctx->f;
  if (mf) {
    p.Xs = ctx->xs_h1; p.ssq_in = ctx->ssq_h1; p.ssq_nb = ctx->NBd;
    p.XsOut = ctx->xs_act;
    st = gemm_mf(ctx, p, EPI_SWIGLU, m);
  } else {
    st = gemm(ctx, p, EPI_SWIGLU, m, false);
  }
  if (st != DEL_OK) return st;
  // 5. down projection + residual (in place: this row now holds h^l)
  p = base_gemm(ctx);
  p.Wt = base + ctx->off_dn; p.NB = ctx->NBd; p.KT = ctx->KTf; p.N = ctx->d; p.K = ctx->f;
  p.X = ctx->act; p.ldx = ctx->fpad;
  p.R = hout; p.ldr = ctx->dpad; p.Y = hout; p.ldy = ctx->dpad;
  if (mf) {
    p.Xs = ctx->xs_act;
    if (l < ctx->L) {   // leave the next layer's gained input behind as split tiles
      p.XsOut = ctx->xs_h; p.gain_out = ctx->gain_attn(li + 1); p.ssq_out = ctx->ssq_h;
    }
    return gemm_mf(ctx, p, EPI_RESID, m);
  }
  return gemm(ctx, p, EPI_RESID, m, false);
}

// Transformer_l on rows [0, m) of the hidden buffer in one wide pass (prefill): the same five steps
// as run_layer on the wide GEMM, every GEMM leaving the next one's split tiles behind.
// `chained`: the previous layer's down projection has left this layer's input tiles in xs_h and
// their sums of squares in ssq_h.
del_status run_layer_wide(del_ctx* ctx, int l, int m, bool chained) {
  const int li = l - 1;
  hipStream_t s = ctx->stream;
  char* base = ctx->arena + (size_t)li * ctx->layer_stride;
  float* hin = ctx->hid_row(l - 1, 0);
  float* hout = ctx->hid_row(l, 0);
  auto wide = [&](GemmP& p, int epi) -> del_status {
    p.M = m;
    p.wide_form = ctx->wide_form;
    const int pr = prof_begin(ctx, 3, epi, m, (int64_t)p.NB * p.KT * 1024);
    if (pr >= 0) { p.ev_start = ctx->prof_ev[2 * pr]; p.ev_stop = ctx->prof_ev[2 * pr + 1]; }
    HIPCHK(launch_gemm_wide(p, epi, s));
    prof_end(ctx, pr);
    return DEL_OK;
  };
  del_status st;
  // 1. RMSNorm + fused QKV + rotary + KV append
  GemmP p = base_gemm(ctx);
  p.Wt = base + ctx->off_qkv; p.NB = ctx->NBqkv; p.KT = ctx->KTd; p.N = ctx->NBqkv * 16; p.K = ctx->d;
  p.Q = ctx->q; p.ldq = ctx->qpad;
  p.Kc = ctx->kc + (size_t)li * ctx->kv_layer_bytes; p.Vc = ctx->vc + (size_t)li * ctx->kv_layer_bytes;
  p.n_q = ctx->nq; p.n_kv = ctx->nkv; p.hd = ctx->hd; p.Tcap = ctx->Tcap;
  p.state = ctx->state; p.row_off = 0; p.rope = ctx->rope;
  void* Kc = p.Kc; void* Vc = p.Vc;
  void* VcT = ctx->vct ? ctx->vct + (size_t)li * ctx->vct_layer_bytes : nullptr;
  p.VcT = VcT; p.TcapT = ctx->TcapT;
  if (chained)
    HIPCHK(launch_rowscale(ctx->ssq_h, ctx->NBd, m, ctx->d, ctx->cfg.rms_eps, ctx->rowscale_w, s));
  else
    HIPCHK(launch_prep_split(hin, m, m, 0, ctx->dpad, ctx->d, ctx->KTd, ctx->gain_attn(li), 1, ctx->cfg.rms_eps, ctx->xs_h,
                             ctx->rowscale_w, s));
  p.Xs = ctx->xs_h; p.rowscale = ctx->rowscale_w;
  if ((st = wide(p, EPI_QKV)) != DEL_OK) return st;
  // 2. causal attention: groups of token rows share the cache reads; then the merge
  AttnP a;
  memset(&a, 0, sizeof(a));
  a.Q = ctx->q; a.ldq = ctx->qpad; a.Kc = Kc; a.Vc = Vc; a.kvdtype = ctx->wd;
  a.n_q = ctx->nq; a.n_kv = ctx->nkv; a.hd = ctx->hd; a.Tcap = ctx->Tcap; a.m = m;
  a.state = ctx->state; a.row_off = 0;
  a.PM = ctx->PM; a.PL = ctx->PL; a.PA = ctx->PA; a.nch_max = WIDE_S; a.ct = ctx->attn_ct;
  a.O = ctx->attn; a.ldo = ctx->qpad;
  a.XsOut = ctx->xs_attn; a.xs_cb_stride = (long long)ctx->KTq * 1024;
  if (VcT) {   // on the matrix cores, straight to the output rows and their tiles
    a.VcT = VcT; a.TcapT = ctx->TcapT;
    HIPCHK(launch_attention_flash(a, s));
  } else {
    const int groups = ctx->nkv * ceil_div(m, 8);
    const int S = std::max(1, std::min(WIDE_S, ceil_div(512, groups)));
    HIPCHK(launch_attention_decode(a, S, s, 8));
    a.nsplit = S;
    HIPCHK(launch_attention_merge(a, s));
  }
  // 3. output projection + residual; leaves the FFN's input tiles
  p = base_gemm(ctx);
  p.Wt = base + ctx->off_o; p.NB = ctx->NBd; p.KT = ctx->KTq; p.N = ctx->d; p.K = ctx->qdim;
  p.R = hin; p.ldr = ctx->dpad; p.Y = hout; p.ldy = ctx->dpad;
  p.Xs = ctx->xs_attn;
  p.XsOut = ctx->xs_h1; p.xs_out_cb_stride = (long long)ctx->KTd * 1024; p.gain_out = ctx->gain_ffn(li);
  p.ssq_out = ctx->ssq_h1;
  if ((st = wide(p, EPI_RESID)) != DEL_OK) return st;
  // 4. RMSNorm + fused gate/up + SiLU(gate) * up
  HIPCHK(launch_rowscale(ctx->ssq_h1, ctx->NBd, m, ctx->d, ctx->cfg.rms_eps, ctx->rowscale_w, s));
  p = base_gemm(ctx);
  p.Wt = base + ctx->off_gu; p.NB = ctx->NBgu; p.KT = ctx->KTd; p.N = ctx->NBgu * 16; p.K = ctx->d;
  p.ACT = ctx->act; p.ldact = ctx->fpad; p.d_ffn = ctx->f;
  p.Xs = ctx->xs_h1; p.rowscale = ctx->rowscale_w;
  p.XsOut = ctx->xs_act; p.xs_out_cb_stride = (long long)ctx->KTf * 1024;
  if ((st = wide(p, EPI_SWIGLU)) != DEL_OK) return st;
  // 5. down projection + residual (in place); leaves the next layer's input tiles
  p = base_gemm(ctx);
  p.Wt = base + ctx->off_dn; p.NB = ctx->NBd; p.KT = ctx->KTf; p.N = ctx->d; p.K = ctx->f;
  p.R = hout; p.ldr = ctx->dpad; p.Y = hout; p.ldy = ctx->dpad;
  p.Xs = ctx->xs_act;
  if (l < ctx->L) {
    p.XsOut = ctx->xs_h; p.xs_out_cb_stride = (long long)ctx->KTd * 1024; p.gain_out = ctx->gain_attn(li + 1);
    p.ssq_out = ctx->ssq_h;
  }
  return wide(p, EPI_RESID);
}

// Transformer_l on rows [0, m) of a round's verify pass: up to 16 rows on the skinny matrix-core GEMMs
// (or the vector path); more (gamma > 15) as one wide pass where the context has one, else on the vector path.
del_status layer_pass(del_ctx* ctx, int l, int m, bool chained) {
  if (m > 16 && ctx->prows >= m && ctx->cfg.use_mfma && ctx->wd == DEL_DTYPE_BF16) return run_layer_wide(ctx, l, m, chained);
  return run_layer(ctx, l, 0, m, chained);
}

GemmP head_gemm(const del_ctx* ctx) {
  GemmP p = base_gemm(ctx);
  p.Wt = ctx->head_t; p.NB = ctx->NBv; p.KT = ctx->KTd; p.N = ctx->V; p.K = ctx->d;
  p.ldx = ctx->dpad; p.gain = ctx->gain_final(); p.rms = 1;
  p.pval = ctx->pval; p.pidx = ctx->pidx; p.psum = ctx->psum;
  return p;
}

// Final norm + LM head + arg-max on one row of the hidden buffer (the draft's head).
// Also the token's confidence (its soft-max probability, Section 4.4) into out_conf.
// emb_next (optional): the token's embedding row goes there too (the next draft step's layer-0 input).
del_status head_one(del_ctx* ctx, int layer, int row, int* out_id, float* out_conf, float* emb_next = nullptr,
                    unsigned long long* note = nullptr, unsigned seq = 0) {
  GemmP p = head_gemm(ctx);
  p.X = ctx->hid_row(layer, row);
  del_status st = gemm(ctx, p, EPI_ARGMAX, 1, false);
  if (st != DEL_OK) return st;
  HIPCHK(launch_argmax_finish(ctx->pval, ctx->pidx, ctx->psum, 1, ctx->NBv, out_id, out_conf, ctx->stream,
                              ctx->embed_t, ctx->wd, ctx->KTd, ctx->V, emb_next, ctx->d, note, seq));
  return DEL_OK;
}

// Shadow tokens (Section 4.2): final norm + LM head + arg-max of rows 0..m-1 of every layer
// 1..L, into shadow_ids[(l-1)*m + i], and their confidences into conf_dev[(l-1)*m + i].
del_status shadow_head(del_ctx* ctx, int m, int row0 = 0) {
  const int R = ctx->L * m;
  const bool mf = ctx->cfg.use_mfma && ctx->wd == DEL_DTYPE_BF16;
  int nparts = ctx->NBv;
  if (mf) {
    HIPCHK(launch_prep_split(ctx->hid_row(1, row0), R, m, (int64_t)ctx->hrows * ctx->dpad, ctx->dpad, ctx->d,
                             ctx->KTd, ctx->gain_final(), 1, ctx->cfg.rms_eps, ctx->xs_shadow, ctx->rowscale,
                             ctx->stream));
    // the head is streamed once per group of column blocks: 8 blocks of 16 rows in the register-blocked form, 16 otherwise
    const int cbs = (R + 15) / 16, per_pass = (ctx->head_form == 4 && ctx->KTd % 4 == 0) ? 8 : 16;
    const int pr = prof_begin(ctx, per_pass == 8 ? 6 : 2, EPI_ARGMAX, R, (int64_t)((cbs + per_pass - 1) / per_pass) * ctx->NBv * ctx->KTd * 1024);
    HIPCHK(launch_head_gemm(ctx->head_t, ctx->NBv, ctx->KTd, ctx->V, ctx->xs_shadow, R, ctx->rowscale, ctx->pval,
                            ctx->pidx, ctx->psum, &nparts, ctx->stream, pr >= 0 ? ctx->prof_ev[2 * pr] : nullptr,
                            pr >= 0 ? ctx->prof_ev[2 * pr + 1] : nullptr, ctx->head_form));
    prof_end(ctx, pr);
  } else {
    for (int l = 1; l <= ctx->L; ++l) {
      GemmP p = head_gemm(ctx);
      p.X = ctx->hid_row(l, row0);
      p.prow0 = (l - 1) * m;
      del_status st = gemm(ctx, p, EPI_ARGMAX, m, false);
      if (st != DEL_OK) return st;
    }
  }
  HIPCHK(launch_argmax_finish(ctx->pval, ctx->pidx, ctx->psum, R, nparts, ctx->shadow_ids, ctx->conf_dev, ctx->stream));
  return DEL_OK;
}

void free_all(del_ctx* c) {
  void* ptrs[] = {c->arena, c->embed_t, (c->head_t != c->embed_t) ? c->head_t : nullptr, c->gains, c->kc, c->vc,
                  c->rope, c->hid, c->q, c->attn, c->act, c->xs_layer, c->xs_shadow, c->rowscale, c->xs_h, c->xs_attn,
                  c->xs_h1, c->xs_act, c->ssq_h, c->ssq_h1, c->PM, c->PL,
                  c->PA, c->pval, c->pidx, c->psum, c->state, c->draft_ids, c->shadow_ids, c->result, c->ids_dev,
                  c->logits_dbg, c->sink, c->stage, c->slog, c->swf, c->srows, c->unif_dev, c->rowscale_w, c->vct};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  if (c->result_host) (void)hipHostFree(c->result_host);   // conf_host and conf_dev point into the result blocks
  if (c->step_host) (void)hipHostFree(c->step_host);
  for (auto& e : c->ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : c->prof_ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& g : c->graphs)
    if (g.second) (void)hipGraphExecDestroy(g.second);
  c->graphs.clear();
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
}

// Run a segment of a round: eagerly (default), or as a HIP graph captured from the very same
// enqueue code the first time this (kind, a, b) is seen and replayed afterwards.
template <class F>
del_status run_segment(del_ctx* ctx, int kind, int a, int b, F&& enqueue) {
  if (!ctx->use_graphs || ctx->prof_on) return enqueue();
  const auto key = std::make_tuple(kind, a, b);
  auto it = ctx->graphs.find(key);
  if (it == ctx->graphs.end()) {
    if (ctx->graphs.size() >= 512) return enqueue();   // bounded cache: run the rest eagerly
    hipGraph_t g = nullptr;
    HIPCHK(hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeRelaxed));
    const del_status st = enqueue();
    const hipError_t e = hipStreamEndCapture(ctx->stream, &g);
    if (st != DEL_OK || e != hipSuccess) {
      if (g) (void)hipGraphDestroy(g);
      return st != DEL_OK ? st : ctx->fail(e, "hipStreamEndCapture");
    }
    hipGraphExec_t ge = nullptr;
    const hipError_t e2 = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
    (void)hipGraphDestroy(g);
    if (e2 != hipSuccess) return ctx->fail(e2, "hipGraphInstantiate");
    it = ctx->graphs.emplace(key, ge).first;
  }
  HIPCHK(hipGraphLaunch(it->second, ctx->stream));
  return DEL_OK;
}

enum { SEG_DRAFT = 0, SEG_VERIFY = 1, SEG_SHADOW = 2, SEG_STEP = 3, SEG_LAST = 4 };

}  // namespace

extern "C" {

const char* del_strerror(del_status s) {
  switch (s) {
    case DEL_OK: return "ok";
    case DEL_E_ARG: return "invalid argument";
    case DEL_E_STATE: return "call out of order";
    case DEL_E_CAPACITY: return "KV cache capacity exceeded";
    case DEL_E_SHAPE: return "tensor shape does not match the configuration";
    case DEL_E_DEVICE: return "HIP error";
    case DEL_E_NOMEM: return "out of memory";
  }
  return "unknown status";
}

const char* del_last_error_text(const del_ctx* ctx) { return ctx ? ctx->err.c_str() : ""; }

del_status del_create(const del_config* cfg, void* hip_stream, del_ctx** out) {
  if (!cfg || !out) return DEL_E_ARG;
  *out = nullptr;
  if (cfg->n_layers < 1 || cfg->d_model < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 ||
      cfg->n_q_heads % cfg->n_kv_heads != 0 || cfg->head_dim < 16 || cfg->head_dim > 128 ||
      cfg->head_dim % 16 != 0 || cfg->d_ffn < 8 || cfg->d_ffn % 8 != 0 || cfg->vocab < 2 ||
      (cfg->weight_dtype != DEL_DTYPE_FP32 && cfg->weight_dtype != DEL_DTYPE_BF16) || cfg->max_context < 2 ||
      cfg->d_max < 0 || cfg->d_max > 63 || cfg->prefill_window < 1 || !(cfg->omega >= 0.0 && cfg->omega <= 1.0) ||
      !(cfg->rope_theta > 0.f) || !(cfg->rms_eps >= 0.f))
    return DEL_E_ARG;
  del_ctx* ctx = new (std::nothrow) del_ctx();
  if (!ctx) return DEL_E_NOMEM;
  ctx->cfg = *cfg;
  ctx->stream = (hipStream_t)hip_stream;
  if (const char* e = getenv("DEL_GRAPHS")) ctx->use_graphs = atoi(e) != 0;
  if (!ctx->stream && ctx->use_graphs) {
    // stream capture needs a stream of its own (default priority); the NULL stream cannot be captured
    if (hipStreamCreateWithFlags(&ctx->stream, hipStreamNonBlocking) == hipSuccess) ctx->own_stream = true;
    else { ctx->stream = nullptr; ctx->use_graphs = false; }
  }
  ctx->L = cfg->n_layers; ctx->d = cfg->d_model; ctx->nq = cfg->n_q_heads; ctx->nkv = cfg->n_kv_heads;
  ctx->hd = cfg->head_dim; ctx->f = cfg->d_ffn; ctx->V = cfg->vocab; ctx->wd = cfg->weight_dtype;
  ctx->esize = ctx->wd == DEL_DTYPE_BF16 ? 2 : 4;
  ctx->KPL = kpl_of(ctx->wd); ctx->TK = tk_of(ctx->wd);
  ctx->qdim = ctx->nq * ctx->hd; ctx->kvdim = ctx->nkv * ctx->hd;
  ctx->KTd = ceil_div(ctx->d, ctx->TK); ctx->KTq = ceil_div(ctx->qdim, ctx->TK); ctx->KTf = ceil_div(ctx->f, ctx->TK);
  // activation rows are padded to 32 floats so that either tile width reads whole tiles
  ctx->dpad = ceil_div(ctx->d, 32) * 32; ctx->qpad = ceil_div(ctx->qdim, 32) * 32; ctx->fpad = ceil_div(ctx->f, 32) * 32;
  ctx->NBqkv = (ctx->qdim + 2 * ctx->kvdim) / 16;
  ctx->NBd = ceil_div(ctx->d, 16);
  ctx->NBgu = ceil_div(ctx->f, 8);
  ctx->NBv = ceil_div(ctx->V, 16);
  ctx->maxrows = std::max(16, cfg->d_max + 1);
  ctx->hrows = ctx->maxrows;
  ctx->Tcap = cfg->max_context;
  ctx->gpad = std::max(ctx->dpad, std::max(ctx->qpad, ctx->fpad));
  ctx->loaded.assign((size_t)(ctx->L + 1) * 12, 0);
  ctx->pol.reset(ctx->L, cfg->d_max, cfg->omega);
  ctx->last_c.assign(ctx->L + 1, 0);
  ctx->last_shadow.assign((size_t)(ctx->L + 1) * (cfg->d_max + 1), 0);
  ctx->last_draft.assign(std::max(1, cfg->d_max), 0);
  ctx->last_conf.assign((size_t)(ctx->L + 1) * (cfg->d_max + 1), 0.f);
  ctx->last_draft_conf.assign((size_t)cfg->d_max + 1, 0.f);
  if (const char* tw = getenv("DEL_TARGET_WAVES")) {
    const int v = atoi(tw);
    if (v >= 64 && v <= 65536) ctx->target_waves = v;
  }
  if (const char* wf = getenv("DEL_WIDE_FORM")) ctx->wide_form = atoi(wf) == 1 ? 1 : 0;
  if (const char* rf = getenv("DEL_ROWS_FORM")) ctx->rows_form = atoi(rf) == 1 ? 1 : 0;
  if (const char* hf = getenv("DEL_HEAD_FORM")) {
    const int v = atoi(hf);
    if (v == 1 || v == 4) ctx->head_form = v;
  }

  const size_t tile = 1024;
  auto al = [](size_t x) { return (x + 4095) & ~(size_t)4095; };
  ctx->off_qkv = 0;
  ctx->off_o = al(ctx->off_qkv + (size_t)ctx->NBqkv * ctx->KTd * tile);
  ctx->off_gu = al(ctx->off_o + (size_t)ctx->NBd * ctx->KTq * tile);
  ctx->off_dn = al(ctx->off_gu + (size_t)ctx->NBgu * ctx->KTd * tile);
  ctx->layer_stride = al(ctx->off_dn + (size_t)ctx->NBd * ctx->KTf * tile);
  ctx->arena_bytes = ctx->layer_stride * ctx->L;
  ctx->vocab_bytes = (size_t)ctx->NBv * ctx->KTd * tile;
  ctx->kv_layer_bytes = (size_t)ctx->nkv * ctx->Tcap * ctx->hd * ctx->esize;
  // attention chunk: as large as the staging registers allow, smaller when that leaves the
  // chip short of work-groups (few kv heads, short context)
  ctx->attn_ct = 64;
  while (ctx->attn_ct * ctx->hd * ctx->esize > 4 * 256 * 16) ctx->attn_ct -= 16;
  while (ctx->attn_ct > 16 && ctx->nkv * ceil_div(ctx->Tcap, ctx->attn_ct) < 512) ctx->attn_ct -= 16;
  if (const char* e = getenv("DEL_ATTN_CT")) {   // tuning override: 16, 32, 48 or 64 rows
    const int v = atoi(e);
    if (v >= 16 && v <= 64 && v % 16 == 0 && v * ctx->hd * ctx->esize <= 4 * 256 * 16) ctx->attn_ct = v;
  }
  ctx->nch_max = ceil_div(ctx->Tcap, ctx->attn_ct);
  if (attention_decode_supported(ctx->wd, ctx->hd, ctx->nq / ctx->nkv)) {
    // about 128 work-groups, at most 8 partials per head for the consumer to merge
    ctx->attn_S = std::max(1, std::min(std::min(8, ctx->nch_max), ceil_div(128, ctx->nkv)));
    if (const char* e = getenv("DEL_ATTN_SPLITS")) {
      const int v = atoi(e);
      if (v >= 0 && v <= std::min(8, ctx->nch_max)) ctx->attn_S = v;   // 0: staged kernels everywhere; 8: what the merge in the output projection takes
    }
    // enough rows give enough work-groups (rows x kv heads >= 192) without splitting the context
    ctx->attn_direct_rows = std::max(2, ceil_div(192, ctx->nkv));
    if (const char* e = getenv("DEL_ATTN_DIRECT_ROWS")) {
      const int v = atoi(e);
      if (v >= 0 && v <= 64) ctx->attn_direct_rows = v;   // 0: always split and merge
    }
    if (const char* e = getenv("DEL_VERIFY_FLASH")) ctx->verify_flash = atoi(e) != 0;
    if (const char* e = getenv("DEL_VERIFY_FLASH_WAVES")) {
      const int v = atoi(e);
      if (v >= 32 && v <= 16384) ctx->verify_flash_waves = v;
    }
    if (const char* e = getenv("DEL_ATTN_DEC_ROWS")) {
      const int v = atoi(e);
      if (v >= 1 && v <= 64) ctx->attn_dec_rows = v;
    }
  }
  // wide prefill passes: bf16 weights on the matrix cores with the register attention kernel
  if (cfg->use_mfma && ctx->wd == DEL_DTYPE_BF16 && ctx->attn_S > 0) {
    int want = 1024;
    if (const char* e = getenv("DEL_PREFILL_ROWS")) want = atoi(e);
    want = std::min(want, ceil_div(ctx->Tcap, 16) * 16);
    if (want >= 32) {
      ctx->prows = want / 16 * 16;
      ctx->hrows = std::max(ctx->maxrows, ctx->prows);
    }
  }
  const int Rmax = ctx->L * ctx->maxrows;
  const int KTmax = std::max(ctx->KTd, std::max(ctx->KTq, ctx->KTf));
  const size_t CBmax = (size_t)ceil_div(ctx->hrows, 16);

#define CK(call)                                                     \
  do {                                                               \
    hipError_t e_ = (call);                                          \
    if (e_ != hipSuccess) {                                          \
      del_status st_ = ctx->fail(e_, #call);                         \
      fprintf(stderr, "del_create: %s\n", ctx->err.c_str());         \
      free_all(ctx);                                                 \
      delete ctx;                                                    \
      return st_;                                                    \
    }                                                                \
  } while (0)
  CK(dmalloc(&ctx->arena, ctx->arena_bytes));
  CK(hipMemsetAsync(ctx->arena, 0, ctx->arena_bytes, ctx->stream));
  CK(dmalloc(&ctx->embed_t, ctx->vocab_bytes));
  CK(hipMemsetAsync(ctx->embed_t, 0, ctx->vocab_bytes, ctx->stream));
  if (cfg->tied_embeddings) {
    ctx->head_t = ctx->embed_t;
  } else {
    CK(dmalloc(&ctx->head_t, ctx->vocab_bytes));
    CK(hipMemsetAsync(ctx->head_t, 0, ctx->vocab_bytes, ctx->stream));
  }
  const size_t gains_bytes = ((size_t)ctx->L * 2 + 1) * ctx->gpad * sizeof(float);
  CK(dmalloc(&ctx->gains, gains_bytes));
  CK(hipMemsetAsync(ctx->gains, 0, gains_bytes, ctx->stream));
  CK(dmalloc(&ctx->kc, ctx->kv_layer_bytes * ctx->L));
  CK(dmalloc(&ctx->vc, ctx->kv_layer_bytes * ctx->L));
  CK(hipMemsetAsync(ctx->kc, 0, ctx->kv_layer_bytes * ctx->L, ctx->stream));
  CK(hipMemsetAsync(ctx->vc, 0, ctx->kv_layer_bytes * ctx->L, ctx->stream));
  {  // rotary table in double precision on the host: angle(p, j) = p * theta^(-2j/hd)
    const int half = ctx->hd / 2;
    std::vector<float2> tab((size_t)ctx->Tcap * half);
    for (int j = 0; j < half; ++j) {
      const double inv = std::pow((double)cfg->rope_theta, -2.0 * j / ctx->hd);
      for (int p = 0; p < ctx->Tcap; ++p) {
        const double a = (double)p * inv;
        tab[(size_t)p * half + j] = make_float2((float)std::cos(a), (float)std::sin(a));
      }
    }
    CK(dmalloc(&ctx->rope, tab.size() * sizeof(float2)));
    CK(hipMemcpy(ctx->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
  }
  const size_t hid_bytes = (size_t)(ctx->L + 1) * ctx->hrows * ctx->dpad * sizeof(float);
  CK(dmalloc(&ctx->hid, hid_bytes));
  CK(hipMemsetAsync(ctx->hid, 0, hid_bytes, ctx->stream));
  CK(dmalloc(&ctx->q, (size_t)ctx->hrows * ctx->qpad * 4));
  CK(dmalloc(&ctx->attn, (size_t)ctx->hrows * ctx->qpad * 4));
  CK(dmalloc(&ctx->act, (size_t)ctx->hrows * ctx->fpad * 4));
  CK(hipMemsetAsync(ctx->q, 0, (size_t)ctx->hrows * ctx->qpad * 4, ctx->stream));
  CK(hipMemsetAsync(ctx->attn, 0, (size_t)ctx->hrows * ctx->qpad * 4, ctx->stream));
  CK(hipMemsetAsync(ctx->act, 0, (size_t)ctx->hrows * ctx->fpad * 4, ctx->stream));
  CK(dmalloc(&ctx->xs_layer, (size_t)KTmax * 2048));
  CK(hipMemsetAsync(ctx->xs_layer, 0, (size_t)KTmax * 2048, ctx->stream));
  {
    uint16_t** bufs[4] = {&ctx->xs_h, &ctx->xs_attn, &ctx->xs_h1, &ctx->xs_act};
    for (auto b : bufs) {   // one set of tiles per block of 16 token rows
      CK(dmalloc(b, CBmax * KTmax * 2048));
      CK(hipMemsetAsync(*b, 0, CBmax * KTmax * 2048, ctx->stream));
    }
    CK(dmalloc(&ctx->ssq_h, CBmax * 16 * ctx->NBd * 4));
    CK(dmalloc(&ctx->ssq_h1, CBmax * 16 * ctx->NBd * 4));
    CK(dmalloc(&ctx->rowscale_w, CBmax * 16 * 4));
    const char* fl = getenv("DEL_PREFILL_FLASH");
    if (ctx->prows > 0 && (ctx->hd == 64 || ctx->hd == 128) && !(fl && atoi(fl) == 0)) {
      ctx->TcapT = ceil_div(ctx->Tcap, 32) * 32;
      ctx->vct_layer_bytes = (size_t)ctx->nkv * ctx->hd * ctx->TcapT * 2;
      CK(dmalloc(&ctx->vct, ctx->vct_layer_bytes * ctx->L));
      CK(hipMemsetAsync(ctx->vct, 0, ctx->vct_layer_bytes * ctx->L, ctx->stream));
    }
  }
  const size_t xs_sh = (size_t)ceil_div(Rmax, 16) * ctx->KTd * 2048;
  CK(dmalloc(&ctx->xs_shadow, xs_sh));
  CK(hipMemsetAsync(ctx->xs_shadow, 0, xs_sh, ctx->stream));
  CK(dmalloc(&ctx->rowscale, (size_t)(Rmax + 16) * 4));
  // attention partials: [row][head][nch_max] for the short passes, [row][head][WIDE_S] for the wide ones
  const size_t prow = std::max((size_t)ctx->maxrows * ctx->nq * ctx->nch_max, (size_t)ctx->hrows * ctx->nq * WIDE_S);
  CK(dmalloc(&ctx->PM, prow * 4));
  CK(dmalloc(&ctx->PL, prow * 4));
  CK(dmalloc(&ctx->PA, prow * ctx->hd * 4));
  CK(dmalloc(&ctx->pval, (size_t)Rmax * ctx->NBv * 4));
  CK(dmalloc(&ctx->pidx, (size_t)Rmax * ctx->NBv * 4));
  CK(dmalloc(&ctx->psum, (size_t)Rmax * ctx->NBv * 4));
  CK(hipHostMalloc((void**)&ctx->step_host, 16, hipHostMallocDefault));
  memset(ctx->step_host, 0, 16);
  CK(dmalloc(&ctx->state, 16));
  CK(hipMemsetAsync(ctx->state, 0, 16, ctx->stream));
  CK(dmalloc(&ctx->draft_ids, (size_t)(cfg->d_max + 1) * 4));
  CK(dmalloc(&ctx->shadow_ids, (size_t)Rmax * 4));
  // a round's results in one block, so that one copy brings them to the host: the counts, drafted and shadow ids
  // (ints), then the shadow and draft confidences (floats); the same layout in pinned host memory
  ctx->res_ints = (size_t)(3 + cfg->d_max + 1 + Rmax);
  ctx->res_words = ctx->res_ints + (size_t)(Rmax + cfg->d_max + 1);
  CK(dmalloc(&ctx->result, ctx->res_words * 4));
  ctx->conf_dev = reinterpret_cast<float*>(ctx->result + ctx->res_ints);
  CK(dmalloc(&ctx->ids_dev, (size_t)ctx->Tcap * 4));
  CK(hipHostMalloc((void**)&ctx->result_host, ctx->res_words * 4, hipHostMallocDefault));
  ctx->conf_host = reinterpret_cast<float*>(ctx->result_host + ctx->res_ints);
  CK(dmalloc(&ctx->logits_dbg, (size_t)ctx->NBv * 16 * 4));
  CK(dmalloc(&ctx->sink, 16));
  {
    const size_t srow_n = (size_t)2 * (cfg->d_max + 1);
    ctx->sld = (int64_t)ctx->NBv * 16;
    CK(dmalloc(&ctx->slog, srow_n * ctx->sld * 4));
    CK(dmalloc(&ctx->swf, srow_n * ctx->sld * 8));
    CK(dmalloc(&ctx->srows, srow_n * sizeof(SampRow)));
    CK(dmalloc(&ctx->unif_dev, (srow_n + 2) * 4));
  }
  for (auto& e : ctx->ev) CK(hipEventCreate(&e));
  CK(hipStreamSynchronize(ctx->stream));
#undef CK
  *out = ctx;
  return DEL_OK;
}

void del_destroy(del_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  free_all(ctx);
  delete ctx;
}

del_status del_load_weights(del_ctx* ctx, const del_tensor* tensors, int32_t n) {
  if (!ctx || (!tensors && n > 0) || n < 0) return DEL_E_ARG;
  // device-resident sources were produced on the caller's streams: wait for them
  for (int i = 0; i < n; ++i)
    if (tensors[i].location == DEL_MEM_DEVICE) { HIPCHK(hipDeviceSynchronize()); break; }
  for (int i = 0; i < n; ++i) {
    const del_tensor& t = tensors[i];
    if (!t.data || t.kind < 0 || t.kind > DEL_T_WD) return DEL_E_ARG;
    if (t.location != DEL_MEM_HOST && t.location != DEL_MEM_DEVICE) return DEL_E_ARG;
    const bool global = t.kind <= DEL_T_FINAL_NORM;
    if (global ? t.layer != -1 : (t.layer < 0 || t.layer >= ctx->L)) return DEL_E_ARG;
    if (t.kind == DEL_T_LM_HEAD && ctx->cfg.tied_embeddings) return DEL_E_ARG;
    int64_t rows = 0, cols = 0;
    char* dst = nullptr;
    int KT = 0, map = MAP_PLAIN, vbase = 0;
    char* lbase = global ? nullptr : ctx->arena + (size_t)t.layer * ctx->layer_stride;
    switch (t.kind) {
      case DEL_T_EMBED: rows = ctx->V; cols = ctx->d; dst = ctx->embed_t; KT = ctx->KTd; break;
      case DEL_T_LM_HEAD: rows = ctx->V; cols = ctx->d; dst = ctx->head_t; KT = ctx->KTd; break;
      case DEL_T_FINAL_NORM: case DEL_T_ATTN_NORM: case DEL_T_FFN_NORM: rows = 1; cols = ctx->d; break;
      case DEL_T_WQ: rows = ctx->qdim; cols = ctx->d; dst = lbase + ctx->off_qkv; KT = ctx->KTd; map = MAP_ROPE; break;
      case DEL_T_WK: rows = ctx->kvdim; cols = ctx->d; dst = lbase + ctx->off_qkv; KT = ctx->KTd; map = MAP_ROPE;
        vbase = ctx->qdim; break;
      case DEL_T_WV: rows = ctx->kvdim; cols = ctx->d; dst = lbase + ctx->off_qkv; KT = ctx->KTd;
        vbase = ctx->qdim + ctx->kvdim; break;
      case DEL_T_WO: rows = ctx->d; cols = ctx->qdim; dst = lbase + ctx->off_o; KT = ctx->KTq; break;
      case DEL_T_WG: rows = ctx->f; cols = ctx->d; dst = lbase + ctx->off_gu; KT = ctx->KTd; map = MAP_GATE; break;
      case DEL_T_WU: rows = ctx->f; cols = ctx->d; dst = lbase + ctx->off_gu; KT = ctx->KTd; map = MAP_UP; break;
      case DEL_T_WD: rows = ctx->d; cols = ctx->f; dst = lbase + ctx->off_dn; KT = ctx->KTf; break;
    }
    if (t.rows != rows || t.cols != cols) return DEL_E_SHAPE;
    const bool is_gain = dst == nullptr;
    const size_t es = is_gain ? 4 : (size_t)ctx->esize;
    const size_t row_bytes = (size_t)cols * es;
    // rows per staged piece: at most 256 MiB of host data in flight on the device
    const int64_t piece = std::max<int64_t>(1, (int64_t)((256ull << 20) / row_bytes));
    for (int64_t r0 = 0; r0 < rows; r0 += piece) {
      const int64_t nr = std::min<int64_t>(piece, rows - r0);
      const char* src = (const char*)t.data + (size_t)r0 * row_bytes;
      if (t.location == DEL_MEM_HOST) {
        const size_t need = (size_t)nr * row_bytes;
        if (need > ctx->stage_bytes) {
          if (ctx->stage) (void)hipFree(ctx->stage);
          ctx->stage = nullptr; ctx->stage_bytes = 0;
          HIPCHK(hipMalloc(&ctx->stage, need));
          ctx->stage_bytes = need;
        }
        HIPCHK(hipMemcpyAsync(ctx->stage, src, need, hipMemcpyHostToDevice, ctx->stream));
        src = (const char*)ctx->stage;
      }
      if (is_gain) {
        float* g = t.kind == DEL_T_FINAL_NORM ? ctx->gain_final()
                   : t.kind == DEL_T_ATTN_NORM ? ctx->gain_attn(t.layer) : ctx->gain_ffn(t.layer);
        HIPCHK(launch_pad_gain((const float*)src, ctx->d, g, ctx->gpad, ctx->stream));
      } else {
        HIPCHK(launch_tile_scatter(src, ctx->wd, r0, nr, cols, map, vbase, ctx->hd, dst, KT, ctx->stream));
      }
      // the staging buffer (or the caller's buffer) is reused right after this call
      HIPCHK(hipStreamSynchronize(ctx->stream));
    }
    ctx->loaded[(size_t)(t.layer + 1) * 12 + t.kind] = 1;
  }
  if (ctx->stage && ctx->all_loaded()) {
    (void)hipFree(ctx->stage);
    ctx->stage = nullptr; ctx->stage_bytes = 0;
  }
  return DEL_OK;
}

del_status del_prefill(del_ctx* ctx, const int32_t* prompt, int32_t n_prompt, int32_t* first_token, int32_t* next_E,
                       int32_t* next_gamma) {
  if (!ctx || !prompt || !first_token || !next_E || !next_gamma || n_prompt < 1) return DEL_E_ARG;
  if (!ctx->all_loaded()) return DEL_E_STATE;
  if (n_prompt + 1 > ctx->Tcap) return DEL_E_CAPACITY;
  for (int i = 0; i < n_prompt; ++i)
    if (prompt[i] < 0 || prompt[i] >= ctx->V) return DEL_E_ARG;
  const int L = ctx->L, P = n_prompt;
  ctx->phase = 0;
  ctx->pol.reset(L, ctx->cfg.d_max, ctx->cfg.omega);
  ctx->rounds = 0;
  HIPCHK(hipMemcpyAsync(ctx->ids_dev, prompt, (size_t)P * 4, hipMemcpyHostToDevice, ctx->stream));
  HIPCHK(launch_set_state(ctx->state, 0, 0, nullptr, -1, ctx->stream));
  const int w = std::min(ctx->cfg.prefill_window, P);
  std::vector<int> shadow((size_t)L * w, 0);  // [l-1][window position]
  std::vector<float> sconf((size_t)L * w, 0.f);
  // passes of up to CH rows (16, or the wide pass's rows); a ragged pass, if any, comes first so that
  // the last ones are full; a pass of more than 16 rows takes the wide path
  const int CH = ctx->prows > 0 ? ctx->prows : 16;
  int start = 0;
  while (start < P) {
    const int mc = (start == 0 && P % CH != 0) ? P % CH : CH;
    // with the feature-major value copy every pass must keep it filled: all passes take the wide path
    const bool widep = ctx->prows > 0 && (mc > 16 || ctx->vct);
    ctx->T = start;   // host mirror of the KV length this pass starts from
    HIPCHK(launch_embed(ctx->embed_t, ctx->wd, ctx->KTd, ctx->V, ctx->ids_dev + start, mc, ctx->hid_row(0, 0),
                        ctx->dpad, ctx->d, ctx->stream));
    for (int l = 1; l <= L; ++l) {
      del_status st = widep ? run_layer_wide(ctx, l, mc, l > 1) : run_layer(ctx, l, 0, mc, l > 1);
      if (st != DEL_OK) return st;
    }
    // rows of this pass inside the statistics window, in groups of up to 16
    for (int r0 = std::max(0, P - w - start); r0 < mc; r0 += 16) {
      const int cnt = std::min(16, mc - r0);
      del_status st = shadow_head(ctx, cnt, r0);
      if (st != DEL_OK) return st;
      HIPCHK(hipMemcpyAsync(ctx->result_host, ctx->shadow_ids, (size_t)L * cnt * 4, hipMemcpyDeviceToHost,
                            ctx->stream));
      HIPCHK(hipMemcpyAsync(ctx->conf_host, ctx->conf_dev, (size_t)L * cnt * 4, hipMemcpyDeviceToHost, ctx->stream));
      HIPCHK(hipStreamSynchronize(ctx->stream));
      for (int i = 0; i < cnt; ++i) {
        const int wpos = start + r0 + i - (P - w);
        for (int l = 1; l <= L; ++l) {
          shadow[(size_t)(l - 1) * w + wpos] = ctx->result_host[(l - 1) * cnt + i];
          sconf[(size_t)(l - 1) * w + wpos] = ctx->conf_host[(l - 1) * cnt + i];
        }
      }
    }
    HIPCHK(launch_set_state(ctx->state, mc, -1, nullptr, -1, ctx->stream));
    ctx->last_rows = mc;
    start += mc;
  }
  // pseudo-round over the window: every layer's shadow token against layer L's
  std::vector<int> c(L + 1, 0);
  for (int l = 1; l <= L; ++l)
    for (int i = 0; i < w; ++i) c[l] += shadow[(size_t)(l - 1) * w + i] == shadow[(size_t)(L - 1) * w + i];
  std::vector<double> tcs(L + 1, 0.0), fcs(L + 1, 0.0);
  for (int l = 1; l <= L; ++l)
    for (int i = 0; i < w; ++i) {
      const bool hit = shadow[(size_t)(l - 1) * w + i] == shadow[(size_t)(L - 1) * w + i];
      (hit ? tcs : fcs)[l] += (double)sconf[(size_t)(l - 1) * w + i];
    }
  ctx->pol.update(c.data(), w, tcs.data(), fcs.data());
  const int first = shadow[(size_t)(L - 1) * w + (w - 1)];
  HIPCHK(launch_set_state(ctx->state, 0, -1, nullptr, first, ctx->stream));
  HIPCHK(hipStreamSynchronize(ctx->stream));
  prof_collect(ctx);
  ctx->T = P; ctx->pending = first; ctx->phase = 1;
  ctx->last_c = c; ctx->last_E = 0; ctx->last_gamma = 0; ctx->last_u = w - 1; ctx->last_n = w;
  *first_token = first; *next_E = ctx->pol.next_E; *next_gamma = ctx->pol.next_gamma;
  return DEL_OK;
}

// After a round's last kernel is queued: wait, read the results back, update the statistics
// (Sections 4.2, 4.4: over the valid positions 0..u, n = u + 1) and the host's mirror of the state.
// sampled: the emitted tokens are the accepted drafts and the drawn last token, and layer E's shadow
// tokens are its greedy ones; otherwise they are the target's tokens and the drafts stand in for
// layer E's shadow tokens.
static del_status finish_round(del_ctx* ctx, int E, int gamma, bool stopped, bool sampled, int32_t* out_tokens,
                               int32_t* n_out) {
  const int L = ctx->L, m = gamma + 1;
  const int Rmax = L * ctx->maxrows;
  HIPCHK(hipStreamSynchronize(ctx->stream));
  prof_collect(ctx);
  (void)hipEventElapsedTime(&ctx->t_draft, ctx->ev[0], ctx->ev[1]);
  (void)hipEventElapsedTime(&ctx->t_verify, ctx->ev[1], ctx->ev[2]);
  (void)hipEventElapsedTime(&ctx->t_shadow, ctx->ev[2], ctx->ev[3]);
  const int* res = ctx->result_host;
  const int u = res[0];
  const int* drafts = res + 3;
  const int* sh = res + 3 + gamma;  // [L][m]
  const int* target = sh + (size_t)(L - 1) * m;
  float* cf = ctx->conf_host;       // [L][m]
  const float* dcf = ctx->conf_host + Rmax;
  // greedy: the drafted tokens are layer E's shadow tokens, their confidences are the draft's too
  if (!sampled)
    for (int i = 0; i < gamma; ++i) cf[(size_t)(E - 1) * m + i] = dcf[i];
  std::vector<int> c(L + 1, 0);
  std::vector<double> tcs(L + 1, 0.0), fcs(L + 1, 0.0);
  for (int l = 1; l <= L; ++l)
    for (int i = 0; i <= u; ++i) {
      const bool hit = sh[(size_t)(l - 1) * m + i] == target[i];
      c[l] += hit;
      (hit ? tcs : fcs)[l] += (double)cf[(size_t)(l - 1) * m + i];
    }
  ctx->pol.update(c.data(), u + 1, tcs.data(), fcs.data());
  if (sampled) {
    for (int i = 0; i < u; ++i) out_tokens[i] = drafts[i];
    out_tokens[u] = res[2];
  } else {
    for (int i = 0; i <= u; ++i) out_tokens[i] = target[i];
  }
  *n_out = u + 1;
  ctx->T = res[1]; ctx->pending = res[2];
  ctx->rounds += 1; ctx->last_rows = m;
  ctx->last_c = c; ctx->last_E = E; ctx->last_gamma = gamma; ctx->last_u = u; ctx->last_n = u + 1;
  ctx->last_stopped = stopped ? 1 : 0;
  const int stride = ctx->cfg.d_max + 1;
  std::fill(ctx->last_shadow.begin(), ctx->last_shadow.end(), 0);
  std::fill(ctx->last_conf.begin(), ctx->last_conf.end(), 0.f);
  for (int l = 1; l <= L; ++l)
    for (int i = 0; i < m; ++i) {
      ctx->last_shadow[(size_t)l * stride + i] = sh[(size_t)(l - 1) * m + i];
      ctx->last_conf[(size_t)l * stride + i] = cf[(size_t)(l - 1) * m + i];
    }
  for (int i = 0; i < gamma; ++i) ctx->last_draft[i] = drafts[i];
  std::fill(ctx->last_draft_conf.begin(), ctx->last_draft_conf.end(), 0.f);
  if (!sampled)
    for (int i = 0; i < gamma + (stopped ? 1 : 0); ++i) ctx->last_draft_conf[i] = dcf[i];
  return DEL_OK;
}

// One round.  tau < 0: draft exactly `gamma` tokens.  tau >= 0: dynamic draft-exiting (Section 4.4;
// Algorithm 1 loop): draft up to `gamma` tokens, stop before appending the first one whose
// confidence is below tau; the stopping step's exit state is the round's last row.
static del_status round_impl(del_ctx* ctx, int E, int gamma, double tau, int32_t* out_tokens, int32_t* n_out,
                             int32_t* gamma_used, int32_t* stopped_early) {
  if (!ctx || !out_tokens || !n_out) return DEL_E_ARG;
  if (ctx->phase != 1) return DEL_E_STATE;
  const int L = ctx->L;
  if (E < 1 || E > L || gamma < 0 || gamma > ctx->cfg.d_max) return DEL_E_ARG;
  if (ctx->T + gamma + 1 > ctx->Tcap) return DEL_E_CAPACITY;
  const bool dynamic = tau >= 0.0;
  const int Rmax = L * ctx->maxrows;
  float* dconf = ctx->conf_dev + Rmax;   // draft confidences
  hipStream_t s = ctx->stream;
  HIPCHK(hipEventRecord(ctx->ev[0], s));
  // one draft step: embed the pending token, layers 1..E on row i, optionally the head
  auto draft_step = [&](int i, bool with_head, bool copy_conf) -> del_status {
    // step 0 embeds the pending token; the head of step i - 1 has already left step i's embedding row
    if (i == 0)
      HIPCHK(launch_embed(ctx->embed_t, ctx->wd, ctx->KTd, ctx->V, ctx->state + 1, 1, ctx->hid_row(0, 0), ctx->dpad,
                          ctx->d, s));
    for (int l = 1; l <= E; ++l) {
      del_status st = run_layer(ctx, l, i, 1, l > 1);
      if (st != DEL_OK) return st;
    }
    if (with_head) {
      // a step the host decides on: its head writes (sequence number, confidence) straight into pinned
      // memory, which the host polls; under graph replay (a baked-in number would be stale) a copy instead
      const bool poll = copy_conf && !ctx->use_graphs;
      unsigned long long* note = reinterpret_cast<unsigned long long*>(ctx->step_host) + 1;
      del_status st = head_one(ctx, E, i, ctx->draft_ids + i, dconf + i, ctx->hid_row(0, i + 1),
                               poll ? note : nullptr, poll ? ++ctx->note_seq : 0);
      if (st != DEL_OK) return st;
      if (copy_conf && !poll) HIPCHK(hipMemcpyAsync(ctx->step_host, dconf + i, 4, hipMemcpyDeviceToHost, s));
    }
    return DEL_OK;
  };
  // ---- draft: auto-regressive steps through layers 1..E + head
  bool stopped = false;
  if (!dynamic) {
    // the last pending token (step gamma) needs no head: only its exit state and KV
    del_status st = run_segment(ctx, SEG_DRAFT, E, gamma, [&]() -> del_status {
      for (int i = 0; i <= gamma; ++i) {
        del_status st2 = draft_step(i, i < gamma, false);
        if (st2 != DEL_OK) return st2;
      }
      return DEL_OK;
    });
    if (st != DEL_OK) return st;
  } else {
    const int cap = gamma;
    for (int i = 0; i <= cap; ++i) {
      if (i == cap) {   // all `cap` tokens appended: the last one still needs its exit state
        del_status st = run_segment(ctx, SEG_LAST, E, i, [&]() { return draft_step(i, false, false); });
        if (st != DEL_OK) return st;
        break;
      }
      // the host decides whether to go on: one small copy and a sync per step
      del_status st = run_segment(ctx, SEG_STEP, E, i, [&]() { return draft_step(i, true, true); });
      if (st != DEL_OK) return st;
      float cf;
      if (!ctx->use_graphs) {
        // poll the word the head writes; past a few milliseconds fall back to waiting for the stream
        const volatile unsigned long long* note = reinterpret_cast<unsigned long long*>(ctx->step_host) + 1;
        const auto t0 = std::chrono::steady_clock::now();
        unsigned long long w = *note;
        for (unsigned spins = 0; (unsigned)(w >> 32) != ctx->note_seq; ++spins) {
          if ((spins & 1023u) == 1023u && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(20)) {
            HIPCHK(hipStreamSynchronize(s));
            w = *note;
            if ((unsigned)(w >> 32) != ctx->note_seq) return ctx->fail(hipErrorUnknown, "draft step left no confidence");
            break;
          }
          w = *note;
        }
        const unsigned bits = (unsigned)w;
        memcpy(&cf, &bits, 4);
      } else {
        HIPCHK(hipStreamSynchronize(s));
        memcpy(&cf, ctx->step_host, 4);
      }
      if ((double)cf < tau) {   // not appended; row i is the last row of the round
        gamma = i;
        stopped = true;
        break;
      }
    }
  }
  const int m = gamma + 1;
  HIPCHK(hipEventRecord(ctx->ev[1], s));
  // ---- verify: the gamma+1 exit states through layers E+1..L
  {
    del_status st = run_segment(ctx, SEG_VERIFY, E, m, [&]() -> del_status {
      for (int l = E + 1; l <= L; ++l) {
        del_status st2 = layer_pass(ctx, l, m, l > E + 1);
        if (st2 != DEL_OK) return st2;
      }
      return DEL_OK;
    });
    if (st != DEL_OK) return st;
  }
  HIPCHK(hipEventRecord(ctx->ev[2], s));
  // ---- shadow tokens of every layer (row L = the target's tokens), acceptance on device,
  //      results to pinned host memory
  {
    del_status st = run_segment(ctx, SEG_SHADOW, E, gamma, [&]() -> del_status {
      del_status st2 = shadow_head(ctx, m);
      if (st2 != DEL_OK) return st2;
      HIPCHK(launch_accept(ctx->state, ctx->draft_ids, ctx->shadow_ids, L, m, E, gamma, ctx->result, s));
      HIPCHK(hipMemcpyAsync(ctx->result_host, ctx->result, ctx->res_words * 4, hipMemcpyDeviceToHost, s));   // ids + confidences
      return DEL_OK;
    });
    if (st != DEL_OK) return st;
  }
  HIPCHK(hipEventRecord(ctx->ev[3], s));
  del_status fst = finish_round(ctx, E, gamma, stopped, false, out_tokens, n_out);
  if (fst != DEL_OK) return fst;
  if (gamma_used) *gamma_used = gamma;
  if (stopped_early) *stopped_early = stopped ? 1 : 0;
  return DEL_OK;
}

del_status del_round(del_ctx* ctx, int32_t E, int32_t gamma, int32_t* out_tokens, int32_t* n_out) {
  return round_impl(ctx, E, gamma, -1.0, out_tokens, n_out, nullptr, nullptr);
}

del_status del_round_dynamic(del_ctx* ctx, int32_t E, double tau, int32_t d_cap, int32_t* out_tokens, int32_t* n_out,
                             int32_t* gamma_used, int32_t* stopped_early) {
  if (!(tau >= 0.0)) return DEL_E_ARG;
  return round_impl(ctx, E, d_cap, tau, out_tokens, n_out, gamma_used, stopped_early);
}

// Logits of rows [row0, row0+m) of layer `layer` into sampling rows [srow0, srow0+m).
static del_status sample_logits(del_ctx* ctx, int layer, int row0, int m, int srow0) {
  GemmP p = head_gemm(ctx);
  p.X = ctx->hid_row(layer, row0);
  p.Y = ctx->slog + (size_t)srow0 * ctx->sld; p.ldy = (int)ctx->sld;
  const bool mf = ctx->cfg.use_mfma && ctx->wd == DEL_DTYPE_BF16 && m > 1;
  return gemm(ctx, p, EPI_STORE, m, mf);
}

static bool sampling_args_ok(double temperature, double top_p) {
  return temperature > 0.0 && top_p > 0.0 && top_p <= 1.0 && std::isfinite(temperature);
}

del_status del_sample_first(del_ctx* ctx, double temperature, double top_p, float r, int32_t* token) {
  if (!ctx || !token || !sampling_args_ok(temperature, top_p) || !(r >= 0.f && r < 1.f)) return DEL_E_ARG;
  if (ctx->phase != 1 || ctx->rounds != 0) return DEL_E_STATE;
  hipStream_t s = ctx->stream;
  const int VB = ctx->cfg.d_max + 1;
  del_status st = sample_logits(ctx, ctx->L, ctx->last_rows - 1, 1, VB);
  if (st != DEL_OK) return st;
  HIPCHK(hipMemcpyAsync(ctx->unif_dev, &r, 4, hipMemcpyHostToDevice, s));
  HIPCHK(launch_samp_rowstats(ctx->slog + (size_t)VB * ctx->sld, ctx->sld, ctx->V, 1, temperature, top_p,
                              ctx->swf + (size_t)VB * ctx->sld, ctx->sld, ctx->srows + VB, ctx->unif_dev,
                              ctx->draft_ids, ctx->state + 1, nullptr, s));
  HIPCHK(hipMemcpyAsync(ctx->step_host, ctx->draft_ids, 4, hipMemcpyDeviceToHost, s));
  HIPCHK(hipStreamSynchronize(s));
  ctx->pending = ctx->step_host[0];
  *token = ctx->pending;
  return DEL_OK;
}

// One sampled round.  tau < 0: draft exactly `gamma` tokens; otherwise `gamma` caps the draft and the
// loop stops, before a token is drawn, at the first step whose confidence is below tau.  uniforms:
// [0, gamma) drafts, [gamma, 2*gamma) acceptances, [2*gamma] the last token.
static del_status round_sample_impl(del_ctx* ctx, int E, int gamma, double tau, double temperature, double top_p,
                                    const float* uniforms, int32_t* out_tokens, int32_t* n_out, int32_t* gamma_used,
                                    int32_t* stopped_early) {
  if (!ctx || !out_tokens || !n_out || !uniforms || !sampling_args_ok(temperature, top_p)) return DEL_E_ARG;
  if (ctx->phase != 1) return DEL_E_STATE;
  const int L = ctx->L;
  if (E < 1 || E > L || gamma < 0 || gamma > ctx->cfg.d_max) return DEL_E_ARG;
  for (int i = 0; i < 2 * gamma + 1; ++i)
    if (!(uniforms[i] >= 0.f && uniforms[i] < 1.f)) return DEL_E_ARG;
  if (ctx->T + gamma + 1 > ctx->Tcap) return DEL_E_CAPACITY;
  hipStream_t s = ctx->stream;
  const int cap = gamma, VB = ctx->cfg.d_max + 1, V = ctx->V;
  const int64_t ld = ctx->sld;
  const bool dynamic = tau >= 0.0;
  const int Rmax = L * ctx->maxrows;
  float* dconf = ctx->conf_dev + Rmax;   // draft confidences
  HIPCHK(hipMemcpyAsync(ctx->unif_dev, uniforms, (size_t)(2 * cap + 1) * 4, hipMemcpyHostToDevice, s));
  HIPCHK(hipEventRecord(ctx->ev[0], s));
  // ---- draft: layers 1..E, the exit layer's logits, a draw from their nucleus
  bool stopped = false;
  for (int i = 0; i <= gamma; ++i) {
    const int* tok = i == 0 ? ctx->state + 1 : ctx->draft_ids + (i - 1);
    HIPCHK(launch_embed(ctx->embed_t, ctx->wd, ctx->KTd, V, tok, 1, ctx->hid_row(0, i), ctx->dpad, ctx->d, s));
    for (int l = 1; l <= E; ++l) {
      del_status st = run_layer(ctx, l, i, 1, l > 1);
      if (st != DEL_OK) return st;
    }
    if (i < gamma) {
      del_status st = sample_logits(ctx, E, i, 1, i);
      if (st != DEL_OK) return st;
      HIPCHK(launch_samp_rowstats(ctx->slog + (size_t)i * ld, ld, V, 1, temperature, top_p, ctx->swf + (size_t)i * ld,
                                  ld, ctx->srows + i, ctx->unif_dev + i, ctx->draft_ids + i, nullptr,
                                  dynamic ? dconf + i : nullptr, s));
      if (dynamic) {   // the host decides whether to go on: one small copy and a sync per step
        HIPCHK(hipMemcpyAsync(ctx->step_host, dconf + i, 4, hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        float cf;
        memcpy(&cf, ctx->step_host, 4);
        if ((double)cf < tau) {   // the token drawn at this step is dropped; row i is the round's last row
          gamma = i;
          stopped = true;
          break;
        }
      }
    }
  }
  const int m = gamma + 1;
  HIPCHK(hipEventRecord(ctx->ev[1], s));
  // ---- verify: the gamma+1 exit states through layers E+1..L
  for (int l = E + 1; l <= L; ++l) {
    del_status st = layer_pass(ctx, l, m, l > E + 1);
    if (st != DEL_OK) return st;
  }
  HIPCHK(hipEventRecord(ctx->ev[2], s));
  // ---- greedy shadow tokens of every layer; the target's distributions; acceptance on the device
  {
    del_status st = shadow_head(ctx, m);
    if (st != DEL_OK) return st;
    st = sample_logits(ctx, L, 0, m, VB);
    if (st != DEL_OK) return st;
    HIPCHK(launch_samp_rowstats(ctx->slog + (size_t)VB * ld, ld, V, m, temperature, top_p, ctx->swf + (size_t)VB * ld, ld,
                                ctx->srows + VB, nullptr, nullptr, nullptr, nullptr, s));
    HIPCHK(launch_samp_accept(ctx->slog, ctx->swf, ctx->srows, ctx->slog + (size_t)VB * ld, ctx->swf + (size_t)VB * ld,
                              ctx->srows + VB, ld, ld, V, gamma, ctx->draft_ids, ctx->unif_dev + cap,
                              ctx->unif_dev + 2 * cap, ctx->state, ctx->shadow_ids, L * m, ctx->result, s));
    HIPCHK(hipMemcpyAsync(ctx->result_host, ctx->result, ctx->res_words * 4, hipMemcpyDeviceToHost, s));   // ids + confidences
  }
  HIPCHK(hipEventRecord(ctx->ev[3], s));
  del_status fst = finish_round(ctx, E, gamma, stopped, true, out_tokens, n_out);
  if (fst != DEL_OK) return fst;
  if (dynamic) {
    const float* dcf = ctx->conf_host + Rmax;
    for (int i = 0; i < gamma + (stopped ? 1 : 0); ++i) ctx->last_draft_conf[i] = dcf[i];
  }
  if (gamma_used) *gamma_used = gamma;
  if (stopped_early) *stopped_early = stopped ? 1 : 0;
  return DEL_OK;
}

del_status del_round_sample(del_ctx* ctx, int32_t E, int32_t gamma, double temperature, double top_p,
                            const float* uniforms, int32_t* out_tokens, int32_t* n_out) {
  return round_sample_impl(ctx, E, gamma, -1.0, temperature, top_p, uniforms, out_tokens, n_out, nullptr, nullptr);
}

del_status del_round_sample_dynamic(del_ctx* ctx, int32_t E, double tau, int32_t d_cap, double temperature,
                                    double top_p, const float* uniforms, int32_t* out_tokens, int32_t* n_out,
                                    int32_t* gamma_used, int32_t* stopped_early) {
  if (!(tau >= 0.0)) return DEL_E_ARG;
  return round_sample_impl(ctx, E, d_cap, tau, temperature, top_p, uniforms, out_tokens, n_out, gamma_used,
                           stopped_early);
}

del_status del_debug_spec_sample(del_ctx* ctx, const float* q_logits, const float* p_logits, int32_t gamma,
                                 double temperature, double top_p, const float* uniforms, int32_t* drafts_out,
                                 int32_t* u, int32_t* last_token) {
  if (!ctx || !p_logits || !uniforms || !u || !last_token || gamma < 0 || gamma > ctx->cfg.d_max ||
      (gamma > 0 && (!q_logits || !drafts_out)) || !sampling_args_ok(temperature, top_p))
    return DEL_E_ARG;
  for (int i = 0; i < 2 * gamma + 1; ++i)
    if (!(uniforms[i] >= 0.f && uniforms[i] < 1.f)) return DEL_E_ARG;
  hipStream_t s = ctx->stream;
  const int VB = ctx->cfg.d_max + 1, V = ctx->V;
  const int64_t ld = ctx->sld;
  HIPCHK(hipStreamSynchronize(s));
  if (gamma > 0)
    HIPCHK(hipMemcpy2D(ctx->slog, (size_t)ld * 4, q_logits, (size_t)V * 4, (size_t)V * 4, gamma, hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy2D(ctx->slog + (size_t)VB * ld, (size_t)ld * 4, p_logits, (size_t)V * 4, (size_t)V * 4, gamma + 1,
                     hipMemcpyHostToDevice));
  HIPCHK(hipMemcpy(ctx->unif_dev, uniforms, (size_t)(2 * gamma + 1) * 4, hipMemcpyHostToDevice));
  // state, drafts and result live in the debug logits buffer, so that the context's own are untouched
  const int DM = ctx->cfg.d_max + 1;
  int* scratch = reinterpret_cast<int*>(ctx->logits_dbg);
  int* st_s = scratch; int* dr_s = scratch + 4; int* rs_s = scratch + 4 + DM;
  const size_t n_scr = (size_t)4 + DM + 3 + DM;
  if ((size_t)ctx->NBv * 16 < n_scr) return DEL_E_CAPACITY;
  HIPCHK(hipMemsetAsync(scratch, 0, n_scr * 4, s));
  if (gamma > 0)
    HIPCHK(launch_samp_rowstats(ctx->slog, ld, V, gamma, temperature, top_p, ctx->swf, ld, ctx->srows, ctx->unif_dev,
                                dr_s, nullptr, nullptr, s));
  HIPCHK(launch_samp_rowstats(ctx->slog + (size_t)VB * ld, ld, V, gamma + 1, temperature, top_p,
                              ctx->swf + (size_t)VB * ld, ld, ctx->srows + VB, nullptr, nullptr, nullptr, nullptr, s));
  HIPCHK(launch_samp_accept(ctx->slog, ctx->swf, ctx->srows, ctx->slog + (size_t)VB * ld, ctx->swf + (size_t)VB * ld,
                            ctx->srows + VB, ld, ld, V, gamma, dr_s, ctx->unif_dev + gamma, ctx->unif_dev + 2 * gamma, st_s,
                            nullptr, 0, rs_s, s));
  HIPCHK(hipStreamSynchronize(s));
  std::vector<int> host(n_scr);
  HIPCHK(hipMemcpy(host.data(), scratch, n_scr * 4, hipMemcpyDeviceToHost));
  *u = host[4 + DM];
  *last_token = host[4 + DM + 2];
  for (int i = 0; i < gamma; ++i) drafts_out[i] = host[4 + i];
  return DEL_OK;
}

}  // extern "C" (re-opened below: the static scratch array has C++ linkage)

// ---- the entry point that allocates nothing ---------------------------------------------------------
// Scratch of del_spec_sample_static: fixed-point weights of up to 2*8+1 logits rows of up to 32768
// tokens, one SampRow per row, and a few integers.  One copy per GPU the library runs on, held until the
// process ends.  Host code never uses the array's name as an address: the device address is looked up
// once per device with hipGetSymbolAddress and kept in static_scratch_ptr.
namespace {
constexpr int STATIC_MAX_VOCAB = 32768, STATIC_MAX_GAMMA = 8;
constexpr size_t ST_ROWS = 2 * STATIC_MAX_GAMMA + 1;
constexpr size_t ST_WF_BYTES = ST_ROWS * (size_t)STATIC_MAX_VOCAB * sizeof(unsigned long long);
constexpr size_t ST_SROW_BYTES = (ST_ROWS * sizeof(SampRow) + 255) / 256 * 256;
constexpr size_t ST_INT_BYTES = 256;
constexpr size_t ST_BYTES = ST_WF_BYTES + ST_SROW_BYTES + ST_INT_BYTES;
constexpr int ST_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[ST_BYTES];
namespace {
void* static_scratch_ptr[ST_MAX_DEVICES] = {};
std::mutex static_scratch_mutex;

// Device address of this GPU's copy of the scratch array (looked up at the first call on the device).
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= ST_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(static_scratch_mutex);
  if (!static_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    static_scratch_ptr[dev] = p;
  }
  *out = static_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

extern "C" {

del_status del_spec_sample_static(const float* q_logits, const float* p_logits, int64_t ld_logits, int32_t vocab,
                                  int32_t gamma, double temperature, double top_p, const float* uniforms,
                                  int32_t* out, void* hip_stream) {
  if (!p_logits || !uniforms || !out || gamma < 0 || vocab < 2 || (gamma > 0 && !q_logits) || ld_logits < vocab ||
      ld_logits % 4 != 0 || !sampling_args_ok(temperature, top_p))
    return DEL_E_ARG;
  // the kernels read the rows in 16-byte pieces
  if (((uintptr_t)p_logits | (uintptr_t)q_logits) % 16 != 0 || (uintptr_t)uniforms % 4 != 0 || (uintptr_t)out % 4 != 0)
    return DEL_E_ARG;
  if (vocab > STATIC_MAX_VOCAB || gamma > STATIC_MAX_GAMMA) return DEL_E_CAPACITY;
  hipStream_t s = (hipStream_t)hip_stream;
  void* base = nullptr;
  if (static_scratch(&base) != hipSuccess) return DEL_E_DEVICE;
  unsigned long long* wf_q = reinterpret_cast<unsigned long long*>(base);
  unsigned long long* wf_p = wf_q + (size_t)STATIC_MAX_GAMMA * STATIC_MAX_VOCAB;
  SampRow* rows_q = reinterpret_cast<SampRow*>(reinterpret_cast<char*>(base) + ST_WF_BYTES);
  SampRow* rows_p = rows_q + STATIC_MAX_GAMMA;
  int* ints = reinterpret_cast<int*>(reinterpret_cast<char*>(base) + ST_WF_BYTES + ST_SROW_BYTES);
  int* state = ints;          // [0] KV length, [1] pending token: the acceptance kernel adds to [0]
  int* drafts = ints + 4;     // [STATIC_MAX_GAMMA]
  const int64_t ldw = STATIC_MAX_VOCAB;
  // the array keeps the last call's contents: what must start at zero is cleared by a kernel (a caller
  // may be capturing this stream into a graph, where memset nodes are not to be used)
  if (launch_set_state(state, 0, 0, nullptr, 0, s) != hipSuccess) return DEL_E_DEVICE;
  if (gamma > 0 && launch_samp_rowstats(q_logits, ld_logits, vocab, gamma, temperature, top_p, wf_q, ldw, rows_q,
                                        uniforms, drafts, nullptr, nullptr, s) != hipSuccess)
    return DEL_E_DEVICE;
  if (launch_samp_rowstats(p_logits, ld_logits, vocab, gamma + 1, temperature, top_p, wf_p, ldw, rows_p, nullptr,
                           nullptr, nullptr, nullptr, s) != hipSuccess)
    return DEL_E_DEVICE;
  if (launch_samp_accept(q_logits, wf_q, rows_q, p_logits, wf_p, rows_p, ld_logits, ldw, vocab, gamma, drafts,
                         uniforms + gamma, uniforms + 2 * gamma, state, nullptr, 0, out, s) != hipSuccess)
    return DEL_E_DEVICE;
  return DEL_OK;
}

del_status del_layer_stats(const del_ctx* ctx, del_stats* out) {
  if (!ctx || !out) return DEL_E_ARG;
  const int L = ctx->L;
  out->n_layers = L; out->rounds = ctx->rounds;
  out->next_E = ctx->pol.next_E; out->next_gamma = ctx->pol.next_gamma;
  out->last_E = ctx->last_E; out->last_gamma = ctx->last_gamma; out->last_u = ctx->last_u; out->last_n = ctx->last_n;
  out->S_n = ctx->pol.Sn;
  for (int l = 0; l <= L; ++l) {
    if (out->S_c) out->S_c[l] = ctx->pol.Sc[l];
    if (out->alpha) out->alpha[l] = ctx->pol.alpha[l];
    if (out->last_c) out->last_c[l] = ctx->last_c[l];
    if (out->tau) out->tau[l] = ctx->pol.tau[l];
    if (out->S_tcs) out->S_tcs[l] = ctx->pol.St[l];
    if (out->S_fcs) out->S_fcs[l] = ctx->pol.Sf[l];
  }
  out->last_stopped = ctx->last_stopped;
  if (out->last_conf) memcpy(out->last_conf, ctx->last_conf.data(), ctx->last_conf.size() * 4);
  if (out->last_draft_conf) memcpy(out->last_draft_conf, ctx->last_draft_conf.data(), ctx->last_draft_conf.size() * 4);
  if (out->last_shadow) memcpy(out->last_shadow, ctx->last_shadow.data(), ctx->last_shadow.size() * 4);
  if (out->last_draft)
    for (int i = 0; i < ctx->cfg.d_max; ++i) out->last_draft[i] = ctx->last_draft[i];
  return DEL_OK;
}

del_status del_set_layer_stats(del_ctx* ctx, const del_stats* in) {
  if (!ctx || !in || !in->S_c) return DEL_E_ARG;
  if (!(in->S_n > 0.0)) return DEL_E_ARG;
  // every input is checked before anything is changed: an error leaves the policy as it was
  const bool conf = in->S_tcs && in->S_fcs;
  for (int l = 1; l <= ctx->L; ++l) {
    if (!(in->S_c[l] >= 0.0)) return DEL_E_ARG;
    if (conf && (!(in->S_tcs[l] >= 0.0) || !(in->S_fcs[l] >= 0.0))) return DEL_E_ARG;
  }
  for (int l = 1; l <= ctx->L; ++l) {
    ctx->pol.Sc[l] = in->S_c[l];
    if (conf) {
      ctx->pol.St[l] = in->S_tcs[l];
      ctx->pol.Sf[l] = in->S_fcs[l];
    }
  }
  ctx->pol.Sn = in->S_n;
  ctx->pol.select();
  return DEL_OK;
}

del_status del_last_timings(const del_ctx* ctx, float* draft_ms, float* verify_ms, float* shadow_ms) {
  if (!ctx) return DEL_E_ARG;
  if (draft_ms) *draft_ms = ctx->t_draft;
  if (verify_ms) *verify_ms = ctx->t_verify;
  if (shadow_ms) *shadow_ms = ctx->t_shadow;
  return DEL_OK;
}

del_status del_debug_hidden(const del_ctx* c, int32_t layer, int32_t row, float* dst) {
  del_ctx* ctx = const_cast<del_ctx*>(c);
  if (!ctx || !dst || layer < 0 || layer > ctx->L || row < 0 || row >= ctx->hrows) return DEL_E_ARG;
  HIPCHK(hipStreamSynchronize(ctx->stream));
  HIPCHK(hipMemcpy(dst, ctx->hid_row(layer, row), (size_t)ctx->d * 4, hipMemcpyDeviceToHost));
  return DEL_OK;
}

del_status del_debug_logits(del_ctx* ctx, int32_t layer, int32_t row, float* dst) {
  if (!ctx || !dst || layer < 0 || layer > ctx->L || row < 0 || row >= ctx->hrows) return DEL_E_ARG;
  if (!ctx->all_loaded()) return DEL_E_STATE;
  GemmP p = head_gemm(ctx);
  p.X = ctx->hid_row(layer, row);
  p.Y = ctx->logits_dbg; p.ldy = ctx->NBv * 16;
  del_status st = gemm(ctx, p, EPI_STORE, 1, false);
  if (st != DEL_OK) return st;
  HIPCHK(hipStreamSynchronize(ctx->stream));
  HIPCHK(hipMemcpy(dst, ctx->logits_dbg, (size_t)ctx->V * 4, hipMemcpyDeviceToHost));
  return DEL_OK;
}

del_status del_debug_last_rows(const del_ctx* ctx, int32_t* rows) {
  if (!ctx || !rows) return DEL_E_ARG;
  *rows = ctx->last_rows;
  return DEL_OK;
}

del_status del_debug_state(const del_ctx* ctx, int32_t* kv_len, int32_t* pending_token) {
  if (!ctx) return DEL_E_ARG;
  if (kv_len) *kv_len = ctx->T;
  if (pending_token) *pending_token = ctx->pending;
  return DEL_OK;
}

del_status del_profile_enable(del_ctx* ctx, int32_t on) {
  if (!ctx) return DEL_E_ARG;
  HIPCHK(hipStreamSynchronize(ctx->stream));
  ctx->prof_on = on != 0;
  ctx->prof.clear();
  ctx->prof_used = 0;
  return DEL_OK;
}

del_status del_profile_read(const del_ctx* ctx, del_prof_entry* out, int32_t cap, int32_t* n) {
  if (!ctx || !n || (cap > 0 && !out)) return DEL_E_ARG;
  const int have = (int)ctx->prof.size();
  *n = have;
  for (int i = 0; i < have && i < cap; ++i) out[i] = ctx->prof[i];
  return DEL_OK;
}

del_status del_policy_step(int32_t n_layers, int32_t d_max, double omega, const int32_t* c, int32_t n,
                           const double* tcs, const double* fcs, double* S_c, double* S_n, double* S_tcs,
                           double* S_fcs, double* alpha, double* tau, int32_t* next_E, int32_t* next_gamma) {
  if (n_layers < 1 || d_max < 0 || !(omega >= 0.0 && omega <= 1.0) || !c || n < 0 || !S_c || !S_n || !alpha ||
      !next_E || !next_gamma)
    return DEL_E_ARG;
  const bool conf = tcs && fcs && S_tcs && S_fcs;
  Policy pol;
  pol.reset(n_layers, d_max, omega);
  std::vector<double> zero(n_layers + 1, 0.0);
  for (int l = 1; l <= n_layers; ++l) {
    pol.Sc[l] = S_c[l];
    if (conf) { pol.St[l] = S_tcs[l]; pol.Sf[l] = S_fcs[l]; }
  }
  pol.Sn = *S_n;
  pol.update(c, n, conf ? tcs : zero.data(), conf ? fcs : zero.data());
  for (int l = 1; l <= n_layers; ++l) {
    S_c[l] = pol.Sc[l];
    alpha[l] = pol.alpha[l];
    if (conf) { S_tcs[l] = pol.St[l]; S_fcs[l] = pol.Sf[l]; }
    if (tau) tau[l] = pol.tau[l];
  }
  *S_n = pol.Sn;
  *next_E = pol.next_E;
  *next_gamma = pol.next_gamma;
  return DEL_OK;
}

del_status del_debug_set_pending(del_ctx* ctx, int32_t token) {
  if (!ctx || token < 0 || token >= ctx->V) return DEL_E_ARG;
  if (ctx->phase != 1) return DEL_E_STATE;
  HIPCHK(launch_set_state(ctx->state, 0, -1, nullptr, token, ctx->stream));
  HIPCHK(hipStreamSynchronize(ctx->stream));
  ctx->pending = token;
  return DEL_OK;
}

del_status del_bench_stream_read(del_ctx* ctx, int64_t bytes, int32_t iters, float* ms_per_iter) {
  if (!ctx || !ms_per_iter || iters < 1 || bytes < 1024) return DEL_E_ARG;
  if ((size_t)bytes > ctx->arena_bytes) bytes = (int64_t)ctx->arena_bytes;
  HIPCHK(launch_stream_read(ctx->arena, bytes, ctx->sink, ctx->stream));  // warm-up
  HIPCHK(hipEventRecord(ctx->ev[0], ctx->stream));
  for (int i = 0; i < iters; ++i) HIPCHK(launch_stream_read(ctx->arena, bytes, ctx->sink, ctx->stream));
  HIPCHK(hipEventRecord(ctx->ev[1], ctx->stream));
  HIPCHK(hipStreamSynchronize(ctx->stream));
  float ms = 0.f;
  HIPCHK(hipEventElapsedTime(&ms, ctx->ev[0], ctx->ev[1]));
  *ms_per_iter = ms / iters;
  return DEL_OK;
}

del_status del_bench_gemv_parts(del_ctx* ctx, int32_t n_blocks, int32_t k_tiles, int32_t waves, int32_t parts,
                                int32_t iters, float* us_per_launch) {
  if (!ctx || !us_per_launch || iters < 1 || n_blocks < 1 || k_tiles < 1 || k_tiles > 480 || parts < 0 || parts > 7 ||
      (waves != 4 && waves != 8 && waves != 16))
    return DEL_E_ARG;
  const size_t mat = (size_t)n_blocks * k_tiles * 1024;
  if (mat > ctx->arena_bytes) return DEL_E_CAPACITY;
  // consecutive launches read different parts of the arena, cycling through at least 1 GiB where the
  // arena has it, so that no launch finds its matrix in a cache
  size_t span = ctx->arena_bytes < ((size_t)1 << 30) ? ctx->arena_bytes : ((size_t)1 << 30);
  if (span < mat) span = mat;
  const int nmat = (int)(span / mat);
  float* buf = nullptr;
  const size_t kf = (size_t)k_tiles * 32, nf = (size_t)n_blocks * 16;
  HIPCHK(hipMalloc((void**)&buf, (2 * kf + 2 * nf) * sizeof(float)));
  float *X = buf, *G = buf + kf, *R = buf + 2 * kf, *Y = R + nf;
  hipError_t e = hipMemsetAsync(buf, 0, (2 * kf + 2 * nf) * sizeof(float), ctx->stream);
  auto go = [&](int i) {
    return launch_gemv_parts((const char*)ctx->arena + (size_t)(i % nmat) * mat, X, G, R, Y, n_blocks, k_tiles, waves, parts,
                             ctx->stream);
  };
  for (int i = 0; i < 3 && e == hipSuccess; ++i) e = go(i);
  if (e == hipSuccess) e = hipEventRecord(ctx->ev[0], ctx->stream);
  for (int i = 0; i < iters && e == hipSuccess; ++i) e = go(i);
  if (e == hipSuccess) e = hipEventRecord(ctx->ev[1], ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev[0], ctx->ev[1]);
  (void)hipFree(buf);
  if (e != hipSuccess) return ctx->fail(e, "del_bench_gemv_parts");
  *us_per_launch = ms * 1e3f / iters;
  return DEL_OK;
}

del_status del_bench_mfma_rate(del_ctx* ctx, int32_t shape, int32_t n_acc, int32_t iters, float* ns_per_instruction) {
  if (!ctx || !ns_per_instruction || iters < 1 || iters > 10000000 || shape < 0 || shape > 1) return DEL_E_ARG;
  const bool ok = shape == 0 ? (n_acc == 2 || n_acc == 4 || n_acc == 8 || n_acc == 16) : (n_acc == 1 || n_acc == 2 || n_acc == 4);
  if (!ok) return DEL_E_ARG;
  float* buf = nullptr;
  const size_t n_init = 512 + 64 * 64, n_all = n_init + 256;
  HIPCHK(hipMalloc((void**)&buf, n_all * sizeof(float)));
  hipError_t e = hipMemsetAsync(buf, 0, n_all * sizeof(float), ctx->stream);
  if (e == hipSuccess) e = launch_mfma_rate(shape, n_acc, buf, buf + n_init, iters, ctx->stream);   // warm-up
  if (e == hipSuccess) e = hipEventRecord(ctx->ev[0], ctx->stream);
  if (e == hipSuccess) e = launch_mfma_rate(shape, n_acc, buf, buf + n_init, iters, ctx->stream);
  if (e == hipSuccess) e = hipEventRecord(ctx->ev[1], ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev[0], ctx->ev[1]);
  (void)hipFree(buf);
  if (e != hipSuccess) return ctx->fail(e, "del_bench_mfma_rate");
  *ns_per_instruction = ms * 1e6f / ((float)iters * (float)n_acc);   // one wave per SIMD: per wave = per SIMD
  return DEL_OK;
}

del_status del_bench_stream_copy(del_ctx* ctx, int64_t bytes, int32_t iters, float* ms_per_iter) {
  if (!ctx || !ms_per_iter || iters < 1 || bytes < 1024) return DEL_E_ARG;
  char* buf = nullptr;
  HIPCHK(hipMalloc((void**)&buf, (size_t)bytes * 2));
  hipError_t e = hipMemsetAsync(buf, 1, (size_t)bytes * 2, ctx->stream);
  if (e == hipSuccess) e = launch_stream_copy(buf, buf + bytes, bytes, ctx->stream);
  if (e == hipSuccess) e = hipEventRecord(ctx->ev[0], ctx->stream);
  for (int i = 0; i < iters && e == hipSuccess; ++i) e = launch_stream_copy(buf, buf + bytes, bytes, ctx->stream);
  if (e == hipSuccess) e = hipEventRecord(ctx->ev[1], ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev[0], ctx->ev[1]);
  (void)hipFree(buf);
  if (e != hipSuccess) return ctx->fail(e, "del_bench_stream_copy");
  *ms_per_iter = ms / iters;
  return DEL_OK;
}

}  // extern "C"
