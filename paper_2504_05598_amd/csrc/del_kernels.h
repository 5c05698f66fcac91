// Internal launcher interface between the host state machine (del_api.hip) and the
// gfx950 kernels (del_kernels.hip).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace del {

// ---- weight tiling -------------------------------------------------------------------
// A matrix [N, K] is stored as tiles of 16 rows x TK input features, 1 KiB each, in the
// order a 64-lane wavefront consumes them: lane l of tile (nb, kt) holds the KPL
// consecutive elements W[row(nb, l%16)][kt*TK + (l/16)*KPL ...].  bf16: KPL=8, TK=32 (this is
// also the A-operand layout of v_mfma_f32_16x16x32_bf16); fp32: KPL=4, TK=16.
// Rows and K are zero-padded to full tiles.
inline int kpl_of(int dtype) { return dtype == 1 ? 8 : 4; }
inline int tk_of(int dtype) { return 4 * kpl_of(dtype); }

// Row maps applied while tiling: which "virtual" row of the fused matrix a source row lands on.
enum RowMap {
  MAP_PLAIN = 0,  // v = base + n
  MAP_ROPE = 1,   // per head: strip t holds j = 8t..8t+7 (rows 0-7) and j + hd/2 (rows 8-15)
  MAP_GATE = 2,   // v = (n/8)*16 + n%8
  MAP_UP = 3      // v = (n/8)*16 + 8 + n%8
};

enum Epi { EPI_STORE = 0, EPI_RESID = 1, EPI_QKV = 2, EPI_SWIGLU = 3, EPI_ARGMAX = 4 };

struct GemmP {
  // weights
  const void* Wt;  // tiled
  int NB, KT;      // 16-row blocks, k tiles
  int N, K;        // valid rows / input features
  int wdtype;      // 0 fp32, 1 bf16
  // activations, vector-ALU path: fp32 rows [M][ldx]; optional gain [KT*TK]; optional RMS norm
  const float* X;
  int ldx, M;
  const float* gain;
  int rms;
  float eps;
  // activations, matrix-core path: hi/lo bf16 split tiles, per-row scale (nullable)
  const uint16_t* Xs;
  const float* rowscale;
  // epilogue
  float* Y; int ldy;            // STORE / RESID destination (first row of this call)
  const float* R; int ldr;      // RESID: residual source
  float* Q; int ldq;            // QKV: rotated queries [M][n_q*hd]
  void* Kc; void* Vc;           // QKV: this layer's caches [n_kv][Tcap][hd] (weight dtype)
  void* VcT; int TcapT;         // QKV, optional: the values also feature-major, [n_kv][hd][TcapT] (bf16)
  int n_q, n_kv, hd, Tcap;
  const int* state;             // state[0] = KV length T
  int ctx_len1;                 // 0: read T from state[0]; otherwise T + 1 as the host knows it (saves the kernel a
                                // dependent load ahead of its rotary-table and cache addresses)
  int row_off;                  // position of row mi is state[0] + row_off + mi
  const float2* rope;           // [Tcap][hd/2] (cos, sin)
  float* ACT; int ldact; int d_ffn;  // SWIGLU
  float* pval; int* pidx;       // ARGMAX partials [rows][NB]
  float* psum;                  // optional: sum of exp(logit - block max) per partial (confidence)
  int prow0;                    // first partial row of this call
  // matrix-core path only: the epilogue can also emit its result rows as the next GEMM's split
  // tiles (RESID: value * gain_out[n]; SWIGLU: the activation), plus, for RESID, the sum of
  // squares of the 16 results per token row (ssq_out[token][NB]) from which the consumer forms
  // the RMS scale (ssq_in / ssq_nb on its side).
  uint16_t* XsOut;
  const float* gain_out;
  float* ssq_out;
  const float* ssq_in; int ssq_nb;
  // wide path (many token rows per launch): XsOut holds one set of tiles per block of 16 token
  // rows, this many 16-bit elements apart
  long long xs_out_cb_stride;
  // vector path, one row: the input row is the attention output given as att_S per-split
  // softmax partials per head (max, sum, weighted values [hd]), merged while staging
  const float* att_PM; const float* att_PL; const float* att_PA;
  int att_S, att_stride, att_hd;
  // host side only: when both are set the launch records the kernel's own start and stop
  // timestamps into these events (per-kernel profiling)
  hipEvent_t ev_start, ev_stop;
  // host side only, wide GEMM: 1 = the two-stage form for every matrix (default 0: the four-deep form where it applies)
  int wide_form;
  // host side only, one-row GEMV: 1 = one row block per work-group for every matrix (default 0: several row blocks per
  // work-group where the shape allows)
  int rows_form;
};

struct AttnP {
  const float* Q; int ldq;      // [m][n_q*hd]
  const void* Kc; const void* Vc;  // this layer's caches
  const void* VcT; int TcapT;      // matrix-core kernel: the values feature-major, [n_kv][hd][TcapT]
  int kvdtype;
  int n_q, n_kv, hd, Tcap, m;
  const int* state; int row_off;
  int ctx_len1;                 // as in GemmP
  float* PM; float* PL; float* PA;  // partials [(mi*n_q+h)][nch_max] (+[hd])
  int nch_max;
  int ct;                       // cache rows per work-group (16, 32, 48 or 64)
  int qb;                       // query rows per batch (set by the launcher)
  int nsplit;                   // > 0: the partials come from the decode kernel, this many per row;
                                // < 0 (decode kernel, one split): write O / XsOut directly, no partials
  float* O; int ldo;            // combined output [m][n_q*hd]
  uint16_t* XsOut;              // optional: the same rows as split tiles (input of the O projection)
  long long xs_cb_stride;       // 16-bit elements between the tiles of consecutive blocks of 16 token rows
  int rw;                       // token rows per work-group of the register kernel (set by the launcher)
  int rps;                      // > 0: the partials come from the matrix-core kernel split into spans of at least
                                // this many cache rows (a multiple of 32); spans past the context hold nothing
};

hipError_t launch_gemm_valu(const GemmP& p, int epi, int waves, hipStream_t s);
// Which kernel the two launchers here take for p: the forms with several row blocks per work-group
// (gemv_rows_k: one row, bf16, 128, 160 or 256 k tiles, at least 256 row blocks; gemm_mfma_rows_k: up to 16 rows,
// 128 k tiles, at least 256 row blocks, any epilogue but the residual one), unless p.rows_form == 1.
bool gemv_rows_applies(const GemmP& p);
bool gemm_mfma_rows_applies(const GemmP& p, int epi, int col_blocks);
hipError_t launch_gemm_mfma(const GemmP& p, int epi, int waves, int col_blocks, hipStream_t s);
// Shadow-head GEMM with fused arg-max over R rows; partials are [R][*n_slabs].  form 4: the register-blocked
// kernel (needs KT % 4 == 0, otherwise the other one runs); any other value: one row block per wave.
hipError_t launch_head_gemm(const void* Wt, int NB, int KT, int N, const uint16_t* Xs, int R, const float* rowscale,
                            float* pval, int* pidx, float* psum, int* n_slabs, hipStream_t s,
                            hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, int form = 1);
// Many token rows at once (prefill): 8 row blocks x up to 256 token rows per work-group, the split
// activation tiles ([cb][kt] for p.M rows) staged through LDS.  epi: EPI_RESID, EPI_QKV or EPI_SWIGLU.
hipError_t launch_gemm_wide(const GemmP& p, int epi, hipStream_t s);
// rowscale[row] = 1 / sqrt(sum_b ssq[row][b] / K + eps) for rows < M.
hipError_t launch_rowscale(const float* ssq, int nb, int M, int K, float eps, float* rowscale, hipStream_t s);
hipError_t launch_prep_split(const float* src, int rows, int rows_per_group, int64_t group_stride,
                             int ld, int K, int KT, const float* gain, int rms, float eps,
                             uint16_t* Xs, float* rowscale, hipStream_t s);
hipError_t launch_attention(const AttnP& p, hipStream_t s);
// rows_per_wg > 1: that many consecutive token rows share a work-group's cache reads (prefill);
// the launcher rounds it down to what the shape's instantiation offers.
hipError_t launch_attention_decode(const AttnP& p, int S, hipStream_t s, int rows_per_wg = 1);
hipError_t launch_attention_merge(const AttnP& p, hipStream_t s);
// Causal attention of p.m token rows on the matrix cores (bf16 caches, head_dim 64 or 128); writes O and
// XsOut directly (no partials).  Needs VcT.
hipError_t launch_attention_flash(const AttnP& p, hipStream_t s);
// The same for m <= 16 token rows (verify), split over the context into S spans of at least rps_min cache rows
// (a multiple of 32): one partial per (row, head, split) in PM / PL / PA, to be merged by launch_attention_merge.
hipError_t launch_attention_flash_split(const AttnP& p, int S, int rps_min, hipStream_t s);
bool attention_decode_supported(int kvdtype, int hd, int G);
hipError_t launch_embed(const void* Et, int wdtype, int KT, int vocab, const int* ids, int m,
                        float* out, int ld, int d_model, hipStream_t s);
// psum / out_conf may be null; out_conf[row] = soft-max probability of the arg-max token.
// emb_out (optional, rows == 1): also writes the winner's embedding row (d_model floats) there.
// note (optional, host-visible memory): row 0's confidence and `seq` as one 8-byte word (seq << 32 | bits).
hipError_t launch_argmax_finish(const float* pval, const int* pidx, const float* psum, int rows, int NB,
                                int* out_ids, float* out_conf, hipStream_t s, const void* Et = nullptr,
                                int wdtype = 0, int KT_e = 0, int vocab = 0, float* emb_out = nullptr,
                                int d_model = 0, unsigned long long* note = nullptr, unsigned seq = 0);
hipError_t launch_accept(int* state, const int* draft_ids, int* shadow_ids, int L, int m, int E,
                         int gamma, int* result, hipStream_t s);
hipError_t launch_set_state(int* state, int add_T, int set_T, const int* pending_src,
                            int pending_val, hipStream_t s);
hipError_t launch_tile_scatter(const void* src, int wdtype, int64_t row0, int64_t nrows, int64_t cols,
                               int map, int vbase, int hd, void* dst, int KT, hipStream_t s);
hipError_t launch_pad_gain(const float* src, int K, float* dst, int Kpad, hipStream_t s);
hipError_t launch_stream_copy(const void* src, void* dst, int64_t bytes, hipStream_t s);
hipError_t launch_stream_read(const void* base, int64_t bytes, float* sink, hipStream_t s);
// The one-row GEMV with parts switched off (bit 0 staging, bit 1 decode + FMA, bit 2 reduce + store) on an
// NB x KT tile matrix at W; X, G: KT*32 floats, R, Y: NB*16 floats.  KT <= 480, waves 4, 8 or 16.
// Issue rate of the bf16 matrix instructions (shape 0: 16x16x32 with 2, 4, 8 or 16 accumulators; 1: 32x32x16 with
// 1, 2 or 4): 256 work-groups of 4 waves run `iters` rounds of n_acc instructions each.
hipError_t launch_mfma_rate(int shape, int n_acc, const float* init, float* out, int iters, hipStream_t s);
hipError_t launch_gemv_parts(const void* W, const float* X, const float* G, const float* R, float* Y, int NB, int KT,
                             int waves, int parts, hipStream_t s);

// ---- speculative sampling (del_sampling.hip) ----
// What the sampling kernels keep of one logits row: token j is in the nucleus when the order key of
// its logit is above kstar, or equal to it with j <= tie_id; its probability is then
// weight[j] / Wkept with weight[j] = exp((z_j - zmax) / temperature) in 2^-44 fixed point.
struct SampRow {
  float zmax;
  unsigned kstar;
  int tie_id;
  int argmax;                    // greedy token (lowest id at the maximum)
  unsigned long long Wkept;      // mass of the nucleus
  unsigned long long Wtot;       // mass of all tokens
  float conf;                    // soft-max probability of the greedy token at temperature 1 (if asked for)
  int pad;
};
// draw_r (optional): also draw one token per row with the uniform number draw_r[row] into draw_tok[row]
// (and into *pending, if given; one row only).
// conf_out (optional): the greedy token's temperature-1 soft-max probability per row.
hipError_t launch_samp_rowstats(const float* Z, int64_t ldz, int V, int rows, double temperature, double top_p,
                                unsigned long long* WF, int64_t ldw, SampRow* out, const float* draw_r, int* draw_tok,
                                int* pending, float* conf_out, hipStream_t s);
hipError_t launch_samp_accept(const float* Zq, const unsigned long long* WFq, const SampRow* rq, const float* Zp,
                              const unsigned long long* WFp, const SampRow* rp, int64_t ldz, int64_t ldw, int V,
                              int gamma, const int* drafts, const float* unif_accept, const float* unif_last, int* state,
                              const int* shadow_ids, int n_shadow, int* result, hipStream_t s);


}  // namespace del
