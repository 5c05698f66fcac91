// gfx950 (CDNA4) kernels of the greedy self-speculative decode round.
//
// Everything here is bound by HBM traffic except the multi-row GEMMs, which use the matrix
// cores.  Weights are streamed exactly once per launch in 1 KiB wave-sized tiles (see
// del_kernels.h); activations stay fp32 on the vector path and are split into bf16 hi + lo
// halves (16 mantissa bits together) on the matrix-core path, accumulating in fp32.
#include "del_kernels.h"
#include <hip/hip_ext.h>

namespace del {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int MAXW = 16;  // waves per work-group at most
constexpr int QBMAX = 32;  // query rows per attention batch at most

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <int KPL> struct WDec;
template <> struct WDec<8> {  // 8 bf16 in a uint4
  static __device__ __forceinline__ void dec(const uint4& w, float* f) {
    f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xFFFF0000u);
    f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xFFFF0000u);
    f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xFFFF0000u);
    f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xFFFF0000u);
  }
};
template <> struct WDec<4> {  // 4 fp32 in a uint4
  static __device__ __forceinline__ void dec(const uint4& w, float* f) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
  }
};

// One embedding row out of the tiled table as fp32: a row's k tile is four 16-byte pieces (lanes g*16 + r
// of the tile), so every thread moves whole pieces.  kpl = 8 (bf16) or 4 (fp32) elements per piece.
__device__ __forceinline__ void gather_embedding(const void* Et, int kpl, int KT, int id, float* out, int d_model,
                                                 int tid, int nthr) {
  const int nb = id >> 4, r = id & 15;
  const int pieces = (d_model + kpl - 1) / kpl;
  for (int c = tid; c < pieces; c += nthr) {
    const int kt = c >> 2, g = c & 3;
    const uint4 raw = ((const uint4*)Et)[((size_t)nb * KT + kt) * 64 + g * 16 + r];
    float v[8];
    if (kpl == 8) {
      WDec<8>::dec(raw, v);
    } else {
      v[0] = __uint_as_float(raw.x); v[1] = __uint_as_float(raw.y);
      v[2] = __uint_as_float(raw.z); v[3] = __uint_as_float(raw.w);
    }
    const int k0 = c * kpl;
    if (k0 + kpl <= d_model) {
      *(float4*)(out + k0) = make_float4(v[0], v[1], v[2], v[3]);
      if (kpl == 8) *(float4*)(out + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      for (int e = 0; e < kpl && k0 + e < d_model; ++e) out[k0 + e] = v[e];
    }
  }
}

template <bool BF16> __device__ __forceinline__ void kv_store(void* base, size_t idx, float v) {
  if (BF16) ((uint16_t*)base)[idx] = f32_to_bf16_rne(v);
  else ((float*)base)[idx] = v;
}

// Eight consecutive features (a quarter of a 32-wide k tile) of one token row -> hi/lo split tiles.
// k8 = index of the group of eight (feature / 8).
__device__ __forceinline__ void split_store8(uint16_t* Xs, int k8, int token, const float* v) {
  uint32_t hi[4], lo[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const uint16_t h0 = f32_to_bf16_rne(v[e]), h1 = f32_to_bf16_rne(v[e + 1]);
    const uint16_t l0 = f32_to_bf16_rne(v[e] - bf16_bits_to_f32(h0));
    const uint16_t l1 = f32_to_bf16_rne(v[e + 1] - bf16_bits_to_f32(h1));
    hi[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    lo[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
  }
  uint16_t* d = Xs + (size_t)(k8 >> 2) * 1024 + ((k8 & 3) * 16 + token) * 8;
  *(uint4*)d = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  *(uint4*)(d + 512) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// ---------------------------------------------------------------------------------------
// Epilogues.  fin[mi][r] holds the finished 16 outputs of row-block nb for token row mi.
// ---------------------------------------------------------------------------------------
// WAVE: run by one wave on its own tile (thread index = lane) instead of the whole work-group.
// XsOut / ssq_out: where this block of 16 token rows puts its split tiles / sums of squares
// (token row mi of the block is row mi there).
template <int EPI, bool BF16KV, bool WAVE = false>
__device__ __forceinline__ void epilogue(const GemmP& p, int nb, float (*fin)[16], int m, int rowbase,
                                         uint16_t* XsOut, float* ssq_out) {
  const int nthr = WAVE ? 64 : blockDim.x;
  const int t0 = WAVE ? (threadIdx.x & 63) : threadIdx.x;
  if (EPI == EPI_STORE || EPI == EPI_RESID) {
    for (int tid = t0; tid < m * 16; tid += nthr) {
      const int mi = tid >> 4, r = tid & 15, n = nb * 16 + r;
      if (n < p.N) {
        float v = fin[mi][r];
        if (EPI == EPI_RESID) v += p.R[(size_t)(rowbase + mi) * p.ldr + n];
        p.Y[(size_t)(rowbase + mi) * p.ldy + n] = v;
        if (EPI == EPI_RESID && XsOut) fin[mi][r] = v;   // keep the residual-added value for the split below
      } else if (EPI == EPI_RESID && XsOut) {
        fin[mi][r] = 0.f;
      }
    }
    if (EPI == EPI_RESID && XsOut) {   // rowbase == 0 on this path (one block of <= 16 token rows)
      if (WAVE) __builtin_amdgcn_wave_barrier(); else __syncthreads();
      for (int tid = t0; tid < m * 2; tid += nthr) {
        const int mi = tid >> 1, half = tid & 1;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int n = nb * 16 + half * 8 + e;
          v[e] = fin[mi][half * 8 + e] * (p.gain_out ? p.gain_out[n] : 1.f);
        }
        split_store8(XsOut, nb * 2 + half, mi, v);
      }
      if (ssq_out) {
        for (int tid = t0; tid < m; tid += nthr) {
          float q = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) q += fin[tid][r] * fin[tid][r];
          ssq_out[(size_t)tid * p.NB + nb] = q;
        }
      }
    }
  } else if (EPI == EPI_QKV) {
    for (int tid = t0; tid < m * 16; tid += nthr) {
      const int mi = tid >> 4, r = tid & 15;
      const int hd = p.hd, half = hd >> 1;
      const int v0 = nb * 16;
      const int hh = v0 / hd, s0 = v0 - hh * hd;
      const int pos = (p.ctx_len1 ? p.ctx_len1 - 1 : p.state[0]) + p.row_off + rowbase + mi;
      if (hh < p.n_q + p.n_kv) {  // rotary heads: rows r and r+8 are the pair (j, j + hd/2)
        if (r < 8) {
          const int j = (s0 >> 4) * 8 + r;
          const float a = fin[mi][r], b = fin[mi][r + 8];
          const float2 cs = p.rope[(size_t)pos * half + j];
          const float ar = a * cs.x - b * cs.y;
          const float br = b * cs.x + a * cs.y;
          if (hh < p.n_q) {
            float* q = p.Q + (size_t)(rowbase + mi) * p.ldq + hh * hd;
            q[j] = ar;
            q[j + half] = br;
          } else {
            const size_t base = ((size_t)(hh - p.n_q) * p.Tcap + pos) * hd;
            kv_store<BF16KV>(p.Kc, base + j, ar);
            kv_store<BF16KV>(p.Kc, base + j + half, br);
          }
        }
      } else {
        const size_t base = ((size_t)(hh - p.n_q - p.n_kv) * p.Tcap + pos) * hd;
        kv_store<BF16KV>(p.Vc, base + s0 + r, fin[mi][r]);
        if (BF16KV && p.VcT)
          ((uint16_t*)p.VcT)[((size_t)(hh - p.n_q - p.n_kv) * hd + s0 + r) * p.TcapT + pos] = f32_to_bf16_rne(fin[mi][r]);
      }
    }
  } else if (EPI == EPI_SWIGLU) {
    for (int tid = t0; tid < m * 8; tid += nthr) {
      const int mi = tid >> 3, r = tid & 7, j = nb * 8 + r;
      float a = 0.f;
      if (j < p.d_ffn) {
        const float gt = fin[mi][r], up = fin[mi][r + 8];
        a = gt / (1.0f + expf(-gt)) * up;
        p.ACT[(size_t)(rowbase + mi) * p.ldact + j] = a;
      }
      if (XsOut) {   // gather the 8 activations of this token row in one lane, store them split
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = __shfl(a, (threadIdx.x & 56) + e);
        if (r == 0) split_store8(XsOut, nb, mi, v);
      }
    }
  } else if (EPI == EPI_ARGMAX) {
    for (int tid = t0; tid < m; tid += nthr) {
      const int mi = tid;
      float best = -INFINITY;
      int bi = 0x7FFFFFFF;
      for (int r = 0; r < 16; ++r) {
        const int n = nb * 16 + r;
        const float v = fin[mi][r];
        if (n < p.N && v > best) { best = v; bi = n; }  // strict >: lowest index wins ties
      }
      const size_t o = (size_t)(p.prow0 + rowbase + mi) * p.NB + nb;
      p.pval[o] = best;
      p.pidx[o] = bi;
      if (p.psum) {   // soft-max denominator of this block relative to its own maximum
        float se = 0.f;
        for (int r = 0; r < 16; ++r)
          if (nb * 16 + r < p.N) se += expf(fin[mi][r] - best);
        p.psum[o] = se;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Weight streaming.  A weight tile is read exactly once per launch, so it is fetched with a
// non-temporal load (no reuse: keeps the stream out of the way of the cached activations),
// and every wave owns a contiguous span of the k tiles of its row block.
// ---------------------------------------------------------------------------------------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int GU = 4;  // tiles in flight per wave and pipeline stage (x2: current + next)

// The k tiles of a row block are split over the waves in whole groups of `grp` tiles, as evenly as the
// group count allows; only the last wave can be left with fewer than `grp` tiles at its end.  (A
// remainder is loaded tile by tile with its latency exposed, so a split in tiles, which leaves one in
// every wave, costs about two memory latencies per launch.)
__device__ __forceinline__ void wave_span(int KT, int nw, int wave, int grp, int& lo, int& hi) {
  const int G = KT / grp;
  lo = (G * wave / nw) * grp;
  hi = wave == nw - 1 ? KT : (G * (wave + 1) / nw) * grp;
}

// ---------------------------------------------------------------------------------------
// The input row of the one-row output projection is the attention output, handed over as att_S <= ATT_SMAX
// per-split softmax partials (max, sum, weighted values): merged while the row is staged.  Request and merge
// are separate steps: all loads of a lane's four features go out at once, with the split index clamped
// instead of a branch around the load, so that a caller can put its weight-tile requests between the two and
// wait for the partials alone; the sums run over the splits in ascending order.
// ---------------------------------------------------------------------------------------
constexpr int ATT_SMAX = 8;
struct AttReq {
  float pm[ATT_SMAX], pl[ATT_SMAX];
  float4 pa[ATT_SMAX];
};
__device__ __forceinline__ void att_request(const GemmP& p, int k, AttReq& r) {
  const int kc = min(k, p.K - 4);            // features past K (padding) merge to zero: any valid address will do
  const int h = kc / p.att_hd, d = kc - h * p.att_hd;
  const size_t row = (size_t)h * p.att_stride;
#pragma unroll
  for (int s = 0; s < ATT_SMAX; ++s) {
    const int sc = min(s, p.att_S - 1);
    r.pm[s] = p.att_PM[row + sc];
    r.pl[s] = p.att_PL[row + sc];
    r.pa[s] = *(const float4*)(p.att_PA + (row + sc) * p.att_hd + d);
  }
}
__device__ __forceinline__ float4 att_merge(const GemmP& p, int k, const AttReq& r) {
  float mx = -INFINITY;
#pragma unroll
  for (int s = 0; s < ATT_SMAX; ++s)
    if (s < p.att_S) mx = fmaxf(mx, r.pm[s]);
  float L = 0.f;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int s = 0; s < ATT_SMAX; ++s)
    if (s < p.att_S) {
      const float ms = r.pm[s];
      const float c = ms > -INFINITY ? expf(ms - mx) : 0.f;
      L += c * r.pl[s];
      a.x += c * r.pa[s].x; a.y += c * r.pa[s].y; a.z += c * r.pa[s].z; a.w += c * r.pa[s].w;
    }
  const float inv = 1.0f / L;
  return k < p.K ? make_float4(a.x * inv, a.y * inv, a.z * inv, a.w * inv) : make_float4(0.f, 0.f, 0.f, 0.f);
}

// ---------------------------------------------------------------------------------------
// Vector-ALU GEMV (M = 1) / skinny GEMM (M = 2; 4 and 8 with 32-bit weights): one work-group per 16-row block; each
// lane accumulates one weight row over its wave's span of k tiles, fp32 throughout.
// M = 1 (the draft path): the gained input row is staged once in LDS (dynamic, KT*TK floats)
// while the first weight tiles are already in flight; M > 1 reads the rows through the cache.
// ---------------------------------------------------------------------------------------
// One weight tile (16 rows x TK inputs, this lane's KPL elements) times the M input rows.
template <int KPL, int M>
__device__ __forceinline__ void valu_tile(const uint4& w, int kt, int g, const float* xs, const GemmP& p, bool has_gain,
                                          float* acc, float* ss) {
  constexpr int TK = 4 * KPL;
  float wf[KPL];
  WDec<KPL>::dec(w, wf);
  const int k0 = kt * TK + g * KPL;
  if (M == 1) {
#pragma unroll
    for (int e = 0; e < KPL; e += 4) {
      const float4 t = *(const float4*)(xs + k0 + e);
      acc[0] += wf[e] * t.x;
      acc[0] += wf[e + 1] * t.y;
      acc[0] += wf[e + 2] * t.z;
      acc[0] += wf[e + 3] * t.w;
    }
  } else {
    float gn[KPL];
#pragma unroll
    for (int e = 0; e < KPL; e += 4) {
      float4 t = has_gain ? *(const float4*)(p.gain + k0 + e) : make_float4(1.f, 1.f, 1.f, 1.f);
      gn[e] = t.x; gn[e + 1] = t.y; gn[e + 2] = t.z; gn[e + 3] = t.w;
    }
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const float* xr = p.X + (size_t)m * p.ldx + k0;
#pragma unroll
      for (int e = 0; e < KPL; e += 4) {
        const float4 t = *(const float4*)(xr + e);
        ss[m] += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
        acc[m] += wf[e] * (t.x * gn[e]);
        acc[m] += wf[e + 1] * (t.y * gn[e + 1]);
        acc[m] += wf[e + 2] * (t.z * gn[e + 2]);
        acc[m] += wf[e + 3] * (t.w * gn[e + 3]);
      }
    }
  }
}

// Waves per work-group by the number of input rows: every row adds an accumulator, a sum of squares and its
// share of the input row to a lane's registers, so the several-row forms run with fewer, larger-register waves
// (at 16 waves they spilled hundreds of registers).
template <int M> struct ValuWaves { static constexpr int max = M == 1 ? 16 : 4; };

template <int KPL, int M, int EPI>
__global__ void __launch_bounds__(64 * ValuWaves<M>::max) gemm_valu_k(GemmP p) {
  constexpr int TK = 4 * KPL;
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[MAXW][M][16];
  __shared__ float ssr[MAXW][M];
  __shared__ float fin[16][16];
  const int tid = threadIdx.x, nw = blockDim.x >> 6, wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 4;
  const int nb = blockIdx.x;
  float acc[M], ss[M];
#pragma unroll
  for (int m = 0; m < M; ++m) { acc[m] = 0.f; ss[m] = 0.f; }
  const bool has_gain = p.gain != nullptr;
  // this wave's span of k tiles: full groups of GU tiles (the last wave: plus a remainder of fewer than GU)
  int kt_lo, kt_hi;
  wave_span(p.KT, nw, wave, GU, kt_lo, kt_hi);
  const int ngroups = (kt_hi - kt_lo) / GU;
  const uint4* wp = (const uint4*)p.Wt + ((size_t)nb * p.KT + kt_lo) * 64 + lane;
  // Order of the first memory requests: the input row (it comes from the cache and is needed by every
  // wave before the first product), then two groups of GU weight tiles per wave (A: even groups, B: odd
  // groups).  Loads complete in order, so the row is in LDS and the barrier passed while the tiles are
  // still arriving, and every wave refills as soon as its own tiles are there; requested after the tiles,
  // the row would arrive behind the whole first burst of the grid and the memory pipe would run dry
  // while the work-group waits at the barrier.
  const int Kp = p.KT * TK, stride = blockDim.x * 4;
  float4 xv[4], gv[4];
  auto stage_load = [&](int base) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = base + j * stride;
      xv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      gv[j] = make_float4(1.f, 1.f, 1.f, 1.f);
      if (k < Kp) {
        if (p.att_S > 0) {
          // the input row is the attention output: merge the S per-split softmax partials here
          // (split by split, in a loop: the batched request of gemv_rows_k would cost this kernel, whose other
          // instantiations run at the register limit, spills)
          if (k < p.K) {
            const int h = k / p.att_hd, d = k - h * p.att_hd;
            const float* pm = p.att_PM + (size_t)h * p.att_stride;
            const float* pl = p.att_PL + (size_t)h * p.att_stride;
            float mx = -INFINITY;
            for (int sidx = 0; sidx < p.att_S; ++sidx) mx = fmaxf(mx, pm[sidx]);
            float L = 0.f;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int sidx = 0; sidx < p.att_S; ++sidx) {
              const float ms = pm[sidx];
              const float c = ms > -INFINITY ? expf(ms - mx) : 0.f;
              L += c * pl[sidx];
              const float4 t = *(const float4*)(p.att_PA + ((size_t)h * p.att_stride + sidx) * p.att_hd + d);
              a.x += c * t.x; a.y += c * t.y; a.z += c * t.z; a.w += c * t.w;
            }
            const float inv = 1.0f / L;
            xv[j] = make_float4(a.x * inv, a.y * inv, a.z * inv, a.w * inv);
          }
        } else {
          xv[j] = *(const float4*)(p.X + k);
        }
        if (has_gain) gv[j] = *(const float4*)(p.gain + k);
      }
    }
  };
  auto stage_store = [&](int base) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = base + j * stride;
      if (k < Kp) {
        const float4 x = xv[j], gg = gv[j];
        ss[0] += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        *(float4*)(xs + k) = make_float4(x.x * gg.x, x.y * gg.y, x.z * gg.z, x.w * gg.w);
      }
    }
  };
  if (M == 1) stage_load(tid * 4);
  uint4 ta[GU], tb[GU];
  if (ngroups > 0) {
#pragma unroll
    for (int u = 0; u < GU; ++u) ta[u] = ld_stream(wp + u * 64);
  }
  if (ngroups > 1) {
#pragma unroll
    for (int u = 0; u < GU; ++u) tb[u] = ld_stream(wp + (GU + u) * 64);
  }
  if (M == 1) {
    // four 16-byte pieces per thread and batch: one batch covers 16 floats x threads, i.e. the whole row
    // for every shape but the widest rows on the smaller work-groups
    stage_store(tid * 4);
    for (int base = tid * 4 + 4 * stride; base < Kp; base += 4 * stride) {
      stage_load(base);
      stage_store(base);
    }
    __syncthreads();
  }
  // Steady state: branch-free, and no register that a load is still filling is ever copied (a copy would
  // make the wave wait for every load in flight): group gi is used from A, A is refilled with group gi + 2,
  // then the same for B with gi + 1 and gi + 3, so two groups (2 * GU KiB per wave) stay in flight.
  auto use = [&](const uint4* tl, int gi) {
#pragma unroll
    for (int u = 0; u < GU; ++u) valu_tile<KPL, M>(tl[u], kt_lo + gi * GU + u, g, xs, p, has_gain, acc, ss);
  };
  auto fill = [&](uint4* tl, int gi) {
    const uint4* wn = wp + (size_t)gi * GU * 64;
#pragma unroll
    for (int u = 0; u < GU; ++u) tl[u] = ld_stream(wn + u * 64);
  };
  int gi = 0;
  for (; gi + 4 <= ngroups; gi += 2) {
    use(ta, gi);
    fill(ta, gi + 2);
    use(tb, gi + 1);
    fill(tb, gi + 3);
  }
  // one to three groups are left, the first two of them already requested
  const int left = ngroups - gi;
  if (left == 3) {
    use(ta, gi);
    fill(ta, gi + 2);
    use(tb, gi + 1);
    use(ta, gi + 2);
  } else if (left == 2) {
    use(ta, gi);
    use(tb, gi + 1);
  } else if (left == 1) {
    use(ta, gi);
  }
  for (int kt = kt_lo + ngroups * GU; kt < kt_hi; ++kt) {
    const uint4 w = ld_stream(wp + (size_t)(kt - kt_lo) * 64);
    valu_tile<KPL, M>(w, kt, g, xs, p, has_gain, acc, ss);
  }
#pragma unroll
  for (int m = 0; m < M; ++m) {
    acc[m] += __shfl_xor(acc[m], 16);
    acc[m] += __shfl_xor(acc[m], 32);
    if (M == 1) {  // every thread staged a distinct slice: reduce over the whole wave
      for (int o = 1; o < 64; o <<= 1) ss[m] += __shfl_xor(ss[m], o);
    } else {       // lanes of one 16-lane group read the same k range: reduce over the groups
      ss[m] += __shfl_xor(ss[m], 16);
      ss[m] += __shfl_xor(ss[m], 32);
    }
  }
  if (lane < 16) {
#pragma unroll
    for (int m = 0; m < M; ++m) red[wave][m][lane] = acc[m];
  }
  if (lane == 0) {
#pragma unroll
    for (int m = 0; m < M; ++m) ssr[wave][m] = ss[m];
  }
  __syncthreads();
  for (int t = tid; t < M * 16; t += blockDim.x) {
    const int mi = t >> 4, r = t & 15;
    float s = 0.f;
    for (int w = 0; w < nw; ++w) s += red[w][mi][r];
    if (p.rms) {
      float q = 0.f;
      for (int w = 0; w < nw; ++w) q += ssr[w][mi];
      s *= 1.0f / sqrtf(q / (float)p.K + p.eps);
    }
    fin[mi][r] = s;
  }
  __syncthreads();
  epilogue<EPI, KPL == 8>(p, nb, fin, M, 0, p.XsOut, p.ssq_out);
}

// ---------------------------------------------------------------------------------------
// One-row GEMV, several row blocks per work-group (bf16 weights, KT = 16 * NG * GUX k tiles: 64 * NG with groups
// of 4 tiles, 160 with NG = 2 groups of 5): the grid is one
// work-group of 16 waves per compute unit and work-group w takes the row blocks w, w + grid, ...  The input
// row is staged once per work-group instead of once per row block, and a wave's tile requests run on across
// the row blocks: each wave owns NG groups of 4 tiles of every row block and keeps two groups in flight in two
// named register sets; the set just used is refilled at once, with the row block's later groups or the next
// row block's first ones, so the reduction and epilogue of a row block run under the next block's loads.  The
// loop over row blocks has no request behind a condition (the last block is a call of its own without refills),
// which lets the compiler keep exact wait counts (a wave waits for one tile at a time).  Against one row block
// per work-group: 17.9 -> 16.8 us (QKV), 30.2 -> 28.3 us (gate/up), 41.0 -> 39.1 us (head) in the measurement
// form of both kernels.
// ---------------------------------------------------------------------------------------
constexpr int ROWS_WAVES = 16;

template <int NG, int EPI, int GUX = GU>
__global__ void __launch_bounds__(1024) gemv_rows_k(GemmP p) {
  static_assert(NG >= 2 && NG % 2 == 0, "the two register sets take the groups of a row block in turn");
  constexpr int KPL = 8, TK = 32;
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[2][ROWS_WAVES][16];
  __shared__ float ssr[ROWS_WAVES];
  __shared__ float fin[16][16];
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, g = lane >> 4;
  const int wg = blockIdx.x, nwg = gridDim.x;
  if (wg >= p.NB) return;                                // uniform, before any barrier
  const int nblk = (p.NB - wg + nwg - 1) / nwg;          // row blocks of this work-group (>= 1)
  const int KT = p.KT;                                   // = 16 * NG * GUX (groups of GUX tiles: 4, or 5 for 160 k tiles)
  const int lo_t = wave * NG * GUX;                      // this wave's k tiles of every row block: [lo_t, lo_t + NG * GUX)
  const bool has_gain = p.gain != nullptr;
  float ss = 0.f;
  // the input row first (it comes from the cache and every wave needs it before its first product), then tiles.
  // The row has KP = KT * 32 floats: NJ float4 per thread, the last one only for the threads that still fall
  // inside the row.  Where it is the attention output, the partials of the first float4 are requested here and
  // merged once the tile requests are out.
  constexpr int XSTRIDE = 64 * ROWS_WAVES * 4, KP = ROWS_WAVES * NG * GUX * TK, NJ = (KP + XSTRIDE - 1) / XSTRIDE;
  auto inside = [&](int j) { return (j + 1) * XSTRIDE <= KP || tid * 4 + j * XSTRIDE < KP; };
  const bool att = p.att_S > 0;
  float4 xv[NJ], gv[NJ];
  AttReq rq;
  if (att) {
    att_request(p, tid * 4, rq);
  } else {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      // (a thread past the row's end reads the row's last float4 and drops it: no branch around the load)
      xv[j] = *(const float4*)(p.X + min(tid * 4 + j * XSTRIDE, KP - 4));
      if (!inside(j)) xv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    gv[j] = has_gain ? *(const float4*)(p.gain + min(tid * 4 + j * XSTRIDE, KP - 4)) : make_float4(1.f, 1.f, 1.f, 1.f);
  const size_t blk_stride = (size_t)nwg * KT * 64;
  const uint4* wp = (const uint4*)p.Wt + ((size_t)wg * KT + lo_t) * 64 + lane;   // this wave's first tile of the current row block
  uint4 ta[GUX], tb[GUX];
  auto fill = [&](uint4* t, const uint4* src) {
#pragma unroll
    for (int u = 0; u < GUX; ++u) t[u] = ld_stream(src + u * 64);
  };
  fill(ta, wp);
  fill(tb, wp + GUX * 64);
  if (att) {
    xv[0] = att_merge(p, tid * 4, rq);
#pragma unroll
    for (int j = 1; j < NJ; ++j) {
      xv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (inside(j)) {
        att_request(p, tid * 4 + j * XSTRIDE, rq);
        xv[j] = att_merge(p, tid * 4 + j * XSTRIDE, rq);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const float4 x = xv[j], gg = gv[j];
    ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    if (inside(j)) *(float4*)(xs + tid * 4 + j * XSTRIDE) = make_float4(x.x * gg.x, x.y * gg.y, x.z * gg.z, x.w * gg.w);
  }
  for (int o = 1; o < 64; o <<= 1) ss += __shfl_xor(ss, o);
  if (lane == 0) ssr[wave] = ss;
  __syncthreads();
  float scale = 1.0f;
  if (p.rms) {
    float q = 0.f;
    for (int w = 0; w < ROWS_WAVES; ++w) q += ssr[w];
    scale = 1.0f / sqrtf(q / (float)p.K + p.eps);
  }
  int par = 0;
  float dummy[1] = {0.f};
  auto use = [&](const uint4* t, int gi, float* acc) {
#pragma unroll
    for (int u = 0; u < GUX; ++u) valu_tile<KPL, 1>(t[u], lo_t + gi * GUX + u, g, xs, p, false, acc, dummy);
  };
  // the finished row block: partial sums of the waves through LDS, then wave 0 alone runs the epilogue on its own
  // LDS patch while the other waves go on with the next row block (the patch is free again by then: wave 0 comes
  // back to it only after the next barrier)
  auto finish = [&](float a, int nb) {
    a += __shfl_xor(a, 16);
    a += __shfl_xor(a, 32);
    if (lane < 16) red[par][wave][lane] = a;
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the partial is in LDS
    __builtin_amdgcn_s_barrier();
    if (wave == 0) {
      if (lane < 16) {
        float s = 0.f;
        for (int w = 0; w < ROWS_WAVES; ++w) s += red[par][w][lane];
        fin[0][lane] = s * scale;
      }
      __builtin_amdgcn_wave_barrier();
      epilogue<EPI, true, true>(p, nb, fin, 1, 0, nullptr, nullptr);
      __builtin_amdgcn_wave_barrier();
    }
    par ^= 1;
  };
  // one row block; `more` (fixed per call site): the refills go on into the next row block
  auto block = [&](int nb, bool more) {
    float acc[1] = {0.f};
    const uint4* wn = wp + blk_stride;
#pragma unroll
    for (int gi = 0; gi < NG; gi += 2) {
      use(ta, gi, acc);
      __builtin_amdgcn_sched_barrier(0);
      if (gi + 2 < NG) fill(ta, wp + (size_t)(gi + 2) * GUX * 64);
      else if (more) fill(ta, wn);
      __builtin_amdgcn_sched_barrier(0);
      use(tb, gi + 1, acc);
      __builtin_amdgcn_sched_barrier(0);
      if (gi + 3 < NG) fill(tb, wp + (size_t)(gi + 3) * GUX * 64);
      else if (more) fill(tb, wn + GUX * 64);
      __builtin_amdgcn_sched_barrier(0);
    }
    finish(acc[0], nb);
    wp = wn;
  };
  int nb = wg;
  for (int b = 0; b + 1 < nblk; ++b, nb += nwg) block(nb, true);
  block(nb, false);
}

// ---------------------------------------------------------------------------------------
// Matrix-core skinny GEMM (bf16 weights): out[16 weight rows][16 token rows] per wave via
// v_mfma_f32_16x16x32_bf16, weights as the A operand straight from the tiled layout, token
// rows as the B operand from hi/lo split tiles ([cb][kt][hi|lo][lane][8], lane = 16*(k/8%4) +
// token).  Two MFMAs per tile (hi, lo).  blockIdx.y selects a block of 16 token rows.
// ---------------------------------------------------------------------------------------
template <int EPI>
__global__ void __launch_bounds__(1024) gemm_mfma_k(GemmP p) {
  constexpr int U = 4;
  __shared__ float red[MAXW][16][16];
  __shared__ float fin[16][16];
  __shared__ float scl[16];
  const int tid = threadIdx.x, nw = blockDim.x >> 6, wave = tid >> 6, lane = tid & 63;
  const int nb = blockIdx.x, cb = blockIdx.y;
  const int mvalid = min(16, p.M - cb * 16);
  const int token = lane & 15, g = lane >> 4;
  // Lanes of token rows beyond the valid ones read the tile of token row 0 of their k group
  // (same cache lines as the active lanes, no extra traffic, no divergent loads); their output
  // columns are never used.
  const int blane = token < mvalid ? lane : (lane & 48);
  int kt_lo, kt_hi;
  wave_span(p.KT, nw, wave, U, kt_lo, kt_hi);
  const int ngroups = (kt_hi - kt_lo) / U;
  const uint4* wp = (const uint4*)p.Wt + ((size_t)nb * p.KT + kt_lo) * 64 + lane;
  const uint4* xp = (const uint4*)p.Xs + ((size_t)cb * p.KT + kt_lo) * 128 + blane;
  floatx4 acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};   // hi and lo products, independent chains
  // two register sets (even and odd groups), never copied: a copy of a register that a load is still
  // filling would make the wave wait for every load in flight
  uint4 a0[U], h0[U], l0[U], a1[U], h1[U], l1[U];
  auto fill = [&](uint4* a, uint4* bh, uint4* bl, int gi) {
    const uint4* wn = wp + (size_t)gi * U * 64;
    const uint4* xn = xp + (size_t)gi * U * 128;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      a[u] = ld_stream(wn + u * 64);
      bh[u] = xn[u * 128];
      bl[u] = xn[u * 128 + 64];
    }
  };
  auto use = [&](const uint4* a, const uint4* bh, const uint4* bl) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, a[u]);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh[u]), acc, 0, 0, 0);
      acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl[u]), acc2, 0, 0, 0);
    }
  };
  if (ngroups > 0) fill(a0, h0, l0, 0);
  if (ngroups > 1) fill(a1, h1, l1, 1);
  if (p.ssq_in) {   // RMS scale per token row from the producer's per-block sums of squares
    for (int mi = wave; mi < mvalid; mi += nw) {
      float q = 0.f;
      for (int b = lane; b < p.ssq_nb; b += 64) q += p.ssq_in[(size_t)mi * p.ssq_nb + b];
      for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
      if (lane == 0) scl[mi] = 1.0f / sqrtf(q / (float)p.K + p.eps);
    }
  }
  // steady state: branch-free, two groups in flight
  int gi = 0;
  for (; gi + 4 <= ngroups; gi += 2) {
    use(a0, h0, l0);
    fill(a0, h0, l0, gi + 2);
    use(a1, h1, l1);
    fill(a1, h1, l1, gi + 3);
  }
  const int left = ngroups - gi;   // one to three groups, the first two already requested
  if (left == 3) {
    use(a0, h0, l0);
    fill(a0, h0, l0, gi + 2);
    use(a1, h1, l1);
    use(a0, h0, l0);
  } else if (left == 2) {
    use(a0, h0, l0);
    use(a1, h1, l1);
  } else if (left == 1) {
    use(a0, h0, l0);
  }
  for (int kt = kt_lo + ngroups * U; kt < kt_hi; ++kt) {
    const uint4 aw = ld_stream(wp + (size_t)(kt - kt_lo) * 64);
    const uint4 h = xp[(size_t)(kt - kt_lo) * 128], l = xp[(size_t)(kt - kt_lo) * 128 + 64];
    const bf16x8 av = __builtin_bit_cast(bf16x8, aw);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, h), acc, 0, 0, 0);
    acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, l), acc2, 0, 0, 0);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] += acc2[j];
  // D layout: lane holds D[4*(lane/16) + j][lane%16], j = 0..3 (rows = weight rows, cols = tokens)
#pragma unroll
  for (int j = 0; j < 4; ++j) red[wave][token][4 * g + j] = acc[j];
  __syncthreads();
  for (int t = tid; t < 256; t += blockDim.x) {
    const int mi = t >> 4, r = t & 15;
    if (mi < mvalid) {
      float s = 0.f;
      for (int w = 0; w < nw; ++w) s += red[w][mi][r];
      if (p.rowscale) s *= p.rowscale[cb * 16 + mi];
      if (p.ssq_in) s *= scl[mi];
      fin[mi][r] = s;
    }
  }
  __syncthreads();
  epilogue<EPI, true>(p, nb, fin, mvalid, cb * 16, p.XsOut, p.ssq_out);
}

// ---------------------------------------------------------------------------------------
// The matrix-core skinny GEMM with several row blocks per work-group (up to 16 token rows, KT = 128):
// as gemv_rows_k, one work-group of 16 waves per compute unit taking the row blocks w, w + grid, ...  A wave
// owns 8 k tiles of every row block; the split activation tiles of those 8 k tiles do not depend on the row
// block, so they are loaded once and stay in registers for all of the work-group's row blocks (the form
// above fetches them again with every weight tile: two of its three loads).  Weight tiles: two named sets
// of 4, refilled as soon as used, running on into the next row block.  Wave 0 sums the waves' 16x16 partials
// and runs the epilogue while the others go on.
// ---------------------------------------------------------------------------------------
template <int EPI>
__global__ void __launch_bounds__(1024) gemm_mfma_rows_k(GemmP p) {
  constexpr int NG = 2;
  __shared__ float red[2][ROWS_WAVES][16][16];
  __shared__ float fin[16][16];
  __shared__ float scl[16];
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int wg = blockIdx.x, nwg = gridDim.x;
  if (wg >= p.NB) return;                                // uniform, before any barrier
  const int nblk = (p.NB - wg + nwg - 1) / nwg;
  const int KT = p.KT;                                   // = 128
  const int mvalid = min(16, p.M);
  const int token = lane & 15, g = lane >> 4;
  const int blane = token < mvalid ? lane : (lane & 48);   // lanes of rows beyond the valid ones re-read token row 0
  const int lo_t = wave * NG * GU;
  // this wave's activation tiles (high and low parts) for its 8 k tiles: loaded once
  uint4 bh[NG * GU], bl[NG * GU];
  const uint4* xp = (const uint4*)p.Xs + (size_t)lo_t * 128 + blane;
#pragma unroll
  for (int i = 0; i < NG * GU; ++i) {
    bh[i] = xp[i * 128];
    bl[i] = xp[i * 128 + 64];
  }
  const size_t blk_stride = (size_t)nwg * KT * 64;
  const uint4* wp = (const uint4*)p.Wt + ((size_t)wg * KT + lo_t) * 64 + lane;
  // weight tiles: two named sets of HS = 2 tiles (the activation tiles leave registers for no more: 16 waves per
  // work-group cap a wave at 128), each refilled as soon as used
  constexpr int HS = 2;
  uint4 ta[HS], tb[HS];
  auto fill = [&](uint4* t, const uint4* src) {
#pragma unroll
    for (int u = 0; u < HS; ++u) t[u] = ld_stream(src + u * 64);
  };
  fill(ta, wp);
  fill(tb, wp + HS * 64);
  if (p.ssq_in) {   // RMS scale per token row from the producer's per-block sums of squares
    for (int mi = wave; mi < mvalid; mi += ROWS_WAVES) {
      float q = 0.f;
      for (int b = lane; b < p.ssq_nb; b += 64) q += p.ssq_in[(size_t)mi * p.ssq_nb + b];
      for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
      if (lane == 0) scl[mi] = 1.0f / sqrtf(q / (float)p.K + p.eps);
    }
  }
  __syncthreads();
  int par = 0;
  auto finish = [&](const floatx4& acc, int nb) {
    // D layout: lane holds D[4*(lane/16) + j][lane%16], j = 0..3 (rows = weight rows, cols = tokens)
#pragma unroll
    for (int j = 0; j < 4; ++j) red[par][wave][token][4 * g + j] = acc[j];
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = lane + 64 * i, mi = t >> 4, r = t & 15;
        if (mi < mvalid) {
          float s = 0.f;
          for (int w = 0; w < ROWS_WAVES; ++w) s += red[par][w][mi][r];
          if (p.rowscale) s *= p.rowscale[mi];
          if (p.ssq_in) s *= scl[mi];
          fin[mi][r] = s;
        }
      }
      __builtin_amdgcn_wave_barrier();
      epilogue<EPI, true, true>(p, nb, fin, mvalid, 0, p.XsOut, p.ssq_out);
      __builtin_amdgcn_wave_barrier();
    }
    par ^= 1;
  };
  auto block = [&](int nb, bool more) {
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    const uint4* wn = wp + blk_stride;
    auto use = [&](const uint4* t, int i0) {
#pragma unroll
      for (int u = 0; u < HS; ++u) {
        const bf16x8 av = __builtin_bit_cast(bf16x8, t[u]);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh[i0 + u]), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl[i0 + u]), acc, 0, 0, 0);
      }
    };
    constexpr int NT = NG * GU;   // this wave's tiles of a row block
#pragma unroll
    for (int i0 = 0; i0 < NT; i0 += 2 * HS) {
      use(ta, i0);
      __builtin_amdgcn_sched_barrier(0);
      if (i0 + 2 * HS < NT) fill(ta, wp + (size_t)(i0 + 2 * HS) * 64);
      else if (more) fill(ta, wn);
      __builtin_amdgcn_sched_barrier(0);
      use(tb, i0 + HS);
      __builtin_amdgcn_sched_barrier(0);
      if (i0 + 3 * HS < NT) fill(tb, wp + (size_t)(i0 + 3 * HS) * 64);
      else if (more) fill(tb, wn + HS * 64);
      __builtin_amdgcn_sched_barrier(0);
    }
    finish(acc, nb);
    wp = wn;
  };
  int nb = wg;
  for (int b = 0; b + 1 < nblk; ++b, nb += nwg) block(nb, true);
  block(nb, false);
}

// ---------------------------------------------------------------------------------------
// Shadow-head GEMM with a fused arg-max (Section 4.2: every layer's hidden states through the
// LM head in one pass): logits of R = L*(gamma+1) rows never leave the chip.  One work-group =
// 8 waves = a slab of 8 consecutive 16-row blocks of the head, times up to 16 column blocks of
// 16 token rows (blockIdx.y picks the group of column blocks).  Each wave streams its own row
// block once (non-temporal); the split activation tiles of the current k tile are staged in
// LDS (double-buffered) and shared by the 8 waves.  Emits per (row, slab) the best logit and
// its index; argmax_finish_k merges the slabs.  The positive per-row RMS scale cannot change an
// arg-max and is left out.
// ---------------------------------------------------------------------------------------
constexpr int HG_W = 8, HG_CB = 16;

__global__ void __launch_bounds__(512) head_gemm_k(const uint4* __restrict__ Wt, int NB, int KT, int N,
                                                   const uint4* __restrict__ Xs, int CB, int R,
                                                   const float* __restrict__ rowscale, float* pval, int* pidx,
                                                   float* psum, int NS) {
  extern __shared__ __align__(16) uint4 bs[];   // [2][HG_CB * 128]
  constexpr int U = 4;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int slab = blockIdx.x, cb0 = blockIdx.y * HG_CB;
  const int ncb = min(HG_CB, CB - cb0);
  const int nb = slab * HG_W + wave;
  const bool rowok = nb < NB;
  // loads are unconditional (clamped addresses) so that the steady-state loop has no branches
  // around memory operations; a wave beyond the last row block re-reads that block and its
  // candidates are masked below
  const uint4* wp = Wt + (size_t)(rowok ? nb : NB - 1) * KT * 64 + lane;
  floatx4 acc[HG_CB];
#pragma unroll
  for (int c = 0; c < HG_CB; ++c) acc[c] = (floatx4){0.f, 0.f, 0.f, 0.f};
  uint4 br[4], a[U], an[U];
  auto loadB = [&](int kt) {   // column blocks beyond ncb are not fetched (the condition is wave-uniform)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int idx = tid + 512 * j, cbi = idx >> 7;
      br[j] = cbi < ncb ? Xs[((size_t)(cb0 + cbi) * KT + kt) * 128 + (idx & 127)] : make_uint4(0, 0, 0, 0);
    }
  };
  auto storeB = [&](int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) bs[buf * (HG_CB * 128) + tid + 512 * j] = br[j];
  };
  // one k tile: prefetch the next activation tiles, multiply, hand them over through LDS
  auto tile = [&](const uint4& aw, int kt) {
    const int cur = kt & 1;
    loadB(min(kt + 1, KT - 1));
    const bf16x8 av = __builtin_bit_cast(bf16x8, aw);
    const uint4* bp = bs + cur * (HG_CB * 128) + lane;
#pragma unroll
    for (int c = 0; c < HG_CB; ++c) {
      if (c < ncb) {
        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bp[c * 128]), acc[c], 0, 0, 0);
        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bp[c * 128 + 64]), acc[c], 0, 0, 0);
      }
    }
    storeB(cur ^ 1);
    __syncthreads();
  };
  const int ngroups = KT / U;
  loadB(0);
  if (ngroups > 0) {
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = ld_stream(wp + u * 64);
  }
  storeB(0);
  __syncthreads();
  for (int gi = 0; gi + 1 < ngroups; ++gi) {
    const uint4* wn = wp + (size_t)(gi + 1) * U * 64;
#pragma unroll
    for (int u = 0; u < U; ++u) an[u] = ld_stream(wn + u * 64);
#pragma unroll
    for (int u = 0; u < U; ++u) tile(a[u], gi * U + u);
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = an[u];
  }
  if (ngroups > 0) {
#pragma unroll
    for (int u = 0; u < U; ++u) tile(a[u], (ngroups - 1) * U + u);
  }
  for (int kt = ngroups * U; kt < KT; ++kt) {
    const uint4 aw = ld_stream(wp + (size_t)kt * 64);
    tile(aw, kt);
  }
  // arg-max: lane holds rows 4g+j of its block for token lane%16 of every column block.  The
  // per-row RMS scale is positive, so it cannot change the arg-max; it is applied because the
  // stored maximum and the soft-max sums (confidence) are in logit units.
  float* wv = (float*)bs;                    // [HG_W][HG_CB][16]
  int* wi = (int*)(wv + HG_W * HG_CB * 16);
  float* ws = (float*)(wi + HG_W * HG_CB * 16);
  const int g = lane >> 4, token = lane & 15;
#pragma unroll
  for (int c = 0; c < HG_CB; ++c) {
    float best = -INFINITY;
    int bi = 0x7FFFFFFF;
    float v[4];
    const int row = (cb0 + c) * 16 + token;
    const float sc = (c < ncb && row < R && rowscale) ? rowscale[row] : 1.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = acc[c][j] * sc;
    if (c < ncb && rowok) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int n = nb * 16 + 4 * g + j;
        if (n < N && v[j] > best) { best = v[j]; bi = n; }
      }
    }
#pragma unroll
    for (int o = 16; o < 64; o <<= 1) {
      const float ov = __shfl_xor(best, o);
      const int oi = __shfl_xor(bi, o);
      if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    float se = 0.f;
    if (psum && c < ncb && rowok) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (nb * 16 + 4 * g + j < N) se += expf(v[j] - best);
    }
    if (psum) {
      se += __shfl_xor(se, 16);
      se += __shfl_xor(se, 32);
    }
    if (g == 0) {
      wv[(wave * HG_CB + c) * 16 + token] = best;
      wi[(wave * HG_CB + c) * 16 + token] = bi;
      ws[(wave * HG_CB + c) * 16 + token] = se;
    }
  }
  __syncthreads();
  if (tid < HG_CB * 16) {
    const int c = tid >> 4, t = tid & 15;
    const int row = (cb0 + c) * 16 + t;
    if (c < ncb && row < R) {
      float best = -INFINITY;
      int bi = 0x7FFFFFFF;
      for (int w = 0; w < HG_W; ++w) {   // ascending row blocks: strict > keeps the lowest index
        const float v = wv[(w * HG_CB + c) * 16 + t];
        const int ix = wi[(w * HG_CB + c) * 16 + t];
        if (v > best || (v == best && ix < bi)) { best = v; bi = ix; }
      }
      pval[(size_t)row * NS + slab] = best;
      pidx[(size_t)row * NS + slab] = bi;
      if (psum) {
        float se = 0.f;
        for (int w = 0; w < HG_W; ++w) {
          const float v = wv[(w * HG_CB + c) * 16 + t];
          if (v > -INFINITY) se += ws[(w * HG_CB + c) * 16 + t] * expf(v - best);
        }
        psum[(size_t)row * NS + slab] = se;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Shadow-head GEMM, register-blocked form.  What bounds the form above is LDS operand traffic: a wave
// owns one row block and reads every activation tile from LDS for a single matrix instruction (about
// 1 KiB of LDS reads per instruction, four SIMDs sharing one LDS port).  Here a wave owns H4_RB = 4 row
// blocks and H4_CB = 8 column blocks (128 accumulator registers), so that an activation tile read from
// LDS feeds 4 instructions, and the k range is split over the waves instead: work-group = the same
// slab of 8 row blocks, wave = (half of the slab, quarter of the k tiles).  Per step every quarter
// consumes its own k tile, whose activation tiles (4 x 8 x 2 KiB) are staged in LDS, double-buffered,
// one barrier per step (KT / 4 barriers per launch instead of KT).  The four quarters are summed
// through LDS at the end; output format as above (per row and slab: best logit, index, soft-max sum).
// Needs KT % 4 == 0.  blockIdx.y picks a group of 8 column blocks (128 token rows).
// ---------------------------------------------------------------------------------------
constexpr int H4_RB = 4, H4_CB = 8, H4_KQ = 4;
constexpr int H4_STAGE = H4_KQ * H4_CB * 128;   // uint4 per stage

__global__ void __launch_bounds__(512) head_gemm4_k(const uint4* __restrict__ Wt, int NB, int KT, int N,
                                                    const uint4* __restrict__ Xs, int CB, int R,
                                                    const float* __restrict__ rowscale, float* pval, int* pidx,
                                                    float* psum, int NS) {
  // two stages as separate arrays: the compiler then knows that the loads filling one stage do not touch
  // the stage being read (otherwise every LDS read after such a load waits for all of them)
  __shared__ __align__(16) uint4 st0[H4_STAGE];
  __shared__ __align__(16) uint4 st1[H4_STAGE];
  uint4* const bs = st0;   // the epilogue reuses stage 0
  // the wave index as a scalar: everything derived from it (row blocks, k quarter, staging sources) then lives
  // in scalar registers and an address is a scalar base plus the lane's 16 bytes; the accumulators leave
  // no vector registers for per-lane pointers
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int rg = wave & 1, kq = wave >> 1;
  const int slab = blockIdx.x, cb0 = blockIdx.y * H4_CB;
  const int ncb = min(H4_CB, CB - cb0);
  const int KTq = KT / H4_KQ, kt0 = kq * KTq;
  const int nb0 = slab * HG_W + rg * H4_RB;
  // loads are unconditional with clamped addresses (no branches around memory operations); row blocks
  // beyond the last one re-read it and are masked in the arg-max
  size_t wrow[H4_RB];   // first tile of this wave's k quarter in each of its row blocks (scalar)
#pragma unroll
  for (int r = 0; r < H4_RB; ++r) wrow[r] = ((size_t)min(nb0 + r, NB - 1) * KT + kt0) * 64;
  floatx4 acc[H4_RB][H4_CB];
#pragma unroll
  for (int r = 0; r < H4_RB; ++r)
#pragma unroll
    for (int c = 0; c < H4_CB; ++c) acc[r][c] = (floatx4){0.f, 0.f, 0.f, 0.f};
  // staging: element idx = tid + 512 j of a stage is (quarter idx / 1024, column block idx / 128 % 8, piece idx % 128)
  // Staging goes from global memory straight into LDS (no registers: the accumulators leave none to
  // spare): element idx = tid + 512 j of a stage is (quarter idx / 1024, column block idx / 128 % 8, piece
  // idx % 128); a wave's 64 lanes fill 64 consecutive 16-byte pieces.  A column block beyond ncb gets a
  // copy of block ncb - 1: its products are computed and never used.
  // (with tid = 64 wave + lane: quarter = j / 2, column block = wave / 2 + 4 (j % 2), piece = 64 (wave % 2) + lane)
  size_t bsrc[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) bsrc[h] = (size_t)(cb0 + min((wave >> 1) + 4 * h, ncb - 1)) * KT * 128 + (wave & 1) * 64;
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;
  auto stageB = [&](int s, uint4* stage) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      __builtin_amdgcn_global_load_lds((gptr_t)(Xs + (bsrc[j & 1] + (size_t)((j >> 1) * KTq + s) * 128) + lane),
                                       (lptr_t)(stage + wave * 64 + 512 * j), 16, 0, 0);
  };
  uint4 a0[H4_RB], a1[H4_RB];
  auto fillA = [&](uint4* a, int s) {
#pragma unroll
    for (int r = 0; r < H4_RB; ++r) a[r] = ld_stream(Wt + (wrow[r] + (size_t)s * 64) + lane);
  };
  // the activation tiles of column block c + 1 are read from LDS while the matrix pipe works on block c
  auto mma = [&](const uint4* a, const uint4* stage) {
    const uint4* bp = stage + kq * (H4_CB * 128) + lane;
    uint4 bh[2], bl[2];
    bh[0] = bp[0];
    bl[0] = bp[64];
#pragma unroll
    for (int c = 0; c < H4_CB; ++c) {
      const int cur = c & 1, nxt = cur ^ 1;
      if (c + 1 < H4_CB) {
        bh[nxt] = bp[(c + 1) * 128];
        bl[nxt] = bp[(c + 1) * 128 + 64];
      }
#pragma unroll
      for (int r = 0; r < H4_RB; ++r)
        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[r]), __builtin_bit_cast(bf16x8, bh[cur]),
                                                            acc[r][c], 0, 0, 0);
#pragma unroll
      for (int r = 0; r < H4_RB; ++r)
        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[r]), __builtin_bit_cast(bf16x8, bl[cur]),
                                                            acc[r][c], 0, 0, 0);
    }
    // schedule: two LDS reads, then eight matrix instructions, eight times over
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int c = 0; c < H4_CB; ++c) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * H4_RB, 0);
    }
  };
  // One step: request the next step's activation tiles into the other stage and the weight tiles of the
  // step after next into the register set that is free, multiply this step's, then wait for the staging
  // (the four weight loads behind it stay in flight) and meet the other waves.  Loads complete in order,
  // so waiting for the staging also waits for every older load: the weight tiles are therefore requested
  // two steps ahead and after the staging loads (three register sets), which gives them two steps to
  // arrive; requested at the end of a step into the set just used (two sets), they had one step, and a
  // step then lasted as long as a loaded HBM access.
  // (the fences pin this order: the wait counts on the four weight loads being the youngest)
  auto step = [&](const uint4* use, uint4* fill, int s, const uint4* cur, uint4* nxt) {
    stageB(min(s + 1, KTq - 1), nxt);
    __builtin_amdgcn_sched_barrier(0);
    fillA(fill, min(s + 2, KTq - 1));
    __builtin_amdgcn_sched_barrier(0);
    mma(use, cur);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F74);   // vmcnt(4): everything but the four loads just issued
    __builtin_amdgcn_s_barrier();
  };
  uint4 a2[H4_RB];
  stageB(0, st0);
  fillA(a0, 0);
  fillA(a1, min(1, KTq - 1));
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
  __builtin_amdgcn_s_barrier();
  int s = 0;
  for (; s + 6 <= KTq; s += 6) {   // stages alternate, register sets rotate: period 6
    step(a0, a2, s, st0, st1);
    step(a1, a0, s + 1, st1, st0);
    step(a2, a1, s + 2, st0, st1);
    step(a0, a2, s + 3, st1, st0);
    step(a1, a0, s + 4, st0, st1);
    step(a2, a1, s + 5, st1, st0);
  }
  const int rem = KTq - s;   // 0..5 steps left, starting again with set 0 and stage 0
  if (rem > 0) step(a0, a2, s, st0, st1);
  if (rem > 1) step(a1, a0, s + 1, st1, st0);
  if (rem > 2) step(a2, a1, s + 2, st0, st1);
  if (rem > 3) step(a0, a2, s + 3, st1, st0);
  if (rem > 4) step(a1, a0, s + 4, st0, st1);
  __syncthreads();
  // sum the four k quarters into the waves of quarter 0, one quarter at a time through LDS
  floatx4* red = (floatx4*)bs;   // [2 row groups][H4_RB][H4_CB][64 lanes]: 64 KiB = stage 0
  for (int q = 1; q < H4_KQ; ++q) {
    if (kq == q) {
#pragma unroll
      for (int r = 0; r < H4_RB; ++r)
#pragma unroll
        for (int c = 0; c < H4_CB; ++c) red[((rg * H4_RB + r) * H4_CB + c) * 64 + lane] = acc[r][c];
    }
    __syncthreads();
    if (kq == 0) {
#pragma unroll
      for (int r = 0; r < H4_RB; ++r)
#pragma unroll
        for (int c = 0; c < H4_CB; ++c) {
          const floatx4 v = red[((rg * H4_RB + r) * H4_CB + c) * 64 + lane];
          acc[r][c][0] += v[0]; acc[r][c][1] += v[1]; acc[r][c][2] += v[2]; acc[r][c][3] += v[3];
        }
    }
    __syncthreads();
  }
  // arg-max by the two waves of quarter 0: a lane holds rows 4g + j of its four row blocks for token
  // lane % 16 of every column block.  The per-row RMS scale is positive (it cannot change the arg-max);
  // it is applied because the stored maximum and the soft-max sums are in logit units.
  float* wv = (float*)bs;                    // [2][H4_CB][16]
  int* wi = (int*)(wv + 2 * H4_CB * 16);
  float* ws = (float*)(wi + 2 * H4_CB * 16);
  const int g = lane >> 4, token = lane & 15;
  if (kq == 0) {
#pragma unroll
    for (int c = 0; c < H4_CB; ++c) {
      const int row = (cb0 + c) * 16 + token;
      const float sc = (c < ncb && row < R && rowscale) ? rowscale[row] : 1.0f;
      float best = -INFINITY;
      int bi = 0x7FFFFFFF;
      if (c < ncb) {
#pragma unroll
        for (int r = 0; r < H4_RB; ++r)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int n = (nb0 + r) * 16 + 4 * g + j;
            const float v = acc[r][c][j] * sc;
            if (nb0 + r < NB && n < N && v > best) { best = v; bi = n; }   // ascending n: strict > keeps the lowest index
          }
      }
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
      float se = 0.f;
      if (psum && c < ncb) {
#pragma unroll
        for (int r = 0; r < H4_RB; ++r)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (nb0 + r < NB && (nb0 + r) * 16 + 4 * g + j < N) se += expf(acc[r][c][j] * sc - best);
        se += __shfl_xor(se, 16);
        se += __shfl_xor(se, 32);
      }
      if (g == 0) {
        wv[(rg * H4_CB + c) * 16 + token] = best;
        wi[(rg * H4_CB + c) * 16 + token] = bi;
        ws[(rg * H4_CB + c) * 16 + token] = se;
      }
    }
  }
  __syncthreads();
  if (tid < H4_CB * 16) {
    const int c = tid >> 4, tk = tid & 15;
    const int row = (cb0 + c) * 16 + tk;
    if (c < ncb && row < R) {
      float best = -INFINITY;
      int bi = 0x7FFFFFFF;
      for (int w = 0; w < 2; ++w) {
        const float v = wv[(w * H4_CB + c) * 16 + tk];
        const int ix = wi[(w * H4_CB + c) * 16 + tk];
        if (v > best || (v == best && ix < bi)) { best = v; bi = ix; }
      }
      pval[(size_t)row * NS + slab] = best;
      pidx[(size_t)row * NS + slab] = bi;
      if (psum) {
        float se = 0.f;
        for (int w = 0; w < 2; ++w) {
          const float v = wv[(w * H4_CB + c) * 16 + tk];
          if (v > -INFINITY) se += ws[(w * H4_CB + c) * 16 + tk] * expf(v - best);
        }
        psum[(size_t)row * NS + slab] = se;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Wide GEMM for passes over many token rows (prefill).  A work-group takes RBW row blocks of the
// matrix times 8 * CPW blocks of 16 token rows.  The weight tiles of a k tile (RBW KiB) are staged
// in LDS, double-buffered, and shared by the 8 waves; every wave owns CPW blocks of token rows,
// whose hi/lo activation tiles it reads straight into registers, so that one weight tile fetched
// from LDS feeds 2 * CPW matrix instructions.  Work-groups that share a slab of the matrix are
// given consecutive slots on one XCD (the slab then comes from that XCD's L2 after its first
// read).  Every wave hands its 16x16 results through a 1 KiB LDS patch of its own to the layer
// epilogues, block of token rows by block of token rows.
// ---------------------------------------------------------------------------------------
template <int EPI, int RBW, int CPW>
__global__ void __launch_bounds__(512) gemm_wide_k(GemmP p, int NS, int NCG) {
  extern __shared__ __align__(16) uint4 as[];   // [2][RBW * 64]; reused by the epilogue ([8 waves][256] floats)
  constexpr int CBW = 8 * CPW;
  constexpr int AL = RBW * 64 / 512;            // 16-byte pieces of the weight tiles per thread
  static_assert(RBW * 64 % 512 == 0 && AL >= 1 && RBW * 64 * 2 * 16 >= 8 * 1024, "RBW must be a multiple of 8");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // slot -> (slab, group of token-row blocks): the NCG groups of a slab follow each other on one XCD
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int cg = local % NCG, slab = (local / NCG) * 8 + xcd;
  if (slab >= NS) return;
  const int NB = p.NB, KT = p.KT;
  const int CB = (p.M + 15) >> 4;
  const int nb0 = slab * RBW, cb0 = cg * CBW + wave * CPW;
  const uint4* Wt = (const uint4*)p.Wt;
  const uint4* Xs = (const uint4*)p.Xs;
  floatx4 acc[RBW][CPW];
#pragma unroll
  for (int r = 0; r < RBW; ++r)
#pragma unroll
    for (int c = 0; c < CPW; ++c) acc[r][c] = (floatx4){0.f, 0.f, 0.f, 0.f};
  // addresses are clamped (row blocks past the matrix, token-row blocks past the pass) so that the
  // loop has no branches around memory operations; such results are dropped in the epilogue
  const uint4* wsrc[AL];
#pragma unroll
  for (int j = 0; j < AL; ++j) {
    const int idx = tid + 512 * j;
    wsrc[j] = Wt + (size_t)min(nb0 + (idx >> 6), NB - 1) * KT * 64 + (idx & 63);
  }
  const uint4* xsrc[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) xsrc[c] = Xs + (size_t)min(cb0 + c, CB - 1) * KT * 128 + lane;
  uint4 ar[AL], bh[CPW], bl[CPW], bhn[CPW], bln[CPW];
#pragma unroll
  for (int j = 0; j < AL; ++j) ar[j] = wsrc[j][0];
#pragma unroll
  for (int c = 0; c < CPW; ++c) { bh[c] = xsrc[c][0]; bl[c] = xsrc[c][64]; }
#pragma unroll
  for (int j = 0; j < AL; ++j) as[tid + 512 * j] = ar[j];
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1, nx = min(kt + 1, KT - 1);
#pragma unroll
    for (int j = 0; j < AL; ++j) ar[j] = wsrc[j][(size_t)nx * 64];
#pragma unroll
    for (int c = 0; c < CPW; ++c) { bhn[c] = xsrc[c][(size_t)nx * 128]; bln[c] = xsrc[c][(size_t)nx * 128 + 64]; }
    const uint4* ap = as + cur * (RBW * 64) + lane;
#pragma unroll
    for (int r = 0; r < RBW; ++r) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, ap[r * 64]);
#pragma unroll
      for (int c = 0; c < CPW; ++c) {
        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh[c]), acc[r][c], 0, 0, 0);
        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl[c]), acc[r][c], 0, 0, 0);
      }
    }
#pragma unroll
    for (int j = 0; j < AL; ++j) as[(cur ^ 1) * (RBW * 64) + tid + 512 * j] = ar[j];
#pragma unroll
    for (int c = 0; c < CPW; ++c) { bh[c] = bhn[c]; bl[c] = bln[c]; }
    __syncthreads();
  }
  // epilogue: lane holds rows 4g+j of a row block for token lane%16 of a block of token rows; each
  // wave works on an LDS patch of its own, so no barrier is needed below
  float (*fin)[16] = reinterpret_cast<float (*)[16]>(reinterpret_cast<float*>(as) + wave * 256);
  const int g = lane >> 4, token = lane & 15;
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    if (cb0 + c >= CB) break;
    const int rowbase = (cb0 + c) * 16;
    const int mvalid = min(16, p.M - rowbase);
    const float sc = (p.rowscale && token < mvalid) ? p.rowscale[rowbase + token] : 1.0f;
    uint16_t* xs_out = p.XsOut ? p.XsOut + (size_t)(cb0 + c) * p.xs_out_cb_stride : nullptr;
    float* ssq_out = p.ssq_out ? p.ssq_out + (size_t)rowbase * p.NB : nullptr;
#pragma unroll
    for (int r = 0; r < RBW; ++r) {
      const int nb = nb0 + r;
      if (nb < NB) {
#pragma unroll
        for (int j = 0; j < 4; ++j) fin[token][4 * g + j] = acc[r][c][j] * sc;
        __builtin_amdgcn_wave_barrier();
        epilogue<EPI, true, true>(p, nb, fin, mvalid, rowbase, xs_out, ssq_out);
        __builtin_amdgcn_wave_barrier();
      }
    }
  }
}

// One wave per token row: the RMS scale from the per-block sums of squares a RESID epilogue left.
__global__ void __launch_bounds__(256) rowscale_k(const float* ssq, int nb, int M, int K, float eps, float* rowscale) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= M) return;
  float q = 0.f;
  for (int b = lane; b < nb; b += 64) q += ssq[(size_t)row * nb + b];
  for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
  if (lane == 0) rowscale[row] = 1.0f / sqrtf(q / (float)K + eps);
}

// The same wide GEMM with the loads four k tiles deep.  In the form above every k tile waits for a memory
// latency: the weight tile is stored to LDS, and the activation registers are copied from a "next" set, inside
// the iteration that requested them.  Here both sit in rings of 4 register sets that are never copied (a copy of
// a register that a load is still filling waits for every load in flight): iteration kt requests tile kt + 3,
// multiplies tile kt and passes the weight tile of kt + 1, requested two iterations earlier, on to LDS (two
// stages).  Needs KT % 4 == 0 (the rings are unrolled) and RBW == 8 (one 16-byte piece of the weight tiles per thread).
template <int EPI, int RBW, int CPW>
__global__ void __launch_bounds__(512) gemm_wide4_k(GemmP p, int NS, int NCG) {
  static_assert(RBW == 8, "one piece of the weight tiles per thread and stage");
  constexpr int CBW = 8 * CPW;
  __shared__ __align__(16) uint4 as0[RBW * 64];   // reused by the epilogue ([8 waves][256] floats)
  __shared__ __align__(16) uint4 as1[RBW * 64];
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int cg = local % NCG, slab = (local / NCG) * 8 + xcd;
  if (slab >= NS) return;
  const int NB = p.NB, KT = p.KT;
  const int CB = (p.M + 15) >> 4;
  const int nb0 = slab * RBW, cb0 = cg * CBW + wave * CPW;
  const uint4* Wt = (const uint4*)p.Wt;
  const uint4* Xs = (const uint4*)p.Xs;
  floatx4 acc[RBW][CPW];
#pragma unroll
  for (int r = 0; r < RBW; ++r)
#pragma unroll
    for (int c = 0; c < CPW; ++c) acc[r][c] = (floatx4){0.f, 0.f, 0.f, 0.f};
  // addresses are clamped (row blocks past the matrix, token-row blocks past the pass, k tiles past the end):
  // no branches around memory operations; such results are dropped or never used
  const size_t wrow = (size_t)min(nb0 + wave, NB - 1) * KT * 64;   // scalar: this wave stages row block nb0 + wave
  size_t xrow[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) xrow[c] = (size_t)min(cb0 + c, CB - 1) * KT * 128;
  // four register sets, named (not indexed) so that every access is to a fixed register
  uint4 ar0, ar1, ar2, ar3, bh0[CPW], bh1[CPW], bh2[CPW], bh3[CPW], bl0[CPW], bl1[CPW], bl2[CPW], bl3[CPW];
  auto request = [&](int kt, uint4& a, uint4* h, uint4* l) {
    const int k = min(kt, KT - 1);
    a = Wt[wrow + (size_t)k * 64 + lane];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      h[c] = Xs[xrow[c] + (size_t)k * 128 + lane];
      l[c] = Xs[xrow[c] + (size_t)k * 128 + 64 + lane];
    }
  };
  auto multiply = [&](const uint4* stage, const uint4* h, const uint4* l) {
    const uint4* ap = stage + lane;
#pragma unroll
    for (int r = 0; r < RBW; ++r) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, ap[r * 64]);
#pragma unroll
      for (int c = 0; c < CPW; ++c) {
        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, h[c]), acc[r][c], 0, 0, 0);
        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, l[c]), acc[r][c], 0, 0, 0);
      }
    }
  };
  request(0, ar0, bh0, bl0);
  request(1, ar1, bh1, bl1);
  request(2, ar2, bh2, bl2);
  as0[tid] = ar0;
  __syncthreads();
  // (the fences keep the requests at the top of an iteration: left alone, the scheduler sinks them below the
  // matrix instructions, next to their first use, and the ring then hides nothing)
  for (int kt = 0; kt < KT; kt += 4) {
    request(kt + 3, ar3, bh3, bl3);
    __builtin_amdgcn_sched_barrier(0);
    multiply(as0, bh0, bl0);
    as1[tid] = ar1;
    __syncthreads();
    request(kt + 4, ar0, bh0, bl0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(as1, bh1, bl1);
    as0[tid] = ar2;
    __syncthreads();
    request(kt + 5, ar1, bh1, bl1);
    __builtin_amdgcn_sched_barrier(0);
    multiply(as0, bh2, bl2);
    as1[tid] = ar3;
    __syncthreads();
    request(kt + 6, ar2, bh2, bl2);
    __builtin_amdgcn_sched_barrier(0);
    multiply(as1, bh3, bl3);
    as0[tid] = ar0;
    __syncthreads();
  }
  // epilogue: lane holds rows 4g+j of a row block for token lane%16 of a block of token rows; each
  // wave works on an LDS patch of its own, so no barrier is needed below
  float (*fin)[16] = reinterpret_cast<float (*)[16]>(reinterpret_cast<float*>(as0) + wave * 256);
  const int g = lane >> 4, token = lane & 15;
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    if (cb0 + c >= CB) break;
    const int rowbase = (cb0 + c) * 16;
    const int mvalid = min(16, p.M - rowbase);
    const float sc = (p.rowscale && token < mvalid) ? p.rowscale[rowbase + token] : 1.0f;
    uint16_t* xs_out = p.XsOut ? p.XsOut + (size_t)(cb0 + c) * p.xs_out_cb_stride : nullptr;
    float* ssq_out = p.ssq_out ? p.ssq_out + (size_t)rowbase * p.NB : nullptr;
#pragma unroll
    for (int r = 0; r < RBW; ++r) {
      const int nb = nb0 + r;
      if (nb < NB) {
#pragma unroll
        for (int j = 0; j < 4; ++j) fin[token][4 * g + j] = acc[r][c][j] * sc;
        __builtin_amdgcn_wave_barrier();
        epilogue<EPI, true, true>(p, nb, fin, mvalid, rowbase, xs_out, ssq_out);
        __builtin_amdgcn_wave_barrier();
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// fp32 rows -> bf16 hi/lo split tiles (+ optional gain and inverse RMS per row).
// One work-group per row.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) prep_split_k(const float* src, int rows_per_group, long long group_stride,
                                                    int ld, int K, int KT, const float* gain, int rms, float eps,
                                                    uint16_t* Xs, float* rowscale) {
  __shared__ float part[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int grp = row / rows_per_group, i = row - grp * rows_per_group;
  const float* x = src + (size_t)grp * group_stride + (size_t)i * ld;
  if (rms) {
    float ss = 0.f;
    for (int k = tid; k < K; k += 256) ss += x[k] * x[k];
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((tid & 63) == 0) part[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) rowscale[row] = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)K + eps);
  } else if (tid == 0) {
    rowscale[row] = 1.0f;
  }
  const int cb = row >> 4, token = row & 15;
  uint16_t* out = Xs + (size_t)cb * KT * 1024;
  for (int k = tid; k < KT * 32; k += 256) {
    float v = 0.f;
    if (k < K) v = gain ? x[k] * gain[k] : x[k];
    const uint16_t hi = f32_to_bf16_rne(v);
    const uint16_t lo = f32_to_bf16_rne(v - bf16_bits_to_f32(hi));
    const int kt = k >> 5, gg = (k & 31) >> 3, e = k & 7;
    const size_t off = (size_t)kt * 1024 + (gg * 16 + token) * 8 + e;
    out[off] = hi;
    out[off + 512] = lo;
  }
}

// ---------------------------------------------------------------------------------------
// Attention over the KV cache, split over the context: one work-group per (chunk of p.ct cache
// rows, kv head).  K and V of the chunk are fetched with all loads in flight at once, staged
// in LDS and shared by every query row of the head group (m token rows x n_q/n_kv heads).
// Emits softmax partials (max, sum, weighted values); attn_combine_k merges the chunks.
// Caches are [n_kv][Tcap][hd].
// ---------------------------------------------------------------------------------------
template <typename KVT>
__global__ void __launch_bounds__(256) attn_partial_k(AttnP p) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int EPW = 4 / sizeof(KVT);  // elements per 32-bit word
  constexpr int NLD = 4;                // 16-byte loads per thread and matrix (64 rows x 256 B at most)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.x, kvh = blockIdx.y;
  const int ct = p.ct;
  const int T0 = (p.ctx_len1 ? p.ctx_len1 - 1 : p.state[0]) + p.row_off;
  const int T_end = T0 + p.m;
  const int t0 = c * ct;
  if (t0 >= T_end) return;
  const int nt = min(ct, T_end - t0);
  const int hd = p.hd, G = p.n_q / p.n_kv, QR = p.m * G;
  const int QB = p.qb;        // query rows per batch (LDS is sized for it)
  const int wpr = hd / EPW;   // words per cache row
  const int ksw = wpr + 1;    // padded LDS row stride in words
  const int rb16 = wpr >> 2;  // 16-byte pieces per cache row
  uint32_t* Ks = (uint32_t*)smem;
  uint32_t* Vs = Ks + ct * ksw;
  float* Qs = (float*)(Vs + ct * ksw);
  float* Ss = Qs + QB * hd;
  const uint4* Kg = (const uint4*)((const KVT*)p.Kc + ((size_t)kvh * p.Tcap + t0) * hd);
  const uint4* Vg = (const uint4*)((const KVT*)p.Vc + ((size_t)kvh * p.Tcap + t0) * hd);
  const int npieces = nt * rb16;
  const float scale = 1.0f / sqrtf((float)hd);
  // few query rows (decode): fetch them now, together with K and V
  const bool qfast = QR * hd <= 4 * 256;
  float qreg[4];
  if (qfast) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = tid + 256 * j;
      qreg[j] = 0.f;
      if (i < QR * hd) {
        const int qi = i / hd, d = i - qi * hd;
        const int mi = qi / G, gi = qi - mi * G;
        qreg[j] = p.Q[(size_t)mi * p.ldq + (kvh * G + gi) * hd + d] * scale;
      }
    }
  }
  uint4 kr[NLD], vr[NLD];
#pragma unroll
  for (int j = 0; j < NLD; ++j) {
    const int i = tid + 256 * j;
    kr[j] = vr[j] = make_uint4(0, 0, 0, 0);
    if (i < npieces) { kr[j] = Kg[i]; vr[j] = Vg[i]; }
  }
#pragma unroll
  for (int j = 0; j < NLD; ++j) {
    const int i = tid + 256 * j;
    if (i < npieces) {
      const int row = i / rb16, w = (i - row * rb16) * 4;
      uint32_t* kd = Ks + row * ksw + w;
      uint32_t* vd = Vs + row * ksw + w;
      kd[0] = kr[j].x; kd[1] = kr[j].y; kd[2] = kr[j].z; kd[3] = kr[j].w;
      vd[0] = vr[j].x; vd[1] = vr[j].y; vd[2] = vr[j].z; vd[3] = vr[j].w;
    }
  }
  if (qfast) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = tid + 256 * j;
      if (i < QR * hd) Qs[i] = qreg[j];
    }
  }
  const int dpairs = hd >> 1;          // PV step: one thread per pair of value dims
  const int nslots = 256 / dpairs;     // query rows processed side by side in the PV step
  const int d2 = tid % dpairs, qslot = tid / dpairs;
  for (int qb = 0; qb < QR; qb += QB) {
    const int nq = min(QB, QR - qb);
    if (!qfast) {
      __syncthreads();
      for (int i = tid; i < nq * hd; i += 256) {
        const int qi = i / hd, d = i - qi * hd;
        const int qr = qb + qi, mi = qr / G, gi = qr - mi * G;
        Qs[qi * hd + d] = p.Q[(size_t)mi * p.ldq + (kvh * G + gi) * hd + d] * scale;
      }
    }
    __syncthreads();
    // scores: one (query row, cache row) pair per thread and step
    for (int pi = tid; pi < nq * ct; pi += 256) {
      const int qi = pi / ct, t = pi - qi * ct;
      const int mi = (qb + qi) / G;
      float s = -INFINITY;
      if (t < nt && t0 + t <= T0 + mi) {
        const uint32_t* krow = Ks + t * ksw;
        const float* qv = Qs + qi * hd;
        float a = 0.f;
        if (sizeof(KVT) == 2) {
          for (int w = 0; w < wpr; ++w) {
            const uint32_t kk = krow[w];
            a += qv[2 * w] * __uint_as_float(kk << 16);
            a += qv[2 * w + 1] * __uint_as_float(kk & 0xFFFF0000u);
          }
        } else {
          for (int w = 0; w < wpr; ++w) a += qv[w] * __uint_as_float(krow[w]);
        }
        s = a;
      }
      Ss[qi * ct + t] = s;
    }
    __syncthreads();
    // softmax numerators per row: one wave per query row, lanes over the cache rows
    for (int qi = wave; qi < nq; qi += 4) {
      float sv = lane < ct ? Ss[qi * ct + lane] : -INFINITY;
      float mx = sv;
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      const float pr = mx > -INFINITY ? expf(sv - mx) : 0.f;   // masked entries: exp(-inf) = 0
      float l = pr;
      for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
      if (lane < ct) Ss[qi * ct + lane] = pr;
      if (lane == 0) {
        const int qr = qb + qi, mi = qr / G, gi = qr - mi * G;
        const size_t prow = ((size_t)mi * p.n_q + kvh * G + gi) * p.nch_max + c;
        p.PM[prow] = mx;
        p.PL[prow] = l;
      }
    }
    __syncthreads();
    // weighted values
    for (int qi = qslot < nslots ? qslot : nq; qi < nq; qi += nslots) {
      const float* pr = Ss + qi * ct;
      float a0 = 0.f, a1 = 0.f;
      if (sizeof(KVT) == 2) {
        const uint32_t* vcol = Vs + d2;
        for (int t = 0; t < nt; ++t) {
          const uint32_t vv = vcol[t * ksw];
          a0 += pr[t] * __uint_as_float(vv << 16);
          a1 += pr[t] * __uint_as_float(vv & 0xFFFF0000u);
        }
      } else {
        const uint32_t* vcol = Vs + 2 * d2;
        for (int t = 0; t < nt; ++t) {
          a0 += pr[t] * __uint_as_float(vcol[t * ksw]);
          a1 += pr[t] * __uint_as_float(vcol[t * ksw + 1]);
        }
      }
      const int qr = qb + qi, mi = qr / G, gi = qr - mi * G;
      const size_t prow = ((size_t)mi * p.n_q + kvh * G + gi) * p.nch_max + c;
      *(float2*)(p.PA + prow * hd + 2 * d2) = make_float2(a0, a1);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Decode attention (one new token row): one work-group per (split of the context, kv head),
// 8 waves.  A wave-wide 16-byte load covers 64/LPR whole cache rows (LPR lanes per row); each
// lane keeps its slice of q in registers, scores are reduced over the LPR lanes of a row, and
// every lane group runs its own online softmax over the rows it sees, so K and V go from HBM
// to registers once with eight 1 KiB loads in flight per wave.  Lane groups and waves are
// merged at the end; the S per-split partials are merged by the consumer (the O projection's
// input staging), so no combine kernel runs on this path.
// ---------------------------------------------------------------------------------------
struct SoftAcc { float m, l; };

// RW > 1 (prefill): RW consecutive token rows share the work-group's cache reads; query q = r * G + g
// is head g of the kv group for token row mi0 + r and sees cache rows up to its own position only.
template <typename KVT, int HD, int G, int RW>
__global__ void __launch_bounds__(512) attn_decode_k(AttnP p) {
  constexpr int NQ = G * RW;
  constexpr int EPL = 16 / sizeof(KVT);   // elements per lane and load
  constexpr int LPR = HD / EPL;           // lanes per cache row
  constexpr int RPL = 64 / LPR;           // cache rows per wave-wide load
  constexpr int UL = 4;                   // loads in flight per wave, matrix and pipeline stage
  constexpr int NWV = RW > 1 ? 4 : 8;           // waves per work-group (launched with 64 * NWV threads)
  __shared__ float sm[NWV][NQ], sl[NWV][NQ];
  __shared__ float sa[NWV][NQ][HD];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int split = blockIdx.x, kvh = blockIdx.y, S = gridDim.x;
  const int mi0 = blockIdx.z * RW;                        // first token row of this work-group
  const int nrow = min(RW, p.m - mi0);                    // rows it really has
  const int T0 = (p.ctx_len1 ? p.ctx_len1 - 1 : p.state[0]) + p.row_off + mi0;   // row mi0 + r attends cache rows <= T0 + r
  const int T_end = T0 + nrow;
  const int rps = ((T_end + S - 1) / S + RPL - 1) / RPL * RPL;   // rows per split, whole loads
  const int t_lo = split * rps, t_hi = min(T_end, t_lo + rps);
  const int rs = lane / LPR, dl = lane % LPR;
  const float scale = 1.0f / sqrtf((float)HD);
  float q[NQ][EPL];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    // a ragged last group re-reads its last row; those queries' results are dropped
    const float* qp = p.Q + (size_t)(mi0 + min(g / G, nrow - 1)) * p.ldq + (size_t)(kvh * G + g % G) * HD + dl * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      const float4 t = *(const float4*)(qp + e);
      q[g][e] = t.x * scale; q[g][e + 1] = t.y * scale; q[g][e + 2] = t.z * scale; q[g][e + 3] = t.w * scale;
    }
  }
  float m[NQ], l[NQ], acc[NQ][EPL];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }
  // row groups of this wave: j = wave, wave + NWV, ...; group j covers rows t_lo + j*RPL ...
  const int ngrp = t_hi > t_lo ? (t_hi - t_lo + RPL - 1) / RPL : 0;
  const uint4* Kg = (const uint4*)((const KVT*)p.Kc + (size_t)kvh * p.Tcap * HD);
  const uint4* Vg = (const uint4*)((const KVT*)p.Vc + (size_t)kvh * p.Tcap * HD);
  // rows past t_hi (a ragged last group) are read from row t_hi - 1 and masked
  auto row_of = [&](int j) { return min(t_lo + j * RPL + rs, t_hi - 1); };
  uint4 kc[UL], vc[UL], kn[UL], vn[UL];
  auto consume = [&](const uint4& kk, const uint4& vv, int j) {
    const int trow = t_lo + j * RPL + rs;
    const bool valid = j < ngrp && trow < t_hi;
    float kf[EPL], vf[EPL];
    if (sizeof(KVT) == 2) { WDec<8>::dec(kk, kf); WDec<8>::dec(vv, vf); }
    else { WDec<4>::dec(kk, kf); WDec<4>::dec(vv, vf); }
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      float sdot = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) sdot += q[g][e] * kf[e];
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) sdot += __shfl_xor(sdot, o);
      if (valid && (RW == 1 || trow <= T0 + g / G)) {
        const float mn = fmaxf(m[g], sdot);
        const float c = expf(m[g] - mn);      // m = -inf at the first row: exp(-inf) = 0
        const float pr = expf(sdot - mn);
        l[g] = l[g] * c + pr;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = acc[g][e] * c + pr * vf[e];
        m[g] = mn;
      }
    }
  };
  if (ngrp > 0) {
    const int nit = (ngrp - wave + NWV * UL - 1) / (NWV * UL);   // iterations of this wave (may be <= 0)
    if (nit > 0) {
#pragma unroll
      for (int u = 0; u < UL; ++u) {
        const int j = min(wave + u * NWV, ngrp - 1);
        const size_t off = (size_t)row_of(j) * LPR + dl;
        kc[u] = Kg[off]; vc[u] = Vg[off];
      }
      for (int it = 0; it < nit; ++it) {
        const int j0 = wave + it * NWV * UL;
#pragma unroll
        for (int u = 0; u < UL; ++u) {   // next iteration's rows (clamped: re-reads the last group at the end)
          const int j = min(j0 + (UL + u) * NWV, ngrp - 1);
          const size_t off = (size_t)row_of(j) * LPR + dl;
          kn[u] = Kg[off]; vn[u] = Vg[off];
        }
#pragma unroll
        for (int u = 0; u < UL; ++u) consume(kc[u], vc[u], j0 + u * NWV);
#pragma unroll
        for (int u = 0; u < UL; ++u) { kc[u] = kn[u]; vc[u] = vn[u]; }
      }
    }
  }
  // merge the lane groups of a wave (same value dims, different rows) ...
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      const float m2 = __shfl_xor(m[g], o), l2 = __shfl_xor(l[g], o);
      const float M = fmaxf(m[g], m2);
      const float c1 = m[g] > -INFINITY ? expf(m[g] - M) : 0.f;
      const float c2 = m2 > -INFINITY ? expf(m2 - M) : 0.f;
      l[g] = l[g] * c1 + l2 * c2;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = acc[g][e] * c1 + __shfl_xor(acc[g][e], o) * c2;
      m[g] = M;
    }
    if (rs == 0) {
      if (dl == 0) { sm[wave][g] = m[g]; sl[wave][g] = l[g]; }
#pragma unroll
      for (int e = 0; e < EPL; ++e) sa[wave][g][dl * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();
  // ... then the waves, in a fixed order; one partial per (query row, split)
  for (int i = tid; i < NQ * HD; i += 64 * NWV) {
    const int g = i / HD, d = i - g * HD;
    if (g / G >= nrow) continue;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NWV; ++w) M = fmaxf(M, sm[w][g]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) {
      const float c = sm[w][g] > -INFINITY ? expf(sm[w][g] - M) : 0.f;
      L += c * sl[w][g];
      A += c * sa[w][g][d];
    }
    const int mi = mi0 + g / G, h = kvh * G + g % G;
    if (S == 1 && p.nsplit < 0) {
      // a single split and the caller wants the result itself: output row and its split tile, no partials
      const float o = A / L;
      p.O[(size_t)mi * p.ldo + h * HD + d] = o;
      if (p.XsOut) {
        const int k = h * HD + d;
        const uint16_t hi = f32_to_bf16_rne(o);
        const uint16_t lo = f32_to_bf16_rne(o - bf16_bits_to_f32(hi));
        uint16_t* dst = p.XsOut + (size_t)(mi >> 4) * p.xs_cb_stride + (size_t)(k >> 5) * 1024 +
                        (((k & 31) >> 3) * 16 + (mi & 15)) * 8 + (k & 7);
        dst[0] = hi;
        dst[512] = lo;
      }
      continue;
    }
    const size_t prow = ((size_t)mi * p.n_q + h) * p.nch_max + split;
    if (d == 0) { p.PM[prow] = M; p.PL[prow] = L; }
    p.PA[prow * HD + d] = A;
  }
}

// ---------------------------------------------------------------------------------------
// Causal attention of many token rows on the matrix cores (prefill).  One wave = 16 consecutive
// token rows of one query head; a work-group = 4 such waves.  Per tile of 32 cache rows:
//   S^T[32 rows][16 queries] = K[32][hd] * Q^T      (A = cache rows as stored, B = queries as
//                                                    bf16 high + low parts, kept in registers)
//   online soft-max per query (a lane holds 8 rows of one query; two cross-lane steps)
//   O^T[hd][16 queries] += V^T[hd][32 rows] * P     (A = the feature-major copy of the values,
//                                                    B = the probabilities, high + low parts)
// The A operand of the first product takes cache row t0 + 8*(i/4) + i%4 (+4 for the second block
// of 16) as its row i, so that the 8 scores a lane ends up with are 8 consecutive cache rows:
// exactly the B operand slice it must supply to the second product.  Nothing passes through LDS.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void split8(const float* v, uint4& hi, uint4& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const uint16_t h0 = f32_to_bf16_rne(v[e]), h1 = f32_to_bf16_rne(v[e + 1]);
    const uint16_t l0 = f32_to_bf16_rne(v[e] - bf16_bits_to_f32(h0));
    const uint16_t l1 = f32_to_bf16_rne(v[e + 1] - bf16_bits_to_f32(h1));
    h[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    l[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
  }
  hi = make_uint4(h[0], h[1], h[2], h[3]);
  lo = make_uint4(l[0], l[1], l[2], l[3]);
}

template <int HD>
__global__ void __launch_bounds__(256) attn_flash_k(AttnP p) {
  constexpr int KT = HD / 32, DT = HD / 16;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4, qi = lane & 15;
  const int h = blockIdx.y, kvh = h / (p.n_q / p.n_kv);
  const int r0 = blockIdx.x * 64 + wave * 16;
  if (r0 >= p.m) return;                       // wave-uniform; the kernel has no barriers
  const int nrow = min(16, p.m - r0);
  const int T0 = (p.ctx_len1 ? p.ctx_len1 - 1 : p.state[0]) + p.row_off;       // cache position of token row 0
  const int pos = T0 + r0 + qi;                // this lane's query attends cache rows <= pos
  const int t_end = T0 + r0 + nrow;            // cache rows this wave needs: [0, t_end)
  // queries: row r0 + qi (a ragged last block re-reads its last row; those results are dropped)
  uint4 qh[KT], ql[KT];
  {
    const float scale = 1.0f / sqrtf((float)HD);
    const float* qp = p.Q + (size_t)(r0 + min(qi, nrow - 1)) * p.ldq + (size_t)h * HD + 8 * g;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const float4 a = *(const float4*)(qp + 32 * kt), b = *(const float4*)(qp + 32 * kt + 4);
      const float v[8] = {a.x * scale, a.y * scale, a.z * scale, a.w * scale,
                          b.x * scale, b.y * scale, b.z * scale, b.w * scale};
      split8(v, qh[kt], ql[kt]);
    }
  }
  floatx4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = (floatx4){0.f, 0.f, 0.f, 0.f};
  float mrun = -INFINITY, lrun = 0.f;
  const uint16_t* Kb = (const uint16_t*)p.Kc + (size_t)kvh * p.Tcap * HD + 8 * g;
  const uint16_t* Vt = (const uint16_t*)p.VcT + ((size_t)kvh * HD + qi) * p.TcapT + 8 * g;
  const int rho = 8 * (qi >> 2) + (qi & 3);
  for (int t0 = 0; t0 < t_end; t0 += 32) {
    floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
    // rows past the wave's last one are read from that last row and masked below
    const uint16_t* k0 = Kb + (size_t)min(t0 + rho, t_end - 1) * HD;
    const uint16_t* k1 = Kb + (size_t)min(t0 + rho + 4, t_end - 1) * HD;
    uint4 a0[KT], a1[KT], av[DT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      a0[kt] = *(const uint4*)(k0 + 32 * kt);
      a1[kt] = *(const uint4*)(k1 + 32 * kt);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) av[dt] = *(const uint4*)(Vt + (size_t)(16 * dt) * p.TcapT + t0);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const bf16x8 x0 = __builtin_bit_cast(bf16x8, a0[kt]), x1 = __builtin_bit_cast(bf16x8, a1[kt]);
      const bf16x8 bh = __builtin_bit_cast(bf16x8, qh[kt]), bl = __builtin_bit_cast(bf16x8, ql[kt]);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x0, bh, s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x1, bh, s1, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x0, bl, s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x1, bl, s1, 0, 0, 0);
    }
    // this lane: scores of cache rows t0 + 8g + e, e = 0..7, for query qi
    float sv[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (t0 + 8 * g + e > pos) sv[e] = -INFINITY;
      mx = fmaxf(mx, sv[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mnew = fmaxf(mrun, mx);          // finite from the first tile on (row 0 is never masked)
    const float c = expf(mrun - mnew);
    float pv[8], ls = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pv[e] = expf(sv[e] - mnew);
      ls += pv[e];
    }
    ls += __shfl_xor(ls, 16);
    ls += __shfl_xor(ls, 32);
    lrun = lrun * c + ls;
    mrun = mnew;
    uint4 ph, pl;
    split8(pv, ph, pl);
    const bf16x8 bh = __builtin_bit_cast(bf16x8, ph), bl = __builtin_bit_cast(bf16x8, pl);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int j = 0; j < 4; ++j) o[dt][j] *= c;
      const bf16x8 x = __builtin_bit_cast(bf16x8, av[dt]);
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, bh, o[dt], 0, 0, 0);
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, bl, o[dt], 0, 0, 0);
    }
  }
  if (qi >= nrow) return;
  // this lane: features 16*dt + 4g + j of head h for token row r0 + qi
  const float inv = 1.0f / lrun;
  const int row = r0 + qi;
  float* orow = p.O + (size_t)row * p.ldo + (size_t)h * HD + 4 * g;
  uint16_t* xs = p.XsOut ? p.XsOut + (size_t)(row >> 4) * p.xs_cb_stride : nullptr;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const float v[4] = {o[dt][0] * inv, o[dt][1] * inv, o[dt][2] * inv, o[dt][3] * inv};
    *(float4*)(orow + 16 * dt) = make_float4(v[0], v[1], v[2], v[3]);
    if (xs) {
      const int k = h * HD + 16 * dt + 4 * g;     // first of 4 consecutive features; k % 4 == 0
      uint16_t hi[4], lo[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        hi[j] = f32_to_bf16_rne(v[j]);
        lo[j] = f32_to_bf16_rne(v[j] - bf16_bits_to_f32(hi[j]));
      }
      uint16_t* dst = xs + (size_t)(k >> 5) * 1024 + (((k & 31) >> 3) * 16 + (row & 15)) * 8 + (k & 7);
      *(uint2*)dst = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
      *(uint2*)(dst + 512) = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
    }
  }
}

// ---------------------------------------------------------------------------------------
// The same matrix-core attention for a few token rows (the verify pass: m <= 16 rows, Section 2
// "verifies all draft tokens in parallel"), split over the context: one wave = all m queries of
// one query head against one span of cache rows, so the cache is read once for all rows and there
// are (splits x query heads) waves to keep in flight.  Each wave leaves a soft-max partial
// (max, sum, weighted values) per (token row, head, split); attn_combine_k merges them.
// ---------------------------------------------------------------------------------------
template <int HD>
__global__ void __launch_bounds__(256) attn_flash_split_k(AttnP p, int S, int rps_min) {
  constexpr int KT = HD / 32, DT = HD / 16;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4, qi = lane & 15;
  const int split = blockIdx.x * 4 + wave;
  if (split >= S) return;                      // wave-uniform; the kernel has no barriers
  const int h = blockIdx.y, kvh = h / (p.n_q / p.n_kv);
  const int nrow = p.m;                        // <= 16, checked by the launcher
  const int T0 = (p.ctx_len1 ? p.ctx_len1 - 1 : p.state[0]) + p.row_off;       // cache position of token row 0
  const int pos = T0 + qi;                     // this lane's query attends cache rows <= pos
  const int t_end = T0 + nrow;                 // cache rows the pass needs: [0, t_end)
  // rows per split: whole tiles of 32, at least what the launcher planned for (attn_combine_k derives the
  // same number from p.rps)
  const int rps = max(rps_min, ((t_end + S - 1) / S + 31) / 32 * 32);
  const int t_lo = split * rps, t_hi = min(t_end, t_lo + rps);
  if (t_lo >= t_end) return;                   // a span past the context: the merge does not read its partial
  uint4 qh[KT], ql[KT];
  {
    const float scale = 1.0f / sqrtf((float)HD);
    const float* qp = p.Q + (size_t)min(qi, nrow - 1) * p.ldq + (size_t)h * HD + 8 * g;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const float4 a = *(const float4*)(qp + 32 * kt), b = *(const float4*)(qp + 32 * kt + 4);
      const float v[8] = {a.x * scale, a.y * scale, a.z * scale, a.w * scale,
                          b.x * scale, b.y * scale, b.z * scale, b.w * scale};
      split8(v, qh[kt], ql[kt]);
    }
  }
  floatx4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = (floatx4){0.f, 0.f, 0.f, 0.f};
  float mrun = -INFINITY, lrun = 0.f;
  const uint16_t* Kb = (const uint16_t*)p.Kc + (size_t)kvh * p.Tcap * HD + 8 * g;
  const uint16_t* Vt = (const uint16_t*)p.VcT + ((size_t)kvh * HD + qi) * p.TcapT + 8 * g;
  const int rho = 8 * (qi >> 2) + (qi & 3);
  // two register sets, filled and used in turn: the rows of the next tile are requested before the current
  // tile is multiplied (a span is two or three tiles: without this each tile costs a full memory latency).
  // Branch-free: an odd tile count runs one more, fully masked, tile on a re-read of the last one.
  auto load = [&](int t0, uint4* a0, uint4* a1, uint4* av) {
    // rows past the pass's last one are read from that last row and masked in the scores
    const uint16_t* k0 = Kb + (size_t)min(t0 + rho, t_end - 1) * HD;
    const uint16_t* k1 = Kb + (size_t)min(t0 + rho + 4, t_end - 1) * HD;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      a0[kt] = *(const uint4*)(k0 + 32 * kt);
      a1[kt] = *(const uint4*)(k1 + 32 * kt);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) av[dt] = *(const uint4*)(Vt + (size_t)(16 * dt) * p.TcapT + t0);
  };
  auto compute = [&](int t0, const uint4* a0, const uint4* a1, const uint4* av) {
    floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const bf16x8 x0 = __builtin_bit_cast(bf16x8, a0[kt]), x1 = __builtin_bit_cast(bf16x8, a1[kt]);
      const bf16x8 bh = __builtin_bit_cast(bf16x8, qh[kt]), bl = __builtin_bit_cast(bf16x8, ql[kt]);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x0, bh, s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x1, bh, s1, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x0, bl, s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x1, bl, s1, 0, 0, 0);
    }
    // this lane: scores of cache rows t0 + 8g + e, e = 0..7, for query qi; rows of the next span (the extra
    // tile of an odd count) and rows the query may not see count for nothing
    float sv[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int row = t0 + 8 * g + e;
      if (row > pos || row >= t_hi) sv[e] = -INFINITY;
      mx = fmaxf(mx, sv[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    // a split may hold no row this query may see (the rows of later tokens only): everything stays
    // at (max = -inf, sum = 0, values = 0), which the merge gives weight 0
    const float mnew = fmaxf(mrun, mx);
    const float c = mrun > -INFINITY ? expf(mrun - mnew) : 0.f;
    float pv[8], ls = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pv[e] = sv[e] > -INFINITY ? expf(sv[e] - mnew) : 0.f;
      ls += pv[e];
    }
    ls += __shfl_xor(ls, 16);
    ls += __shfl_xor(ls, 32);
    lrun = lrun * c + ls;
    mrun = mnew;
    uint4 ph, pl;
    split8(pv, ph, pl);
    const bf16x8 bh = __builtin_bit_cast(bf16x8, ph), bl = __builtin_bit_cast(bf16x8, pl);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int j = 0; j < 4; ++j) o[dt][j] *= c;
      const bf16x8 x = __builtin_bit_cast(bf16x8, av[dt]);
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, bh, o[dt], 0, 0, 0);
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, bl, o[dt], 0, 0, 0);
    }
  };
  {
    const int last = t_lo + (t_hi - t_lo - 1) / 32 * 32;   // first row of the span's last tile
    uint4 ka0[KT], ka1[KT], va[DT], kb0[KT], kb1[KT], vb[DT];
    load(t_lo, ka0, ka1, va);
    for (int t0 = t_lo; t0 < t_hi; t0 += 64) {
      load(min(t0 + 32, last), kb0, kb1, vb);
      compute(t0, ka0, ka1, va);
      load(min(t0 + 64, last), ka0, ka1, va);
      compute(t0 + 32, kb0, kb1, vb);
    }
  }
  if (qi >= nrow) return;
  // this lane: features 16*dt + 4g + j of head h for token row qi, as an unnormalised partial
  const size_t prow = ((size_t)qi * p.n_q + h) * p.nch_max + split;
  if (g == 0) { p.PM[prow] = mrun; p.PL[prow] = lrun; }
  float* pa = p.PA + prow * HD + 4 * g;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) *(float4*)(pa + 16 * dt) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
}

__global__ void __launch_bounds__(128) attn_combine_k(AttnP p) {
  const int row = blockIdx.x;  // mi * n_q + h
  const int d = threadIdx.x;
  if (d >= p.hd) return;
  const int T_end = (p.ctx_len1 ? p.ctx_len1 - 1 : p.state[0]) + p.row_off + p.m;
  int nch = p.nsplit > 0 ? p.nsplit : (T_end + p.ct - 1) / p.ct;   // partials per row
  if (p.rps > 0) {   // matrix-core kernel, split by spans of rows: only the spans that reach into the context
    const int rps = max(p.rps, ((T_end + p.nsplit - 1) / p.nsplit + 31) / 32 * 32);
    nch = min(nch, (T_end + rps - 1) / rps);
  }
  const float* pm = p.PM + (size_t)row * p.nch_max;
  const float* pl = p.PL + (size_t)row * p.nch_max;
  const float* pa = p.PA + (size_t)row * p.nch_max * p.hd + d;
  // every chunk below nch has written its partial (fully masked ones: max = -inf, sum = 0, values = 0),
  // so the loops are branch-free and their loads independent
  float M = -INFINITY;
#pragma unroll 8
  for (int c = 0; c < nch; ++c) M = fmaxf(M, pm[c]);
  float L = 0.f, acc = 0.f;
#pragma unroll 8
  for (int c = 0; c < nch; ++c) {
    const float mc = pm[c];
    const float w = mc > -INFINITY ? expf(mc - M) : 0.f;
    L += w * pl[c];
    acc += w * pa[(size_t)c * p.hd];
  }
  const int mi = row / p.n_q, h = row - mi * p.n_q;
  const float o = acc / L;
  p.O[(size_t)mi * p.ldo + h * p.hd + d] = o;
  if (p.XsOut) {
    const int k = h * p.hd + d;
    const uint16_t hi = f32_to_bf16_rne(o);
    const uint16_t lo = f32_to_bf16_rne(o - bf16_bits_to_f32(hi));
    uint16_t* dst = p.XsOut + (size_t)(mi >> 4) * p.xs_cb_stride + (size_t)(k >> 5) * 1024 +
                    (((k & 31) >> 3) * 16 + (mi & 15)) * 8 + (k & 7);
    dst[0] = hi;
    dst[512] = lo;
  }
}

// ---------------------------------------------------------------------------------------
// Small kernels
// ---------------------------------------------------------------------------------------
template <int KPL>
__global__ void __launch_bounds__(256) embed_k(const void* Et, int KT, int vocab, const int* ids, float* out, int ld,
                                               int d_model) {
  const int row = blockIdx.x;
  int id = ids[row];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  gather_embedding(Et, KPL, KT, id, out + (size_t)row * ld, d_model, threadIdx.x, 256);
}

// Merge the per-row-block (max, index) partials of one logits row; lowest index wins ties.
// With psum (per-block sums of exp(logit - block max)) also the confidence of the arg-max token:
// its soft-max probability 1 / sum_b psum[b] * exp(max_b - max) (Section 4.4).
// emb_out (optional, one row): the winner's embedding row goes there as fp32 (the next draft step's input),
// read from the tiled embedding Et (kpl = 8 bf16 or 4 fp32 elements per lane and tile).
__global__ void __launch_bounds__(256) argmax_finish_k(const float* pval, const int* pidx, const float* psum, int NB,
                                                       int* out_ids, float* out_conf, const void* Et, int kpl,
                                                       int KT_e, int vocab, float* emb_out, int d_model,
                                                       unsigned long long* note, unsigned seq) {
  __shared__ float sv[256];
  __shared__ int si[256];
  const int row = blockIdx.x, tid = threadIdx.x;
  float best = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int b = tid; b < NB; b += 256) {
    const float v = pval[(size_t)row * NB + b];
    const int ix = pidx[(size_t)row * NB + b];
    if (v > best || (v == best && ix < bi)) { best = v; bi = ix; }
  }
  sv[tid] = best; si[tid] = bi;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      const float v = sv[tid + s];
      const int ix = si[tid + s];
      if (v > sv[tid] || (v == sv[tid] && ix < si[tid])) { sv[tid] = v; si[tid] = ix; }
    }
    __syncthreads();
  }
  const float M = sv[0];
  const int winner = si[0];
  if (tid == 0) out_ids[row] = winner;
  if (emb_out && row == 0) {
    const int id = winner < 0 ? 0 : (winner >= vocab ? vocab - 1 : winner);
    gather_embedding(Et, kpl, KT_e, id, emb_out, d_model, tid, 256);
  }
  if (psum && out_conf) {
    __syncthreads();
    float se = 0.f;
    for (int b = tid; b < NB; b += 256) {
      const float v = pval[(size_t)row * NB + b];
      if (v > -INFINITY) se += psum[(size_t)row * NB + b] * expf(v - M);
    }
    sv[tid] = se;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
      if (tid < s) sv[tid] += sv[tid + s];
      __syncthreads();
    }
    if (tid == 0) {
      const float cf = 1.0f / sv[0];
      out_conf[row] = cf;
      // for a host that polls pinned memory instead of waiting for the stream: sequence number and
      // confidence in one 8-byte store
      if (note && row == 0)
        __hip_atomic_store(note, ((unsigned long long)seq << 32) | __float_as_uint(cf), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}

// Greedy acceptance on the device (Section 2, greedy special case): u = first i < gamma
// with draft[i] != target[i], else gamma; the KV length advances by u + 1 and the pending
// input token becomes the target's token at u.  The drafted tokens are layer E's shadow
// tokens by construction, so they overwrite that row (both were computed from the same
// hidden state, but by different kernels).
// result: [0]=u, [1]=new T, [2]=pending, [3..3+gamma) drafts, then shadow [L][m]
__global__ void accept_k(int* state, const int* draft_ids, int* shadow_ids, int L, int m, int E, int gamma,
                         int* result) {
  // one wave: the drafts stand in for layer E's shadow tokens, then the first mismatch, then the copies
  const int t = threadIdx.x;
  if (blockIdx.x != 0 || t >= 64) return;
  int* srow = shadow_ids + (size_t)(E - 1) * m;
  for (int i = t; i < gamma; i += 64) srow[i] = draft_ids[i];
  const int* target = shadow_ids + (size_t)(L - 1) * m;
  // lane i < gamma looks at draft i (gamma <= 64 is checked by the launcher)
  const bool miss = t < gamma && draft_ids[t] != target[t];
  const unsigned long long mm = __ballot(miss);
  const int u = mm ? __ffsll((long long)mm) - 1 : gamma;
  const int T = state[0] + u + 1;
  const int next = target[u];
  __builtin_amdgcn_wave_barrier();
  if (t == 0) {
    state[0] = T;
    state[1] = next;
    result[0] = u;
    result[1] = T;
    result[2] = next;
  }
  for (int i = t; i < gamma; i += 64) result[3 + i] = draft_ids[i];
  // layer E's row was rewritten above by this same wave; its stores precede these loads in program order
  __threadfence_block();
  for (int i = t; i < L * m; i += 64) result[3 + gamma + i] = shadow_ids[i];
}

__global__ void set_state_k(int* state, int add_T, int set_T, const int* pending_src, int pending_val) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  if (set_T >= 0) state[0] = set_T;
  state[0] += add_T;
  if (pending_src) state[1] = *pending_src;
  else if (pending_val >= 0) state[1] = pending_val;
}

// Natural row-major [nrows, cols] (rows row0.. of the tensor) -> tiled layout, with the row map.
template <int KPL, typename T>
__global__ void __launch_bounds__(256) tile_scatter_k(const T* src, long long row0, long long nrows, long long cols,
                                                      int map, int vbase, int hd, T* dst, int KT) {
  const long long chunks_per_row = (cols + KPL - 1) / KPL;
  const long long total = nrows * chunks_per_row;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long ln = i / chunks_per_row;
    const int kc = (int)(i - ln * chunks_per_row);
    const long long n = row0 + ln;
    long long v;
    if (map == MAP_ROPE) {
      const int half = hd >> 1;
      const long long head = n / hd;
      const int j = (int)(n - head * hd);
      const int b = j / half, jj = j - b * half;
      v = vbase + head * hd + (jj >> 3) * 16 + b * 8 + (jj & 7);
    } else if (map == MAP_GATE) {
      v = (n >> 3) * 16 + (n & 7);
    } else if (map == MAP_UP) {
      v = (n >> 3) * 16 + 8 + (n & 7);
    } else {
      v = vbase + n;
    }
    const long long nb = v >> 4;
    const int r = (int)(v & 15);
    const int kt = kc >> 2, g = kc & 3;
    T* d = dst + (((size_t)nb * KT + kt) * 64 + g * 16 + r) * KPL;
    const T* s = src + (size_t)ln * cols + (size_t)kc * KPL;
#pragma unroll
    for (int e = 0; e < KPL; ++e) d[e] = ((long long)kc * KPL + e < cols) ? s[e] : (T)0;
  }
}

__global__ void pad_gain_k(const float* src, int K, float* dst, int Kpad) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k < Kpad) dst[k] = k < K ? src[k] : 0.f;
}

// Pure streaming read with the GEMV access pattern (non-temporal 1 KiB loads per wave, each wave
// a contiguous span, 8 loads in flight): the achievable-bandwidth ceiling of the weight stream.
__global__ void __launch_bounds__(512) stream_read_k(const uint4* base, long long n_tiles, float* sink) {
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * 512 + threadIdx.x) >> 6;
  const long long n_waves = ((long long)gridDim.x * 512) >> 6;
  const long long per = (n_tiles + n_waves - 1) / n_waves;
  const long long t0 = wave * per, t1 = t0 + per < n_tiles ? t0 + per : n_tiles;
  uint32_t acc = 0;
  long long t = t0;
  for (; t + 8 <= t1; t += 8) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld_stream(base + (t + u) * 64 + lane);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; t < t1; ++t) {
    const uint4 v = ld_stream(base + t * 64 + lane);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = 1.f;  // practically never; keeps the loads alive
}

// Plain copy of n 16-byte pieces (reads n*16 bytes, writes n*16 bytes): the known-size kernel
// against which the profiler's HBM byte counters are calibrated.
__global__ void __launch_bounds__(256) stream_copy_k(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) dst[i] = src[i];
}

// The one-row GEMV with parts of it switched off, for measurement only (results are not used): where a
// launch spends its time beyond the weight stream.  PARTS bit 0: the input row and gain staged through
// LDS (with the sum of squares); bit 1: bf16 decode and fp32 FMA (with the staged row, or with constants
// when bit 0 is off); bit 2: cross-wave reduction, RMS scale, residual add and store.  PARTS = 0 leaves
// the tile loads in the GEMV's geometry and schedule (two groups of GU tiles per wave in flight).
template <int PARTS>
__global__ void __launch_bounds__(1024) gemv_parts_k(const uint4* __restrict__ W, const float* __restrict__ X,
                                                    const float* __restrict__ G, const float* __restrict__ R,
                                                    float* __restrict__ Y, int KT) {
  constexpr bool STG = PARTS & 1, CMP = PARTS & 2, RED = PARTS & 4;
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[MAXW][16];
  __shared__ float ssr[MAXW];
  const int tid = threadIdx.x, nw = blockDim.x >> 6, wave = tid >> 6, lane = tid & 63, g = lane >> 4, nb = blockIdx.x;
  int kt_lo, kt_hi;
  wave_span(KT, nw, wave, GU, kt_lo, kt_hi);
  const int ngroups = (kt_hi - kt_lo) / GU;
  const uint4* wp = W + ((size_t)nb * KT + kt_lo) * 64 + lane;
  float acc = 0.f, ss = 0.f;
  const int Kp = KT * 32, stride = blockDim.x * 4;
  float4 xv[4], gv[4];
  auto stage_load = [&](int base) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kk = base + j * stride;
      xv[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      gv[j] = make_float4(1.f, 1.f, 1.f, 1.f);
      if (kk < Kp) { xv[j] = *(const float4*)(X + kk); gv[j] = *(const float4*)(G + kk); }
    }
  };
  auto stage_store = [&](int base) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kk = base + j * stride;
      if (kk < Kp) {
        const float4 x = xv[j], gg = gv[j];
        ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        *(float4*)(xs + kk) = make_float4(x.x * gg.x, x.y * gg.y, x.z * gg.z, x.w * gg.w);
      }
    }
  };
  if (STG) stage_load(tid * 4);
  uint4 ta[GU], tb[GU];
  if (ngroups > 0) {
#pragma unroll
    for (int u = 0; u < GU; ++u) ta[u] = ld_stream(wp + u * 64);
  }
  if (ngroups > 1) {
#pragma unroll
    for (int u = 0; u < GU; ++u) tb[u] = ld_stream(wp + (GU + u) * 64);
  }
  if (STG) {
    stage_store(tid * 4);
    for (int base = tid * 4 + 4 * stride; base < Kp; base += 4 * stride) { stage_load(base); stage_store(base); }
    __syncthreads();
  }
  auto tile = [&](const uint4& w, int kt) {
    if (CMP) {
      float wf[8];
      WDec<8>::dec(w, wf);
      float4 a = make_float4(1.f, 2.f, 3.f, 4.f), b = make_float4(.5f, .25f, .125f, 2.f);
      if (STG) { a = *(const float4*)(xs + kt * 32 + g * 8); b = *(const float4*)(xs + kt * 32 + g * 8 + 4); }
      acc += wf[0] * a.x; acc += wf[1] * a.y; acc += wf[2] * a.z; acc += wf[3] * a.w;
      acc += wf[4] * b.x; acc += wf[5] * b.y; acc += wf[6] * b.z; acc += wf[7] * b.w;
    } else {
      acc += __uint_as_float((w.x ^ w.y ^ w.z ^ w.w) & 0x3fffffffu);
    }
  };
  auto use = [&](const uint4* tl, int gi) {
#pragma unroll
    for (int u = 0; u < GU; ++u) tile(tl[u], kt_lo + gi * GU + u);
  };
  auto fill = [&](uint4* tl, int gi) {
    const uint4* wn = wp + (size_t)gi * GU * 64;
#pragma unroll
    for (int u = 0; u < GU; ++u) tl[u] = ld_stream(wn + u * 64);
  };
  int gi = 0;
  for (; gi + 4 <= ngroups; gi += 2) { use(ta, gi); fill(ta, gi + 2); use(tb, gi + 1); fill(tb, gi + 3); }
  const int left = ngroups - gi;
  if (left == 3) { use(ta, gi); fill(ta, gi + 2); use(tb, gi + 1); use(ta, gi + 2); }
  else if (left == 2) { use(ta, gi); use(tb, gi + 1); }
  else if (left == 1) { use(ta, gi); }
  for (int kt = kt_lo + ngroups * GU; kt < kt_hi; ++kt) tile(ld_stream(wp + (size_t)(kt - kt_lo) * 64), kt);
  if (!RED) {
    if (acc == 123.456f || ss == 77.f) Y[nb * 16 + (lane & 15)] = acc;   // practically never; keeps the work alive
    return;
  }
  acc += __shfl_xor(acc, 16);
  acc += __shfl_xor(acc, 32);
  for (int o = 1; o < 64; o <<= 1) ss += __shfl_xor(ss, o);
  if (lane < 16) red[wave][lane] = acc;
  if (lane == 0) ssr[wave] = ss;
  __syncthreads();
  if (tid < 16) {
    float s = 0.f, q = 0.f;
    for (int w = 0; w < nw; ++w) s += red[w][tid];
    for (int w = 0; w < nw; ++w) q += ssr[w];
    s *= 1.0f / sqrtf(q / (float)(KT * 32) + 1e-5f);
    Y[nb * 16 + tid] = s + R[nb * 16 + tid];
  }
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
template <int KPL, int M, int EPI>
static hipError_t launch_valu_e(const GemmP& p, int waves, hipStream_t s) {
  while (waves > ValuWaves<M>::max) waves >>= 1;
  dim3 grid(p.NB), block(64 * waves);
  const size_t lds = M == 1 ? (size_t)p.KT * 4 * KPL * sizeof(float) : 0;
  if (lds > 48 * 1024) {  // beyond the default dynamic LDS limit: raise it for this kernel (once is enough)
    static size_t raised = 0;
    if (lds > raised) {
      hipError_t e = hipFuncSetAttribute((const void*)gemm_valu_k<KPL, M, EPI>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised = lds;
    }
  }
  if (p.ev_start && p.ev_stop)
    hipExtLaunchKernelGGL((gemm_valu_k<KPL, M, EPI>), grid, block, (uint32_t)lds, s, p.ev_start, p.ev_stop, 0, p);
  else
    hipLaunchKernelGGL((gemm_valu_k<KPL, M, EPI>), grid, block, lds, s, p);
  return hipGetLastError();
}

// The several-row-blocks-per-work-group form: bf16, one row, KT = 128, 160 or 256, at least one row block per
// work-group of a grid of ROWS_GRID; p.rows_form == 1 keeps the other kernel.
constexpr int ROWS_GRID = 256;   // one work-group per compute unit of the MI355X
template <int NG, int EPI, int GUX = GU>
static hipError_t launch_rows_e(const GemmP& p, hipStream_t s) {
  const size_t lds = (size_t)p.KT * 32 * sizeof(float);
  static size_t raised = 0;
  if (lds > 48 * 1024 && lds > raised) {
    hipError_t e = hipFuncSetAttribute((const void*)gemv_rows_k<NG, EPI, GUX>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised = lds;
  }
  const dim3 grid(p.NB < ROWS_GRID ? p.NB : ROWS_GRID), block(64 * ROWS_WAVES);
  if (p.ev_start && p.ev_stop)
    hipExtLaunchKernelGGL((gemv_rows_k<NG, EPI, GUX>), grid, block, (uint32_t)lds, s, p.ev_start, p.ev_stop, 0, p);
  else
    hipLaunchKernelGGL((gemv_rows_k<NG, EPI, GUX>), grid, block, lds, s, p);
  return hipGetLastError();
}
template <int NG, int GUX = GU>
static hipError_t launch_rows(const GemmP& p, int epi, hipStream_t s) {
  switch (epi) {
    case EPI_STORE: return launch_rows_e<NG, EPI_STORE, GUX>(p, s);
    case EPI_RESID: return launch_rows_e<NG, EPI_RESID, GUX>(p, s);
    case EPI_QKV: return launch_rows_e<NG, EPI_QKV, GUX>(p, s);
    case EPI_SWIGLU: return launch_rows_e<NG, EPI_SWIGLU, GUX>(p, s);
    case EPI_ARGMAX: return launch_rows_e<NG, EPI_ARGMAX, GUX>(p, s);
    default: return hipErrorInvalidValue;
  }
}

template <int KPL, int M>
static hipError_t launch_valu_m(const GemmP& p, int epi, int waves, hipStream_t s) {
  switch (epi) {
    case EPI_STORE: return launch_valu_e<KPL, M, EPI_STORE>(p, waves, s);
    case EPI_RESID: return launch_valu_e<KPL, M, EPI_RESID>(p, waves, s);
    case EPI_QKV: return launch_valu_e<KPL, M, EPI_QKV>(p, waves, s);
    case EPI_SWIGLU: return launch_valu_e<KPL, M, EPI_SWIGLU>(p, waves, s);
    case EPI_ARGMAX: return launch_valu_e<KPL, M, EPI_ARGMAX>(p, waves, s);
    default: return hipErrorInvalidValue;
  }
}

template <int KPL>
static hipError_t launch_valu_k(const GemmP& p, int epi, int waves, hipStream_t s) {
  if (p.M == 1) return launch_valu_m<KPL, 1>(p, epi, waves, s);
  if (p.M == 2) return launch_valu_m<KPL, 2>(p, epi, waves, s);
  // four and eight rows with 32-bit weights only: with 16-bit weights (twice the values per tile) they do not fit
  // a lane's registers
  if constexpr (KPL == 4) {
    if (p.M == 4) return launch_valu_m<KPL, 4>(p, epi, waves, s);
    if (p.M == 8) return launch_valu_m<KPL, 8>(p, epi, waves, s);
  }
  return hipErrorInvalidValue;
}

bool gemv_rows_applies(const GemmP& p) {
  return p.wdtype == 1 && p.M == 1 && p.rows_form != 1 && p.NB >= ROWS_GRID && !p.XsOut && (p.KT == 128 || p.KT == 160 || p.KT == 256);
}
bool gemm_mfma_rows_applies(const GemmP& p, int epi, int col_blocks) {
  // (not with the residual epilogue: that instantiation does not fit 128 registers, and its matrices have one row
  // block per work-group anyway)
  return col_blocks == 1 && p.KT == 128 && p.NB >= ROWS_GRID && p.rows_form != 1 && epi != EPI_RESID;
}

hipError_t launch_gemm_valu(const GemmP& p, int epi, int waves, hipStream_t s) {
  if (waves < 1 || waves > MAXW || p.NB <= 0 || p.KT <= 0) return hipErrorInvalidValue;
  // attention partials as the input row: at most ATT_SMAX splits, whole float4 groups of features inside a head
  if (p.att_S > 0 && (p.att_S > ATT_SMAX || p.att_S > p.att_stride || p.K < 4 || p.att_hd % 4 || p.K % p.att_hd ||
                      !p.att_PM || !p.att_PL || !p.att_PA))
    return hipErrorInvalidValue;
  if (gemv_rows_applies(p))
    return p.KT == 128 ? launch_rows<2>(p, epi, s) : p.KT == 160 ? launch_rows<2, 5>(p, epi, s) : launch_rows<4>(p, epi, s);
  return p.wdtype == 1 ? launch_valu_k<8>(p, epi, waves, s) : launch_valu_k<4>(p, epi, waves, s);
}

hipError_t launch_gemm_mfma(const GemmP& p, int epi, int waves, int col_blocks, hipStream_t s) {
  if (waves < 1 || waves > MAXW || p.NB <= 0 || p.KT <= 0 || p.wdtype != 1 || col_blocks < 1 ||
      p.M > col_blocks * 16 || p.M <= (col_blocks - 1) * 16)
    return hipErrorInvalidValue;
  const bool timed = p.ev_start && p.ev_stop;
  if (gemm_mfma_rows_applies(p, epi, col_blocks)) {
    // several row blocks per work-group, the activation tiles held in registers
    const dim3 rgrid(ROWS_GRID), rblock(64 * ROWS_WAVES);
#define MFMA_ROWS(E)                                                                                              \
  if (timed) hipExtLaunchKernelGGL((gemm_mfma_rows_k<E>), rgrid, rblock, 0, s, p.ev_start, p.ev_stop, 0, p);       \
  else hipLaunchKernelGGL((gemm_mfma_rows_k<E>), rgrid, rblock, 0, s, p);                                           \
  return hipGetLastError();
    switch (epi) {
      case EPI_STORE: MFMA_ROWS(EPI_STORE)
      case EPI_QKV: MFMA_ROWS(EPI_QKV)
      case EPI_SWIGLU: MFMA_ROWS(EPI_SWIGLU)
      case EPI_ARGMAX: MFMA_ROWS(EPI_ARGMAX)
      default: return hipErrorInvalidValue;
    }
#undef MFMA_ROWS
  }
  dim3 grid(p.NB, col_blocks), block(64 * waves);
  switch (epi) {
    case EPI_STORE:
      if (timed) hipExtLaunchKernelGGL((gemm_mfma_k<EPI_STORE>), grid, block, 0, s, p.ev_start, p.ev_stop, 0, p);
      else hipLaunchKernelGGL((gemm_mfma_k<EPI_STORE>), grid, block, 0, s, p);
      break;
    case EPI_RESID:
      if (timed) hipExtLaunchKernelGGL((gemm_mfma_k<EPI_RESID>), grid, block, 0, s, p.ev_start, p.ev_stop, 0, p);
      else hipLaunchKernelGGL((gemm_mfma_k<EPI_RESID>), grid, block, 0, s, p);
      break;
    case EPI_QKV:
      if (timed) hipExtLaunchKernelGGL((gemm_mfma_k<EPI_QKV>), grid, block, 0, s, p.ev_start, p.ev_stop, 0, p);
      else hipLaunchKernelGGL((gemm_mfma_k<EPI_QKV>), grid, block, 0, s, p);
      break;
    case EPI_SWIGLU:
      if (timed) hipExtLaunchKernelGGL((gemm_mfma_k<EPI_SWIGLU>), grid, block, 0, s, p.ev_start, p.ev_stop, 0, p);
      else hipLaunchKernelGGL((gemm_mfma_k<EPI_SWIGLU>), grid, block, 0, s, p);
      break;
    case EPI_ARGMAX:
      if (timed) hipExtLaunchKernelGGL((gemm_mfma_k<EPI_ARGMAX>), grid, block, 0, s, p.ev_start, p.ev_stop, 0, p);
      else hipLaunchKernelGGL((gemm_mfma_k<EPI_ARGMAX>), grid, block, 0, s, p);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

namespace {
template <int EPI, int RBW, int CPW>
hipError_t launch_wide_inst(const GemmP& p, hipStream_t s) {
  const int CB = (p.M + 15) / 16, NS = (p.NB + RBW - 1) / RBW, NCG = (CB + 8 * CPW - 1) / (8 * CPW);
  dim3 grid((NS + 7) / 8 * 8 * NCG), block(512);
  const bool deep = p.wide_form != 1;
  // loads four k tiles deep (static LDS) where an iteration is short against a memory latency: one block of token
  // rows per wave.  With two blocks per wave the iteration is twice as long, two work-groups per CU already hide
  // the latency, and the rings' registers would leave room for one work-group only (measured: 330 -> 348 us on
  // gate/up, 214 -> 244 us on QKV, against 219 -> 123 us on the output and down projections).
  if (deep && CPW == 1 && p.KT % 4 == 0) {
    if (p.ev_start && p.ev_stop)
      hipExtLaunchKernelGGL((gemm_wide4_k<EPI, RBW, CPW>), grid, block, 0, s, p.ev_start, p.ev_stop, 0, p, NS, NCG);
    else
      hipLaunchKernelGGL((gemm_wide4_k<EPI, RBW, CPW>), grid, block, 0, s, p, NS, NCG);
    return hipGetLastError();
  }
  const size_t lds = (size_t)2 * RBW * 64 * sizeof(uint4);
  static bool raised = false;
  if (!raised) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_wide_k<EPI, RBW, CPW>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised = true;
  }
  if (p.ev_start && p.ev_stop)
    hipExtLaunchKernelGGL((gemm_wide_k<EPI, RBW, CPW>), grid, block, (uint32_t)lds, s, p.ev_start, p.ev_stop, 0, p, NS,
                          NCG);
  else
    hipLaunchKernelGGL((gemm_wide_k<EPI, RBW, CPW>), grid, block, lds, s, p, NS, NCG);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_gemm_wide(const GemmP& p, int epi, hipStream_t s) {
  if (p.NB <= 0 || p.KT <= 0 || p.M < 1 || p.wdtype != 1 || !p.Xs) return hipErrorInvalidValue;
  // a work-group's tile: 8 row blocks x 256 token rows; x 128 for the matrices with few rows (output and
  // down projection), which doubles their work-groups.  (16 row blocks x 256 rows halves the activation
  // traffic but leaves one work-group per CU and measured slower.)
  const bool small = p.NB < 512;
  switch (epi) {
    case EPI_RESID: return small ? launch_wide_inst<EPI_RESID, 8, 1>(p, s) : launch_wide_inst<EPI_RESID, 8, 2>(p, s);
    case EPI_QKV: return small ? launch_wide_inst<EPI_QKV, 8, 1>(p, s) : launch_wide_inst<EPI_QKV, 8, 2>(p, s);
    case EPI_SWIGLU: return small ? launch_wide_inst<EPI_SWIGLU, 8, 1>(p, s) : launch_wide_inst<EPI_SWIGLU, 8, 2>(p, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_rowscale(const float* ssq, int nb, int M, int K, float eps, float* rowscale, hipStream_t s) {
  if (M < 1 || nb < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rowscale_k, dim3((M + 3) / 4), dim3(256), 0, s, ssq, nb, M, K, eps, rowscale);
  return hipGetLastError();
}

hipError_t launch_head_gemm(const void* Wt, int NB, int KT, int N, const uint16_t* Xs, int R, const float* rowscale,
                            float* pval, int* pidx, float* psum, int* n_slabs, hipStream_t s, hipEvent_t ev_start,
                            hipEvent_t ev_stop, int form) {
  if (NB <= 0 || KT <= 0 || R <= 0) return hipErrorInvalidValue;
  const int CB = (R + 15) / 16, NS = (NB + HG_W - 1) / HG_W;
  *n_slabs = NS;
  // form 4: the register-blocked kernel (4 row blocks x 8 column blocks per wave, k split over the waves)
  const bool blocked = form == 4 && KT % 4 == 0;
  const size_t lds = blocked ? 0 : (size_t)2 * HG_CB * 128 * sizeof(uint4);   // the blocked kernel's stages are static
  static bool raised = false;
  if (!blocked && !raised) {
    hipError_t e = hipFuncSetAttribute((const void*)head_gemm_k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised = true;
  }
  const dim3 grid(NS, blocked ? (CB + H4_CB - 1) / H4_CB : (CB + HG_CB - 1) / HG_CB);
  if (blocked) {
    if (ev_start && ev_stop)
      hipExtLaunchKernelGGL(head_gemm4_k, grid, dim3(512), (uint32_t)lds, s, ev_start, ev_stop, 0, (const uint4*)Wt, NB, KT, N,
                            (const uint4*)Xs, CB, R, rowscale, pval, pidx, psum, NS);
    else
      hipLaunchKernelGGL(head_gemm4_k, grid, dim3(512), lds, s, (const uint4*)Wt, NB, KT, N, (const uint4*)Xs, CB, R,
                         rowscale, pval, pidx, psum, NS);
  } else if (ev_start && ev_stop) {
    hipExtLaunchKernelGGL(head_gemm_k, grid, dim3(512), (uint32_t)lds, s, ev_start, ev_stop, 0, (const uint4*)Wt, NB, KT, N,
                          (const uint4*)Xs, CB, R, rowscale, pval, pidx, psum, NS);
  } else {
    hipLaunchKernelGGL(head_gemm_k, grid, dim3(512), lds, s, (const uint4*)Wt, NB, KT, N, (const uint4*)Xs, CB, R, rowscale,
                       pval, pidx, psum, NS);
  }
  return hipGetLastError();
}

hipError_t launch_prep_split(const float* src, int rows, int rows_per_group, int64_t group_stride, int ld, int K,
                             int KT, const float* gain, int rms, float eps, uint16_t* Xs, float* rowscale,
                             hipStream_t s) {
  if (rows <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(prep_split_k, dim3(rows), dim3(256), 0, s, src, rows_per_group, (long long)group_stride, ld, K,
                     KT, gain, rms, eps, Xs, rowscale);
  return hipGetLastError();
}

static size_t attn_lds_bytes(int hd, int esize, int ct, int qb) {
  const int wpr = hd * esize / 4;
  return (size_t)2 * ct * (wpr + 1) * 4 + (size_t)qb * hd * 4 + (size_t)qb * ct * 4;
}

// Decode path (m == 1) for the shapes the register kernel is built for; S = number of splits.
// Returns hipErrorNotSupported for other shapes (the caller falls back to the staged kernels).
hipError_t launch_attention_decode(const AttnP& p, int S, hipStream_t s, int rows_per_wg) {
  if (p.m < 1 || S < 1 || S > p.nch_max) return hipErrorInvalidValue;
  const int G = p.n_q / p.n_kv;
  const bool many = rows_per_wg > 1;
  // one work-group per (split, kv head, group of token rows); G * rows per group <= 8 queries
#define DEL_ATT(KVT, HD, GG, RW)                                                                    \
  hipLaunchKernelGGL((attn_decode_k<KVT, HD, GG, RW>), dim3(S, p.n_kv, (p.m + RW - 1) / RW), dim3(RW > 1 ? 256 : 512), 0, s, p)
  if (p.kvdtype == 1 && p.hd == 128 && G == 1) { if (many) DEL_ATT(uint16_t, 128, 1, 8); else DEL_ATT(uint16_t, 128, 1, 1); }
  else if (p.kvdtype == 1 && p.hd == 64 && G == 4) { if (many) DEL_ATT(uint16_t, 64, 4, 2); else DEL_ATT(uint16_t, 64, 4, 1); }
  else if (p.kvdtype == 1 && p.hd == 128 && G == 8) DEL_ATT(uint16_t, 128, 8, 1);
  else if (p.kvdtype == 0 && p.hd == 64 && G == 1) { if (many) DEL_ATT(float, 64, 1, 4); else DEL_ATT(float, 64, 1, 1); }
  else return hipErrorNotSupported;
#undef DEL_ATT
  return hipGetLastError();
}

bool attention_decode_supported(int kvdtype, int hd, int G) {
  return (kvdtype == 1 && hd == 128 && (G == 1 || G == 8)) || (kvdtype == 1 && hd == 64 && G == 4) ||
         (kvdtype == 0 && hd == 64 && G == 1);
}

hipError_t launch_attention_flash(const AttnP& p, hipStream_t s) {
  if (p.m < 1 || p.kvdtype != 1 || !p.VcT || p.TcapT % 32 != 0 || p.TcapT < p.Tcap || p.n_q % p.n_kv != 0 ||
      (p.hd != 64 && p.hd != 128))
    return hipErrorInvalidValue;
  dim3 grid((p.m + 63) / 64, p.n_q), block(256);
  if (p.hd == 128) hipLaunchKernelGGL((attn_flash_k<128>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((attn_flash_k<64>), grid, block, 0, s, p);
  return hipGetLastError();
}

// Few token rows (m <= 16) on the matrix cores, S context splits of at least rps_min rows (a multiple of 32)
// each: writes S partials per (row, head); the caller merges them with launch_attention_merge (nsplit = S).
hipError_t launch_attention_flash_split(const AttnP& p, int S, int rps_min, hipStream_t s) {
  if (p.m < 1 || p.m > 16 || p.kvdtype != 1 || !p.VcT || p.TcapT % 32 != 0 || p.TcapT < p.Tcap || p.n_q % p.n_kv != 0 ||
      (p.hd != 64 && p.hd != 128) || S < 1 || S > p.nch_max || rps_min < 32 || rps_min % 32 != 0)
    return hipErrorInvalidValue;
  dim3 grid((S + 3) / 4, p.n_q), block(256);
  if (p.hd == 128) hipLaunchKernelGGL((attn_flash_split_k<128>), grid, block, 0, s, p, S, rps_min);
  else hipLaunchKernelGGL((attn_flash_split_k<64>), grid, block, 0, s, p, S, rps_min);
  return hipGetLastError();
}

// Merge p.nsplit partials per row (written by the decode kernel) into O (and XsOut).
hipError_t launch_attention_merge(const AttnP& p, hipStream_t s) {
  if (p.nsplit < 1 || p.nsplit > p.nch_max || p.hd > 128) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_combine_k, dim3(p.m * p.n_q), dim3(128), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_attention(const AttnP& p, hipStream_t s) {
  const int es = p.kvdtype == 1 ? 2 : 4;
  // the staging registers hold ct rows of at most 4 x 256 threads x 16 bytes per matrix
  if (p.hd > 128 || p.hd % 16 != 0 || p.m < 1 || p.n_q % p.n_kv != 0 || p.ct < 16 || p.ct > 64 || p.ct % 16 != 0 ||
      p.ct * p.hd * es > 4 * 256 * 16)
    return hipErrorInvalidValue;
  dim3 grid(p.nch_max, p.n_kv), block(256);
  AttnP q = p;
  const int QR = p.m * (p.n_q / p.n_kv);
  q.qb = QR >= QBMAX ? QBMAX : ((QR + 3) & ~3);   // few query rows: less LDS, more work-groups per CU
  if (p.kvdtype == 1)
    hipLaunchKernelGGL((attn_partial_k<uint16_t>), grid, block, attn_lds_bytes(p.hd, 2, p.ct, q.qb), s, q);
  else
    hipLaunchKernelGGL((attn_partial_k<float>), grid, block, attn_lds_bytes(p.hd, 4, p.ct, q.qb), s, q);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_combine_k, dim3(p.m * p.n_q), dim3(128), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_embed(const void* Et, int wdtype, int KT, int vocab, const int* ids, int m, float* out, int ld,
                        int d_model, hipStream_t s) {
  if (wdtype == 1)
    hipLaunchKernelGGL((embed_k<8>), dim3(m), dim3(256), 0, s, Et, KT, vocab, ids, out, ld, d_model);
  else
    hipLaunchKernelGGL((embed_k<4>), dim3(m), dim3(256), 0, s, Et, KT, vocab, ids, out, ld, d_model);
  return hipGetLastError();
}

hipError_t launch_argmax_finish(const float* pval, const int* pidx, const float* psum, int rows, int NB, int* out_ids,
                                float* out_conf, hipStream_t s, const void* Et, int wdtype, int KT_e, int vocab,
                                float* emb_out, int d_model, unsigned long long* note, unsigned seq) {
  if ((emb_out && (rows != 1 || !Et)) || (note && !(psum && out_conf))) return hipErrorInvalidValue;
  hipLaunchKernelGGL(argmax_finish_k, dim3(rows), dim3(256), 0, s, pval, pidx, psum, NB, out_ids, out_conf, Et,
                     wdtype == 1 ? 8 : 4, KT_e, vocab, emb_out, d_model, note, seq);
  return hipGetLastError();
}

hipError_t launch_accept(int* state, const int* draft_ids, int* shadow_ids, int L, int m, int E, int gamma,
                         int* result, hipStream_t s) {
  if (gamma > 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(accept_k, dim3(1), dim3(64), 0, s, state, draft_ids, shadow_ids, L, m, E, gamma, result);
  return hipGetLastError();
}

hipError_t launch_set_state(int* state, int add_T, int set_T, const int* pending_src, int pending_val,
                            hipStream_t s) {
  hipLaunchKernelGGL(set_state_k, dim3(1), dim3(64), 0, s, state, add_T, set_T, pending_src, pending_val);
  return hipGetLastError();
}

hipError_t launch_tile_scatter(const void* src, int wdtype, int64_t row0, int64_t nrows, int64_t cols, int map,
                               int vbase, int hd, void* dst, int KT, hipStream_t s) {
  const int kpl = wdtype == 1 ? 8 : 4;
  const int64_t total = nrows * ((cols + kpl - 1) / kpl);
  if (total <= 0) return hipSuccess;
  const int64_t want = (total + 255) / 256;
  const int blocks = (int)(want < 65535 * 4 ? want : 65535 * 4);
  if (wdtype == 1)
    hipLaunchKernelGGL((tile_scatter_k<8, uint16_t>), dim3(blocks), dim3(256), 0, s, (const uint16_t*)src,
                       (long long)row0, (long long)nrows, (long long)cols, map, vbase, hd, (uint16_t*)dst, KT);
  else
    hipLaunchKernelGGL((tile_scatter_k<4, float>), dim3(blocks), dim3(256), 0, s, (const float*)src, (long long)row0,
                       (long long)nrows, (long long)cols, map, vbase, hd, (float*)dst, KT);
  return hipGetLastError();
}

hipError_t launch_pad_gain(const float* src, int K, float* dst, int Kpad, hipStream_t s) {
  hipLaunchKernelGGL(pad_gain_k, dim3((Kpad + 255) / 256), dim3(256), 0, s, src, K, dst, Kpad);
  return hipGetLastError();
}

hipError_t launch_stream_copy(const void* src, void* dst, int64_t bytes, hipStream_t s) {
  const long long n = bytes / 16;
  if (n <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stream_copy_k, dim3(256 * 16), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* base, int64_t bytes, float* sink, hipStream_t s) {
  const long long n_tiles = bytes / 1024;
  if (n_tiles <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stream_read_k, dim3(256 * 8), dim3(512), 0, s, (const uint4*)base, n_tiles, sink);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Measurement kernel: issue rate of the two bf16 matrix instructions with NACC independent accumulators per
// wave and no memory traffic in the loop (one wave per SIMD, one work-group per compute unit).  SHAPE 0:
// v_mfma_f32_16x16x32_bf16 (the instruction the weight tiles are laid out for), 1: v_mfma_f32_32x32x16_bf16.
// The accumulators start from memory so that they are distinct values; results are discarded.
// ---------------------------------------------------------------------------------------
typedef float floatx16 __attribute__((ext_vector_type(16)));
template <int SHAPE, int NACC>
__global__ void __launch_bounds__(256) mfma_rate_k(const float* init, float* out, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
  {
    const uint4 ua = *(const uint4*)(init + 4 * lane), ub = *(const uint4*)(init + 256 + 4 * lane);
    a = __builtin_bit_cast(bf16x8, ua);
    b = __builtin_bit_cast(bf16x8, ub);
  }
  float s = 0.f;
  if (SHAPE == 0) {
    floatx4 acc[NACC];
#pragma unroll
    for (int n = 0; n < NACC; ++n)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[n][j] = init[512 + (n * 4 + j) * 64 + lane];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int n = 0; n < NACC; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[n], 0, 0, 0);
    }
#pragma unroll
    for (int n = 0; n < NACC; ++n) s += acc[n][0] + acc[n][1] + acc[n][2] + acc[n][3];
  } else {
    floatx16 acc[NACC];
#pragma unroll
    for (int n = 0; n < NACC; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[n][j] = init[512 + (n * 16 + j) * 64 + lane];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int n = 0; n < NACC; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
#pragma unroll
    for (int n = 0; n < NACC; ++n)
#pragma unroll
      for (int j = 0; j < 16; ++j) s += acc[n][j];
  }
  if (s == 12345.678f) out[threadIdx.x] = s;   // keeps the loop alive; the buffers hold zeros
}

// init: 512 + 64 * 64 floats (zeros will do), out: 256 floats
hipError_t launch_mfma_rate(int shape, int n_acc, const float* init, float* out, int iters, hipStream_t s) {
  const dim3 grid(256), block(256);
#define MFMA_RATE(S, N)                                                                     \
  if (shape == S && n_acc == N) {                                                           \
    hipLaunchKernelGGL((mfma_rate_k<S, N>), grid, block, 0, s, init, out, iters);           \
    return hipGetLastError();                                                               \
  }
  MFMA_RATE(0, 2) MFMA_RATE(0, 4) MFMA_RATE(0, 8) MFMA_RATE(0, 16)
  MFMA_RATE(1, 1) MFMA_RATE(1, 2) MFMA_RATE(1, 4)
#undef MFMA_RATE
  return hipErrorInvalidValue;
}

hipError_t launch_gemv_parts(const void* W, const float* X, const float* G, const float* R, float* Y, int NB, int KT,
                             int waves, int parts, hipStream_t s) {
  if (NB < 1 || KT < 1 || KT > 480 || (waves != 4 && waves != 8 && waves != 16) || parts < 0 || parts > 7)
    return hipErrorInvalidValue;
  const dim3 grid(NB), block(64 * waves);
  const size_t lds = (size_t)KT * 32 * sizeof(float);
  switch (parts) {
#define GP(v) case v: hipLaunchKernelGGL((gemv_parts_k<v>), grid, block, lds, s, (const uint4*)W, X, G, R, Y, KT); break;
    GP(0) GP(1) GP(2) GP(3) GP(4) GP(5) GP(6) GP(7)
#undef GP
  }
  return hipGetLastError();
}

}  // namespace del
