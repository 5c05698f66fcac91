// Speculative sampling on the device (DEL paper, Section 2, "Speculative decoding": draft tokens are
// drawn from the draft distribution q, accepted with probability min(1, p/q), a rejected position is
// redrawn from max(0, p - q), and after gamma acceptances one more token is drawn from p).
//
// A logits row becomes a distribution by soft-max(logits / temperature) restricted to the nucleus of
// mass top_p: tokens ordered by falling logit (lower id first among equals), the shortest leading run
// whose mass reaches top_p.  Every decision here is taken on exact integers: the weight
// exp((z - zmax) / temperature) of a token is computed in fp64 and stored as a 2^-44 fixed-point
// integer, so that sums do not depend on the order of addition and a run gives the same tokens every
// time.  The nucleus cut is found by a select over histograms of masses, not by a sort: a first pass
// of 256 bins linear in the logit, then 8-bit digits of the logits' order-preserving bit patterns
// inside the bin that holds the cut.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "del_kernels.h"

namespace del {

namespace {

constexpr int SB = 1024;                       // threads of every kernel in this file
constexpr double FIX = 17592186044416.0;       // 2^44
constexpr int SWD = 16;                        // loads a thread keeps in flight in a sweep

typedef unsigned long long u64;

__device__ __forceinline__ unsigned order_key(float z) {
  const unsigned b = __float_as_uint(z + 0.0f);   // -0 -> +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ bool kept(const SampRow& r, float z, int j) {
  const unsigned k = order_key(z);
  return k > r.kstar || (k == r.kstar && j <= r.tie_id);
}

// Exclusive scan of one value per thread over the block (Hillis-Steele in LDS); `buf` holds SB
// entries.  Returns the exclusive prefix; *total gets the block's sum.
template <typename T>
__device__ T block_exscan(T v, T* buf, T* total) {
  const int t = threadIdx.x;
  buf[t] = v;
  __syncthreads();
  for (int off = 1; off < SB; off <<= 1) {
    T add = t >= off ? buf[t - off] : (T)0;
    __syncthreads();
    buf[t] += add;
    __syncthreads();
  }
  const T incl = buf[t];
  *total = buf[SB - 1];
  __syncthreads();
  return incl - v;
}

// f(j, z[j]) for every j < V, ids interleaved over the threads (coalesced), SWD loads in flight.
template <typename F>
__device__ __forceinline__ void sweep(const float* z, int V, F f) {
  int j = threadIdx.x;
  for (; j + (SWD - 1) * SB < V; j += SWD * SB) {
    float v[SWD];
#pragma unroll
    for (int k = 0; k < SWD; ++k) v[k] = z[j + k * SB];
#pragma unroll
    for (int k = 0; k < SWD; ++k) f(j + k * SB, v[k]);
  }
  for (; j < V; j += SB) f(j, z[j]);
}

// The same with the token's fixed-point weight: f(j, z[j], wf[j]).
template <typename F>
__device__ __forceinline__ void sweep_w(const float* z, const u64* wf, int V, F f) {
  int j = threadIdx.x;
  for (; j + (SWD - 1) * SB < V; j += SWD * SB) {
    float v[SWD];
    u64 w[SWD];
#pragma unroll
    for (int k = 0; k < SWD; ++k) { v[k] = z[j + k * SB]; w[k] = wf[j + k * SB]; }
#pragma unroll
    for (int k = 0; k < SWD; ++k) f(j + k * SB, v[k], w[k]);
  }
  for (; j < V; j += SB) f(j, z[j], wf[j]);
}

struct PickLds {
  u64 buf[SB];        // scratch of the block scans and reductions
  u64 wtot[SB / 64];  // mass of each wave's segment
  int found;
};

// Four masses of ids j..j+3 (j a multiple of 4) of a row restricted to its nucleus.
struct KeptMass {
  const float* z; const u64* wf; SampRow R; int V;
  __device__ __forceinline__ void operator()(int j, u64* m) const {
    if (j + 3 < V) {
      const float4 zz = *reinterpret_cast<const float4*>(z + j);
      const ulonglong2 a = *reinterpret_cast<const ulonglong2*>(wf + j);
      const ulonglong2 b = *reinterpret_cast<const ulonglong2*>(wf + j + 2);
      m[0] = kept(R, zz.x, j) ? a.x : 0ull;
      m[1] = kept(R, zz.y, j + 1) ? a.y : 0ull;
      m[2] = kept(R, zz.z, j + 2) ? b.x : 0ull;
      m[3] = kept(R, zz.w, j + 3) ? b.y : 0ull;
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) m[k] = (j + k < V && kept(R, z[j + k], j + k)) ? wf[j + k] : 0ull;
    }
  }
};

// Draw by inverse cumulative mass in id order: the first id whose cumulative mass exceeds
// floor(r * total).  mass4(j, m) gives the masses of ids j..j+3.  Each wave owns a contiguous
// segment of the ids, 256 per step (4 per lane, 16-byte loads): first every wave sums its segment,
// then the wave whose segment holds the target walks it again with a wave scan per step.
// Every thread returns the id (-1 if the total is 0); *total_out receives the total mass.
template <typename F>
__device__ int pick_by_fraction(const F& mass4, int V, double r, PickLds* L, u64* total_out) {
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  constexpr int NW = SB / 64;
  const int S = ((V + NW - 1) / NW + 255) & ~255;     // ids per wave, a multiple of 256
  const int s0 = min(V, w * S), s1 = min(V, s0 + S);
  u64 part = 0;
  for (int base = s0; base < s1; base += 512) {
    u64 m[8];
    mass4(base + 4 * lane, m);
    if (base + 256 < s1) mass4(base + 256 + 4 * lane, m + 4);
    else m[4] = m[5] = m[6] = m[7] = 0;
    part += ((m[0] + m[1]) + (m[2] + m[3])) + ((m[4] + m[5]) + (m[6] + m[7]));
  }
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
  if (lane == 0) L->wtot[w] = part;
  if (t == 0) L->found = -1;
  __syncthreads();
  u64 total = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) total += L->wtot[i];
  *total_out = total;
  if (total == 0) { __syncthreads(); return -1; }
  u64 target = (u64)floor(r * (double)total);
  if (target >= total) target = total - 1;
  u64 excl = 0;
  for (int i = 0; i < w; ++i) excl += L->wtot[i];
  if (part > 0 && excl <= target && target < excl + part) {   // this wave's segment holds the target
    u64 run = excl;
    for (int base = s0; base < s1; base += 256) {
      u64 m[4];
      mass4(base + 4 * lane, m);
      const u64 g = (m[0] + m[1]) + (m[2] + m[3]);
      u64 inc = g;
      for (int off = 1; off < 64; off <<= 1) {
        const u64 o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
      }
      const unsigned long long hit = __ballot(run + inc > target);
      if (hit) {
        if (lane == __ffsll((long long)hit) - 1) {
          u64 c = run + inc - g;
          int k = 0;
          for (; k < 3; ++k) {
            c += m[k];
            if (c > target) break;
          }
          L->found = base + 4 * lane + k;
        }
        break;
      }
      run += __shfl(inc, 63, 64);
    }
  }
  __syncthreads();
  const int f = L->found;
  __syncthreads();
  return f;
}

// The first bin, in scan order, at which `above` plus the bins' running mass reaches `target`; scan
// position s looks at bin s (descending == false) or 255 - s.  Run by the first wave; the result goes
// to *sel and the mass of the bins before it, added to `above`, to *above_out.
__device__ __forceinline__ void select_bin(const u64* hist, u64 above, u64 target, bool descending, int* sel,
                                           u64* above_out) {
  const int l = threadIdx.x;
  if (l >= 64) return;
  u64 h[4], g = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int sidx = 4 * l + i;
    h[i] = hist[descending ? 255 - sidx : sidx];
    g += h[i];
  }
  u64 inc = g;
  for (int off = 1; off < 64; off <<= 1) {
    const u64 o = __shfl_up(inc, off, 64);
    if (l >= off) inc += o;
  }
  const unsigned long long hit = __ballot(above + inc >= target);
  const int lane = hit ? __ffsll((long long)hit) - 1 : 63;
  if (l == lane) {
    u64 a = above + inc - g;
    int i = 0;
    for (; i < 3; ++i) {
      if (a + h[i] >= target) break;
      a += h[i];
    }
    const int sidx = 4 * l + i;
    *sel = descending ? 255 - sidx : sidx;
    *above_out = a;
  }
}

}  // namespace

// One block per logits row: maximum, greedy token, its temperature-1 soft-max probability, the
// fixed-point weights of all tokens, and the nucleus (threshold key, tie cut, kept mass).  With
// draw_r: also draws a token from the row's nucleus with the uniform number draw_r[row] into
// draw_tok[row] (and into *pending, if given).
__global__ void __launch_bounds__(SB) samp_rowstats_k(const float* Z, long long ldz, int V, double inv_temp,
                                                      double top_p, u64* WF, long long ldw, SampRow* rows,
                                                      const float* draw_r, int* draw_tok, int* pending,
                                                      float* conf_out) {
  __shared__ PickLds pl;
  __shared__ double dbuf[SB];
  __shared__ u64 hist[256];
  __shared__ unsigned bmin[256], bmax[256];
  __shared__ float s_max, s_min;
  __shared__ int s_arg, s_sel;
  __shared__ u64 s_above;
  u64* sbuf = pl.buf;
  const int row = blockIdx.x, t = threadIdx.x;
  const float* z = Z + (long long)row * ldz;
  u64* wf = WF + (long long)row * ldw;
  // ---- maximum, the lowest id that attains it, and the minimum
  float mx = -INFINITY, mn = INFINITY;
  int arg = 0x7fffffff;
  sweep(z, V, [&](int j, float zj) {
    const float v = zj + 0.0f;
    if (v > mx) { mx = v; arg = j; }
    mn = fminf(mn, v);
  });
  float* fb = reinterpret_cast<float*>(dbuf);
  float* fb2 = fb + SB;
  int* ib = reinterpret_cast<int*>(sbuf);
  fb[t] = mx; fb2[t] = mn; ib[t] = arg;
  __syncthreads();
  for (int off = SB / 2; off > 0; off >>= 1) {
    if (t < off) {
      const float o = fb[t + off];
      const int oi = ib[t + off];
      if (o > fb[t] || (o == fb[t] && oi < ib[t])) { fb[t] = o; ib[t] = oi; }
      fb2[t] = fminf(fb2[t], fb2[t + off]);
    }
    __syncthreads();
  }
  if (t == 0) { s_max = fb[0]; s_min = fb2[0]; s_arg = ib[0]; }
  __syncthreads();
  const float zmax = s_max;
  const float zmin = s_min;
  // ---- weights and their total; on the way the first pass of the nucleus search: 256 bins linear
  //      in the logit between the row's maximum (bin 0) and minimum, which spreads the row evenly
  //      (the bit patterns of a narrow range would fall into a few bins and serialise the
  //      atomics); each bin also records the smallest and largest key it received
  const bool nucleus = top_p < 1.0;
  const float scale = zmax > zmin ? 256.0f / (zmax - zmin) : 0.0f;
  if (t < 256) { hist[t] = 0; bmin[t] = 0xffffffffu; bmax[t] = 0u; }
  __syncthreads();
  u64 wsum = 0;
  double s1 = 0.0;   // temperature-1 partition sum, only when the confidence is asked for
  sweep(z, V, [&](int j, float zj) {
    const float zc = zj + 0.0f;
    const double dz = (double)zc - (double)zmax;
    if (conf_out) s1 += exp(dz);
    const u64 w = (u64)rint(exp(dz * inv_temp) * FIX);
    wf[j] = w;
    wsum += w;
    if (nucleus) {
      const int b = min(255, (int)((zmax - zc) * scale));
      const unsigned k = order_key(zc);
      atomicAdd(&hist[b], w);
      atomicMin(&bmin[b], k);
      atomicMax(&bmax[b], k);
    }
  });
  __syncthreads();
  sbuf[t] = wsum;
  __syncthreads();
  for (int off = SB / 2; off > 0; off >>= 1) {
    if (t < off) sbuf[t] += sbuf[t + off];
    __syncthreads();
  }
  const u64 Wtot = sbuf[0];
  __syncthreads();
  float conf = 0.f;
  if (conf_out) {
    dbuf[t] = s1;
    __syncthreads();
    for (int off = SB / 2; off > 0; off >>= 1) {
      if (t < off) dbuf[t] += dbuf[t + off];
      __syncthreads();
    }
    conf = (float)(1.0 / dbuf[0]);
    __syncthreads();
  }
  unsigned kstar = 0;
  int tie_id = V;
  u64 Wkept = Wtot;
  if (nucleus) {
    // ---- radix select: the key at which the mass of higher-ranked tokens first reaches top_p
    u64 target = (u64)ceil(top_p * (double)Wtot);
    if (target < 1) target = 1;
    if (target > Wtot) target = Wtot;
    select_bin(hist, 0, target, false, &s_sel, &s_above);
    __syncthreads();
    u64 above = s_above;
    const unsigned klo = bmin[s_sel], khi = bmax[s_sel];
    __syncthreads();
    // then 8-bit digits of the keys inside [klo, khi], from the highest bit in which the two differ
    const unsigned kdiff = klo ^ khi;
    const int top = kdiff ? 31 - __clz((int)kdiff) : 0;
    const int shift0 = top > 7 ? top - 7 : 0;
    unsigned mask = shift0 + 8 >= 32 ? 0u : ~((1u << (shift0 + 8)) - 1u);
    unsigned prefix = khi & mask;
    int n_last = 0, id_last = V;
    u64 w_last = 0;
    for (int shift = shift0; shift >= 0; shift = shift >= 8 ? shift - 8 : (shift > 0 ? 0 : -1)) {
      if (t < 256) hist[t] = 0;
      __syncthreads();
      if (shift == 0 && t < 256) { bmin[t] = 0xffffffffu; bmax[t] = 0u; }   // now: lowest id, count
      __syncthreads();
      sweep_w(z, wf, V, [&](int j, float zj, u64 w) {
        const unsigned k = order_key(zj);
        if (k >= klo && k <= khi && (k & mask) == prefix) {
          const unsigned dgt = (k >> shift) & 255u;
          atomicAdd(&hist[dgt], w);
          if (shift == 0) { atomicMin(&bmin[dgt], (unsigned)j); atomicAdd(&bmax[dgt], 1u); }
        }
      });
      __syncthreads();
      select_bin(hist, above, target, true, &s_sel, &s_above);
      __syncthreads();
      above = s_above;
      n_last = (int)bmax[s_sel]; id_last = (int)bmin[s_sel]; w_last = hist[s_sel];
      prefix = (prefix & ~(255u << shift)) | ((unsigned)s_sel << shift);
      mask |= 255u << shift;
      __syncthreads();
    }
    kstar = prefix;
    if (n_last == 1) {
      // the usual case: one token carries the threshold key
      tie_id = id_last;
      Wkept = above + w_last;
    } else {
      if (t == 0) s_sel = V;
      // tokens whose key equals kstar share one logit, hence one weight: keep the first `need` of them
      const int C = (V + SB - 1) / SB;
      const int j0 = min(V, t * C), j1 = min(V, j0 + C);
      int cnt = 0;
      u64 w_each = 0;
      for (int j = j0; j < j1; ++j)
        if (order_key(z[j]) == kstar) { ++cnt; w_each = wf[j]; }
      sbuf[t] = w_each;
      __syncthreads();
      for (int off = SB / 2; off > 0; off >>= 1) {
        if (t < off) sbuf[t] = sbuf[t] > sbuf[t + off] ? sbuf[t] : sbuf[t + off];
        __syncthreads();
      }
      w_each = sbuf[0];
      __syncthreads();
      int n_eq;
      int* ibuf = reinterpret_cast<int*>(dbuf);
      const int excl = block_exscan<int>(cnt, ibuf, &n_eq);
      int need = n_eq;
      if (w_each > 0) {
        const u64 want = target > above ? target - above : 1;
        const u64 q = (want + w_each - 1) / w_each;
        need = q < (u64)n_eq ? (int)q : n_eq;
        if (need < 1) need = 1;
      }
      if (cnt > 0 && excl < need && need <= excl + cnt) {
        int c = excl;
        for (int j = j0; j < j1; ++j)
          if (order_key(z[j]) == kstar && ++c == need) { s_sel = j; break; }
      }
      __syncthreads();
      tie_id = s_sel;
      Wkept = above + (u64)need * w_each;
      __syncthreads();
    }
  }
  SampRow R;
  R.zmax = zmax; R.kstar = kstar; R.tie_id = tie_id; R.argmax = s_arg;
  R.Wkept = Wkept; R.Wtot = Wtot; R.conf = conf; R.pad = 0;
  if (t == 0) {
    rows[row] = R;
    if (conf_out) conf_out[row] = conf;
  }
  if (draw_r) {
    u64 total;
    const int tok = pick_by_fraction(KeptMass{z, wf, R, V}, V, (double)draw_r[row], &pl, &total);
    if (t == 0) {
      const int tk = tok >= 0 ? tok : R.argmax;
      draw_tok[row] = tk;
      if (pending) *pending = tk;
    }
  }
}

// Acceptance of gamma drafted tokens and the round's last token; commits the KV length and the
// pending token.  Rows 0..gamma-1 of (Zq, WFq, rq) are the draft steps, rows 0..gamma of
// (Zp, WFp, rp) the target's.  unif_accept[0..gamma) decide the acceptances, *unif_last draws the last token.
// result: [0]=u, [1]=new KV length, [2]=last token, [3..3+gamma)=drafts, then the L*m shadow tokens.
__global__ void __launch_bounds__(SB) samp_accept_k(const float* Zq, const u64* WFq, const SampRow* rq,
                                                    const float* Zp, const u64* WFp, const SampRow* rp,
                                                    long long ldz, long long ldw, int V, int gamma,
                                                    const int* drafts, const float* unif_accept,
                                                    const float* unif_last, int* state, const int* shadow_ids,
                                                    int n_shadow, int* result) {
  __shared__ PickLds pl;
  __shared__ int s_rej[64];
  __shared__ int s_u;
  const int t = threadIdx.x;
  // every drafted token's test on its own thread; u = the first that fails
  if (t < 64) {
    int rej = 0;
    if (t < gamma) {
      const int x = drafts[t];
      const SampRow q = rq[t], p = rp[t];
      const double qx = (double)WFq[(long long)t * ldw + x] / (double)q.Wkept;
      const double px = kept(p, Zp[(long long)t * ldz + x], x)
                            ? (double)WFp[(long long)t * ldw + x] / (double)p.Wkept : 0.0;
      rej = !((double)unif_accept[t] * qx < px);
    }
    s_rej[t] = rej;
  }
  __syncthreads();
  if (t == 0) {
    int u = gamma;
    for (int i = 0; i < gamma; ++i)
      if (s_rej[i]) { u = i; break; }
    s_u = u;
  }
  __syncthreads();
  const int u = s_u;
  const double r = (double)*unif_last;
  const float* zp = Zp + (long long)u * ldz;
  const u64* wp = WFp + (long long)u * ldw;
  const SampRow P = rp[u];
  int tok = -1;
  if (u < gamma) {
    const float* zq = Zq + (long long)u * ldz;
    const u64* wq = WFq + (long long)u * ldw;
    const SampRow Q = rq[u];
    const double ip = 1.0 / (double)P.Wkept, iq = 1.0 / (double)Q.Wkept;
    const KeptMass mp{zp, wp, P, V}, mq{zq, wq, Q, V};
    auto res4 = [&](int j, u64* m) {
      u64 a[4], b[4];
      mp(j, a);
      mq(j, b);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const double d = (double)a[k] * ip - (double)b[k] * iq;
        m[k] = d > 0.0 ? (u64)rint(d * FIX) : 0ull;
      }
    };
    u64 total;
    tok = pick_by_fraction(res4, V, r, &pl, &total);
  }
  if (tok < 0) {
    u64 total;
    tok = pick_by_fraction(KeptMass{zp, wp, P, V}, V, r, &pl, &total);
    if (tok < 0) tok = P.argmax;
  }
  if (t == 0) {
    const int T = state[0] + u + 1;
    state[0] = T;
    state[1] = tok;
    result[0] = u; result[1] = T; result[2] = tok;
  }
  for (int i = t; i < gamma; i += SB) result[3 + i] = drafts[i];
  for (int i = t; i < n_shadow; i += SB) result[3 + gamma + i] = shadow_ids[i];
}

hipError_t launch_samp_rowstats(const float* Z, int64_t ldz, int V, int rows, double temperature, double top_p,
                                unsigned long long* WF, int64_t ldw, SampRow* out, const float* draw_r, int* draw_tok,
                                int* pending, float* conf_out, hipStream_t s) {
  if (rows <= 0 || V <= 0 || !(temperature > 0.0) || !(top_p > 0.0) || (draw_r && !draw_tok))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(samp_rowstats_k, dim3(rows), dim3(SB), 0, s, Z, (long long)ldz, V, 1.0 / temperature, top_p, WF,
                     (long long)ldw, out, draw_r, draw_tok, pending, conf_out);
  return hipGetLastError();
}

hipError_t launch_samp_accept(const float* Zq, const unsigned long long* WFq, const SampRow* rq, const float* Zp,
                              const unsigned long long* WFp, const SampRow* rp, int64_t ldz, int64_t ldw, int V,
                              int gamma, const int* drafts, const float* unif_accept, const float* unif_last, int* state,
                              const int* shadow_ids, int n_shadow, int* result, hipStream_t s) {
  if (gamma < 0 || gamma > 64 || V <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(samp_accept_k, dim3(1), dim3(SB), 0, s, Zq, WFq, rq, Zp, WFp, rp, (long long)ldz, (long long)ldw,
                     V, gamma, drafts, unif_accept, unif_last, state, shadow_ids, n_shadow, result);
  return hipGetLastError();
}

}  // namespace del
