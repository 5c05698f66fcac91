// Speculative sampling on the device (DEL paper, Section 2, "Speculative decoding": draft tokens are
// drawn from the draft distribution q, accepted with probability min(1, p/q), a rejected position is
// redrawn from max(0, p - q), and after gamma acceptances one more token is drawn from p).
//
// A logits row becomes a distribution by soft-max(logits / temperature) restricted to the nucleus of
// mass top_p: tokens ordered by falling logit (lower id first among equals), the shortest leading run
// whose mass reaches top_p.  Every decision here is taken on exact integers: the weight
// exp((z - zmax) / temperature) of a token is computed in fp64 and stored as a 2^-44 fixed-point
// integer, so that sums do not depend on the order of addition and a run gives the same tokens every
// time.  The nucleus cut is found by a radix select over the logits' order-preserving bit patterns
// (four passes of 8 bits, a 256-bin histogram of masses each), not by a sort.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "del_kernels.h"

namespace del {

namespace {

constexpr int SB = 1024;                       // threads of every kernel in this file
constexpr double FIX = 17592186044416.0;       // 2^44

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

// First id, in id order, whose cumulative mass exceeds `target` (0 <= target < total mass).
// mass(j) is evaluated twice per id.  Every thread returns the id.
template <typename F>
__device__ int pick_by_mass(F mass, int V, u64 target, u64* buf, int* found) {
  const int C = (V + SB - 1) / SB;
  const int j0 = min(V, (int)threadIdx.x * C), j1 = min(V, j0 + C);
  u64 sum = 0;
  for (int j = j0; j < j1; ++j) sum += mass(j);
  u64 total;
  const u64 excl = block_exscan<u64>(sum, buf, &total);
  if (threadIdx.x == 0) *found = -1;
  __syncthreads();
  if (sum > 0 && excl <= target && target < excl + sum) {
    u64 c = excl;
    for (int j = j0; j < j1; ++j) {
      c += mass(j);
      if (c > target) { *found = j; break; }
    }
  }
  __syncthreads();
  int f = *found;
  __syncthreads();
  return f;
}

}  // namespace

// One block per logits row: maximum, greedy token, its temperature-1 soft-max probability, the
// fixed-point weights of all tokens, and the nucleus (threshold key, tie cut, kept mass).
__global__ void __launch_bounds__(SB) samp_rowstats_k(const float* Z, long long ldz, int V, double inv_temp,
                                                      double top_p, u64* WF, long long ldw, SampRow* rows) {
  __shared__ u64 sbuf[SB];
  __shared__ double dbuf[SB];
  __shared__ u64 hist[256];
  __shared__ float s_max;
  __shared__ int s_arg, s_sel;
  __shared__ u64 s_above;
  const int row = blockIdx.x, t = threadIdx.x;
  const float* z = Z + (long long)row * ldz;
  u64* wf = WF + (long long)row * ldw;
  // ---- maximum and the lowest id that attains it
  float mx = -INFINITY;
  int arg = 0x7fffffff;
  for (int j = t; j < V; j += SB) {
    const float v = z[j] + 0.0f;
    if (v > mx) { mx = v; arg = j; }
  }
  float* fb = reinterpret_cast<float*>(dbuf);
  int* ib = reinterpret_cast<int*>(sbuf);
  fb[t] = mx; ib[t] = arg;
  __syncthreads();
  for (int off = SB / 2; off > 0; off >>= 1) {
    if (t < off) {
      const float o = fb[t + off];
      const int oi = ib[t + off];
      if (o > fb[t] || (o == fb[t] && oi < ib[t])) { fb[t] = o; ib[t] = oi; }
    }
    __syncthreads();
  }
  if (t == 0) { s_max = fb[0]; s_arg = ib[0]; }
  __syncthreads();
  const float zmax = s_max;
  // ---- weights, their total, and the temperature-1 partition sum
  double s1 = 0.0;
  u64 wsum = 0;
  for (int j = t; j < V; j += SB) {
    const double dz = (double)(z[j] + 0.0f) - (double)zmax;
    s1 += exp(dz);
    const u64 w = (u64)rint(exp(dz * inv_temp) * FIX);
    wf[j] = w;
    wsum += w;
  }
  dbuf[t] = s1; sbuf[t] = wsum;
  __syncthreads();
  for (int off = SB / 2; off > 0; off >>= 1) {
    if (t < off) { dbuf[t] += dbuf[t + off]; sbuf[t] += sbuf[t + off]; }
    __syncthreads();
  }
  const double S1 = dbuf[0];
  const u64 Wtot = sbuf[0];
  __syncthreads();
  unsigned kstar = 0;
  int tie_id = V;
  u64 Wkept = Wtot;
  if (top_p < 1.0) {
    // ---- radix select: the key at which the mass of higher-ranked tokens first reaches top_p
    u64 target = (u64)ceil(top_p * (double)Wtot);
    if (target < 1) target = 1;
    if (target > Wtot) target = Wtot;
    unsigned prefix = 0, mask = 0;
    u64 above = 0, mass_eq = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (t < 256) hist[t] = 0;
      __syncthreads();
      for (int j = t; j < V; j += SB) {
        const unsigned k = order_key(z[j]);
        if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], wf[j]);
      }
      __syncthreads();
      if (t == 0) {
        u64 a = above;
        int sel = 0;
        for (int b = 255; b >= 0; --b) {
          if (a + hist[b] >= target) { sel = b; break; }
          a += hist[b];
        }
        s_sel = sel; s_above = a;
      }
      __syncthreads();
      above = s_above;
      mass_eq = hist[s_sel];
      prefix |= (unsigned)s_sel << shift;
      mask |= 255u << shift;
      __syncthreads();
    }
    kstar = prefix;
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
    (void)mass_eq;
  }
  if (t == 0) {
    SampRow r;
    r.zmax = zmax; r.kstar = kstar; r.tie_id = tie_id; r.argmax = s_arg;
    r.Wkept = Wkept; r.Wtot = Wtot; r.conf = (float)(1.0 / S1); r.pad = 0;
    rows[row] = r;
  }
}

// Draw one token from a row's nucleus distribution with the uniform number *r: the first id whose
// cumulative kept mass exceeds r * (kept mass).  Writes the token and its weight.
__global__ void __launch_bounds__(SB) samp_draw_k(const float* z, int V, const u64* wf, const SampRow* row,
                                                  const float* r, int* token_out, u64* weight_out,
                                                  int* state_pending) {
  __shared__ u64 buf[SB];
  __shared__ int found;
  const SampRow R = *row;
  const u64 target = (u64)floor((double)*r * (double)R.Wkept);
  const int tok = pick_by_mass([&](int j) -> u64 { return kept(R, z[j], j) ? wf[j] : 0ull; }, V,
                               target < R.Wkept ? target : R.Wkept - 1, buf, &found);
  if (threadIdx.x == 0) {
    const int tk = tok >= 0 ? tok : R.argmax;
    *token_out = tk;
    if (weight_out) *weight_out = wf[tk];
    if (state_pending) *state_pending = tk;
  }
}

// Acceptance of gamma drafted tokens and the round's last token; commits the KV length and the
// pending token.  Rows 0..gamma-1 of (Zq, WFq, rq) are the draft steps, rows 0..gamma of
// (Zp, WFp, rp) the target's.  unif[0..gamma) decide the acceptances, unif[gamma] draws the last token.
// result: [0]=u, [1]=new KV length, [2]=last token, [3..3+gamma)=drafts, then the L*m shadow tokens.
__global__ void __launch_bounds__(SB) samp_accept_k(const float* Zq, const u64* WFq, const SampRow* rq,
                                                    const float* Zp, const u64* WFp, const SampRow* rp,
                                                    long long ldz, long long ldw, int V, int gamma,
                                                    const int* drafts, const float* unif, int* state,
                                                    const int* shadow_ids, int n_shadow, int* result) {
  __shared__ u64 buf[SB];
  __shared__ int found, s_u;
  const int t = threadIdx.x;
  if (t == 0) {
    int u = gamma;
    for (int i = 0; i < gamma; ++i) {
      const int x = drafts[i];
      const SampRow q = rq[i], p = rp[i];
      const double qx = (double)WFq[(long long)i * ldw + x] / (double)q.Wkept;
      const double px = kept(p, Zp[(long long)i * ldz + x], x)
                            ? (double)WFp[(long long)i * ldw + x] / (double)p.Wkept : 0.0;
      if (!((double)unif[i] * qx < px)) { u = i; break; }
    }
    s_u = u;
  }
  __syncthreads();
  const int u = s_u;
  const double r = (double)unif[gamma];
  const float* zp = Zp + (long long)u * ldz;
  const u64* wp = WFp + (long long)u * ldw;
  const SampRow P = rp[u];
  int tok = -1;
  if (u < gamma) {
    const float* zq = Zq + (long long)u * ldz;
    const u64* wq = WFq + (long long)u * ldw;
    const SampRow Q = rq[u];
    const double ip = 1.0 / (double)P.Wkept, iq = 1.0 / (double)Q.Wkept;
    auto res = [&](int j) -> u64 {
      const double pj = kept(P, zp[j], j) ? (double)wp[j] * ip : 0.0;
      const double qj = kept(Q, zq[j], j) ? (double)wq[j] * iq : 0.0;
      const double d = pj - qj;
      return d > 0.0 ? (u64)rint(d * FIX) : 0ull;
    };
    // total residual mass, then the draw
    const int C = (V + SB - 1) / SB;
    const int j0 = min(V, t * C), j1 = min(V, j0 + C);
    u64 sum = 0;
    for (int j = j0; j < j1; ++j) sum += res(j);
    u64 total;
    (void)block_exscan<u64>(sum, buf, &total);
    if (total > 0) {
      const u64 target = (u64)floor(r * (double)total);
      tok = pick_by_mass(res, V, target < total ? target : total - 1, buf, &found);
    }
  }
  if (tok < 0) {
    const u64 target = (u64)floor(r * (double)P.Wkept);
    tok = pick_by_mass([&](int j) -> u64 { return kept(P, zp[j], j) ? wp[j] : 0ull; }, V,
                       target < P.Wkept ? target : P.Wkept - 1, buf, &found);
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
                                unsigned long long* WF, int64_t ldw, SampRow* out, hipStream_t s) {
  if (rows <= 0 || V <= 0 || !(temperature > 0.0) || !(top_p > 0.0)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(samp_rowstats_k, dim3(rows), dim3(SB), 0, s, Z, (long long)ldz, V, 1.0 / temperature, top_p, WF,
                     (long long)ldw, out);
  return hipGetLastError();
}

hipError_t launch_samp_draw(const float* z, int V, const unsigned long long* wf, const SampRow* row, const float* r,
                            int* token_out, unsigned long long* weight_out, int* state_pending, hipStream_t s) {
  hipLaunchKernelGGL(samp_draw_k, dim3(1), dim3(SB), 0, s, z, V, wf, row, r, token_out, weight_out, state_pending);
  return hipGetLastError();
}

hipError_t launch_samp_accept(const float* Zq, const unsigned long long* WFq, const SampRow* rq, const float* Zp,
                              const unsigned long long* WFp, const SampRow* rp, int64_t ldz, int64_t ldw, int V,
                              int gamma, const int* drafts, const float* unif, int* state, const int* shadow_ids,
                              int n_shadow, int* result, hipStream_t s) {
  if (gamma < 0 || V <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(samp_accept_k, dim3(1), dim3(SB), 0, s, Zq, WFq, rq, Zp, WFp, rp, (long long)ldz, (long long)ldw,
                     V, gamma, drafts, unif, state, shadow_ids, n_shadow, result);
  return hipGetLastError();
}

}  // namespace del
