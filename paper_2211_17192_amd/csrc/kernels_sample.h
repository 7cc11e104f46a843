// Sampling kernels: section 2.2 standardisation (temperature softmax / argmax),
// inverse-CDF draws from caller-supplied uniforms, and the accept / resample
// part of Algorithm 1 fused into one launch (row statistics in parallel, then
// the last-finishing workgroup of a sequence takes the decisions, draws the
// extra token and commits / rolls back the sequence state).
//
// Arithmetic of a standardised row z at temperature T > 0:
//   m = max_k z_k,  e_k = exp((z_k - m) / T)  (fp32 hardware exp2 path),
//   S = sum_k e_k (fp64),  prob_k = e_k * (1/S) (fp64).
// Sums and cumulative sums are carried in fp64, so the blocked summation order
// differs from a sequential one only far below the resolution of the uniforms.
// T == 0 uses integer argmax compares (ties to the lowest index).
#pragma once
#include <limits.h>
#include "common.h"

namespace sd {

constexpr int SAMPLE_THREADS = 1024;
constexpr int SAMPLE_CHUNK = 256;           // vocabulary entries per scan chunk (64 lanes x 4)
constexpr int SAMPLE_MAX_CHUNKS = 1024;     // vocab <= 262144
constexpr int SAMPLE_COUNTER_STRIDE = 64;    // uint32 elements between the tickets of two sequences
constexpr int SAMPLE_REG_F4 = 8;            // a row up to 32768 entries is held in registers

struct RowStat {
  float  m;      // max logit
  int    arg;    // lowest index attaining it
  double S;      // sum of e_k over the kept entries
  float  thr;    // entries with a logit below it are dropped (top-k / nucleus); -inf: none
  float  pad;
};

struct SampleSmem {
  float  redf[16];
  double redd[16];
  int    redi[16];
  int    flag;
  int    n;
  int    chunk;          // scan: chunk that holds the threshold
  int    token;
  double before;         // scan: cumulative weight before that chunk
  double total;
  double ctot[SAMPLE_MAX_CHUNKS];
};

__device__ __forceinline__ float exp_scaled(float z, float m, float invT, float thr) {
  return (z >= thr) ? __expf((z - m) * invT) : 0.0f;      // padding (-inf) passes the test and gives 0
}

// Order-preserving map of a float onto unsigned integers, and back.
__device__ __forceinline__ unsigned float_key(float z) {
  const unsigned u = __float_as_uint(z);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(unsigned k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// A row of up to 32768 entries fits the registers of one 1024-thread workgroup:
// thread tid holds float4 number it * 1024 + tid, it = 0..7.  In terms of the
// 256-entry scan chunks, v[it] of wavefront w is lane-slice `lane` of chunk it * 16 + w.
__device__ __forceinline__ bool row_fits_regs(const float* z, int V) {
  return ((V & 3) == 0) && ((reinterpret_cast<uintptr_t>(z) & 15) == 0) &&
         (V <= SAMPLE_REG_F4 * 4 * SAMPLE_THREADS) && (blockDim.x == SAMPLE_THREADS);
}
__device__ __forceinline__ void load_row_regs(const float* __restrict__ z, int V, float4 (&v)[SAMPLE_REG_F4]) {
  const float4* z4 = reinterpret_cast<const float4*>(z);
  const int n4 = V >> 2, tid = threadIdx.x;
#pragma unroll
  for (int it = 0; it < SAMPLE_REG_F4; ++it) {
    const int i = it * SAMPLE_THREADS + tid;
    const float4 t = z4[min(i, n4 - 1)];           // unconditional load, padding by select
    v[it] = (i < n4) ? t : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  }
}
// top_k > 0 / 0 < top_p < 1 (section 2.2: top-k and nucleus sampling as an adjusted
// distribution): the kept set is {z >= thr}.  Top-k: thr = k-th largest logit, found bit by
// bit on the order-preserving integer key (32 counting passes over the registers).  Nucleus,
// applied to what top-k left: thr = the largest value whose upper set still carries top_p of
// the mass, found the same way with sums in place of counts.  Ties with the last kept entry
// are kept.  Argmax sampling ignores both.
__device__ __forceinline__ RowStat row_stats_regs(const float4 (&v)[SAMPLE_REG_F4], float invT, bool greedy,
                                                  SampleSmem& sm, int top_k = 0, float top_p = 0.0f, int V = 0) {
  const int tid = threadIdx.x;
  RowStat st; st.arg = 0; st.S = 0.0; st.thr = -INFINITY; st.pad = 0.0f;
  float m = -INFINITY;
#pragma unroll
  for (int it = 0; it < SAMPLE_REG_F4; ++it)
    m = fmaxf(m, fmaxf(fmaxf(v[it].x, v[it].y), fmaxf(v[it].z, v[it].w)));
  m = block_reduce(m, sm.redf, OpMaxF(), -INFINITY);
  st.m = m;
  if (greedy) {
    int a = INT_MAX;
#pragma unroll
    for (int it = SAMPLE_REG_F4 - 1; it >= 0; --it) {
      const int k = (it * SAMPLE_THREADS + tid) * 4;
      if (v[it].w == m) a = k + 3;
      if (v[it].z == m) a = k + 2;
      if (v[it].y == m) a = k + 1;
      if (v[it].x == m) a = k;
    }
    st.arg = block_reduce(a, sm.redi, OpMinI(), INT_MAX);
    return st;
  }
  float thr = -INFINITY;
  if (top_k > 0 && top_k < V) {
    unsigned tau = 0u;
    for (int bit = 31; bit >= 0; --bit) {
      const unsigned cand = tau | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int it = 0; it < SAMPLE_REG_F4; ++it)
        cnt += (int)(float_key(v[it].x) >= cand) + (int)(float_key(v[it].y) >= cand) +
               (int)(float_key(v[it].z) >= cand) + (int)(float_key(v[it].w) >= cand);
      cnt = block_reduce(cnt, sm.redi, OpSumI(), 0);
      if (cnt >= top_k) tau = cand;
    }
    thr = key_float(tau);
  }
  float s = 0.0f;
#pragma unroll
  for (int it = 0; it < SAMPLE_REG_F4; ++it)       // exp(-inf) = 0 for the padding
    s += (exp_scaled(v[it].x, m, invT, thr) + exp_scaled(v[it].y, m, invT, thr)) +
         (exp_scaled(v[it].z, m, invT, thr) + exp_scaled(v[it].w, m, invT, thr));
  double S = block_reduce((double)s, sm.redd, OpSumD(), 0.0);
  if (top_p > 0.0f && top_p < 1.0f) {
    const double target = (double)top_p * S;
    const float floor_thr = thr;                   // what top-k dropped stays dropped
    unsigned tau = 0u;
    for (int bit = 31; bit >= 0; --bit) {
      const unsigned cand = tau | (1u << bit);
      const float ct = fmaxf(key_float(cand), floor_thr);
      float part = 0.0f;
#pragma unroll
      for (int it = 0; it < SAMPLE_REG_F4; ++it)
        part += (exp_scaled(v[it].x, m, invT, ct) + exp_scaled(v[it].y, m, invT, ct)) +
                (exp_scaled(v[it].z, m, invT, ct) + exp_scaled(v[it].w, m, invT, ct));
      const double mass = block_reduce((double)part, sm.redd, OpSumD(), 0.0);
      if (mass >= target) { tau = cand; S = mass; }
    }
    thr = fmaxf(key_float(tau), floor_thr);
  }
  st.S = S;
  st.thr = thr;
  return st;
}

// max / argmax / sum-of-exponentials of one logits row; every thread gets it.
// Rows of up to 32768 entries are read from memory exactly once.
__device__ __forceinline__ RowStat row_stats(const float* __restrict__ z, int V, float invT,
                                             bool greedy, SampleSmem& sm, int top_k = 0, float top_p = 0.0f) {
  const int tid = threadIdx.x, nt = blockDim.x;
  RowStat st; st.arg = 0; st.S = 0.0; st.thr = -INFINITY; st.pad = 0.0f;
  if (row_fits_regs(z, V)) {
    float4 v[SAMPLE_REG_F4];
    load_row_regs(z, V, v);
    return row_stats_regs(v, invT, greedy, sm, top_k, top_p, V);
  }
  // longer rows: no top-k / nucleus (the host side refuses the combination)
  float m = -INFINITY;
  for (int i = tid; i < V; i += nt) m = fmaxf(m, z[i]);
  m = block_reduce(m, sm.redf, OpMaxF(), -INFINITY);
  st.m = m;
  if (greedy) {
    int a = INT_MAX;
    for (int i = tid; i < V; i += nt) if (z[i] == m) a = min(a, i);
    st.arg = block_reduce(a, sm.redi, OpMinI(), INT_MAX);
    return st;
  }
  double s = 0.0;
  for (int i = tid; i < V; i += nt) s += (double)exp_scaled(z[i], m, invT, -INFINITY);
  st.S = block_reduce(s, sm.redd, OpSumD(), 0.0);
  return st;
}

// The four weights of entries k..k+3: prob_p, minus prob_q clipped at zero when
// a draft row is given (the unnormalised adjusted distribution of section 2.3).
struct RowPair {
  const float* zp; const float* zq;     // zq == nullptr: plain row
  float mp, mq;
  float tp, tq;                         // drop thresholds of the two rows
  double invSp, invSq;
  float invT;
  int V;
  bool vec;
};

__device__ __forceinline__ void load4(const RowPair& rp, int k, float (&zp)[4], float (&zq)[4]) {
  if (rp.vec && k + 3 < rp.V) {
    const float4 a = *reinterpret_cast<const float4*>(rp.zp + k);
    zp[0] = a.x; zp[1] = a.y; zp[2] = a.z; zp[3] = a.w;
    if (rp.zq) {
      const float4 b = *reinterpret_cast<const float4*>(rp.zq + k);
      zq[0] = b.x; zq[1] = b.y; zq[2] = b.z; zq[3] = b.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      zp[e] = (k + e < rp.V) ? rp.zp[k + e] : -INFINITY;
      zq[e] = (rp.zq && k + e < rp.V) ? rp.zq[k + e] : -INFINITY;
    }
  }
}

__device__ __forceinline__ void calc4(const RowPair& rp, int k, const float (&zp)[4], const float (&zq)[4],
                                      double (&w)[4]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    double p = (k + e < rp.V) ? (double)exp_scaled(zp[e], rp.mp, rp.invT, rp.tp) * rp.invSp : 0.0;
    if (rp.zq) {
      const double q = (k + e < rp.V) ? (double)exp_scaled(zq[e], rp.mq, rp.invT, rp.tq) * rp.invSq : 0.0;
      p -= q;
      p = p > 0.0 ? p : 0.0;
    }
    w[e] = p;
  }
}

__device__ __forceinline__ void weights4(const RowPair& rp, int k, double (&w)[4]) {
  float zp[4], zq[4];
  load4(rp, k, zp, zq);
  calc4(rp, k, zp, zq, w);
}

// Wavefront 0: scan the chunk totals (lane l owns chunks [l*cpl, (l+1)*cpl)), find the
// chunk in which the cumulative weight first exceeds u * total, and leave in sm:
// total, chunk (or -1 - last chunk with positive weight when round-off keeps the
// threshold out of reach) and the cumulative weight before that chunk.
__device__ __forceinline__ void scan_chunk_totals(int nchunks, float u, SampleSmem& sm) {
  const int lane = threadIdx.x & 63;
  const int cpl = (nchunks + 63) / 64;
  const int c0 = min(nchunks, lane * cpl), c1 = min(nchunks, c0 + cpl);
  double local = 0.0;
  for (int c = c0; c < c1; ++c) local += sm.ctot[c];
  double inc = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double t = __shfl_up(inc, o, WAVE);
    if (lane >= o) inc += t;
  }
  const double total = __shfl(inc, 63, WAVE);
  const double theta = (double)u * total;
  double cum = inc - local;
  int found = INT_MAX;
  double before = 0.0;
  for (int c = c0; c < c1; ++c) {
    const double nx = cum + sm.ctot[c];
    if (found == INT_MAX && nx > theta) { found = c; before = cum; }
    cum = nx;
  }
  const int first = wave_min(found);
  int lastpos = -1;
  for (int c = c0; c < c1; ++c) if (sm.ctot[c] > 0.0) lastpos = c;
  lastpos = wave_max(lastpos);
  if (found == first && first != INT_MAX) { sm.chunk = first; sm.before = before; }
  if (lane == 0) {
    sm.total = total;
    if (first == INT_MAX) { sm.chunk = -1 - lastpos; sm.before = 0.0; }
  }
}

// One wavefront: entry by entry scan of a 256-entry chunk (lane holds entries k..k+3 with
// weights w).  Returns in every lane the first entry whose cumulative weight exceeds theta,
// or, in fallback mode / if none does, the last entry with positive weight.
__device__ __forceinline__ int pick_in_chunk(const double (&w)[4], int k, int V, bool fallback, double theta,
                                             double before) {
  const int lane = threadIdx.x & 63;
  const double local = (w[0] + w[1]) + (w[2] + w[3]);
  double inc = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double t = __shfl_up(inc, o, WAVE);
    if (lane >= o) inc += t;
  }
  int cand = INT_MAX;
  if (!fallback) {
    double cum = before + (inc - local);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      cum += w[e];
      if (cand == INT_MAX && cum > theta && k + e < V) cand = k + e;
    }
    cand = wave_min(cand);
  }
  if (cand == INT_MAX) {
    int lp = -1;
#pragma unroll
    for (int e = 0; e < 4; ++e) if (w[e] > 0.0 && k + e < V) lp = k + e;
    cand = wave_max(lp);
  }
  return cand;
}

// Inverse-CDF draw: smallest k with cumulative weight > u * total weight, in
// vocabulary order.  Chunks of 256 consecutive entries are summed by one
// wavefront each (coalesced 1 KB reads), the chunk totals are scanned, and only
// the chunk that holds the threshold is scanned entry by entry.  Returns -1 in
// every thread if the total weight is not positive (the caller then falls back
// to the unadjusted row).
__device__ __forceinline__ int icdf_row(const float* zp, const RowStat& sp, const float* zq,
                                        const RowStat& sq, float invT, int V, float u,
                                        SampleSmem& sm, double qscale = 1.0) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
  RowPair rp;
  rp.zp = zp; rp.zq = zq; rp.mp = sp.m; rp.mq = sq.m; rp.tp = sp.thr; rp.tq = sq.thr;
  rp.invSp = 1.0 / sp.S; rp.invSq = zq ? qscale / sq.S : 0.0;     // q enters the residual as qscale * q
  rp.invT = invT; rp.V = V;
  rp.vec = ((V & 3) == 0) && ((reinterpret_cast<uintptr_t>(zp) & 15) == 0) &&
           (zq == nullptr || (reinterpret_cast<uintptr_t>(zq) & 15) == 0);
  const int nchunks = (V + SAMPLE_CHUNK - 1) / SAMPLE_CHUNK;
  __syncthreads();
  constexpr int CB = 4;                          // chunks whose loads a wavefront keeps in flight
  for (int cb = wave; cb < nchunks; cb += nw * CB) {
    float zpv[CB][4], zqv[CB][4];
#pragma unroll
    for (int u = 0; u < CB; ++u) {
      const int c = cb + u * nw;
      if (c < nchunks) load4(rp, c * SAMPLE_CHUNK + lane * 4, zpv[u], zqv[u]);
    }
#pragma unroll
    for (int u = 0; u < CB; ++u) {
      const int c = cb + u * nw;
      if (c < nchunks) {
        double w[4];
        calc4(rp, c * SAMPLE_CHUNK + lane * 4, zpv[u], zqv[u], w);
        const double t = wave_sum((w[0] + w[1]) + (w[2] + w[3]));
        if (lane == 0) sm.ctot[c] = t;
      }
    }
  }
  __syncthreads();
  if (wave == 0) scan_chunk_totals(nchunks, u, sm);
  __syncthreads();
  const double total = sm.total;
  if (!(total > 0.0)) return -1;
  const int chunk = sm.chunk;
  if (wave == 0) {
    const bool fallback = chunk < 0;          // threshold not reached by round-off
    const int c = fallback ? (-1 - chunk) : chunk;
    const int k = c * SAMPLE_CHUNK + lane * 4;
    double w[4];
    weights4(rp, k, w);
    const int tok = pick_in_chunk(w, k, V, fallback, (double)u * total, sm.before);
    if (lane == 0) sm.token = tok;
  }
  __syncthreads();
  return sm.token;
}

// Inverse-CDF draw from rows held in registers (see row_fits_regs for the layout):
// same arithmetic and summation order as icdf_row, without touching memory.
__device__ __forceinline__ void weights_of(const float4& zp, const float4& zq, bool with_q, float mp, float mq,
                                           float tp, float tq, double invSp, double invSq, float invT,
                                           double (&w)[4]) {
  const float a[4] = {zp.x, zp.y, zp.z, zp.w}, b[4] = {zq.x, zq.y, zq.z, zq.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    double p = (double)exp_scaled(a[e], mp, invT, tp) * invSp;    // padding: exp(-inf) = 0
    if (with_q) {
      p -= (double)exp_scaled(b[e], mq, invT, tq) * invSq;
      p = p > 0.0 ? p : 0.0;
    }
    w[e] = p;
  }
}

__device__ __forceinline__ int icdf_regs(const float4 (&vp)[SAMPLE_REG_F4], const RowStat& sp,
                                         const float4 (&vq)[SAMPLE_REG_F4], const RowStat& sq, bool with_q,
                                         float invT, int V, float u, SampleSmem& sm, double qscale = 1.0) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NW = SAMPLE_THREADS / 64;
  const double invSp = 1.0 / sp.S, invSq = with_q ? qscale / sq.S : 0.0;
  const int nchunks = (V + SAMPLE_CHUNK - 1) / SAMPLE_CHUNK;
  __syncthreads();
#pragma unroll
  for (int it = 0; it < SAMPLE_REG_F4; ++it) {
    const int c = it * NW + wave;
    double w[4];
    weights_of(vp[it], vq[it], with_q, sp.m, sq.m, sp.thr, sq.thr, invSp, invSq, invT, w);
    const double t = wave_sum((w[0] + w[1]) + (w[2] + w[3]));
    if (lane == 0 && c < nchunks) sm.ctot[c] = t;
  }
  __syncthreads();
  if (wave == 0) scan_chunk_totals(nchunks, u, sm);
  __syncthreads();
  const double total = sm.total;
  if (!(total > 0.0)) return -1;
  const int chunk = sm.chunk;
  const bool fallback = chunk < 0;            // threshold not reached by round-off
  const int c = fallback ? (-1 - chunk) : chunk;
  if (wave == c % NW) {
    double w[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int it = 0; it < SAMPLE_REG_F4; ++it)
      if (it == c / NW) weights_of(vp[it], vq[it], with_q, sp.m, sq.m, sp.thr, sq.thr, invSp, invSq, invT, w);
    const int tok = pick_in_chunk(w, c * SAMPLE_CHUNK + lane * 4, V, fallback, (double)u * total, sm.before);
    if (lane == 0) sm.token = tok;
  }
  __syncthreads();
  return sm.token;
}

// ---------------------------------------------------------------------------
// Draw one token from one logits row: x_i ~ q_i of the draft loop, or the
// plain-decoding draw t ~ p.
//   mode 0: store the token as guess number `slot` (st->x[slot])
//   mode 1: commit it (standard decoding): len += 1
// Several sequences: sequence b reads the row at logits + b * seq_stride (floats) and uses
// prm[b], st[b].
// ---------------------------------------------------------------------------
// The draw is spread over SAMPLE_SPLIT workgroups per row.  One workgroup is bound by its own
// instruction stream (32 exponentials per thread, twice, and the fp64 weights: 8.5 us on one CU for
// a 32128-entry row), so here every workgroup finds the row's maximum itself (a cheap pass over the
// whole row), then takes one register slice of the row: chunks w * 16 .. w * 16 + 15 for workgroup
// w, one wavefront per 256-entry chunk as in icdf_regs.  The chunk totals go to `tot`
// ([sequence][SAMPLE_MAX_CHUNKS] doubles); the workgroup that arrives last (ticket: one counter
// per sequence, SAMPLE_COUNTER_STRIDE words apart, zero before and after) scans them and walks
// the chunk that holds u * total.  The weights are exp((z - m) / T) without the division by
// their sum: both sides of "cumulative weight > u * total" carry the same factor.
// Argmax sampling, top-k / nucleus and rows that do not fit the registers are left to workgroup 0,
// which then does the whole row (statistics and draw from registers, one read of the row); the others leave at once.  grid = (SAMPLE_SPLIT, sequences).
constexpr int SAMPLE_SPLIT = SAMPLE_REG_F4;

__device__ __forceinline__ void commit_draw(SeqState* st, int mode, int slot, int tok) {
  if (mode == 0) {
    st->x[slot] = tok;
  } else {
    st->prev_tok = st->last_tok;
    st->last_tok = tok;
    st->len += 1;
    st->n = 0;
    st->out[0] = tok;
  }
}

static __global__ __launch_bounds__(SAMPLE_THREADS) void sample_row_split_kernel(
    const float* __restrict__ logits, int V, const StepParams* __restrict__ prm, int uniform_idx,
    SeqState* __restrict__ st, int mode, int slot, size_t seq_stride, double* __restrict__ tot,
    unsigned int* __restrict__ ticket) {
  __shared__ SampleSmem sm;
  const int w = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  logits += (size_t)blockIdx.y * seq_stride;
  prm += blockIdx.y;
  st += blockIdx.y;
  tot += (size_t)blockIdx.y * SAMPLE_MAX_CHUNKS;
  ticket += (size_t)blockIdx.y * SAMPLE_COUNTER_STRIDE;
  const float T = prm->temperature;
  const bool greedy = (T == 0.0f);
  const float invT = greedy ? 1.0f : 1.0f / T;
  const bool filtered = prm->top_k > 0 || (prm->top_p > 0.0f && prm->top_p < 1.0f);
  if (greedy || filtered || !row_fits_regs(logits, V)) {      // uniform over the grid's workgroups of this row
    if (w != 0) return;
    int tok;
    if (row_fits_regs(logits, V)) {
      float4 v[SAMPLE_REG_F4];
      load_row_regs(logits, V, v);
      const RowStat rs = row_stats_regs(v, invT, greedy, sm, prm->top_k, prm->top_p, V);
      tok = greedy ? rs.arg : icdf_regs(v, rs, v, rs, false, invT, V, prm->uniforms[uniform_idx], sm);
    } else {
      const RowStat rs = row_stats(logits, V, invT, greedy, sm);
      tok = greedy ? rs.arg : icdf_row(logits, rs, nullptr, rs, invT, V, prm->uniforms[uniform_idx], sm);
    }
    if (tid == 0) commit_draw(st, mode, slot, tok);
    return;
  }
  const float4* z4 = reinterpret_cast<const float4*>(logits);
  const int n4 = V >> 2, nchunks = (V + SAMPLE_CHUNK - 1) / SAMPLE_CHUNK;
  const float4 pad = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  // the row's maximum, and this workgroup's slice (float4 number w * 1024 + tid: lane-slice `lane` of chunk w * 16 + wave)
  float m = -INFINITY;
  float4 mine = pad;
  {
    float4 v[SAMPLE_REG_F4];
    load_row_regs(logits, V, v);
#pragma unroll
    for (int it = 0; it < SAMPLE_REG_F4; ++it) {
      m = fmaxf(m, fmaxf(fmaxf(v[it].x, v[it].y), fmaxf(v[it].z, v[it].w)));
      if (it == w) mine = v[it];
    }
  }
  m = block_reduce(m, sm.redf, OpMaxF(), -INFINITY);
  const int c = w * (SAMPLE_THREADS / 64) + wave;
  {
    const double t = wave_sum(((double)exp_scaled(mine.x, m, invT, -INFINITY) + (double)exp_scaled(mine.y, m, invT, -INFINITY)) +
                              ((double)exp_scaled(mine.z, m, invT, -INFINITY) + (double)exp_scaled(mine.w, m, invT, -INFINITY)));
    if (lane == 0 && c < nchunks) tot[c] = t;
  }
  if (!last_block_arrives(ticket, SAMPLE_SPLIT, &sm.flag)) return;
  for (int i = tid; i < nchunks; i += SAMPLE_THREADS) sm.ctot[i] = tot[i];
  __syncthreads();
  const float u = prm->uniforms[uniform_idx];
  if (wave == 0) scan_chunk_totals(nchunks, u, sm);
  __syncthreads();
  if (wave == 0) {
    const double total = sm.total;
    const int chunk = sm.chunk;
    const bool fallback = chunk < 0;            // threshold not reached by round-off
    const int cc = fallback ? (-1 - chunk) : chunk;
    const int i4 = cc * (SAMPLE_CHUNK / 4) + lane;
    const float4 t4 = z4[min(i4, n4 - 1)];
    const float4 z = (i4 < n4) ? t4 : pad;
    const double wv[4] = {(double)exp_scaled(z.x, m, invT, -INFINITY), (double)exp_scaled(z.y, m, invT, -INFINITY),
                          (double)exp_scaled(z.z, m, invT, -INFINITY), (double)exp_scaled(z.w, m, invT, -INFINITY)};
    const int tok = pick_in_chunk(wv, i4 * 4, V, fallback, (double)u * total, sm.before);
    if (lane == 0) commit_draw(st, mode, slot, tok);
  }
}

// ---------------------------------------------------------------------------
// Accept / resample (Algorithm 1, second half).  grid = (2*gamma+1, rows):
// block (j, b) computes the statistics of logits row j of sequence b (j <=
// gamma: p_{j+1}; j > gamma: q_{j-gamma}); the last block of a sequence to
// finish then
//   * evaluates r_i <= p_i(x_i)/q_i(x_i) for all i in one wavefront and takes
//     n = index of the first rejection from the ballot,
//   * draws t from norm(max(0, p_{n+1} - q_{n+1})) (n < gamma) or p_{gamma+1},
//   * writes n and t, and, when `st` is given, commits the sequence:
//     out = x_1..x_n, t; len += n+1 (which is the KV roll-back: cache rows
//     beyond the committed length are dead and get overwritten).
// x, r, s: explicit arrays [rows, gamma] / [rows] or, when prm/st are given,
// taken from the device-resident step parameters and state.
// ---------------------------------------------------------------------------
// MODE 0: everything in one launch (ticket).  MODE 1: row statistics only.  MODE 2: the
// per-sequence tail only, grid (1, rows).  MODE 3: the acceptance probabilities beta_i as a
// side output, grid (gamma, rows), after the statistics exist.  A device-scope atomic costs about 0.08 us of
// chip-wide throughput, so with many sequences two launches (1 + 2) beat rows * (2*gamma+1)
// tickets; with one sequence the single launch wins.
template <int MODE>
static __global__ __launch_bounds__(SAMPLE_THREADS) void spec_verify_kernel(
    const float* __restrict__ p_logits, const float* __restrict__ q_logits,
    const int* __restrict__ x_in, const float* __restrict__ r_in, const float* __restrict__ s_in,
    int gamma, int V, float temperature, float lenience_in, double log_lenience_in, int top_k_in, float top_p_in,
    const StepParams* __restrict__ prm,
    RowStat* __restrict__ stats, unsigned int* __restrict__ counters,
    int* __restrict__ out_n, int* __restrict__ out_t, float* __restrict__ beta_out,
    SeqState* __restrict__ st) {
  __shared__ SampleSmem sm;
  __shared__ RowStat srow[2 * 15 + 1];
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int nrows = 2 * gamma + 1;
  if (prm) prm += b;                     // in-model use: per-sequence parameters and state
  if (st) st += b;
  const float T = prm ? prm->temperature : temperature;
  const bool greedy = (T == 0.0f);
  const float invT = greedy ? 1.0f : 1.0f / T;
  const double len = (double)(prm ? prm->lenience : lenience_in);            // appendix A.5, 1 = exact
  const double log_len = prm ? prm->log_lenience : log_lenience_in;
  const int top_k = prm ? prm->top_k : top_k_in;                             // section 2.2, same for p and q
  const float top_p = prm ? prm->top_p : top_p_in;
  const float* P = p_logits + (size_t)b * (gamma + 1) * V;
  const float* Q = q_logits + (size_t)b * gamma * V;
  RowStat* my_stats = stats + (size_t)b * nrows;

  if (MODE == 3) {
    // beta_{j+1} = sum_x min(p(x) / l, q(x)): the probability that guess j+1 is accepted
    // (section 3.1; with lenience, appendix A.5).  Needs the statistics of a MODE 0 / 1 launch.
    if (j >= gamma) return;
    const RowStat sp = my_stats[j];
    const float* zp = P + (size_t)j * V;
    float* dst = st ? st->beta : beta_out + (size_t)b * gamma;
    if (greedy) {                                // one-hot q at its argmax: accepted or not
      const int aq = row_stats(Q + (size_t)j * V, V, 1.0f, true, sm).arg;   // argmax sampling keeps no q statistics
      if (tid == 0) {
        const bool acc = (len < 1.0) ? ((double)zp[aq] - (double)sp.m >= log_len) : (aq == sp.arg);
        dst[j] = acc ? 1.0f : 0.0f;
      }
      return;
    }
    const RowStat sq = my_stats[gamma + 1 + j];
    const float* zq = Q + (size_t)j * V;
    const double ip = (1.0 / sp.S) / len, iq = 1.0 / sq.S;
    double acc = 0.0;
    for (int k = tid; k < V; k += SAMPLE_THREADS) {
      const double pv = (double)exp_scaled(zp[k], sp.m, invT, sp.thr) * ip;
      const double qv = (double)exp_scaled(zq[k], sq.m, invT, sq.thr) * iq;
      acc += pv < qv ? pv : qv;
    }
    acc = block_reduce(acc, sm.redd, OpSumD(), 0.0);
    if (tid == 0) dst[j] = (float)acc;
    return;
  }

  if (MODE != 2 && !(greedy && j > gamma)) {          // argmax sampling never looks at q rows
    const float* z = (j <= gamma) ? P + (size_t)j * V : Q + (size_t)(j - gamma - 1) * V;
    const RowStat rs = row_stats(z, V, invT, greedy, sm, top_k, top_p);
    if (tid == 0) my_stats[j] = rs;
  }
  if (MODE == 1) return;
  // one counter per sequence, 256 bytes apart
  if (MODE == 0 && !last_block_arrives(counters + (size_t)b * SAMPLE_COUNTER_STRIDE, (unsigned)nrows, &sm.flag)) return;

  // ---- tail: one workgroup per sequence ----
  if (tid < nrows) srow[tid] = my_stats[tid];
  __syncthreads();
  const int* x = st ? st->x : x_in + (size_t)b * gamma;
  const float* r = prm ? prm->uniforms + gamma : r_in + (size_t)b * gamma;
  const float s = greedy ? 0.5f : (prm ? prm->uniforms[2 * gamma] : s_in[b]);

  if (tid < WAVE) {                       // wavefront 0: one lane per guess
    bool reject = false;
    if (tid < gamma) {
      const int xi = min(max(x[tid], 0), V - 1);
      if (greedy) {
        // lenient argmax sampling: keep x when p(x) >= l * max p, p = softmax of the raw logits
        reject = (len < 1.0) ? ((double)P[(size_t)tid * V + xi] - (double)srow[tid].m < log_len)
                             : (srow[tid].arg != xi);
      } else {
        const RowStat sp = srow[tid], sq = srow[gamma + 1 + tid];
        const double p = (double)exp_scaled(P[(size_t)tid * V + xi], sp.m, invT, sp.thr) * (1.0 / sp.S);
        const double q = (double)exp_scaled(Q[(size_t)tid * V + xi], sq.m, invT, sq.thr) * (1.0 / sq.S);
        const double lq = q * len;
        const double ratio = (lq > 0.0) ? p / lq : INFINITY;
        reject = ((double)r[tid] > ratio);
      }
    }
    const unsigned long long mask = __ballot(reject);
    if (tid == 0) sm.n = mask ? (__ffsll((long long)mask) - 1) : gamma;
  }
  __syncthreads();
  const int n = sm.n;
  int t;
  int fell_back = 0;
  if (greedy) {
    t = srow[n].arg;
  } else {
    const float* zp = P + (size_t)n * V;
    const float* zq = Q + (size_t)min(n, gamma - 1) * V;
    const RowStat sq = srow[gamma + 1 + min(n, gamma - 1)];
    if (row_fits_regs(zp, V) && row_fits_regs(zq, V)) {
      float4 vp[SAMPLE_REG_F4], vq[SAMPLE_REG_F4];
      load_row_regs(zp, V, vp);
      load_row_regs(zq, V, vq);               // unconditional; unused when all guesses were kept
      t = icdf_regs(vp, srow[n], vq, sq, n < gamma, invT, V, s, sm, len);
      if (t < 0) { fell_back = 1; t = icdf_regs(vp, srow[n], vq, sq, false, invT, V, s, sm); }
    } else if (n < gamma) {
      t = icdf_row(zp, srow[n], zq, sq, invT, V, s, sm, len);
      if (t < 0) { fell_back = 1; t = icdf_row(zp, srow[n], nullptr, srow[n], invT, V, s, sm); }
    } else {
      t = icdf_row(zp, srow[n], nullptr, srow[n], invT, V, s, sm);
    }
  }
  if (tid == 0) {
    if (out_n) out_n[b] = n;
    if (out_t) out_t[b] = t;
    if (st) {
      const int last = st->last_tok;
      for (int i = 0; i < 16; ++i) st->out[i] = (i < n) ? x[i] : (i == n ? t : -1);
      st->prev_tok = (n >= 1) ? x[n - 1] : last;
      st->last_tok = t;
      st->len += n + 1;
      st->n = n;
      st->fallbacks += fell_back;
    }
  }
}

}  // namespace sd
