// Row set-up + embedding: decides which tokens a forward processes, from the
// device-resident sequence state, and writes their embeddings into the fp32
// residual stream.  Keeping this on the device lets one captured graph serve
// every iteration.
#pragma once
#include "common.h"

namespace sd {

enum {
  ROWS_VERIFY = 0,       // Mp scoring of Algorithm 1: [last token, x_1..x_gamma] at len-1 ..
  ROWS_DRAFT_FIRST = 1,  // first Mq step: the last two committed tokens at len-2, len-1
  ROWS_DRAFT_NEXT = 2,   // Mq step i >= 2: x_{i-1} at len-2+i
  ROWS_BASELINE = 3,     // standard decoding: last token at len-1
  ROWS_PREFILL = 4       // prompt[start .. start+R) at start ..
};

// grid = R workgroups.  row_pos[r] < 0 marks a padding row (first draft step of
// a one-token sequence): it is embedded as token 0 at position 0 and ignored.
// For RMSNorm models the kernel also writes xg = x * gain of the first norm in
// the storage type and the row's sum of squares (one partial: ss[0][r]).
// Several sequences: the launch covers sequences seq0, seq0+1, ... with rps rows
// each, one after the other: workgroup b (sequence seq0 + b / rps) writes row b of
// x / xg / row_pos / ..., and the sum of squares of its row into the block of ss that
// belongs to the row's slab of MAX_ROWS rows (ss_stride floats per slab); `st` is the array
// of sequence states.  row_seq[r] (when given) receives the row's sequence, logit_row[r] the
// row of the logits buffer its LM-head output belongs in (< 0: not needed):
// p rows [seq][gamma+1], q rows [seq][gamma], one row per sequence for plain decoding.
template <typename T>
static __global__ __launch_bounds__(256) void embed_kernel(
    int mode, int step, const SeqState* __restrict__ st, const int* __restrict__ prompt, int start,
    const T* __restrict__ tok_emb, const T* __restrict__ pos_emb, int d, int vocab,
    float* __restrict__ x, int* __restrict__ row_pos, const T* __restrict__ gain_next,
    T* __restrict__ xg, float* __restrict__ ss,
    int rps, int seq0, int gamma, int* __restrict__ row_seq, int* __restrict__ logit_row,
    int ss_stride) {
  __shared__ float red[16];
  const int j = (int)blockIdx.x % rps, sl = (int)blockIdx.x / rps, seq = seq0 + sl;
  const int r = blockIdx.x, slab = r / MAX_ROWS, r16 = r % MAX_ROWS;     // row, its slab, row within the slab
  st += seq;
  int tok, pos, lrow = -1;
  switch (mode) {
    case ROWS_VERIFY:      tok = (j == 0) ? st->last_tok : st->x[j - 1]; pos = st->len - 1 + j; lrow = seq * (gamma + 1) + j; break;
    case ROWS_DRAFT_FIRST: tok = (j == 0) ? st->prev_tok : st->last_tok; pos = st->len - 2 + j; lrow = (j == 1) ? seq * gamma : -1; break;
    case ROWS_DRAFT_NEXT:  tok = st->x[step - 1]; pos = st->len - 1 + step; lrow = seq * gamma + step; break;
    case ROWS_BASELINE:    tok = st->last_tok; pos = st->len - 1; lrow = seq; break;
    default:               tok = prompt[start + r]; pos = start + r; break;
  }
  if (threadIdx.x == 0 && row_seq) { row_seq[r] = seq; logit_row[r] = lrow; }
  if (threadIdx.x == 0) row_pos[r] = pos;
  if (pos < 0) { tok = 0; pos = 0; }
  tok = min(max(tok, 0), vocab - 1);
  const T* e = tok_emb + (size_t)tok * d;
  const T* p = pos_emb ? pos_emb + (size_t)pos * d : nullptr;
  float q = 0.0f;
  // 8 consecutive elements per thread and step, four steps in flight: the row
  // comes from cold memory and the loop would otherwise pay its latency per step
  const int ngroups = d >> 3;                       // d is a multiple of 32
  for (int g0 = threadIdx.x; g0 < ngroups; g0 += blockDim.x * 4) {
    float v[4][8], w[4][8], gn[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int g = g0 + u * blockDim.x;
      if (g < ngroups) {
        load8<T>(e + g * 8, v[u]);
        if (p) load8<T>(p + g * 8, w[u]);
        if (xg) load8<T>(gain_next + g * 8, gn[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int g = g0 + u * blockDim.x;
      if (g < ngroups) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          float val = v[u][k];
          if (p) val += w[u][k];
          x[(size_t)r * d + g * 8 + k] = val;
          if (xg) Store<T>::st(xg + (size_t)r * d + g * 8 + k, val * gn[u][k]);
          q += val * val;
        }
      }
    }
  }
  if (ss) {
    q = block_reduce(q, red, OpSumF(), 0.0f);
    if (threadIdx.x == 0) ss[(size_t)slab * ss_stride + r16] = q;
  }
}

// Negligible-cost approximation model (an n-gram table): the draft logits of guess `step`
// of sequence b are the table row selected by the previous token (bigram; row_of == nullptr:
// one row for every context, a unigram model).  grid = (slices, sequences); the row is
// copied to dst + b * seq_stride, where the sampling kernels expect the draft's logits.
static __global__ __launch_bounds__(256) void table_row_kernel(
    const float* __restrict__ table, const int* __restrict__ row_of, int n_rows, int V,
    const SeqState* __restrict__ st, int step, float* __restrict__ dst, size_t seq_stride) {
  st += blockIdx.y;
  int prev = (step == 0) ? st->last_tok : st->x[step - 1];
  prev = min(max(prev, 0), V - 1);
  int row = (row_of != nullptr) ? row_of[prev] : 0;
  row = min(max(row, 0), n_rows - 1);
  const float* src = table + (size_t)row * V;
  float* out = dst + (size_t)blockIdx.y * seq_stride;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < V; i += gridDim.x * blockDim.x) out[i] = src[i];
}

// Copying draft (section 3.6): the context is the committed tokens hist[0, len) of sequence b
// followed by this iteration's guesses x[0, step).  Its last `match` tokens are searched among
// their earlier occurrences; the most recent one that has a successor decides: the draft's
// logits row is 0 at that successor and -inf elsewhere.  Without an occurrence the row is the
// table row (as in table_row_kernel) or, with no table, all zeros: the uniform model.
// grid = (slices, sequences); every workgroup repeats the search and writes its slice.
static __global__ __launch_bounds__(256) void copy_row_kernel(
    const int* __restrict__ hist, int hist_stride, int match, const float* __restrict__ table,
    const int* __restrict__ row_of, int n_rows, int V, const SeqState* __restrict__ st, int step,
    float* __restrict__ dst, size_t seq_stride) {
  st += blockIdx.y;
  const int* h = hist + (size_t)blockIdx.y * hist_stride;
  const int L = min(max(st->len, 0), hist_stride), S = L + step;
  auto tok = [&](int i) { return i < L ? h[i] : st->x[min(i - L, 15)]; };
  __shared__ int found;
  if (threadIdx.x == 0) found = -1;
  __syncthreads();
  int best = -1;
  for (int j = threadIdx.x; j + match < S; j += blockDim.x) {      // occurrence at [j, j+match), successor j+match
    bool same = true;
    for (int t = 0; t < match; ++t) same = same && tok(j + t) == tok(S - match + t);
    if (same) best = j;
  }
  if (best >= 0) atomicMax(&found, best);
  __syncthreads();
  float* out = dst + (size_t)blockIdx.y * seq_stride;
  const int i0 = blockIdx.x * blockDim.x + threadIdx.x, di = gridDim.x * blockDim.x;
  if (found >= 0) {
    const int x = min(max(tok(found + match), 0), V - 1);
    for (int i = i0; i < V; i += di) out[i] = (i == x) ? 0.0f : -INFINITY;
  } else if (table != nullptr) {
    int prev = (step == 0) ? st->last_tok : st->x[step - 1];
    prev = min(max(prev, 0), V - 1);
    int row = (row_of != nullptr) ? row_of[prev] : 0;
    row = min(max(row, 0), n_rows - 1);
    const float* src = table + (size_t)row * V;
    for (int i = i0; i < V; i += di) out[i] = src[i];
  } else {
    for (int i = i0; i < V; i += di) out[i] = 0.0f;
  }
}

// Keeps the token history that copy_row_kernel searches: after an iteration of Algorithm 1
// (spec != 0) the n+1 emitted tokens, after a plain decoding step the one new token, at the
// positions they were committed to.  grid = sequences, 32 threads.
static __global__ void hist_append_kernel(int* __restrict__ hist, int hist_stride, const SeqState* __restrict__ st, int spec) {
  st += blockIdx.x;
  int* h = hist + (size_t)blockIdx.x * hist_stride;
  const int L = st->len, t = threadIdx.x;
  const int cnt = spec ? min(max(st->n, 0), 15) + 1 : 1;
  const int pos = L - cnt + t;
  if (t < cnt && pos >= 0 && pos < hist_stride) h[pos] = spec ? st->out[t] : st->last_tok;
}

// Pure streaming read (measurement): the grid's wavefronts walk the buffer in the GEMMs' access
// shape, 1 KB per wavefront and load, `depth` KB in flight per wavefront, every byte exactly once
// (n_blocks 1-KB blocks, wavefront w of W takes blocks w, w + W, ... in runs of `run` blocks).
// The sum lands in *sink only if it equals a value it cannot have, so the loads are not removed.
static __global__ __launch_bounds__(512) void stream_read_kernel(const f32x4* __restrict__ src, size_t n_blocks, float* sink) {
  const int lane = threadIdx.x & 63;
  const size_t W = (size_t)gridDim.x * (blockDim.x >> 6), w = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const size_t per_wave = (n_blocks + W - 1) / W;            // consecutive blocks per wavefront
  const size_t b0 = w * per_wave, b1 = (b0 + per_wave < n_blocks) ? b0 + per_wave : n_blocks;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int U = 8;
  for (size_t b = b0; b < b1; b += U) {
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {                            // unconditional loads, out-of-range ones re-read the last block
      const size_t bb = (b + u < b1) ? b + u : b1 - 1;
      v[u] = __builtin_nontemporal_load(src + bb * 64 + lane);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (b + u < b1) acc += v[u];
  }
  if (acc.x + acc.y + acc.z + acc.w == 1.2345e-31f) *sink = acc.x;
}

// Relative-position bias by causal distance: out[h][max_len - 1 - d] = rel_bias[h][bucket_lut[d]] for
// d in [0, max_len), three zeros after it (rows of max_len + 3 floats): consecutive keys of one query
// position are consecutive entries.
template <typename T>
static __global__ void bias_by_key_kernel(const T* __restrict__ rel_bias, const int* __restrict__ bucket_lut, int rel_buckets,
                                          int max_len, int n_heads, float* __restrict__ out) {
  const int row = max_len + 3;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_heads * row) return;
  const int h = i / row, e = i % row;
  out[i] = (e < max_len) ? Store<T>::ld(rel_bias + (size_t)h * rel_buckets + bucket_lut[max_len - 1 - e]) : 0.0f;
}

static __global__ void fill_u32_kernel(unsigned int* p, unsigned int v, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace sd
