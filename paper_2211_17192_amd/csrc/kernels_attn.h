// Multi-query decode attention for the (gamma+1)-row forward.
//
// The R query rows (positions row_pos[0..R)) of every head attend causally to
// the paged KV cache (self-attention; the rows' own keys were appended by the
// QKV projection just before) or to a fixed block of encoder keys
// (cross-attention).  Work is split flash-decoding style:
//   grid = (key chunks of 64, kv heads); a workgroup scores its 64 keys against
//   all rows of its kv head (4 lanes per key, each holding a quarter of the
//   head dimension), forms chunk-local softmax numerators, multiplies by V,
//   and writes an unnormalised partial (m, l, O).  The last workgroup of a kv
//   head to finish merges the partials in chunk order and writes the output.
// Chunks sit at absolute key positions and every reduction order is fixed, so
// a row's result does not depend on R or on the other rows: a row computed
// alone (plain decoding) is bit-identical to the same row among gamma+1.
// KV layout per layer: [page][K|V][kv_head][slot][d_head]; a (kv head, page)
// is a contiguous page_size * d_head block, so key reads are coalesced.
#pragma once
#include "common.h"

namespace sd {

constexpr int ATTN_THREADS = 256;
constexpr int ATTN_CHUNK = 64;

struct AttnArgs {
  const void* q;            // T [R][H*dh]
  void* out;                // T [R][H*dh]
  const void* kv_pool;      // self: this layer's pages
  const void* ck; const void* cv;   // cross: T [kv_len][H*dh] each
  const int* page_table;
  int page_size;
  const int* row_pos;       // [R]; self: causal limit of each row, < 0 = padding row
  int R, H, Hkv;
  int cross;                // 1: cross-attention over kv_len keys, no mask, no bias
  int kv_len;
  float scale;
  const void* rel_bias;     // T [H][rel_buckets] or nullptr
  const int* bucket_lut;    // [max_len] bucket of each causal distance
  int rel_buckets;
  float* part_o;            // [Hkv][nchunks][RG][dh]
  float* part_ml;           // [Hkv][nchunks][RG][2]
  unsigned int* counters;   // [Hkv]
};

template <typename T, int DH>
static __global__ __launch_bounds__(ATTN_THREADS) void attn_kernel(const AttnArgs a) {
  extern __shared__ float lds[];
  __shared__ int s_flag;
  __shared__ int s_pos[MAX_ROWS];
  constexpr int DP = DH / 4;                       // head-dim elements per lane in the score phase
  constexpr int NG = ATTN_THREADS / DH;            // key groups in the PV phase
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, hkv = blockIdx.y, nchunks_max = gridDim.x;
  const int G = a.H / a.Hkv, RG = a.R * G;

  if (tid < MAX_ROWS) s_pos[tid] = (tid < a.R) ? (a.cross ? 0 : a.row_pos[tid]) : -1;
  __syncthreads();
  int kv_len = a.kv_len;
  if (!a.cross) {
    int mx = -1;
    for (int r = 0; r < a.R; ++r) mx = max(mx, s_pos[r]);
    kv_len = mx + 1;
  }
  const int active = (kv_len + ATTN_CHUNK - 1) / ATTN_CHUNK;
  if (chunk >= active) return;                     // whole workgroup leaves together

  float* q_s = lds;                                // [RG][DH]
  float* s_s = q_s + RG * DH;                      // [RG][64]
  float* o_s = s_s + RG * ATTN_CHUNK;              // [NG][RG][DH]
  float* ml_s = o_s + NG * RG * DH;                // [RG][2]

  const T* qg = static_cast<const T*>(a.q);
  for (int i = tid; i < RG * DH; i += ATTN_THREADS) {
    const int rg = i / DH, d = i % DH, r = rg / G, h = hkv * G + rg % G;
    q_s[i] = Store<T>::ld(qg + (size_t)r * a.H * DH + h * DH + d);
  }
  __syncthreads();

  // ---- scores: 4 lanes per key ----
  {
    const int kl = tid >> 2, part = tid & 3;
    const int key = chunk * ATTN_CHUNK + kl;
    const bool key_ok = key < kv_len;
    float kreg[DP];
    if (key_ok) {
      const T* kp;
      if (a.cross) {
        kp = static_cast<const T*>(a.ck) + (size_t)key * a.H * DH + hkv * DH;
      } else {
        const int page = a.page_table[key / a.page_size], slot = key % a.page_size;
        kp = static_cast<const T*>(a.kv_pool) +
             ((((size_t)page * 2 + 0) * a.Hkv + hkv) * a.page_size + slot) * DH;
      }
#pragma unroll
      for (int e = 0; e < DP; e += 8) {
        float v[8];
        load8<T>(kp + part * DP + e, v);
#pragma unroll
        for (int f = 0; f < 8; ++f) kreg[e + f] = v[f];
      }
    } else {
#pragma unroll
      for (int e = 0; e < DP; ++e) kreg[e] = 0.0f;
    }
    for (int rg = 0; rg < RG; ++rg) {
      const float* qr = q_s + rg * DH + part * DP;
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < DP; ++e) dot += qr[e] * kreg[e];
      dot += __shfl_xor(dot, 1, WAVE);
      dot += __shfl_xor(dot, 2, WAVE);
      if (part == 0) {
        const int r = rg / G, pos = s_pos[r];
        float sc = -INFINITY;
        if (key_ok && pos >= 0 && (a.cross || key <= pos)) {
          sc = a.scale * dot;
          if (a.rel_bias != nullptr) {
            const int h = hkv * G + rg % G;
            sc += Store<T>::ld(static_cast<const T*>(a.rel_bias) + h * a.rel_buckets +
                               a.bucket_lut[pos - key]);
          }
        }
        s_s[rg * ATTN_CHUNK + kl] = sc;
      }
    }
  }
  __syncthreads();

  // ---- chunk-local softmax numerators: one wavefront per row, lane = key ----
  for (int rg = wave; rg < RG; rg += ATTN_THREADS / 64) {
    const float sc = s_s[rg * ATTN_CHUNK + lane];
    const float m = wave_max(sc);
    const float p = (m == -INFINITY) ? 0.0f : __expf(sc - m);
    const float l = wave_sum(p);
    s_s[rg * ATTN_CHUNK + lane] = p;
    if (lane == 0) { ml_s[rg * 2] = m; ml_s[rg * 2 + 1] = l; }
  }
  __syncthreads();

  // ---- P * V: thread = (key group, head-dim element) ----
  {
    const int d = tid % DH, g = tid / DH;
    for (int rb = 0; rb < RG; rb += MAX_ROWS) {
      float acc[MAX_ROWS];
#pragma unroll
      for (int i = 0; i < MAX_ROWS; ++i) acc[i] = 0.0f;
      const int nr = min(MAX_ROWS, RG - rb);
      for (int kl = g; kl < ATTN_CHUNK; kl += NG) {
        const int key = chunk * ATTN_CHUNK + kl;
        if (key >= kv_len) break;
        const T* vp;
        if (a.cross) {
          vp = static_cast<const T*>(a.cv) + (size_t)key * a.H * DH + hkv * DH;
        } else {
          const int page = a.page_table[key / a.page_size], slot = key % a.page_size;
          vp = static_cast<const T*>(a.kv_pool) +
               ((((size_t)page * 2 + 1) * a.Hkv + hkv) * a.page_size + slot) * DH;
        }
        const float v = Store<T>::ld(vp + d);
#pragma unroll
        for (int i = 0; i < MAX_ROWS; ++i)
          if (i < nr) acc[i] += s_s[(rb + i) * ATTN_CHUNK + kl] * v;
      }
#pragma unroll
      for (int i = 0; i < MAX_ROWS; ++i)
        if (i < nr) o_s[(g * RG + rb + i) * DH + d] = acc[i];
    }
  }
  __syncthreads();
  float* po = a.part_o + ((size_t)hkv * nchunks_max + chunk) * RG * DH;
  float* pml = a.part_ml + ((size_t)hkv * nchunks_max + chunk) * RG * 2;
  for (int i = tid; i < RG * DH; i += ATTN_THREADS) {
    float s = 0.0f;
#pragma unroll
    for (int g = 0; g < NG; ++g) s += o_s[g * RG * DH + i];
    po[i] = s;
  }
  for (int i = tid; i < RG * 2; i += ATTN_THREADS) pml[i] = ml_s[i];

  if (!last_block_arrives(a.counters + hkv, (unsigned)active, &s_flag)) return;

  // ---- merge the chunk partials of this kv head, in chunk order ----
  T* og = static_cast<T*>(a.out);
  const float* bo = a.part_o + (size_t)hkv * nchunks_max * RG * DH;
  const float* bml = a.part_ml + (size_t)hkv * nchunks_max * RG * 2;
  for (int i = tid; i < RG * DH; i += ATTN_THREADS) {
    const int rg = i / DH, d = i % DH, r = rg / G, h = hkv * G + rg % G;
    float M = -INFINITY;
    for (int c = 0; c < active; ++c) M = fmaxf(M, bml[((size_t)c * RG + rg) * 2]);
    float L = 0.0f, O = 0.0f;
    if (M != -INFINITY) {
      for (int c = 0; c < active; ++c) {
        const float mc = bml[((size_t)c * RG + rg) * 2];
        if (mc == -INFINITY) continue;
        const float w = __expf(mc - M);
        L += w * bml[((size_t)c * RG + rg) * 2 + 1];
        O += w * bo[(size_t)c * RG * DH + i];
      }
    }
    Store<T>::st(og + (size_t)r * a.H * DH + h * DH + d, (L > 0.0f) ? O / L : 0.0f);
  }
}

}  // namespace sd
