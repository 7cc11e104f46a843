// Multi-query decode attention for the (gamma+1)-row forward.
//
// The R query rows (positions row_pos[0..R)) of every head attend causally to
// the paged KV cache (self-attention; the rows' own keys were appended by the
// QKV projection just before) or to a fixed block of encoder keys
// (cross-attention).
//
// One workgroup of 1024 threads owns one kv head and walks its keys in blocks
// of 512 with an online softmax (running max m, denominator l, unnormalised
// output O per row).  There is no split over workgroups and therefore no
// cross-workgroup merge: device-scope atomics cost about a quarter of a
// microsecond each on this chip when they queue on one address, which is more
// than the whole kernel should take.  Per block of keys:
//   scores  2 lanes per key, each holding half of the head dimension of its key
//           in registers and dotting it with every query row (rows in LDS);
//   softmax one wavefront per row over the 512 scores;
//   P*V     thread = (key group, head-dim element); coalesced V rows; the 16
//           (8 for d_head 128) key groups are added in fixed order through LDS.
// Key blocks sit at absolute positions and all reduction orders are fixed, so
// a row's result does not depend on R or on the other rows: a row computed
// alone (plain decoding) is bit-identical to the same row among gamma+1.
// KV layout per layer: [page][K|V][kv_head][slot][d_head]; a (kv head, page)
// is a contiguous page_size * d_head block, so key reads are coalesced.
#pragma once
#include "common.h"

namespace sd {

constexpr int ATTN_THREADS = 1024;
constexpr int ATTN_BLOCK = 512;            // keys per pass
constexpr int ATTN_MAX_RG = 24;            // query rows x heads per kv head that fit in LDS

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
};

// dynamic LDS (floats): q [RG][DH] | s [RG][512] | o [NG][16][DH] | m, l, f [3][RG] | acc [RG][DH]
template <typename T, int DH>
static __global__ __launch_bounds__(ATTN_THREADS) void attn_kernel(const AttnArgs a) {
  extern __shared__ float lds[];
  __shared__ int s_pos[MAX_ROWS];
  constexpr int DP = DH / 2;                       // head-dim elements per lane in the score phase
  constexpr int NG = ATTN_THREADS / DH;            // key groups in the P*V phase
  constexpr int NW = ATTN_THREADS / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hkv = blockIdx.x;
  const int G = a.H / a.Hkv, RG = a.R * G;

  if (tid < MAX_ROWS) s_pos[tid] = (tid < a.R) ? (a.cross ? 0 : a.row_pos[tid]) : -1;
  float* q_s = lds;                                // [RG][DH]
  float* s_s = q_s + RG * DH;                      // [RG][512]
  float* o_s = s_s + RG * ATTN_BLOCK;              // [NG][16][DH]
  float* m_s = o_s + NG * MAX_ROWS * DH;           // [RG] running max
  float* l_s = m_s + RG;                           // [RG] running denominator
  float* f_s = l_s + RG;                           // [RG] rescale factor of this pass
  float* acc_s = f_s + RG;                         // [RG][DH] running output

  const T* qg = static_cast<const T*>(a.q);
  for (int i = tid; i < RG * DH; i += ATTN_THREADS) {
    const int rg = i / DH, d = i % DH, r = rg / G, h = hkv * G + rg % G;
    q_s[i] = Store<T>::ld(qg + (size_t)r * a.H * DH + h * DH + d);
    acc_s[i] = 0.0f;
  }
  if (tid < RG) { m_s[tid] = -INFINITY; l_s[tid] = 0.0f; }
  __syncthreads();
  int kv_len = a.kv_len;
  if (!a.cross) {
    int mx = -1;
    for (int r = 0; r < a.R; ++r) mx = max(mx, s_pos[r]);
    kv_len = mx + 1;
  }

  for (int k0 = 0; k0 < kv_len; k0 += ATTN_BLOCK) {
    // ---- scores: 2 lanes per key ----
    {
      const int kl = tid >> 1, part = tid & 1;
      const int key = k0 + kl;
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
          s_s[rg * ATTN_BLOCK + kl] = sc;
        }
      }
    }
    __syncthreads();

    // ---- online softmax: one wavefront per row, 8 scores per lane ----
    for (int rg = wave; rg < RG; rg += NW) {
      float sc[ATTN_BLOCK / 64];
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < ATTN_BLOCK / 64; ++i) { sc[i] = s_s[rg * ATTN_BLOCK + i * 64 + lane]; mx = fmaxf(mx, sc[i]); }
      mx = wave_max(mx);
      const float m_old = m_s[rg];
      const float m_new = fmaxf(m_old, mx);
      float sum = 0.0f;
#pragma unroll
      for (int i = 0; i < ATTN_BLOCK / 64; ++i) {
        const float p = (sc[i] == -INFINITY) ? 0.0f : __expf(sc[i] - m_new);
        s_s[rg * ATTN_BLOCK + i * 64 + lane] = p;
        sum += p;
      }
      sum = wave_sum(sum);
      if (lane == 0) {
        const float f = (m_old == -INFINITY) ? 0.0f : __expf(m_old - m_new);
        f_s[rg] = f;
        l_s[rg] = l_s[rg] * f + sum;
        m_s[rg] = m_new;
      }
    }
    __syncthreads();

    // ---- P * V: thread = (key group, head-dim element), 16 rows at a time ----
    {
      const int d = tid % DH, g = tid / DH;
      const int nkeys = min(ATTN_BLOCK, kv_len - k0);
      for (int rb = 0; rb < RG; rb += MAX_ROWS) {
        float acc[MAX_ROWS];
#pragma unroll
        for (int i = 0; i < MAX_ROWS; ++i) acc[i] = 0.0f;
        const int nr = min(MAX_ROWS, RG - rb);
        for (int kl = g; kl < nkeys; kl += NG) {
          const int key = k0 + kl;
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
            if (i < nr) acc[i] += s_s[(rb + i) * ATTN_BLOCK + kl] * v;
        }
#pragma unroll
        for (int i = 0; i < MAX_ROWS; ++i)
          if (i < nr) o_s[(g * MAX_ROWS + i) * DH + d] = acc[i];
        __syncthreads();
        for (int i = tid; i < nr * DH; i += ATTN_THREADS) {      // key groups in fixed order
          float t = 0.0f;
#pragma unroll
          for (int gg = 0; gg < NG; ++gg) t += o_s[gg * MAX_ROWS * DH + i];
          const int idx = rb * DH + i;
          acc_s[idx] = acc_s[idx] * f_s[idx / DH] + t;
        }
        __syncthreads();
      }
    }
  }

  T* og = static_cast<T*>(a.out);
  for (int i = tid; i < RG * DH; i += ATTN_THREADS) {
    const int rg = i / DH, d = i % DH, r = rg / G, h = hkv * G + rg % G;
    const float L = l_s[rg];
    Store<T>::st(og + (size_t)r * a.H * DH + h * DH + d, (L > 0.0f) ? acc_s[i] / L : 0.0f);
  }
}

}  // namespace sd
