// Skinny GEMM for the (gamma+1)-row forward: Y[R,N] = X[R,K] * W[N,K]^T with
// R <= 16 rows.  The path is HBM-bound on the weights (about R flop per byte),
// so the kernel is organised around streaming W exactly once:
//
//  * W is re-tiled at load time into MFMA operand order
//      Wt[N/16][K/32][64 lanes][8 elements],
//    lane l of a tile holding W[n0 + l%16][k0 + (l/16)*8 .. +8], so a wavefront
//    fetches one contiguous 1 KB (bf16) block per MFMA with 16-byte loads and
//    its whole K-slice is one contiguous stream.
//  * The weights sit on the MFMA "A" side (16 output features), the R
//    activation rows on the 16-wide "B" side; fp32 accumulation.
//  * A workgroup works through 16-feature tiles (tile = block, block + grid,
//    ...) with a two-stage software pipeline: the loads of the next chunk, or of
//    the next tile's first chunk, are in flight while the current one is
//    multiplied, reduced and written out.  Its S wavefronts split K and the
//    partial tiles are added through LDS in wave order 0..S-1.  S depends on
//    (N, K) only, never on R, so a row's result is bit-identical whether it is
//    computed alone or among gamma+1 rows.
//  * Vector-memory loads complete in issue order as far as the wait counter can
//    tell, so the kernel keeps them branch-free and issues whatever the epilogue
//    reads (residual, bias, gain, rotary table) BEFORE the prefetch of the next
//    chunk; otherwise every epilogue would drain the prefetch.
//  * RMSNorm is folded around the GEMM: the producer of the residual stream
//    (embedding or a residual-add epilogue) also writes xg = x * gain of the
//    next norm in the storage type and, per 16-feature tile, the partial sums
//    of x^2; the consumer multiplies plain xg rows and scales its output rows
//    by 1/rms, which it gets by adding the partials in tile order.  No pass
//    over x, no barrier before the weight stream starts.
//  * LayerNorm (mean subtraction) is applied as a prologue on the fp32 rows.
//  * Epilogues: bias, tanh-GELU, gated GELU / SwiGLU (two weight streams, one
//    activation stream), residual add, rotary + scatter of q / k / v (k and v
//    go straight into the paged KV cache), logit scaling.
#pragma once
#include "common.h"

namespace sd {

enum { PRO_NONE = 0, PRO_POST = 1, PRO_LN = 2 };
enum { EPI_STORE = 0, EPI_QKV = 1, EPI_RESID = 2, EPI_ACT = 3, EPI_GATED = 4, EPI_LOGITS = 5 };
enum { ACT_GELU = 0, ACT_SILU = 1 };

struct GemmArgs {
  const void* W;          // tiled weights, N/16 tiles
  const void* W2;         // EPI_GATED: the "up" weights, tiled alike
  const void* X;          // PRO_NONE / PRO_POST: T [R][K]; PRO_LN: float [R][K]
  const void* gain;       // T [K]   (PRO_LN)
  const void* beta;       // T [K]   (PRO_LN)
  const void* bias;       // T [N] or nullptr
  const float* ss_in;     // PRO_POST: [n_part][16] partial sums of x^2 of the input rows
  int n_part;
  int R, K, N;
  int ksteps_per_wave;    // ceil((K/32) / waves)
  float eps;
  void* out;              // STORE/ACT/GATED: T [R][ldo]; RESID, LOGITS: float [R][ldo]
  int ldo;
  float scale;            // EPI_LOGITS
  int act;                // EPI_GATED
  int hm_rows, hm_row0;   // EPI_STORE: > 0 selects the head-major layout (uses d_head)
  // EPI_RESID extras for a following RMSNorm (all optional)
  void* xg_out;           // T [R][ldo]: (x + y) * gain_next
  const void* gain_next;  // T [N]
  float* ss_out;          // [N/16][16] partial sums of (x + y)^2 per tile and row
  // EPI_QKV
  void* q_out;            // T [R][nq]
  int nq, nkv;            // features [0,nq) q, [nq,nq+nkv) k, [nq+nkv,nq+2nkv) v
  void* kv_pool;          // this layer's pages: [page][2][n_kv_heads][page_size][d_head]
  const int* page_table;
  int page_size, n_kv_heads, d_head;
  const int* row_pos;     // [R] position of each row; < 0: row is padding
  // several sequences in one launch (all optional)
  const int* row_seq;     // EPI_QKV: [R] sequence of each row; its page table starts at page_table + seq * pt_stride
  int pt_stride;
  const int* out_row;     // EPI_LOGITS: [R] row of `out` each input row goes to, < 0: dropped
  // gemm_wide_kernel: nrt slabs of 16 rows, one after the other in every row-indexed
  // buffer; slabs hold R rows each, the last one R_last; the partial-sum blocks of two
  // slabs lie ss_stride floats apart
  int nrt, R_last, ss_stride;
  const float* rope;      // [max_len][d_head/2][2] (cos, sin) or nullptr
  // gemm_split_kernel / gemm_split_finish_kernel: the K chunks' partial tiles,
  // [nchunk][nrt][streams * N/16][64 lanes][4] floats, and the number of chunks
  float* partial;
  int nchunk;
  const float* rs_in;     // PRO_POST: 1 / rms of every row, [nrt * 16] (rows_to_fragments_kernel writes it)
  // gemm_gated_wide_kernel: when set, the output goes here in fragment order
  // ([N/32][GEMM_WIDE_RT][64 lanes][8], what the FFN-out product reads) instead of row-major into `out`
  void* out_frag;
};

template <typename T> struct Mma;
template <> struct Mma<bf16> {
  typedef bf16x8 Frag;
  static __device__ __forceinline__ Frag load(const bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
  static __device__ __forceinline__ Frag load_stream(const bf16* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p));
  }
  static __device__ __forceinline__ Frag from_floats(const float (&v)[8]) {
    Frag f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (bf16)v[e];
    return f;
  }
  static __device__ __forceinline__ Frag select(bool keep, const Frag& f) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 bits = __builtin_bit_cast(u32x4, f);
    const unsigned m = keep ? 0xFFFFFFFFu : 0u;
    return __builtin_bit_cast(Frag, bits & m);
  }
  static __device__ __forceinline__ f32x4 mma(const Frag& a, const Frag& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mma<float> {
  struct Frag { float v[8]; };
  static __device__ __forceinline__ Frag load(const float* p) { Frag f; load8<float>(p, f.v); return f; }
  static __device__ __forceinline__ Frag load_stream(const float* p) { return load(p); }
  static __device__ __forceinline__ Frag from_floats(const float (&v)[8]) {
    Frag f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = v[e];
    return f;
  }
  static __device__ __forceinline__ Frag select(bool keep, const Frag& f) {
    Frag r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r.v[e] = keep ? f.v[e] : 0.0f;
    return r;
  }
  // eight 16x16x4 steps; step e contracts the k indices {kq*8 + e}, the same
  // set on both operands
  static __device__ __forceinline__ f32x4 mma(const Frag& a, const Frag& b, f32x4 c) {
#pragma unroll
    for (int e = 0; e < 8; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[e], b.v[e], c, 0, 0, 0);
    return c;
  }
};

// The 8 elements of a fragment as floats (what load8 gives for the same 8 elements).
template <typename T> __device__ __forceinline__ void frag_to_floats(const typename Mma<T>::Frag& f, float (&o)[8]);
template <> __device__ __forceinline__ void frag_to_floats<bf16>(const bf16x8& f, float (&o)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (float)f[e];
}
template <> __device__ __forceinline__ void frag_to_floats<float>(const Mma<float>::Frag& f, float (&o)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f.v[e];
}

// The same row must come out bit-identical from every kernel that can compute it (one slab or
// several), so the arithmetic of the epilogues and of the LayerNorm prologue is written once and
// with floating-point contraction off: left to itself the compiler fuses a multiply and an add
// into an FMA in one kernel and not in another, and the last bit of a rotated key then differs.
__device__ __forceinline__ float gelu_tanh(float x) {
#pragma clang fp contract(off)
  return 0.5f * x * (1.0f + tanhf(0.7978845608028654f * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float silu(float x) {
#pragma clang fp contract(off)
  return x / (1.0f + expf(-x));
}
// rotary embedding of one element: y with its pair partner `other`, (cos, sin) of the position
__device__ __forceinline__ float rope_rotate(float y, float other, float c, float sn, bool odd) {
#pragma clang fp contract(off)
  const float yc = y * c, os = other * sn;
  return odd ? (os + yc) : (yc - os);
}
// a square that stays a product: the sums of squares behind the norms must not depend on whether
// the compiler fuses the square into the addition that follows it
__device__ __forceinline__ float square(float x) {
#pragma clang fp contract(off)
  const float q = x * x;
  return q;
}
// variance accumulation of the LayerNorm prologue
__device__ __forceinline__ float add_square(float acc, float x) {
#pragma clang fp contract(off)
  const float q = x * x;
  return acc + q;
}
// LayerNorm of one element
__device__ __forceinline__ float ln_apply(float v, float mu, float rstd, float g, float b) {
#pragma clang fp contract(off)
  const float n = (v - mu) * rstd;
  const float ng = n * g;
  return ng + b;
}

// k-steps per chunk of the software pipeline (a chunk's loads go out together, unconditionally:
// k-steps beyond a wavefront's slice re-read its last one).  8 for long K-slices; a wavefront
// whose whole slice is 4 k-steps or fewer (d_model 512 over 4 wavefronts) takes chunks of 4, so
// that half of its loads are not duplicates: 7 % off the small draft model's forward.
constexpr int GEMM_UNROLL = 8;
constexpr int GEMM_UNROLL_SHORT = 4;
constexpr int GEMM_PART_REGS = 16;          // partial sums of x^2 an epilogue thread adds from LDS: 16 x 16 tiles
constexpr int GEMM_PART_STAGE = 16 * GEMM_PART_REGS;   // tiles whose partial sums are staged in LDS (d_model <= 4096)

// Launched with 4 or 8 wavefronts; threads 0..255 (t = row * 16 + feature) run the epilogue.
// U: k-steps per chunk (GEMM_UNROLL or GEMM_UNROLL_SHORT; it changes what is in flight, never the
// order of a row's additions).
template <typename T, int PRO, int EPI, int U = GEMM_UNROLL>
static __global__ __launch_bounds__(512) void gemm_kernel(const GemmArgs a) {
  extern __shared__ float lds[];
  constexpr int ND = (EPI == EPI_GATED) ? 2 : 1;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, S = blockDim.x >> 6;
  const int j = lane & 15, kq = lane >> 4;           // B side: row j, k-quarter kq
  const int KS = a.K >> 5;
  const int ks0 = min(KS, wave * a.ksteps_per_wave), ks1 = min(KS, ks0 + a.ksteps_per_wave);
  const int nchunks = (a.ksteps_per_wave + U - 1) / U;          // same for every wave
  const int ntiles = a.N >> 4;
  const int my_tiles = (ntiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  float* part = lds;                                 // [2][S][ND][256], double-buffered per tile
  float* stat = lds + 2 * S * ND * 256;              // [S][16]
  float* ybuf = stat + S * 16;                       // [256]
  const bool row_ok = (j < a.R);
  const bool epi_thread = tid < 256;
  const int e_row = (tid >> 4) & 15, e_f = tid & 15;  // epilogue role of this thread
  const int e_rowc = min(e_row, a.R - 1);             // clamped: loads stay in bounds

  float mu = 0.0f, rstd = 1.0f;

  typedef typename Mma<T>::Frag Frag;
  struct Buf { Frag fa[ND][U]; Frag fb[U]; };

  // All loads are unconditional: a branch around a load makes the compiler wait
  // for every outstanding load before the next multiply, which would undo the
  // pipelining.  Out-of-range rows / k-steps re-read a valid address and are
  // replaced by zeros with a select when they are used.
  const int jr = min(j, a.R - 1);
  auto make_b = [&](int ks, bool valid) -> Frag {
    const int k = ks * 32 + kq * 8;
    if (PRO != PRO_LN) {
      return Mma<T>::load(static_cast<const T*>(a.X) + (size_t)jr * a.K + k);
    } else {
      float v[8], g[8], bb[8];
      load8<float>(static_cast<const float*>(a.X) + (size_t)jr * a.K + k, v);
      load8<T>(static_cast<const T*>(a.gain) + k, g);
      load8<T>(static_cast<const T*>(a.beta) + k, bb);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = ln_apply(v[e], mu, rstd, g[e], bb[e]);
      return Mma<T>::select(valid && row_ok, Mma<T>::from_floats(v));
    }
  };

  // chunk g of this workgroup's work list: tile blockIdx.x + (g / nchunks) * gridDim.x,
  // k-steps ks0 + (g % nchunks) * U ... of this wave's K-slice
  const int ks_last = max(ks1 - 1, 0);
  // (WHAT: 1 = the weights, 2 = the activations, 3 = both, interleaved per k-step)
  auto load_chunk_part = [&](Buf& b, int g, auto what) {
    constexpr int WHAT = decltype(what)::value;
    const int ti = g / nchunks, c = g - ti * nchunks;
    const size_t tile = (size_t)blockIdx.x + (size_t)ti * gridDim.x;
    const T* w0 = static_cast<const T*>(a.W) + (tile * KS) * 512 + lane * 8;
    const T* w1 = (ND == 2) ? static_cast<const T*>(a.W2) + (tile * KS) * 512 + lane * 8 : nullptr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ks = ks0 + c * U + u;
      const int ksc = min(ks, ks_last);
      if (WHAT & 1) {
        b.fa[0][u] = Mma<T>::load_stream(w0 + (size_t)ksc * 512);
        if (ND == 2) b.fa[ND - 1][u] = Mma<T>::load_stream(w1 + (size_t)ksc * 512);
      }
      if (WHAT & 2) b.fb[u] = make_b(ksc, ks < ks1);
    }
  };
  auto load_chunk = [&](Buf& b, int g) { load_chunk_part(b, g, std::integral_constant<int, 3>()); };

  const int G = my_tiles * nchunks;
  Buf b0, b1;
  // ---- PRO_POST: 1 / rms of every row, once per workgroup.  The producer left one partial sum
  // of x^2 per 16-feature tile and row ([n_part][16] floats, written by n_part different
  // workgroups).  Thread t of the four epilogue wavefronts fetches block t with four 16-byte
  // loads that go straight into LDS (no registers; the whole array crosses the memory system once
  // per workgroup, 1 KB per wavefront and load); epilogue thread (row, f) then adds the partials
  // f, f + 16, ... in ascending order and the 16 lanes of the row: the order the batched kernels
  // use too.  (Letting every epilogue thread load its 16 partials itself, 64 bytes apart, made 256
  // workgroups send a thousand requests each to the same 256 cache lines: 1.3 us per launch.)
  // The loads go out ahead of the weights, so that the in-order return of loads does not hold the
  // weight stream back, and are read under the barrier the first tile's end needs anyway.
  // LDS layout: load i of wavefront w fills ssb[(4 i + w) * 256 ..] with one 16-byte piece per
  // lane: partial (p, row) sits at (((row / 4) * 4 + p / 64) * 64 + p % 64) * 4 + row % 4.
  float rs_row = 1.0f;
  float* ssb = ybuf + 256;                       // GEMM_PART_STAGE * 16 floats
  if (PRO == PRO_POST && epi_thread) {
    const float* blk = a.ss_in + (size_t)min(tid, a.n_part - 1) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(blk + 4 * i),
                                       (__attribute__((address_space(3))) void*)(ssb + (4 * i + wave) * 256), 16, 0, 0);
  }
  // A LayerNorm model's rows cannot be normalised before their statistics are known, but the first
  // chunk's weights depend on nothing: they are asked for first and arrive while the statistics
  // (two passes over the rows, two barriers) are computed.
  if (PRO == PRO_LN) {
    if (G > 0) load_chunk_part(b0, 0, std::integral_constant<int, 1>());
    // ---- statistics of the fp32 rows, reduced across the workgroup ----
    if (sizeof(T) == 2 && nchunks == 1) {            // (fp32 fragments are twice the registers: general path)
      // A wavefront's whole K-slice is one chunk (small d_model): the rows' elements, gains and
      // offsets are fetched ONCE, with the weights, and both passes of the statistics and the
      // normalised fragments come out of registers -- the same additions in the same order as
      // the general path below, without its two further trips to memory.
      const float* x = static_cast<const float*>(a.X) + (size_t)jr * a.K + kq * 8;
      float xv[U][8];
      typename Mma<T>::Frag gv[U], bv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = min(ks0 + u, ks_last) * 32;
        load8<float>(x + k, xv[u]);
        gv[u] = Mma<T>::load(static_cast<const T*>(a.gain) + k + kq * 8);
        bv[u] = Mma<T>::load(static_cast<const T*>(a.beta) + k + kq * 8);
      }
      float s = 0.0f;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ks0 + u < ks1) {
#pragma unroll
          for (int e = 0; e < 8; ++e) s += xv[u][e];
        }
      s = lane_combine<16>(s, OpSumF()); s = lane_combine<32>(s, OpSumF());
      if (kq == 0) stat[wave * 16 + j] = s;
      __syncthreads();
      float t = 0.0f;
      for (int w = 0; w < S; ++w) t += stat[w * 16 + j];
      mu = t / (float)a.K;
      __syncthreads();
      float s2 = 0.0f;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ks0 + u < ks1) {
#pragma unroll
          for (int e = 0; e < 8; ++e) s2 = add_square(s2, xv[u][e] - mu);
        }
      s2 = lane_combine<16>(s2, OpSumF()); s2 = lane_combine<32>(s2, OpSumF());
      if (kq == 0) stat[wave * 16 + j] = s2;
      __syncthreads();
      float t2 = 0.0f;
      for (int w = 0; w < S; ++w) t2 += stat[w * 16 + j];
      rstd = 1.0f / sqrtf(t2 / (float)a.K + a.eps);
      if (G > 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float v[8], g[8], bb[8];
          frag_to_floats<T>(gv[u], g); frag_to_floats<T>(bv[u], bb);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = ln_apply(xv[u][e], mu, rstd, g[e], bb[e]);
          b0.fb[u] = Mma<T>::select((ks0 + u < ks1) && row_ok, Mma<T>::from_floats(v));
        }
      }
    } else {
      const float* x = static_cast<const float*>(a.X) + (size_t)min(j, a.R - 1) * a.K + kq * 8;
      float s = 0.0f;
#pragma unroll 4
      for (int ks = ks0; ks < ks1; ++ks) {
        float v[8]; load8<float>(x + ks * 32, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) s += v[e];
      }
      s = lane_combine<16>(s, OpSumF()); s = lane_combine<32>(s, OpSumF());
      if (kq == 0) stat[wave * 16 + j] = s;
      __syncthreads();
      float t = 0.0f;
      for (int w = 0; w < S; ++w) t += stat[w * 16 + j];
      mu = t / (float)a.K;
      __syncthreads();
      float s2 = 0.0f;
#pragma unroll 4
      for (int ks = ks0; ks < ks1; ++ks) {
        float v[8]; load8<float>(x + ks * 32, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) s2 = add_square(s2, v[e] - mu);
      }
      s2 = lane_combine<16>(s2, OpSumF()); s2 = lane_combine<32>(s2, OpSumF());
      if (kq == 0) stat[wave * 16 + j] = s2;
      __syncthreads();
      float t2 = 0.0f;
      for (int w = 0; w < S; ++w) t2 += stat[w * 16 + j];
      rstd = 1.0f / sqrtf(t2 / (float)a.K + a.eps);
      if (G > 0) load_chunk_part(b0, 0, std::integral_constant<int, 2>());
    }
  } else if (G > 0) {
    load_chunk(b0, 0);
  }
  int e_pos = -1;
  size_t e_kvbase = 0;                            // EPI_QKV: cache offset of this row's page / slot
  if (EPI == EPI_QKV && epi_thread) {
    e_pos = (e_row < a.R) ? a.row_pos[e_rowc] : -1;
    const int pc = max(e_pos, 0);
    const int pt0 = (a.row_seq != nullptr) ? a.row_seq[e_rowc] * a.pt_stride : 0;
    const int page = a.page_table[pt0 + pc / a.page_size], slot = pc % a.page_size;
    e_kvbase = (size_t)page * 2 * a.n_kv_heads * a.page_size * a.d_head + (size_t)slot * a.d_head;
  }

  // ---- per-tile epilogue inputs, issued before the prefetch of the next chunk ----
  float pre_res = 0.0f, pre_bias = 0.0f, pre_gain = 0.0f, pre_cos = 1.0f, pre_sin = 0.0f;
  auto prefetch_epilogue = [&](int ti) {
    if (!epi_thread) return;
    const int n = ((int)blockIdx.x + ti * (int)gridDim.x) * 16 + e_f;
    if (a.bias != nullptr) pre_bias = Store<T>::ld(static_cast<const T*>(a.bias) + n);
    if (EPI == EPI_RESID) {
      pre_res = static_cast<const float*>(a.out)[(size_t)e_rowc * a.ldo + n];
      if (a.xg_out != nullptr) pre_gain = Store<T>::ld(static_cast<const T*>(a.gain_next) + n);
    }
    if (EPI == EPI_QKV && a.rope != nullptr) {
      const int nn = (n < a.nq) ? n : (n < a.nq + a.nkv ? n - a.nq : n - a.nq - a.nkv);
      const float* cs = a.rope + ((size_t)max(e_pos, 0) * (a.d_head >> 1) + ((nn % a.d_head) >> 1)) * 2;
      pre_cos = cs[0]; pre_sin = cs[1];
    }
  };

  f32x4 acc[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d) acc[d] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Adds the K-slices of a finished tile in wave order and applies the epilogue.
  auto finish_tile = [&](int ti) {
    const int tile = (int)blockIdx.x + ti * (int)gridDim.x;
    float* pt = part + (ti & 1) * S * ND * 256;
    // accumulator layout: lane holds features (lane/16)*4 + r, r = 0..3, of row lane%16
#pragma unroll
    for (int d = 0; d < ND; ++d) {
#pragma unroll
      for (int r = 0; r < 4; ++r) pt[(wave * ND + d) * 256 + j * 16 + kq * 4 + r] = acc[d][r];
      acc[d] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();
    if (epi_thread) {
      const int t = tid, row = e_row, f = e_f, n = tile * 16 + f;
      if (PRO == PRO_POST && ti == 0) {
        float q = 0.0f;
#pragma unroll
        for (int u = 0; u < GEMM_PART_REGS; ++u) {
          const int p = e_f + 16 * u;
          const int pc = min(p, a.n_part - 1);
          const float v = ssb[((((e_row >> 2) << 2) + (pc >> 6)) * 64 + (pc & 63)) * 4 + (e_row & 3)];
          q += (p < a.n_part) ? v : 0.0f;
        }
        for (int p = e_f + 16 * GEMM_PART_REGS; p < a.n_part; p += 16) q += a.ss_in[p * 16 + e_rowc];
        q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
        q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
        q = row_first(q);                          // the total the batched kernels use: the first lane's
        rs_row = 1.0f / sqrtf(q / (float)a.K + a.eps);
      }
      float y[ND];
#pragma unroll
      for (int d = 0; d < ND; ++d) {
        float s = 0.0f;
        for (int w = 0; w < S; ++w) s += pt[(w * ND + d) * 256 + t];
        y[d] = s;
      }
      if (PRO == PRO_POST) {
#pragma unroll
        for (int d = 0; d < ND; ++d) y[d] *= rs_row;
      }
      y[0] += pre_bias;
      if (EPI == EPI_QKV) {
        ybuf[t] = y[0];
      } else if (EPI == EPI_RESID) {
        float xn = 0.0f;
        if (row < a.R) {
          xn = pre_res + y[0];
          static_cast<float*>(a.out)[(size_t)row * a.ldo + n] = xn;
          if (a.xg_out != nullptr) Store<T>::st(static_cast<T*>(a.xg_out) + (size_t)row * a.ldo + n, xn * pre_gain);
        }
        if (a.ss_out != nullptr) {
          float q = square(xn);
          q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
          q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
          if (f == 0) a.ss_out[tile * 16 + row] = q;
        }
      } else if (row < a.R) {
        if (EPI == EPI_STORE) {
          if (a.hm_rows > 0)       // head-major: [head][hm_rows][d_head], this launch's rows start at hm_row0
            Store<T>::st(static_cast<T*>(a.out) +
                             ((size_t)(n / a.d_head) * a.hm_rows + a.hm_row0 + row) * a.d_head + n % a.d_head, y[0]);
          else
            Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, y[0]);
        } else if (EPI == EPI_ACT) {
          Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, gelu_tanh(y[0]));
        } else if (EPI == EPI_GATED) {
          const float g = (a.act == ACT_GELU) ? gelu_tanh(y[0]) : silu(y[0]);
          Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, g * y[ND - 1]);
        } else if (EPI == EPI_LOGITS) {
          const int orow = (a.out_row != nullptr) ? a.out_row[row] : row;
          if (orow >= 0) static_cast<float*>(a.out)[(size_t)orow * a.ldo + n] = a.scale * y[0];
        }
      }
    }
    if (EPI == EPI_QKV) {
      __syncthreads();
      if (epi_thread && e_row < a.R) {
        const int t = tid, n = tile * 16 + e_f;
        float y = ybuf[t];
        const bool is_q = n < a.nq, is_k = !is_q && n < a.nq + a.nkv;
        const int nn = is_q ? n : (is_k ? n - a.nq : n - a.nq - a.nkv);
        const int head = nn / a.d_head, d = nn % a.d_head;
        if (a.rope != nullptr && (is_q || is_k) && e_pos >= 0) {
          const float other = ybuf[t ^ 1];
          y = rope_rotate(y, other, pre_cos, pre_sin, (d & 1) != 0);
        }
        if (is_q) {
          Store<T>::st(static_cast<T*>(a.q_out) + (size_t)e_row * a.nq + n, y);
        } else if (e_pos >= 0) {
          const size_t idx = e_kvbase + ((size_t)(is_k ? 0 : 1) * a.n_kv_heads + head) * a.page_size * a.d_head + d;
          Store<T>::st(static_cast<T*>(a.kv_pool) + idx, y);
        }
      }
    }
  };

  auto compute_chunk = [&](const Buf& b, int g) {
    const int ti = g / nchunks, c = g - ti * nchunks;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool valid = (ks0 + c * U + u < ks1) && row_ok;
      const Frag fb = (PRO == PRO_LN) ? b.fb[u] : Mma<T>::select(valid, b.fb[u]);
      acc[0] = Mma<T>::mma(b.fa[0][u], fb, acc[0]);
      if (ND == 2) acc[ND - 1] = Mma<T>::mma(b.fa[ND - 1][u], fb, acc[ND - 1]);
    }
    if (c == nchunks - 1) finish_tile(ti);
  };
  // chunk g closes its tile: fetch what that tile's epilogue reads, before the
  // loads of chunk g + 1 go out
  auto before_prefetch = [&](int g) {
    const int ti = g / nchunks;
    if (g - ti * nchunks == nchunks - 1) prefetch_epilogue(ti);
  };

  // ---- software pipeline over the work list: the loads of chunk g+1 (possibly
  // the first chunk of the next tile) are in flight while chunk g is multiplied
  // and while a finished tile is reduced and written out ----
  for (int g = 0; g < G; g += 2) {
    before_prefetch(g);
    if (g + 1 < G) load_chunk(b1, g + 1);
    compute_chunk(b0, g);
    if (g + 1 < G) {
      before_prefetch(g + 1);
      if (g + 2 < G) load_chunk(b0, g + 2);
      compute_chunk(b1, g + 1);
    }
  }
}

// ---------------------------------------------------------------------------
// The same product for up to GEMM_WIDE_RT slabs of 16 rows in one launch (several
// sequences decoded together give more than 16 rows).  Same K split over wavefronts
// and same order of additions per row as gemm_kernel: a row's result does not depend on
// the kernel it went through.
//
// What bounds this kernel is not HBM but the traffic of activation fragments from L2:
// every KB of weights needs a KB of activations per slab.  Two measures (a
// micro-benchmark of the bare loop gave 1.4 TB/s of weights with six row-major fragments
// per weight KB, 2.7 with the fragments contiguous, 3.9 with three contiguous ones):
//  * the activations come in fragment order, Xf[K/32][GEMM_WIDE_RT][64 lanes][8]
//    (rows_to_fragments_kernel writes it just before the launch), so a fragment is one
//    contiguous KB instead of 16 rows x 64 B;
//  * every fragment is used for two weight streams: the gate and up matrices of a gated
//    FFN, else two neighbouring 16-feature tiles.
// PRO_LN (LayerNorm prologue) still reads the fp32 rows directly.
// Main loop: a ring of k-step slots refilled right after use; no branches around loads.
// ---------------------------------------------------------------------------
constexpr int GEMM_WIDE_U = 2;

// LDS of the wide kernel: the partial tiles of every wavefront, stream and slab, the QKV
// staging rows, and per-row constants.
__host__ __device__ constexpr size_t gemm_wide_lds_bytes(int S) {
  return (size_t)(S * 2 * GEMM_WIDE_RT * 256 + 2 * GEMM_WIDE_RT * 256 + S * 16 + GEMM_WIDE_RT * 16 * 4) * sizeof(float);
}

// Row-major activations [nrt * 16][K] -> fragment order [K/32][GEMM_WIDE_RT][64][8].
// One thread moves the 8 elements of one lane of one fragment.  With rs_out, the workgroups
// nrt .. 2 nrt - 1 of the grid also leave 1 / rms of every row of slab (block - nrt) there, from
// the partial sums of squares ss_in (added in gemm_kernel's order), for the split GEMM's
// finish kernel.
template <typename T>
static __global__ __launch_bounds__(256) void rows_to_fragments_kernel(const T* __restrict__ X, T* __restrict__ Xf,
                                                                      int nrt, int K, const float* __restrict__ ss_in,
                                                                      int n_part, int ss_stride, float eps,
                                                                      float* __restrict__ rs_out) {
  if (rs_out != nullptr && (int)blockIdx.x >= nrt && (int)blockIdx.x < 2 * nrt) {
    const int rt = (int)blockIdx.x - nrt, row = threadIdx.x >> 4, f = threadIdx.x & 15;
    const float* ss = ss_in + (size_t)rt * ss_stride;
    float q = 0.0f;
#pragma unroll 8
    for (int p = f; p < n_part; p += 16) q += ss[p * 16 + row];
    q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
    q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
    if (f == 0) rs_out[rt * 16 + row] = 1.0f / sqrtf(q / (float)K + eps);
  }
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int lane = idx & 63, f = idx >> 6;
  const int KS = K >> 5;
  if (f >= KS * nrt) return;
  const int ks = f / nrt, rt = f - ks * nrt;
  const int j = lane & 15, kq = lane >> 4;
  float v[8];
  load8<T>(X + (size_t)(rt * 16 + j) * K + ks * 32 + kq * 8, v);
  T* dst = Xf + (((size_t)ks * GEMM_WIDE_RT + rt) * 64 + lane) * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) Store<T>::st(dst + e, v[e]);
}

template <typename T, int PRO, int EPI>
static __global__ __launch_bounds__(512) void gemm_wide_kernel(const GemmArgs a) {
  extern __shared__ float lds[];
  constexpr int ND = (EPI == EPI_GATED) ? 2 : 1;
  constexpr int U = GEMM_WIDE_U, RT = GEMM_WIDE_RT;   // a deeper ring (4 k-steps) measured the same
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, S = blockDim.x >> 6;
  const int j = lane & 15, kq = lane >> 4;
  const int KS = a.K >> 5;
  const int ks0 = min(KS, wave * a.ksteps_per_wave), ks1 = min(KS, ks0 + a.ksteps_per_wave);
  const int ntiles = a.N >> 4;
  // work items: pairs of weight streams.  Gated FFN: (gate, up) of tile p; else tiles 2p, 2p+1.
  const int npairs = (ND == 2) ? ntiles : (ntiles + 1) / 2;
  const int my_pairs = (npairs - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  auto stream_tile = [&](int pair, int st) { return (ND == 2) ? pair : 2 * pair + st; };
  float* part = lds;                                 // [S][2][RT][256]
  float* ybuf = part + S * 2 * RT * 256;             // [2][RT][256]
  float* stat = ybuf + 2 * RT * 256;                 // [S][16]
  float* rs_s = stat + S * 16;                       // [RT * 16] 1 / rms of every row (PRO_POST)
  int* pos_s = reinterpret_cast<int*>(rs_s + RT * 16);          // [RT * 16] position of every row (EPI_QKV)
  unsigned long long* kvb_s = reinterpret_cast<unsigned long long*>(pos_s + RT * 16);   // [RT * 16] cache offset
  const int nrt = a.nrt;
  auto slab_rows = [&](int rt) { return (rt == nrt - 1) ? a.R_last : a.R; };

  // B side: clamped slab / row of this lane
  int jr[RT];
  bool jok[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rc = min(rt, nrt - 1), rows = slab_rows(rc);
    jr[rt] = rc * 16 + min(j, rows - 1);
    jok[rt] = (rt < nrt) && (j < rows);
  }
  // Epilogue side: thread t owns output e = t % 256 (row e / 16, feature e % 16) of the slabs
  // t / 256, t / 256 + blockDim / 256, ... of both streams
  const int e_row = (tid >> 4) & 15, e_f = tid & 15, e_idx = tid & 255;
  const int es_step = (int)blockDim.x >> 8, es0 = tid >> 8;          // 1 or 2; 0 or 1

  // ---- PRO_LN: statistics of the fp32 rows, slab by slab ----
  float mu[RT], rstd[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) { mu[rt] = 0.0f; rstd[rt] = 1.0f; }
  if (PRO == PRO_LN) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const float* x = static_cast<const float*>(a.X) + (size_t)jr[rt] * a.K + kq * 8;
      float s1 = 0.0f;
      for (int ks = ks0; ks < ks1; ++ks) {
        float v[8]; load8<float>(x + ks * 32, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) s1 += v[e];
      }
      s1 = lane_combine<16>(s1, OpSumF()); s1 = lane_combine<32>(s1, OpSumF());
      __syncthreads();
      if (kq == 0) stat[wave * 16 + j] = s1;
      __syncthreads();
      float t = 0.0f;
      for (int w = 0; w < S; ++w) t += stat[w * 16 + j];
      mu[rt] = t / (float)a.K;
      float s2 = 0.0f;
      for (int ks = ks0; ks < ks1; ++ks) {
        float v[8]; load8<float>(x + ks * 32, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) s2 = add_square(s2, v[e] - mu[rt]);
      }
      s2 = lane_combine<16>(s2, OpSumF()); s2 = lane_combine<32>(s2, OpSumF());
      __syncthreads();
      if (kq == 0) stat[wave * 16 + j] = s2;
      __syncthreads();
      float t2 = 0.0f;
      for (int w = 0; w < S; ++w) t2 += stat[w * 16 + j];
      rstd[rt] = 1.0f / sqrtf(t2 / (float)a.K + a.eps);
    }
  }

  typedef typename Mma<T>::Frag Frag;
  struct Slot { Frag fa[2]; Frag fb[RT]; };
  auto make_b = [&](int ks, bool valid, int rt) -> Frag {
    if (PRO != PRO_LN) {             // fragment order: one contiguous KB per (k-step, slab)
      const int rc = min(rt, nrt - 1);
      return Mma<T>::load(static_cast<const T*>(a.X) + (((size_t)ks * RT + rc) * 64 + lane) * 8);
    } else {
      const int k = ks * 32 + kq * 8;
      float v[8], g[8], bb[8];
      load8<float>(static_cast<const float*>(a.X) + (size_t)jr[rt] * a.K + k, v);
      load8<T>(static_cast<const T*>(a.gain) + k, g);
      load8<T>(static_cast<const T*>(a.beta) + k, bb);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = ln_apply(v[e], mu[rt], rstd[rt], g[e], bb[e]);
      return Mma<T>::select(valid && jok[rt], Mma<T>::from_floats(v));
    }
  };

  const int ks_last = max(ks1 - 1, 0);
  const int kpw = a.ksteps_per_wave;
  const int Q = my_pairs * kpw;                      // steps of this wavefront (the same for all)
  // cursor of the next step to load: pair index on this workgroup's list and k-step within the
  // wavefront's K slice, advanced without divisions; past the end it stays on the last step
  int l_pi = 0, l_kk = 0;
  auto load_step = [&](Slot& sl) {
    const int pair = (int)blockIdx.x + l_pi * (int)gridDim.x;
    const int ks = ks0 + l_kk, ksc = min(ks, ks_last);
    const size_t t0 = (size_t)stream_tile(pair, 0), t1 = (size_t)min(stream_tile(pair, 1), ntiles - 1);
    sl.fa[0] = Mma<T>::load_stream(static_cast<const T*>(a.W) + (t0 * KS + ksc) * 512 + lane * 8);
    sl.fa[1] = Mma<T>::load_stream(static_cast<const T*>(ND == 2 ? a.W2 : a.W) + (t1 * KS + ksc) * 512 + lane * 8);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) sl.fb[rt] = make_b(ksc, ks < ks1, rt);
    const bool last = (l_pi == my_pairs - 1) && (l_kk == kpw - 1);
    const bool wrap = (l_kk == kpw - 1) && !last;
    l_kk = last ? l_kk : (wrap ? 0 : l_kk + 1);
    l_pi = wrap ? l_pi + 1 : l_pi;
  };

  Slot ring[U];
#pragma unroll
  for (int u = 0; u < U; ++u) load_step(ring[u]);

  // ---- per row, tile-independent epilogue inputs, kept in LDS ----
  for (int r = tid >> 4; r < nrt * 16; r += (int)blockDim.x >> 4) {      // 16 lanes per row
    const int rt = r >> 4, r16 = r & 15, rows = slab_rows(rt);
    const int rc = rt * 16 + min(r16, rows - 1);                         // clamped: loads stay in bounds
    if (PRO == PRO_POST) {
      const float* ss = a.ss_in + (size_t)rt * a.ss_stride;
      float q = 0.0f;
      for (int p = e_f; p < a.n_part; p += 16) q += ss[p * 16 + (rc & 15)];
      q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
      q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
      if (e_f == 0) rs_s[r] = 1.0f / sqrtf(q / (float)a.K + a.eps);
    }
    if (EPI == EPI_QKV && e_f == 0) {
      const int pos = (r16 < rows) ? a.row_pos[rc] : -1;
      const int pc = max(pos, 0);
      const int pt0 = (a.row_seq != nullptr) ? a.row_seq[rc] * a.pt_stride : 0;
      const int page = a.page_table[pt0 + pc / a.page_size], slot = pc % a.page_size;
      pos_s[r] = pos;
      kvb_s[r] = (unsigned long long)page * 2 * a.n_kv_heads * a.page_size * a.d_head + (unsigned long long)slot * a.d_head;
    }
  }
  // (the first barrier of finish_pair orders these writes before their use)

  const bool has_bias = a.bias != nullptr, has_gain = (EPI == EPI_RESID) && a.xg_out != nullptr;

  f32x4 acc[2][RT];
#pragma unroll
  for (int d = 0; d < 2; ++d)
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[d][rt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // One barrier before the partial tiles are written (the previous pair's epilogue has read
  // them), one after; every thread then finishes its outputs of its slabs.
  auto finish_pair = [&](int pi) {
    const int pair = (int)blockIdx.x + pi * (int)gridDim.x;
    __syncthreads();
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int r = 0; r < 4; ++r) part[((wave * 2 + d) * RT + rt) * 256 + j * 16 + kq * 4 + r] = acc[d][rt][r];
        acc[d][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    __syncthreads();
    const int f = e_f;
    constexpr int NOUT = (ND == 2) ? 1 : 2;         // output tiles of the pair
#pragma unroll
    for (int o = 0; o < NOUT; ++o) {
      const int tile = stream_tile(pair, o);
      if (tile < ntiles) {                           // uniform over the workgroup
        const int n = tile * 16 + f;
        const float bias = has_bias ? Store<T>::ld(static_cast<const T*>(a.bias) + n) : 0.0f;
        const float gain = has_gain ? Store<T>::ld(static_cast<const T*>(a.gain_next) + n) : 0.0f;
        for (int rt = es0; rt < nrt; rt += es_step) {
          const int row = rt * 16 + e_row;
          const bool ok = e_row < slab_rows(rt);
          float y[2];
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            float s1 = 0.0f;
            const int st = (ND == 2) ? d : o;
            for (int w = 0; w < S; ++w) s1 += part[((w * 2 + st) * RT + rt) * 256 + e_idx];
            y[d] = s1;
          }
          if (PRO == PRO_POST) {
            const float r1 = rs_s[row];
            y[0] *= r1; y[1] *= r1;
          }
          y[0] += bias;
          if (EPI == EPI_QKV) {
            ybuf[(o * RT + rt) * 256 + e_idx] = y[0];
          } else if (EPI == EPI_RESID) {
            float xn = 0.0f;
            if (ok) {
              xn = static_cast<const float*>(a.out)[(size_t)row * a.ldo + n] + y[0];
              static_cast<float*>(a.out)[(size_t)row * a.ldo + n] = xn;
              if (a.xg_out != nullptr) Store<T>::st(static_cast<T*>(a.xg_out) + (size_t)row * a.ldo + n, xn * gain);
            }
            if (a.ss_out != nullptr) {
              float q = square(xn);
              q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
              q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
              if (f == 0) a.ss_out[(size_t)rt * a.ss_stride + tile * 16 + e_row] = q;
            }
          } else if (ok) {
            if (EPI == EPI_STORE) {
              Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, y[0]);
            } else if (EPI == EPI_ACT) {
              Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, gelu_tanh(y[0]));
            } else if (EPI == EPI_GATED) {
              const float g = (a.act == ACT_GELU) ? gelu_tanh(y[0]) : silu(y[0]);
              Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, g * y[1]);
            } else if (EPI == EPI_LOGITS) {
              const int orow = (a.out_row != nullptr) ? a.out_row[row] : row;
              if (orow >= 0) static_cast<float*>(a.out)[(size_t)orow * a.ldo + n] = a.scale * y[0];
            }
          }
        }
      }
    }
    if (EPI == EPI_QKV) {
      __syncthreads();
#pragma unroll
      for (int o = 0; o < NOUT; ++o) {
        const int tile = stream_tile(pair, o);
        if (tile < ntiles) {
          const int n = tile * 16 + f;
          const bool is_q = n < a.nq, is_k = !is_q && n < a.nq + a.nkv;
          const int nn = is_q ? n : (is_k ? n - a.nq : n - a.nq - a.nkv);
          const int head = nn / a.d_head, d = nn % a.d_head;
          for (int rt = es0; rt < nrt; rt += es_step) {
            const int row = rt * 16 + e_row;
            if (e_row < slab_rows(rt)) {
              const int pos = pos_s[row];
              float y = ybuf[(o * RT + rt) * 256 + e_idx];
              if (a.rope != nullptr && (is_q || is_k) && pos >= 0) {
                const float* cs = a.rope + ((size_t)pos * (a.d_head >> 1) + (d >> 1)) * 2;
                const float other = ybuf[(o * RT + rt) * 256 + (e_idx ^ 1)];
                y = rope_rotate(y, other, cs[0], cs[1], (d & 1) != 0);
              }
              if (is_q) {
                Store<T>::st(static_cast<T*>(a.q_out) + (size_t)row * a.nq + n, y);
              } else if (pos >= 0) {
                const size_t idx = (size_t)kvb_s[row] + ((size_t)(is_k ? 0 : 1) * a.n_kv_heads + head) * a.page_size * a.d_head + d;
                Store<T>::st(static_cast<T*>(a.kv_pool) + idx, y);
              }
            }
          }
        }
      }
    }
  };

  const int Qpad = (Q + U - 1) / U * U;
  int c_pi = 0, c_kk = 0;                          // the step being multiplied
  for (int q0 = 0; q0 < Qpad; q0 += U) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int q = q0 + u;
      const bool kvalid = (q < Q) && (ks0 + c_kk < ks1);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const Frag fb = (PRO == PRO_LN) ? Mma<T>::select(q < Q, ring[u].fb[rt]) : Mma<T>::select(kvalid && jok[rt], ring[u].fb[rt]);
        acc[0][rt] = Mma<T>::mma(ring[u].fa[0], fb, acc[0][rt]);
        acc[1][rt] = Mma<T>::mma(ring[u].fa[1], fb, acc[1][rt]);
      }
      load_step(ring[u]);
      const bool tile_end = (q < Q) && (c_kk == kpw - 1);
      if (tile_end) finish_pair(c_pi);
      c_pi = tile_end ? c_pi + 1 : c_pi;
      c_kk = (c_kk == kpw - 1) ? 0 : c_kk + 1;
    }
  }
}

// Re-tile a row-major [N][K] weight into MFMA operand order (see above).
// One thread moves 8 consecutive K-elements.
template <typename T>
static __global__ void retile_kernel(const T* __restrict__ src, T* __restrict__ dst, int N, int K) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // index of an 8-element group
  const size_t total = (size_t)N * K / 8;
  if (i >= total) return;
  const int KS = K >> 5;
  const int lane = (int)(i & 63);
  const size_t blk = i >> 6;                   // tile * KS + ks
  const int ks = (int)(blk % KS);
  const size_t tile = blk / KS;
  const size_t n = tile * 16 + (lane & 15);
  const size_t k = (size_t)ks * 32 + (lane >> 4) * 8;
  const T* s = src + n * K + k;
  T* d = dst + i * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) d[e] = s[e];
}

// ---------------------------------------------------------------------------
// Several slabs, second design: the wavefronts of a workgroup share the activations.
// gemm_wide_kernel splits K over the wavefronts of a workgroup, so every wavefront pulls its
// own activation fragments from L2 (a KB per slab for every KB of weights), and that traffic
// bounds it.  Here a workgroup takes one K chunk (the k-steps one wavefront of gemm_kernel
// would take) of NW tiles, one per wavefront (two weight streams for a gated FFN: the
// gate and up tiles; NW = 8, or 12 when that makes the grid fit the chip in one round): the chunk's activation fragments pass through LDS once per workgroup,
// SplitShape<T>::SUB k-steps at a time, and serve all its wavefronts; a weight register is
// reloaded for the next pass right after its multiply.  Each wavefront leaves the partial tile of its chunk in
// global memory; gemm_split_finish_kernel adds the chunks in wavefront order and applies
// the epilogue, so a row's sums are those of gemm_kernel, bit for bit.
// grid = (ceil(tiles / NW), chunks); dynamic LDS = SUB * nrt fragments.
template <typename T> struct SplitShape { static constexpr int SUB = 16 / (int)sizeof(T); };   // k-steps per pass: 8 of bf16, 4 of fp32 (8 KB of activation fragments per slab)

template <typename T, int NS, int NW>
static __global__ __launch_bounds__(64 * NW) void gemm_split_kernel(const GemmArgs a) {
  typedef typename Mma<T>::Frag Frag;
  extern __shared__ float lds[];
  Frag* xs = reinterpret_cast<Frag*>(lds);          // [SUB][nrt][64 lanes]
  constexpr int SUB = SplitShape<T>::SUB, RT = GEMM_WIDE_RT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KS = a.K >> 5, ntiles = a.N >> 4, nrt = a.nrt;
  const int chunk = blockIdx.y;
  const int ks0 = min(KS, chunk * a.ksteps_per_wave), ks1 = min(KS, ks0 + a.ksteps_per_wave);
  const int tile = (int)blockIdx.x * NW + wave, tilec = min(tile, ntiles - 1);
  const int ks_last = max(ks1 - 1, 0);
  const T* wbase[NS];
  wbase[0] = static_cast<const T*>(a.W) + ((size_t)tilec * KS) * 512 + lane * 8;
  if (NS == 2) wbase[NS - 1] = static_cast<const T*>(a.W2) + ((size_t)tilec * KS) * 512 + lane * 8;
  const Frag* xf = reinterpret_cast<const Frag*>(a.X);            // [KS][RT][64 lanes]

  f32x4 acc[NS][RT];
#pragma unroll
  for (int st = 0; st < NS; ++st)
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[st][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // All loads are unconditional and clamped: no branch around loads.
  Frag wf[NS][SUB];
#pragma unroll
  for (int st = 0; st < NS; ++st)
#pragma unroll
    for (int u = 0; u < SUB; ++u) wf[st][u] = Mma<T>::load_stream(wbase[st] + (size_t)min(ks0 + u, ks_last) * 512);
  // this thread's share of a pass's activation fragments (SUB * nrt * 64 of them over the workgroup)
  constexpr int NT = 64 * NW, XPT = (SUB * RT * 64 + NT - 1) / NT;
  Frag xr[XPT];
  const int nfrag = SUB * nrt * 64;
  auto load_x = [&](int ksb) {
#pragma unroll
    for (int m = 0; m < XPT; ++m) {
      const int i = min(tid + NT * m, nfrag - 1);
      const int u = i / (nrt * 64), rem = i - u * (nrt * 64);
      xr[m] = xf[(size_t)min(ksb + u, ks_last) * (RT * 64) + rem];
    }
  };
  load_x(ks0);
  for (int ksb = ks0; ksb < ks1; ksb += SUB) {
    __syncthreads();                                 // the previous pass has been multiplied
#pragma unroll
    for (int m = 0; m < XPT; ++m)
      if (tid + NT * m < nfrag) xs[tid + NT * m] = xr[m];
    __syncthreads();
    load_x(ksb + SUB);                               // the next pass's activations are in flight while this one is multiplied
#pragma unroll
    for (int u = 0; u < SUB; ++u) {
      if (ksb + u < ks1) {                           // uniform; k-steps in order, as gemm_kernel takes them
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          if (rt < nrt) {
            const Frag fb = xs[(u * nrt + rt) * 64 + lane];
#pragma unroll
            for (int st = 0; st < NS; ++st) acc[st][rt] = Mma<T>::mma(wf[st][u], fb, acc[st][rt]);
          }
        }
      }
      // this register's k-step of the next pass is on its way while the rest of this pass is multiplied
#pragma unroll
      for (int st = 0; st < NS; ++st) wf[st][u] = Mma<T>::load_stream(wbase[st] + (size_t)min(ksb + SUB + u, ks_last) * 512);
    }
  }
  if (tile < ntiles) {
#pragma unroll
    for (int st = 0; st < NS; ++st)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        if (rt < nrt)
          *reinterpret_cast<f32x4*>(a.partial + ((((size_t)chunk * nrt + rt) * (NS * ntiles) + (size_t)st * ntiles + tile) * 64 + lane) * 4) = acc[st][rt];
  }
}

// Adds the chunks' partial tiles in chunk order and applies the epilogue of one (tile, slab):
// grid = (tiles, slabs), thread t = row * 16 + feature.  The partial tiles are requested first;
// the row's constants (norm factor, cache position) arrive while they are on their way.
template <typename T, int PRO, int EPI>
static __global__ __launch_bounds__(256) void gemm_split_finish_kernel(const GemmArgs a) {
  constexpr int ND = (EPI == EPI_GATED) ? 2 : 1;
  const int tid = threadIdx.x, e_row = tid >> 4, f = tid & 15;
  const int tile = blockIdx.x, rt = blockIdx.y, nrt = a.nrt, ntiles = a.N >> 4;
  const int rows = (rt == nrt - 1) ? a.R_last : a.R;
  const int row = rt * 16 + e_row, rc = rt * 16 + min(e_row, rows - 1);      // clamped: loads stay in bounds
  const bool ok = e_row < rows;
  const int n = tile * 16 + f;
  // accumulator layout: lane (row, feature / 4) holds features 4 (lane / 16) + r of row lane % 16
  const int pidx = (e_row + 16 * (f >> 2)) * 4 + (f & 3);
  float pv[ND][8];                                   // at most 8 chunks
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int w = 0; w < 8; ++w)
      pv[d][w] = a.partial[((((size_t)min(w, a.nchunk - 1) * nrt + rt) * (ND * ntiles) + (size_t)d * ntiles + tile) * 256) + pidx];
  const float bias = (a.bias != nullptr) ? Store<T>::ld(static_cast<const T*>(a.bias) + n) : 0.0f;
  const float r1 = (PRO == PRO_POST) ? a.rs_in[rc] : 1.0f;
  float y[2] = {0.0f, 0.0f};
#pragma unroll
  for (int d = 0; d < ND; ++d) {
    float s1 = 0.0f;
#pragma unroll
    for (int w = 0; w < 8; ++w) if (w < a.nchunk) s1 += pv[d][w];
    y[d] = s1;
  }
  if (PRO == PRO_POST) { y[0] *= r1; y[1] *= r1; }
  y[0] += bias;
  if (EPI == EPI_QKV) {
    const int pos = ok ? a.row_pos[rc] : -1;
    const bool is_q = n < a.nq, is_k = !is_q && n < a.nq + a.nkv;
    const int nn = is_q ? n : (is_k ? n - a.nq : n - a.nq - a.nkv);
    const int head = nn / a.d_head, d = nn % a.d_head;
    float v = y[0];
    const float other = __shfl_xor(v, 1, 64);        // the other half of the rotary pair: feature f ^ 1 of the same row
    if (a.rope != nullptr && (is_q || is_k) && pos >= 0) {
      const float* cs = a.rope + ((size_t)pos * (a.d_head >> 1) + (d >> 1)) * 2;
      v = rope_rotate(v, other, cs[0], cs[1], (d & 1) != 0);
    }
    if (ok) {
      if (is_q) {
        Store<T>::st(static_cast<T*>(a.q_out) + (size_t)row * a.nq + n, v);
      } else if (pos >= 0) {
        const int pt0 = (a.row_seq != nullptr) ? a.row_seq[rc] * a.pt_stride : 0;
        const int page = a.page_table[pt0 + pos / a.page_size], slot = pos % a.page_size;
        const size_t base = (size_t)page * 2 * a.n_kv_heads * a.page_size * a.d_head + (size_t)slot * a.d_head;
        Store<T>::st(static_cast<T*>(a.kv_pool) + base + ((size_t)(is_k ? 0 : 1) * a.n_kv_heads + head) * a.page_size * a.d_head + d, v);
      }
    }
  } else if (EPI == EPI_RESID) {
    float xn = 0.0f;
    if (ok) {
      xn = static_cast<const float*>(a.out)[(size_t)row * a.ldo + n] + y[0];
      static_cast<float*>(a.out)[(size_t)row * a.ldo + n] = xn;
      if (a.xg_out != nullptr)
        Store<T>::st(static_cast<T*>(a.xg_out) + (size_t)row * a.ldo + n, xn * Store<T>::ld(static_cast<const T*>(a.gain_next) + n));
    }
    if (a.ss_out != nullptr) {
      float q = square(xn);
      q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
      q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
      if (f == 0) a.ss_out[(size_t)rt * a.ss_stride + tile * 16 + e_row] = q;
    }
  } else if (ok) {
    if (EPI == EPI_STORE) {
      Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, y[0]);
    } else if (EPI == EPI_GATED) {
      const float g = (a.act == ACT_GELU) ? gelu_tanh(y[0]) : silu(y[0]);
      Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n, g * y[1]);
    }
  }
}

// Gated FFN-in over several slabs: there are enough tiles to fill the chip without splitting K
// over workgroups, and the partial tiles of a split would be many (chunks x 2 streams x d_ff).
// A workgroup of four wavefronts takes four tiles (gate and up stream each) through ALL of K,
// the activation fragments passing through LDS as in gemm_split_kernel; every wavefront keeps
// gemm_kernel's sums: the k-steps of a chunk go into `acc` in order, and at a chunk's end `acc`
// is added to the running total, chunks in order -- the additions gemm_kernel's epilogue
// makes -- so the results stay bit-identical.  One workgroup per CU, one wavefront per SIMD: nothing
// hides a stall, so the number of slabs is a template parameter (no branch inside a pass), the
// activation fragments of k-step u + 1 are read from LDS while k-step u is multiplied, a weight
// register is reloaded for the next pass right after its multiply (no second copy), and running
// totals and accumulators both live in registers (a wavefront alone on its SIMD has 512).
// Epilogue out of registers: norm factor (from rows_to_fragments_kernel), activation, product.
// grid = ceil(tiles / 4); dynamic LDS = SUB * NRT fragments.
constexpr int GEMM_GATED_NW = 4;
template <typename T> __host__ __device__ constexpr size_t gemm_gated_lds_bytes(int nrt) {
  return (size_t)SplitShape<T>::SUB * nrt * 64 * 8 * sizeof(T);
}
// EPI == EPI_LOGITS: the same walk for the LM head; a wavefront's two streams are the tiles 2 t and
// 2 t + 1 of the one weight matrix, the epilogue scales and routes the rows (out_row).
template <typename T, int EPI, int NRT>
static __global__ __launch_bounds__(64 * GEMM_GATED_NW) void gemm_gated_wide_kernel(const GemmArgs a) {
  typedef typename Mma<T>::Frag Frag;
  extern __shared__ float lds[];
  constexpr int SUB = SplitShape<T>::SUB, RT = GEMM_WIDE_RT, NW = GEMM_GATED_NW, NT = 64 * NW;
  constexpr int nrt = NRT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, kq = lane >> 4;
  const int KS = a.K >> 5, ntiles = a.N >> 4, kpw = a.ksteps_per_wave;
  Frag* xs = reinterpret_cast<Frag*>(lds);                        // [SUB][NRT][64 lanes]
  // work item = pair of streams: (gate, up) of tile `item`, or tiles 2 item and 2 item + 1
  const int nitems = (EPI == EPI_GATED) ? ntiles : (ntiles + 1) / 2;
  const int item = (int)blockIdx.x * NW + wave, itemc = min(item, nitems - 1);
  const int tile0 = (EPI == EPI_GATED) ? itemc : 2 * itemc, tile1 = (EPI == EPI_GATED) ? itemc : min(2 * itemc + 1, ntiles - 1);
  const T* wbase[2];
  wbase[0] = static_cast<const T*>(a.W) + ((size_t)tile0 * KS) * 512 + lane * 8;
  wbase[1] = static_cast<const T*>((EPI == EPI_GATED) ? a.W2 : a.W) + ((size_t)tile1 * KS) * 512 + lane * 8;
  const Frag* xf = reinterpret_cast<const Frag*>(a.X);            // [KS][RT][64 lanes]

  f32x4 acc[2][NRT], tot[2][NRT];
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) { acc[st][rt] = f32x4{0.f, 0.f, 0.f, 0.f}; tot[st][rt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
  Frag wf[2][SUB];
  // this thread's share of a pass's activation fragments: fragment i = tid + NT m is (k-step
  // i / (NRT * 64), slab and lane i % (NRT * 64)); the split is the same for every pass
  constexpr int NFRAG = SUB * NRT * 64, XPT = (NFRAG + NT - 1) / NT;
  Frag xr[XPT];
  auto load_x = [&](int ksb) {                       // unconditional, clamped: no branch around loads
#pragma unroll
    for (int m = 0; m < XPT; ++m) {
      const int i = min(tid + NT * m, NFRAG - 1);
      const int u = i / (NRT * 64), rem = i - u * (NRT * 64);       // (a division by a constant)
      xr[m] = xf[(size_t)min(ksb + u, KS - 1) * (RT * 64) + rem];
    }
  };
  // a pass never crosses a chunk's end: its k-steps are [ksb, ksb + len)
  auto pass_len = [&](int ksb) { return min(SUB, min(KS, (ksb / kpw + 1) * kpw) - ksb); };
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int u = 0; u < SUB; ++u) wf[st][u] = Mma<T>::load_stream(wbase[st] + (size_t)min(u, KS - 1) * 512);
  load_x(0);
  int chunks_done = 0;
  for (int ksb = 0; ksb < KS;) {
    const int len = pass_len(ksb), next = ksb + len;
    __syncthreads();                                 // the previous pass has been multiplied
#pragma unroll
    for (int m = 0; m < XPT; ++m)
      if (NFRAG % NT == 0 || tid + NT * m < NFRAG) xs[tid + NT * m] = xr[m];
    __syncthreads();
    load_x(next);
    if (len == SUB) {                                // (uniform) a whole pass, straight-line
      constexpr int NB = (NRT <= 5) ? 2 : 1;         // six slabs: no registers left for a second set of fragments
      Frag fb[NB][NRT];
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) fb[0][rt] = xs[rt * 64 + lane];
#pragma unroll
      for (int u = 0; u < SUB; ++u) {
        if (NB == 2 && u + 1 < SUB) {
#pragma unroll
          for (int rt = 0; rt < NRT; ++rt) fb[(u + 1) & 1][rt] = xs[((u + 1) * NRT + rt) * 64 + lane];
        }
        if (NB == 1 && u > 0) {
#pragma unroll
          for (int rt = 0; rt < NRT; ++rt) fb[0][rt] = xs[(u * NRT + rt) * 64 + lane];
        }
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          acc[0][rt] = Mma<T>::mma(wf[0][u], fb[u & (NB - 1)][rt], acc[0][rt]);
          acc[1][rt] = Mma<T>::mma(wf[1][u], fb[u & (NB - 1)][rt], acc[1][rt]);
        }
        // this register's next k-step is on its way while the rest of the pass is multiplied
        wf[0][u] = Mma<T>::load_stream(wbase[0] + (size_t)min(next + u, KS - 1) * 512);
        wf[1][u] = Mma<T>::load_stream(wbase[1] + (size_t)min(next + u, KS - 1) * 512);
      }
    } else {                                         // the short pass at a chunk's end
#pragma unroll
      for (int u = 0; u < SUB; ++u) {
        if (u < len) {                               // uniform
#pragma unroll
          for (int rt = 0; rt < NRT; ++rt) {
            const Frag fb = xs[(u * NRT + rt) * 64 + lane];
            acc[0][rt] = Mma<T>::mma(wf[0][u], fb, acc[0][rt]);
            acc[1][rt] = Mma<T>::mma(wf[1][u], fb, acc[1][rt]);
          }
        }
        wf[0][u] = Mma<T>::load_stream(wbase[0] + (size_t)min(next + u, KS - 1) * 512);
        wf[1][u] = Mma<T>::load_stream(wbase[1] + (size_t)min(next + u, KS - 1) * 512);
      }
    }
    if (next == KS || next % kpw == 0) {             // the chunk is complete: add it, chunks in order
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
#pragma unroll
          for (int r = 0; r < 4; ++r) tot[st][rt][r] += acc[st][rt][r];
          acc[st][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      ++chunks_done;
    }
    ksb = next;
  }
  if (item >= nitems) return;
  // accumulator layout: lane holds features 4 kq + r, r = 0..3, of row j
  const int n0 = tile0 * 16 + kq * 4;
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    {
      const int rows = (rt == nrt - 1) ? a.R_last : a.R;
      if (j < rows) {
        const int row = rt * 16 + j;
        const float r1 = a.rs_in[row];
        f32x4 t0 = tot[0][rt], t1 = tot[1][rt];
        for (int c = chunks_done; c < a.nchunk; ++c)      // chunks beyond K are empty in gemm_kernel too: it adds their zeros
#pragma unroll
          for (int r = 0; r < 4; ++r) { t0[r] += 0.0f; t1[r] += 0.0f; }
        if (EPI == EPI_LOGITS) {
          const int orow = (a.out_row != nullptr) ? a.out_row[row] : row;
          if (orow >= 0) {
#pragma unroll
            for (int st = 0; st < 2; ++st) {
              if (st == 1 && 2 * item + 1 >= ntiles) break;          // an odd number of tiles: no second stream
              const int n1 = (2 * item + st) * 16 + kq * 4;
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                float y = (st ? t1[r] : t0[r]) * r1;
                y += (a.bias != nullptr) ? Store<T>::ld(static_cast<const T*>(a.bias) + n1 + r) : 0.0f;
                static_cast<float*>(a.out)[(size_t)orow * a.ldo + n1 + r] = a.scale * y;
              }
            }
          }
          continue;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float y0 = t0[r] * r1;
          const float y1 = t1[r] * r1;
          y0 += (a.bias != nullptr) ? Store<T>::ld(static_cast<const T*>(a.bias) + n0 + r) : 0.0f;
          const float g = (a.act == ACT_GELU) ? gelu_tanh(y0) : silu(y0);
          if (a.out_frag != nullptr)     // element (row, n): k-step n / 32, lane (row % 16) + 16 ((n % 32) / 8), element n % 8
            Store<T>::st(static_cast<T*>(a.out_frag) + ((((size_t)((n0 + r) >> 5) * RT + rt) * 64 + j + 16 * (((n0 + r) & 31) >> 3)) * 8 + ((n0 + r) & 7)), g * y1);
          else
            Store<T>::st(static_cast<T*>(a.out) + (size_t)row * a.ldo + n0 + r, g * y1);
        }
      }
    }
  }
}

}  // namespace sd
