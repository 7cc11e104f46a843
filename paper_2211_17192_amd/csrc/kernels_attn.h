// Multi-query decode attention for the (gamma+1)-row forward.
//
// The R query rows (positions row_pos[0..R)) of every head attend causally to
// the paged KV cache (self-attention; the rows' own keys were appended by the
// QKV projection just before) or to a fixed block of encoder keys
// (cross-attention).
//
// One workgroup of 256, 512 or 1024 threads owns one kv head (and a few of the query rows:
// rows are independent, so splitting them needs no merge) and walks its keys in blocks
// (one key per 2 threads, per 4 for d_head 128) with an online softmax (running max m,
// denominator l, unnormalised output O per row).  There is no split over
// workgroups and therefore no cross-workgroup merge: device-scope atomics cost
// about a quarter of a microsecond each on this chip when they queue on one
// address, which is more than the whole kernel should take.  The kernel is
// latency-bound, so every thread issues all its K and V loads of a key block
// up front with 16-byte loads and no branches (they do not depend on the
// scores), and the rest runs out of registers and LDS:
//   scores  LPK lanes per key, each holding a slice of the head dimension of
//           its key in registers and dotting it with every query row (in LDS);
//   softmax one wavefront per row over the block's scores;
//   P*V     thread = (group of KPT consecutive keys, 8 head-dim elements); the
//           groups of a wavefront are added by lane shuffles, the wavefronts in
//           fixed order through LDS.
// Key blocks sit at absolute positions and all reduction orders are fixed, so
// a row's result does not depend on R or on the other rows: a row computed
// alone (plain decoding) is bit-identical to the same row among gamma+1.
// KV layout per layer: [page][K|V][kv_head][slot][d_head]; a (kv head, page)
// is a contiguous page_size * d_head block.  Cross keys / values: [head][key][d_head].
#pragma once
#include "common.h"

namespace sd {


constexpr int ATTN_LDS_DIST = 4096;        // causal distances whose bias bucket is cached in LDS
constexpr int ATTN_MAX_RG = 32;            // query rows x heads per kv head: two 16-row MFMA tiles; 150 KB of LDS in attn_kernel at d_head 64

// LPK lanes per key and DP head-dim elements per lane in the score phase (a workgroup of THREADS
// threads takes THREADS / LPK keys per block); KPT consecutive keys per thread in the P*V phase;
// RPP rows per P*V pass (bounds the LDS reduction buffer [wavefronts][RPP][DH] to 64 KB).
template <int DH> struct AttnShape;
template <> struct AttnShape<32>  { static constexpr int LPK = 2, DP = 16, KPT = 2, RPP = 16; };
template <> struct AttnShape<64>  { static constexpr int LPK = 2, DP = 32, KPT = 4, RPP = 16; };
template <> struct AttnShape<128> { static constexpr int LPK = 4, DP = 32, KPT = 4, RPP = 8; };
constexpr int attn_block_keys(int dh, int threads = 1024) { return threads / (dh == 128 ? 4 : 2); }
constexpr int attn_rows_per_pass(int dh) { return dh == 128 ? 8 : 16; }

struct AttnArgs {
  const void* q;            // T [R][H*dh]
  void* out;                // T [R][H*dh]
  const void* kv_pool;      // self: this layer's pages
  const void* ck; const void* cv;   // cross: T [H][kv_len][dh] each
  const int* page_table;
  int page_size, n_pages;   // page_size a power of two >= 16; n_pages entries per sequence in page_table
  const int* row_pos;       // [R]; self: causal limit of each row, < 0 = padding row
  int R, H, Hkv;
  int G, g_mul;             // query heads per kv head; 65536 / G + 1: x / G == (x * g_mul) >> 16 for x < 1024
  int rows_per_wg;          // grid.y = ceil(R / rows_per_wg): rows are independent, no merge needed
  // several sequences in one launch: grid.z = sequences, R rows each, one after the other
  // (sequence z: rows z * R ..); sequence z uses the page table at page_table + (seq0 + z) * pt_stride
  int seq0, pt_stride;
  // long contexts: the keys of a (sequence, kv head) are cut into nsplit ranges of split_keys keys
  // (a multiple of the key block) that different workgroups take (grid.y = row groups x nsplit);
  // each leaves its running maximum, denominator and unnormalised output in `partial`
  // ([sequence][kv head][split][ATTN_MAX_RG][d_head + 2] floats) and attn_merge_kernel combines
  // them.  nsplit is fixed per model (from max_len), so the split never depends on the other rows.
  int nsplit, split_keys;
  float* partial;
  // attn_merge_kernel: when set, the merged output goes here in the batched GEMMs' fragment order
  // ([H * d_head / 32][GEMM_WIDE_RT][64 lanes][8]: element (row, n) at k-step n / 32, slab row / 16,
  // lane (row % 16) + 16 ((n % 32) / 8), element n % 8) instead of row-major into `out`
  void* out_frag;
  int cross;                // 1: cross-attention over kv_len keys, no mask, no bias
  int kv_len;
  float scale;
  const void* rel_bias;     // T [H][rel_buckets] or nullptr
  // attn_mma_kernel: the same bias laid out by distance: [H][bias_off + 4] floats, entry bias_off - d
  // for causal distance d = position - key in [0, bias_off], zeros after it
  const float* bias_by_key;
  int bias_off;
  const int* bucket_lut;    // [n_pages * page_size <= ATTN_LDS_DIST] bucket of each causal distance
  int rel_buckets;
  // attn_mma_kernel, mode ATTN_CROSS_PROJ: the kernel computes its head's queries itself from the
  // RMSNorm input of the cross-attention block, exactly as gemm_kernel<bf16, PRO_POST, EPI_STORE>
  // would (`q` is not read): pj_w = the projection's weights in MFMA tile order, pj_x = the rows
  // times the norm's gain [R][pj_K], pj_ss = [pj_npart][16] partial sums of squares of the rows,
  // pj_q_off = where in dynamic LDS (in floats) the 16 x d_head query rows go
  const void* pj_w; const void* pj_x; const float* pj_ss;
  int pj_K, pj_npart, pj_q_off;
  float pj_eps;
};

// THREADS (256, 512 or 1024) sets the key block: THREADS / LPK keys per pass, so a launch takes the
// smallest workgroup whose block covers the contexts it expects; CROSS compiles the cross-attention
// addressing (fixed keys, no mask, no bias) apart from the paged one.
// The kernel is a chain of latencies, so everything the first key block needs from memory leaves
// in one go before anything waits: the rows' positions and the page-table entries (cached reads),
// then the K and V rows (threads whose key lies beyond the context re-read the block's first key,
// whose page entry every thread holds, and get probability 0), then the queries and the bias tables on their way to LDS.  The next block's page entries are
// asked for a block ahead, its keys as soon as the scores have used the current ones, its values
// after the last P*V pass.
// dynamic LDS (floats): q [RG][DH] | s [RG][KB] | o [THREADS/64][RPP][DH] | m, l, f [3][RG] | acc [RG][DH]
template <typename T, int DH, int THREADS, bool CROSS>
static __global__ __launch_bounds__(THREADS) void attn_kernel(const AttnArgs a) {
  extern __shared__ float lds[];
  __shared__ int s_pos[MAX_ROWS];
  __shared__ float s_bias[4 * 64];                 // rel_bias rows of this kv head's query heads
  __shared__ unsigned char s_bucket[ATTN_LDS_DIST];
  typedef AttnShape<DH> SH;
  constexpr int LPK = SH::LPK, KB = THREADS / LPK, DP = SH::DP, KPT = SH::KPT, RPP = SH::RPP;
  constexpr int OCT = DH / 8;                      // 8-element slices of a V row
  constexpr int NW = THREADS / 64;
  static_assert((THREADS / OCT) * KPT == KB, "P*V mapping must cover the key block");
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hkv = blockIdx.x;
  // rows are independent: blockIdx.y takes rows [r0, r0 + R) of the launch
  const int split = (a.nsplit > 1) ? (int)blockIdx.y % a.nsplit : 0;
  const int rs = ((a.nsplit > 1) ? (int)blockIdx.y / a.nsplit : (int)blockIdx.y) * a.rows_per_wg;   // first row within the sequence
  const int R = min(a.rows_per_wg, a.R - rs);
  const int r0 = (int)blockIdx.z * a.R + rs;      // first row within the launch
  const int* page_table = a.page_table + (size_t)(a.seq0 + blockIdx.z) * a.pt_stride;
  const int G = a.H / a.Hkv, RG = R * G;
  const int kl_s = tid / LPK, part = tid % LPK;    // score phase: key within block, slice
  const int oct = tid % OCT, grp = tid / OCT;      // P*V phase: V slice, key group (KPT keys)
  const int page_shift = __ffs(a.page_size) - 1, page_mask = a.page_size - 1;
  const int key_cap = CROSS ? a.kv_len : a.n_pages * a.page_size;   // keys that exist in memory
  const int k_begin = split * a.split_keys;

  // ---- (1) positions and page entries ----
  int my_pos = -1;                                 // lane r of every wavefront: the causal limit of row r
  if (lane < R) my_pos = CROSS ? 0 : a.row_pos[r0 + lane];
  int pg0 = 0, pgk = 0, pgv[KPT];                 // page of the block's first key, of this thread's K key and V keys
  auto load_pages = [&](int k0) {
    if (CROSS) return;
    pg0 = page_table[k0 >> page_shift];
    pgk = page_table[min(k0 + kl_s, key_cap - 1) >> page_shift];
#pragma unroll
    for (int u = 0; u < KPT; ++u) pgv[u] = page_table[min(k0 + grp * KPT + u, key_cap - 1) >> page_shift];
  };
  auto row_ptr = [&](int key, int page, int which) -> const T* {   // which: 0 = K, 1 = V
    if (CROSS) return static_cast<const T*>(which ? a.cv : a.ck) + ((size_t)hkv * a.kv_len + key) * DH;
    return static_cast<const T*>(a.kv_pool) +
           ((((size_t)page * 2 + which) * a.Hkv + hkv) * a.page_size + (key & page_mask)) * DH;
  };
  // ---- (2) K and V rows of a block: unconditional 16-byte loads (a branch per load would serialise them) ----
  float kreg[DP];
  float vreg[KPT][8];                              // keys grp * KPT + u
  int kv_len = a.kv_len;                           // keys this workgroup attends to end here
  auto issue_k = [&](int k0) {
    const bool ok = k0 + kl_s < kv_len;
    const T* kp = row_ptr(ok ? k0 + kl_s : k0, ok ? pgk : pg0, 0) + part * DP;
#pragma unroll
    for (int e = 0; e < DP; e += 8) {
      float v[8];
      load8<T>(kp + e, v);
#pragma unroll
      for (int f = 0; f < 8; ++f) kreg[e + f] = v[f];
    }
  };
  auto issue_v = [&](int k0) {
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
      const bool ok = k0 + grp * KPT + u < kv_len;
      load8<T>(row_ptr(ok ? k0 + grp * KPT + u : k0, ok ? pgv[u] : pg0, 1) + oct * 8, vreg[u]);
    }
  };
#pragma unroll
  for (int u = 0; u < KPT; ++u) pgv[u] = 0;
  load_pages(k_begin);
  if (!CROSS) kv_len = wave_max(my_pos) + 1;
  const int kv_all = kv_len;                       // the context; kv_len: where this key range ends
  if (a.nsplit > 1) kv_len = min(kv_len, k_begin + a.split_keys);
  issue_k(k_begin);
  issue_v(k_begin);

  // ---- (3) queries and tables into LDS ----
  float* q_s = lds;                                // [RG][DH]
  float* s_s = q_s + RG * DH;                      // [RG][KB]
  float* o_s = s_s + RG * KB;                      // [NW][RPP][DH]
  float* m_s = o_s + NW * RPP * DH;                // [RG] running max
  float* l_s = m_s + RG;                           // [RG] running denominator
  float* f_s = l_s + RG;                           // [RG] rescale factor of this pass
  float* acc_s = f_s + RG;                         // [RG][DH] running output
  if (tid < MAX_ROWS) s_pos[tid] = my_pos;
  const T* qg = static_cast<const T*>(a.q);
  for (int i = tid; i < RG * DH; i += THREADS) {
    const int rg = i / DH, d = i % DH, r = rg / G, h = hkv * G + rg % G;
    q_s[i] = Store<T>::ld(qg + (size_t)(r0 + r) * a.H * DH + h * DH + d);
    acc_s[i] = 0.0f;
  }
  if (tid < RG) { m_s[tid] = -INFINITY; l_s[tid] = 0.0f; }
  // relative-position bias: table rows and distance -> bucket map (the distances this context
  // can hold) into LDS, so the score loop has no global loads
  const bool use_bias = !CROSS && a.rel_bias != nullptr;
  if (use_bias) {
    for (int i = tid; i < G * a.rel_buckets; i += THREADS)
      s_bias[i] = Store<T>::ld(static_cast<const T*>(a.rel_bias) + (size_t)(hkv * G) * a.rel_buckets + i);
    const int n_dist = min(ATTN_LDS_DIST, kv_all);
    for (int i = tid; i < n_dist; i += THREADS) s_bucket[i] = (unsigned char)a.bucket_lut[i];
  }
  if (a.nsplit > 1 && k_begin >= kv_len) {       // nothing in this key range yet: an empty partial
    float* pp = a.partial + ((((size_t)blockIdx.z * a.Hkv + hkv) * a.nsplit + split) * ATTN_MAX_RG + (size_t)rs * G) * (DH + 2);
    if (tid < RG) { pp[(size_t)tid * (DH + 2) + DH] = -INFINITY; pp[(size_t)tid * (DH + 2) + DH + 1] = 0.0f; }
    return;
  }
  __syncthreads();

  for (int k0 = k_begin; k0 < kv_len; k0 += KB) {
    const int nkeys = min(KB, kv_len - k0);
    const bool more = k0 + KB < kv_len;
    if (more) load_pages(k0 + KB);
    const bool key_ok = kl_s < nkeys;

    // ---- scores ----
    for (int rg = 0; rg < RG; ++rg) {
      const float4* qr = reinterpret_cast<const float4*>(q_s + rg * DH + part * DP);
      float4 q4[DP / 4];
#pragma unroll
      for (int e = 0; e < DP / 4; ++e) q4[e] = qr[e];
      float dot = 0.0f;
#pragma unroll
      for (int e = 0; e < DP / 4; ++e) {
        dot += q4[e].x * kreg[4 * e]; dot += q4[e].y * kreg[4 * e + 1];
        dot += q4[e].z * kreg[4 * e + 2]; dot += q4[e].w * kreg[4 * e + 3];
      }
      dot = lane_combine<1>(dot, OpSumF());
      if (LPK == 4) dot = lane_combine<2>(dot, OpSumF());
      if (part == 0) {
        const int r = rg / G, pos = s_pos[r], key = k0 + kl_s;
        float sc = -INFINITY;
        if (key_ok && pos >= 0 && (CROSS || key <= pos)) {
          sc = a.scale * dot;
          if (use_bias) sc += s_bias[(rg % G) * a.rel_buckets + (int)s_bucket[pos - key]];
        }
        s_s[rg * KB + kl_s] = sc;
      }
    }
    if (more) issue_k(k0 + KB);
    __syncthreads();

    // ---- online softmax: one wavefront per row ----
    for (int rg = wave; rg < RG; rg += NW) {
      float sc[KB / 64];
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < KB / 64; ++i) { sc[i] = s_s[rg * KB + i * 64 + lane]; mx = fmaxf(mx, sc[i]); }
      mx = wave_max(mx);
      const float m_old = m_s[rg];
      const float m_new = fmaxf(m_old, mx);
      float sum = 0.0f;
#pragma unroll
      for (int i = 0; i < KB / 64; ++i) {
        const float p = (sc[i] == -INFINITY) ? 0.0f : __expf(sc[i] - m_new);
        s_s[rg * KB + i * 64 + lane] = p;
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

    // ---- P * V out of registers, RPP rows per pass ----
    for (int rb = 0; rb < RG; rb += RPP) {
      const int nr = min(RPP, RG - rb);
      for (int i = 0; i < nr; ++i) {
        float pk[KPT];
        if (KPT == 4) {
          const float4 p4 = *reinterpret_cast<const float4*>(s_s + (rb + i) * KB + grp * KPT);
          pk[0] = p4.x; pk[1] = p4.y; pk[KPT - 2] = p4.z; pk[KPT - 1] = p4.w;
        } else {
          const float2 p2 = *reinterpret_cast<const float2*>(s_s + (rb + i) * KB + grp * KPT);
          pk[0] = p2.x; pk[KPT - 1] = p2.y;
        }
        float t[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = 0.0f;
#pragma unroll
        for (int u = 0; u < KPT; ++u)              // keys in ascending order
#pragma unroll
          for (int e = 0; e < 8; ++e) t[e] += pk[u] * vreg[u][e];
        // add the key groups of this wavefront (ascending lane distance: fixed order)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (OCT <= 4) t[e] = lane_combine<4>(t[e], OpSumF());
          if (OCT <= 8) t[e] = lane_combine<8>(t[e], OpSumF());
          t[e] = lane_combine<16>(t[e], OpSumF());
          t[e] = lane_combine<32>(t[e], OpSumF());
        }
        if (lane < OCT) {
          float* o = o_s + ((size_t)wave * RPP + i) * DH + oct * 8;
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = t[e];
        }
      }
      if (more && rb + RPP >= RG) issue_v(k0 + KB);
      __syncthreads();
      for (int i = tid; i < nr * DH; i += THREADS) {           // wavefronts = key ranges, ascending
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) t += o_s[w * RPP * DH + i];
        const int idx = rb * DH + i;
        acc_s[idx] = acc_s[idx] * f_s[idx / DH] + t;
      }
      __syncthreads();
    }
  }

  if (a.nsplit > 1) {            // leave the partial result of this key range for the merge
    float* pp = a.partial + ((((size_t)blockIdx.z * a.Hkv + hkv) * a.nsplit + split) * ATTN_MAX_RG + (size_t)rs * G) * (DH + 2);
    for (int i = tid; i < RG * DH; i += THREADS) pp[(size_t)(i / DH) * (DH + 2) + i % DH] = acc_s[i];
    if (tid < RG) { pp[(size_t)tid * (DH + 2) + DH] = m_s[tid]; pp[(size_t)tid * (DH + 2) + DH + 1] = l_s[tid]; }
    return;
  }
  T* og = static_cast<T*>(a.out);
  for (int i = tid; i < RG * DH; i += THREADS) {
    const int rg = i / DH, d = i % DH, r = rg / G, h = hkv * G + rg % G;
    const float L = l_s[rg];
    Store<T>::st(og + (size_t)(r0 + r) * a.H * DH + h * DH + d, (L > 0.0f) ? acc_s[i] / L : 0.0f);
  }
}

// bf16 attention on the matrix cores.  attn_kernel is a chain of a few hundred vector
// instructions per wavefront, and a wavefront issues one every four cycles at best: at decode
// sizes that chain, not memory, is most of its time.  Here the two products are MFMAs and the
// operands go from the cache rows straight into their fragments, so a 32-key step is a few dozen
// instructions.  A workgroup has NW (4 or 8) wavefronts that never synchronise inside the key
// loop; each walks every NW-th 32-key step of its key range with its own running maximum,
// denominator and output, all in registers (more wavefronts than that lose more at the merge
// than they gain on the steps):
//   S^T = K Q^T   16x16x32 MFMA, A = 16 keys x 32 features straight from the cache rows,
//                 B = the query rows (rows x heads of the kv head, zero-padded to 16 or 32),
//                 kept in registers for the whole kernel.  Which features a lane holds is free
//                 as long as both operands agree: in k-step s the four quarters of a key read
//                 64 contiguous bytes of its row (features 32 s + 8 kq ..).  A lane ends up with
//                 the scores of one query row for 8 keys, so the softmax needs two lane
//                 exchanges per step only.
//   O^T = V^T P   A = 16 features x 32 keys: V is key-major in the cache, so every wavefront
//                 copies its 32 x d_head tile into a private LDS region with fully coalesced
//                 16-byte loads and reads the fragments back with gfx950's transposing LDS read
//                 (ds_read_b64_tr_b16: two per 16-feature tile instead of eight 2-byte reads);
//                 B = the probabilities the lane
//                 already holds, each as the sum of two bf16 numbers (two MFMAs).
// The wavefronts' results are merged through LDS, in wavefront order; a launch without key ranges
// (nsplit == 1) normalises and writes the output rows, one with key ranges leaves (m, l, O) in
// `partial` for attn_merge_kernel exactly as attn_kernel does.  Every row's arithmetic is
// independent of the other rows.  MODE: causal self-attention over the paged cache, the same with
// the relative-position bias, or cross-attention (the fixed encoder keys, no mask, no bias).
// The bias of (head, key - position) comes from a table the host lays out by distance
// (bias_by_key: [head][max_len + 3], entry max_len - 1 - distance, zero-padded), so the four
// consecutive keys a lane scores per 16-key tile are one 16-byte read, asked for with the step's
// K and V rows: no tables in LDS, no barrier before the loop.
// Memory latency: the rows' positions, the first step's page entries and the queries leave
// together; the K and V rows follow as soon as the positions (hence the context length) are
// known; page entries of later steps are asked for a step ahead.  No page table in LDS.
// (Computing a key's address without the table when a sequence's pages lie in order, and loading
// the first step's rows before the context length is known - clamped to the cache's extent, rows
// past the context zeroed on their way through LDS - was tried: 0.3 us faster at 120 keys, 0.3 us
// slower at 60, where two of four wavefronts then pull never-written rows from cold memory.)
// grid = (kv heads, sequences, row groups or key ranges).
// dynamic LDS: max(NW x 32 x (d_head + 8) bf16 staging, NW x RG x (d_head + 2) floats for the merge).
__device__ __forceinline__ bf16x8 ld_frag(const bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ bf16x8 zero_frag() {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  return __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
}
// D[m][n] += sum_k A[m][k] B[n][k]: lane (lane % 16, lane / 16) holds A[m][8 kq .. 8 kq + 8) and the
// same of B; element r of the result is D[4 (lane / 16) + r][lane % 16]
__device__ __forceinline__ f32x4 mma_bf16(const bf16x8& a, const bf16x8& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
constexpr float ATTN_MMA_SLACK = 6.0f;       // how far scores may outgrow the softmax reference point before it moves
constexpr size_t attn_mma_lds_bytes(int rg, int dh, int nw) {
  const size_t stage = (size_t)nw * 32 * (dh + 8) * 2, merge = (size_t)nw * rg * (dh + 2) * 4;
  return stage > merge ? stage : merge;
}

constexpr int ATTN_SELF = 0, ATTN_SELF_BIAS = 1, ATTN_CROSS = 2, ATTN_CROSS_PROJ = 3;
// ATTN_CROSS_PROJ (d_head 64, one row tile, one query head per kv head, K <= 512): cross-attention of a
// small model whose query projection is done here instead of in a launch of its own.  A head's 64
// query features are 4 tiles x K/32 k-steps of weights, 64 KB at K = 512: the wavefronts fetch them
// with the first keys and values, multiply them exactly as gemm_kernel would -- four K-slices per
// tile, chunks of four k-steps with the k-steps past a slice masked, the slices' partial tiles added
// in order, the row's 1/rms from the partial sums of squares in gemm_kernel's order, rounding to
// bf16 -- and hand the rows to the score product through LDS.  Bit-identical to the two launches.
constexpr int ATTN_PJ_S = 4, ATTN_PJ_U = 4;            // gemm_kernel's wavefronts and chunk at K <= 512
constexpr size_t attn_mma_proj_lds_bytes(int rg, int nw) {
  const size_t base = attn_mma_lds_bytes(rg, 64, nw), part = (size_t)4 * ATTN_PJ_S * 256 * 4;
  return ((base > part ? base : part) + 15) / 16 * 16 + 16 * 64 * 2;
}
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // four floats at any 4-byte boundary

template <int DH, int NRT, int NW, int MODE>
// (four wavefronts: capped at 128 registers so that two workgroups share a CU, which the long
// contexts' key ranges need: one workgroup per CU took two rounds there)
static __global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_mma_kernel(const AttnArgs a) {
  extern __shared__ float lds[];
  constexpr bool PROJ = MODE == ATTN_CROSS_PROJ;
  constexpr bool CROSS = MODE == ATTN_CROSS || PROJ, BIAS = MODE == ATTN_SELF_BIAS, TABLE = !CROSS;   // TABLE: paged keys
  constexpr int KSQ = DH / 32;                     // k-steps of the score product
  constexpr int DT = DH / 16;                      // 16-feature tiles of the output
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, kq = lane >> 4;
  const int hkv = blockIdx.x;
  const int seq = blockIdx.y;
  // z: the key ranges of a launch that has them (it has one row group), else the row groups
  const int split = (a.nsplit > 1) ? (int)blockIdx.z : 0;
  const int rs = (a.nsplit > 1) ? 0 : (int)blockIdx.z * a.rows_per_wg;
  const int R = min(a.rows_per_wg, a.R - rs);
  const int r0 = seq * a.R + rs;
  const int G = a.G, RG = R * G;
  const int* page_table = TABLE ? a.page_table + (size_t)(a.seq0 + seq) * a.pt_stride : nullptr;
  const int page_shift = __ffs(a.page_size) - 1, page_mask = a.page_size - 1;
  const int last_page = a.n_pages - 1;
  const int k_begin = split * a.split_keys;
  const int kb0 = k_begin + wave * 32;

  // ---- positions, the first step's page entries, the queries: one round of loads ----
  int my_pos = -1;                                  // lane r: the causal limit of row r
  if (!CROSS && lane < R) my_pos = a.row_pos[r0 + lane];
  int pg[2] = {0, 0};                               // TABLE: pages of keys kb .. kb + 15 and kb + 16 .. kb + 31 of the step to load
  auto ask_pages = [&](int kb, int (&out)[2]) {
    if (!TABLE) return;
    out[0] = page_table[min(kb >> page_shift, last_page)];
    out[1] = page_table[min((kb + 16) >> page_shift, last_page)];
  };
  ask_pages(kb0, pg);
  // ---- PROJ: the loads of the query projection leave first ----
  constexpr int PJ_PER_WAVE = PROJ ? (DH / 16) * ATTN_PJ_S / NW : 1;      // (tile, K-slice) units per wavefront
  bf16x8 pj_w[PJ_PER_WAVE][ATTN_PJ_U], pj_b[PJ_PER_WAVE][ATTN_PJ_U];
  float pj_ss[16];
  const int pj_KS = PROJ ? a.pj_K >> 5 : 0, pj_kpw = (pj_KS + ATTN_PJ_S - 1) / ATTN_PJ_S;
  if (PROJ) {
    const bf16* W = static_cast<const bf16*>(a.pj_w);
    const bf16* xb = static_cast<const bf16*>(a.pj_x) + (size_t)(r0 + min(j, R - 1)) * a.pj_K + kq * 8;
#pragma unroll
    for (int i = 0; i < PJ_PER_WAVE; ++i) {
      const int u = wave + NW * i, tile = hkv * (DH / 16) + (u >> 2), w = u & 3;
      const int ks0 = min(pj_KS, w * pj_kpw), ks1 = min(pj_KS, ks0 + pj_kpw), ks_last = max(ks1 - 1, 0);
#pragma unroll
      for (int uu = 0; uu < ATTN_PJ_U; ++uu) {
        const int ksc = min(ks0 + uu, ks_last);
        pj_w[i][uu] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(W + ((size_t)tile * pj_KS + ksc) * 512 + lane * 8));
        pj_b[i][uu] = ld_frag(xb + ksc * 32);
      }
    }
    if (tid < 256) {                                // thread (row, f) of the projection's epilogue: partials f, f + 16, ..
      const int rowc = r0 + min(tid >> 4, R - 1), f = tid & 15;
#pragma unroll
      for (int u = 0; u < 16; ++u) pj_ss[u] = a.pj_ss[min(f + 16 * u, a.pj_npart - 1) * 16 + rowc];
    }
  }
  // query rows of this lane: rg = rt * 16 + j; features (4 s + kq) * 8 .. + 8 in k-step s
  bf16x8 qf[NRT][KSQ];
  int pos[NRT], gq[NRT];
  const float* brow[NRT];                           // BIAS: this lane's head in bias_by_key
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int rg = rt * 16 + j;
    const bool ok = rg < RG;
    const int rgc = ok ? rg : 0;
    const int rr = (rgc * a.g_mul) >> 16;           // rgc / G
    gq[rt] = rgc - rr * G;
    pos[rt] = ok ? (CROSS ? 0x7fffffff : a.row_pos[r0 + rr]) : -1;
    brow[rt] = BIAS ? a.bias_by_key + (size_t)(hkv * G + gq[rt]) * (a.bias_off + 4) : nullptr;
    const bf16* qp = static_cast<const bf16*>(a.q) + (size_t)(r0 + rr) * a.H * DH + (size_t)(hkv * G + gq[rt]) * DH + kq * 8;
#pragma unroll
    for (int s = 0; s < KSQ; ++s) qf[rt][s] = (ok && !PROJ) ? ld_frag(qp + s * 32) : zero_frag();
  }
  auto row_ptr = [&](int key, int page, int which) -> const bf16* {   // which: 0 = K, 1 = V
    if (CROSS) return static_cast<const bf16*>(which ? a.cv : a.ck) + ((size_t)hkv * a.kv_len + key) * DH;
    return static_cast<const bf16*>(a.kv_pool) + ((((size_t)page * 2 + which) * a.Hkv + hkv) * a.page_size + (key & page_mask)) * DH;
  };
  // The loads of a step are issued one step ahead, into the registers the previous step has
  // just finished with (V after its transposition at the top of the step, K after the score
  // product), so a wavefront's load latency overlaps a whole step of its own arithmetic.
  bf16x8 kf[2][KSQ];
  bf16x8 vr[DH / 16];
  constexpr int VKPL = 64 / (DH / 8);               // keys one V load of the wavefront covers
  const int vpiece = lane % (DH / 8), vkey = lane / (DH / 8);
  int kv_len = a.kv_len;
  int pg_last = 0;                                  // TABLE: page of the last key, what loads past the range re-read
  // TABLE: a step's 32 keys start at a multiple of 32 and pages hold a multiple of 16 keys, so keys
  // 0..15 of the step are consecutive slots of one page and keys 16..31 of one page: two page
  // entries per step.  (Past the range kb is clamped and every lane re-reads the last key itself.)
  auto halves = [&](int kb, int which, const bf16* (&half)[2], int& nk) {
    const bool in = kb < kv_len;
    const int kc = in ? kb : max(kv_len - 1, 0);
    nk = max(min(32, kv_len - kc), 1);
    const bool in1 = kb + 16 < kv_len;
    half[0] = row_ptr(kc, in ? pg[0] : pg_last, which);
    half[1] = row_ptr(in1 ? kb + 16 : max(kv_len - 1, 0), in1 ? pg[1] : pg_last, which);
  };
  auto load_k = [&](int kb) {
    const bf16* half[2] = {nullptr, nullptr}; int nk = 0;
    if (TABLE) halves(kb, 0, half, nk);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const bf16* kp;
      if (TABLE) {
        const int kk = min(kt * 16 + j, nk - 1);
        kp = ((kk < 16) ? half[0] + kk * DH : half[1] + (kk - 16) * DH) + kq * 8;
      } else {
        kp = row_ptr(min(kb + kt * 16 + j, a.kv_len - 1), 0, 0) + kq * 8;
      }
#pragma unroll
      for (int s = 0; s < KSQ; ++s) kf[kt][s] = ld_frag(kp + s * 32);      // the four quarters read 64 contiguous bytes
    }
  };
  auto load_v = [&](int kb) {                       // load c: VKPL keys, each row read by DH/8 consecutive lanes
    const bf16* half[2] = {nullptr, nullptr}; int nk = 0;
    if (TABLE) halves(kb, 1, half, nk);
#pragma unroll
    for (int c = 0; c < DH / 16; ++c) {
      if (TABLE) {
        const int kk = min(c * VKPL + vkey, nk - 1);
        vr[c] = ld_frag(((kk < 16) ? half[0] + kk * DH : half[1] + (kk - 16) * DH) + vpiece * 8);
      } else {
        vr[c] = ld_frag(row_ptr(min(kb + c * VKPL + vkey, a.kv_len - 1), 0, 1) + vpiece * 8);
      }
    }
  };
  int pos_min = 0x7fffffff;                         // a step whose keys all lie at or below it needs no mask
  if (!CROSS) {
    kv_len = wave_max(my_pos) + 1;
    pos_min = wave_min(lane < R ? my_pos : 0x7fffffff);
  }
  float* pp = a.partial + ((((size_t)seq * a.Hkv + hkv) * a.nsplit + split) * ATTN_MAX_RG + (size_t)rs * G) * (DH + 2);
  if (a.nsplit > 1) {
    if (k_begin >= kv_len) {                        // nothing in this key range yet: an empty partial
      if (tid < RG) { pp[(size_t)tid * (DH + 2) + DH] = -INFINITY; pp[(size_t)tid * (DH + 2) + DH + 1] = 0.0f; }
      return;
    }
    kv_len = min(kv_len, k_begin + a.split_keys);
  }
  if (TABLE) pg_last = page_table[min(max(kv_len - 1, 0) >> page_shift, last_page)];

  float m_run[NRT], l_run[NRT];
  f32x4 o[DT][NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    m_run[rt] = -INFINITY; l_run[rt] = 0.0f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // V tile of the step, row-major with padded rows: [32 keys][DH + 8] bf16 (rows stay 8-byte aligned,
  // which the transposing reads of a fragment need).
  constexpr int VRS = DH + 8;
  unsigned short* vt = reinterpret_cast<unsigned short*>(lds) + (size_t)wave * 32 * VRS;
  // bias of this lane's keys kb + kt*16 + kq*4 + 0..3 for row rt: table entries (key - pos) + bias_off ..,
  // clamped where every one of them is masked anyway (key > pos)
  f32x4 bz[2][NRT];
  auto load_bias = [&](int kb) {
    if (!BIAS) return;
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        const int i0 = min(kb + kt * 16 + kq * 4 - pos[rt] + a.bias_off, a.bias_off);
        bz[kt][rt] = *reinterpret_cast<const f32x4_a4*>(brow[rt] + i0);
      }
  };
  if (kb0 < kv_len) { load_k(kb0); load_v(kb0); }   // a wavefront without keys loads nothing
  if (kb0 < kv_len) load_bias(kb0);
  ask_pages(kb0 + NW * 32, pg);
  if (PROJ) {
    // ---- the projection itself, while the first keys and values are on their way ----
    float* pj_part = lds;                            // [4 tiles][4 slices][256]; the staging region is not in use yet
    unsigned short* pj_q = reinterpret_cast<unsigned short*>(lds + a.pj_q_off);     // [16 rows][DH] bf16
#pragma unroll
    for (int i = 0; i < PJ_PER_WAVE; ++i) {
      const int u = wave + NW * i, w = u & 3;
      const int ks0 = min(pj_KS, w * pj_kpw), ks1 = min(pj_KS, ks0 + pj_kpw);
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int uu = 0; uu < ATTN_PJ_U; ++uu) {
        const bool valid = (ks0 + uu < ks1) && (j < R);
        acc = mma_bf16(pj_w[i][uu], valid ? pj_b[i][uu] : zero_frag(), acc);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) pj_part[u * 256 + j * 16 + kq * 4 + r] = acc[r];     // u = tile * 4 + slice
    }
    __syncthreads();
    if (tid < 256) {
      const int row = tid >> 4, f = tid & 15;
      float q = 0.0f;
#pragma unroll
      for (int u = 0; u < 16; ++u) q += (f + 16 * u < a.pj_npart) ? pj_ss[u] : 0.0f;
      q = lane_combine<1>(q, OpSumF()); q = lane_combine<2>(q, OpSumF());
      q = lane_combine<4>(q, OpSumF()); q = lane_combine<8>(q, OpSumF());
      q = row_first(q);
      const float rs_row = 1.0f / sqrtf(q / (float)a.pj_K + a.pj_eps);
#pragma unroll
      for (int t = 0; t < DH / 16; ++t) {
        float y = 0.0f;
#pragma unroll
        for (int w = 0; w < ATTN_PJ_S; ++w) y += pj_part[(t * ATTN_PJ_S + w) * 256 + tid];
        y *= rs_row;
        y += 0.0f;                                   // (gemm_kernel adds its absent bias as zero)
        const bf16 yb = (bf16)y;
        pj_q[row * DH + t * 16 + f] = __builtin_bit_cast(unsigned short, yb);
      }
    }
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      const int rg = rt * 16 + j;                    // (one query head per kv head: row group = row)
#pragma unroll
      for (int s = 0; s < KSQ; ++s)
        qf[rt][s] = (rg < RG) ? *reinterpret_cast<const bf16x8*>(pj_q + rg * DH + s * 32 + kq * 8) : zero_frag();
    }
    // (pj_part was last read before the barrier above, so the staging region is free; pj_q lies beyond
    // everything the rest of the kernel writes)
  }

  for (int kb = kb0; kb < kv_len; kb += NW * 32) {
    const int nkeys = min(32, kv_len - kb);
    const int kb_next = kb + NW * 32;
    int pgn[2] = {0, 0};
    ask_pages(kb_next + NW * 32, pgn);
    // ---- V tile -> LDS, transposed; then its registers take the next step's tile ----
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");     // the reads of the previous step are done
#pragma unroll
    for (int c = 0; c < DH / 16; ++c) *reinterpret_cast<bf16x8*>(vt + (c * VKPL + vkey) * VRS + vpiece * 8) = vr[c];
    load_v(kb_next);                                 // no branch around loads: the compiler would wait for all of them
    // ---- scores: sc[kt][rt][r] = S[key kb + kt*16 + kq*4 + r][row rt*16 + j] ----
    f32x4 sc[2][NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        sc[kt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KSQ; ++s) sc[kt][rt] = mma_bf16(kf[kt][s], qf[rt][s], sc[kt][rt]);
      }
    load_k(kb_next);
    pg[0] = pgn[0]; pg[1] = pgn[1];
    f32x4 bias[2][NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) bias[kt][rt] = BIAS ? bz[kt][rt] : f32x4{0.f, 0.f, 0.f, 0.f};
    load_bias(kb_next);                              // (its index clamp keeps reads past the range in bounds)
    float p[2][NRT][4];
    float f[NRT];
    bool rescale = false;
    const bool all_visible = nkeys == 32 && kb + 31 <= pos_min;     // uniform
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      float mx = -INFINITY;
      if (all_visible) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            p[kt][rt][r] = a.scale * sc[kt][rt][r];
            if (BIAS) p[kt][rt][r] += bias[kt][rt][r];
            mx = fmaxf(mx, p[kt][rt][r]);
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int kl = kt * 16 + kq * 4 + r;
            const bool ok = kl < nkeys && kb + kl <= pos[rt];
            float v = a.scale * sc[kt][rt][r];
            if (BIAS) v += bias[kt][rt][r];
            p[kt][rt][r] = ok ? v : -INFINITY;
            mx = fmaxf(mx, p[kt][rt][r]);
          }
      }
      mx = lane_combine<16>(mx, OpMaxF());
      mx = lane_combine<32>(mx, OpMaxF());
      // the reference point m_run only moves when the scores outgrow it by more than
      // ATTN_MMA_SLACK: probabilities stay below e^slack, and most steps need no rescaling
      const float m_new = (mx > m_run[rt] + ATTN_MMA_SLACK || m_run[rt] == -INFINITY) ? fmaxf(m_run[rt], mx) : m_run[rt];
      f[rt] = (m_new == m_run[rt]) ? 1.0f : ((m_run[rt] == -INFINITY) ? 0.0f : __expf(m_run[rt] - m_new));
      rescale = rescale || (f[rt] != 1.0f);
      float sum = 0.0f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float e = (p[kt][rt][r] == -INFINITY) ? 0.0f : __expf(p[kt][rt][r] - m_new);
          p[kt][rt][r] = e;
          sum += e;
        }
      l_run[rt] = l_run[rt] * f[rt] + sum;          // this lane's keys only; the quarters are added at the end
      m_run[rt] = m_new;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");     // this step's V tile has landed in LDS
    // ---- O^T = f O^T + V^T P;  p as the sum of two bf16 numbers (16 mantissa bits): the
    //      matrix cores have time to spare ----
    bf16x8 pf[NRT], pl[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = p[e >> 2][rt][e & 3];
        pf[rt][e] = (bf16)v;
        pl[rt][e] = (bf16)(v - (float)pf[rt][e]);
      }
    if (__builtin_amdgcn_ballot_w64(rescale) != 0ull) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
          for (int r = 0; r < 4; ++r) o[dt][rt][r] *= f[rt];
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      // vf[e] = V[key (e/4) 16 + 4 kq + e%4][feature dt 16 + j]: two transposing LDS reads.  In each
      // block of 16 lanes, lane s hands in the address of four consecutive 16-bit elements D[s][0..3]
      // and lane i gets back D[i/4 + 4 e][i%4], e = 0..3; with lane s pointing at
      // V[key0 + s/4][dt 16 + 4 (s%4) ..], lane j receives keys key0 .. key0 + 3 of feature dt 16 + j.
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const unsigned short* vp = vt + (kq * 4 + (j >> 2)) * VRS + dt * 16 + 4 * (j & 3);
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)vp);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 16 * VRS));
      const s16x8 vb = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8 vf = __builtin_bit_cast(bf16x8, vb);
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        o[dt][rt] = mma_bf16(vf, pl[rt], o[dt][rt]);
        o[dt][rt] = mma_bf16(vf, pf[rt], o[dt][rt]);
      }
    }
  }

  // ---- merge the wavefronts: each leaves (m, l, O) of its keys in LDS ----
  __syncthreads();                                  // staging region no longer in use
  float* mg = lds + (size_t)wave * RG * (DH + 2);
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    float l = lane_combine<16>(l_run[rt], OpSumF());
    l = lane_combine<32>(l, OpSumF());
    const int rg = rt * 16 + j;
    if (rg < RG) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) mg[(size_t)rg * (DH + 2) + dt * 16 + kq * 4 + r] = o[dt][rt][r];
      if (kq == 0) { mg[(size_t)rg * (DH + 2) + DH] = m_run[rt]; mg[(size_t)rg * (DH + 2) + DH + 1] = l; }
    }
  }
  __syncthreads();
  if (a.nsplit > 1) {
    for (int i = tid; i < RG * (DH + 2); i += 64 * NW) {
      const int rg = i / (DH + 2), d = i % (DH + 2);
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < NW; ++w) m = fmaxf(m, lds[((size_t)w * RG + rg) * (DH + 2) + DH]);
      float out = m;                                   // d == DH: the maximum itself
      if (d != DH) {
        out = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {                 // wavefronts in order; d == DH + 1 sums the denominators
          const float mw = lds[((size_t)w * RG + rg) * (DH + 2) + DH];
          if (mw != -INFINITY) out += lds[((size_t)w * RG + rg) * (DH + 2) + d] * __expf(mw - m);
        }
      }
      pp[i] = out;
    }
    return;
  }
  bf16* og = static_cast<bf16*>(a.out);
  for (int i = tid; i < RG * DH; i += 64 * NW) {
    const int rg = i / DH, d = i % DH;
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) m = fmaxf(m, lds[((size_t)w * RG + rg) * (DH + 2) + DH]);
    float L = 0.0f, acc = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {                     // wavefronts in order
      const float* row = lds + ((size_t)w * RG + rg) * (DH + 2);
      const float mw = row[DH];
      if (mw != -INFINITY) {
        const float e = __expf(mw - m);
        L += row[DH + 1] * e;
        acc += row[d] * e;
      }
    }
    const int rr = (rg * a.g_mul) >> 16, gg = rg - rr * G;
    og[(size_t)(r0 + rr) * a.H * DH + (size_t)(hkv * G + gg) * DH + d] = (bf16)((L > 0.0f) ? acc / L : 0.0f);
  }
}

// Combines the partial results of the key ranges of one (sequence, kv head): with
// m = max m_s, the output is sum_s acc_s e^(m_s - m) / sum_s l_s e^(m_s - m), ranges taken in
// order.  grid = (kv heads, rows x query heads of the kv head, sequences), one thread per feature.
template <typename T, int DH>
static __global__ __launch_bounds__(DH) void attn_merge_kernel(const AttnArgs a) {
  const int hkv = blockIdx.x, G = a.H / a.Hkv, rg = blockIdx.y, d = threadIdx.x;
  const int r_base = (int)blockIdx.z * a.R;
  const float* pp = a.partial + ((((size_t)blockIdx.z * a.Hkv + hkv) * a.nsplit) * ATTN_MAX_RG + rg) * (DH + 2);
  const size_t stride = (size_t)ATTN_MAX_RG * (DH + 2);
  float m = -INFINITY;
  for (int sp = 0; sp < a.nsplit; ++sp) m = fmaxf(m, pp[sp * stride + DH]);
  float L = 0.0f, o = 0.0f;
  for (int sp = 0; sp < a.nsplit; ++sp) {
    const float* q = pp + sp * stride;
    const float ms = q[DH];
    if (ms != -INFINITY) {                         // empty ranges left no output behind
      const float w = __expf(ms - m);
      L += q[DH + 1] * w;
      o += q[d] * w;
    }
  }
  const int r = rg / G, h = hkv * G + rg % G;
  const float res = (L > 0.0f) ? o / L : 0.0f;
  if (a.out_frag != nullptr) {
    const int row = r_base + r, n = h * DH + d;
    Store<T>::st(static_cast<T*>(a.out_frag) + ((((size_t)(n >> 5) * GEMM_WIDE_RT + (row >> 4)) * 64 + (row & 15) + 16 * ((n & 31) >> 3)) * 8 + (n & 7)), res);
  } else {
    Store<T>::st(static_cast<T*>(a.out) + (size_t)(r_base + r) * a.H * DH + h * DH + d, res);
  }
}

}  // namespace sd
