// Host side of the speculative-decoding library: workspace layout, weight
// loading / re-tiling, and the launch sequences of prefill, one run of
// Algorithm 1 (sd_step) and one plain decoding step (sd_step_baseline).
// The C ABI is declared and documented in include/sd.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <functional>
#include <map>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/sd.h"
#include "kernels_attn.h"
#include "kernels_gemm.h"
#include "kernels_misc.h"
#include "kernels_sample.h"

namespace {

using namespace sd;

thread_local std::string g_load_error;
static_assert(sd::ATTN_MAX_RG == SD_ATTN_MAX_ROWS_X_GROUP, "sd.h states the attention kernels' row limit");
int g_num_cus = 256;                 // compute units of the device, read at load

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Bump allocator over the caller's workspace; with base == nullptr it only sizes.
struct Arena {
  char* base;
  size_t off = 0;
  explicit Arena(void* b) : base(static_cast<char*>(b)) {}
  void* take(size_t bytes) {
    off = align_up(off);
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

struct LayerW {
  void *ln1g = nullptr, *ln1b = nullptr, *wqkv = nullptr, *bqkv = nullptr, *wo = nullptr, *bo = nullptr;
  void *lncg = nullptr, *cq = nullptr, *ck = nullptr, *cv = nullptr, *co = nullptr;
  void *ln2g = nullptr, *ln2b = nullptr, *w1 = nullptr, *wu = nullptr, *b1 = nullptr, *w2 = nullptr, *b2 = nullptr;
  void* kv = nullptr;                       // [page][2][Hkv][PS][dh]
  void *cross_k = nullptr, *cross_v = nullptr;   // [H][enc_len][dh]
};

struct Model {
  sd_model_cfg cfg{};
  size_t esz = 4;
  int nq = 0, nkv = 0, n_pages = 0, page_size = 0;
  void *tok_emb = nullptr, *pos_emb = nullptr, *head = nullptr, *lnfg = nullptr, *lnfb = nullptr, *rel_bias = nullptr;
  int* bucket_lut = nullptr;
  float* bias_by_key = nullptr; // T5DEC: rel_bias by causal distance, [n_heads][max_len + 3] (attn_mma_kernel)
  float* rope = nullptr;
  std::vector<LayerW> L;
  int batch = 1;               // sequences; each owns n_pages pages of every layer's pool
  int rows_cap = MAX_ROWS;     // activation rows: one group of MAX_ROWS rows per sequence at most
  int* page_table = nullptr;   // [batch][n_pages]
  bool pages_in_order = true;  // sequence b's table is b * n_pages + 0, 1, 2, ...; false (SD_FLAG_SCATTER_PAGES): back to front
  int *row_seq = nullptr, *logit_row = nullptr;   // [rows_cap], written by the embedding kernel
  void* xfrag = nullptr;       // activations of one wide GEMM in fragment order
  float* wide_partial = nullptr;   // partial tiles of the K chunks of one split GEMM
  float* wide_rs = nullptr;        // 1 / rms of the rows of one split GEMM
  void* xfrag2 = nullptr;          // a batched kernel's output that the next product reads, in fragment order
  int attn_nsplit = 1, attn_split_keys = 0;   // long contexts: key ranges per (sequence, kv head)
  float* attn_partial = nullptr;
  float* x = nullptr;
  void* xg = nullptr;          // x * gain of the next RMSNorm, storage type
  float* ss = nullptr;         // [d_model/16][16] partial sums of x^2
  void *qbuf = nullptr, *attn = nullptr, *ffn = nullptr;
  int* row_pos = nullptr;
  int* prompt = nullptr;
};

bool cfg_ok(const sd_model_cfg& c, std::string& why) {
  auto bad = [&](const char* m) { why = m; return false; };
  if (c.arch < 0 || c.arch > 2) return bad("unknown arch");
  if (c.dtype != SD_F32 && c.dtype != SD_BF16) return bad("unknown dtype");
  if (c.n_layers < 1 || c.d_model < 32 || c.n_heads < 1 || c.n_kv_heads < 1 || c.d_ff < 32 ||
      c.vocab < 16 || c.max_len < 2)
    return bad("non-positive size");
  if (c.d_head != 32 && c.d_head != 64 && c.d_head != 128) return bad("d_head must be 32, 64 or 128");
  if (c.n_heads % c.n_kv_heads) return bad("n_heads must be a multiple of n_kv_heads");
  if (c.arch != SD_ARCH_GQA && c.n_heads != c.n_kv_heads) return bad("grouped KV heads need SD_ARCH_GQA");
  if (c.n_heads / c.n_kv_heads > 4) return bad("at most 4 query heads per KV head");
  if (c.d_model % 32 || c.d_ff % 32 || (c.n_heads * c.d_head) % 32) return bad("dims must be multiples of 32");
  if (c.vocab % 16) return bad("vocab must be a multiple of 16");
  if (c.vocab > SAMPLE_CHUNK * SAMPLE_MAX_CHUNKS) return bad("vocab too large");
  if (c.arch == SD_ARCH_T5DEC && (c.enc_len < 1 || c.rel_buckets < 2 || c.rel_buckets % 2 ||
                                  c.rel_max_dist <= c.rel_buckets / 2))
    return bad("T5DEC needs enc_len, rel_buckets, rel_max_dist");
  if (c.arch == SD_ARCH_T5DEC && c.rel_buckets > 64) return bad("at most 64 relative-position buckets");
  if (c.arch == SD_ARCH_T5DEC && c.max_len > ATTN_LDS_DIST - 64) return bad("max_len too large for the relative-position table");
  if (c.arch != SD_ARCH_T5DEC && c.enc_len != 0) return bad("enc_len only for T5DEC");
  if (!(c.norm_eps > 0.0f)) return bad("norm_eps must be positive");
  return true;
}

// Lays a model out in the arena (or sizes it).
void plan_model(Arena& A, Model& m, const sd_model_cfg& c, int page_size, int batch) {
  m.cfg = c;
  m.batch = batch;
  m.rows_cap = MAX_ROWS * batch;
  m.esz = (c.dtype == SD_BF16) ? 2 : 4;
  const size_t e = m.esz, d = c.d_model, ff = c.d_ff, V = c.vocab;
  m.nq = c.n_heads * c.d_head;
  m.nkv = c.n_kv_heads * c.d_head;
  m.page_size = page_size;
  m.n_pages = (c.max_len + page_size - 1) / page_size;
  m.tok_emb = A.take(V * d * e);
  m.head = A.take(V * d * e);
  m.lnfg = A.take(d * e);
  if (c.arch == SD_ARCH_GPT) { m.lnfb = A.take(d * e); m.pos_emb = A.take((size_t)c.max_len * d * e); }
  if (c.arch == SD_ARCH_T5DEC) {
    m.rel_bias = A.take((size_t)c.n_heads * c.rel_buckets * e);
    m.bucket_lut = static_cast<int*>(A.take((size_t)c.max_len * sizeof(int)));
    m.bias_by_key = static_cast<float*>(A.take((size_t)c.n_heads * (c.max_len + 3) * sizeof(float)));
  }
  if (c.arch == SD_ARCH_GQA) m.rope = static_cast<float*>(A.take((size_t)c.max_len * c.d_head * sizeof(float)));
  m.L.assign(c.n_layers, LayerW());
  for (auto& l : m.L) {
    l.ln1g = A.take(d * e); l.ln2g = A.take(d * e);
    l.wqkv = A.take((size_t)(m.nq + 2 * m.nkv) * d * e);
    l.wo = A.take(d * m.nq * e);
    l.w2 = A.take(d * ff * e);
    if (c.arch == SD_ARCH_GPT) {
      l.ln1b = A.take(d * e); l.ln2b = A.take(d * e);
      l.bqkv = A.take((size_t)(m.nq + 2 * m.nkv) * e);
      l.bo = A.take(d * e); l.b1 = A.take(ff * e); l.b2 = A.take(d * e);
      l.w1 = A.take(ff * d * e);
    } else {
      l.w1 = A.take(ff * d * e);            // gate
      l.wu = A.take(ff * d * e);
    }
    if (c.arch == SD_ARCH_T5DEC) {
      l.lncg = A.take(d * e);
      l.cq = A.take(m.nq * d * e); l.ck = A.take(m.nq * d * e); l.cv = A.take(m.nq * d * e);
      l.co = A.take(d * m.nq * e);
      l.cross_k = A.take((size_t)c.enc_len * m.nq * e);
      l.cross_v = A.take((size_t)c.enc_len * m.nq * e);
    }
    l.kv = A.take((size_t)batch * m.n_pages * 2 * c.n_kv_heads * page_size * c.d_head * e);
  }
  const size_t rows = (size_t)m.rows_cap;
  m.page_table = static_cast<int*>(A.take((size_t)batch * m.n_pages * sizeof(int)));
  m.x = static_cast<float*>(A.take(rows * d * sizeof(float)));
  m.xg = A.take(rows * d * e);
  m.ss = static_cast<float*>(A.take((size_t)batch * (d / 16) * 16 * sizeof(float)));   // [group][d/16][16]
  m.qbuf = A.take(rows * m.nq * e);
  m.attn = A.take(rows * m.nq * e);
  m.ffn = A.take(rows * ff * e);
  m.row_pos = static_cast<int*>(A.take(rows * sizeof(int)));
  m.row_seq = static_cast<int*>(A.take(rows * sizeof(int)));
  m.logit_row = static_cast<int*>(A.take(rows * sizeof(int)));
  // contexts beyond 1024 positions: key ranges of 512 keys taken by different workgroups
  m.attn_split_keys = 512;
  m.attn_nsplit = (c.max_len > 1024) ? std::min(16, (c.max_len + m.attn_split_keys - 1) / m.attn_split_keys) : 1;
  if (m.attn_nsplit > 1) {
    m.attn_split_keys = ((c.max_len + m.attn_nsplit - 1) / m.attn_nsplit + 511) / 512 * 512;
    m.attn_partial = static_cast<float*>(A.take((size_t)batch * c.n_kv_heads * m.attn_nsplit * ATTN_MAX_RG *
                                                (c.d_head + 2) * sizeof(float)));
  }
  if (batch > 1) {
    m.xfrag = A.take((size_t)std::max({(size_t)d, (size_t)m.nq, ff}) * GEMM_WIDE_RT * 16 * e);
    const size_t tiles = std::max((size_t)d, (size_t)(m.nq + 2 * m.nkv)) / 16;    // the products split_ok() lets through
    m.wide_partial = static_cast<float*>(A.take((size_t)8 * GEMM_WIDE_RT * tiles * 256 * sizeof(float)));
    m.wide_rs = static_cast<float*>(A.take((size_t)GEMM_WIDE_RT * 16 * sizeof(float)));
    m.xfrag2 = A.take((size_t)std::max({(size_t)d, (size_t)m.nq, ff}) * GEMM_WIDE_RT * 16 * e);
  }
  m.prompt = static_cast<int*>(A.take((size_t)c.max_len * sizeof(int)));
}

}  // namespace

struct sd_ctx {
  Model p, q;
  sd_runtime_cfg rt{};
  hipStream_t stream = nullptr;
  bool own_stream = false;
  SeqState* d_state = nullptr;
  StepParams* d_params = nullptr;
  float *p_logits = nullptr, *q_logits = nullptr;
  RowStat* d_stats = nullptr;
  unsigned int* d_counter = nullptr;
  double* d_draw_tot = nullptr;          // sample_row_split_kernel: chunk totals [batch][SAMPLE_MAX_CHUNKS]
  unsigned int* d_draw_ticket = nullptr; // and its tickets, SAMPLE_COUNTER_STRIDE words per sequence
  SeqState* h_state = nullptr;       // pinned
  StepParams* h_params = nullptr;    // pinned
  int batch = 1;
  // host mirror of the sequences
  // per sequence: prefilled?  Mq cache behind the committed tokens (after plain decoding steps or
  // steps whose drafts did not come from Mq; only that sequence's prefill brings it back)?
  std::vector<int> len, last_tok, ready, mq_stale;
  bool all_ready() const { for (int r : ready) if (!r) return false; return true; }
  bool any_stale() const { for (int m : mq_stale) if (m) return true; return false; }
  int last_gamma = 0, last_kind = -1;   // for sd_debug_logits
  hipGraphExec_t graphs[SD_MAX_GAMMA + 1] = {};
  hipGraphExec_t graph_baseline = nullptr;
  hipEvent_t ev[4] = {};
  std::vector<hipEvent_t> kev;       // 2 per Mp layer: around the gated FFN-in GEMM (SD_FLAG_PROFILE)
  bool time_ffn = false;             // set while the verify forward of a profiled step is enqueued
  int skip_ops = 0;                  // sd_time_forward: SD_OP_* launches left out of the forward being recorded
  sd_stats stats{};
  sd_sampling sampling{1.0f, 0, 0.0f};
  // negligible-cost draft: logits table in place of Mq's forward (caller-owned device memory)
  const float* draft_table = nullptr;
  const int* draft_row_of = nullptr;
  int draft_rows = 0;
  // copying draft: the committed tokens of every sequence, [batch][hist_stride], kept on the
  // device while copy_match > 0; hist_len = how many of them the device holds
  int* d_hist = nullptr;
  int hist_stride = 0, copy_match = 0;
  std::vector<int> hist_len;
  bool no_mq() const { return draft_table != nullptr || copy_match > 0; }
  // acceptance statistics for the choice of gamma: they describe the pair and the task, not one
  // sequence, so sd_reset leaves them alone
  int64_t tune_accepted = 0, tune_tested = 0, tune_beta_count = 0;
  double tune_beta_sum = 0.0;
  std::string err;
};

namespace {

void plan_ctx(Arena& A, sd_ctx& c, const sd_model_cfg& pc, const sd_model_cfg& qc, const sd_runtime_cfg& rt) {
  const size_t B = (size_t)rt.batch;
  c.batch = rt.batch;
  plan_model(A, c.p, pc, rt.page_size, rt.batch);
  plan_model(A, c.q, qc, rt.page_size, rt.batch);
  c.d_state = static_cast<SeqState*>(A.take(B * sizeof(SeqState)));
  c.d_params = static_cast<StepParams*>(A.take(B * sizeof(StepParams)));
  c.p_logits = static_cast<float*>(A.take(B * (rt.max_gamma + 1) * pc.vocab * sizeof(float)));   // [seq][gamma+1][V]
  c.q_logits = static_cast<float*>(A.take(B * rt.max_gamma * pc.vocab * sizeof(float)));         // [seq][gamma][V]
  c.d_stats = static_cast<RowStat*>(A.take(B * (2 * SD_MAX_GAMMA + 1) * sizeof(RowStat)));
  c.d_counter = static_cast<unsigned int*>(A.take(B * SAMPLE_COUNTER_STRIDE * sizeof(unsigned int)));
  c.d_draw_tot = static_cast<double*>(A.take(B * SAMPLE_MAX_CHUNKS * sizeof(double)));
  c.d_draw_ticket = static_cast<unsigned int*>(A.take(B * SAMPLE_COUNTER_STRIDE * sizeof(unsigned int)));
  c.hist_stride = pc.max_len;
  c.d_hist = static_cast<int*>(A.take(B * (size_t)pc.max_len * sizeof(int)));
}

bool rt_ok(const sd_runtime_cfg& rt, std::string& why) {
  if (rt.batch < 1 || rt.batch > SD_MAX_BATCH) { why = "batch out of range"; return false; }
  if (rt.max_gamma < 1 || rt.max_gamma > SD_MAX_GAMMA) { why = "max_gamma out of range"; return false; }
  if (rt.page_size < 16 || (rt.page_size & (rt.page_size - 1))) { why = "page_size must be a power of two >= 16"; return false; }
  return true;
}

sd_status fail(sd_ctx* c, sd_status s, const std::string& msg) {
  if (c) c->err = msg; else g_load_error = msg;
  return s;
}

#define HIP_TRY(ctx, expr)                                                              \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      return fail(ctx, SD_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_));     \
  } while (0)

// ------------------------------------------------------------------ launches
// Wavefronts per workgroup (they split K): 8 when each still gets a full chunk of
// k-steps, else 4.  Depends on K only, so a row's reduction order never changes.
int pick_waves(int ksteps) { return (ksteps >= 8 * GEMM_UNROLL) ? 8 : 4; }

template <typename T, int PRO, int EPI>
void launch_gemm_t(hipStream_t s, GemmArgs a) {
  const int tiles = a.N / 16, KS = a.K / 32;
  const int S = pick_waves(KS);
  a.ksteps_per_wave = (KS + S - 1) / S;
  const int ND = (EPI == EPI_GATED) ? 2 : 1;
  const size_t lds = (size_t)(2 * S * ND * 256 + S * 16 + 256 + (PRO == PRO_POST ? GEMM_PART_STAGE * 16 : 0)) * sizeof(float);
  // one resident workgroup of 8 wavefronts per CU (more only when they are smaller), each
  // taking the same number of tiles
  const int capacity = g_num_cus * std::max(1, 8 / S);
  const int per_wg = (tiles + capacity - 1) / capacity;
  const int grid = (tiles + per_wg - 1) / per_wg;
  if (a.ksteps_per_wave <= GEMM_UNROLL_SHORT)
    hipLaunchKernelGGL((gemm_kernel<T, PRO, EPI, GEMM_UNROLL_SHORT>), dim3(grid), dim3(64 * S), lds, s, a);
  else
    hipLaunchKernelGGL((gemm_kernel<T, PRO, EPI, GEMM_UNROLL>), dim3(grid), dim3(64 * S), lds, s, a);
}

// Several 16-row slabs in one launch (a.nrt of them, set by the caller).
template <typename T, int PRO, int EPI>
void launch_gemm_wide_t(hipStream_t s, GemmArgs a) {
  const int tiles = a.N / 16, KS = a.K / 32;
  const int S = pick_waves(KS);                  // the same K split as the one-slab kernel: same sums
  a.ksteps_per_wave = (KS + S - 1) / S;
  const size_t lds = gemm_wide_lds_bytes(S);
  // work items are pairs of weight streams (gate + up of a tile, else two neighbouring tiles);
  // one resident workgroup per CU (the partial tiles of six slabs take most of its LDS)
  const int pairs = (EPI == EPI_GATED) ? tiles : (tiles + 1) / 2;
  const int per_wg = (pairs + g_num_cus - 1) / g_num_cus;
  const int grid = (pairs + per_wg - 1) / per_wg;
  hipLaunchKernelGGL((gemm_wide_kernel<T, PRO, EPI>), dim3(grid), dim3(64 * S), lds, s, a);
}

// Split design: K chunks over workgroups (the one-slab kernel's chunks), then the finish kernel.
template <typename T, int PRO, int EPI>
void launch_gemm_split_t(hipStream_t s, GemmArgs a, float* partial) {
  const int tiles = a.N / 16, KS = a.K / 32;
  const int S = pick_waves(KS);                  // the same K split as the one-slab kernel: same sums
  a.ksteps_per_wave = (KS + S - 1) / S;
  a.nchunk = S;
  a.partial = partial;
  constexpr int NS = (EPI == EPI_GATED) ? 2 : 1;
  const size_t lds = (size_t)SplitShape<T>::SUB * a.nrt * 64 * 8 * sizeof(T);
  // 8 tiles per workgroup, 12 when 8 would need a second round of workgroups and 12 does not
  const bool wide12 = ((tiles + 7) / 8) * S > g_num_cus && ((tiles + 11) / 12) * S <= g_num_cus;
  if (wide12) hipLaunchKernelGGL((gemm_split_kernel<T, NS, 12>), dim3((tiles + 11) / 12, S), dim3(768), lds, s, a);
  else hipLaunchKernelGGL((gemm_split_kernel<T, NS, 8>), dim3((tiles + 7) / 8, S), dim3(512), lds, s, a);
  hipLaunchKernelGGL((gemm_split_finish_kernel<T, PRO, EPI>), dim3(tiles, a.nrt), dim3(256), 0, s, a);
}

// Gated FFN-in over several slabs: no split over workgroups, every wavefront walks all of K.
template <typename T, int EPI>
void launch_gemm_gated_wide(hipStream_t s, GemmArgs a) {
  const int tiles = (EPI == EPI_GATED) ? a.N / 16 : (a.N / 16 + 1) / 2, KS = a.K / 32;
  const int S = pick_waves(KS);                  // the chunks whose sums the one-slab kernel adds
  a.ksteps_per_wave = (KS + S - 1) / S;
  a.nchunk = S;
  const dim3 grid((tiles + GEMM_GATED_NW - 1) / GEMM_GATED_NW), block(64 * GEMM_GATED_NW);
  const size_t lds = gemm_gated_lds_bytes<T>(a.nrt);       // at most 48 KB: within the default limit
  static_assert(gemm_gated_lds_bytes<T>(GEMM_WIDE_RT) <= 64 * 1024, "gated wide kernel: dynamic LDS");
  switch (a.nrt) {                                         // the slab count is a template parameter of the kernel
#define SD_NRT(N_) case N_: hipLaunchKernelGGL((gemm_gated_wide_kernel<T, EPI, N_>), grid, block, lds, s, a); break
    SD_NRT(1); SD_NRT(2); SD_NRT(3); SD_NRT(4); SD_NRT(5); SD_NRT(6);
#undef SD_NRT
    default: break;                                        // (callers pass 1 .. GEMM_WIDE_RT)
  }
}

// Which products take the split design (activations in fragment order, RMSNorm or no norm).
inline bool split_ok(int pro, int epi) {
  // (a gated FFN's partial tiles are too many: 8 chunks x 2 streams x d_ff; it stays with gemm_wide_kernel)
  return (pro == PRO_POST && epi == EPI_QKV) || (pro == PRO_NONE && epi == EPI_RESID);
}

template <typename T>
void launch_gemm_split(hipStream_t s, int pro, int epi, const GemmArgs& a, float* partial) {
#define SD_CASE(P, E) if (pro == P && epi == E) return launch_gemm_split_t<T, P, E>(s, a, partial)
  SD_CASE(PRO_POST, EPI_QKV); SD_CASE(PRO_NONE, EPI_RESID);     // (split_ok() admits no others)
#undef SD_CASE
}

// The wide kernel's LDS exceeds the default 64 KB limit of dynamic LDS.
template <typename T>
hipError_t allow_wide_lds() {
  hipError_t e = hipSuccess;
#define SD_CASE(P, E)                                                                                          \
  if (e == hipSuccess)                                                                                         \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_wide_kernel<T, P, E>),                         \
                            hipFuncAttributeMaxDynamicSharedMemorySize,                                       \
                            (int)gemm_wide_lds_bytes(8))
  SD_CASE(PRO_LN, EPI_QKV); SD_CASE(PRO_POST, EPI_QKV);
  SD_CASE(PRO_NONE, EPI_RESID);
  SD_CASE(PRO_LN, EPI_ACT); SD_CASE(PRO_POST, EPI_GATED);
  SD_CASE(PRO_LN, EPI_LOGITS); SD_CASE(PRO_POST, EPI_LOGITS);
#undef SD_CASE
  return e;
}

template <typename T>
void launch_gemm_wide(hipStream_t s, int pro, int epi, const GemmArgs& a) {
#define SD_CASE(P, E) if (pro == P && epi == E) return launch_gemm_wide_t<T, P, E>(s, a)
  SD_CASE(PRO_LN, EPI_QKV); SD_CASE(PRO_POST, EPI_QKV);
  SD_CASE(PRO_NONE, EPI_RESID);
  SD_CASE(PRO_LN, EPI_ACT); SD_CASE(PRO_POST, EPI_GATED);
  SD_CASE(PRO_LN, EPI_LOGITS); SD_CASE(PRO_POST, EPI_LOGITS);
#undef SD_CASE
}

template <typename T>
void launch_gemm(hipStream_t s, int pro, int epi, const GemmArgs& a) {
#define SD_CASE(P, E) if (pro == P && epi == E) return launch_gemm_t<T, P, E>(s, a)
  SD_CASE(PRO_LN, EPI_QKV); SD_CASE(PRO_POST, EPI_QKV);
  SD_CASE(PRO_NONE, EPI_RESID); SD_CASE(PRO_NONE, EPI_STORE); SD_CASE(PRO_POST, EPI_STORE);
  SD_CASE(PRO_LN, EPI_ACT); SD_CASE(PRO_POST, EPI_GATED);
  SD_CASE(PRO_LN, EPI_LOGITS); SD_CASE(PRO_POST, EPI_LOGITS);
#undef SD_CASE
}

size_t attn_lds_bytes(int RG, int DH, int threads) {
  return (size_t)(RG * DH + RG * attn_block_keys(DH, threads) + (threads / 64) * attn_rows_per_pass(DH) * DH +
                  3 * RG + RG * DH) * sizeof(float);
}

// Threads per workgroup of attn_kernel: the smallest size whose key block covers `keys`.
int attn_threads(int DH, int keys) {
  for (int t : {256, 512})
    if (attn_block_keys(DH, t) >= keys) return t;
  return 1024;
}

template <typename T, int DH>
void launch_attn_kernel(hipStream_t s, const AttnArgs& a, dim3 grid, int threads, size_t lds) {
#define SD_ATTN(TH)                                                                                  \
  if (threads == TH) {                                                                               \
    if (a.cross) hipLaunchKernelGGL((attn_kernel<T, DH, TH, true>), grid, dim3(TH), lds, s, a);      \
    else hipLaunchKernelGGL((attn_kernel<T, DH, TH, false>), grid, dim3(TH), lds, s, a);             \
    return;                                                                                          \
  }
  SD_ATTN(256) SD_ATTN(512) SD_ATTN(1024)
#undef SD_ATTN
}

// The matrix-core kernel: four wavefronts per workgroup, eight when the expected context is more than
// eight 32-key steps (measured at 512 encoder keys: 6.5 us against 6.8 with four and 7.7 with sixteen).
int attn_mma_waves(int keys) { return (keys + 31) / 32 > 8 ? 8 : 4; }
template <int DH, int NRT>
void launch_attn_mma(hipStream_t s, const AttnArgs& a, dim3 grid, int nw, size_t lds) {
  const int mode = a.cross ? (a.pj_w != nullptr ? ATTN_CROSS_PROJ : ATTN_CROSS) : (a.bias_by_key != nullptr ? ATTN_SELF_BIAS : ATTN_SELF);
  if constexpr (DH == 64 && NRT == 1) {
    if (mode == ATTN_CROSS_PROJ) {
      if (nw == 4) hipLaunchKernelGGL((attn_mma_kernel<64, 1, 4, ATTN_CROSS_PROJ>), grid, dim3(256), lds, s, a);
      else hipLaunchKernelGGL((attn_mma_kernel<64, 1, 8, ATTN_CROSS_PROJ>), grid, dim3(512), lds, s, a);
      return;
    }
  }
#define SD_MMA(NW_, MODE_)                                                                                \
  if (nw == NW_ && mode == MODE_) {                                                                       \
    hipLaunchKernelGGL((attn_mma_kernel<DH, NRT, NW_, MODE_>), grid, dim3(64 * NW_), lds, s, a);          \
    return;                                                                                               \
  }
  SD_MMA(4, ATTN_SELF) SD_MMA(4, ATTN_SELF_BIAS) SD_MMA(4, ATTN_CROSS)
  SD_MMA(8, ATTN_SELF) SD_MMA(8, ATTN_SELF_BIAS) SD_MMA(8, ATTN_CROSS)
#undef SD_MMA
}

template <typename T>
void launch_attn(hipStream_t s, const Model& m, AttnArgs a, int nseq) {
  const int G = a.H / a.Hkv, DH = m.cfg.d_head;
  a.G = G; a.g_mul = 65536 / G + 1;
  // few kv heads leave most CUs idle: split the (independent) rows over more workgroups
  a.rows_per_wg = (nseq * a.Hkv * ((a.R + 1) / 2) <= g_num_cus) ? std::min(2, a.R) : a.R;
  if (a.cross || m.attn_nsplit <= 1) { a.nsplit = 1; a.split_keys = 0; a.partial = nullptr; }
  else { a.nsplit = m.attn_nsplit; a.split_keys = m.attn_split_keys; a.partial = m.attn_partial; }
  if (a.nsplit > 1) a.rows_per_wg = a.R;          // the key ranges already spread the work
  // The workgroup is sized for the context: all of the encoder's keys in one block for cross-attention,
  // half of max_len for self-attention (a sequence that grows to max_len spends half its life below
  // that; longer contexts take more blocks).  Fixed per model, so every forward of a model, plain or
  // (gamma+1)-row, adds a row's keys in the same order.
  const int threads = a.cross ? attn_threads(DH, a.kv_len) : (a.nsplit > 1 ? 1024 : attn_threads(DH, (m.cfg.max_len + 1) / 2));
  const size_t lds = attn_lds_bytes(a.rows_per_wg * G, DH, threads);
  const dim3 grid(a.Hkv, ((a.R + a.rows_per_wg - 1) / a.rows_per_wg) * a.nsplit, nseq);
  // bf16 with d_head 64 or 128: the matrix-core kernel (key ranges: four wavefronts per range, as
  // the ranges already spread the work)
  if (std::is_same<T, bf16>::value && (DH == 64 || DH == 128)) {
    const int RG = a.rows_per_wg * G;
    const int nw = (a.nsplit > 1) ? 4 : attn_mma_waves(a.cross ? a.kv_len : (m.cfg.max_len + 1) / 2);
    if (a.pj_w != nullptr && !(a.cross && DH == 64 && RG <= 16 && G == 1)) a.pj_w = nullptr;   // (callers check; never project elsewhere)
    size_t ll = attn_mma_lds_bytes(RG, DH, nw);
    if (a.pj_w != nullptr) {
      ll = attn_mma_proj_lds_bytes(RG, nw);
      a.pj_q_off = (int)((ll - 16 * 64 * 2) / 4);
    }
    const dim3 lg(grid.x, grid.z, grid.y);          // key ranges in z, the slowest index: the fullest ranges start first
    if (DH == 64 && RG <= 16) launch_attn_mma<64, 1>(s, a, lg, nw, ll);
    else if (DH == 64) launch_attn_mma<64, 2>(s, a, lg, nw, ll);
    else if (RG <= 16) launch_attn_mma<128, 1>(s, a, lg, nw, ll);
    else launch_attn_mma<128, 2>(s, a, lg, nw, ll);
  } else if (DH == 32) launch_attn_kernel<T, 32>(s, a, grid, threads, lds);
  else if (DH == 64) launch_attn_kernel<T, 64>(s, a, grid, threads, lds);
  else launch_attn_kernel<T, 128>(s, a, grid, threads, lds);
  if (a.nsplit > 1) {
    const dim3 mg(a.Hkv, a.R * G, nseq);
    if (DH == 32) hipLaunchKernelGGL((attn_merge_kernel<T, 32>), mg, dim3(32), 0, s, a);
    else if (DH == 64) hipLaunchKernelGGL((attn_merge_kernel<T, 64>), mg, dim3(64), 0, s, a);
    else hipLaunchKernelGGL((attn_merge_kernel<T, 128>), mg, dim3(128), 0, s, a);
  }
}

// The attention kernel keeps up to ATTN_MAX_RG query rows in more than 64 KB of LDS.
// Each instantiation gets the most it can ask for, ATTN_MAX_RG query rows at its own d_head (the
// reduction buffer [16 wavefronts][rows per pass][d_head] makes d_head 64 the largest).
constexpr size_t ATTN_STATIC_LDS = MAX_ROWS * 4 + 4 * 64 * 4 + ATTN_LDS_DIST;   // the kernel's __shared__ arrays
constexpr size_t LDS_PER_CU = 160 * 1024;
template <typename T, int DH, int TH>
hipError_t allow_attn_lds_t() {
  const size_t bytes = attn_lds_bytes(ATTN_MAX_RG, DH, TH);
  if (bytes + ATTN_STATIC_LDS > LDS_PER_CU) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<T, DH, TH, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<T, DH, TH, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  return e;
}
template <typename T, int DH>
hipError_t allow_attn_lds() {
  hipError_t e = allow_attn_lds_t<T, DH, 256>();
  if (e == hipSuccess) e = allow_attn_lds_t<T, DH, 512>();
  if (e == hipSuccess) e = allow_attn_lds_t<T, DH, 1024>();
  return e;
}
// The matrix-core kernel with eight wavefronts, 24 query rows and d_head 128 merges through 100 KB of LDS.
template <int DH, int NRT, int NW, int MODE>
hipError_t allow_mma_lds() {
  const size_t bytes = attn_mma_lds_bytes(NRT == 1 ? 16 : ATTN_MAX_RG, DH, NW);
  static_assert(attn_mma_lds_bytes(ATTN_MAX_RG, 128, 8) <= LDS_PER_CU, "matrix-core attention: LDS budget");
  if (bytes <= 64 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mma_kernel<DH, NRT, NW, MODE>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}
template <int DH, int NRT, int NW>
hipError_t allow_mma_lds_modes() {
  hipError_t e = allow_mma_lds<DH, NRT, NW, ATTN_SELF>();
  if (e == hipSuccess) e = allow_mma_lds<DH, NRT, NW, ATTN_SELF_BIAS>();
  if (e == hipSuccess) e = allow_mma_lds<DH, NRT, NW, ATTN_CROSS>();
  return e;
}
template <int DH>
hipError_t allow_mma_lds_dh() {
  hipError_t e = allow_mma_lds_modes<DH, 1, 4>();
  if (e == hipSuccess) e = allow_mma_lds_modes<DH, 1, 8>();
  if (e == hipSuccess) e = allow_mma_lds_modes<DH, 2, 4>();
  if (e == hipSuccess) e = allow_mma_lds_modes<DH, 2, 8>();
  return e;
}
template <typename T>
hipError_t allow_big_lds() {
  hipError_t e = allow_attn_lds<T, 32>();
  if (e == hipSuccess) e = allow_attn_lds<T, 64>();
  if (e == hipSuccess) e = allow_attn_lds<T, 128>();
  if (e == hipSuccess) e = allow_mma_lds_dh<64>();
  if (e == hipSuccess) e = allow_mma_lds_dh<128>();
  return e;
}

// Rows one prefill pass may carry so that rows x (query heads per kv head) fits the attention kernel.
int prefill_rows(const sd_model_cfg& c) { return std::min(MAX_ROWS, ATTN_MAX_RG / (c.n_heads / c.n_kv_heads)); }

// Which rows a forward processes: sequences seq0 .. seq0+nseq-1 with rps rows each, chosen
// by (mode, step) from the device-resident sequence states (ROWS_PREFILL: rps prompt tokens
// of sequence seq0 from position start).  gamma fixes where the LM-head rows land in the
// logits buffers ([seq][gamma+1][V] for Mp, [seq][gamma][V] for Mq).
struct Rows { int mode, step, rps, start, seq0, nseq, gamma; };

// One forward of model m; with `logits` the LM head runs on every row and each row's
// output goes where the embedding kernel's row map says (or nowhere).
// The rows of the sequences lie one after the other (sequence s: rows s * rps ..) and are cut into
// slabs ("groups") of MAX_ROWS rows for the GEMMs; a sequence may straddle two slabs, which no
// kernel minds: every row carries its own position, sequence and output row.
template <typename T>
void forward(sd_ctx* c, Model& m, const Rows& rw, float* logits) {
  hipStream_t s = c->stream;
  const sd_model_cfg& f = m.cfg;
  const int d = f.d_model;
  const size_t e = m.esz;
  const bool rms = (f.arch != SD_ARCH_GPT);
  const int pro = rms ? PRO_POST : PRO_LN;
  const int n_layers = (int)m.L.size();
  const int skip = c->skip_ops;                     // measurement only (sd_time_forward); 0 in every decoding call
  const int rows_total = rw.nseq * rw.rps;
  const int n_groups = (rows_total + MAX_ROWS - 1) / MAX_ROWS;
  struct Grp { int R; float* x; char* xg; float* ss; char *qbuf, *attn, *ffn; int *row_pos, *row_seq, *logit_row; };
  auto group = [&](int g) {
    Grp q;
    q.R = std::min(MAX_ROWS, rows_total - g * MAX_ROWS);
    const size_t off = (size_t)g * MAX_ROWS;
    q.x = m.x + off * d;
    q.xg = static_cast<char*>(m.xg) + off * d * e;
    q.ss = m.ss + (size_t)g * (d / 16) * 16;
    q.qbuf = static_cast<char*>(m.qbuf) + off * m.nq * e;
    q.attn = static_cast<char*>(m.attn) + off * m.nq * e;
    q.ffn = static_cast<char*>(m.ffn) + off * f.d_ff * e;
    q.row_pos = m.row_pos + off; q.row_seq = m.row_seq + off; q.logit_row = m.logit_row + off;
    return q;
  };
  {
    const Grp q = group(0);                         // one launch: the kernel places each row in its slab
    hipLaunchKernelGGL((embed_kernel<T>), dim3(rw.nseq * rw.rps), dim3(256), 0, s, rw.mode, rw.step, c->d_state, m.prompt,
                       rw.start, static_cast<const T*>(m.tok_emb), static_cast<const T*>(m.pos_emb), d, f.vocab, q.x,
                       q.row_pos, static_cast<const T*>(rms ? m.L[0].ln1g : nullptr),
                       reinterpret_cast<T*>(rms ? q.xg : nullptr), rms ? q.ss : nullptr,
                       rw.rps, rw.seq0, rw.gamma, q.row_seq, q.logit_row, (d / 16) * 16);
  }
  // One GEMM over every group: groups are 16-row slabs one after the other in all row-indexed
  // buffers, so up to GEMM_WIDE_RT of them go into one launch of the wide kernel (weights
  // streamed once for all of them); a single group takes the one-slab kernel.
  const int R_full = MAX_ROWS, R_tail = rows_total - (n_groups - 1) * MAX_ROWS;
  // frag_in: the producer left this product's activations in fragment order already (one launch only)
  const void* frag_in = nullptr;
  bool out_frag_next = false, produced_frag = false;   // ask the gated kernel for fragment-order output / it complied
  auto gemm_groups = [&](int pro_, int epi_, const std::function<void(GemmArgs&, const Grp&)>& fill) {
    if (n_groups == 1) {
      GemmArgs a{};
      fill(a, group(0));
      launch_gemm<T>(s, pro_, epi_, a);
      return;
    }
    for (int g0 = 0; g0 < n_groups; g0 += GEMM_WIDE_RT) {
      GemmArgs a{};
      fill(a, group(g0));
      a.nrt = std::min(GEMM_WIDE_RT, n_groups - g0);
      a.R = R_full;
      a.R_last = (g0 + a.nrt == n_groups) ? R_tail : R_full;
      a.ss_stride = (d / 16) * 16;
      if (frag_in != nullptr && pro_ == PRO_NONE && n_groups <= GEMM_WIDE_RT) {
        a.X = frag_in;
      } else if (pro_ != PRO_LN) {                // the wide kernel reads the activations in fragment order
        const int frags = (a.K / 32) * a.nrt;
        const int blocks = (frags * 64 + 255) / 256;
        const bool want_rs = pro_ == PRO_POST && (split_ok(pro_, epi_) || epi_ == EPI_GATED || epi_ == EPI_LOGITS) && blocks >= 2 * a.nrt;
        hipLaunchKernelGGL((rows_to_fragments_kernel<T>), dim3(blocks), dim3(256), 0, s,
                           static_cast<const T*>(a.X), static_cast<T*>(m.xfrag), a.nrt, a.K, a.ss_in, a.n_part,
                           a.ss_stride, a.eps, want_rs ? m.wide_rs : nullptr);
        a.X = m.xfrag;
        a.rs_in = want_rs ? m.wide_rs : nullptr;
      }
      if (pro_ == PRO_POST && epi_ == EPI_GATED && a.rs_in != nullptr) {
        if (out_frag_next && n_groups <= GEMM_WIDE_RT) { a.out_frag = m.xfrag2; produced_frag = true; }
        launch_gemm_gated_wide<T, EPI_GATED>(s, a);
      } else if (pro_ == PRO_POST && epi_ == EPI_LOGITS && a.rs_in != nullptr) {
        launch_gemm_gated_wide<T, EPI_LOGITS>(s, a);
      }
      else if (split_ok(pro_, epi_) && (pro_ != PRO_POST || a.rs_in != nullptr)) launch_gemm_split<T>(s, pro_, epi_, a, m.wide_partial);
      else launch_gemm_wide<T>(s, pro_, epi_, a);
    }
  };
  int n_part = 1;                                   // partial sums of x^2 the next norm has to add
  // input of a normed GEMM: LayerNorm reads the fp32 rows, RMSNorm the pre-scaled rows + partials
  auto normed = [&](GemmArgs& a, const Grp& q, const void* gain, const void* beta) {
    a.R = q.R;
    a.eps = f.norm_eps;
    if (rms) { a.X = q.xg; a.ss_in = q.ss; a.n_part = n_part; }
    else { a.X = q.x; a.gain = gain; a.beta = beta; }
  };
  // residual add that also prepares the input of the next norm
  auto resid = [&](const void* W, bool from_ffn, const void* bias, int K, const void* gain_next) {
    gemm_groups(PRO_NONE, EPI_RESID, [&](GemmArgs& o, const Grp& q) {
      o.R = q.R; o.W = W; o.X = from_ffn ? q.ffn : q.attn; o.bias = bias; o.K = K; o.N = d; o.out = q.x; o.ldo = d;
      if (rms) { o.xg_out = q.xg; o.gain_next = gain_next; o.ss_out = q.ss; }
    });
    n_part = d / 16;
  };
  for (int li = 0; li < n_layers; ++li) {
    const LayerW& l = m.L[li];
    // q, k, v projections (+ rotary) with k, v appended to the cache
    if (!(skip & SD_OP_QKV)) gemm_groups(pro, EPI_QKV, [&](GemmArgs& a, const Grp& q) {
      normed(a, q, l.ln1g, l.ln1b);
      a.W = l.wqkv; a.bias = l.bqkv; a.K = d; a.N = m.nq + 2 * m.nkv;
      a.q_out = q.qbuf; a.nq = m.nq; a.nkv = m.nkv; a.kv_pool = l.kv; a.page_table = m.page_table;
      a.page_size = m.page_size; a.n_kv_heads = f.n_kv_heads; a.d_head = f.d_head; a.row_pos = q.row_pos;
      a.rope = m.rope;
      if (m.batch > 1) { a.row_seq = q.row_seq; a.pt_stride = m.n_pages; }
    });
    // Small models: the cross-attention kernel computes its own queries (ATTN_CROSS_PROJ), one launch
    // less per layer.  The conditions are the kernel's: bf16, heads of 64, one query head per kv head,
    // one slab of rows, K = d_model <= 512 (gemm_kernel then runs four wavefronts with chunks of four
    // k-steps, which the kernel reproduces).
    const bool fuse_cross_q = f.arch == SD_ARCH_T5DEC && std::is_same<T, bf16>::value && f.d_head == 64 &&
                              f.n_heads == f.n_kv_heads && n_groups == 1 && d <= 512 && d % 32 == 0 &&
                              !(c->rt.flags & SD_FLAG_SEPARATE_CROSS_Q);
    auto attention = [&](bool cross) {
      {
        const Grp q = group(0);                     // one launch over all sequences (grid.z)
        AttnArgs a{};
        a.q = q.qbuf; a.out = q.attn; a.kv_pool = l.kv; a.page_table = m.page_table; a.page_size = m.page_size; a.n_pages = m.n_pages;
        a.row_pos = q.row_pos; a.R = rw.rps; a.H = f.n_heads; a.Hkv = f.n_kv_heads; a.cross = 0; a.kv_len = 0;
        a.scale = (f.arch == SD_ARCH_T5DEC) ? 1.0f : 1.0f / sqrtf((float)f.d_head);
        a.rel_bias = m.rel_bias; a.bucket_lut = m.bucket_lut; a.rel_buckets = f.rel_buckets;
        a.bias_by_key = m.bias_by_key; a.bias_off = f.max_len - 1;
        a.seq0 = rw.seq0; a.pt_stride = m.n_pages;
        if (cross) { a.cross = 1; a.ck = l.cross_k; a.cv = l.cross_v; a.kv_len = f.enc_len; a.scale = 1.0f; a.rel_bias = nullptr; a.bias_by_key = nullptr; }
        if (cross && fuse_cross_q && !(skip & SD_OP_CROSS_Q)) {
          a.pj_w = l.cq; a.pj_x = q.xg; a.pj_ss = q.ss; a.pj_K = d; a.pj_npart = n_part; a.pj_eps = f.norm_eps;
        }
        // long contexts end in the merge kernel, which can leave its output in fragment order for
        // the batched O projection (no re-tile)
        if (!cross && m.attn_nsplit > 1 && n_groups > 1 && n_groups <= GEMM_WIDE_RT) { a.out_frag = m.xfrag2; produced_frag = true; }
        launch_attn<T>(s, m, a, rw.nseq);
      }
    };
    if (!(skip & SD_OP_ATTN)) attention(false);
    frag_in = produced_frag ? m.xfrag2 : nullptr;
    produced_frag = false;
    if (!(skip & SD_OP_O)) resid(l.wo, false, l.bo, m.nq, (f.arch == SD_ARCH_T5DEC) ? l.lncg : l.ln2g);
    else n_part = d / 16;
    frag_in = nullptr;
    if (f.arch == SD_ARCH_T5DEC) {
      for (int g = 0; g < n_groups && !(skip & SD_OP_CROSS_Q) && !fuse_cross_q; ++g) {
        const Grp q = group(g);
        GemmArgs cq{};
        normed(cq, q, l.lncg, nullptr);
        cq.W = l.cq; cq.K = d; cq.N = m.nq; cq.out = q.qbuf; cq.ldo = m.nq;
        launch_gemm<T>(s, PRO_POST, EPI_STORE, cq);
      }
      if (!(skip & SD_OP_CROSS_ATTN)) attention(true);
      if (!(skip & SD_OP_CROSS_O)) resid(l.co, false, nullptr, m.nq, l.ln2g);
    }
    {
      const bool gpt = (f.arch == SD_ARCH_GPT);
      const bool timed = !gpt && c->time_ffn && &m == &c->p && 2 * li + 1 < (int)c->kev.size();
      if (timed) hipEventRecord(c->kev[2 * li], s);
      out_frag_next = true;                        // the FFN-out product reads fragments: skip its re-tile
      if (!(skip & SD_OP_FFN_IN)) gemm_groups(gpt ? PRO_LN : PRO_POST, gpt ? EPI_ACT : EPI_GATED, [&](GemmArgs& h, const Grp& q) {
        normed(h, q, l.ln2g, l.ln2b);
        h.K = d; h.N = f.d_ff; h.out = q.ffn; h.ldo = f.d_ff; h.W = l.w1;
        if (gpt) h.bias = l.b1;
        else { h.W2 = l.wu; h.act = (f.arch == SD_ARCH_T5DEC) ? ACT_GELU : ACT_SILU; }
      });
      if (timed) hipEventRecord(c->kev[2 * li + 1], s);
    }
    out_frag_next = false;
    frag_in = produced_frag ? m.xfrag2 : nullptr;
    produced_frag = false;
    if (!(skip & SD_OP_FFN_OUT)) resid(l.w2, true, l.b2, f.d_ff, (li + 1 < n_layers) ? m.L[li + 1].ln1g : m.lnfg);
    else n_part = d / 16;
    frag_in = nullptr;
  }
  if (logits != nullptr && !(skip & SD_OP_HEAD)) {
    gemm_groups(pro, EPI_LOGITS, [&](GemmArgs& a, const Grp& q) {
      normed(a, q, m.lnfg, m.lnfb);
      a.W = m.head; a.K = d; a.N = f.vocab; a.out = logits; a.ldo = f.vocab; a.scale = f.logit_scale;
      a.out_row = q.logit_row;
    });
  }
}

void forward_any(sd_ctx* c, Model& m, const Rows& rw, float* logits) {
  if (m.cfg.dtype == SD_BF16) forward<bf16>(c, m, rw, logits);
  else forward<float>(c, m, rw, logits);
}

// Cross-attention keys / values of every layer from the encoder output.
template <typename T>
void cross_kv(sd_ctx* c, Model& m, const void* enc) {
  const sd_model_cfg& f = m.cfg;
  for (const LayerW& l : m.L)
    for (int which = 0; which < 2; ++which)
      for (int r0 = 0; r0 < f.enc_len; r0 += MAX_ROWS) {
        GemmArgs g{};
        g.R = std::min(MAX_ROWS, f.enc_len - r0);
        g.W = which ? l.cv : l.ck;
        g.X = static_cast<const char*>(enc) + (size_t)r0 * f.d_model * m.esz;
        g.K = f.d_model; g.N = m.nq;
        g.out = which ? l.cross_v : l.cross_k;       // [head][enc_len][d_head]: one contiguous block per head
        g.hm_rows = f.enc_len; g.hm_row0 = r0; g.d_head = f.d_head;
        launch_gemm<T>(c->stream, PRO_NONE, EPI_STORE, g);
      }
}

// One draw per sequence from the row at logits + b * seq_stride (mode 0: guess number `slot`; 1: commit).
void launch_draw(sd_ctx* c, const float* logits, int uniform_idx, int mode, int slot, size_t seq_stride) {
  hipLaunchKernelGGL(sample_row_split_kernel, dim3(SAMPLE_SPLIT, c->batch), dim3(SAMPLE_THREADS), 0, c->stream, logits,
                     c->p.cfg.vocab, c->d_params, uniform_idx, c->d_state, mode, slot, seq_stride, c->d_draw_tot, c->d_draw_ticket);
}

// The launch sequence of one run of Algorithm 1 for every sequence (everything between the
// upload of the step parameters and the download of the states).
void enqueue_step(sd_ctx* c, int gamma, bool profile) {
  hipStream_t s = c->stream;
  const int V = c->p.cfg.vocab, B = c->batch;
  if (profile) hipEventRecord(c->ev[0], s);
  for (int i = 0; i < gamma; ++i) {              // q_i <- Mq(prefix + x_<i), x_i ~ q_i
    if (c->copy_match > 0)                       // copied from the context, else the table / uniform
      hipLaunchKernelGGL(copy_row_kernel, dim3(std::min(32, (V + 255) / 256), B), dim3(256), 0, s, c->d_hist, c->hist_stride,
                         c->copy_match, c->draft_table, c->draft_row_of, c->draft_rows, V, c->d_state, i,
                         c->q_logits + (size_t)i * V, (size_t)gamma * V);
    else if (c->draft_table)                     // table lookup instead of a forward
      hipLaunchKernelGGL(table_row_kernel, dim3(std::min(32, (V + 255) / 256), B), dim3(256), 0, s, c->draft_table,
                         c->draft_row_of, c->draft_rows, V, c->d_state, i, c->q_logits + (size_t)i * V, (size_t)gamma * V);
    else if (i == 0) forward_any(c, c->q, Rows{ROWS_DRAFT_FIRST, 0, 2, 0, 0, B, gamma}, c->q_logits);
    else forward_any(c, c->q, Rows{ROWS_DRAFT_NEXT, i, 1, 0, 0, B, gamma}, c->q_logits);
    launch_draw(c, c->q_logits + (size_t)i * V, i, 0, i, (size_t)gamma * V);
  }
  if (profile) hipEventRecord(c->ev[1], s);
  // p_1..p_{gamma+1} in one forward
  c->time_ffn = profile;
  forward_any(c, c->p, Rows{ROWS_VERIFY, 0, gamma + 1, 0, 0, B, gamma}, c->p_logits);
  c->time_ffn = false;
  if (profile) hipEventRecord(c->ev[2], s);
#define SD_VERIFY(MODE, GRID)                                                                                        \
  hipLaunchKernelGGL(spec_verify_kernel<MODE>, GRID, dim3(SAMPLE_THREADS), 0, s, c->p_logits, c->q_logits,             \
                     (const int*)nullptr, (const float*)nullptr, (const float*)nullptr, gamma, V, 0.0f, 1.0f, 0.0, 0,  \
                     0.0f, c->d_params, c->d_stats, c->d_counter, (int*)nullptr, (int*)nullptr, (float*)nullptr,       \
                     c->d_state)
  if (B * (2 * gamma + 1) <= 64) {              // few tickets: one launch
    SD_VERIFY(0, dim3(2 * gamma + 1, B));
  } else {                                       // many sequences: statistics, then one tail workgroup each
    SD_VERIFY(1, dim3(2 * gamma + 1, B));
    SD_VERIFY(2, dim3(1, B));
  }
  if (c->rt.flags & SD_FLAG_BETA) SD_VERIFY(3, dim3(gamma, B));   // side output: beta_i of every guess, into the states
#undef SD_VERIFY
  if (c->copy_match > 0) hipLaunchKernelGGL(hist_append_kernel, dim3(B), dim3(32), 0, s, c->d_hist, c->hist_stride, c->d_state, 1);
  if (profile) hipEventRecord(c->ev[3], s);
}

void enqueue_baseline(sd_ctx* c) {
  const int V = c->p.cfg.vocab, B = c->batch;
  forward_any(c, c->p, Rows{ROWS_BASELINE, 0, 1, 0, 0, B, 0}, c->p_logits);
  launch_draw(c, c->p_logits, 0, 1, 0, (size_t)V);
  if (c->copy_match > 0) hipLaunchKernelGGL(hist_append_kernel, dim3(B), dim3(32), 0, c->stream, c->d_hist, c->hist_stride, c->d_state, 0);
}

// ------------------------------------------------------------------ loading
struct TensorMap {
  std::map<std::string, const sd_tensor*> m;
  TensorMap(const sd_tensor* t, int n) { for (int i = 0; i < n; ++i) if (t[i].name) m[t[i].name] = &t[i]; }
};

template <typename T>
sd_status put(hipStream_t s, const TensorMap& tm, const Model& m, const std::string& name, void* dst,
              int64_t rows, int64_t cols, bool tiled, std::string& err) {
  auto it = tm.m.find(name);
  if (it == tm.m.end()) { err = "missing tensor " + name; return SD_EINVAL; }
  const sd_tensor* t = it->second;
  const bool shape_ok = (cols == 0) ? (t->ndim == 1 && t->shape[0] == rows)
                                    : (t->ndim == 2 && t->shape[0] == rows && t->shape[1] == cols);
  if (!shape_ok || t->dtype != m.cfg.dtype || t->dev == nullptr) { err = "bad shape / dtype / pointer: " + name; return SD_EINVAL; }
  const size_t n = (size_t)rows * (cols ? cols : 1);
  if (tiled) {
    const size_t groups = n / 8;
    hipLaunchKernelGGL((retile_kernel<T>), dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s,
                       static_cast<const T*>(t->dev), static_cast<T*>(dst), (int)rows, (int)cols);
  } else if (hipMemcpyAsync(dst, t->dev, n * sizeof(T), hipMemcpyDeviceToDevice, s) != hipSuccess) {
    err = "copy failed: " + name; return SD_EHIP;
  }
  return SD_OK;
}

template <typename T>
sd_status load_model(hipStream_t s, Model& m, const sd_tensor* w, int n, std::string& err) {
  const TensorMap tm(w, n);
  const sd_model_cfg& f = m.cfg;
  const int64_t d = f.d_model, ff = f.d_ff, V = f.vocab;
  sd_status st;
#define PUT(name, dst, r, cc, tiled) \
  if ((st = put<T>(s, tm, m, name, dst, r, cc, tiled, err)) != SD_OK) return st
  PUT("tok_emb", m.tok_emb, V, d, false);
  PUT("head", m.head, V, d, true);
  PUT("lnf.g", m.lnfg, d, 0, false);
  if (f.arch == SD_ARCH_GPT) { PUT("lnf.b", m.lnfb, d, 0, false); PUT("pos_emb", m.pos_emb, f.max_len, d, false); }
  if (f.arch == SD_ARCH_T5DEC) PUT("rel_bias", m.rel_bias, f.n_heads, f.rel_buckets, false);
  for (int i = 0; i < f.n_layers; ++i) {
    LayerW& l = m.L[i];
    const std::string p = "l" + std::to_string(i) + ".";
    char* qkv = static_cast<char*>(l.wqkv);
    PUT(p + "ln1.g", l.ln1g, d, 0, false);
    PUT(p + "ln2.g", l.ln2g, d, 0, false);
    PUT(p + "wq", qkv, m.nq, d, true);
    PUT(p + "wk", qkv + (size_t)m.nq * d * m.esz, m.nkv, d, true);
    PUT(p + "wv", qkv + (size_t)(m.nq + m.nkv) * d * m.esz, m.nkv, d, true);
    PUT(p + "wo", l.wo, d, m.nq, true);
    PUT(p + "w2", l.w2, d, ff, true);
    if (f.arch == SD_ARCH_GPT) {
      char* b = static_cast<char*>(l.bqkv);
      PUT(p + "ln1.b", l.ln1b, d, 0, false);
      PUT(p + "ln2.b", l.ln2b, d, 0, false);
      PUT(p + "bq", b, m.nq, 0, false);
      PUT(p + "bk", b + (size_t)m.nq * m.esz, m.nkv, 0, false);
      PUT(p + "bv", b + (size_t)(m.nq + m.nkv) * m.esz, m.nkv, 0, false);
      PUT(p + "bo", l.bo, d, 0, false);
      PUT(p + "w1", l.w1, ff, d, true);
      PUT(p + "b1", l.b1, ff, 0, false);
      PUT(p + "b2", l.b2, d, 0, false);
    } else {
      PUT(p + "wg", l.w1, ff, d, true);
      PUT(p + "wu", l.wu, ff, d, true);
    }
    if (f.arch == SD_ARCH_T5DEC) {
      PUT(p + "lnc.g", l.lncg, d, 0, false);
      PUT(p + "cq", l.cq, m.nq, d, true);
      PUT(p + "ck", l.ck, m.nq, d, true);
      PUT(p + "cv", l.cv, m.nq, d, true);
      PUT(p + "co", l.co, d, m.nq, true);
    }
  }
#undef PUT
  // host-built tables
  // sequence b owns pages b * n_pages .. of every pool: in order, or (m.pages_in_order false) back to front
  std::vector<int> pt((size_t)m.batch * m.n_pages);
  for (int b = 0; b < m.batch; ++b)
    for (int i = 0; i < m.n_pages; ++i)
      pt[(size_t)b * m.n_pages + i] = b * m.n_pages + (m.pages_in_order ? i : m.n_pages - 1 - i);
  if (hipMemcpy(m.page_table, pt.data(), pt.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess) { err = "page table upload"; return SD_EHIP; }
  if (f.arch == SD_ARCH_T5DEC) {
    // causal distance -> bucket: one distance per bucket in the first half,
    // logarithmic spacing up to rel_max_dist in the second, then saturation
    std::vector<int> lut(f.max_len);
    const int half = f.rel_buckets / 2;
    for (int rel = 0; rel < f.max_len; ++rel) {
      int b = rel;
      if (rel >= half) {
        b = half + (int)std::floor(std::log((double)rel / half) / std::log((double)f.rel_max_dist / half) *
                                   (f.rel_buckets - half));
        if (b > f.rel_buckets - 1) b = f.rel_buckets - 1;
      }
      lut[rel] = b;
    }
    if (hipMemcpy(m.bucket_lut, lut.data(), lut.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess) { err = "bucket table upload"; return SD_EHIP; }
    const int row = f.max_len + 3;                  // after rel_bias on the same stream
    hipLaunchKernelGGL((bias_by_key_kernel<T>), dim3((unsigned)((f.n_heads * row + 255) / 256)), dim3(256), 0, s,
                       static_cast<const T*>(m.rel_bias), m.bucket_lut, f.rel_buckets, f.max_len, f.n_heads, m.bias_by_key);
    if (hipGetLastError() != hipSuccess) { err = "bias table"; return SD_EHIP; }
  }
  if (f.arch == SD_ARCH_GQA) {
    std::vector<float> cs((size_t)f.max_len * f.d_head);
    for (int pos = 0; pos < f.max_len; ++pos)
      for (int i = 0; i < f.d_head / 2; ++i) {
        const double ang = (double)pos * std::pow((double)f.rope_theta, -2.0 * i / f.d_head);
        cs[((size_t)pos * (f.d_head / 2) + i) * 2] = (float)std::cos(ang);
        cs[((size_t)pos * (f.d_head / 2) + i) * 2 + 1] = (float)std::sin(ang);
      }
    if (hipMemcpy(m.rope, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) { err = "rope table upload"; return SD_EHIP; }
  }
  return SD_OK;
}

sd_status sync_state_to_host(sd_ctx* c) {
  HIP_TRY(c, hipMemcpyAsync(c->h_state, c->d_state, (size_t)c->batch * sizeof(SeqState), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return SD_OK;
}

// Records what `enqueue` puts on the context's stream into an executable graph.  Whatever fails,
// the stream has left capture mode when this returns and *exec is a valid graph or nullptr.
template <typename F>
sd_status capture_graph(sd_ctx* c, hipGraphExec_t* exec, F&& enqueue) {
  hipGraph_t g = nullptr;
  *exec = nullptr;
  HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
  enqueue();
  hipError_t e = hipStreamEndCapture(c->stream, &g);     // ends the capture also when it reports an error
  if (e == hipSuccess) e = hipGraphInstantiate(exec, g, nullptr, nullptr, 0);
  if (g) hipGraphDestroy(g);
  if (e != hipSuccess) {
    *exec = nullptr;
    (void)hipGetLastError();
    return fail(c, SD_EHIP, std::string("graph capture / instantiate: ") + hipGetErrorString(e));
  }
  return SD_OK;
}

// The device and the host disagree about a sequence after a launch: nothing can be trusted any
// more, so every sequence has to be reset and prefilled before the next step.
sd_status poisoned(sd_ctx* c, const char* what) {
  for (auto& r : c->ready) r = 0;
  return fail(c, SD_EHIP, std::string(what) + ": reset and prefill every sequence");
}

}  // namespace

// ====================================================================== C ABI
extern "C" size_t sd_workspace_bytes(const sd_model_cfg* p_cfg, const sd_model_cfg* q_cfg,
                                     const sd_runtime_cfg* rt) {
  std::string why;
  if (!p_cfg || !q_cfg || !rt || !cfg_ok(*p_cfg, why) || !cfg_ok(*q_cfg, why) || !rt_ok(*rt, why)) return 0;
  if (p_cfg->vocab != q_cfg->vocab) return 0;
  sd_ctx tmp;
  Arena A(nullptr);
  plan_ctx(A, tmp, *p_cfg, *q_cfg, *rt);
  return align_up(A.off);
}

extern "C" sd_status sd_load_models(sd_ctx** out, const sd_model_cfg* p_cfg, const sd_tensor* p_w, int32_t n_p,
                                    const sd_model_cfg* q_cfg, const sd_tensor* q_w, int32_t n_q,
                                    const sd_runtime_cfg* rt) {
  if (!out || !p_cfg || !q_cfg || !rt || !p_w || !q_w || n_p < 1 || n_q < 1) return fail(nullptr, SD_EINVAL, "null argument");
  *out = nullptr;
  std::string why;
  if (!cfg_ok(*p_cfg, why)) return fail(nullptr, SD_EINVAL, "Mp config: " + why);
  if (!cfg_ok(*q_cfg, why)) return fail(nullptr, SD_EINVAL, "Mq config: " + why);
  if (!rt_ok(*rt, why)) return fail(nullptr, SD_EINVAL, "runtime config: " + why);
  if (p_cfg->vocab != q_cfg->vocab) return fail(nullptr, SD_EINVAL, "Mp and Mq must share the vocabulary");
  if (rt->batch > 1 && (p_cfg->arch == SD_ARCH_T5DEC || q_cfg->arch == SD_ARCH_T5DEC))
    return fail(nullptr, SD_EINVAL, "T5DEC models take one sequence (one encoder output per context)");
  if ((rt->max_gamma + 1) * (p_cfg->n_heads / p_cfg->n_kv_heads) > ATTN_MAX_RG ||
      2 * (q_cfg->n_heads / q_cfg->n_kv_heads) > ATTN_MAX_RG)
    return fail(nullptr, SD_EINVAL, "(max_gamma+1) x (query heads per kv head) exceeds the attention kernel's limit");
  if (!rt->workspace || (reinterpret_cast<uintptr_t>(rt->workspace) & 255)) return fail(nullptr, SD_EINVAL, "workspace must be 256-byte aligned");
  const size_t need = sd_workspace_bytes(p_cfg, q_cfg, rt);
  if (rt->workspace_bytes < need) return fail(nullptr, SD_ENOMEM, "workspace too small: need " + std::to_string(need));
  sd_ctx* c = new (std::nothrow) sd_ctx();
  if (!c) return fail(nullptr, SD_ENOMEM, "host allocation failed");
  c->rt = *rt;
  Arena A(rt->workspace);
  plan_ctx(A, *c, *p_cfg, *q_cfg, *rt);
  auto bail = [&](sd_status s, const std::string& m) { sd_free(c); return fail(nullptr, s, m); };
  if (rt->stream) c->stream = static_cast<hipStream_t>(rt->stream);
  else {                       // a stream of the context's own (not the legacy default stream, which cannot be captured)
    if (hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking) != hipSuccess) return bail(SD_EHIP, "stream creation failed");
    c->own_stream = true;
  }
  const size_t B = (size_t)rt->batch;
  c->len.assign(B, 0); c->last_tok.assign(B, -1); c->ready.assign(B, 0); c->hist_len.assign(B, 0); c->mq_stale.assign(B, 0);
  if (hipHostMalloc(reinterpret_cast<void**>(&c->h_state), B * sizeof(SeqState), hipHostMallocDefault) != hipSuccess ||
      hipHostMalloc(reinterpret_cast<void**>(&c->h_params), B * sizeof(StepParams), hipHostMallocDefault) != hipSuccess)
    return bail(SD_EHIP, "pinned allocation failed");
  std::memset(c->h_state, 0, B * sizeof(SeqState));
  std::memset(c->h_params, 0, B * sizeof(StepParams));
  for (auto& e : c->ev) if (hipEventCreate(&e) != hipSuccess) return bail(SD_EHIP, "event creation failed");
  if (p_cfg->arch != SD_ARCH_GPT) {
    c->kev.assign(2 * (size_t)p_cfg->n_layers, nullptr);
    for (auto& e : c->kev) if (hipEventCreate(&e) != hipSuccess) return bail(SD_EHIP, "event creation failed");
  }
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      g_num_cus = cus;
  }
  if (allow_big_lds<bf16>() != hipSuccess || allow_big_lds<float>() != hipSuccess ||
      allow_wide_lds<bf16>() != hipSuccess || allow_wide_lds<float>() != hipSuccess)
    return bail(SD_EHIP, "cannot raise the LDS limit");
  std::string err;
  c->p.pages_in_order = c->q.pages_in_order = (rt->flags & SD_FLAG_SCATTER_PAGES) == 0;
  sd_status st = (p_cfg->dtype == SD_BF16) ? load_model<bf16>(c->stream, c->p, p_w, n_p, err)
                                           : load_model<float>(c->stream, c->p, p_w, n_p, err);
  if (st != SD_OK) return bail(st, "Mp: " + err);
  st = (q_cfg->dtype == SD_BF16) ? load_model<bf16>(c->stream, c->q, q_w, n_q, err)
                                 : load_model<float>(c->stream, c->q, q_w, n_q, err);
  if (st != SD_OK) return bail(st, "Mq: " + err);
  {
    const size_t n = B * SAMPLE_COUNTER_STRIDE;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, c->d_counter, 0u, n);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, c->d_draw_ticket, 0u, n);
  }
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) return bail(SD_EHIP, std::string("load: ") + hipGetErrorString(e));
  *out = c;
  return SD_OK;
}

extern "C" void sd_free(sd_ctx* c) {
  if (!c) return;
  if (c->stream) hipStreamSynchronize(c->stream);
  for (auto& g : c->graphs) if (g) hipGraphExecDestroy(g);
  if (c->graph_baseline) hipGraphExecDestroy(c->graph_baseline);
  for (auto& e : c->ev) if (e) hipEventDestroy(e);
  for (auto& e : c->kev) if (e) hipEventDestroy(e);
  if (c->h_state) hipHostFree(c->h_state);
  if (c->h_params) hipHostFree(c->h_params);
  if (c->own_stream && c->stream) hipStreamDestroy(c->stream);
  delete c;
}

extern "C" const char* sd_last_error(const sd_ctx* c) { return c ? c->err.c_str() : g_load_error.c_str(); }

extern "C" sd_status sd_reset(sd_ctx* c, int32_t row) {
  if (!c) return SD_EINVAL;
  if (row < -1 || row >= c->batch) return fail(c, SD_EINVAL, "row must be -1 or a sequence index");
  for (int b = 0; b < c->batch; ++b)
    if (row == -1 || row == b) { c->ready[b] = 0; c->len[b] = 0; c->last_tok[b] = -1; c->hist_len[b] = 0; }
  if (row == -1) c->stats = sd_stats{};
  return SD_OK;
}

extern "C" sd_status sd_prefill(sd_ctx* c, int32_t row, const int32_t* prompt, int32_t n,
                                const void* enc_p, const void* enc_q) {
  if (!c) return SD_EINVAL;
  if (row < 0 || row >= c->batch || !prompt || n < 1) return fail(c, SD_EINVAL, "row must be a sequence index, prompt non-empty");
  const sd_model_cfg &pc = c->p.cfg, &qc = c->q.cfg;
  if ((pc.arch == SD_ARCH_T5DEC) != (enc_p != nullptr) || (qc.arch == SD_ARCH_T5DEC) != (enc_q != nullptr))
    return fail(c, SD_EINVAL, "encoder output must be given exactly for T5DEC models");
  const int room = std::min(pc.max_len, qc.max_len);
  if (n + c->rt.max_gamma + 1 > room) return fail(c, SD_ERANGE, "prompt + max_gamma + 1 exceeds max_len");
  for (int i = 0; i < n; ++i) if (prompt[i] < 0 || prompt[i] >= pc.vocab) return fail(c, SD_ERANGE, "token id out of range");
  c->ready[row] = 0; c->hist_len[row] = 0;
  Model* ms[2] = {&c->p, &c->q};
  const void* encs[2] = {enc_p, enc_q};
  for (int k = 0; k < 2; ++k) {
    Model& m = *ms[k];
    HIP_TRY(c, hipMemcpyAsync(m.prompt, prompt, (size_t)n * sizeof(int), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (m.cfg.arch == SD_ARCH_T5DEC) {
      if (m.cfg.dtype == SD_BF16) cross_kv<bf16>(c, m, encs[k]); else cross_kv<float>(c, m, encs[k]);
    }
    const int step = prefill_rows(m.cfg);
    for (int s0 = 0; s0 < n - 1; s0 += step)
      forward_any(c, m, Rows{ROWS_PREFILL, 0, std::min(step, n - 1 - s0), s0, row, 1, 0}, nullptr);
  }
  SeqState st{};
  st.len = n; st.last_tok = prompt[n - 1]; st.prev_tok = (n >= 2) ? prompt[n - 2] : 0;
  for (int i = 0; i < 16; ++i) { st.x[i] = 0; st.out[i] = -1; }
  c->h_state[row] = st;
  HIP_TRY(c, hipMemcpyAsync(c->d_state + row, c->h_state + row, sizeof(SeqState), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipMemcpyAsync(c->d_hist + (size_t)row * c->hist_stride, prompt, (size_t)n * sizeof(int), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  HIP_TRY(c, hipGetLastError());
  c->ready[row] = 1; c->len[row] = n; c->last_tok[row] = prompt[n - 1]; c->hist_len[row] = n;
  c->mq_stale[row] = 0;                             // both caches were just filled for this sequence
  return SD_OK;
}

static sd_status check_uniforms(sd_ctx* c, float temperature, const float* u, int n) {
  if (!(temperature >= 0.0f) || !std::isfinite(temperature)) return fail(c, SD_EINVAL, "temperature must be finite and >= 0");
  if (temperature > 0.0f && !u) return fail(c, SD_EINVAL, "uniforms required when temperature > 0");
  if (u) for (int i = 0; i < n; ++i) if (!(u[i] > 0.0f && u[i] < 1.0f)) return fail(c, SD_ERANGE, "uniform outside (0,1)");
  return SD_OK;
}

extern "C" sd_status sd_step(sd_ctx* c, const int32_t* prefix, int32_t prefix_len, int32_t gamma,
                             float temperature, const float* uniforms, int32_t* out_tokens, int32_t* out_n) {
  if (!c) return SD_EINVAL;
  if (!out_tokens || !out_n) return fail(c, SD_EINVAL, "null output");
  if (gamma < 1 || gamma > c->rt.max_gamma) return fail(c, SD_EINVAL, "gamma out of range");
  const int B = c->batch;
  if (!c->all_ready()) return fail(c, SD_ESTATE, "sd_step before every sequence was prefilled");
  if (!c->no_mq() && c->any_stale()) return fail(c, SD_ESTATE, "Mq cache is stale (after sd_step_baseline or drafts without Mq): reset and prefill");
  if (c->copy_match > 0)
    for (int b = 0; b < B; ++b)
      if (c->hist_len[b] != c->len[b]) return fail(c, SD_ESTATE, "token history incomplete: choose the copying draft before prefill");
  if (prefix && B > 1) return fail(c, SD_EINVAL, "the prefix check is for single-sequence contexts");
  if (prefix && (prefix_len != c->len[0] || prefix[prefix_len - 1] != c->last_tok[0]))
    return fail(c, SD_ESTATE, "prefix does not match the committed sequence");
  const int nu = 2 * gamma + 1;
  sd_status st = check_uniforms(c, temperature, uniforms, B * nu);
  if (st != SD_OK) return st;
  for (int b = 0; b < B; ++b)
    if (c->len[b] + gamma + 1 > std::min(c->p.cfg.max_len, c->q.cfg.max_len)) return fail(c, SD_ERANGE, "sequence would exceed max_len");

  for (int b = 0; b < B; ++b) {
    StepParams& hp = c->h_params[b];
    hp.temperature = temperature;
    hp.lenience = c->sampling.lenience;
    hp.log_lenience = std::log((double)c->sampling.lenience);
    hp.top_k = c->sampling.top_k; hp.top_p = c->sampling.top_p;
    for (int i = 0; i < nu; ++i) hp.uniforms[i] = uniforms ? uniforms[(size_t)b * nu + i] : 0.5f;
  }
  const size_t pbytes = (size_t)B * sizeof(StepParams), sbytes = (size_t)B * sizeof(SeqState);
  const bool profile = (c->rt.flags & SD_FLAG_PROFILE) != 0;
  const bool graph = (c->rt.flags & SD_FLAG_GRAPH) != 0 && !profile;
  if (graph) {
    if (!c->graphs[gamma]) {
      st = capture_graph(c, &c->graphs[gamma], [&] {
        hipMemcpyAsync(c->d_params, c->h_params, pbytes, hipMemcpyHostToDevice, c->stream);
        enqueue_step(c, gamma, false);
        hipMemcpyAsync(c->h_state, c->d_state, sbytes, hipMemcpyDeviceToHost, c->stream);
      });
      if (st != SD_OK) return st;
    }
    HIP_TRY(c, hipGraphLaunch(c->graphs[gamma], c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  } else {
    HIP_TRY(c, hipMemcpyAsync(c->d_params, c->h_params, pbytes, hipMemcpyHostToDevice, c->stream));
    enqueue_step(c, gamma, profile);
    if ((st = sync_state_to_host(c)) != SD_OK) return st;
  }
  HIP_TRY(c, hipGetLastError());
  for (int b = 0; b < B; ++b) {
    const SeqState& hs = c->h_state[b];
    if (hs.n < 0 || hs.n > gamma || hs.len != c->len[b] + hs.n + 1) return poisoned(c, "device state inconsistent after step");
  }
  int64_t fallbacks = 0;
  for (int b = 0; b < B; ++b) {
    const SeqState& hs = c->h_state[b];
    out_n[b] = hs.n;
    for (int i = 0; i <= gamma; ++i) out_tokens[(size_t)b * (gamma + 1) + i] = (i <= hs.n) ? hs.out[i] : -1;
    c->len[b] = hs.len; c->last_tok[b] = hs.last_tok;
    if (c->copy_match > 0) c->hist_len[b] = hs.len;
    c->stats.tokens += hs.n + 1; c->stats.accepted += hs.n;
    fallbacks += hs.fallbacks;
    const int tested = std::min(hs.n + 1, gamma);          // guesses whose test decided something
    c->stats.tested += tested;
    c->tune_tested += tested; c->tune_accepted += hs.n;
    if (c->rt.flags & SD_FLAG_BETA) {
      double bsum = 0.0;
      for (int i = 0; i < tested; ++i) bsum += (double)hs.beta[i];
      c->stats.beta_sum += bsum; c->stats.beta_count += tested;
      c->tune_beta_sum += bsum; c->tune_beta_count += tested;
    }
  }
  c->stats.fallbacks = fallbacks;
  if (c->no_mq()) c->mq_stale.assign((size_t)B, 1);      // Mq did not see these tokens
  c->last_gamma = gamma; c->last_kind = 0;
  c->stats.steps += 1;
  if (profile) {
    float a = 0, b = 0, d = 0;
    hipEventElapsedTime(&a, c->ev[0], c->ev[1]); hipEventElapsedTime(&b, c->ev[1], c->ev[2]);
    hipEventElapsedTime(&d, c->ev[2], c->ev[3]);
    c->stats.draft_ms = a; c->stats.verify_ms = b; c->stats.accept_ms = d;
    for (size_t i = 0; i + 1 < c->kev.size(); i += 2) {
      float k = 0;
      if (hipEventElapsedTime(&k, c->kev[i], c->kev[i + 1]) == hipSuccess) { c->stats.ffn_in_ms_sum += k; c->stats.ffn_in_launches += 1; }
    }
  }
  return SD_OK;
}

extern "C" sd_status sd_step_baseline(sd_ctx* c, float temperature, const float* uniforms, int32_t* out_token) {
  if (!c) return SD_EINVAL;
  if (!out_token) return fail(c, SD_EINVAL, "null output");
  const int B = c->batch;
  if (!c->all_ready()) return fail(c, SD_ESTATE, "sd_step_baseline before every sequence was prefilled");
  sd_status st = check_uniforms(c, temperature, uniforms, B);
  if (st != SD_OK) return st;
  for (int b = 0; b < B; ++b)
    if (c->len[b] + 1 > c->p.cfg.max_len) return fail(c, SD_ERANGE, "sequence would exceed max_len");
  for (int b = 0; b < B; ++b) {
    StepParams& hp = c->h_params[b];
    hp.temperature = temperature;
    hp.lenience = 1.0f; hp.log_lenience = 0.0;
    hp.top_k = c->sampling.top_k; hp.top_p = c->sampling.top_p;
    hp.uniforms[0] = uniforms ? uniforms[b] : 0.5f;
  }
  const size_t pbytes = (size_t)B * sizeof(StepParams), sbytes = (size_t)B * sizeof(SeqState);
  if ((c->rt.flags & SD_FLAG_GRAPH) != 0) {
    if (!c->graph_baseline) {
      st = capture_graph(c, &c->graph_baseline, [&] {
        hipMemcpyAsync(c->d_params, c->h_params, pbytes, hipMemcpyHostToDevice, c->stream);
        enqueue_baseline(c);
        hipMemcpyAsync(c->h_state, c->d_state, sbytes, hipMemcpyDeviceToHost, c->stream);
      });
      if (st != SD_OK) return st;
    }
    HIP_TRY(c, hipGraphLaunch(c->graph_baseline, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  } else {
    HIP_TRY(c, hipMemcpyAsync(c->d_params, c->h_params, pbytes, hipMemcpyHostToDevice, c->stream));
    enqueue_baseline(c);
    if ((st = sync_state_to_host(c)) != SD_OK) return st;
  }
  HIP_TRY(c, hipGetLastError());
  for (int b = 0; b < B; ++b)
    if (c->h_state[b].len != c->len[b] + 1) return poisoned(c, "device state inconsistent after baseline step");
  for (int b = 0; b < B; ++b) {
    out_token[b] = c->h_state[b].last_tok;
    if (c->copy_match > 0 && c->hist_len[b] == c->len[b]) c->hist_len[b] = c->h_state[b].len;
    c->len[b] = c->h_state[b].len; c->last_tok[b] = c->h_state[b].last_tok;
  }
  c->mq_stale.assign((size_t)B, 1);
  c->last_kind = 2;
  return SD_OK;
}

extern "C" sd_status sd_debug_logits(sd_ctx* c, int32_t which, float* host_out, size_t n) {
  if (!c || !host_out) return SD_EINVAL;
  const size_t V = c->p.cfg.vocab;
  const float* src = nullptr;
  size_t rows = 0;
  const size_t B = (size_t)c->batch;
  if (which == 0 && c->last_kind == 0) { src = c->p_logits; rows = B * (c->last_gamma + 1); }
  else if (which == 1 && c->last_kind == 0) { src = c->q_logits; rows = B * c->last_gamma; }
  else if (which == 2 && c->last_kind == 2) { src = c->p_logits; rows = B; }
  else return fail(c, SD_ESTATE, "no such logits from the last call");
  if (n > rows * V) return fail(c, SD_EINVAL, "more floats requested than the last call produced");
  HIP_TRY(c, hipMemcpy(host_out, src, n * sizeof(float), hipMemcpyDeviceToHost));
  return SD_OK;
}

extern "C" sd_status sd_set_flags(sd_ctx* c, int32_t flags) {
  if (!c) return SD_EINVAL;
  if (flags & ~(SD_FLAG_GRAPH | SD_FLAG_PROFILE | SD_FLAG_BETA | SD_FLAG_SCATTER_PAGES | SD_FLAG_SEPARATE_CROSS_Q)) return fail(c, SD_EINVAL, "unknown flag");
  flags = (flags & ~SD_FLAG_SCATTER_PAGES) | (c->rt.flags & SD_FLAG_SCATTER_PAGES);    // the cache layout is fixed at load
  if ((flags ^ c->rt.flags) & (SD_FLAG_BETA | SD_FLAG_SEPARATE_CROSS_Q)) {            // the captured iteration changes
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (auto& g : c->graphs) if (g) { hipGraphExecDestroy(g); g = nullptr; }
    if (c->graph_baseline) { hipGraphExecDestroy(c->graph_baseline); c->graph_baseline = nullptr; }
  }
  c->rt.flags = flags;
  return SD_OK;
}

extern "C" sd_status sd_set_table_draft(sd_ctx* c, const float* table, const int32_t* row_of, int32_t n_rows) {
  if (!c) return SD_EINVAL;
  if (table != nullptr && n_rows < 1) return fail(c, SD_EINVAL, "a draft table needs at least one row");
  if (table == nullptr && (row_of != nullptr || n_rows != 0)) return fail(c, SD_EINVAL, "no table: row_of must be NULL and n_rows 0");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (auto& g : c->graphs) if (g) { hipGraphExecDestroy(g); g = nullptr; }     // the captured draft loop changes
  // (steps taken without Mq mark the sequences' Mq caches stale: going back to Mq needs them prefilled again)
  c->draft_table = table; c->draft_row_of = table ? row_of : nullptr; c->draft_rows = table ? n_rows : 0;
  return SD_OK;
}

extern "C" sd_status sd_set_copy_draft(sd_ctx* c, int32_t match) {
  if (!c) return SD_EINVAL;
  if (match < 0 || match > SD_MAX_COPY_MATCH) return fail(c, SD_EINVAL, "match must lie in [0, SD_MAX_COPY_MATCH]");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (auto& g : c->graphs) if (g) { hipGraphExecDestroy(g); g = nullptr; }     // the captured launches change
  if (c->graph_baseline) { hipGraphExecDestroy(c->graph_baseline); c->graph_baseline = nullptr; }
  c->copy_match = match;
  return SD_OK;
}

extern "C" sd_status sd_set_sampling(sd_ctx* c, const sd_sampling* opt) {
  if (!c || !opt) return SD_EINVAL;
  if (!(opt->lenience > 0.0f && opt->lenience <= 1.0f)) return fail(c, SD_EINVAL, "lenience must lie in (0, 1]");
  if (opt->top_k < 0 || !(opt->top_p >= 0.0f && opt->top_p <= 1.0f)) return fail(c, SD_EINVAL, "top_k must be >= 0 and top_p in [0, 1]");
  const bool filter = opt->top_k > 0 || (opt->top_p > 0.0f && opt->top_p < 1.0f);
  if (filter && (c->p.cfg.vocab > SAMPLE_REG_F4 * 4 * SAMPLE_THREADS || (c->p.cfg.vocab & 3)))
    return fail(c, SD_EINVAL, "top-k / nucleus need vocab <= 32768 and vocab % 4 == 0");
  c->sampling = *opt;
  return SD_OK;
}

// Theorem 3.8 for one gamma; alpha -> 1 has the limit (gamma + 1) / (gamma c + 1).
static double improvement_factor(double alpha, double c, int gamma) {
  double tokens = 0.0, a = 1.0;                          // 1 + alpha + ... + alpha^gamma (Eq. 1)
  for (int i = 0; i <= gamma; ++i) { tokens += a; a *= alpha; }
  return tokens / ((double)gamma * c + 1.0);
}

extern "C" sd_status sd_choose_gamma(double alpha, double cost, int32_t gamma_max, int32_t* gamma, double* improvement) {
  if (!gamma || gamma_max < 1 || !(alpha >= 0.0 && alpha < 1.0) || !(cost >= 0.0) || !std::isfinite(cost)) return SD_EINVAL;
  int best = 1;
  double best_v = improvement_factor(alpha, cost, 1);
  for (int g = 2; g <= gamma_max; ++g) {
    const double v = improvement_factor(alpha, cost, g);
    if (v > best_v) { best_v = v; best = g; }
  }
  *gamma = best;
  if (improvement) *improvement = best_v;
  return SD_OK;
}

extern "C" sd_status sd_measure_cost(sd_ctx* c, int32_t reps, double* mq_us, double* mp_us) {
  if (!c || !mq_us || !mp_us) return SD_EINVAL;
  if (reps < 1 || reps > 1000) return fail(c, SD_EINVAL, "reps must be 1..1000");
  if (!c->all_ready() || c->any_stale()) return fail(c, SD_ESTATE, "sd_measure_cost needs a prefilled sequence with a valid Mq cache");
  if (c->no_mq()) return fail(c, SD_ESTATE, "sd_measure_cost times Mq: clear the table / copying draft first");
  const int V = c->p.cfg.vocab, B = c->batch;
  if (c->rt.max_gamma < 2) return fail(c, SD_EINVAL, "sd_measure_cost needs max_gamma >= 2 (it runs a second draft step)");
  for (int b = 0; b < B; ++b)
    if (c->len[b] + 2 > std::min(c->p.cfg.max_len, c->q.cfg.max_len)) return fail(c, SD_ERANGE, "no room behind the committed sequence");
  // step parameters for the draws: whatever temperature was used last is fine, the uniforms must be valid
  for (int b = 0; b < B; ++b) {
    StepParams& hp = c->h_params[b];
    hp.uniforms[0] = 0.5f; hp.uniforms[1] = 0.5f;
    if (!(hp.temperature >= 0.0f)) hp.temperature = 1.0f;
    hp.lenience = c->sampling.lenience;
    hp.log_lenience = std::log((double)c->sampling.lenience);
    hp.top_k = c->sampling.top_k; hp.top_p = c->sampling.top_p;
  }
  HIP_TRY(c, hipMemcpyAsync(c->d_params, c->h_params, (size_t)B * sizeof(StepParams), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  double us[2] = {0.0, 0.0};
  for (int which = 0; which < 2; ++which) {
    hipGraphExec_t ge = nullptr;
    const sd_status cs = capture_graph(c, &ge, [&] {
      if (which == 0) {      // a draft step that is not the first of an iteration: guess x_1 in, q_2 and x_2 out
        forward_any(c, c->q, Rows{ROWS_DRAFT_NEXT, 1, 1, 0, 0, B, 2}, c->q_logits);     // rows [seq][2][V], second of each
        launch_draw(c, c->q_logits + (size_t)V, 1, 0, 1, (size_t)2 * V);
      } else {               // standard decoding's forward and draw; the draw lands in a guess slot, nothing is committed
        forward_any(c, c->p, Rows{ROWS_BASELINE, 0, 1, 0, 0, B, 0}, c->p_logits);
        launch_draw(c, c->p_logits, 0, 0, 1, (size_t)V);
      }
    });
    if (cs != SD_OK) return cs;
    hipError_t e = hipSuccess;
    hipGraphLaunch(ge, c->stream);                       // warm-up
    hipEventRecord(c->ev[0], c->stream);
    for (int i = 0; i < reps; ++i) hipGraphLaunch(ge, c->stream);
    hipEventRecord(c->ev[1], c->stream);
    e = hipStreamSynchronize(c->stream);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev[0], c->ev[1]);
    hipGraphExecDestroy(ge);
    if (e != hipSuccess) return fail(c, SD_EHIP, std::string("sd_measure_cost: ") + hipGetErrorString(e));
    us[which] = 1e3 * (double)ms / (double)reps;
  }
  c->last_kind = -1;                                     // the logits buffers no longer hold a step's rows
  *mq_us = us[0]; *mp_us = us[1];
  return SD_OK;
}

extern "C" sd_status sd_autotune_gamma(sd_ctx* c, int32_t reps, int32_t* gamma, double* alpha, double* cost,
                                       double* improvement) {
  if (!c || !gamma) return SD_EINVAL;
  if (c->tune_tested < 1) return fail(c, SD_ESTATE, "no acceptance test recorded yet: run sd_step first");
  double a = (c->tune_beta_count > 0) ? c->tune_beta_sum / (double)c->tune_beta_count
                                      : (double)c->tune_accepted / (double)c->tune_tested;
  a = std::min(std::max(a, 0.0), 1.0 - 1e-9);
  double mq = 0.0, mp = 0.0;
  sd_status st = sd_measure_cost(c, reps, &mq, &mp);
  if (st != SD_OK) return st;
  const double cc = mq / mp;
  st = sd_choose_gamma(a, cc, c->rt.max_gamma, gamma, improvement);
  if (st != SD_OK) return fail(c, st, "sd_choose_gamma rejected the measured alpha / c");
  if (alpha) *alpha = a;
  if (cost) *cost = cc;
  return SD_OK;
}

extern "C" sd_status sd_time_ffn_in(sd_ctx* c, int32_t rows, int32_t reps, double* us_per_launch) {
  if (!c || !us_per_launch) return SD_EINVAL;
  if (rows < 1 || rows > MAX_ROWS || reps < 1 || reps > 1000) return fail(c, SD_EINVAL, "rows must be 1..16, reps 1..1000");
  Model& m = c->p;
  const sd_model_cfg& f = m.cfg;
  const bool rms = f.arch != SD_ARCH_GPT;
  hipGraphExec_t ge = nullptr;
  const sd_status cs = capture_graph(c, &ge, [&] {
  for (const LayerW& l : m.L) {
    GemmArgs h{};
    h.R = rows; h.eps = f.norm_eps; h.K = f.d_model; h.N = f.d_ff; h.out = m.ffn; h.ldo = f.d_ff; h.W = l.w1;
    if (rms) {
      h.X = m.xg; h.ss_in = m.ss; h.n_part = f.d_model / 16;
      h.W2 = l.wu; h.act = (f.arch == SD_ARCH_T5DEC) ? ACT_GELU : ACT_SILU;
      if (f.dtype == SD_BF16) launch_gemm<bf16>(c->stream, PRO_POST, EPI_GATED, h);
      else launch_gemm<float>(c->stream, PRO_POST, EPI_GATED, h);
    } else {
      h.X = m.x; h.gain = l.ln2g; h.beta = l.ln2b; h.bias = l.b1;
      if (f.dtype == SD_BF16) launch_gemm<bf16>(c->stream, PRO_LN, EPI_ACT, h);
      else launch_gemm<float>(c->stream, PRO_LN, EPI_ACT, h);
    }
  }
  });
  if (cs != SD_OK) return cs;
  hipError_t e = hipSuccess;
  hipGraphLaunch(ge, c->stream);                       // warm-up
  hipEventRecord(c->ev[0], c->stream);
  for (int i = 0; i < reps; ++i) hipGraphLaunch(ge, c->stream);
  hipEventRecord(c->ev[1], c->stream);
  e = hipStreamSynchronize(c->stream);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev[0], c->ev[1]);
  hipGraphExecDestroy(ge);
  if (e != hipSuccess) return fail(c, SD_EHIP, std::string("sd_time_ffn_in: ") + hipGetErrorString(e));
  *us_per_launch = 1e3 * (double)ms / ((double)reps * (double)m.L.size());
  return SD_OK;
}

extern "C" sd_status sd_time_forward(sd_ctx* c, int32_t which, int32_t rows, int32_t skip_ops, int32_t reps,
                                     double* us_per_forward) {
  if (!c || !us_per_forward) return SD_EINVAL;
  if (which < 0 || which > 1 || reps < 1 || reps > 1000 || (skip_ops & ~SD_OP_ALL)) return fail(c, SD_EINVAL, "which must be 0 / 1, reps 1..1000, skip_ops a set of SD_OP_* bits");
  const int B = c->batch;
  const int max_rows = (which == 0) ? c->rt.max_gamma + 1 : 2;
  if (rows < 1 || rows > max_rows) return fail(c, SD_EINVAL, "rows must be 1..max_gamma+1 for Mp, 1..2 for Mq");
  if (!c->all_ready() || (which == 1 && c->any_stale())) return fail(c, SD_ESTATE, "sd_time_forward needs every sequence prefilled (and a valid Mq cache to time Mq)");
  for (int b = 0; b < B; ++b)
    if (c->len[b] + rows > std::min(c->p.cfg.max_len, c->q.cfg.max_len)) return fail(c, SD_ERANGE, "no room behind the committed sequence");
  hipGraphExec_t ge = nullptr;
  c->skip_ops = skip_ops;
  const sd_status cs = capture_graph(c, &ge, [&] {
    if (which == 0) {
      if (rows == 1) forward_any(c, c->p, Rows{ROWS_BASELINE, 0, 1, 0, 0, B, 0}, c->p_logits);
      else forward_any(c, c->p, Rows{ROWS_VERIFY, 0, rows, 0, 0, B, rows - 1}, c->p_logits);
    } else {
      if (rows == 1) forward_any(c, c->q, Rows{ROWS_DRAFT_NEXT, 1, 1, 0, 0, B, 2}, c->q_logits);
      else forward_any(c, c->q, Rows{ROWS_DRAFT_FIRST, 0, 2, 0, 0, B, 2}, c->q_logits);
    }
  });
  c->skip_ops = 0;
  if (cs != SD_OK) return cs;
  hipGraphLaunch(ge, c->stream);                       // warm-up
  hipEventRecord(c->ev[0], c->stream);
  for (int i = 0; i < reps; ++i) hipGraphLaunch(ge, c->stream);
  hipEventRecord(c->ev[1], c->stream);
  hipError_t e = hipStreamSynchronize(c->stream);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev[0], c->ev[1]);
  hipGraphExecDestroy(ge);
  c->last_kind = -1;                                   // the logits buffers no longer hold a step's rows
  if (e != hipSuccess) return fail(c, SD_EHIP, std::string("sd_time_forward: ") + hipGetErrorString(e));
  *us_per_forward = 1e3 * (double)ms / (double)reps;
  return SD_OK;
}

extern "C" sd_status sd_time_stream_read(sd_ctx* c, int32_t which, int32_t reps, double* us_per_pass, double* bytes_per_pass) {
  if (!c || !us_per_pass || !bytes_per_pass) return SD_EINVAL;
  if (which < 0 || which > 1 || reps < 1 || reps > 1000) return fail(c, SD_EINVAL, "which must be 0 / 1, reps 1..1000");
  const Model& m = which ? c->q : c->p;
  // the model's weights as the library holds them: from the output table to the end of the last layer's weights
  const char* lo = static_cast<const char*>(m.head);
  const LayerW& last = m.L.back();
  const char* hi = static_cast<const char*>(last.kv);
  if (hi <= lo) return fail(c, SD_EINVAL, "unexpected workspace layout");
  const size_t n_blocks = (size_t)(hi - lo) / 1024;
  float* sink = reinterpret_cast<float*>(c->d_counter);      // never written: the kernel's condition cannot hold
  hipLaunchKernelGGL(stream_read_kernel, dim3(g_num_cus), dim3(512), 0, c->stream, reinterpret_cast<const f32x4*>(lo), n_blocks, sink);
  hipEventRecord(c->ev[0], c->stream);
  for (int i = 0; i < reps; ++i)
    hipLaunchKernelGGL(stream_read_kernel, dim3(g_num_cus), dim3(512), 0, c->stream, reinterpret_cast<const f32x4*>(lo), n_blocks, sink);
  hipEventRecord(c->ev[1], c->stream);
  hipError_t e = hipStreamSynchronize(c->stream);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev[0], c->ev[1]);
  if (e != hipSuccess) return fail(c, SD_EHIP, std::string("sd_time_stream_read: ") + hipGetErrorString(e));
  *us_per_pass = 1e3 * (double)ms / (double)reps;
  *bytes_per_pass = (double)n_blocks * 1024.0;
  return SD_OK;
}

extern "C" sd_status sd_get_stats(sd_ctx* c, sd_stats* out) {
  if (!c || !out) return SD_EINVAL;
  *out = c->stats;
  return SD_OK;
}

#include "spec_sample_api.hip"
