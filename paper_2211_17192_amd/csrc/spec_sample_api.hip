// C-ABI entry points of the stand-alone accept / resample kernel (the second
// half of Algorithm 1 on explicit logits).  See include/sd.h.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include <mutex>
#include <string>
#include "../../include/sd.h"
#include "kernels_misc.h"
#include "kernels_sample.h"

namespace {
size_t scratch_align(size_t v, size_t a) { return (v + a - 1) / a * a; }
}

extern "C" size_t sd_spec_sample_scratch_bytes(int32_t rows, int32_t gamma) {
  if (rows < 1 || gamma < 1 || gamma > SD_MAX_GAMMA) return 0;
  return scratch_align((size_t)rows * sd::SAMPLE_COUNTER_STRIDE * sizeof(unsigned int), 256) +
         (size_t)rows * (2 * gamma + 1) * sizeof(sd::RowStat);
}

namespace {
// Argument checks shared by the entry points; fills the resolved options.
struct SampleOpts { float len; double log_len; int top_k; float top_p; };
sd_status check_sample_args(const float* p_logits, const float* q_logits, const int32_t* x, const float* r,
                            const float* s, int32_t rows, int32_t gamma, int32_t vocab, float temperature,
                            const sd_sampling* opt, const int32_t* out_n, const int32_t* out_t, SampleOpts& o) {
  if (!p_logits || !q_logits || !x || !out_n || !out_t) return SD_EINVAL;
  if (rows < 1 || rows > 65535 || gamma < 1 || gamma > SD_MAX_GAMMA || vocab < 1 ||
      vocab > sd::SAMPLE_CHUNK * sd::SAMPLE_MAX_CHUNKS) return SD_EINVAL;
  if (!(temperature >= 0.0f)) return SD_EINVAL;
  if (temperature > 0.0f && (!r || !s)) return SD_EINVAL;
  o.len = opt ? opt->lenience : 1.0f;
  if (!(o.len > 0.0f && o.len <= 1.0f)) return SD_EINVAL;
  o.log_len = std::log((double)o.len);
  o.top_k = opt ? opt->top_k : 0;
  o.top_p = opt ? opt->top_p : 0.0f;
  if (o.top_k < 0 || !(o.top_p >= 0.0f && o.top_p <= 1.0f)) return SD_EINVAL;
  if ((o.top_k > 0 || (o.top_p > 0.0f && o.top_p < 1.0f)) &&
      (vocab > sd::SAMPLE_REG_F4 * 4 * sd::SAMPLE_THREADS || (vocab & 3) ||
       (reinterpret_cast<uintptr_t>(p_logits) & 15) || (reinterpret_cast<uintptr_t>(q_logits) & 15)))
    return SD_EINVAL;                            // the filters run on rows held in registers
  return SD_OK;
}

// The launches of one call; counters: one ticket per row, SAMPLE_COUNTER_STRIDE words apart, zero
// before the call (the one-launch form leaves them zero again); stats: rows x (2 gamma + 1).
sd_status launch_spec_sample(const float* p_logits, const float* q_logits, const int32_t* x, const float* r,
                             const float* s, int32_t rows, int32_t gamma, int32_t vocab, float temperature,
                             const SampleOpts& o, int32_t* out_n, int32_t* out_t, float* beta,
                             unsigned int* counters, sd::RowStat* stats, hipStream_t s_) {
  const dim3 grid(2 * gamma + 1, rows), block(sd::SAMPLE_THREADS);
#define SD_VERIFY(MODE, GRID)                                                                                   \
  hipLaunchKernelGGL(sd::spec_verify_kernel<MODE>, GRID, block, 0, s_, p_logits, q_logits, x, r, s, gamma, vocab, \
                     temperature, o.len, o.log_len, o.top_k, o.top_p, (const sd::StepParams*)nullptr, stats, counters, out_n, out_t,  \
                     beta, (sd::SeqState*)nullptr)
  if (rows * (2 * gamma + 1) <= 64) {           // few tickets: one launch
    SD_VERIFY(0, grid);
  } else {                                       // many sequences: statistics, then one tail workgroup each
    SD_VERIFY(1, grid);
    SD_VERIFY(2, dim3(1, rows));
  }
  if (beta) SD_VERIFY(3, dim3(gamma, rows));
#undef SD_VERIFY
  return hipGetLastError() == hipSuccess ? SD_OK : SD_EHIP;
}
}  // namespace

extern "C" sd_status sd_spec_sample_ex(const float* p_logits, const float* q_logits, const int32_t* x,
                                       const float* r, const float* s, int32_t rows, int32_t gamma,
                                       int32_t vocab, float temperature, const sd_sampling* opt,
                                       int32_t* out_n, int32_t* out_t, float* beta, void* scratch, void* stream) {
  if (!scratch) return SD_EINVAL;
  SampleOpts o{};
  const sd_status st = check_sample_args(p_logits, q_logits, x, r, s, rows, gamma, vocab, temperature, opt, out_n, out_t, o);
  if (st != SD_OK) return st;
  unsigned int* counters = static_cast<unsigned int*>(scratch);
  sd::RowStat* stats = reinterpret_cast<sd::RowStat*>(
      static_cast<char*>(scratch) + scratch_align((size_t)rows * sd::SAMPLE_COUNTER_STRIDE * sizeof(unsigned int), 256));
  return launch_spec_sample(p_logits, q_logits, x, r, s, rows, gamma, vocab, temperature, o, out_n, out_t, beta,
                            counters, stats, static_cast<hipStream_t>(stream));
}

extern "C" sd_status sd_spec_sample(const float* p_logits, const float* q_logits, const int32_t* x,
                                    const float* r, const float* s, int32_t rows, int32_t gamma,
                                    int32_t vocab, float temperature, int32_t* out_n,
                                    int32_t* out_t, void* scratch, void* stream) {
  return sd_spec_sample_ex(p_logits, q_logits, x, r, s, rows, gamma, vocab, temperature, nullptr, out_n, out_t,
                           nullptr, scratch, stream);
}

// ---------------------------------------------------------------------------
// The same call for callers that cannot allocate: its scratch (tickets and row
// statistics) is a fixed array in device memory that belongs to the library.
// Every GPU the library runs on holds its own copy at its own address; host code
// must not hand the array's name to a kernel, it asks the runtime for the address
// once per device and uses that pointer from then on.
// ---------------------------------------------------------------------------
namespace {
constexpr int STATIC_ROWS = SD_SPEC_SAMPLE_STATIC_MAX_ROWS;
constexpr size_t STATIC_COUNTER_BYTES = (size_t)STATIC_ROWS * sd::SAMPLE_COUNTER_STRIDE * sizeof(unsigned int);
constexpr size_t STATIC_STAT_BYTES = (size_t)STATIC_ROWS * (2 * SD_MAX_GAMMA + 1) * sizeof(sd::RowStat);
static_assert(STATIC_COUNTER_BYTES % 256 == 0, "the statistics start 256-byte aligned");
static __device__ __align__(256) unsigned char scratch[STATIC_COUNTER_BYTES + STATIC_STAT_BYTES];   // 250 KB

constexpr int STATIC_MAX_DEVICES = 64;
void* g_scratch_ptr[STATIC_MAX_DEVICES] = {};    // device address of `scratch` on each device, once known
std::mutex g_scratch_mutex;

// The address of this device's copy of `scratch` (nullptr + *err on failure).
void* static_scratch_address(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || ptr == nullptr) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" sd_status sd_spec_sample_static(const float* p_logits, const float* q_logits, const int32_t* x,
                                           const float* r, const float* s, int32_t rows, int32_t gamma,
                                           int32_t vocab, float temperature, const sd_sampling* opt,
                                           int32_t* out_n, int32_t* out_t, float* beta, void* stream) {
  SampleOpts o{};
  const sd_status st = check_sample_args(p_logits, q_logits, x, r, s, rows, gamma, vocab, temperature, opt, out_n, out_t, o);
  if (st != SD_OK) return st;
  if (rows > STATIC_ROWS) {
    g_load_error = "sd_spec_sample_static takes at most " + std::to_string(STATIC_ROWS) + " rows per call (got " +
                   std::to_string(rows) + "): split the call, or use sd_spec_sample_ex with a scratch buffer of your own";
    return SD_ERANGE;
  }
  hipError_t e = hipSuccess;
  void* ptr = static_scratch_address(&e);
  if (ptr == nullptr) {
    g_load_error = std::string("sd_spec_sample_static: address of the scratch array: ") + hipGetErrorString(e);
    return SD_EHIP;
  }
  hipStream_t s_ = static_cast<hipStream_t>(stream);
  unsigned int* counters = static_cast<unsigned int*>(ptr);
  sd::RowStat* stats = reinterpret_cast<sd::RowStat*>(static_cast<char*>(ptr) + STATIC_COUNTER_BYTES);
  // the tickets must start at zero whatever an earlier (possibly failed) call left: a fill kernel,
  // not a memset, so that the call can be recorded into a graph
  const size_t words = (size_t)rows * sd::SAMPLE_COUNTER_STRIDE;
  hipLaunchKernelGGL(sd::fill_u32_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s_, counters, 0u, words);
  return launch_spec_sample(p_logits, q_logits, x, r, s, rows, gamma, vocab, temperature, o, out_n, out_t, beta,
                            counters, stats, s_);
}
