// C-ABI entry points of the stand-alone accept / resample kernel (the second
// half of Algorithm 1 on explicit logits).  See include/sd.h.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include "../../include/sd.h"
#include "kernels_sample.h"

namespace {
size_t scratch_align(size_t v, size_t a) { return (v + a - 1) / a * a; }
}

extern "C" size_t sd_spec_sample_scratch_bytes(int32_t rows, int32_t gamma) {
  if (rows < 1 || gamma < 1 || gamma > SD_MAX_GAMMA) return 0;
  return scratch_align((size_t)rows * sd::SAMPLE_COUNTER_STRIDE * sizeof(unsigned int), 256) +
         (size_t)rows * (2 * gamma + 1) * sizeof(sd::RowStat);
}

extern "C" sd_status sd_spec_sample_ex(const float* p_logits, const float* q_logits, const int32_t* x,
                                       const float* r, const float* s, int32_t rows, int32_t gamma,
                                       int32_t vocab, float temperature, const sd_sampling* opt,
                                       int32_t* out_n, int32_t* out_t, float* beta, void* scratch, void* stream) {
  if (!p_logits || !q_logits || !x || !out_n || !out_t || !scratch) return SD_EINVAL;
  if (rows < 1 || rows > 65535 || gamma < 1 || gamma > SD_MAX_GAMMA || vocab < 1 ||
      vocab > sd::SAMPLE_CHUNK * sd::SAMPLE_MAX_CHUNKS) return SD_EINVAL;
  if (!(temperature >= 0.0f)) return SD_EINVAL;
  if (temperature > 0.0f && (!r || !s)) return SD_EINVAL;
  const float len = opt ? opt->lenience : 1.0f;
  if (!(len > 0.0f && len <= 1.0f)) return SD_EINVAL;
  const double log_len = std::log((double)len);
  const int top_k = opt ? opt->top_k : 0;
  const float top_p = opt ? opt->top_p : 0.0f;
  if (top_k < 0 || !(top_p >= 0.0f && top_p <= 1.0f)) return SD_EINVAL;
  if ((top_k > 0 || (top_p > 0.0f && top_p < 1.0f)) &&
      (vocab > sd::SAMPLE_REG_F4 * 4 * sd::SAMPLE_THREADS || (vocab & 3) ||
       (reinterpret_cast<uintptr_t>(p_logits) & 15) || (reinterpret_cast<uintptr_t>(q_logits) & 15)))
    return SD_EINVAL;                            // the filters run on rows held in registers
  unsigned int* counters = static_cast<unsigned int*>(scratch);
  sd::RowStat* stats = reinterpret_cast<sd::RowStat*>(
      static_cast<char*>(scratch) + scratch_align((size_t)rows * sd::SAMPLE_COUNTER_STRIDE * sizeof(unsigned int), 256));
  const dim3 grid(2 * gamma + 1, rows), block(sd::SAMPLE_THREADS);
  hipStream_t s_ = static_cast<hipStream_t>(stream);
#define SD_VERIFY(MODE, GRID)                                                                                   \
  hipLaunchKernelGGL(sd::spec_verify_kernel<MODE>, GRID, block, 0, s_, p_logits, q_logits, x, r, s, gamma, vocab, \
                     temperature, len, log_len, top_k, top_p, (const sd::StepParams*)nullptr, stats, counters, out_n, out_t,  \
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

extern "C" sd_status sd_spec_sample(const float* p_logits, const float* q_logits, const int32_t* x,
                                    const float* r, const float* s, int32_t rows, int32_t gamma,
                                    int32_t vocab, float temperature, int32_t* out_n,
                                    int32_t* out_t, void* scratch, void* stream) {
  return sd_spec_sample_ex(p_logits, q_logits, x, r, s, rows, gamma, vocab, temperature, nullptr, out_n, out_t,
                           nullptr, scratch, stream);
}
