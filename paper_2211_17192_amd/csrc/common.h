// Device-side helpers shared by the gfx950 kernels: storage-type traits,
// wavefront (64 lanes) and workgroup reductions, the ticket used by kernels
// whose last-finishing workgroup runs a tail phase.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

constexpr int WAVE = 64;
constexpr int MAX_ROWS = 16;          // rows one forward handles = one MFMA column tile

typedef __bf16 bf16;
typedef float  f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Device-resident decoding state of one sequence (section 2.3 / Algorithm 1:
// the committed prefix is summarised by its length and last two tokens; x
// holds the guesses of the running iteration).
struct SeqState {
  int32_t len;                 // committed tokens
  int32_t last_tok;            // token at position len-1
  int32_t prev_tok;            // token at position len-2 (undefined when len < 2)
  int32_t n;                   // accepted guesses of the last iteration
  int32_t x[16];               // guesses x_1..x_gamma of this iteration
  int32_t out[16];             // tokens emitted by the last iteration, -1 padded
  int32_t fallbacks;           // zero-residual fallbacks taken so far
  int32_t pad[3];
};

// Per-call parameters that change between iterations; they live in device
// memory so that a captured graph can be replayed unchanged.
struct StepParams {
  float temperature;
  float uniforms[2 * 15 + 1];  // [0,g) draft draws, [g,2g) accept tests, [2g] final draw
};

template <typename T> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Store<bf16> {
  static __device__ __forceinline__ float ld(const bf16* p) { return (float)*p; }
  static __device__ __forceinline__ void st(bf16* p, float v) { *p = (bf16)v; }
};

// Round a value the way it would be stored in T and read back.
template <typename T> __device__ __forceinline__ float round_to(float v);
template <> __device__ __forceinline__ float round_to<float>(float v) { return v; }
template <> __device__ __forceinline__ float round_to<bf16>(float v) { return (float)(bf16)v; }

// Load 8 consecutive elements of T (16-byte aligned for bf16, 32 for float) as floats.
template <typename T> __device__ __forceinline__ void load8(const T* p, float (&o)[8]);
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&o)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
template <> __device__ __forceinline__ void load8<bf16>(const bf16* p, float (&o)[8]) {
  const bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (float)v[e];
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, WAVE));
  return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, WAVE));
  return v;
}

// Workgroup-wide reductions over up to 16 waves.  `red` is LDS scratch of at
// least 16 elements of the value type; every thread gets the result.  The
// combine order is fixed (wave 0..n-1), so results are run-to-run identical.
template <typename V, typename Op>
__device__ __forceinline__ V block_reduce(V v, V* red, Op op, V identity) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = op(v, __shfl_xor(v, o, WAVE));
  __syncthreads();                       // protect `red` from the previous use
  if (lane == 0) red[wave] = v;
  __syncthreads();
  V r = identity;
  for (int w = 0; w < nw; ++w) r = op(r, red[w]);
  return r;
}

struct OpSumF { __device__ float operator()(float a, float b) const { return a + b; } };
struct OpSumD { __device__ double operator()(double a, double b) const { return a + b; } };
struct OpMaxF { __device__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpMinI { __device__ int operator()(int a, int b) const { return min(a, b); } };
struct OpMaxI { __device__ int operator()(int a, int b) const { return max(a, b); } };

// Ticket: returns true in every thread of exactly one workgroup, the one that
// arrives last among `expected`; that workgroup sees all global writes the
// others made before their call.  It also re-arms the counter for the next use.
__device__ __forceinline__ bool last_block_arrives(unsigned int* counter, unsigned int expected,
                                                   int* lds_flag) {
  // The barrier orders every thread's earlier global writes before thread 0's
  // device-scope release; one wavefront pays for the cache write-back /
  // invalidate instead of all of them.
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t =
        __hip_atomic_fetch_add(counter, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (t == expected - 1u);
    if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *lds_flag = last;
  }
  __syncthreads();
  return *lds_flag != 0;
}

}  // namespace sd
