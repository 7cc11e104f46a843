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
// Slabs of MAX_ROWS rows one batched GEMM launch takes; also the slab count of the fragment-order
// activation buffers ([K/32][GEMM_WIDE_RT][64 lanes][8]) that the producing kernels may write directly.
constexpr int GEMM_WIDE_RT = 6;

struct SeqState {
  int32_t len;                 // committed tokens
  int32_t last_tok;            // token at position len-1
  int32_t prev_tok;            // token at position len-2 (undefined when len < 2)
  int32_t n;                   // accepted guesses of the last iteration
  int32_t x[16];               // guesses x_1..x_gamma of this iteration
  int32_t out[16];             // tokens emitted by the last iteration, -1 padded
  int32_t fallbacks;           // zero-residual fallbacks taken so far
  int32_t pad[3];
  float   beta[16];            // acceptance probabilities beta_1..beta_gamma of the last iteration (when asked for)
};

// Per-call parameters that change between iterations; they live in device
// memory so that a captured graph can be replayed unchanged.
struct StepParams {
  double log_lenience;         // ln(lenience), for the argmax-sampling variant of the lenient test
  float temperature;
  float lenience;              // factor l of the lenient acceptance test, 1 = the exact algorithm
  float uniforms[2 * 15 + 1];  // [0,g) draft draws, [g,2g) accept tests, [2g] final draw
  float top_p;                 // nucleus mass, outside (0,1) = off
  int32_t top_k;               // top-k sampling, 0 = off
  int32_t pad;
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

// ---------------------------------------------------------------------------
// Cross-lane combines that stay in the vector ALU: DPP quad permutes and row
// rotations inside a row of 16 lanes, and the gfx950 half-swap instructions
// across rows.  (ds_bpermute-based shuffles go through the LDS pipe, which the
// attention and sampling kernels need for data.)  lane_combine<OFF>(v, op)
// returns op(v, v of the partner lane) in every lane; the partner is lane^OFF
// for OFF in {1, 2, 8, 16, 32} and lane+4 (mod 16, same row) for OFF == 4.
// ---------------------------------------------------------------------------
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

template <int OFF> __device__ __forceinline__ unsigned dpp_partner(unsigned v) {
  constexpr int ctrl = (OFF == 1) ? 0xB1 : (OFF == 2) ? 0x4E : (OFF == 4) ? 0x124 : 0x128;
  return (unsigned)__builtin_amdgcn_mov_dpp((int)v, ctrl, 0xf, 0xf, true);
}
template <int OFF> __device__ __forceinline__ u32x2 half_swap(unsigned v) {
  if (OFF == 16) return __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return __builtin_amdgcn_permlane32_swap(v, v, false, false);
}

template <typename V> struct Words;
template <> struct Words<float> {
  static constexpr int N = 1;
  static __device__ __forceinline__ void split(float v, unsigned (&w)[2]) { w[0] = __float_as_uint(v); w[1] = 0; }
  static __device__ __forceinline__ float join(const unsigned (&w)[2]) { return __uint_as_float(w[0]); }
};
template <> struct Words<int> {
  static constexpr int N = 1;
  static __device__ __forceinline__ void split(int v, unsigned (&w)[2]) { w[0] = (unsigned)v; w[1] = 0; }
  static __device__ __forceinline__ int join(const unsigned (&w)[2]) { return (int)w[0]; }
};
template <> struct Words<double> {
  static constexpr int N = 2;
  static __device__ __forceinline__ void split(double v, unsigned (&w)[2]) {
    const unsigned long long u = (unsigned long long)__double_as_longlong(v);
    w[0] = (unsigned)u; w[1] = (unsigned)(u >> 32);
  }
  static __device__ __forceinline__ double join(const unsigned (&w)[2]) {
    return __longlong_as_double((long long)(((unsigned long long)w[1] << 32) | w[0]));
  }
};

template <int OFF, typename V, typename Op>
__device__ __forceinline__ V lane_combine(V v, Op op) {
  unsigned w[2];
  Words<V>::split(v, w);
  if (OFF < 16) {
    unsigned o[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < Words<V>::N; ++i) o[i] = dpp_partner<OFF>(w[i]);
    return op(v, Words<V>::join(o));
  } else {
    unsigned x[2] = {0, 0}, y[2] = {0, 0};     // {own, partner} in an order that depends on the lane
#pragma unroll
    for (int i = 0; i < Words<V>::N; ++i) { const u32x2 r = half_swap<OFF>(w[i]); x[i] = r.x; y[i] = r.y; }
    return op(Words<V>::join(x), Words<V>::join(y));
  }
}

// The value that lane 0 of this lane's row of 16 holds.  (After the four in-row steps of a sum every
// lane holds a total, but the rotation of the OFF == 4 step gives the quads two different
// association orders; code that must agree bit for bit with code that reads lane 0's total
// takes lane 0's too.)
__device__ __forceinline__ float row_first(float v) {
  const int w = __builtin_bit_cast(int, v);
  const int a = __builtin_amdgcn_readlane(w, 0), b = __builtin_amdgcn_readlane(w, 16);
  const int c = __builtin_amdgcn_readlane(w, 32), d = __builtin_amdgcn_readlane(w, 48);
  const int lane = (int)(threadIdx.x & 63);
  return __builtin_bit_cast(float, lane < 16 ? a : (lane < 32 ? b : (lane < 48 ? c : d)));
}

// All 64 lanes get op over the wavefront (op must be commutative; the
// association order is fixed per lane, so results are run-to-run identical).
template <typename V, typename Op>
__device__ __forceinline__ V wave_allreduce(V v, Op op) {
  v = lane_combine<1>(v, op); v = lane_combine<2>(v, op); v = lane_combine<4>(v, op);
  v = lane_combine<8>(v, op); v = lane_combine<16>(v, op); v = lane_combine<32>(v, op);
  return v;
}

struct OpSumF { __device__ float operator()(float a, float b) const { return a + b; } };
struct OpSumD { __device__ double operator()(double a, double b) const { return a + b; } };
struct OpMaxF { __device__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpMinI { __device__ int operator()(int a, int b) const { return min(a, b); } };
struct OpSumI { __device__ int operator()(int a, int b) const { return a + b; } };
struct OpMaxI { __device__ int operator()(int a, int b) const { return max(a, b); } };

__device__ __forceinline__ float wave_sum(float v) { return wave_allreduce(v, OpSumF()); }
__device__ __forceinline__ double wave_sum(double v) { return wave_allreduce(v, OpSumD()); }
__device__ __forceinline__ float wave_max(float v) { return wave_allreduce(v, OpMaxF()); }
__device__ __forceinline__ int wave_min(int v) { return wave_allreduce(v, OpMinI()); }
__device__ __forceinline__ int wave_max(int v) { return wave_allreduce(v, OpMaxI()); }

// Workgroup-wide reductions over up to 16 waves.  `red` is LDS scratch of at
// least 16 elements of the value type; every thread gets the result.  The
// combine order is fixed (wave 0..n-1), so results are run-to-run identical.
template <typename V, typename Op>
__device__ __forceinline__ V block_reduce(V v, V* red, Op op, V identity) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_allreduce(v, op);
  __syncthreads();                       // protect `red` from the previous use
  if (lane == 0) red[wave] = v;
  __syncthreads();
  V r = identity;
  for (int w = 0; w < nw; ++w) r = op(r, red[w]);
  return r;
}

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
