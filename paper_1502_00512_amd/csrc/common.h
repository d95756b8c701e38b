// Shared device/host definitions of the gfx950 RNNLM library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rnnlm_dev {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// Padding granularities of every internal buffer (elements). All GEMM operands live in
// buffers whose dimensions are multiples of these, with the padding kept at zero (or, where
// stated, merely finite), so the contraction kernels carry no bounds checks.
constexpr int PAD_H = 256;  // hidden dimension
constexpr int PAD_V = 256;  // vocabulary dimension
constexpr int PAD_B = 32;   // streams per timestep
constexpr int PAD_M = 256;  // rows of a window (T * padded B)

__host__ __device__ inline long round_up(long a, long b) { return (a + b - 1) / b * b; }

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int BK = 32;  // K extent of one LDS tile (128 bytes)
  static constexpr int VEC = 4;  // elements per 16-byte access
};
template <>
struct Elem<bf16_t> {
  static constexpr int BK = 64;
  static constexpr int VEC = 8;
};

__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return (float)v; }
template <typename T>
__device__ inline T from_f32(float v);
template <>
__device__ inline float from_f32<float>(float v) { return v; }
template <>
__device__ inline bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // round-to-nearest-even

// Barrier and ticket counters of the persistent recurrent kernels.  Every counter has a 256-byte line to itself:
// polls queue at the address they read, and with the counters of all eight XCDs in one line (or all workgroups
// of the chip polling one word) an arrival took several microseconds to become visible to the pollers instead
// of under one.  kind 0 (x = 0): the whole grid's counter of the chip-wide exchange; kind 1: step barrier of the
// group on XCD x; kind 2: ticket dispenser of XCD x; kinds 3 and 4: the two levels of the resident kernel's
// chip-wide barrier (arrivals of XCD x's workgroups; XCDs that have fully arrived, one copy per XCD).
constexpr int SYNC_WORDS = 5 * 8 * 64;
__host__ __device__ inline int sync_word(int kind, int x) { return (kind * 8 + x) * 64; }

__device__ inline float sigmoidf_(float a) { return 1.0f / (1.0f + __expf(-a)); }

}  // namespace rnnlm_dev
