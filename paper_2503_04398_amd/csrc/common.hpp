// Shared host/device helpers of the library: status handling, config validation, workspace carving,
// bf16 conversion.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "semmoe.h"

namespace semmoe {

constexpr int kWave = 64;

// ---- status -------------------------------------------------------------------------------------
void set_last_hip_error(hipError_t e);

#define SEMMOE_HIP(expr)                                  \
  do {                                                    \
    hipError_t _e = (expr);                               \
    if (_e != hipSuccess) {                               \
      ::semmoe::set_last_hip_error(_e);                   \
      return SEMMOE_EHIP;                                 \
    }                                                     \
  } while (0)

#define SEMMOE_LAUNCH_CHECK() SEMMOE_HIP(hipGetLastError())

// Shape rules every call shares.  `need_ffn`: d and F are used; `need_T`: cfg->T is used.
int32_t validate_config(const semmoe_config* cfg, bool need_T, bool need_rows, bool need_ffn);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline size_t act_bytes(const semmoe_config* cfg) { return cfg->dtype == SEMMOE_BF16 ? 2 : 4; }

// Sequential carving of the caller's workspace.
struct Carver {
  char* base;
  size_t size, off;
  bool ok;
  Carver(void* ws, size_t bytes) : base(static_cast<char*>(ws)), size(bytes), off(0), ok(ws != nullptr) {}
  template <typename T>
  T* take(size_t n) {
    size_t start = align_up(off, 256);
    size_t end = start + n * sizeof(T);
    if (!ok || end > size) {
      ok = false;
      off = end;
      return nullptr;
    }
    off = end;
    return reinterpret_cast<T*>(base + start);
  }
};

// Workspace needs per call (bytes), shared by semmoe_workspace_bytes and the calls themselves.
constexpr int kTokBlock = 256;  // tokens per workgroup in the index kernels
size_t ws_route(const semmoe_config* cfg);
size_t ws_reshuffle(const semmoe_config* cfg);
size_t ws_dispatch(const semmoe_config* cfg);
size_t ws_ffn(const semmoe_config* cfg);
size_t ws_request(const semmoe_config* cfg);
int tuning_value(int key);  // current value of a SEMMOE_TUNE_* knob (-1: default)

// ---- device helpers -----------------------------------------------------------------------------
typedef uint16_t bf16_t;  // storage of a bf16 value

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(static_cast<uint32_t>(v) << 16); }

// round to nearest, ties to even (inputs are finite)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

}  // namespace semmoe
