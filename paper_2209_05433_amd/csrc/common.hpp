// Internal declarations shared by the translation units of libfp8mm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fp8mm.h"

namespace fp8mm {

// Records the message returned by fp8_last_error() on this thread and returns `code`.
int fail(int code, const char* fmt, ...);
void clear_error();

// Turns the state of the HIP runtime after a launch into a status code.
int check_launch(const char* what);

inline bool valid_format(int f) { return f == FP8_E4M3 || f == FP8_E5M2; }
inline bool valid_dtype(int d) { return d == FP8_F32 || d == FP8_BF16; }

// Which implementation the cast kernel uses for the FP8 rounding step.
//   kCastBits : integer bit manipulation written from the format definition
//   kCastCvt  : the gfx950 v_cvt_pk_{fp8,bf8}_f32 instructions, with the saturation and
//               special-value rules applied around them
// The converter path is the default (it was checked against the bit path on all 2^32 inputs);
// the knob FP8_KNOB_CAST_PATH overrides it.
enum CastPath { kCastBits = 0, kCastCvt = 1, kCastBitsStrict = 2 /* non-saturating, kernels only */ };
CastPath cast_path();

// Current value of a tuning knob (fp8_knob_t).  The knobs are process-wide atomics, seeded once
// from the environment (FP8MM_CAST_PATH, FP8MM_TILE_N, FP8MM_GROUP_M, FP8MM_GEMM, FP8MM_SPLIT_K)
// and changed through fp8_set_knob(); no launch path reads the environment.
int knob(int which);

// ---- launchers (each enqueues on `stream` and returns a status) -------------------------
int launch_amax(const void* x, size_t n, int in_dtype, float* amax_out, hipStream_t stream);
int launch_amax_scale(const void* x, size_t n, int in_dtype, int fmt, float* amax_out, float* scale_out, void* workspace,
                      hipStream_t stream);
int launch_amax_scale_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt, float* amax_out,
                            float* scale_out, void* workspace, hipStream_t stream);
int launch_quantize_multi(int count, const void* const* x, const size_t* n, int in_dtype, const int* fmt,
                          const float* scale_dev, uint8_t* const* q_out, hipStream_t stream);
float scale_from_amax_host(float amax, int fmt);
int launch_scale_from_amax(const float* amax, int fmt, float* scale_out, hipStream_t stream);
int launch_quantize(const void* x, size_t n, int in_dtype, int fmt, float scale,
                    const float* scale_dev, bool saturate, uint8_t* q_out, hipStream_t stream);
int launch_quantize_amax(const void* x, size_t n, int in_dtype, int fmt, const float* scale_dev, uint8_t* q_out,
                         float* amax_out, hipStream_t stream);
int launch_quantize_sr(const void* x, size_t n, int in_dtype, int fmt, float scale, const float* scale_dev,
                       uint64_t seed, uint8_t* q_out, hipStream_t stream);
int launch_scale_from_history(const float* hist, size_t len, int fmt, float* scale_out, hipStream_t stream);
int launch_scale_n(const float* amax, size_t n, int fmt, float* scale_out, hipStream_t stream);
int launch_amax_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, float* amax_out, hipStream_t stream);
int launch_quantize_rows(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt, const float* scale_dev,
                         uint8_t* q_out, hipStream_t stream);
int launch_quantize_transpose(const void* x, int64_t rows, int64_t cols, int in_dtype, int fmt, const float* scale_dev,
                              uint8_t* q_out, uint8_t* qt_out, hipStream_t stream);
int launch_dequantize(const uint8_t* q, size_t n, int fmt, float scale, const float* scale_dev,
                      int out_dtype, void* out, hipStream_t stream);

}  // namespace fp8mm
