// Internal helpers of libw2l (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/w2l.h"

namespace w2l {

typedef unsigned short bf16_t;  // raw bits: upper half of an IEEE float

void note_hip_error(hipError_t e);
// status of the launch just made on this thread
inline int launch_status() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    return W2L_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int out_len(int T, int s) { return (T + s - 1) / s; }
inline size_t dtype_size(int dt) { return dt == W2L_BF16 ? 2 : 4; }
inline bool valid_dtype(int dt) { return dt == W2L_F32 || dt == W2L_BF16; }

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, size_t i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
    static __device__ __forceinline__ void store(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }
};

// ---- internal entry points shared between translation units -----------------------
int conv_fwd_generic(const void* x, const void* w, const float* bias, void* y, int B, int T, int Cin,
                     int Cout, int k, int s, int dt, int ydt, hipStream_t st);
int conv_dgrad_generic(const void* dy, const void* w, void* dx, int B, int T, int Cin, int Cout, int k,
                       int s, int dt, int dydt, hipStream_t st);
int conv_wgrad_generic(const void* x, const void* dy, float* dw, int B, int T, int Cin, int Cout, int k,
                       int s, int dt, int dydt, int accumulate, hipStream_t st);
// column sums of dy[rows,Cout] -> dbias, two deterministic stages; scratch holds DBIAS_CHUNKS*Cout floats
enum { DBIAS_CHUNKS = 64 };
int dbias_reduce(const void* dy, float* dbias, long long rows, int Cout, int dydt, int accumulate,
                 float* scratch, hipStream_t st);


// MFMA (bf16 operands, fp32 accumulate) paths; *_ok() says whether a shape is taken
bool conv_fwd_mfma_ok(int B, int T, int Cin, int Cout, int k, int s);
int conv_fwd_mfma(const void* x, const void* w, const float* bias, void* y, int B, int T, int Cin, int Cout,
                  int k, int s, int ydt, hipStream_t st);
bool conv_dgrad_mfma_ok(int B, int T, int Cin, int Cout, int k, int s);
int conv_dgrad_mfma(const void* dy, const void* w, void* dx, int B, int T, int Cin, int Cout, int k, int s,
                    hipStream_t st);
bool conv_wgrad_mfma_ok(int B, int T, int Cin, int Cout, int k, int s);
size_t conv_wgrad_mfma_workspace(int B, int T, int Cin, int Cout, int k, int s);
int conv_wgrad_mfma(const void* x, const void* dy, float* dw, int B, int T, int Cin, int Cout, int k, int s,
                    int accumulate, void* ws, hipStream_t st);

}  // namespace w2l
