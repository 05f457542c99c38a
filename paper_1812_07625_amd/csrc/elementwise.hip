// Bandwidth-bound kernels of the network: gated linear unit and per-frame log-softmax.
// (The paper's tensor library fuses such chains of simple ops into one kernel, Sec. 2.1;
// here each is one hand-fused pass: every input read once, every output written once.)
#include "common.h"

namespace w2l {
namespace {

__device__ __forceinline__ float sigmoidf_(float u) { return 1.f / (1.f + __expf(-u)); }

// ---- GLU ---------------------------------------------------------------------------
// Vector path: 8 channels per thread (16-byte bf16 loads, 2x16-byte fp32 loads).
struct alignas(16) bf16x8 { bf16_t v[8]; };
struct alignas(16) f32x4 { float v[4]; };

template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* o) {
        bf16x8 r = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = bf16_to_f32(r.v[i]);
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float* o) {
        bf16x8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r.v[i] = f32_to_bf16(o[i]);
        *reinterpret_cast<bf16x8*>(p) = r;
    }
};
template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float* p, float* o) {
        f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[i] = a.v[i]; o[4 + i] = b.v[i]; }
    }
    static __device__ __forceinline__ void store(float* p, const float* o) {
        f32x4 a, b;
#pragma unroll
        for (int i = 0; i < 4; ++i) { a.v[i] = o[i]; b.v[i] = o[4 + i]; }
        *reinterpret_cast<f32x4*>(p) = a;
        *reinterpret_cast<f32x4*>(p + 4) = b;
    }
};

template <typename T>
__global__ __launch_bounds__(256) void glu_fwd_vec(const T* __restrict__ y, T* __restrict__ h,
                                                   long long rows, int H)
{
    const int hv = H / 8;
    const long long total = rows * hv;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / hv;
        const int c = (int)(i - r * hv) * 8;
        float a[8], g[8], o[8];
        Vec8<T>::load(y + r * 2 * H + c, a);
        Vec8<T>::load(y + r * 2 * H + H + c, g);
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = a[j] * sigmoidf_(g[j]);
        Vec8<T>::store(h + r * H + c, o);
    }
}
template <typename T>
__global__ __launch_bounds__(256) void glu_fwd_scalar(const T* __restrict__ y, T* __restrict__ h,
                                                      long long rows, int H)
{
    const long long total = rows * H;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / H;
        const int c = (int)(i - r * H);
        const float a = Elem<T>::load(y, r * 2 * H + c), g = Elem<T>::load(y, r * 2 * H + H + c);
        Elem<T>::store(h, i, a * sigmoidf_(g));
    }
}
template <typename T>
__global__ __launch_bounds__(256) void glu_bwd_vec(const T* __restrict__ y, const T* __restrict__ dh,
                                                   T* __restrict__ dy, long long rows, int H)
{
    const int hv = H / 8;
    const long long total = rows * hv;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / hv;
        const int c = (int)(i - r * hv) * 8;
        float a[8], g[8], d[8], da[8], dg[8];
        Vec8<T>::load(y + r * 2 * H + c, a);
        Vec8<T>::load(y + r * 2 * H + H + c, g);
        Vec8<T>::load(dh + r * H + c, d);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float sg = sigmoidf_(g[j]);
            da[j] = d[j] * sg;
            dg[j] = d[j] * a[j] * sg * (1.f - sg);
        }
        Vec8<T>::store(dy + r * 2 * H + c, da);
        Vec8<T>::store(dy + r * 2 * H + H + c, dg);
    }
}
template <typename T>
__global__ __launch_bounds__(256) void glu_bwd_scalar(const T* __restrict__ y, const T* __restrict__ dh,
                                                      T* __restrict__ dy, long long rows, int H)
{
    const long long total = rows * H;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / H;
        const int c = (int)(i - r * H);
        const float a = Elem<T>::load(y, r * 2 * H + c), g = Elem<T>::load(y, r * 2 * H + H + c);
        const float d = Elem<T>::load(dh, i), sg = sigmoidf_(g);
        Elem<T>::store(dy, r * 2 * H + c, d * sg);
        Elem<T>::store(dy, r * 2 * H + H + c, d * a * sg * (1.f - sg));
    }
}

inline unsigned grid_for(long long items)
{
    long long b = (items + 255) / 256;
    const long long cap = 256 * 16;  // 16 workgroups per CU keep enough loads in flight
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (unsigned)b;
}

// ---- log-softmax: one wavefront per row ----------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <typename T>
__global__ __launch_bounds__(256) void logsoftmax_fwd_k(const T* __restrict__ z, float* __restrict__ lp,
                                                        long long rows, int C)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (blockIdx.x * (long long)blockDim.x + threadIdx.x) >> 6;
    const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
    for (long long r = wave; r < rows; r += nwaves) {
        const T* zr = z + r * C;
        float m = -INFINITY;
        for (int c = lane; c < C; c += 64) m = fmaxf(m, Elem<T>::load(zr, c));
        m = wave_max(m);
        float s = 0.f;
        for (int c = lane; c < C; c += 64) s += expf(Elem<T>::load(zr, c) - m);
        s = wave_sum(s);
        const float lse = m + logf(s);
        for (int c = lane; c < C; c += 64) lp[r * C + c] = Elem<T>::load(zr, c) - lse;
    }
}
__global__ __launch_bounds__(256) void logsoftmax_bwd_k(const float* __restrict__ lp,
                                                        const float* __restrict__ dlp,
                                                        float* __restrict__ dz, long long rows, int C)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (blockIdx.x * (long long)blockDim.x + threadIdx.x) >> 6;
    const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
    for (long long r = wave; r < rows; r += nwaves) {
        float s = 0.f;
        for (int c = lane; c < C; c += 64) s += dlp[r * C + c];
        s = wave_sum(s);
        for (int c = lane; c < C; c += 64) dz[r * C + c] = dlp[r * C + c] - expf(lp[r * C + c]) * s;
    }
}

}  // namespace
}  // namespace w2l

using namespace w2l;

extern "C" int w2l_glu_fwd(const void* y, void* h, long long rows, int Cout, int dtype, void* stream)
{
    if (!y || !h) return W2L_ERR_NULL;
    if (rows <= 0 || Cout <= 0 || (Cout & 1)) return W2L_ERR_SHAPE;
    if (!valid_dtype(dtype)) return W2L_ERR_DTYPE;
    if (!aligned16(y) || !aligned16(h)) return W2L_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int H = Cout / 2;
    const bool vec = (H % 8) == 0;
    const long long items = vec ? rows * (H / 8) : rows * H;
    const dim3 g(grid_for(items)), b(256);
    if (dtype == W2L_BF16) {
        if (vec) hipLaunchKernelGGL(glu_fwd_vec<bf16_t>, g, b, 0, st, (const bf16_t*)y, (bf16_t*)h, rows, H);
        else hipLaunchKernelGGL(glu_fwd_scalar<bf16_t>, g, b, 0, st, (const bf16_t*)y, (bf16_t*)h, rows, H);
    } else {
        if (vec) hipLaunchKernelGGL(glu_fwd_vec<float>, g, b, 0, st, (const float*)y, (float*)h, rows, H);
        else hipLaunchKernelGGL(glu_fwd_scalar<float>, g, b, 0, st, (const float*)y, (float*)h, rows, H);
    }
    return launch_status();
}

extern "C" int w2l_glu_bwd(const void* y, const void* dh, void* dy, long long rows, int Cout, int dtype,
                           void* stream)
{
    if (!y || !dh || !dy) return W2L_ERR_NULL;
    if (rows <= 0 || Cout <= 0 || (Cout & 1)) return W2L_ERR_SHAPE;
    if (!valid_dtype(dtype)) return W2L_ERR_DTYPE;
    if (!aligned16(y) || !aligned16(dh) || !aligned16(dy)) return W2L_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int H = Cout / 2;
    const bool vec = (H % 8) == 0;
    const long long items = vec ? rows * (H / 8) : rows * H;
    const dim3 g(grid_for(items)), b(256);
    if (dtype == W2L_BF16) {
        if (vec) hipLaunchKernelGGL(glu_bwd_vec<bf16_t>, g, b, 0, st, (const bf16_t*)y, (const bf16_t*)dh, (bf16_t*)dy, rows, H);
        else hipLaunchKernelGGL(glu_bwd_scalar<bf16_t>, g, b, 0, st, (const bf16_t*)y, (const bf16_t*)dh, (bf16_t*)dy, rows, H);
    } else {
        if (vec) hipLaunchKernelGGL(glu_bwd_vec<float>, g, b, 0, st, (const float*)y, (const float*)dh, (float*)dy, rows, H);
        else hipLaunchKernelGGL(glu_bwd_scalar<float>, g, b, 0, st, (const float*)y, (const float*)dh, (float*)dy, rows, H);
    }
    return launch_status();
}

extern "C" int w2l_logsoftmax_fwd(const void* z, float* lp, long long rows, int C, int z_dtype, void* stream)
{
    if (!z || !lp) return W2L_ERR_NULL;
    if (rows <= 0 || C <= 0 || C > 4096) return W2L_ERR_SHAPE;
    if (!valid_dtype(z_dtype)) return W2L_ERR_DTYPE;
    if (!aligned16(z) || !aligned16(lp)) return W2L_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const dim3 g(grid_for(rows * 64)), b(256);
    if (z_dtype == W2L_BF16)
        hipLaunchKernelGGL(logsoftmax_fwd_k<bf16_t>, g, b, 0, st, (const bf16_t*)z, lp, rows, C);
    else
        hipLaunchKernelGGL(logsoftmax_fwd_k<float>, g, b, 0, st, (const float*)z, lp, rows, C);
    return launch_status();
}

extern "C" int w2l_logsoftmax_bwd(const float* lp, const float* dlp, float* dz, long long rows, int C,
                                  void* stream)
{
    if (!lp || !dlp || !dz) return W2L_ERR_NULL;
    if (rows <= 0 || C <= 0 || C > 4096) return W2L_ERR_SHAPE;
    if (!aligned16(lp) || !aligned16(dlp) || !aligned16(dz)) return W2L_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(logsoftmax_bwd_k, dim3(grid_for(rows * 64)), dim3(256), 0, st, lp, dlp, dz, rows, C);
    return launch_status();
}
