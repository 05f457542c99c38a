// Bandwidth-bound kernels of the network: gated linear unit and per-frame log-softmax.
// (The paper's tensor library fuses such chains of simple ops into one kernel, Sec. 2.1;
// here each is one hand-fused pass: every input read once, every output written once.)
#include "common.h"

namespace w2l {
namespace {


// ---- GLU ---------------------------------------------------------------------------
// Vector path: 8 channels per thread (16-byte bf16 loads, 2x16-byte fp32 loads).
struct alignas(16) bf16x8 { bf16_t v[8]; };
struct alignas(16) f32x4 { float v[4]; };

template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* o) {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        // plain load: the producer kernel has usually just written these values and they are still in the memory-side cache
        const u4 r = *reinterpret_cast<const u4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = bf16_to_f32((bf16_t)(r[i] & 0xffffu));
            o[2 * i + 1] = bf16_to_f32((bf16_t)(r[i] >> 16));
        }
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float* o) {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        u4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (unsigned)f32_to_bf16(o[2 * i]) | ((unsigned)f32_to_bf16(o[2 * i + 1]) << 16);
        __builtin_nontemporal_store(r, reinterpret_cast<u4*>(p));
    }
};
template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float* p, float* o) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 a = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p)), b = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p) + 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[i] = a[i]; o[4 + i] = b[i]; }
    }
    static __device__ __forceinline__ void store(float* p, const float* o) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        f4 a, b;
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = o[i]; b[i] = o[4 + i]; }
        __builtin_nontemporal_store(a, reinterpret_cast<f4*>(p));
        __builtin_nontemporal_store(b, reinterpret_cast<f4*>(p) + 1);
    }
};

// Output rows run over every frame of the output allocation: B*pitch + slack frames.  Frame f
// belongs to utterance b = f / pitch at time t = f % pitch - halo; it is real iff 0 <= t < Tp
// (then its dense source row is b*Tp + t), otherwise it is a halo/slack frame and gets zeros.
struct RowMap {
    int Tp, pitch, halo;
    long long real_frames;  // B * pitch
    // IDX: long long, or unsigned where every frame index fits (the 64-bit division is slow)
    template <typename IDX>
    __device__ __forceinline__ long long src(IDX f) const
    {
        if (pitch == Tp) return (long long)f < real_frames ? (long long)f : -1;
        if ((long long)f >= real_frames) return -1;
        const IDX b = f / (IDX)pitch;
        const int t = (int)(f - b * (IDX)pitch) - halo;
        return (t >= 0 && t < Tp) ? (long long)b * Tp + t : -1;
    }
};

// IDX: the type of the flat element index -- unsigned where the element count fits 32 bits (the launchers
// choose): a 64-bit division per element costs more than the rest of the element's work
template <typename T, int V, typename IDX>  // V = 8 (vector path, H % 8 == 0) or 1
__global__ __launch_bounds__(256) void glu_fwd_k(const T* __restrict__ y, T* __restrict__ h, long long out_rows,
                                                 int H, RowMap map)
{
    const int hv = H / V;
    const IDX total = (IDX)(out_rows * hv);
    for (IDX i = blockIdx.x * (IDX)blockDim.x + threadIdx.x; i < total; i += (IDX)gridDim.x * blockDim.x) {
        const IDX f = i / (IDX)hv;
        const int c = (int)(i - f * hv) * V;
        const long long r = map.src(f);
        float o[V];
        if (r >= 0) {
            float a[V], g[V];
            if (V == 8) {
                Vec8<T>::load(y + r * 2 * H + c, a);
                Vec8<T>::load(y + r * 2 * H + H + c, g);
            } else {
                a[0] = Elem<T>::load(y, r * 2 * H + c);
                g[0] = Elem<T>::load(y, r * 2 * H + H + c);
            }
#pragma unroll
            for (int j = 0; j < V; ++j) o[j] = a[j] * sigmoidf_(g[j]);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) o[j] = 0.f;
        }
        if (V == 8) Vec8<T>::store(h + (size_t)f * H + c, o);
        else Elem<T>::store(h, (size_t)f * H + c, o[0]);
    }
}

template <typename T, int V, typename IDX>
__global__ __launch_bounds__(256) void glu_bwd_k(const T* __restrict__ y, const T* __restrict__ dh,
                                                 T* __restrict__ dy, long long out_rows, int H, RowMap map)
{
    const int hv = H / V;
    const IDX total = (IDX)(out_rows * hv);
    for (IDX i = blockIdx.x * (IDX)blockDim.x + threadIdx.x; i < total; i += (IDX)gridDim.x * blockDim.x) {
        const IDX f = i / (IDX)hv;
        const int c = (int)(i - f * hv) * V;
        const long long r = map.src(f);
        float da[V], dg[V];
        if (r >= 0) {
            float a[V], g[V], d[V];
            if (V == 8) {
                Vec8<T>::load(y + r * 2 * H + c, a);
                Vec8<T>::load(y + r * 2 * H + H + c, g);
                Vec8<T>::load(dh + r * H + c, d);
            } else {
                a[0] = Elem<T>::load(y, r * 2 * H + c);
                g[0] = Elem<T>::load(y, r * 2 * H + H + c);
                d[0] = Elem<T>::load(dh, r * H + c);
            }
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float sg = sigmoidf_(g[j]);
                da[j] = d[j] * sg;
                dg[j] = d[j] * a[j] * sg * (1.f - sg);
            }
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) { da[j] = 0.f; dg[j] = 0.f; }
        }
        if (V == 8) {
            Vec8<T>::store(dy + (size_t)f * 2 * H + c, da);
            Vec8<T>::store(dy + (size_t)f * 2 * H + H + c, dg);
        } else {
            Elem<T>::store(dy, (size_t)f * 2 * H + c, da[0]);
            Elem<T>::store(dy, (size_t)f * 2 * H + H + c, dg[0]);
        }
    }
}

// dense [B*Tp, C] -> haloed layout (zeros in halo and slack frames); C % 8 == 0, bf16
__global__ __launch_bounds__(256) void pad_layout_k(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                                    long long out_rows, int C, RowMap map, int* __restrict__ clear,
                                                    int nclear)
{
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < nclear; i += blockDim.x) clear[i] = 0;
    const int cv = C / 8;
    const long long total = out_rows * cv;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long f = i / cv;
        const int c = (int)(i - f * cv) * 8;
        const long long r = map.src(f);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r >= 0) v = *reinterpret_cast<const uint4*>(src + r * C + c);
        *reinterpret_cast<uint4*>(dst + f * C + c) = v;
    }
}

// two tensors with the same time layout in one launch (the weight gradient stages x and dy)
__global__ __launch_bounds__(256) void pad_layout2_k(const bf16_t* __restrict__ src0, bf16_t* __restrict__ dst0, int C0,
                                                     const bf16_t* __restrict__ src1, bf16_t* __restrict__ dst1, int C1,
                                                     long long out_rows, RowMap map)
{
    const int cv0 = C0 / 8, cv1 = C1 / 8;
    const long long n0 = out_rows * cv0, total = n0 + out_rows * cv1;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const bool second = i >= n0;
        const long long e = second ? i - n0 : i;
        const int cv = second ? cv1 : cv0, C = second ? C1 : C0;
        const bf16_t* src = second ? src1 : src0;
        bf16_t* dst = second ? dst1 : dst0;
        const long long f = e / cv;
        const int c = (int)(e - f * cv) * 8;
        const long long r = map.src(f);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r >= 0) v = *reinterpret_cast<const uint4*>(src + r * C + c);
        *reinterpret_cast<uint4*>(dst + f * C + c) = v;
    }
}

// the same for any dtype and channel count, one element per thread
template <typename T>
__global__ __launch_bounds__(256) void pad_layout_any_k(const T* __restrict__ src, T* __restrict__ dst, long long out_rows,
                                                        int C, RowMap map)
{
    const long long total = out_rows * C;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long f = i / C;
        const long long r = map.src(f);
        dst[i] = r >= 0 ? src[r * C + (i - f * C)] : T(0);
    }
}

// Operand preparation for data gradients the MFMA kernels do not take as they come (fp32 dy, a channel count that
// is not a multiple of 64, a strided layer): dy -> bf16, haloed, channels padded with zeros to Cp.
template <typename T>
__global__ __launch_bounds__(256) void prep_dy_k(const T* __restrict__ src, bf16_t* __restrict__ dst, long long out_rows,
                                                 int C, int Cp, RowMap map, int* __restrict__ clear, int nclear)
{
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < nclear; i += blockDim.x) clear[i] = 0;
    // one thread writes 8 channels (16 bytes); Cp is a multiple of 64
    const int cv = Cp / 8;
    const long long total = out_rows * cv;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long f = i / cv;
        const int c = (int)(i - f * cv) * 8;
        const long long r = map.src(f);
        bf16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = (r >= 0 && c + e < C) ? f32_to_bf16(Elem<T>::load(src, r * C + c + e)) : (bf16_t)0;
        *reinterpret_cast<uint4*>(dst + f * Cp + c) = *reinterpret_cast<const uint4*>(v);
    }
}
// w[Cout][k][Cin] -> w'[Cp][kf][s * Cin]: w'[co][jj][ph * Cin + ci] = w[co][s * jj + ph][ci], zero where the tap
// s * jj + ph does not exist or co >= Cout (s = 1: a copy with zero rows appended).
__global__ __launch_bounds__(256) void prep_w_k(const bf16_t* __restrict__ w, bf16_t* __restrict__ dst, int Cout, int k,
                                                int Cin, int Cp, int kf, int s)
{
    const long long total = (long long)Cp * kf * s * Cin;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const int ci = (int)(i % Cin);
        const long long q = i / Cin;
        const int ph = (int)(q % s);
        const long long q2 = q / s;
        const int jj = (int)(q2 % kf), co = (int)(q2 / kf);
        const int j = s * jj + ph;
        dst[i] = (co < Cout && j < k) ? w[((size_t)co * k + j) * Cin + ci] : (bf16_t)0;
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

namespace w2l {

namespace {
template <typename T, int V, typename IDX>
void launch_glu_fwd(dim3 g, hipStream_t st, const void* y, void* h, long long out_rows, int H, const RowMap& map)
{
    hipLaunchKernelGGL((glu_fwd_k<T, V, IDX>), g, dim3(256), 0, st, (const T*)y, (T*)h, out_rows, H, map);
}
template <typename T, int V, typename IDX>
void launch_glu_bwd(dim3 g, hipStream_t st, const void* y, const void* dh, void* dy, long long out_rows, int H, const RowMap& map)
{
    hipLaunchKernelGGL((glu_bwd_k<T, V, IDX>), g, dim3(256), 0, st, (const T*)y, (const T*)dh, (T*)dy, out_rows, H, map);
}
}  // namespace

int glu_fwd_layout(const void* y, void* h, int B, int Tp, int Cout, int dtype, int pitch, int halo, int slack,
                   hipStream_t st)
{
    const int H = Cout / 2;
    const bool vec = (H % 8) == 0;
    const long long out_rows = (long long)B * pitch + slack;
    const RowMap map{Tp, pitch, halo, (long long)B * pitch};
    const long long items = vec ? out_rows * (H / 8) : out_rows * H;
    const dim3 g(grid_for(items));
    const bool small = items < (1LL << 31);  // 32-bit element indices
#define W2L_GLU(T_, V_)                                                                    \
    {                                                                                      \
        if (small) launch_glu_fwd<T_, V_, unsigned>(g, st, y, h, out_rows, H, map);        \
        else launch_glu_fwd<T_, V_, long long>(g, st, y, h, out_rows, H, map);             \
    }
    if (dtype == W2L_BF16) {
        if (vec) W2L_GLU(bf16_t, 8) else W2L_GLU(bf16_t, 1)
    } else {
        if (vec) W2L_GLU(float, 8) else W2L_GLU(float, 1)
    }
#undef W2L_GLU
    return launch_status();
}

int glu_bwd_layout(const void* y, const void* dh, void* dy, int B, int Tp, int Cout, int dtype, int pitch, int halo,
                   int slack, hipStream_t st)
{
    const int H = Cout / 2;
    const bool vec = (H % 8) == 0;
    const long long out_rows = (long long)B * pitch + slack;
    const RowMap map{Tp, pitch, halo, (long long)B * pitch};
    const long long items = vec ? out_rows * (H / 8) : out_rows * H;
    const dim3 g(grid_for(items));
    const bool small = items < (1LL << 31);
#define W2L_GLU(T_, V_)                                                                    \
    {                                                                                      \
        if (small) launch_glu_bwd<T_, V_, unsigned>(g, st, y, dh, dy, out_rows, H, map);   \
        else launch_glu_bwd<T_, V_, long long>(g, st, y, dh, dy, out_rows, H, map);        \
    }
    if (dtype == W2L_BF16) {
        if (vec) W2L_GLU(bf16_t, 8) else W2L_GLU(bf16_t, 1)
    } else {
        if (vec) W2L_GLU(float, 8) else W2L_GLU(float, 1)
    }
#undef W2L_GLU
    return launch_status();
}

}  // namespace w2l

namespace w2l {
int pad_layout_bf16(const void* src, void* dst, int B, int Tp, int C, int pitch, int halo, int slack, hipStream_t st,
                    int* clear, int nclear)
{
    const long long out_rows = (long long)B * pitch + slack;
    const RowMap map{Tp, pitch, halo, (long long)B * pitch};
    hipLaunchKernelGGL(pad_layout_k, dim3(grid_for(out_rows * (C / 8))), dim3(256), 0, st, (const bf16_t*)src,
                       (bf16_t*)dst, out_rows, C, map, clear, nclear);
    return launch_status();
}

int pad_layout(const void* src, void* dst, int B, int Tp, int C, int dtype, int pitch, int halo, int slack, hipStream_t st)
{
    if (dtype == W2L_BF16 && C % 8 == 0) return pad_layout_bf16(src, dst, B, Tp, C, pitch, halo, slack, st);
    const long long out_rows = (long long)B * pitch + slack;
    const RowMap map{Tp, pitch, halo, (long long)B * pitch};
    const dim3 g(grid_for(out_rows * C)), b(256);
    if (dtype == W2L_BF16)
        hipLaunchKernelGGL(pad_layout_any_k<bf16_t>, g, b, 0, st, (const bf16_t*)src, (bf16_t*)dst, out_rows, C, map);
    else
        hipLaunchKernelGGL(pad_layout_any_k<float>, g, b, 0, st, (const float*)src, (float*)dst, out_rows, C, map);
    return launch_status();
}

int prep_dgrad_dy(const void* src, int src_dtype, void* dst, int B, int Tp, int C, int Cp, int pitch, int halo, int slack,
                  hipStream_t st, int* clear, int nclear)
{
    const long long out_rows = (long long)B * pitch + slack;
    const RowMap map{Tp, pitch, halo, (long long)B * pitch};
    if (src_dtype == W2L_BF16 && C == Cp) return pad_layout_bf16(src, dst, B, Tp, C, pitch, halo, slack, st, clear, nclear);
    const dim3 g(grid_for(out_rows * (Cp / 8))), b(256);
    if (src_dtype == W2L_BF16)
        hipLaunchKernelGGL(prep_dy_k<bf16_t>, g, b, 0, st, (const bf16_t*)src, (bf16_t*)dst, out_rows, C, Cp, map, clear, nclear);
    else
        hipLaunchKernelGGL(prep_dy_k<float>, g, b, 0, st, (const float*)src, (bf16_t*)dst, out_rows, C, Cp, map, clear, nclear);
    return launch_status();
}

int prep_dgrad_w(const void* w, void* dst, int Cout, int k, int Cin, int Cp, int kf, int s, hipStream_t st)
{
    hipLaunchKernelGGL(prep_w_k, dim3(grid_for((long long)Cp * kf * s * Cin)), dim3(256), 0, st, (const bf16_t*)w,
                       (bf16_t*)dst, Cout, k, Cin, Cp, kf, s);
    return launch_status();
}

int pad_layout2_bf16(const void* src0, void* dst0, int C0, const void* src1, void* dst1, int C1, int B, int Tp, int pitch,
                     int halo, int slack, hipStream_t st)
{
    if (C0 % 8 || C1 % 8) return W2L_ERR_SHAPE;
    const long long out_rows = (long long)B * pitch + slack;
    const RowMap map{Tp, pitch, halo, (long long)B * pitch};
    hipLaunchKernelGGL(pad_layout2_k, dim3(grid_for(out_rows * ((C0 + C1) / 8))), dim3(256), 0, st, (const bf16_t*)src0,
                       (bf16_t*)dst0, C0, (const bf16_t*)src1, (bf16_t*)dst1, C1, out_rows, map);
    return launch_status();
}
}  // namespace w2l

extern "C" int w2l_glu_fwd(const void* y, void* h, long long rows, int Cout, int dtype, void* stream)
{
    if (!y || !h) return W2L_ERR_NULL;
    if (rows <= 0 || rows > 2147483647LL || Cout <= 0 || (Cout & 1)) return W2L_ERR_SHAPE;
    if (!valid_dtype(dtype)) return W2L_ERR_DTYPE;
    if (!aligned16(y) || !aligned16(h)) return W2L_ERR_ALIGN;
    return glu_fwd_layout(y, h, 1, (int)rows, Cout, dtype, (int)rows, 0, 0, (hipStream_t)stream);
}

extern "C" int w2l_glu_bwd(const void* y, const void* dh, void* dy, long long rows, int Cout, int dtype,
                           void* stream)
{
    if (!y || !dh || !dy) return W2L_ERR_NULL;
    if (rows <= 0 || rows > 2147483647LL || Cout <= 0 || (Cout & 1)) return W2L_ERR_SHAPE;
    if (!valid_dtype(dtype)) return W2L_ERR_DTYPE;
    if (!aligned16(y) || !aligned16(dh) || !aligned16(dy)) return W2L_ERR_ALIGN;
    return glu_bwd_layout(y, dh, dy, 1, (int)rows, Cout, dtype, (int)rows, 0, 0, (hipStream_t)stream);
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

// ---- SGD with momentum ----------------------------------------------------------------
// 22 bytes of HBM traffic per parameter (read w, v, grad; write w, v and the bf16 copy): 16-byte accesses, two
// groups of four parameters per thread (a whole grid apart, all six loads issued before the first use) and a grid
// that covers the tensor in one pass.  A wavefront that loads, computes, stores and ends keeps more of the memory
// system busy than one that loops: 6.4 TB/s against 4.6 for a grid-stride loop over a grid capped at 4096 blocks.
namespace {
constexpr int SGD_PER_THREAD = 2;
__global__ __launch_bounds__(256) void sgd_momentum_k(float* __restrict__ w, float* __restrict__ v,
                                                      const float* __restrict__ g, w2l::bf16_t* __restrict__ lowp,
                                                      long long n, float lr, float mu, float wd)
{
    const long long n4 = n / 4;
    // every value is touched exactly once: streaming (non-temporal) loads and stores keep it out of the caches
    typedef float f4 __attribute__((ext_vector_type(4)));
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const long long t0 = blockIdx.x * (long long)blockDim.x + threadIdx.x, stride = (long long)gridDim.x * blockDim.x;
    f4 wv[SGD_PER_THREAD], vv[SGD_PER_THREAD], gv[SGD_PER_THREAD];
#pragma unroll
    for (int u = 0; u < SGD_PER_THREAD; ++u) {
        const long long i = t0 + u * stride;
        if (i < n4) {
            wv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(w) + i);
            vv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(v) + i);
            gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g) + i);
        }
    }
#pragma unroll
    for (int u = 0; u < SGD_PER_THREAD; ++u) {
        const long long i = t0 + u * stride;
        if (i < n4) {
            f4 &wq = wv[u], &vq = vv[u];
            const f4 gq = gv[u];
            vq.x = mu * vq.x + (gq.x + wd * wq.x); wq.x -= lr * vq.x;
            vq.y = mu * vq.y + (gq.y + wd * wq.y); wq.y -= lr * vq.y;
            vq.z = mu * vq.z + (gq.z + wd * wq.z); wq.z -= lr * vq.z;
            vq.w = mu * vq.w + (gq.w + wd * wq.w); wq.w -= lr * vq.w;
            __builtin_nontemporal_store(wq, reinterpret_cast<f4*>(w) + i);
            __builtin_nontemporal_store(vq, reinterpret_cast<f4*>(v) + i);
            if (lowp) {
                u2 o;
                o.x = (unsigned)w2l::f32_to_bf16(wq.x) | ((unsigned)w2l::f32_to_bf16(wq.y) << 16);
                o.y = (unsigned)w2l::f32_to_bf16(wq.z) | ((unsigned)w2l::f32_to_bf16(wq.w) << 16);
                __builtin_nontemporal_store(o, reinterpret_cast<u2*>(lowp) + i);
            }
        }
    }
    // tail (n % 4 values)
    const long long t = n4 * 4 + t0;
    if (t < n) {
        const float vn = mu * v[t] + (g[t] + wd * w[t]);
        const float wn = w[t] - lr * vn;
        v[t] = vn;
        w[t] = wn;
        if (lowp) lowp[t] = w2l::f32_to_bf16(wn);
    }
}
}  // namespace

extern "C" int w2l_sgd_momentum_step(float* w, float* v, const float* grad, void* w_lowp, long long n, float lr,
                                     float momentum, float weight_decay, void* stream)
{
    using namespace w2l;
    if (!w || !v || !grad) return W2L_ERR_NULL;
    if (n < 0) return W2L_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(v) || !aligned16(grad) || (w_lowp && !aligned16(w_lowp))) return W2L_ERR_ALIGN;
    if (n == 0) return W2L_OK;
    const long long n4 = n / 4 > 0 ? n / 4 : 1;
    const long long blocks = (n4 + 256 * SGD_PER_THREAD - 1) / (256 * SGD_PER_THREAD);
    if (blocks > 2147483647LL) return W2L_ERR_SHAPE;
    hipLaunchKernelGGL(sgd_momentum_k, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, w, v, grad,
                       static_cast<bf16_t*>(w_lowp), n, lr, momentum, weight_decay);
    return launch_status();
}
