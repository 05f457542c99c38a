// Shape-agnostic temporal-convolution kernels (fp32 or bf16 operands, fp32 accumulation).
//
// These back every shape the MFMA kernels do not take (fp32 tensors, channel counts
// that are not multiples of 8, strided data gradients).  Each of the three passes is
// the GEMM C[m,n] = sum_r A(m,r) * B(r,n) over a 64x64 output tile per workgroup,
// 16-deep LDS panels, 4x4 outputs per thread; the operand functors fold the
// convolution's indexing (tap offset, stride, zero padding) into the loads, so no
// unfolded copy of the input is ever made.
//
// Definitions (the paper names the op in Sec. 2.3 without a formula):
//   fwd   y[b,t',co]  = bias[co] + sum_{j,ci} w[co,j,ci] * x[b, s t' + j - p, ci]
//   dgrad dx[b,t,ci]  = sum_{j,co} w[co,j,ci] * dy[b,(t+p-j)/s,co]   (divisible, in range)
//   wgrad dw[co,j,ci] = sum_{b,t'} dy[b,t',co] * x[b, s t' + j - p, ci]
#include "common.h"

namespace w2l {
namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <class AF, class BF, class EP, bool A_RFAST, bool B_RFAST>
__global__ __launch_bounds__(256) void gemm_tiled(AF af, BF bf, EP ep, int M, int N, int R)
{
    __shared__ float As[TK][TM + 1];
    __shared__ float Bs[TK][TN + 1];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int r0 = 0; r0 < R; r0 += TK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * 256;
            int rr, mm;
            if (A_RFAST) { rr = e % TK; mm = e / TK; } else { mm = e % TM; rr = e / TM; }
            const int m = m0 + mm, r = r0 + rr;
            As[rr][mm] = (m < M && r < R) ? af(m, r) : 0.f;
            int nn;
            if (B_RFAST) { rr = e % TK; nn = e / TK; } else { nn = e % TN; rr = e / TN; }
            const int n = n0 + nn;
            const int r2 = r0 + rr;
            Bs[rr][nn] = (n < N && r2 < R) ? bf(r2, n) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int rr = 0; rr < TK; ++rr) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[rr][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[rr][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) ep(m, n, acc[i][j]);
        }
}

// ---- operand functors (time-axis layout: element ((b*pitch + halo + t) * C + c)) ---------
template <typename T>
struct XWindow {  // A(m=(b,t'), r=(j,ci)) = x[b, s t' + j - p, ci]
    const T* x; int T_, Tp, Cin, s, p, pitch, halo;
    __device__ float operator()(int m, int r) const {
        const int b = m / Tp, tp = m - b * Tp;
        const int j = r / Cin, ci = r - j * Cin;
        const int t = s * tp + j - p;
        if (t < 0 || t >= T_) return 0.f;
        return Elem<T>::load(x, ((size_t)b * pitch + halo + t) * Cin + ci);
    }
};
template <typename T>
struct WRows {  // B(r=(j,ci), n=co) = w[co, j, ci]
    const T* w; int KC;
    __device__ float operator()(int r, int n) const { return Elem<T>::load(w, (size_t)n * KC + r); }
};
template <typename T>
struct DyWindow {  // A(m=(b,t), r=(j,co)) = dy[b, (t+p-j)/s, co]
    const T* dy; int T_, Tp, Cout, s, p, pitch, halo;
    __device__ float operator()(int m, int r) const {
        const int b = m / T_, t = m - b * T_;
        const int j = r / Cout, co = r - j * Cout;
        const int u = t + p - j;
        if (u < 0) return 0.f;
        const int tp = u / s;
        if (tp * s != u || tp >= Tp) return 0.f;
        return Elem<T>::load(dy, ((size_t)b * pitch + halo + tp) * Cout + co);
    }
};
template <typename T>
struct WCols {  // B(r=(j,co), n=ci) = w[co, j, ci]
    const T* w; int Cin, Cout, k;
    __device__ float operator()(int r, int n) const {
        const int j = r / Cout, co = r - j * Cout;
        return Elem<T>::load(w, ((size_t)co * k + j) * Cin + n);
    }
};
template <typename T>
struct DyT {  // A(m=co, r=(b,t')) = dy[b,t',co]
    const T* dy; int Tp, Cout, pitch, halo;
    __device__ float operator()(int m, int r) const {
        const int b = r / Tp, tp = r - b * Tp;
        return Elem<T>::load(dy, ((size_t)b * pitch + halo + tp) * Cout + m);
    }
};
template <typename T>
struct XShift {  // B(r=(b,t'), n=(j,ci)) = x[b, s t' + j - p, ci]
    const T* x; int T_, Tp, Cin, s, p, pitch, halo;
    __device__ float operator()(int r, int n) const {
        const int b = r / Tp, tp = r - b * Tp;
        const int j = n / Cin, ci = n - j * Cin;
        const int t = s * tp + j - p;
        if (t < 0 || t >= T_) return 0.f;
        return Elem<T>::load(x, ((size_t)b * pitch + halo + t) * Cin + ci);
    }
};
template <typename T>
struct StoreRows {  // out[b, t, n] = v (+ bias[n]); m = (b,t) over `frames` frames per utterance
    T* y; const float* bias; int N, frames, pitch, halo;
    __device__ void operator()(int m, int n, float v) const {
        const int b = m / frames, t = m - b * frames;
        Elem<T>::store(y, ((size_t)b * pitch + halo + t) * N + n, v + (bias ? bias[n] : 0.f));
    }
};
struct StoreAcc {
    float* d; int N; int accumulate;
    __device__ void operator()(int m, int n, float v) const {
        const size_t i = (size_t)m * N + n;
        d[i] = accumulate ? d[i] + v : v;
    }
};

template <class AF, class BF, class EP, bool AR, bool BR>
int launch(AF af, BF bf, EP ep, long long M, long long N, long long R, hipStream_t st)
{
    const long long gy = (M + TM - 1) / TM, gx = (N + TN - 1) / TN;
    if (gy > 65535 || gx > 2147483647LL || M * 1 > 2147483647LL || R > 2147483647LL) return W2L_ERR_SHAPE;
    hipLaunchKernelGGL((gemm_tiled<AF, BF, EP, AR, BR>), dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, st,
                       af, bf, ep, (int)M, (int)N, (int)R);
    return launch_status();
}

template <typename TI, typename TO>
int fwd_t(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, hipStream_t st)
{
    XWindow<TI> af{(const TI*)x, d.T, d.Tp, d.Cin, d.s, d.p, d.x_pitch, d.x_halo};
    WRows<TI> bf{(const TI*)w, d.k * d.Cin};
    StoreRows<TO> ep{(TO*)y, bias, d.Cout, d.Tp, d.y_pitch, d.y_halo};
    return launch<XWindow<TI>, WRows<TI>, StoreRows<TO>, true, true>(af, bf, ep, (long long)d.B * d.Tp, d.Cout,
                                                                      (long long)d.k * d.Cin, st);
}
template <typename TW, typename TDY>
int dgrad_t(const ConvDesc& d, const void* dy, const void* w, void* dx, hipStream_t st)
{
    DyWindow<TDY> af{(const TDY*)dy, d.T, d.Tp, d.Cout, d.s, d.p, d.y_pitch, d.y_halo};
    WCols<TW> bf{(const TW*)w, d.Cin, d.Cout, d.k};
    StoreRows<TW> ep{(TW*)dx, nullptr, d.Cin, d.T, d.x_pitch, d.x_halo};
    return launch<DyWindow<TDY>, WCols<TW>, StoreRows<TW>, true, false>(af, bf, ep, (long long)d.B * d.T, d.Cin,
                                                                         (long long)d.k * d.Cout, st);
}
template <typename TX, typename TDY>
int wgrad_t(const ConvDesc& d, const void* x, const void* dy, float* dw, int accumulate, hipStream_t st)
{
    DyT<TDY> af{(const TDY*)dy, d.Tp, d.Cout, d.y_pitch, d.y_halo};
    XShift<TX> bf{(const TX*)x, d.T, d.Tp, d.Cin, d.s, d.p, d.x_pitch, d.x_halo};
    StoreAcc ep{dw, d.k * d.Cin, accumulate};
    return launch<DyT<TDY>, XShift<TX>, StoreAcc, false, false>(af, bf, ep, d.Cout, (long long)d.k * d.Cin,
                                                                 (long long)d.B * d.Tp, st);
}

// ---- weight gradient for narrow outputs (Cout <= 32, e.g. the 29 grapheme classes) ---------
// dw[co, n=(j,ci)] = sum_{r=(b,t')} dy[r,co] * x[b, s t' + j - p, ci].  A 64-wide GEMM tile would
// leave all but one tile row empty and serialise the whole reduction in a handful of
// workgroups; here the reduction is cut into SKINNY_CHUNKS row ranges (grid.y), every thread
// owns one column n and keeps all Cout partial sums in registers, and a second pass adds the
// chunks in a fixed order.
constexpr int SKINNY_ROWS = 32;  // dy rows staged in LDS per pass

template <typename TX, typename TDY>
__global__ __launch_bounds__(256) void wgrad_skinny_stage1(const TX* __restrict__ x, const TDY* __restrict__ dy,
                                                           float* __restrict__ part, ConvDesc d)
{
    // 64 columns per workgroup; its four wavefronts take every fourth row of the chunk, so four times as many
    // row loads are in flight per column (the kernel lives on memory latency), and add up through LDS at the end
    __shared__ float dyt[SKINNY_ROWS][32];
    __shared__ float red[3][32][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int N = d.k * d.Cin, R = d.B * d.Tp;
    const int n = blockIdx.x * 64 + lane;
    const int per = (R + gridDim.y - 1) / gridDim.y;
    const int r_begin = per * blockIdx.y, r_end = (r_begin + per < R) ? r_begin + per : R;
    const int j = (n < N) ? n / d.Cin : 0, ci = (n < N) ? n - j * d.Cin : 0;
    float acc[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) acc[c] = 0.f;
    for (int r0 = r_begin; r0 < r_end; r0 += SKINNY_ROWS) {
        for (int e = threadIdx.x; e < SKINNY_ROWS * 32; e += 256) {
            const int rr = e >> 5, c = e & 31, r = r0 + rr;
            float v = 0.f;
            if (r < r_end && c < d.Cout) {
                const int b = r / d.Tp, tp = r - b * d.Tp;
                v = Elem<TDY>::load(dy, ((size_t)b * d.y_pitch + d.y_halo + tp) * d.Cout + c);
            }
            dyt[rr][c] = v;
        }
        __syncthreads();
        if (n < N) {
            // this wavefront's eight rows of the pass: their x values are loaded together (independent loads, one
            // latency); a row outside the utterance or past the chunk contributes 0 (its dy row in LDS is 0 as well)
            float xv[SKINNY_ROWS / 4];
#pragma unroll
            for (int u = 0; u < SKINNY_ROWS / 4; ++u) {
                const int rq = r0 + wave + 4 * u;
                const int r = min(rq, r_end - 1);
                const int b = r / d.Tp, tp = r - b * d.Tp;
                const int t = d.s * tp + j - d.p;
                const bool ok = t >= 0 && t < d.T && rq < r_end;
                const float v = Elem<TX>::load(x, ((size_t)b * d.x_pitch + d.x_halo + (ok ? t : 0)) * d.Cin + ci);
                xv[u] = ok ? v : 0.f;
            }
#pragma unroll
            for (int u = 0; u < SKINNY_ROWS / 4; ++u)
#pragma unroll
                for (int c = 0; c < 32; ++c) acc[c] = fmaf(dyt[wave + 4 * u][c], xv[u], acc[c]);
        }
        __syncthreads();
    }
    if (wave > 0) {
#pragma unroll
        for (int c = 0; c < 32; ++c) red[wave - 1][c][lane] = acc[c];
    }
    __syncthreads();
    if (wave == 0 && n < N)
        for (int c = 0; c < d.Cout; ++c)
            part[((size_t)blockIdx.y * d.Cout + c) * N + n] = ((acc[c] + red[0][c][lane]) + red[1][c][lane]) + red[2][c][lane];
}
__global__ __launch_bounds__(256) void wgrad_skinny_stage2(const float* __restrict__ part, float* __restrict__ dw,
                                                           int chunks, long long total, int accumulate)
{
    const long long i = blockIdx.x * 256LL + threadIdx.x;
    if (i >= total) return;
    float acc = 0.f;
#pragma unroll 8
    for (int c = 0; c < chunks; ++c) acc += part[(size_t)c * total + i];  // independent loads, added in order
    dw[i] = accumulate ? dw[i] + acc : acc;
}

// ---- dbias: deterministic two-stage column sum -------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1(const T* dy, float* part, long long rows, int Cout)
{
    // block: 64 columns x 4 row lanes; grid.y = row chunks
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int rl = threadIdx.x >> 6;
    const long long per = (rows + gridDim.y - 1) / gridDim.y;
    const long long r0 = per * blockIdx.y, r1 = (r0 + per < rows) ? r0 + per : rows;
    float acc = 0.f;
    if (c < Cout)
        for (long long r = r0 + rl; r < r1; r += 4) acc += Elem<T>::load(dy, (size_t)r * Cout + c);
    __shared__ float sm[4][64];
    sm[rl][threadIdx.x & 63] = acc;
    __syncthreads();
    if (rl == 0 && c < Cout)
        part[(size_t)blockIdx.y * Cout + c] = (sm[0][threadIdx.x] + sm[1][threadIdx.x]) +
                                              (sm[2][threadIdx.x] + sm[3][threadIdx.x]);
}
// bf16, Cout % 8 == 0.  A workgroup owns 32 columns (4 lanes x 16-byte loads) of one of
// DBIAS_VCHUNKS row ranges, 64 row lanes each; the 64 partial sums per column are added in a
// fixed tree through LDS; colsum_stage2 then adds the chunks in order.
constexpr int DBIAS_VCHUNKS = 16;
__global__ __launch_bounds__(256) void colsum_bf16_stage1(const bf16_t* __restrict__ dy, float* __restrict__ part,
                                                          long long rows, int Cout)
{
    const int cg = threadIdx.x & 3, rl = threadIdx.x >> 2;
    const int c0 = blockIdx.x * 32 + cg * 8;
    const long long per = (rows + gridDim.y - 1) / gridDim.y;
    const long long r0 = per * blockIdx.y, r1 = (r0 + per < rows) ? r0 + per : rows;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    if (c0 < Cout)
        for (long long r = r0 + rl; r < r1; r += 64) {
            const uint4 v = *reinterpret_cast<const uint4*>(dy + r * Cout + c0);
            const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[2 * j] += __uint_as_float(u[j] << 16);
                acc[2 * j + 1] += __uint_as_float(u[j] & 0xffff0000u);
            }
        }
    __shared__ float sm[64][33];
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[rl][cg * 8 + j] = acc[j];
    __syncthreads();
    for (int half = 32; half > 0; half >>= 1) {
        for (int e = threadIdx.x; e < half * 32; e += 256) {
            const int r = e >> 5, c = e & 31;
            sm[r][c] += sm[r + half][c];
        }
        __syncthreads();
    }
    if (threadIdx.x < 32) {
        const int c = blockIdx.x * 32 + threadIdx.x;
        if (c < Cout) part[(size_t)blockIdx.y * Cout + c] = sm[0][threadIdx.x];
    }
}
__global__ void colsum_stage2(const float* part, float* dbias, int chunks, int Cout, int accumulate)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= Cout) return;
    float acc = 0.f;
    for (int i0 = 0; i0 < chunks; i0 += 16) {
        float v[16];  // independent loads, then added in order
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = (i0 + u < chunks) ? part[(size_t)(i0 + u) * Cout + c] : 0.f;
#pragma unroll
        for (int u = 0; u < 16; ++u) acc += v[u];
    }
    dbias[c] = accumulate ? dbias[c] + acc : acc;
}

}  // namespace

int conv_fwd_generic(const ConvDesc& d, const void* x, const void* w, const float* bias, void* y, int dt, int ydt,
                     hipStream_t st)
{
    if (dt == W2L_F32 && ydt == W2L_F32) return fwd_t<float, float>(d, x, w, bias, y, st);
    if (dt == W2L_BF16 && ydt == W2L_BF16) return fwd_t<bf16_t, bf16_t>(d, x, w, bias, y, st);
    if (dt == W2L_BF16 && ydt == W2L_F32) return fwd_t<bf16_t, float>(d, x, w, bias, y, st);
    return W2L_ERR_DTYPE;
}
int conv_dgrad_generic(const ConvDesc& d, const void* dy, const void* w, void* dx, int dt, int dydt, hipStream_t st)
{
    if (dt == W2L_F32 && dydt == W2L_F32) return dgrad_t<float, float>(d, dy, w, dx, st);
    if (dt == W2L_BF16 && dydt == W2L_BF16) return dgrad_t<bf16_t, bf16_t>(d, dy, w, dx, st);
    if (dt == W2L_BF16 && dydt == W2L_F32) return dgrad_t<bf16_t, float>(d, dy, w, dx, st);
    return W2L_ERR_DTYPE;
}
int conv_wgrad_generic(const ConvDesc& d, const void* x, const void* dy, float* dw, int dt, int dydt, int accumulate,
                       hipStream_t st)
{
    if (dt == W2L_F32 && dydt == W2L_F32) return wgrad_t<float, float>(d, x, dy, dw, accumulate, st);
    if (dt == W2L_BF16 && dydt == W2L_BF16) return wgrad_t<bf16_t, bf16_t>(d, x, dy, dw, accumulate, st);
    if (dt == W2L_BF16 && dydt == W2L_F32) return wgrad_t<bf16_t, float>(d, x, dy, dw, accumulate, st);
    return W2L_ERR_DTYPE;
}
size_t conv_wgrad_skinny_scratch(int Cin, int Cout, int k)
{
    return Cout <= 32 ? round_up((size_t)SKINNY_CHUNKS * Cout * k * Cin * 4, 256) : 0;
}
int conv_wgrad_skinny(const ConvDesc& d, const void* x, const void* dy, float* dw, int dt, int dydt, int accumulate,
                      float* scratch, hipStream_t st)
{
    const long long N = (long long)d.k * d.Cin;
    const dim3 g1((unsigned)((N + 63) / 64), SKINNY_CHUNKS);
    if (dt == W2L_F32 && dydt == W2L_F32)
        hipLaunchKernelGGL((wgrad_skinny_stage1<float, float>), g1, dim3(256), 0, st, (const float*)x, (const float*)dy, scratch, d);
    else if (dt == W2L_BF16 && dydt == W2L_BF16)
        hipLaunchKernelGGL((wgrad_skinny_stage1<bf16_t, bf16_t>), g1, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dy, scratch, d);
    else if (dt == W2L_BF16 && dydt == W2L_F32)
        hipLaunchKernelGGL((wgrad_skinny_stage1<bf16_t, float>), g1, dim3(256), 0, st, (const bf16_t*)x, (const float*)dy, scratch, d);
    else
        return W2L_ERR_DTYPE;
    int rc = launch_status();
    if (rc) return rc;
    const long long total = (long long)d.Cout * N;
    hipLaunchKernelGGL(wgrad_skinny_stage2, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, scratch, dw,
                       (int)SKINNY_CHUNKS, total, accumulate);
    return launch_status();
}
int dbias_reduce(const void* dy, float* dbias, long long rows, int Cout, int dydt, int accumulate,
                 float* scratch, hipStream_t st)
{
    if (dydt == W2L_BF16 && Cout % 8 == 0) {
        hipLaunchKernelGGL(colsum_bf16_stage1, dim3((Cout + 31) / 32, DBIAS_VCHUNKS), dim3(256), 0, st,
                           (const bf16_t*)dy, scratch, rows, Cout);
        int rc = launch_status();
        if (rc) return rc;
        hipLaunchKernelGGL(colsum_stage2, dim3((Cout + 255) / 256), dim3(256), 0, st, scratch, dbias,
                           (int)DBIAS_VCHUNKS, Cout, accumulate);
        return launch_status();
    }
    const dim3 g1((Cout + 63) / 64, DBIAS_CHUNKS);
    if (dydt == W2L_F32)
        hipLaunchKernelGGL(colsum_stage1<float>, g1, dim3(256), 0, st, (const float*)dy, scratch, rows, Cout);
    else if (dydt == W2L_BF16)
        hipLaunchKernelGGL(colsum_stage1<bf16_t>, g1, dim3(256), 0, st, (const bf16_t*)dy, scratch, rows, Cout);
    else
        return W2L_ERR_DTYPE;
    int rc = launch_status();
    if (rc) return rc;
    hipLaunchKernelGGL(colsum_stage2, dim3((Cout + 255) / 256), dim3(256), 0, st, scratch, dbias,
                       (int)DBIAS_CHUNKS, Cout, accumulate);
    return launch_status();
}

}  // namespace w2l
