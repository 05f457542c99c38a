// Log-mel filterbank features on the GPU (paper Sec. 2.2 lists log-mels among the feature types
// computed on the fly before every network evaluation, Sec. 4.1 uses them as the network input;
// the paper computes them on host threads and fixes no constant -- the recipe is this library's
// reading: frames wholly inside the signal, Hamming window, zero-padded DFT, power spectrum,
// triangular filters equally spaced on the mel scale m = 2595 log10(1 + f/700), natural log).
//
// One wavefront per frame, four frames in flight per workgroup, a workgroup covers 16 consecutive
// frames of one utterance (their samples overlap, so they come from L2 / the same cache lines).
// The DFT is a radix-2 Stockham (self-sorting, out-of-place) FFT between two LDS buffers owned by
// the wavefront: log2(nfft) stages of nfft/2 butterflies, no workgroup barrier inside.  Twiddle
// factors, the window and the mel points are computed once per workgroup (sincospi / cospi on
// exact binary fractions; the mel points in double) -- there is no table in memory.  A lane then
// owns mel bands (lane, lane + 64, ...) and adds its weighted bins in ascending order, so the
// result does not depend on scheduling.
#include "common.h"

namespace w2l {
namespace {

constexpr int FRAMES_PER_WG = 16;

struct LogmelDims {
    int B, Nmax, Tmax, F, sr, win, hop, nfft, log2n;
    float fmin, fmax, floor;
};

template <typename T> __device__ __forceinline__ void store_as(T* p, float v) { Elem<T>::store(p, 0, v); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }

template <typename TO>
__global__ __launch_bounds__(256) void logmel_k(const float* __restrict__ wav, const int* __restrict__ wav_len,
                                                TO* __restrict__ feat, int* __restrict__ feat_len, LogmelDims d)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int b = blockIdx.y, t0 = blockIdx.x * FRAMES_PER_WG;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = d.nfft, H = N / 2;
    float2* tw = reinterpret_cast<float2*>(smem);                 // [N/2]  exp(-2 pi i k / N)
    float* window = reinterpret_cast<float*>(tw + H);             // [win]
    float* pts = window + ((d.win + 1) & ~1);                     // [F+2]  mel points in Hz
    float2* bufs = reinterpret_cast<float2*>(pts + ((d.F + 2 + 1) & ~1));  // per wavefront: two buffers of N, 8-byte aligned
    float2* x = bufs + (size_t)wave * 2 * N;
    float2* y = x + N;
    float* power = reinterpret_cast<float*>(bufs + (size_t)4 * 2 * N) + (size_t)wave * (H + 1);  // [N/2+1]

    int n = wav_len[b];
    n = n < 0 ? 0 : (n > d.Nmax ? d.Nmax : n);
    int T = n < d.win ? 0 : 1 + (n - d.win) / d.hop;
    T = T > d.Tmax ? d.Tmax : T;
    if (blockIdx.x == 0 && tid == 0) feat_len[b] = T;
    TO* fb = feat + (size_t)b * d.Tmax * d.F;
    if (t0 >= T) {  // nothing but padding in this workgroup's frames
        for (int e = tid; e < FRAMES_PER_WG * d.F; e += 256) {
            const int t = t0 + e / d.F;
            if (t < d.Tmax) store_as(fb + (size_t)t0 * d.F + e, 0.f);
        }
        return;
    }
    for (int k = tid; k < H; k += 256) {
        float s, c;
        sincospif(2.f * (float)k / (float)N, &s, &c);  // the argument is an exact binary fraction
        tw[k] = make_float2(c, -s);
    }
    for (int i = tid; i < d.win; i += 256) window[i] = 0.54f - 0.46f * cospif(2.f * (float)i / (float)(d.win - 1));
    for (int i = tid; i < d.F + 2; i += 256) {
        const double mlo = 2595.0 * log10(1.0 + (double)d.fmin / 700.0), mhi = 2595.0 * log10(1.0 + (double)d.fmax / 700.0);
        const double m = mlo + (mhi - mlo) * (double)i / (double)(d.F + 1);
        pts[i] = (float)(700.0 * (pow(10.0, m / 2595.0) - 1.0));
    }
    __syncthreads();

    const float* wb = wav + (size_t)b * d.Nmax;
    const float bin_hz = (float)d.sr / (float)N;
    for (int t = t0 + wave; t < t0 + FRAMES_PER_WG && t < d.Tmax; t += 4) {
        TO* out = fb + (size_t)t * d.F;
        if (t >= T) {
            for (int f = lane; f < d.F; f += 64) store_as(out + f, 0.f);
            continue;
        }
        const float* seg = wb + (size_t)t * d.hop;
        for (int i = lane; i < N; i += 64) x[i] = make_float2(i < d.win ? seg[i] * window[i] : 0.f, 0.f);
        __builtin_amdgcn_wave_barrier();
        // Stockham radix-2, decimation in frequency: at a stage the sequence length is len = N / s;
        // butterfly (p, q), p < len/2, q < s, takes src[q + s p], src[q + s (p + len/2)] and writes
        // dst[q + s 2p] = a + b, dst[q + s (2p+1)] = (a - b) exp(-2 pi i p / len); exp(..) = tw[p s].
        float2* src = x;
        float2* dst = y;
        for (int ls = 0; ls < d.log2n; ++ls) {
            const int s = 1 << ls;
            for (int j = lane; j < H; j += 64) {
                const int p = j >> ls, q = j & (s - 1);
                const float2 a = src[q + s * p], c = src[q + s * p + H];
                const float2 w = tw[p << ls];
                dst[q + s * 2 * p] = make_float2(a.x + c.x, a.y + c.y);
                dst[q + s * (2 * p + 1)] = cmul(make_float2(a.x - c.x, a.y - c.y), w);
            }
            __builtin_amdgcn_wave_barrier();
            float2* tmp = src; src = dst; dst = tmp;
        }
        for (int k = lane; k <= H; k += 64) {
            const float2 v = src[k];
            power[k] = v.x * v.x + v.y * v.y;
        }
        __builtin_amdgcn_wave_barrier();
        for (int f = lane; f < d.F; f += 64) {
            const float lo = pts[f], ce = pts[f + 1], hi = pts[f + 2];
            const float ru = 1.f / (ce - lo), rd = 1.f / (hi - ce);
            int k0 = (int)(lo / bin_hz), k1 = (int)(hi / bin_hz) + 1;  // a superset of the bins with a positive weight
            k0 = k0 < 0 ? 0 : k0;
            k1 = k1 > H ? H : k1;
            float acc = 0.f;
            for (int k = k0; k <= k1; ++k) {
                const float fr = (float)k * bin_hz;
                const float wgt = fmaxf(0.f, fminf((fr - lo) * ru, (hi - fr) * rd));
                acc = fmaf(wgt, power[k], acc);
            }
            store_as(out + f, logf(fmaxf(acc, d.floor)));
        }
        __builtin_amdgcn_wave_barrier();
    }
}

size_t logmel_lds_bytes(int nfft, int win, int F)
{
    return (size_t)(nfft / 2) * 8 + (size_t)((win + 1) & ~1) * 4 + (size_t)((F + 2 + 1) & ~1) * 4 + (size_t)4 * 2 * nfft * 8 +
           (size_t)4 * (nfft / 2 + 1) * 4;
}

}  // namespace
}  // namespace w2l

using namespace w2l;

extern "C" int w2l_logmel_num_frames(int n_samples, int win, int hop)
{
    if (win <= 0 || hop <= 0 || n_samples < win) return 0;
    return 1 + (n_samples - win) / hop;
}

extern "C" int w2l_logmel_fwd(const float* wav, const int* wav_len, void* feat, int* feat_len, int B, int Nmax, int Tmax,
                              int n_mels, int sample_rate, int win, int hop, int nfft, float fmin, float fmax, float floor,
                              int dtype, void* stream)
{
    if (!wav || !wav_len || !feat || !feat_len) return W2L_ERR_NULL;
    if (B <= 0 || B > 65535 || Nmax <= 0 || Tmax <= 0 || n_mels <= 0 || n_mels > 256 || sample_rate <= 0 || win < 2 ||
        hop <= 0 || nfft < 128 || nfft > 1024 || (nfft & (nfft - 1)) || win > nfft || !(fmin >= 0.f) || !(fmax > fmin) ||
        fmax > 0.5f * (float)sample_rate || !(floor > 0.f))
        return W2L_ERR_SHAPE;
    if (!valid_dtype(dtype)) return W2L_ERR_DTYPE;
    int log2n = 0;
    while ((1 << log2n) < nfft) ++log2n;
    LogmelDims d{B, Nmax, Tmax, n_mels, sample_rate, win, hop, nfft, log2n, fmin, fmax, floor};
    const size_t lds = logmel_lds_bytes(nfft, win, n_mels);
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((Tmax + FRAMES_PER_WG - 1) / FRAMES_PER_WG, B), block(256);
    if (dtype == W2L_BF16) {
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)logmel_k<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
        }
        hipLaunchKernelGGL(logmel_k<bf16_t>, grid, block, lds, st, wav, wav_len, (bf16_t*)feat, feat_len, d);
    } else {
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)logmel_k<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
        }
        hipLaunchKernelGGL(logmel_k<float>, grid, block, lds, st, wav, wav_len, (float*)feat, feat_len, d);
    }
    return launch_status();
}
