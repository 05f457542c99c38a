// Log-mel filterbank features on the GPU (paper Sec. 2.2 lists log-mels among the feature types
// computed on the fly before every network evaluation, Sec. 4.1 uses them as the network input;
// the paper computes them on host threads and fixes no constant -- the recipe is this library's
// reading: frames wholly inside the signal, Hamming window, zero-padded DFT, power spectrum,
// triangular filters equally spaced on the mel scale m = 2595 log10(1 + f/700), natural log).
//
// One wavefront per frame, four frames in flight per workgroup, a workgroup covers a run of consecutive
// frames of one utterance (their samples overlap, so they come from L2 / the same cache lines).
// The DFT of the real, zero-padded frame is taken as a complex FFT of half the size on
// z[n] = x[2n] + i x[2n+1], followed by the usual split into the spectrum of x.  The FFT is a
// radix-4 Stockham (self-sorting, out-of-place) transform between two LDS buffers owned by the
// wavefront, with one radix-2 pass when the size is not a power of four: for nfft = 512 that is
// four passes of 64 butterflies, one per lane, and no workgroup barrier.  Twiddle factors, the
// window, the mel points and the band weights are computed once per workgroup (sincospi / cospi
// on exact binary fractions; the mel points in double) -- there is no table in memory.  A lane
// then owns mel bands (lane, lane + 64, ...) and adds its weighted bins in ascending order, so the
// result does not depend on scheduling.
#include "common.h"

namespace w2l {
namespace {


struct LogmelDims {
    int B, Nmax, Tmax, F, sr, win, hop, nfft;
    int fpw;  // frames per workgroup (a multiple of 4)
    float fmin, fmax, floor;
};

template <typename T> __device__ __forceinline__ void store_as(T* p, float v) { Elem<T>::store(p, 0, v); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }

// LDS layout (floats unless noted), shared by the kernel and the host-side size
struct LogmelLds {
    int tw, window, pts, k0, off, wgt, bufs, power, total;  // offsets in bytes
};
__host__ __device__ inline LogmelLds logmel_lds(int nfft, int win, int F)
{
    auto up8 = [](int v) { return (v + 7) & ~7; };
    LogmelLds l;
    int o = 0;
    l.tw = o;     o += up8((3 * nfft / 4 + 1) * 8);          // float2 exp(-2 pi i k / nfft), k <= 3 nfft / 4
    l.window = o; o += up8(win * 4);
    l.pts = o;    o += up8((F + 2) * 4);                     // mel points in Hz
    l.k0 = o;     o += up8(F * 4);                           // int: first bin of a band
    l.off = o;    o += up8((F + 1) * 4);                     // int: start of a band's weights in wgt
    l.wgt = o;    o += up8((nfft + 2 + 4 * F) * 4);          // band weights, band after band
    l.bufs = o;   o += 4 * 2 * (nfft / 2) * 8;               // per wavefront: two float2 buffers of nfft/2
    l.power = o;  o += up8(4 * (nfft / 2 + 1) * 4);          // per wavefront: nfft/2 + 1
    l.total = o;
    return l;
}

template <typename TO>
__global__ __launch_bounds__(256) void logmel_k(const float* __restrict__ wav, const int* __restrict__ wav_len,
                                                TO* __restrict__ feat, int* __restrict__ feat_len, LogmelDims d)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int b = blockIdx.y, t0 = blockIdx.x * d.fpw;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = d.nfft, M = N / 2;
    const LogmelLds L = logmel_lds(N, d.win, d.F);
    float2* tw = reinterpret_cast<float2*>(smem + L.tw);
    float* window = reinterpret_cast<float*>(smem + L.window);
    float* pts = reinterpret_cast<float*>(smem + L.pts);
    int* bk0 = reinterpret_cast<int*>(smem + L.k0);
    int* boff = reinterpret_cast<int*>(smem + L.off);
    float* bw = reinterpret_cast<float*>(smem + L.wgt);
    float2* x = reinterpret_cast<float2*>(smem + L.bufs) + (size_t)wave * 2 * M;
    float2* y = x + M;
    float* power = reinterpret_cast<float*>(smem + L.power) + (size_t)wave * (M + 1);

    int n = wav_len[b];
    n = n < 0 ? 0 : (n > d.Nmax ? d.Nmax : n);
    int T = n < d.win ? 0 : 1 + (n - d.win) / d.hop;
    T = T > d.Tmax ? d.Tmax : T;
    if (blockIdx.x == 0 && tid == 0) feat_len[b] = T;
    TO* fb = feat + (size_t)b * d.Tmax * d.F;
    if (t0 >= T) {  // nothing but padding in this workgroup's frames
        for (int e = tid; e < d.fpw * d.F; e += 256) {
            const int t = t0 + e / d.F;
            if (t < d.Tmax) store_as(fb + (size_t)t0 * d.F + e, 0.f);
        }
        return;
    }
    // ---- per workgroup: twiddles, window, mel points, band weights
    for (int k = tid; k <= 3 * N / 4; k += 256) {
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
    const float bin_hz = (float)d.sr / (float)N;
    for (int f = tid; f < d.F; f += 256) {  // bins of a band: a superset of those with a positive weight
        int k0 = (int)(pts[f] / bin_hz), k1 = (int)(pts[f + 2] / bin_hz) + 1;
        k0 = k0 < 0 ? 0 : k0;
        k1 = k1 > M ? M : k1;
        bk0[f] = k0;
        boff[f + 1] = k1 - k0 + 1;  // the count, for now
    }
    __syncthreads();
    int my_off[1];
    my_off[0] = 0;
    if (tid <= d.F)                  // start of band tid's weights = sum of the counts before it (F <= 256: one band per thread)
        for (int g = 0; g < tid; ++g) my_off[0] += boff[g + 1];
    __syncthreads();
    if (tid <= d.F) boff[tid] = my_off[0];
    __syncthreads();
    for (int f = tid; f < d.F; f += 256) {
        const float lo = pts[f], ce = pts[f + 1], hi = pts[f + 2];
        const float ru = 1.f / (ce - lo), rd = 1.f / (hi - ce);
        const int k0 = bk0[f], cnt = boff[f + 1] - boff[f];
        for (int i = 0; i < cnt; ++i) {
            const float fr = (float)(k0 + i) * bin_hz;
            bw[boff[f] + i] = fmaxf(0.f, fminf((fr - lo) * ru, (hi - fr) * rd));
        }
    }
    __syncthreads();

    const float* wb = wav + (size_t)b * d.Nmax;
    for (int t = t0 + wave; t < t0 + d.fpw && t < d.Tmax; t += 4) {
        TO* out = fb + (size_t)t * d.F;
        if (t >= T) {
            for (int f = lane; f < d.F; f += 64) store_as(out + f, 0.f);
            continue;
        }
        const float* seg = wb + (size_t)t * d.hop;
        for (int i = lane; i < M; i += 64) {
            const int e = 2 * i;
            x[i] = make_float2(e < d.win ? seg[e] * window[e] : 0.f, e + 1 < d.win ? seg[e + 1] * window[e + 1] : 0.f);
        }
        __builtin_amdgcn_wave_barrier();
        // Stockham radix-4, decimation in frequency, on M points: at a pass the sequence length is
        // len = M / s; butterfly (p, q), p < len/4, q < s, takes src[q + s (p + r len/4)], r = 0..3,
        // and writes dst[q + s (4p + r)] with the factors exp(-2 pi i r p / len) = tw[2 r p s].
        float2* src = x;
        float2* dst = y;
        int len = M, s = 1, ls = 0;
        for (; len >= 4; len >>= 2, s <<= 2, ls += 2) {
            const int m = len >> 2;
            for (int j = lane; j < (M >> 2); j += 64) {
                const int p = j >> ls, q = j & (s - 1);
                const float2* in = src + q + s * p;
                const float2 a = in[0], bb = in[s * m], c = in[2 * s * m], dd = in[3 * s * m];
                const int ti = 2 * p * s;
                const float2 apc = cadd(a, c), amc = csub(a, c), bpd = cadd(bb, dd), bmd = csub(bb, dd);
                const float2 jbmd = make_float2(-bmd.y, bmd.x);  // i (b - d)
                float2* o = dst + q + s * 4 * p;
                o[0] = cadd(apc, bpd);
                o[s] = cmul(tw[ti], csub(amc, jbmd));
                o[2 * s] = cmul(tw[2 * ti], csub(apc, bpd));
                o[3 * s] = cmul(tw[3 * ti], cadd(amc, jbmd));
            }
            __builtin_amdgcn_wave_barrier();
            float2* tmp = src; src = dst; dst = tmp;
        }
        if (len == 2) {  // one radix-2 pass: s = M / 2
            for (int q = lane; q < s; q += 64) {
                const float2 a = src[q], c = src[q + s];
                dst[q] = cadd(a, c);
                dst[q + s] = csub(a, c);
            }
            __builtin_amdgcn_wave_barrier();
            float2* tmp = src; src = dst; dst = tmp;
        }
        // spectrum of the real frame from the spectrum Z of the packed one:
        //   X[k] = (Z[k] + conj Z[M-k]) / 2 - (i / 2) exp(-2 pi i k / N) (Z[k] - conj Z[M-k]),  k = 0..M
        for (int k = lane; k <= M; k += 64) {
            const float2 zk = src[k & (M - 1)], zm = src[(M - k) & (M - 1)];
            const float2 e = make_float2(0.5f * (zk.x + zm.x), 0.5f * (zk.y - zm.y));
            const float2 o = make_float2(0.5f * (zk.x - zm.x), 0.5f * (zk.y + zm.y));
            const float2 r = cmul(tw[k], make_float2(o.y, -o.x));  // (-i) o, turned by the twiddle
            const float re = e.x + r.x, im = e.y + r.y;
            power[k] = re * re + im * im;
        }
        __builtin_amdgcn_wave_barrier();
        for (int f = lane; f < d.F; f += 64) {
            const int k0 = bk0[f], o0 = boff[f], cnt = boff[f + 1] - o0;
            float acc = 0.f;
            for (int i = 0; i < cnt; ++i) acc = fmaf(bw[o0 + i], power[k0 + i], acc);
            store_as(out + f, logf(fmaxf(acc, d.floor)));
        }
        __builtin_amdgcn_wave_barrier();
    }
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
    if (B <= 0 || B > 65535 || Nmax <= 0 || Tmax <= 0 || n_mels <= 0 || n_mels > 255 || sample_rate <= 0 || win < 2 ||
        hop <= 0 || nfft < 128 || nfft > 1024 || (nfft & (nfft - 1)) || win > nfft || !(fmin >= 0.f) || !(fmax > fmin) ||
        fmax > 0.5f * (float)sample_rate || !(floor > 0.f))
        return W2L_ERR_SHAPE;
    if (!valid_dtype(dtype)) return W2L_ERR_DTYPE;
    // the per-workgroup set-up is shared by fpw frames; about a thousand workgroups keep four of them
    // (sixteen wavefronts) on every CU, which is what hides the LDS round trips of the FFT passes
    long long fpw = ((long long)B * Tmax + 999) / 1000;
    fpw = fpw < 4 ? 4 : (fpw > 256 ? 256 : fpw);
    fpw = (fpw + 3) / 4 * 4;
    LogmelDims d{B, Nmax, Tmax, n_mels, sample_rate, win, hop, nfft, (int)fpw, fmin, fmax, floor};
    const size_t lds = (size_t)logmel_lds(nfft, win, n_mels).total;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((Tmax + (int)fpw - 1) / (int)fpw, B), block(256);
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
