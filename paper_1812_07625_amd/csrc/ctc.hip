// CTC criterion on the GPU (paper Sec. 2.3; the paper runs its CTC on host cores,
// Sec. 4.1 -- this keeps the whole criterion on the device, so no device<->host round
// trip sits between the network's forward and backward passes).
//
// Three kernels, all deterministic (no floating-point atomics):
//   1. (logits only) per-frame log-softmax into the workspace;
//   2. ctc_lattice: one workgroup per (utterance, direction).  alpha runs forward in
//      time, beta is the same recursion on the reversed label sequence and reversed
//      time, so the two run concurrently and the serial chain is T_b steps, not 2 T_b.
//      States live in LDS; scores are kept in the base-2 log domain so that the
//      log-sum-exp maps onto the hardware exp2/log2 instructions; the running values
//      are held in fp64 (their magnitude grows with t, the increments do not) while
//      every transcendental is evaluated in fp32 on differences.  Score rows are
//      prefetched into LDS a chunk of frames ahead, off the dependency chain;
//   3. ctc_grad: one wavefront per frame combines alpha_t and beta_t into the state
//      posteriors, normalises them per frame, and sums them per class in a fixed
//      order given by a (class, position) sort of the target.
#include "common.h"

namespace w2l {
namespace {

constexpr double LOG2E = 1.4426950408889634074;
constexpr double LN2 = 0.69314718055994530942;
constexpr int PF = 8;           // prefetch registers per thread
constexpr int MAX_CHUNK = 16;   // frames of scores staged per chunk
constexpr int GRAD_ROWS = 16;   // frames per ctc_grad workgroup (4 per wavefront)

struct CtcDims {
    int B, Tp, C, Lmax, blank;
    int Sp;  // lattice row pitch = 2*Lmax+1
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// log2( 2^a + 2^b + 2^c ), any of them may be -inf
__device__ __forceinline__ double lse3_log2(double a, double b, double c)
{
    const double m = fmax(a, fmax(b, c));
    if (m == -INFINITY) return -INFINITY;
    const float sum = fast_exp2((float)(a - m)) + fast_exp2((float)(b - m)) + fast_exp2((float)(c - m));
    return m + (double)fast_log2(sum);
}

__global__ void ctc_lattice(const float* __restrict__ lp, const int* __restrict__ targets,
                            const int* __restrict__ in_len, const int* __restrict__ tgt_len,
                            float* __restrict__ loss, double* __restrict__ logp2_out,
                            double* __restrict__ alpha, double* __restrict__ beta, CtcDims d, int chunk)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int dir = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, NT = blockDim.x;
    const int T = in_len[b], L = tgt_len[b];
    __shared__ int bad_len, bad;
    if (tid == 0) {
        bad_len = (T < 0 || T > d.Tp || L < 0 || L > d.Lmax) ? 1 : 0;
        bad = 0;
    }
    __syncthreads();
    if (bad_len) {
        if (dir == 0 && tid == 0) { loss[b] = NAN; logp2_out[b] = NAN; }
        return;
    }
    const int S = 2 * L + 1;
    // LDS carve-up: two state vectors (2 leading -inf pads each), class of each state
    // (bit 30 = "may skip from s-2"), two score chunks
    double* st0 = reinterpret_cast<double*>(smem_raw);
    double* st1 = st0 + (2 * d.Lmax + 3);
    int* cls = reinterpret_cast<int*>(st1 + (2 * d.Lmax + 3));
    float* sc0 = reinterpret_cast<float*>(cls + (2 * d.Lmax + 1));
    float* sc1 = sc0 + (size_t)chunk * d.C;

    const int* lab = targets + (size_t)b * d.Lmax;
    for (int i = tid; i < L; i += NT) {
        const int l = lab[i];
        if (l < 0 || l >= d.C || l == d.blank) bad = 1;
    }
    __syncthreads();
    if (bad) {
        if (dir == 0 && tid == 0) { loss[b] = NAN; logp2_out[b] = NAN; }
        return;
    }
    // state index q runs in this direction's own order; actual state s = dir ? S-1-q : q
    for (int q = tid; q < S; q += NT) {
        const int s = dir ? S - 1 - q : q;
        int c = d.blank, skip = 0;
        if (s & 1) {
            c = lab[(s - 1) >> 1];
            if (q >= 2) {
                const int s2 = dir ? s + 2 : s - 2;
                skip = (lab[(s2 - 1) >> 1] != c);
            }
        }
        cls[q] = c | (skip << 30);
    }
    for (int q = tid; q < S + 2; q += NT) { st0[q] = -INFINITY; st1[q] = -INFINITY; }

    if (T == 0) {
        if (dir == 0 && tid == 0) {
            loss[b] = (L == 0) ? 0.f : INFINITY;
            logp2_out[b] = (L == 0) ? 0.0 : -INFINITY;
        }
        return;
    }

    const float* lpb = lp + (size_t)b * d.Tp * d.C;
    double* lat = (dir ? beta : alpha) + (size_t)b * d.Tp * d.Sp;
    const int rowsz = d.C;
    const int chunk_elems = chunk * rowsz;
    // frame visited at step i
    auto frame = [&](int i) { return dir ? T - 1 - i : i; };

    // chunk 0 synchronously
    for (int e = tid; e < chunk_elems; e += NT) {
        const int r = e / rowsz, c = e - r * rowsz;
        sc0[e] = (r < T) ? lpb[(size_t)frame(r) * rowsz + c] : 0.f;
    }
    __syncthreads();

    double* prev = st0;
    double* cur = st1;
    float pf[PF];
    for (int step = 0; step < T; ++step) {
        const int cidx = step / chunk, within = step - cidx * chunk;
        float* sc = (cidx & 1) ? sc1 : sc0;
        if (within == 0) {  // start fetching the next chunk; consumed `chunk` steps from now
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const int e = tid + i * NT;
                pf[i] = 0.f;
                if (e < chunk_elems) {
                    const int r = e / rowsz, c = e - r * rowsz;
                    const int fs = (cidx + 1) * chunk + r;
                    if (fs < T) pf[i] = lpb[(size_t)frame(fs) * rowsz + c];
                }
            }
        }
        const int t = frame(step);
        const float* row = sc + (size_t)within * rowsz;
        for (int q = tid; q < S; q += NT) {
            const int cw = cls[q];
            const int c = cw & 0x3fffffff;
            const double sc2 = (double)row[c] * LOG2E;
            double v;
            if (step == 0) {
                v = (q < 2) ? sc2 : -INFINITY;
            } else {
                const double a0 = prev[q + 2], a1 = prev[q + 1];
                const double a2 = (cw >> 30) ? prev[q] : -INFINITY;
                v = lse3_log2(a0, a1, a2) + sc2;
            }
            cur[q + 2] = v;
            lat[(size_t)t * d.Sp + (dir ? S - 1 - q : q)] = v;
        }
        if (within == chunk - 1) {
            float* nxt = (cidx & 1) ? sc0 : sc1;
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const int e = tid + i * NT;
                if (e < chunk_elems) nxt[e] = pf[i];
            }
        }
        // LDS-only hand-over: wait for this wavefront's LDS traffic, then barrier.  A full
        // __syncthreads() would also wait for the lattice stores above, putting HBM write
        // latency on the T-step dependency chain.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        double* tmp = prev; prev = cur; cur = tmp;
    }
    if (dir == 0 && tid == 0) {
        const double lp2 = lse3_log2(prev[S - 1 + 2], (S > 1) ? prev[S - 2 + 2] : -INFINITY, -INFINITY);
        logp2_out[b] = lp2;
        loss[b] = (lp2 == -INFINITY) ? INFINITY : (float)(-lp2 * LN2);
    }
}

__device__ __forceinline__ float wsum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(256) void ctc_grad(const float* __restrict__ lp, const int* __restrict__ targets,
                                                const int* __restrict__ in_len,
                                                const int* __restrict__ tgt_len,
                                                const float* __restrict__ loss,
                                                const double* __restrict__ logp2_in,
                                                const double* __restrict__ alpha,
                                                const double* __restrict__ beta, float* __restrict__ grad,
                                                CtcDims d, int is_logits, float grad_scale)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int b = blockIdx.y, t0 = blockIdx.x * GRAD_ROWS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* gb = grad + (size_t)b * d.Tp * d.C;
    const float ls = loss[b];
    const int T = in_len[b];
    const bool live = isfinite(ls) && T > 0;  // NaN (invalid) and +inf (no alignment) give zero rows
    if (!live) {
        for (int e = tid; e < GRAD_ROWS * d.C; e += 256) {
            const int t = t0 + e / d.C;
            if (t < d.Tp) gb[(size_t)t0 * d.C + e] = 0.f;
        }
        return;
    }
    const int L = tgt_len[b], S = 2 * L + 1;
    int* lab = reinterpret_cast<int*>(smem_raw);       // [Lmax]
    int* order = lab + d.Lmax;                         // [Lmax] label positions sorted by (class, position)
    int* cstart = order + d.Lmax;                      // [C+1]
    float* ebuf = reinterpret_cast<float*>(cstart + d.C + 1) + (size_t)wave * d.Sp;  // [4][Sp]

    for (int i = tid; i < L; i += 256) lab[i] = targets[(size_t)b * d.Lmax + i];
    for (int c = tid; c <= d.C; c += 256) cstart[c] = 0;
    __syncthreads();
    for (int i = tid; i < L; i += 256) atomicAdd(&cstart[lab[i] + 1], 1);  // integer: order-independent
    __syncthreads();
    if (tid == 0)
        for (int c = 0; c < d.C; ++c) cstart[c + 1] += cstart[c];
    __syncthreads();
    for (int i = tid; i < L; i += 256) {
        const int c = lab[i];
        int r = cstart[c];
        for (int j = 0; j < i; ++j) r += (lab[j] == c);
        order[r] = i;
    }
    __syncthreads();

    const double logp2 = logp2_in[b];
    const float* lpb = lp + (size_t)b * d.Tp * d.C;
    for (int rr = wave; rr < GRAD_ROWS; rr += 4) {
        const int t = t0 + rr;
        if (t >= d.Tp) break;
        float* grow = gb + (size_t)t * d.C;
        if (t >= T) {
            for (int c = lane; c < d.C; c += 64) grow[c] = 0.f;
            continue;
        }
        const double* ar = alpha + ((size_t)b * d.Tp + t) * d.Sp;
        const double* br = beta + ((size_t)b * d.Tp + t) * d.Sp;
        const float* lrow = lpb + (size_t)t * d.C;
        float z = 0.f, zb = 0.f;
        for (int s = lane; s < S; s += 64) {
            const int c = (s & 1) ? lab[(s - 1) >> 1] : d.blank;
            const double a = ar[s], bt = br[s];
            float e = 0.f;
            if (a != -INFINITY && bt != -INFINITY)
                e = fast_exp2((float)(a + bt - (double)lrow[c] * LOG2E - logp2));
            ebuf[s] = e;
            z += e;
            if (!(s & 1)) zb += e;
        }
        z = wsum(z);
        zb = wsum(zb);
        const float inv = z > 0.f ? 1.f / z : 0.f;
        __builtin_amdgcn_wave_barrier();
        for (int c = lane; c < d.C; c += 64) {
            float g;
            if (c == d.blank) {
                g = zb;
            } else {
                g = 0.f;
                for (int q = cstart[c]; q < cstart[c + 1]; ++q) g += ebuf[2 * order[q] + 1];
            }
            g *= inv;
            grow[c] = is_logits ? grad_scale * (__expf(lrow[c]) - g) : -grad_scale * g;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

size_t lattice_lds_bytes(int Lmax, int C, int chunk)
{
    return (size_t)2 * 8 * (2 * Lmax + 3) + (size_t)4 * (2 * Lmax + 1) + (size_t)2 * 4 * chunk * C;
}
size_t grad_lds_bytes(int Lmax, int C)
{
    return (size_t)4 * (2 * Lmax + C + 1) + (size_t)4 * 4 * (2 * Lmax + 1);
}
void lattice_launch_shape(int Lmax, int C, int* nt, int* chunk)
{
    int need = 2 * Lmax + 1;
    if ((C + PF - 1) / PF > need) need = (C + PF - 1) / PF;
    int t = (need + 63) / 64 * 64;
    if (t < 64) t = 64;
    if (t > 1024) t = 1024;
    int ch = PF * t / C;
    if (ch > MAX_CHUNK) ch = MAX_CHUNK;
    if (ch < 1) ch = 1;
    *nt = t;
    *chunk = ch;
}

struct WsLayout { size_t lp, logp, alpha, beta, total; };
WsLayout ws_layout(int B, int Tp, int C, int Lmax)
{
    WsLayout w;
    size_t off = 0;
    w.lp = off; off += round_up((size_t)B * Tp * C * 4, 256);
    w.logp = off; off += round_up((size_t)B * 8, 256);
    const size_t lat = round_up((size_t)B * Tp * (2 * (size_t)Lmax + 1) * 8, 256);
    w.alpha = off; off += lat;
    w.beta = off; off += lat;
    w.total = off;
    return w;
}

}  // namespace
}  // namespace w2l

using namespace w2l;

extern "C" size_t w2l_ctc_workspace_bytes(int B, int Tp, int C, int Lmax)
{
    if (B <= 0 || Tp <= 0 || C <= 0 || Lmax <= 0) return 0;
    return ws_layout(B, Tp, C, Lmax).total;
}

extern "C" int w2l_ctc_check_targets_host(const int* targets, const int* in_len, const int* tgt_len, int B,
                                          int Tp, int C, int Lmax, int blank)
{
    if (!targets || !in_len || !tgt_len) return W2L_ERR_NULL;
    if (B <= 0 || Tp <= 0 || C <= 0 || Lmax <= 0 || blank < 0 || blank >= C) return W2L_ERR_SHAPE;
    for (int b = 0; b < B; ++b) {
        if (in_len[b] < 0 || in_len[b] > Tp || tgt_len[b] < 0 || tgt_len[b] > Lmax) return W2L_ERR_TARGET;
        for (int i = 0; i < tgt_len[b]; ++i) {
            const int l = targets[(size_t)b * Lmax + i];
            if (l < 0 || l >= C || l == blank) return W2L_ERR_TARGET;
        }
    }
    return W2L_OK;
}

extern "C" int w2l_ctc_fwd_bwd(const float* input, int is_logits, const int* targets, const int* in_len,
                               const int* tgt_len, float* loss, float* grad, int B, int Tp, int C, int Lmax,
                               int blank, float grad_scale, void* workspace, size_t ws_bytes, void* stream)
{
    if (!input || !targets || !in_len || !tgt_len || !loss || !grad) return W2L_ERR_NULL;
    if (B <= 0 || Tp <= 0 || C <= 0 || C > 4096 || Lmax <= 0 || Lmax > 3000 || blank < 0 || blank >= C ||
        B > 65535)
        return W2L_ERR_SHAPE;
    if (!aligned16(input) || !aligned16(targets) || !aligned16(grad)) return W2L_ERR_ALIGN;
    const WsLayout w = ws_layout(B, Tp, C, Lmax);
    if (!workspace || ws_bytes < w.total || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return W2L_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const float* lp = input;
    if (is_logits) {
        float* lpw = reinterpret_cast<float*>(ws + w.lp);
        int rc = w2l_logsoftmax_fwd(input, lpw, (long long)B * Tp, C, W2L_F32, stream);
        if (rc) return rc;
        lp = lpw;
    }
    double* logp = reinterpret_cast<double*>(ws + w.logp);
    double* alpha = reinterpret_cast<double*>(ws + w.alpha);
    double* beta = reinterpret_cast<double*>(ws + w.beta);
    CtcDims d{B, Tp, C, Lmax, blank, 2 * Lmax + 1};

    int nt, chunk;
    lattice_launch_shape(Lmax, C, &nt, &chunk);
    const size_t lds1 = lattice_lds_bytes(Lmax, C, chunk), lds2 = grad_lds_bytes(Lmax, C);
    if (lds1 > 160 * 1024 || lds2 > 160 * 1024) return W2L_ERR_SHAPE;
    hipError_t e;
    if (lds1 > 48 * 1024) {
        e = hipFuncSetAttribute((const void*)ctc_lattice, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    }
    if (lds2 > 48 * 1024) {
        e = hipFuncSetAttribute((const void*)ctc_grad, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    }
    hipLaunchKernelGGL(ctc_lattice, dim3(2, B), dim3(nt), lds1, st, lp, targets, in_len, tgt_len, loss, logp,
                       alpha, beta, d, chunk);
    int rc = launch_status();
    if (rc) return rc;
    hipLaunchKernelGGL(ctc_grad, dim3((Tp + GRAD_ROWS - 1) / GRAD_ROWS, B), dim3(256), lds2, st, lp, targets,
                       in_len, tgt_len, loss, logp, alpha, beta, grad, d, is_logits, grad_scale);
    return launch_status();
}
