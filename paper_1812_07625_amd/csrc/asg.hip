// ASG criterion on the GPU (AutoSegCriterion: paper Sec. 2.3 lists it beside CTC as the
// original wav2letter criterion with learned parameters, and cites its source; the paper
// prints no formula).  Definition used here: unnormalised emissions f[t][c], a learned
// transition matrix g[i][j] (class j at frame t-1 followed by class i at frame t), no blank;
//   loss = FCC - FAL,
//   FCC = log-sum of exp(score) over all C^T frame labellings          (fully connected lattice)
//   FAL = the same over the monotone alignments of the target            (forced alignment lattice)
//   score(pi) = sum_t f[t][pi_t] + sum_{t>=1} g[pi_t][pi_{t-1}]
// and the gradients are differences of node / edge occupancies of the two lattices.
//
// Kernels, all deterministic (no floating-point atomics):
//   1. asg_lattice: one workgroup per (utterance, lattice, direction).  Forward and backward run
//      concurrently (backward = the same recursion on reversed time with the transposed
//      transitions, and for FAL the reversed target), so the serial chain is T_b steps.  Rows are
//      stored as base-2 logs, fp32, relative to a double-precision offset per frame; "log zero" is
//      a large negative finite number.
//      FAL: log domain (hardware exp2/log2), one lane per target position, the value of the
//      position to the left by a DPP wavefront shift; wavefronts overlap by BLK mirrored positions
//      so that nothing crosses a wavefront boundary inside a block of BLK frames (16 or 12), at
//      whose end the largest state moves into the offset; the block's emission rows come from LDS.
//      FCC: while the transition scores span at most LINEAR_RANGE bits the states are plain numbers
//      and a step is a matrix-vector product with exact power-of-two rescaling (up to 32 classes:
//      lane rotations and swaps only, on one wavefront, with a second wavefront doing all memory
//      work and bookkeeping; up to 64: one wavefront, through a small LDS array); beyond that
//      range a log-domain recursion with a full log-sum-exp per state takes over.
//   2. asg_grad_em: per frame, node occupancies of both lattices, each normalised per frame;
//      FAL positions are summed per class in a fixed order ((class, position) sort).
//   3. asg_trans_partial: per (utterance, 32 frames), edge occupancies summed over the frames:
//      FCC per class pair, FAL per target position (stay / advance).
//   4. asg_trans_utt: per utterance, FCC edge sums minus FAL edge sums as a C x C table (the FAL
//      sums are scattered with 64-bit fixed-point integer atomics, which are order-independent).
//   5. asg_trans_reduce: sum over utterances in a fixed order.
#include <type_traits>
#include "common.h"

namespace w2l {
namespace {

constexpr double LOG2E = 1.4426950408889634074;
constexpr double LN2 = 0.69314718055994530942;
constexpr float NEG = -1.0e30f;       // log zero: absorbs every finite addend, never turns into NaN
constexpr float NEG_TEST = -1.0e29f;  // anything below is "log zero"
constexpr int AHEAD = 16;             // frames of scores held in registers ahead of the recursion; period of the
                                      // hand-over between wavefronts and of the renormalisation
constexpr int CP = 64;                // pitch of an FCC lattice row; the class limit
constexpr int GRAD_UNROLL = 4;        // target positions per lane whose loads asg_grad_em issues together
constexpr int CHUNK = 32;             // frames per asg_trans_partial workgroup

struct AsgDims {
    int B, Tp, C, Lmax;
    int Sp;   // FAL lattice row pitch = Lmax + 4 (the last four are spare slots); Tp + 1 rows per utterance
    int nch;  // frame chunks per utterance
};

// workspace pointers
struct AsgWs {
    float *fal[2], *fcc[2];          // lattices per direction: [B][Tp+1][Sp] and [B][Tp+1][CP]
    double *faloff[2], *fccoff[2];   // [B][Tp+1] offsets of the rows
    double* terms;                   // [B][2]: FCC, FAL in base-2 units
    int* status;                     // [B]: 0 live, 1 no alignment, 2 invalid
    float *izf, *iza;                // [B][Tp] inverse per-frame normalisers of the node occupancies
    float *partF, *partA, *tabD;     // [B][nch][C*C], [B][nch][2][Lmax], [B][C*C] (per-utterance d loss / d g)
    int *order, *cstart;             // [B][Lmax] target positions sorted by (class, position); [B][C+1] start of every class in it
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float lse2_log2(float a, float b)
{
    const float m = fmaxf(a, b);
    return m + fast_log2(1.f + fast_exp2(fminf(a, b) - m));
}
__device__ __forceinline__ float wave_max_f(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
// value of the lane to the left (lane - 1); lane 0 gets `edge`
__device__ __forceinline__ float from_left_lane(float v, float edge)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(edge), __float_as_int(v), 0x138 /* wave_shr:1 */,
                                                      0xf, 0xf, false));
}

// Wavefront reductions on the DPP path (no LDS traffic, no wait counters): four row shifts
// leave each row's result in its lane 15, two row broadcasts carry it to lane 63, one lane
// read hands it to every lane.  Lanes a step does not reach keep `old` (the identity).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float old, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_max_bcast(float v)
{
    v = fmaxf(v, dpp_f<0x111, 0xf>(v, v));  // row_shr:1
    v = fmaxf(v, dpp_f<0x112, 0xf>(v, v));  // row_shr:2
    v = fmaxf(v, dpp_f<0x114, 0xf>(v, v));  // row_shr:4
    v = fmaxf(v, dpp_f<0x118, 0xf>(v, v));  // row_shr:8
    v = fmaxf(v, dpp_f<0x142, 0xa>(v, v));  // row_bcast:15 into rows 1 and 3
    v = fmaxf(v, dpp_f<0x143, 0xc>(v, v));  // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_min_bcast(float v) { return -wave_max_bcast(-v); }
__device__ __forceinline__ float wave_sum_bcast(float v)
{
    v += dpp_f<0x111, 0xf>(0.f, v);
    v += dpp_f<0x112, 0xf>(0.f, v);
    v += dpp_f<0x114, 0xf>(0.f, v);
    v += dpp_f<0x118, 0xf>(0.f, v);
    v += dpp_f<0x142, 0xa>(0.f, v);
    v += dpp_f<0x143, 0xc>(0.f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// ---- forced alignment lattice, one direction.  Position i (in this direction's order) is held
// by lane group gi = i / PPT; a_t[i] = f[t][y_i] + lse( a_{t-1}[i] + g_stay[i], a_{t-1}[i-1] + g_adv[i] ).
// Frame 0 comes out of the recursion itself: "before frame 0" all mass sits on a virtual
// position -1 that can only advance (into position 0, at no cost).  Mirror lanes, score ring,
// spare slots and renormalisation as described at the top of the file.
template <int PPT, int BLK, int NQ>
__device__ __forceinline__ void fal_lattice(const float* __restrict__ em, const float* __restrict__ trans,
                                            const int* __restrict__ lab, int T, int L, int dir,
                                            float* __restrict__ lat, double* __restrict__ offs, double* term_out,
                                            const AsgDims& d, float (*xbuf)[16][AHEAD][4], float (*wmax)[16], float* tbl)
{
    constexpr int HALO = BLK, OWN = 64 - BLK;  // mirror lanes / owned lanes of a wavefront
    constexpr int PITCH = BLK + 1;             // table entries per class (one of padding against bank conflicts)
    const int tid = threadIdx.x, NT = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int gi = wave * OWN + lane - HALO;
    const bool owner = lane >= HALO;
    const float log2e = (float)LOG2E;
    int cls[PPT], slot[PPT];
    bool cnt[PPT];
    float gs[PPT], ga[PPT], a[PPT];
#pragma unroll
    for (int j = 0; j < PPT; ++j) {
        const int i = gi * PPT + j;
        const bool real = i >= 0 && i < L;
        const int li = dir ? L - 1 - i : i;
        cls[j] = real ? lab[li] : 0;
        gs[j] = real ? trans[(size_t)cls[j] * d.C + cls[j]] * log2e : NEG;
        ga[j] = NEG;
        if (real && i >= 1) {
            const int prev = lab[dir ? li + 1 : li - 1];  // the position entered from, in this direction
            ga[j] = (dir ? trans[(size_t)prev * d.C + cls[j]] : trans[(size_t)cls[j] * d.C + prev]) * log2e;
        } else if (i == 0) {
            ga[j] = 0.f;
        }
        slot[j] = (real && owner) ? i : d.Lmax + j;
        cnt[j] = real && owner;
        a[j] = (i == -1) ? 0.f : NEG;
    }
    auto frame = [&](int step) { return dir ? T - 1 - step : step; };
    double offset = 0;  // true log2 value = relative value + offset
    const int nwaves = NT >> 6;
    const int tblocks = (T + BLK - 1) / BLK;
    const long long rstep = dir ? -(long long)d.Sp : d.Sp;
    float* rptr = lat + (size_t)frame(0) * d.Sp;
    float* const spare = lat + (size_t)d.Tp * d.Sp;

    // The emission rows of a block of BLK frames are staged in LDS by the whole workgroup (scaled to
    // base-2 logs, class-major: a step's read is the lane's fixed address plus a constant), in two
    // buffers; the rows are requested two blocks ahead and written to LDS at the block boundary, so
    // the recursion itself issues no vector loads and never waits on the memory counter that its own
    // lattice stores keep busy.  Element e of a block: step k = e / C, class c = e % C; in memory
    // the rows of a block are adjacent (reversed for the backward direction); steps past the last
    // frame are clamped to a valid address (what they read only feeds the spare row).
    const int nel = BLK * d.C, per_buf = d.C * PITCH, last_el = T * d.C - 1;
    int goff[NQ], loff[NQ];
    float raw0[NQ], raw1[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int e = min(tid + q * NT, nel - 1);
        const int k = e / d.C, c = e - k * d.C;
        goff[q] = dir ? c - k * d.C : e;
        loff[q] = (tid + q * NT < nel) ? c * PITCH + k : -1;
    }
    auto load_rows = [&](int tb, float (&raw)[NQ]) {
        const int base = dir ? (T - 1 - tb * BLK) * d.C : tb * BLK * d.C;
#pragma unroll
        for (int q = 0; q < NQ; ++q) raw[q] = em[min(max(base + goff[q], 0), last_el)];
    };
    auto write_rows = [&](int buf, const float (&raw)[NQ]) {
#pragma unroll
        for (int q = 0; q < NQ; ++q)
            if (loff[q] >= 0) tbl[buf * per_buf + loff[q]] = raw[q] * log2e;
    };
    const float* tl[PPT];
#pragma unroll
    for (int j = 0; j < PPT; ++j) tl[j] = tbl + cls[j] * PITCH;

    auto block = [&](int tb, float (&next)[NQ], float (&load)[NQ]) {
        const int cur = (tb & 1) * per_buf;
        load_rows(tb + 2, load);
        float sn[PPT];
#pragma unroll
        for (int j = 0; j < PPT; ++j) sn[j] = tl[j][cur];
#pragma unroll
        for (int k = 0; k < BLK; ++k) {
            const int step = tb * BLK + k;
            float s[PPT];
#pragma unroll
            for (int j = 0; j < PPT; ++j) s[j] = sn[j];
            if (k + 1 < BLK) {  // the next frame's scores, one step ahead
#pragma unroll
                for (int j = 0; j < PPT; ++j) sn[j] = tl[j][cur + k + 1];
            }
            float* const row = step < T ? rptr : spare;
            rptr += rstep;
            float carry = from_left_lane(a[PPT - 1], NEG);
#pragma unroll
            for (int j = 0; j < PPT; ++j) {
                const float o = a[j];
                const float n = s[j] + lse2_log2(o + gs[j], carry + ga[j]);
                carry = o;
                a[j] = n;
                row[slot[j]] = n;
            }
        }
        if (tid < BLK) {
            const int step = tb * BLK + tid;
            offs[step < T ? frame(step) : d.Tp] = offset;
        }
        // the rows in flight are not touched before the steps are done (tied to a value the last step produced)
#pragma unroll
        for (int q = 0; q < NQ; ++q) asm volatile("" : "+v"(next[q]), "+v"(a[0]));
        // ---- block boundary: refresh the mirror lanes from the left neighbour, renormalise
        const int par = tb & 1;
        float m = NEG;
#pragma unroll
        for (int j = 0; j < PPT; ++j) m = fmaxf(m, cnt[j] ? a[j] : NEG);
        m = wave_max_bcast(m);
        if (nwaves > 1) {
            if (lane == 0) wmax[par][wave] = m;
            if (lane >= OWN) {
#pragma unroll
                for (int j = 0; j < PPT; ++j) xbuf[par][wave][lane - OWN][j] = a[j];
            }
        }
        write_rows((tb + 1) & 1, next);
        __syncthreads();
        if (nwaves > 1) {
            if (wave > 0 && !owner) {
#pragma unroll
                for (int j = 0; j < PPT; ++j) a[j] = xbuf[par][wave - 1][lane][j];
            }
            m = wmax[par][0];
            for (int w2 = 1; w2 < nwaves; ++w2) m = fmaxf(m, wmax[par][w2]);
        }
        if (m > NEG_TEST) {  // uniform over the workgroup
#pragma unroll
            for (int j = 0; j < PPT; ++j) a[j] = a[j] > NEG_TEST ? a[j] - m : NEG;
            offset += (double)m;
        }
    };
    load_rows(0, raw0);
    write_rows(0, raw0);
    load_rows(1, raw1);
    __syncthreads();
    for (int tb = 0; tb < tblocks; tb += 2) {
        block(tb, raw1, raw0);
        if (tb + 1 < tblocks) block(tb + 1, raw0, raw1);
    }
    if (dir == 0) {  // FAL = a_{T-1}[L-1], read back from the stored row of the last frame
        __syncthreads();
        if (tid == 0) {
            const float v = L >= 1 ? __builtin_nontemporal_load(lat + (size_t)(T - 1) * d.Sp + (L - 1)) : NEG;
            const double off = __builtin_nontemporal_load(offs + (T - 1));
            *term_out = v < NEG_TEST ? -INFINITY : (double)v + off;
        }
    }
}

// ---- fully connected lattice, one direction (one wavefront; two in the rotation path further down).
//   A_0[i] = f[0][i];  A_t[i] = f[t][i] + lse_j( A_{t-1}[j] + G[i][j] ),  G = g (forward) or g^T (backward)
// Up to 32 classes: two lanes per class (lane = 2 * class + half), each taking half of the source
// classes j, combined with one DPP lane swap; up to 64 classes: one lane per class.  A step
// publishes the states through a small LDS array and reads the sources back as broadcast 16-byte
// reads (one wavefront: LDS operations execute in order, no barrier needed).
// Two recursions write the same rows (base-2 log of the state relative to the row's offset):
//  * linear, when the transition scores span at most LINEAR_RANGE bits: the states are kept as
//    plain numbers, a step is the matrix-vector product  n[i] = 2^(f'[i]) * sum_j E[i][j] a[j]  with
//    E = 2^(G - max G) <= 1 and f' = f[t] - max_i f[t][i]; every second step the result is scaled
//    by the power of two that brings the largest input state to [0.5, 1) -- exact, and tracked in
//    the offset.  Under that bound a step changes the largest state by a factor between
//    2^-(LINEAR_RANGE+1) and 2^7, so between two scalings the largest state stays above 2^-62:
//    what is flushed to zero is below 2^-64 of the largest state and could regain at most
//    2^LINEAR_RANGE of that in later frames;
//  * log domain otherwise: a full log-sum-exp per state and step (one exp2 per source class), which
//    takes any range of scores.
constexpr float LINEAR_RANGE = 30.f;  // bits, about 21 nats

__device__ __forceinline__ float swap_pair(float v)  // value of lane ^ 1
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1 /* quad_perm:[1,0,3,2] */, 0xf, 0xf, false));
}

// acc (+)= e * (x of the lane R places around this lane's row of 16): one DPP instruction per source.
// The _FIRST form sits behind two wait states: the first DPP read of a register that a vector
// instruction has just written.
#define W2L_DPP_TAIL(R) " row_ror:" #R " row_mask:0xf bank_mask:0xf bound_ctrl:1"
#define W2L_FMAC_ROR(acc, x, e, R) asm volatile("v_fmac_f32_dpp %0, %1, %2" W2L_DPP_TAIL(R) : "+v"(acc) : "v"(x), "v"(e))
#define W2L_MUL_ROR(acc, x, e, R) asm volatile("v_mul_f32_dpp %0, %1, %2" W2L_DPP_TAIL(R) : "=v"(acc) : "v"(x), "v"(e))
#define W2L_MUL_ROR_FIRST(acc, x, e, R) \
    asm volatile("s_nop 1\n\tv_mul_f32_dpp %0, %1, %2" W2L_DPP_TAIL(R) : "=v"(acc) : "v"(x), "v"(e))
// one link of the maximum over lanes 0..31 of non-negative floats (their bit patterns order like
// unsigned integers; result in lane 31 after row_shr:1,2,4,8 and row_bcast:15).  Two other
// instructions must separate it from the previous write of u.
#define W2L_MAX_LINK(u, CTRL) asm volatile("v_max_u32_dpp %0, %0, %0 " CTRL " bank_mask:0xf" : "+v"(u))
template <int R>
__device__ __forceinline__ int ror_i(int x)
{
    return R == 0 ? x : __builtin_amdgcn_update_dpp(0, x, 0x120 + (R == 0 ? 1 : R), 0xf, 0xf, true);
}
// Linear recursion for up to 32 classes without LDS: class = lane & 31, so a row of 16 lanes
// holds 16 classes and both halves of the wavefront hold every class.  A lane reaches the 16
// states of a row with DPP row rotations; lanes 0..31 sum over the source classes of their own
// row, lanes 32..63 -- after one row swap (v_permlane16_swap) -- over those of the other row, and
// one half swap (v_permlane32_swap) adds the two.  Which lane a rotation or a swap delivers is not
// assumed: the same operations are applied to the lane numbers first and the transition factors
// are laid out to match.  All 64 lanes end a step with the new state of their class.
// Two wavefronts share the work.  Wavefront 0 runs the recursion and touches no global memory: it
// reads a frame's normalised emission factors from an LDS ring and leaves the new (linear) states
// and the step's scaling exponent in another.  Wavefront 1 works one block of AHEAD frames ahead
// and one behind: it loads the emission rows of the next block, takes their per-frame maximum and
// exponentials, and turns the states of the previous block into the stored base-2 logs, the
// double-precision row offsets and, at the last frame, the lattice's total.  One workgroup
// barrier per block; both wavefronts pass the same number of them.
struct FccRings {
    float e[2][AHEAD][32];   // emission factors 2^(f log2 e - mx) of a block, by class
    float n[2][AHEAD][32];   // states after each frame of a block, by class
    float mx[4][AHEAD];      // per-frame maximum of the scaled emissions (kept until the block is written out)
    int ex[2][AHEAD];        // exponent taken off the input states at each (even) step of a block
};
__device__ __forceinline__ void fcc_linear_rows(const float* __restrict__ em, const float* __restrict__ trans, int T, int dir,
                                                float* __restrict__ lat, double* __restrict__ offs, double* term_out,
                                                const AsgDims& d, float gmax, FccRings& ring)
{
    const int lane = threadIdx.x & 63, ci = lane & 31, role = threadIdx.x >> 6;
    const bool real = ci < d.C, upper = lane >= 32;
    const float log2e = (float)LOG2E;
    const int tblocks = (T + AHEAD - 1) / AHEAD;
    auto frame = [&](int step) { return dir ? T - 1 - step : step; };
    if (role == 1) {
        // ---- wavefront 1: lanes 0..31 take the even frames of a block, lanes 32..63 the odd ones
        const int cl = real ? ci : 0;
        auto request = [&](int tb, float (&s)[AHEAD / 2]) {  // emission rows of block tb (frames past the end: the last frame again)
#pragma unroll
            for (int q = 0; q < AHEAD / 2; ++q) {
                const int step = tb * AHEAD + 2 * q + (upper ? 1 : 0);
                s[q] = em[(size_t)frame(step < T ? step : T - 1) * d.C + cl];
            }
        };
        auto prepare = [&](int tb, const float (&s)[AHEAD / 2]) {  // emission factors of block tb from its rows
#pragma unroll
            for (int q = 0; q < AHEAD / 2; ++q) {
                const int k = 2 * q + (upper ? 1 : 0);
                const float x = real ? s[q] * log2e : NEG;
                float m = x;
                m = fmaxf(m, dpp_f<0x111, 0xf>(m, m));  // row_shr:1
                m = fmaxf(m, dpp_f<0x112, 0xf>(m, m));  // row_shr:2
                m = fmaxf(m, dpp_f<0x114, 0xf>(m, m));  // row_shr:4
                m = fmaxf(m, dpp_f<0x118, 0xf>(m, m));  // row_shr:8
                m = fmaxf(m, dpp_f<0x142, 0xa>(m, m));  // row_bcast:15: lanes 31 and 63 hold the maximum of their half
                const float m_lo = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 31));
                const float m_hi = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 63));
                const float mk = upper ? m_hi : m_lo;
                ring.e[tb & 1][k][ci] = fast_exp2(x - mk);
                if (ci == 0) ring.mx[tb & 3][k] = mk;
            }
        };
        double offset = 0;
        const double gmax_d = (double)gmax;
        auto shr_d = [](double v, auto ctrl) {  // the value of the lane `n` to the left within a row of 16; 0 where there is none
            constexpr int CTRL = decltype(ctrl)::value;
            const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, true);
            const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, true);
            return __hiloint2double(hi, lo);
        };
        auto write_out = [&](int tb) {  // rows and offsets of block tb
            // offsets: lane k of every row of 16 lanes takes frame k's increment; an inclusive scan over the row
            // (double precision) gives all 16 offsets at once, and lanes 0..15 store them
            const int kk = lane & 15, step_k = tb * AHEAD + kk;
            const int exk = (kk & 1) ? 0 : ring.ex[tb & 1][kk];
            double run = (double)ring.mx[tb & 3][kk] + (step_k == 0 ? 0.0 : gmax_d + (double)exk);
            run += shr_d(run, std::integral_constant<int, 0x111>{});  // row_shr:1
            run += shr_d(run, std::integral_constant<int, 0x112>{});  // row_shr:2
            run += shr_d(run, std::integral_constant<int, 0x114>{});  // row_shr:4
            run += shr_d(run, std::integral_constant<int, 0x118>{});  // row_shr:8
            const double off = offset + run;
            if (lane < AHEAD) offs[step_k < T ? (size_t)frame(step_k) : (size_t)d.Tp] = off;  // frames past the end: the spare row
            offset = __shfl(off, AHEAD - 1, 64);
            const bool last = dir == 0 && tb == tblocks - 1;  // this block holds frame T-1: the lattice's total
            const double off_last = last ? __shfl(off, (T - 1) - tb * AHEAD, 64) : 0.0;
#pragma unroll
            for (int q = 0; q < AHEAD / 2; ++q) {
                const int k = 2 * q + (upper ? 1 : 0), step = tb * AHEAD + k;
                const float n = ring.n[tb & 1][k][ci];
                const size_t r = step < T ? (size_t)frame(step) : (size_t)d.Tp;
                lat[r * CP + ci] = fmaxf(fast_log2(n), NEG);
                if (last) {  // FCC = log2 sum_i 2^(A_{T-1}[i])
                    float sx = real ? n : 0.f;
                    sx += dpp_f<0x111, 0xf>(0.f, sx);
                    sx += dpp_f<0x112, 0xf>(0.f, sx);
                    sx += dpp_f<0x114, 0xf>(0.f, sx);
                    sx += dpp_f<0x118, 0xf>(0.f, sx);
                    sx += dpp_f<0x142, 0xa>(0.f, sx);  // lanes 31 and 63: the sum over their half
                    if (step == T - 1 && ci == 31) *term_out = (double)fast_log2(sx) + off_last;
                }
            }
        };
        // rows are requested two blocks before the recursion needs their factors: a block to arrive, a block to be worked on
        float rows0[AHEAD / 2], rows1[AHEAD / 2];
        request(0, rows0);
        request(1, rows1);
        prepare(0, rows0);
        __syncthreads();
        for (int tb = 0; tb < tblocks; tb += 2) {
            request(tb + 2, rows0);
            prepare(tb + 1, rows1);
            if (tb > 0) write_out(tb - 1);
            __syncthreads();
            if (tb + 1 < tblocks) {
                request(tb + 3, rows1);
                prepare(tb + 2, rows0);
                write_out(tb);
                __syncthreads();
            }
        }
        write_out(tblocks - 1);
        return;
    }
    // ---- wavefront 0: the recursion
    // The row swap returns two registers.  Applied to the lane numbers it tells which of the two a
    // lane has to take: lanes 0..31 the one that still holds their own number, lanes 32..63 the one
    // that holds a lane of the other row.  (The half swap needs no such choice: the sum of its two
    // results is the sum of both halves in every lane.)
    const auto sw16 = __builtin_amdgcn_permlane16_swap((unsigned)lane, (unsigned)lane, false, false);
    const bool take0 = upper ? ((sw16[0] ^ (unsigned)lane) & 16u) != 0 : sw16[0] == (unsigned)lane;
    const int xid = (int)((take0 ? sw16[0] : sw16[1]) & 31u);  // class whose state this lane feeds into the rotations
    float E[16];  // factors by rotation
    auto factor = [&](int src) {
        if (!real || src >= d.C) return 0.f;
        return fast_exp2((dir ? trans[(size_t)src * d.C + ci] : trans[(size_t)ci * d.C + src]) * log2e - gmax);
    };
#define W2L_E(R) E[R] = factor(ror_i<R>(xid));
    W2L_E(0) W2L_E(1) W2L_E(2) W2L_E(3) W2L_E(4) W2L_E(5) W2L_E(6) W2L_E(7)
    W2L_E(8) W2L_E(9) W2L_E(10) W2L_E(11) W2L_E(12) W2L_E(13) W2L_E(14) W2L_E(15)
#undef W2L_E
    float a = 0.f;
    __syncthreads();
    for (int tb = 0; tb < tblocks; ++tb) {
        const float* eb = &ring.e[tb & 1][0][ci];
        float* nb = &ring.n[tb & 1][0][ci];
        int* xb = &ring.ex[tb & 1][0];
        float e_next = eb[0];
#pragma unroll
        for (int k = 0; k < AHEAD; ++k) {
            const float s2 = e_next;
            if (k + 1 < AHEAD) e_next = eb[(k + 1) * 32];  // the next frame's factors, one step ahead
            // every second step: the exponent of the largest input state (0 for an all-zero input), folded
            // into the emission factor.  The five links of that reduction are dependent DPP instructions;
            // they are spread between the independent multiply-adds below, which cover their wait states.
            const bool scale = !(k & 1);
            unsigned mb = __float_as_uint(a);
            const auto o16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(a), false, false);
            const float x = __uint_as_float(take0 ? o16[0] : o16[1]);
            float acc[4];  // four chains: a dependent fma would wait for the one before it
            acc[0] = x * E[0];
            W2L_MUL_ROR_FIRST(acc[1], x, E[1], 1);
            W2L_MUL_ROR(acc[2], x, E[2], 2);
            W2L_MUL_ROR(acc[3], x, E[3], 3);
            if (scale) W2L_MAX_LINK(mb, "row_shr:1 row_mask:0xf");
            W2L_FMAC_ROR(acc[0], x, E[4], 4);
            W2L_FMAC_ROR(acc[1], x, E[5], 5);
            W2L_FMAC_ROR(acc[2], x, E[6], 6);
            if (scale) W2L_MAX_LINK(mb, "row_shr:2 row_mask:0xf");
            W2L_FMAC_ROR(acc[3], x, E[7], 7);
            W2L_FMAC_ROR(acc[0], x, E[8], 8);
            W2L_FMAC_ROR(acc[1], x, E[9], 9);
            if (scale) W2L_MAX_LINK(mb, "row_shr:4 row_mask:0xf");
            W2L_FMAC_ROR(acc[2], x, E[10], 10);
            W2L_FMAC_ROR(acc[3], x, E[11], 11);
            W2L_FMAC_ROR(acc[0], x, E[12], 12);
            if (scale) W2L_MAX_LINK(mb, "row_shr:8 row_mask:0xf");
            W2L_FMAC_ROR(acc[1], x, E[13], 13);
            W2L_FMAC_ROR(acc[2], x, E[14], 14);
            W2L_FMAC_ROR(acc[3], x, E[15], 15);
            if (scale) W2L_MAX_LINK(mb, "row_bcast:15 row_mask:0xa");
            const int ex = scale ? __builtin_amdgcn_frexp_expf(__uint_as_float((unsigned)__builtin_amdgcn_readlane((int)mb, 31))) : 0;
            const float e = scale ? __builtin_amdgcn_ldexpf(s2, -ex) : s2;
            if (scale) xb[k] = ex;  // every lane the same value to the same place
            const float part = (acc[0] + acc[1]) + (acc[2] + acc[3]);
            const auto o32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(part), __float_as_uint(part), false, false);
            const float raw = __uint_as_float(o32[0]) + __uint_as_float(o32[1]);  // lower half + upper half, in every lane
            const float n = (k == 0 && tb == 0) ? s2 : e * raw;
            a = n;
            nb[k * 32] = n;  // both halves store the same values to the same places: no lane masking in the loop
        }
        __syncthreads();
    }
}

template <int CMAX>
__device__ __forceinline__ void fcc_lattice(const float* __restrict__ em, const float* __restrict__ trans, int T, int dir,
                                            float* __restrict__ lat, double* __restrict__ offs, double* term_out,
                                            const AsgDims& d, float* abuf, FccRings& ring)
{
    constexpr int LPC = CMAX <= 32 ? 2 : 1;  // lanes per class
    constexpr int NSRC = CMAX / LPC;         // source classes per lane
    const int lane = threadIdx.x & 63;
    const int ci = lane / LPC, half = lane % LPC;
    const bool real = ci < d.C;
    const bool writer = real && half == 0;
    const float log2e = (float)LOG2E;
    float G[NSRC];
    float gmax = NEG, gmin = -NEG;
#pragma unroll
    for (int jj = 0; jj < NSRC; ++jj) {
        const int j = half * NSRC + jj;
        const bool on = real && j < d.C;
        G[jj] = on ? (dir ? trans[(size_t)j * d.C + ci] : trans[(size_t)ci * d.C + j]) * log2e : NEG;
        gmax = on ? fmaxf(gmax, G[jj]) : gmax;
        gmin = on ? fminf(gmin, G[jj]) : gmin;
    }
    gmax = wave_max_bcast(gmax);
    gmin = wave_min_bcast(gmin);
    const bool linear = gmax - gmin <= LINEAR_RANGE;  // uniform (false also for NaN or infinite scores)
    if (CMAX <= 32 && linear) {
        fcc_linear_rows(em, trans, T, dir, lat, offs, term_out, d, gmax, ring);
        return;
    }
    if (threadIdx.x >= 64) return;  // the other paths run on one wavefront
    auto frame = [&](int step) { return dir ? T - 1 - step : step; };
    const int cl = real ? ci : 0;
    float sc[AHEAD];
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) sc[k] = em[(size_t)frame(k < T ? k : T - 1) * d.C + cl];
    double offset = 0;  // true log2 value = stored value + offset
    const int tblocks = (T + AHEAD - 1) / AHEAD;
    const long long sstep = dir ? -(long long)d.C : d.C, rstep = dir ? -(long long)CP : CP;
    const float* sptr = em + (size_t)frame(AHEAD - 1 < T ? AHEAD - 1 : T - 1) * d.C;
    float* rptr = lat + (size_t)frame(0) * CP;
    float* const spare = lat + (size_t)d.Tp * CP;
    const float4* src = reinterpret_cast<const float4*>(abuf + half * NSRC);
    float v[NSRC];
    auto gather = [&](float a) {  // publish this lane's state, read this lane's source states
        abuf[ci] = a;
        __builtin_amdgcn_wave_barrier();  // compiler-level ordering only: the store stays ahead of the reads
#pragma unroll
        for (int q = 0; q < NSRC / 4; ++q) {
            const float4 x = src[q];
            v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
        }
        __builtin_amdgcn_wave_barrier();  // ... and the reads ahead of the next store
    };

    if (linear) {
#pragma unroll
        for (int jj = 0; jj < NSRC; ++jj) G[jj] = (real && half * NSRC + jj < d.C) ? fast_exp2(G[jj] - gmax) : 0.f;  // E
        float a = 0.f;
        for (int tb = 0; tb < tblocks; ++tb) {
            // the block's 16 frames of scores at once: per-frame maximum (16 interleaved DPP
            // reductions) and normalised emission factors; then the ring is refilled for the next block
            float s2[AHEAD], mx[AHEAD];
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = s2[k] = real ? sc[k] * log2e : NEG;
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = fmaxf(mx[k], dpp_f<0x111, 0xf>(mx[k], mx[k]));
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = fmaxf(mx[k], dpp_f<0x112, 0xf>(mx[k], mx[k]));
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = fmaxf(mx[k], dpp_f<0x114, 0xf>(mx[k], mx[k]));
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = fmaxf(mx[k], dpp_f<0x118, 0xf>(mx[k], mx[k]));
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = fmaxf(mx[k], dpp_f<0x142, 0xa>(mx[k], mx[k]));
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) mx[k] = fmaxf(mx[k], dpp_f<0x143, 0xc>(mx[k], mx[k]));
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) {
                mx[k] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx[k]), 63));
                s2[k] = fast_exp2(s2[k] - mx[k]);  // e
                const int step = tb * AHEAD + k;
                sptr += (step + AHEAD < T) ? sstep : 0;
                sc[k] = sptr[cl];
            }
#pragma unroll
            for (int k = 0; k < AHEAD; ++k) {
                const int step = tb * AHEAD + k;
                float* const row = step < T ? rptr : spare;
                rptr += rstep;
                gather(a);
                const float e = s2[k];
                // every second step: the exponent of the largest input state (0 for an all-zero input)
                const int ex = (k & 1) ? 0 : __builtin_amdgcn_frexp_expf(wave_max_bcast(a));
                float acc[4] = {0.f, 0.f, 0.f, 0.f};  // four chains: a dependent fma would wait for the one before it
#pragma unroll
                for (int jj = 0; jj < NSRC; ++jj) acc[jj & 3] = fmaf(v[jj], G[jj], acc[jj & 3]);
                float raw = (acc[0] + acc[1]) + (acc[2] + acc[3]);
                if (LPC == 2) raw += swap_pair(raw);
                const float n = step == 0 ? e : ((k & 1) ? e * raw : __builtin_amdgcn_ldexpf(e * raw, -ex));
                offset += (double)mx[k] + (step == 0 ? 0.0 : (double)gmax + (double)ex);
                if (dir == 0 && step == T - 1) {  // FCC = log2 sum_i 2^(A_{T-1}[i])
                    const float sx = wave_sum_bcast(writer ? n : 0.f);
                    if (lane == 0) *term_out = (double)fast_log2(sx) + offset;
                }
                a = n;
                if (half == 0) row[ci] = fmaxf(fast_log2(n), NEG);
                if (lane == 0) offs[step < T ? frame(step) : d.Tp] = offset;
            }
        }
        return;
    }

    float a = NEG;
    for (int tb = 0; tb < tblocks; ++tb) {
#pragma unroll
        for (int k = 0; k < AHEAD; ++k) {
            const int step = tb * AHEAD + k;
            const float s = real ? sc[k] * log2e : NEG;
            sptr += (step + AHEAD < T) ? sstep : 0;
            sc[k] = sptr[cl];
            float* const row = step < T ? rptr : spare;
            rptr += rstep;
            gather(a);
            // four interleaved chains for the maximum and for the sum
            float m4[4] = {NEG, NEG, NEG, NEG};
#pragma unroll
            for (int jj = 0; jj < NSRC; ++jj) {
                v[jj] += G[jj];
                m4[jj & 3] = fmaxf(m4[jj & 3], v[jj]);
            }
            float m = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
            if (LPC == 2) m = fmaxf(m, swap_pair(m));
            float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jj = 0; jj < NSRC; ++jj) s4[jj & 3] += fast_exp2(v[jj] - m);
            float sum = (s4[0] + s4[1]) + (s4[2] + s4[3]);
            if (LPC == 2) sum += swap_pair(sum);
            const float n = step == 0 ? s : s + (m + fast_log2(sum));
            if (dir == 0 && step == T - 1) {  // FCC = lse_i A_{T-1}[i]
                const float x = real ? n : NEG;
                const float mx = wave_max_bcast(x);
                const float sx = wave_sum_bcast(writer ? fast_exp2(x - mx) : 0.f);
                if (lane == 0) *term_out = (double)(mx + fast_log2(sx)) + offset;
            }
            a = real ? n : NEG;
            if (half == 0) row[ci] = a;
        }
        if (lane < AHEAD) {
            const int step = tb * AHEAD + lane;
            offs[step < T ? frame(step) : d.Tp] = offset;
        }
        const float m = wave_max_bcast(a);
        if (m > NEG_TEST) {
            a = a > NEG_TEST ? a - m : NEG;
            offset += (double)m;
        }
    }
}

// grid (4, B): x = 0/1 FAL forward/backward, 2/3 FCC forward/backward
template <int PPT, int CMAX, int MAXT, int BLK, int NQ>
__global__ __launch_bounds__(MAXT) void asg_lattice(const float* __restrict__ em, const float* __restrict__ trans,
                                                    const int* __restrict__ targets, const int* __restrict__ in_len,
                                                    const int* __restrict__ tgt_len, AsgWs w, AsgDims d)
{
    __shared__ float xbuf[2][16][AHEAD][4];
    __shared__ float ftbl[2 * CP * (AHEAD + 1)];  // forced alignment: emission rows of two blocks of frames, class-major
    __shared__ float wmax[2][16];
    __shared__ __align__(16) float abuf[64];
    __shared__ FccRings ring;
    __shared__ int bad;
    const int kind = blockIdx.x >> 1, dir = blockIdx.x & 1, b = blockIdx.y;
    const int tid = threadIdx.x, NT = blockDim.x;
    const int T = in_len[b], L = tgt_len[b];
    const bool bad_len = T < 0 || T > d.Tp || L < 0 || L > d.Lmax;  // uniform
    if (tid == 0) bad = 0;
    __syncthreads();
    const int* lab = targets + (size_t)b * d.Lmax;
    if (!bad_len)
        for (int i = tid; i < L; i += NT) {
            const int l = lab[i];
            if (l < 0 || l >= d.C) bad = 1;
        }
    __syncthreads();
    if (bad_len || bad) {
        if (blockIdx.x == 0 && tid == 0) w.status[b] = 2;
        return;
    }
    if (T == 0 || L == 0 || L > T) {  // nothing to run: no alignment, or no frames and no labels (loss 0)
        if (blockIdx.x == 0 && tid == 0) {
            w.status[b] = (T == 0 && L == 0) ? 0 : 1;
            w.terms[2 * b] = 0.0;
            w.terms[2 * b + 1] = (T == 0 && L == 0) ? 0.0 : -INFINITY;
        }
        return;
    }
    if (blockIdx.x == 0 && tid == 0) w.status[b] = 0;
    if (kind == 2) {
        // fifth workgroup of the utterance, beside the four recursions: the target positions sorted by
        // (class, position) and the start of every class in that order -- the fixed summation order of
        // the emission-gradient kernel.  A plain rank count (no atomics): position i goes to
        // #{j : y_j < y_i} + #{j < i : y_j = y_i}.
        int* ord = w.order + (size_t)b * d.Lmax;
        int* cst = w.cstart + (size_t)b * (d.C + 1);
        for (int i = tid; i < L; i += NT) {
            const int c = lab[i];
            int r = 0;
            for (int j = 0; j < L; ++j) {
                const int l = lab[j];
                r += (l < c || (l == c && j < i)) ? 1 : 0;
            }
            ord[r] = i;
        }
        for (int c = tid; c <= d.C; c += NT) {
            int r = 0;
            for (int j = 0; j < L; ++j) r += lab[j] < c ? 1 : 0;
            cst[c] = r;
        }
        return;
    }
    const float* emb = em + (size_t)b * d.Tp * d.C;
    if (kind == 0) {
        fal_lattice<PPT, BLK, NQ>(emb, trans, lab, T, L, dir, w.fal[dir] + (size_t)b * (d.Tp + 1) * d.Sp,
                                  w.faloff[dir] + (size_t)b * (d.Tp + 1), w.terms + 2 * b + 1, d, xbuf, wmax, ftbl);
    } else {
        if (tid >= 128) return;  // two wavefronts: the recursion and its helper (the launch has at least two)
        fcc_lattice<CMAX>(emb, trans, T, dir, w.fcc[dir] + (size_t)b * (d.Tp + 1) * CP,
                          w.fccoff[dir] + (size_t)b * (d.Tp + 1), w.terms + 2 * b, d, abuf, ring);
    }
}

// Node occupancies and the loss.  One wavefront per frame; a workgroup of 4 wavefronts takes `rows_per_wg` consecutive frames of one utterance.
//   grad_em[t][c] = grad_scale * ( P_fcc(pi_t = c) - P_fal(pi_t = c) )
__global__ __launch_bounds__(256) void asg_grad_em(const float* __restrict__ em, const int* __restrict__ targets,
                                                   const int* __restrict__ in_len, const int* __restrict__ tgt_len,
                                                   float* __restrict__ loss, float* __restrict__ grad, AsgWs w, AsgDims d,
                                                   int rows_per_wg, float grad_scale)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int b = blockIdx.y, t0 = blockIdx.x * rows_per_wg;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* gb = grad + (size_t)b * d.Tp * d.C;
    const int status = w.status[b];
    const int T = in_len[b];
    const double fcc2 = w.terms[2 * b], fal2 = w.terms[2 * b + 1];
    if (blockIdx.x == 0 && tid == 0)
        loss[b] = status == 2 ? NAN : (status == 1 ? INFINITY : (float)((fcc2 - fal2) * LN2));
    const int t_end = min(t0 + rows_per_wg, d.Tp);
    if (status != 0 || t0 >= T) {
        for (int e = t0 * d.C + tid; e < t_end * d.C; e += 256) gb[e] = 0.f;
        return;
    }
    const int L = tgt_len[b];
    int* lab = reinterpret_cast<int*>(smem_raw);  // [Lmax]
    int* order = lab + d.Lmax;                    // [Lmax] positions sorted by (class, position)
    int* cstart = order + d.Lmax;                 // [C+1]
    float* ebuf = reinterpret_cast<float*>(cstart + d.C + 1) + (size_t)wave * d.Sp;  // [4][Sp]
    for (int i = tid; i < L; i += 256) {
        lab[i] = targets[(size_t)b * d.Lmax + i];
        order[i] = w.order[(size_t)b * d.Lmax + i];
    }
    for (int c = tid; c <= d.C; c += 256) cstart[c] = w.cstart[(size_t)b * (d.C + 1) + c];
    __syncthreads();

    const float log2e = (float)LOG2E;
    const size_t rowb = (size_t)b * (d.Tp + 1);
    for (int t = t0 + wave; t < t_end; t += 4) {
        float* grow = gb + (size_t)t * d.C;
        if (t >= T) {
            for (int c = lane; c < d.C; c += 64) grow[c] = 0.f;
            continue;
        }
        const float* erow = em + ((size_t)b * d.Tp + t) * d.C;
        // fully connected: lane = class
        const float shiftF = (float)(w.fccoff[0][rowb + t] + w.fccoff[1][rowb + t] - fcc2);
        float pf = 0.f;
        if (lane < d.C) {
            const float av = w.fcc[0][(rowb + t) * CP + lane], bv = w.fcc[1][(rowb + t) * CP + lane];
            if (av > NEG_TEST && bv > NEG_TEST) pf = fast_exp2((av + bv) + (shiftF - erow[lane] * log2e));
        }
        const float zf = wave_sum_bcast(pf);
        // forced alignment: lanes stride over the positions (backward rows are stored in reversed order);
        // the loads of GRAD_UNROLL positions per lane are issued together
        const float shiftA = (float)(w.faloff[0][rowb + t] + w.faloff[1][rowb + t] - fal2);
        const float* ar = w.fal[0] + (rowb + t) * d.Sp;
        const float* br = w.fal[1] + (rowb + t) * d.Sp;
        float za = 0.f;
        for (int s0 = lane; s0 < L; s0 += 64 * GRAD_UNROLL) {
            float av[GRAD_UNROLL], bv[GRAD_UNROLL], sc[GRAD_UNROLL];
#pragma unroll
            for (int u = 0; u < GRAD_UNROLL; ++u) {
                const int sidx = min(s0 + 64 * u, L - 1);  // clamped lanes repeat a valid position and are dropped below
                av[u] = ar[sidx];
                bv[u] = br[L - 1 - sidx];
                sc[u] = erow[lab[sidx]];
            }
#pragma unroll
            for (int u = 0; u < GRAD_UNROLL; ++u) {
                const int sidx = s0 + 64 * u;
                float e = 0.f;
                if (av[u] > NEG_TEST && bv[u] > NEG_TEST) e = fast_exp2((av[u] + bv[u]) + (shiftA - sc[u] * log2e));
                if (sidx < L) {
                    ebuf[sidx] = e;
                    za += e;
                }
            }
        }
        za = wave_sum_bcast(za);
        const float izf = zf > 0.f ? 1.f / zf : 0.f, iza = za > 0.f ? 1.f / za : 0.f;
        if (lane == 0) {
            w.izf[(size_t)b * d.Tp + t] = izf;
            w.iza[(size_t)b * d.Tp + t] = iza;
        }
        __builtin_amdgcn_wave_barrier();
        if (lane < d.C) {
            float g = 0.f;
            for (int q = cstart[lane]; q < cstart[lane + 1]; ++q) g += ebuf[order[q]];
            grow[lane] = grad_scale * (pf * izf - g * iza);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Edge occupancies summed over a chunk of frames.  Workgroup (chunk, utterance).
//   FCC: partF[i*C+j] = sum_t P_fcc(pi_t = i, pi_{t-1} = j)
//   FAL: partA[0][s]  = sum_t P_fal(position s at t-1 and at t),  partA[1][s] = sum_t P_fal(s-1 at t-1, s at t)
// An edge's weight is exp2( fwd_{t-1}[source] + g + bwd_t[destination] - total ), normalised by the
// node normaliser of frame t (the edge occupancies of a frame sum to the same 1).
__global__ __launch_bounds__(256) void asg_trans_partial(const float* __restrict__ trans, const int* __restrict__ targets,
                                                         const int* __restrict__ in_len, const int* __restrict__ tgt_len,
                                                         AsgWs w, AsgDims d)
{
    __shared__ float sA[CHUNK + 1][CP];  // forward rows t0-1 .. t0+CHUNK-1
    __shared__ float sB[CHUNK][CP];      // backward rows t0 .. t0+CHUNK-1
    __shared__ float wF[CHUNK], wA[CHUNK];
    const int ch = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int C2 = d.C * d.C;
    float* pF = w.partF + ((size_t)b * d.nch + ch) * C2;
    float* pA = w.partA + ((size_t)b * d.nch + ch) * 2 * d.Lmax;
    const int T = in_len[b], L = tgt_len[b];
    const int t0 = ch * CHUNK;
    const int tlo = t0 < 1 ? 1 : t0, thi = t0 + CHUNK < T ? t0 + CHUNK : T;  // frames [tlo, thi)
    if (w.status[b] != 0 || tlo >= thi) {
        for (int p = tid; p < C2; p += 256) pF[p] = 0.f;
        for (int s = tid; s < 2 * d.Lmax; s += 256) pA[s] = 0.f;
        return;
    }
    const size_t rowb = (size_t)b * (d.Tp + 1);
    const double fcc2 = w.terms[2 * b], fal2 = w.terms[2 * b + 1];
    for (int e = tid; e < (CHUNK + 1) * CP; e += 256) {
        const int r = e / CP, c = e - r * CP, t = t0 - 1 + r;
        sA[r][c] = (t >= 0 && t < T && c < d.C) ? w.fcc[0][(rowb + t) * CP + c] : NEG;
    }
    for (int e = tid; e < CHUNK * CP; e += 256) {
        const int r = e / CP, c = e - r * CP, t = t0 + r;
        sB[r][c] = (t < T && c < d.C) ? w.fcc[1][(rowb + t) * CP + c] : NEG;
    }
    if (tid < CHUNK) {
        const int t = t0 + tid;
        float f = NEG, a = NEG;
        if (t >= tlo && t < thi) {
            const float izf = w.izf[(size_t)b * d.Tp + t], iza = w.iza[(size_t)b * d.Tp + t];
            if (izf > 0.f) f = (float)(w.fccoff[0][rowb + t - 1] + w.fccoff[1][rowb + t] - fcc2) + fast_log2(izf);
            if (iza > 0.f) a = (float)(w.faloff[0][rowb + t - 1] + w.faloff[1][rowb + t] - fal2) + fast_log2(iza);
        }
        wF[tid] = f;
        wA[tid] = a;
    }
    __syncthreads();
    const float log2e = (float)LOG2E;
    for (int p = tid; p < C2; p += 256) {
        const int i = p / d.C, j = p - i * d.C;
        const float g2 = trans[p] * log2e;
        float acc = 0.f;
        for (int r = tlo - t0; r < thi - t0; ++r) acc += fast_exp2((sA[r][j] + sB[r][i]) + (g2 + wF[r]));
        pF[p] = acc;
    }
    const int* lab = targets + (size_t)b * d.Lmax;
    for (int s = tid; s < d.Lmax; s += 256) {
        float stay = 0.f, adv = 0.f;
        if (s < L) {
            const int c = lab[s];
            const float gs = trans[(size_t)c * d.C + c] * log2e;
            const float ga = s >= 1 ? trans[(size_t)c * d.C + lab[s - 1]] * log2e : NEG;
            const float* a0 = w.fal[0] + rowb * d.Sp + s;                // forward row t-1 is read at a0[(t-1) * Sp]
            const float* b0 = w.fal[1] + rowb * d.Sp + (L - 1 - s);      // backward rows are stored in reversed order
            for (int t = tlo; t < thi; t += 8) {   // loads of eight frames in flight together
                float x0[8], x1[8], y[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int tt = t + u < thi ? t + u : thi - 1;
                    x0[u] = a0[(size_t)(tt - 1) * d.Sp];
                    x1[u] = s >= 1 ? a0[(size_t)(tt - 1) * d.Sp - 1] : NEG;
                    y[u] = b0[(size_t)tt * d.Sp];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (t + u >= thi) break;
                    const float bv = y[u] + wA[t + u - t0];
                    stay += fast_exp2((x0[u] + bv) + gs);
                    adv += fast_exp2((x1[u] + bv) + ga);
                }
            }
        }
        pA[s] = stay;
        pA[d.Lmax + s] = adv;
    }
}

// Per utterance: d loss_b / d g as a C x C table.  FAL edge sums (added over the chunks in
// order) are scattered into the table as 64-bit fixed-point numbers with integer atomics -- integer
// addition does not depend on the order, so the result is reproducible -- and subtracted from
// the FCC edge sums (added over the chunks in order).
constexpr double FIXED_ONE = 4294967296.0;  // 2^32: occupancies up to 2^31 frames, resolved to 2.3e-10
__global__ __launch_bounds__(256) void asg_trans_utt(const int* __restrict__ targets, const int* __restrict__ tgt_len,
                                                     AsgWs w, AsgDims d)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int b = blockIdx.x, tid = threadIdx.x, C2 = d.C * d.C;
    float* tab = w.tabD + (size_t)b * C2;
    if (w.status[b] != 0) {
        for (int p = tid; p < C2; p += 256) tab[p] = 0.f;
        return;
    }
    const int L = tgt_len[b];
    unsigned long long* fal = reinterpret_cast<unsigned long long*>(smem_raw);  // [C*C]
    for (int p = tid; p < C2; p += 256) fal[p] = 0ull;
    __syncthreads();
    const int* lab = targets + (size_t)b * d.Lmax;
    const float* pA = w.partA + (size_t)b * d.nch * 2 * d.Lmax;
    for (int s = tid; s < L; s += 256) {
        float stay = 0.f, adv = 0.f;
#pragma unroll 8
        for (int ch = 0; ch < d.nch; ++ch) {
            stay += pA[(size_t)ch * 2 * d.Lmax + s];
            adv += pA[(size_t)ch * 2 * d.Lmax + d.Lmax + s];
        }
        const int c = lab[s];
        atomicAdd(&fal[c * d.C + c], (unsigned long long)(long long)__double2ll_rn((double)stay * FIXED_ONE));
        if (s >= 1)
            atomicAdd(&fal[c * d.C + lab[s - 1]], (unsigned long long)(long long)__double2ll_rn((double)adv * FIXED_ONE));
    }
    __syncthreads();
    const float* pF = w.partF + (size_t)b * d.nch * C2;
    for (int p = tid; p < C2; p += 256) {
        float f = 0.f;
#pragma unroll 8
        for (int ch = 0; ch < d.nch; ++ch) f += pF[(size_t)ch * C2 + p];
        tab[p] = f - (float)((double)(long long)fal[p] * (1.0 / FIXED_ONE));
    }
}

//   grad_trans[p] = grad_scale * sum_b tabD[b][p], added in the order b = 0, 1, ...
__global__ __launch_bounds__(64) void asg_trans_reduce(float* __restrict__ grad_trans, AsgWs w, AsgDims d, float grad_scale)
{
    const int p = blockIdx.x * 64 + threadIdx.x, C2 = d.C * d.C;
    if (p >= C2) return;
    float acc = 0.f;
#pragma unroll 8
    for (int b = 0; b < d.B; ++b) acc += w.tabD[(size_t)b * C2 + p];
    grad_trans[p] = grad_scale * acc;
}

struct WsLayout { size_t fal[2], fcc[2], faloff[2], fccoff[2], terms, status, izf, iza, partF, partA, tabD, order, cstart, total; };
WsLayout ws_layout(int B, int Tp, int C, int Lmax)
{
    WsLayout w;
    size_t off = 0;
    const size_t rows = (size_t)B * (Tp + 1);
    const int nch = (Tp + CHUNK - 1) / CHUNK;
    for (int q = 0; q < 2; ++q) { w.fal[q] = off; off += round_up(rows * ((size_t)Lmax + 4) * 4, 256); }
    for (int q = 0; q < 2; ++q) { w.fcc[q] = off; off += round_up(rows * CP * 4, 256); }
    for (int q = 0; q < 2; ++q) { w.faloff[q] = off; off += round_up(rows * 8, 256); }
    for (int q = 0; q < 2; ++q) { w.fccoff[q] = off; off += round_up(rows * 8, 256); }
    w.terms = off; off += round_up((size_t)B * 16, 256);
    w.status = off; off += round_up((size_t)B * 4, 256);
    w.izf = off; off += round_up((size_t)B * Tp * 4, 256);
    w.iza = off; off += round_up((size_t)B * Tp * 4, 256);
    w.partF = off; off += round_up((size_t)B * nch * C * C * 4, 256);
    w.partA = off; off += round_up((size_t)B * nch * 2 * Lmax * 4, 256);
    w.tabD = off; off += round_up((size_t)B * C * C * 4, 256);
    w.order = off; off += round_up((size_t)B * Lmax * 4, 256);
    w.cstart = off; off += round_up((size_t)B * (C + 1) * 4, 256);
    w.total = off;
    return w;
}

// Which asg_lattice<PPT, CMAX, MAXT, BLK, NQ> variant a problem takes, and its launch shape.
// Forced alignment: one lane per PPT target positions, 64 - BLK of them per wavefront.  A step is bound by
// instruction issue, so a wavefront wants a SIMD of its own: the smallest PPT that fits four wavefronts, with
// blocks of 16 frames if that fits and of 12 (52 owned lanes) otherwise; longer targets take four positions
// per lane on as many wavefronts as they need.  (The register budget, MAXT, follows the workgroup size.)
// NQ: emission-row elements a thread stages per block (BLK * C <= 1024 <= 8 threads).
struct AsgLaunch { int ppt, blk, nt, nq, cmax, maxt; };
AsgLaunch asg_launch_config(int C, int Lmax)
{
    int ppt = 4, blk = 16;
    for (int p = 1; p <= 4; p *= 2) {
        if (Lmax <= 4 * 48 * p) { ppt = p; blk = 16; break; }
        if (Lmax <= 4 * 52 * p) { ppt = p; blk = 12; break; }
    }
    const int own = 64 - blk;
    int nt = 64 * (((Lmax + ppt - 1) / ppt + own - 1) / own);
    if (nt < 128) nt = 128;  // the fully connected lattice runs on two wavefronts
    const int maxt = nt > 256 ? 1024 : 256;
    if (maxt == 1024) { ppt = 4; blk = 16; }
    const int nq = blk * C <= 2 * nt ? 2 : 8;
    return AsgLaunch{ppt, blk, nt, nq, C <= 32 ? 32 : 64, maxt};
}

template <int PPT, int MAXT, int BLK>
void launch_lattice(int cmax, int nq, dim3 grid, dim3 block, hipStream_t st, const float* em, const float* trans,
                    const int* targets, const int* in_len, const int* tgt_len, const AsgWs& w, const AsgDims& d)
{
#define W2L_ASG_LAUNCH(C_, Q_) \
    hipLaunchKernelGGL((asg_lattice<PPT, C_, MAXT, BLK, Q_>), grid, block, 0, st, em, trans, targets, in_len, tgt_len, w, d)
    // only the combinations asg_launch_config() can produce are compiled: with at most 32 classes a block of 12
    // frames (or a workgroup of more than 256 threads) always stages 2 values per thread, and with more than
    // 32 classes a block of 16 frames on at most 256 threads always stages 8
    if (cmax <= 32) {
        if constexpr (BLK == 12 || MAXT == 1024) {
            W2L_ASG_LAUNCH(32, 2);
        } else {
            if (nq == 2) W2L_ASG_LAUNCH(32, 2); else W2L_ASG_LAUNCH(32, 8);
        }
    } else {
        if constexpr (BLK == 16 && MAXT == 256) {
            W2L_ASG_LAUNCH(64, 8);
        } else {
            if (nq == 2) W2L_ASG_LAUNCH(64, 2); else W2L_ASG_LAUNCH(64, 8);
        }
    }
#undef W2L_ASG_LAUNCH
}

}  // namespace
}  // namespace w2l

using namespace w2l;

extern "C" size_t w2l_asg_workspace_bytes(int B, int Tp, int C, int Lmax)
{
    if (B <= 0 || Tp <= 0 || C <= 0 || C > CP || Lmax <= 0) return 0;
    return ws_layout(B, Tp, C, Lmax).total;
}

extern "C" int w2l_asg_launch_config(int C, int Lmax, int* positions_per_lane, int* class_lanes, int* max_threads,
                                     int* frames_per_block, int* row_values_per_thread, int* threads)
{
    if (!positions_per_lane || !class_lanes || !max_threads || !frames_per_block || !row_values_per_thread || !threads)
        return W2L_ERR_NULL;
    if (C <= 0 || C > CP || Lmax <= 0 || Lmax > 3000) return W2L_ERR_SHAPE;
    const AsgLaunch cfg = asg_launch_config(C, Lmax);
    if (cfg.nt > 1024) return W2L_ERR_SHAPE;
    *positions_per_lane = cfg.ppt;
    *class_lanes = cfg.cmax;
    *max_threads = cfg.maxt;
    *frames_per_block = cfg.blk;
    *row_values_per_thread = cfg.nq;
    *threads = cfg.nt;
    return W2L_OK;
}

extern "C" int w2l_asg_check_targets_host(const int* targets, const int* in_len, const int* tgt_len, int B, int Tp,
                                          int C, int Lmax)
{
    if (!targets || !in_len || !tgt_len) return W2L_ERR_NULL;
    if (B <= 0 || Tp <= 0 || C <= 0 || Lmax <= 0) return W2L_ERR_SHAPE;
    for (int b = 0; b < B; ++b) {
        if (in_len[b] < 0 || in_len[b] > Tp || tgt_len[b] < 0 || tgt_len[b] > Lmax) return W2L_ERR_TARGET;
        for (int i = 0; i < tgt_len[b]; ++i) {
            const int l = targets[(size_t)b * Lmax + i];
            if (l < 0 || l >= C) return W2L_ERR_TARGET;
        }
    }
    return W2L_OK;
}

extern "C" int w2l_asg_fwd_bwd(const float* emissions, const float* trans, const int* targets, const int* in_len,
                               const int* tgt_len, float* loss, float* grad_emissions, float* grad_trans, int B, int Tp,
                               int C, int Lmax, float grad_scale, void* workspace, size_t ws_bytes, void* stream)
{
    if (!emissions || !trans || !targets || !in_len || !tgt_len || !loss || !grad_emissions) return W2L_ERR_NULL;
    if (B <= 0 || Tp <= 0 || C <= 0 || C > CP || Lmax <= 0 || Lmax > 3000 || B > 65535) return W2L_ERR_SHAPE;
    if (!aligned16(emissions) || !aligned16(targets) || !aligned16(grad_emissions)) return W2L_ERR_ALIGN;
    const WsLayout l = ws_layout(B, Tp, C, Lmax);
    if (!workspace || ws_bytes < l.total || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return W2L_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    AsgDims d{B, Tp, C, Lmax, Lmax + 4, (Tp + CHUNK - 1) / CHUNK};
    AsgWs w;
    for (int q = 0; q < 2; ++q) {
        w.fal[q] = reinterpret_cast<float*>(ws + l.fal[q]);
        w.fcc[q] = reinterpret_cast<float*>(ws + l.fcc[q]);
        w.faloff[q] = reinterpret_cast<double*>(ws + l.faloff[q]);
        w.fccoff[q] = reinterpret_cast<double*>(ws + l.fccoff[q]);
    }
    w.terms = reinterpret_cast<double*>(ws + l.terms);
    w.status = reinterpret_cast<int*>(ws + l.status);
    w.izf = reinterpret_cast<float*>(ws + l.izf);
    w.iza = reinterpret_cast<float*>(ws + l.iza);
    w.partF = reinterpret_cast<float*>(ws + l.partF);
    w.partA = reinterpret_cast<float*>(ws + l.partA);
    w.tabD = reinterpret_cast<float*>(ws + l.tabD);
    w.order = reinterpret_cast<int*>(ws + l.order);
    w.cstart = reinterpret_cast<int*>(ws + l.cstart);

    const size_t lds_em = (size_t)4 * (2 * Lmax + C + 1) + (size_t)4 * 4 * (Lmax + 4);
    const size_t lds_tab = (size_t)8 * C * C;
    if (lds_em > 160 * 1024) return W2L_ERR_SHAPE;
    if (lds_em > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)asg_grad_em, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_em);
        if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    }
    const AsgLaunch cfg = asg_launch_config(C, Lmax);
    if (cfg.nt > 1024) return W2L_ERR_SHAPE;
    const int nt = cfg.nt, nq = cfg.nq;
    const dim3 g1(5, B), b1(nt);  // four recursions and the sort of the target
    if (cfg.maxt == 1024) launch_lattice<4, 1024, 16>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    else if (cfg.ppt == 1 && cfg.blk == 16) launch_lattice<1, 256, 16>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    else if (cfg.ppt == 1) launch_lattice<1, 256, 12>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    else if (cfg.ppt == 2 && cfg.blk == 16) launch_lattice<2, 256, 16>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    else if (cfg.ppt == 2) launch_lattice<2, 256, 12>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    else if (cfg.blk == 16) launch_lattice<4, 256, 16>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    else launch_lattice<4, 256, 12>(C, nq, g1, b1, st, emissions, trans, targets, in_len, tgt_len, w, d);
    int rc = launch_status();
    if (rc) return rc;
    // frames per emission-gradient workgroup: one per wavefront while the per-workgroup copy of the target's
    // sort (2 Lmax + C + 1 integers) is small beside the frames' own lattice rows, more otherwise
    const int rows_per_wg = (2 * Lmax + C + 1 <= 1024) ? 4 : 16;
    hipLaunchKernelGGL(asg_grad_em, dim3((Tp + rows_per_wg - 1) / rows_per_wg, B), dim3(256), lds_em, st, emissions, targets,
                       in_len, tgt_len, loss, grad_emissions, w, d, rows_per_wg, grad_scale);
    rc = launch_status();
    if (rc || !grad_trans) return rc;
    hipLaunchKernelGGL(asg_trans_partial, dim3(d.nch, B), dim3(256), 0, st, trans, targets, in_len, tgt_len, w, d);
    rc = launch_status();
    if (rc) return rc;
    hipLaunchKernelGGL(asg_trans_utt, dim3(B), dim3(256), lds_tab, st, targets, tgt_len, w, d);
    rc = launch_status();
    if (rc) return rc;
    hipLaunchKernelGGL(asg_trans_reduce, dim3((C * C + 63) / 64), dim3(64), 0, st, grad_trans, w, d, grad_scale);
    return launch_status();
}
