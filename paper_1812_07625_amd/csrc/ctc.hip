// CTC criterion on the GPU (paper Sec. 2.3; the paper runs its CTC on host cores,
// Sec. 4.1 -- this keeps the whole criterion on the device, so no device<->host round
// trip sits between the network's forward and backward passes).
//
// Three kernels, all deterministic (no floating-point atomics):
//   1. (logits only) per-frame log-softmax into the workspace;
//   2. ctc_lattice: one workgroup per (utterance, direction).  alpha runs forward in
//      time, beta is the same recursion on the reversed label sequence and reversed time,
//      so the two run concurrently and the serial chain is T_b steps, not 2 T_b.
//      A state is kept as a pair (v, e): its value is v * 2^e with v a float and e a 32-bit
//      integer -- the range of the log domain without a transcendental on the chain.  The
//      sum of predecessors aligns their exponents with v_ldexp and adds; the frame's score
//      enters as 2^(lp * log2 e) split into an integer exponent and a mantissa in [1, 2).
//      All terms are non-negative, so a mantissa never shrinks and grows by at most 6x per
//      frame: once per block of frames each lane moves the exponent of its own mantissas
//      into e.  Exponents carry a bias and a zero state has v = 0 and exponent 0, below
//      every real one, which keeps the step free of branches; the lattice rows hold the
//      (v, e) pairs.  A third workgroup per utterance sorts the target for kernel 3;
//   3. ctc_grad: one wavefront per frame combines alpha_t and beta_t (mantissas
//      multiplied, exponents added, log P taken off) into the state posteriors, normalises
//      them per frame, and sums them per class in a fixed order given by a (class, position)
//      sort of the target.
#include <mutex>
#include "common.h"

namespace w2l {
namespace {

constexpr double LN2 = 0.69314718055994530942;

struct CtcDims {
    int B, Tp, C, Lmax, blank;
    int len_div;  // in_len[] counts frames before the network's total stride: the criterion sees ceil(in_len / len_div)
    int Sp;    // lattice row pitch in states = 2*Lmax+4 (the last pair is a spare); a state is 8 bytes
    int rows;  // lattice rows per utterance = Tp + 2*LAT_PAD: frame t is row LAT_PAD + t
};

__device__ __forceinline__ int crit_len(int n, int div) { return (n < 0 || div <= 1) ? n : (n + div - 1) / div; }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// value of the lane to the left (lane - 1); lane 0 gets 0
__device__ __forceinline__ int from_left_lane_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x138 /* wave_shr:1 */, 0xf, 0xf, true);
}
__device__ __forceinline__ float from_left_lane(float v) { return __int_as_float(from_left_lane_i(__float_as_int(v))); }

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int LAT_PAD = 16;  // spare lattice rows at either end of an utterance = the longest block of frames

// A state's exponent is kept with a bias, so that 0 can stand for "zero state" (the value a lane
// shift fills in at the edge) and compares below every real exponent.  True exponents stay within
// +-MAX_FRAMES * 65536 = +-2^29 of zero, and the bias (which falls by EXP_DRIFT per frame, see below) within
// (2^29, 2^30]: a real state's biased exponent is positive and fits 31 bits.
constexpr int EXP_BIAS = 1 << 30;
constexpr int MAX_FRAMES = 8192;
constexpr float MIN_LOG2 = -65535.f;               // scores are clamped to 2^+-65535; below: probability zero
// A score enters the step as (mantissa, q) with q = EXP_DRIFT - exponent > 0, and the step takes q off a state's
// biased exponent with one saturating unsigned subtraction: the bias of every state falls by EXP_DRIFT per frame
// (row t of alpha carries EXP_BIAS - (t + 1) EXP_DRIFT, row t of beta EXP_BIAS - (T - t) EXP_DRIFT), a zero state
// stays at 0, and a zero score (q = Q_ZERO) sends any state to 0.  With MAX_FRAMES frames of scores clamped to
// 2^+-65535 a real state's biased exponent stays within (0, 2^30 + 2^16).
constexpr int EXP_DRIFT = 65536;
constexpr unsigned Q_ZERO = 0xffffffffu;
__device__ __forceinline__ int sub_sat(int e, unsigned q) { return (int)__builtin_elementwise_sub_sat((unsigned)e, q); }

// exp(s) = 2^(s log2 e) = 2^fl * 2^frac: fl an integer in [-65535, 65535] (the product is clamped there), frac in
// [0, 1] up to an ulp.  The rounding error of the product -- 0.004 for a score of -45000 -- and the tail of log2 e
// are recovered with an fma, so frac is good to fp32 whatever the size of the score.  Returns false for a score
// below 2^MIN_LOG2 (-inf included): probability zero.
constexpr float LOG2E_HI = 1.44269502162933349609375f;   // log2 e rounded to fp32
constexpr float LOG2E_LO = 1.92596299112661746e-8f;      // what the rounding dropped
__device__ __forceinline__ bool score_split(float s, float& fl, float& frac)
{
    const float xh = s * LOG2E_HI;
    const float xl = __builtin_fmaf(s, LOG2E_HI, -xh) + s * LOG2E_LO;
    const float x = fminf(fmaxf(xh, MIN_LOG2), -MIN_LOG2);
    fl = floorf(x);
    frac = (x - fl) + xl;
    return xh >= MIN_LOG2;
}

// v * 2^e for a (v, e) pair as a double-precision base-2 log; -inf for a zero state
__device__ __forceinline__ double pair_log2(float v, int e) { return v > 0.f ? (double)fast_log2(v) + (double)e : -INFINITY; }

// One workgroup per (utterance, direction).  The extended sequence is cut into pairs
// (blank 2i, label 2i+1); a lane holds PPT consecutive pairs in registers, so per frame it needs
// exactly one value from outside: the label state of the pair to its left, which a DPP
// whole-wavefront shift delivers from the neighbouring lane.  No value crosses a wavefront
// boundary inside a block of BLK frames: the first BLK lanes of every wavefront but the first
// recompute the pairs owned by the last lanes of the wavefront on its left (wavefront 0 owns all 64).  Their leftmost input
// is missing, so they go stale from the left at one pair per frame -- after BLK frames
// the staleness has not yet reached the lanes the wavefront owns -- and once per block they are
// refreshed through LDS, at the one barrier of the block.  States to the right of the target's
// last pair are computed too (nothing reads them; a state depends only on states to its left);
// states left of pair 0 stay zero.  beta is the same recursion on the reversed sequence and
// reversed time (state index q counts from the end), stored in its own q order.
// The step body is straight-line code with a fixed number of memory operations: lanes that own
// no real pair write to a spare pair, and the steps between the last frame and the end of its
// block of BLK frames run on like the others -- their rows land in the LAT_PAD spare
// rows that every utterance's lattice has at either end (alpha runs off the far end, beta off
// the near one) or in rows t >= T_b that nobody reads.
// Stored per frame and state: the pair (v, biased e), the integer as the bits of the second float.
// NQ > 0 (the class rows of a block of frames fit NQ values per thread): the scores do not come
// through per-lane loads at all.  The workgroup keeps the rows lp[t, 0..C-1] of the current
// block of BLK frames in LDS, already split into (mantissa, exponent), class-major
// (the frames of one class are adjacent, so a step's read is the lane's fixed address plus a
// constant), in two buffers: the rows of the next block are loaded (coalesced) before the
// block's steps start and written to the other buffer after them, so the recursion itself issues
// no vector loads and never waits on the memory counter that its own lattice stores keep busy.
// NQ == 0 (large alphabets): the scores lp[t, blank] and lp[t, label] are gathered per lane
// BLK frames early into a register ring.
// BLK = 16, or 12 where that brings the target onto four wavefronts (64 + 3 (64 - BLK) owned lanes):
// the step is bound by instruction issue -- one wavefront alone on its SIMD issues the ~25
// instructions of a step at the 4-cycle cadence -- so a fifth wavefront, which has to share a
// SIMD, costs more than a hand-over between wavefronts every 12 frames instead of every 16.
template <int PPT, int NQ, int BLK>
__global__ __launch_bounds__(1024) void ctc_lattice(const float* __restrict__ lp, const int* __restrict__ targets,
                                                    const int* __restrict__ in_len, const int* __restrict__ tgt_len,
                                                    float* __restrict__ loss, double* __restrict__ logp2_out,
                                                    float2* __restrict__ alpha, float2* __restrict__ beta,
                                                    int* __restrict__ sort_order, int* __restrict__ sort_start, CtcDims d)
{
    constexpr bool TABLE = NQ > 0;
    constexpr int HALO_LANES = BLK;             // lanes of a wavefront that mirror the wavefront on its left
    constexpr int OWN_LANES = 64 - HALO_LANES;  // lanes whose states a wavefront owns (and stores)
    constexpr int TABLE_PITCH = BLK + 1;        // table entries per class (one of padding against bank conflicts)
    __shared__ float xbuf[2][16][HALO_LANES][4 * PPT];  // [block parity][wavefront][lane - OWN_LANES][v, e of blank, label]
    __shared__ int bad_len, bad;
    extern __shared__ __align__(16) unsigned char dyn_smem[];
    float2* const tbl = reinterpret_cast<float2*>(dyn_smem);  // TABLE: [2][C][TABLE_PITCH] (pm, q)
    const int dir = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, NT = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int T = crit_len(in_len[b], d.len_div), L = tgt_len[b];
    if (tid == 0) {
        bad_len = (T < 0 || T > d.Tp || L < 0 || L > d.Lmax) ? 1 : 0;
        bad = 0;
    }
    __syncthreads();
    if (bad_len) {
        if (dir == 0 && tid == 0) { loss[b] = NAN; logp2_out[b] = NAN; }
        return;
    }
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
    if (T == 0) {
        if (dir == 0 && tid == 0) {
            loss[b] = (L == 0) ? 0.f : INFINITY;
            logp2_out[b] = (L == 0) ? 0.0 : -INFINITY;
        }
        return;
    }
    if (dir == 2) {
        // third workgroup of the utterance, beside the two recursions: the label positions sorted by
        // (class, position) and the start of every class in that order -- the fixed summation order
        // of the gradient kernel.  A plain rank count (no atomics): position i goes to
        // #{j : l_j < l_i} + #{j < i : l_j = l_i}.
        int* ord = sort_order + (size_t)b * d.Lmax;
        int* cst = sort_start + (size_t)b * (d.C + 1);
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
    // pair i (in this direction's order) = states q = 2i (blank), 2i+1 (label i, absent for i = L)
    // this lane's group of PPT pairs: wavefront 0 has nobody on its left and owns all 64 of its lanes' groups
    const int gi = wave == 0 ? lane : 64 + (wave - 1) * OWN_LANES + lane - HALO_LANES;
    const bool owner = wave == 0 || lane >= HALO_LANES;  // not a mirror of the wavefront on the left
    int cls[PPT];        // class of the label state
    bool skip[PPT];      // label state may be entered from the label of the pair to the left
    unsigned slot[PPT];  // byte offset of the pair in a lattice row (the spare pair for lanes that own no real pair)
    float vb[PPT], vl[PPT];
    int eb[PPT], el[PPT];  // biased exponents; 0 for a zero state
#pragma unroll
    for (int j = 0; j < PPT; ++j) {
        const int i = gi * PPT + j;
        const bool real = gi >= 0 && i <= L, has_l = gi >= 0 && i < L;
        const int li = dir ? L - 1 - i : i;          // label index in the target
        cls[j] = has_l ? lab[li] : d.blank;
        skip[j] = has_l && i >= 1 && lab[dir ? li + 1 : li - 1] != cls[j];
        slot[j] = 16u * (unsigned)((real && owner) ? i : d.Lmax + 1);
        // the state "before frame 0": all mass in front of pair 0, so that frame 0 comes out of the recursion itself
        const bool start = gi >= 0 && i == 0;
        vb[j] = start ? 1.f : 0.f;
        eb[j] = start ? EXP_BIAS : 0;
        vl[j] = 0.f;
        el[j] = 0;
    }
    const float* lpb = lp + (size_t)b * d.Tp * d.C;
    float2* lat = (dir ? beta : alpha) + ((size_t)b * d.rows + LAT_PAD) * d.Sp;  // row of frame 0
    auto frame = [&](int step) { return dir ? T - 1 - step : step; };

    const int nwaves = NT >> 6;
    const int tblocks = (T + BLK - 1) / BLK;
    // running pointers instead of per-step index arithmetic: the lattice row written next
    // (and, without the table, the score row fetched next, clamped at the last frame)
    const long long sstep = dir ? -(long long)d.C : d.C;
    // A lattice row is addressed as the utterance's slice (spare rows included) + the row's byte offset (uniform,
    // advanced once per step) + the lane's byte offset: one 32-bit add per store.
    char* const lat_slice = reinterpret_cast<char*>((dir ? beta : alpha) + (size_t)b * d.rows * d.Sp);
    const int row_bytes = d.Sp * (int)sizeof(float2), rstep = dir ? -row_bytes : row_bytes;
    int rptr = (LAT_PAD + frame(0)) * row_bytes;
    // exp(lp) = 2^(lp log2 e) = pm * 2^pe with pm in [1, 2); a score below 2^MIN_LOG2 (-inf included) is probability zero
    auto split = [&](float s, float& pm, unsigned& pq) {
        float fl, frac;
        const bool pos = score_split(s, fl, frac);
        pq = pos ? (unsigned)(EXP_DRIFT - (int)fl) : Q_ZERO;
        pm = pos ? fast_exp2(frac) : 0.f;
    };
    // one frame of the recursion for this lane's pairs, given the split scores.  A sum of states brings
    // them to their largest exponent (exact) and adds; a zero state (v = 0, exponent 0, far below any
    // real state's biased exponent) drops out by itself, and a sum of zeros stays at exponent 0
    // through the max() (a zero score's exponent pulls any sum below 0).
    auto advance = [&](int row, float pmb, unsigned qb, const float (&pml)[PPT], const unsigned (&ql)[PPT]) {
        // label state (previous frame) of the pair to the left of this lane's first pair
        float cv = from_left_lane(vl[PPT - 1]);
        int ce = from_left_lane_i(el[PPT - 1]);
#pragma unroll
        for (int j = 0; j < PPT; ++j) {
            const float obv = vb[j], olv = vl[j];
            const int obe = eb[j], ole = el[j];
            // blank: from itself and from the label on its left
            const int E1 = max(obe, ce);
            const float s1 = __builtin_amdgcn_ldexpf(obv, obe - E1) + __builtin_amdgcn_ldexpf(cv, ce - E1);
            // label: from itself, and from its blank alone or, where the label on its left differs, from the sum
            // just formed for the blank (its blank + that label)
            const float xv = skip[j] ? s1 : obv;
            const int xe = skip[j] ? E1 : obe;
            const int E2 = max(ole, xe);
            const float s2 = __builtin_amdgcn_ldexpf(olv, ole - E2) + __builtin_amdgcn_ldexpf(xv, xe - E2);
            cv = olv;
            ce = ole;
            vb[j] = pmb * s1;
            eb[j] = sub_sat(E1, qb);
            vl[j] = pml[j] * s2;
            el[j] = sub_sat(E2, ql[j]);
            const u32x4 st = {__float_as_uint(vb[j]), (unsigned)eb[j], __float_as_uint(vl[j]), (unsigned)el[j]};
            *reinterpret_cast<u32x4*>(lat_slice + (unsigned)(row + (int)slot[j])) = st;
        }
    };
    // block boundary: every lane moves the exponents of its mantissas into e; the mirror lanes
    // are refreshed from the left neighbour (one workgroup barrier)
    auto boundary = [&](int tb, bool sync_always, auto&& before_barrier) {
#pragma unroll
        for (int j = 0; j < PPT; ++j) {
            const int xb = __builtin_amdgcn_frexp_expf(vb[j]), xl = __builtin_amdgcn_frexp_expf(vl[j]);  // 0 for a zero state
            vb[j] = __builtin_amdgcn_ldexpf(vb[j], -xb);
            eb[j] += xb;
            vl[j] = __builtin_amdgcn_ldexpf(vl[j], -xl);
            el[j] += xl;
        }
        const int par = tb & 1;
        if (nwaves > 1 && lane >= OWN_LANES) {
#pragma unroll
            for (int j = 0; j < PPT; ++j) {
                float* q = &xbuf[par][wave][lane - OWN_LANES][4 * j];
                q[0] = vb[j]; q[1] = __int_as_float(eb[j]); q[2] = vl[j]; q[3] = __int_as_float(el[j]);
            }
        }
        before_barrier();  // work that only has to be done by the barrier: issued while the hand-over writes are on their way
        if (nwaves > 1 || sync_always) __syncthreads();
        if (nwaves > 1 && wave > 0 && !owner) {
#pragma unroll
            for (int j = 0; j < PPT; ++j) {
                const float* q = &xbuf[par][wave - 1][lane][4 * j];
                vb[j] = q[0]; eb[j] = __float_as_int(q[1]); vl[j] = q[2]; el[j] = __float_as_int(q[3]);
            }
        }
    };

    if constexpr (TABLE) {
        // element e of a block's rows: step k = e / C of the block, class c = e % C.  In memory the
        // rows of a block are adjacent (in reversed order for beta), so an element's address is the
        // block's base plus a per-thread constant; steps past the last frame are clamped to a
        // valid address (whatever they read only feeds the spare rows).
        const int nel = BLK * d.C, per_buf = d.C * TABLE_PITCH, last = T * d.C - 1;
        int goff[NQ], loff[NQ];
        float raw0[NQ], raw1[NQ];  // rows in flight: loaded two blocks before the block that uses them
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int e = min(tid + q * NT, nel - 1);
            const int k = e / d.C, c = e - k * d.C;
            goff[q] = dir ? c - k * d.C : e;
            loff[q] = (tid + q * NT < nel) ? c * TABLE_PITCH + k : -1;
        }
        auto load_rows = [&](int tb, float (&raw)[NQ]) {
            const int base = dir ? (T - 1 - tb * BLK) * d.C : tb * BLK * d.C;
#pragma unroll
            for (int q = 0; q < NQ; ++q) raw[q] = lpb[min(max(base + goff[q], 0), last)];
        };
        auto write_rows = [&](int buf, const float (&raw)[NQ]) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                float pm;
                unsigned pq;
                split(raw[q], pm, pq);
                if (loff[q] >= 0) tbl[buf * per_buf + loff[q]] = make_float2(pm, __uint_as_float(pq));
            }
        };
        const float2* tb_blank = tbl + d.blank * TABLE_PITCH;
        const float2* tb_label[PPT];
#pragma unroll
        for (int j = 0; j < PPT; ++j) tb_label[j] = tbl + cls[j] * TABLE_PITCH;
        // block tb: its scores are in table buffer tb & 1; the rows of block tb + 2 are requested into
        // `load`, the rows of block tb + 1 (requested a block ago) are in `next` and go into the other buffer
        auto block = [&](int tb, float (&next)[NQ], float (&load)[NQ]) {
            const int cur = (tb & 1) * per_buf;
            load_rows(tb + 2, load);
            {
                float2 nb = tb_blank[cur], nl[PPT];  // scores of the block's first frame
#pragma unroll
                for (int j = 0; j < PPT; ++j) nl[j] = tb_label[j][cur];
#pragma unroll
                for (int k = 0; k < BLK; ++k) {
                    const float pmb = nb.x;
                    const unsigned peb = __float_as_uint(nb.y);
                    float pml[PPT];
                    unsigned pel[PPT];
#pragma unroll
                    for (int j = 0; j < PPT; ++j) { pml[j] = nl[j].x; pel[j] = __float_as_uint(nl[j].y); }
                    if (k + 1 < BLK) {  // the next frame's scores, one step ahead
                        nb = tb_blank[cur + k + 1];
#pragma unroll
                        for (int j = 0; j < PPT; ++j) nl[j] = tb_label[j][cur + k + 1];
                    }
                    advance(rptr, pmb, peb, pml, pel);
                    rptr += rstep;
                }
            }
            // the rows in flight are not touched before the steps are done (tied to a value the last step
            // produced): their wait must not move ahead of the steps
#pragma unroll
            for (int q = 0; q < NQ; ++q) asm volatile("" : "+v"(next[q]), "+v"(vb[0]));
            boundary(tb, true, [&] { write_rows((tb + 1) & 1, next); });
        };
        load_rows(0, raw0);
        write_rows(0, raw0);
        load_rows(1, raw1);
        __syncthreads();
        for (int tb = 0; tb < tblocks; tb += 2) {
            block(tb, raw1, raw0);
            if (tb + 1 < tblocks) block(tb + 1, raw0, raw1);
        }
    } else {
        float sb[BLK], sl[PPT][BLK];
#pragma unroll
        for (int k = 0; k < BLK; ++k) {
            const int f = frame(k < T ? k : T - 1);
            sb[k] = lpb[(size_t)f * d.C + d.blank];
#pragma unroll
            for (int j = 0; j < PPT; ++j) sl[j][k] = lpb[(size_t)f * d.C + cls[j]];
        }
        const float* sptr = lpb + (size_t)frame(BLK - 1 < T ? BLK - 1 : T - 1) * d.C;
        for (int tb = 0; tb < tblocks; ++tb) {
#pragma unroll
            for (int k = 0; k < BLK; ++k) {
                const int step = tb * BLK + k;
                float pmb, pml[PPT];
                unsigned peb, pel[PPT];
                split(sb[k], pmb, peb);
#pragma unroll
                for (int j = 0; j < PPT; ++j) split(sl[j][k], pml[j], pel[j]);
                {   // refill this ring slot for step + BLK (past the end: the last frame again)
                    sptr += (step + BLK < T) ? sstep : 0;
                    sb[k] = sptr[d.blank];
#pragma unroll
                    for (int j = 0; j < PPT; ++j) sl[j][k] = sptr[cls[j]];
                }
                advance(rptr, pmb, peb, pml, pel);
                rptr += rstep;
            }
            boundary(tb, false, [] {});
        }
    }
    // log P = log( alpha_{T-1}(S-1) + alpha_{T-1}(S-2) ): blank of pair L, label of pair L-1, read back
    // from the stored lattice row of the last frame (written by this workgroup)
    if (dir == 0) {
        __syncthreads();
        if (tid == 0) {
            const float2* last = lat + (size_t)(T - 1) * d.Sp;
            const float fbv = __builtin_nontemporal_load(&last[2 * L].x);
            const int fbe = __float_as_int(__builtin_nontemporal_load(&last[2 * L].y));
            const float flv = L > 0 ? __builtin_nontemporal_load(&last[2 * L - 1].x) : 0.f;
            const int fle = L > 0 ? __float_as_int(__builtin_nontemporal_load(&last[2 * L - 1].y)) : 0;
            const int E = max(fbe, fle);
            const float sum = __builtin_amdgcn_ldexpf(fbv, fbe - E) + __builtin_amdgcn_ldexpf(flv, fle - E);
            const double lp2 = pair_log2(sum, E - EXP_BIAS + T * EXP_DRIFT);
            logp2_out[b] = lp2;
            loss[b] = sum > 0.f ? (float)(-lp2 * LN2) : INFINITY;
        }
    }
}

__device__ __forceinline__ float wsum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One wavefront per frame; a workgroup of 4 wavefronts takes `rows_per_wg` consecutive frames of one
// utterance.  The loads of a frame (both lattice rows, the gathered scores) are issued together,
// GRAD_UNROLL states per lane at a time.
constexpr int GRAD_UNROLL = 4;
__global__ __launch_bounds__(256) void ctc_grad(const float* __restrict__ lp, const int* __restrict__ targets,
                                                const int* __restrict__ in_len,
                                                const int* __restrict__ tgt_len,
                                                const float* __restrict__ loss,
                                                const double* __restrict__ logp2_in,
                                                const float2* __restrict__ alpha,
                                                const float2* __restrict__ beta,
                                                const int* __restrict__ sort_order,
                                                const int* __restrict__ sort_start, float* __restrict__ grad,
                                                CtcDims d, int rows_per_wg, int is_logits, float grad_scale)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int b = blockIdx.y, t0 = blockIdx.x * rows_per_wg;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* gb = grad + (size_t)b * d.Tp * d.C;
    const float ls = loss[b];
    const int T = crit_len(in_len[b], d.len_div);
    const bool live = isfinite(ls) && T > 0;  // NaN (invalid) and +inf (no alignment) give zero rows
    const int t_end = min(t0 + rows_per_wg, d.Tp);
    if (!live || t0 >= T) {
        for (int e = t0 * d.C + tid; e < t_end * d.C; e += 256) gb[e] = 0.f;
        return;
    }
    const int L = tgt_len[b], S = 2 * L + 1;
    int* lab = reinterpret_cast<int*>(smem_raw);       // [Lmax]
    int* order = lab + d.Lmax;                         // [Lmax] label positions sorted by (class, position)
    int* cstart = order + d.Lmax;                      // [C+1]
    float* ebuf = reinterpret_cast<float*>(cstart + d.C + 1) + (size_t)wave * d.Sp;  // [4][Sp]

    for (int i = tid; i < L; i += 256) {
        lab[i] = targets[(size_t)b * d.Lmax + i];
        order[i] = sort_order[(size_t)b * d.Lmax + i];
    }
    for (int c = tid; c <= d.C; c += 256) cstart[c] = sort_start[(size_t)b * (d.C + 1) + c];
    __syncthreads();

    const double logp2 = logp2_in[b];
    // log P split into an integer (taken off the integer exponents exactly) and a fraction
    const int iref = (int)floor(logp2);
    const float shift = (float)((double)iref - logp2);
    const float* lpb = lp + (size_t)b * d.Tp * d.C;
    for (int t = t0 + wave; t < t_end; t += 4) {
        float* grow = gb + (size_t)t * d.C;
        if (t >= T) {
            for (int c = lane; c < d.C; c += 64) grow[c] = 0.f;
            continue;
        }
        const float2* ar = alpha + ((size_t)b * d.rows + LAT_PAD + t) * d.Sp;
        const float2* br = beta + ((size_t)b * d.rows + LAT_PAD + t) * d.Sp;
        const float* lrow = lpb + (size_t)t * d.C;
        float z = 0.f, zb = 0.f;
        for (int s0 = lane; s0 < S; s0 += 64 * GRAD_UNROLL) {
            float2 a[GRAD_UNROLL], bt[GRAD_UNROLL];
            float sc[GRAD_UNROLL];
#pragma unroll
            for (int u = 0; u < GRAD_UNROLL; ++u) {
                const int s = min(s0 + 64 * u, S - 1);  // clamped lanes repeat a valid state and are dropped below
                const int c = (s & 1) ? lab[(s - 1) >> 1] : d.blank;
                a[u] = ar[s];
                bt[u] = br[S - 1 - s];  // beta rows are stored in reversed state order
                sc[u] = lrow[c];
            }
#pragma unroll
            for (int u = 0; u < GRAD_UNROLL; ++u) {
                const int s = s0 + 64 * u;
                float e = 0.f;
                // alpha and beta both carry the frame's own score: one of them is taken off again, split exactly
                // as the lattice kernel split it (integer part off the integer exponents, so nothing large cancels in fp32)
                if (a[u].x > 0.f && bt[u].x > 0.f) {
                    float fl, frac;
                    score_split(sc[u], fl, frac);
                    // both exponents carry the bias: taken off in wrap-around arithmetic
                    const int ex = (int)((unsigned)__float_as_int(a[u].y) + (unsigned)__float_as_int(bt[u].y) - 2u * (unsigned)EXP_BIAS +
                                        (unsigned)(T + 1) * (unsigned)EXP_DRIFT);
                    e = fast_exp2((fast_log2(a[u].x * bt[u].x) + (float)(ex - iref - (int)fl)) + (shift - frac));
                }
                if (s < S) {
                    ebuf[s] = e;
                    z += e;
                    if (!(s & 1)) zb += e;
                }
            }
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

size_t grad_lds_bytes(int Lmax, int C)
{
    return (size_t)4 * (2 * Lmax + C + 1) + (size_t)4 * 4 * (2 * Lmax + 4);
}

// Which ctc_lattice<PPT, NQ, BLK> variant a problem takes, and its launch shape.
// One lane per PPT (blank, label) pairs of the extended target: 64 lanes of the first wavefront, 64 - BLK of
// every further one.  The step is bound by instruction issue, so a wavefront wants a SIMD of its own: the
// smallest PPT that fits four wavefronts, with blocks of 16 frames if that fits (208 lanes) and of 12 (220
// lanes) otherwise; targets beyond 220 * 4 pairs take four pairs per lane on as many wavefronts as they need.
// NQ > 0 (score table in LDS): a block's class rows must fit 8 elements per thread and, in two buffers, 64 KB.
struct CtcLaunch { int ppt, blk, nt, nq; size_t lds; };
CtcLaunch ctc_launch_config(int C, int Lmax)
{
    const int pairs = Lmax + 1;
    int ppt = 4, blk = 16;
    for (int p = 1; p <= 4; p *= 2) {
        if (pairs <= (64 + 3 * 48) * p) { ppt = p; blk = 16; break; }
        if (pairs <= (64 + 3 * 52) * p) { ppt = p; blk = 12; break; }
    }
    const int own = 64 - blk, groups = (pairs + ppt - 1) / ppt;
    const int nt = 64 * (groups <= 64 ? 1 : 1 + (groups - 64 + own - 1) / own);
    const long long nel = (long long)blk * C;
    const size_t table_bytes = (size_t)2 * C * (blk + 1) * 8;
    const int nq = (nel <= 8LL * nt && table_bytes <= 64 * 1024) ? (nel <= 2LL * nt ? 2 : (nel <= 4LL * nt ? 4 : 8)) : 0;
    return CtcLaunch{ppt, blk, nt, nq, nq ? table_bytes : 0};
}

struct WsLayout { size_t lp, logp, order, cstart, alpha, beta, total; };
WsLayout ws_layout(int B, int Tp, int C, int Lmax)
{
    WsLayout w;
    size_t off = 0;
    w.lp = off; off += round_up((size_t)B * Tp * C * 4, 256);
    w.logp = off; off += round_up((size_t)B * 8, 256);
    w.order = off; off += round_up((size_t)B * Lmax * 4, 256);
    w.cstart = off; off += round_up((size_t)B * (C + 1) * 4, 256);
    const size_t lat = round_up((size_t)B * (Tp + 2 * LAT_PAD) * (2 * (size_t)Lmax + 4) * 8, 256);
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

extern "C" int w2l_ctc_launch_config(int C, int Lmax, int* pairs_per_lane, int* table_values_per_thread,
                                     int* frames_per_block, int* threads)
{
    if (!pairs_per_lane || !table_values_per_thread || !frames_per_block || !threads) return W2L_ERR_NULL;
    if (C <= 0 || C > 4096 || Lmax <= 0 || Lmax > 3000) return W2L_ERR_SHAPE;
    const CtcLaunch cfg = ctc_launch_config(C, Lmax);
    if (cfg.nt > 1024) return W2L_ERR_SHAPE;
    *pairs_per_lane = cfg.ppt;
    *table_values_per_thread = cfg.nq;
    *frames_per_block = cfg.blk;
    *threads = cfg.nt;
    return W2L_OK;
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

namespace {
int ctc_check_args(const float* input, const int* targets, const int* in_len, const int* tgt_len, const float* loss,
                   const float* grad, int B, int Tp, int C, int Lmax, int blank)
{
    if (!input || !targets || !in_len || !tgt_len || !loss || !grad) return W2L_ERR_NULL;
    if (B <= 0 || Tp <= 0 || Tp > MAX_FRAMES || C <= 0 || C > 4096 || Lmax <= 0 || Lmax > 3000 || blank < 0 ||
        blank >= C || B > 65535)
        return W2L_ERR_SHAPE;
    if (!aligned16(input) || !aligned16(targets) || !aligned16(grad)) return W2L_ERR_ALIGN;
    return W2L_OK;
}

// the three launches, arguments already checked; workspace: ws_layout().total bytes of device memory
int ctc_run(const float* input, int is_logits, const int* targets, const int* in_len, const int* tgt_len, float* loss,
            float* grad, int B, int Tp, int C, int Lmax, int blank, float grad_scale, void* workspace, void* stream,
            int len_div = 1)
{
    const WsLayout w = ws_layout(B, Tp, C, Lmax);
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
    float2* alpha = reinterpret_cast<float2*>(ws + w.alpha);
    float2* beta = reinterpret_cast<float2*>(ws + w.beta);
    int* sort_order = reinterpret_cast<int*>(ws + w.order);
    int* sort_start = reinterpret_cast<int*>(ws + w.cstart);
    CtcDims d{B, Tp, C, Lmax, blank, len_div, 2 * Lmax + 4, Tp + 2 * LAT_PAD};

    const size_t lds2 = grad_lds_bytes(Lmax, C);
    if (lds2 > 160 * 1024) return W2L_ERR_SHAPE;
    if (lds2 > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)ctc_grad, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }
    }
    const CtcLaunch cfg = ctc_launch_config(C, Lmax);
    if (cfg.nt > 1024) return W2L_ERR_SHAPE;
    const int ppt = cfg.ppt, blk = cfg.blk, nt = cfg.nt, nq = cfg.nq;
    const dim3 g1(3, B), b1(nt);  // alpha, beta, and the sort of the target for the gradient kernel
    const size_t lds1 = cfg.lds;
#define W2L_CTC_LAUNCH(P_, Q_, B_)                                                                                    \
    {                                                                                                                 \
        if (lds1 > 32 * 1024) {                                                                                       \
            hipError_t e = hipFuncSetAttribute((const void*)ctc_lattice<P_, Q_, B_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1); \
            if (e != hipSuccess) { note_hip_error(e); return W2L_ERR_LAUNCH; }                                        \
        }                                                                                                             \
        hipLaunchKernelGGL((ctc_lattice<P_, Q_, B_>), g1, b1, lds1, st, lp, targets, in_len, tgt_len, loss, logp, alpha, beta, sort_order, sort_start, d); \
    }
#define W2L_CTC_LAUNCH_Q(P_, B_)                                                                                      \
    {                                                                                                                 \
        if (nq == 2) W2L_CTC_LAUNCH(P_, 2, B_) else if (nq == 4) W2L_CTC_LAUNCH(P_, 4, B_)                             \
        else if (nq == 8) W2L_CTC_LAUNCH(P_, 8, B_) else W2L_CTC_LAUNCH(P_, 0, B_)                                    \
    }
#define W2L_CTC_LAUNCH_P(P_)                                                                                          \
    {                                                                                                                 \
        if (blk == 16) W2L_CTC_LAUNCH_Q(P_, 16) else W2L_CTC_LAUNCH_Q(P_, 12)                                          \
    }
    if (ppt == 1) W2L_CTC_LAUNCH_P(1) else if (ppt == 2) W2L_CTC_LAUNCH_P(2) else W2L_CTC_LAUNCH_P(4)
#undef W2L_CTC_LAUNCH_P
#undef W2L_CTC_LAUNCH_Q
#undef W2L_CTC_LAUNCH
    int rc = launch_status();
    if (rc) return rc;
    // frames per gradient workgroup: one per wavefront while the per-workgroup copy of the target's sort
    // (2 Lmax + C + 1 integers) is small beside the frames' own lattice rows, more otherwise
    const int rows_per_wg = (2 * Lmax + C + 1 <= 1024) ? 4 : 16;
    hipLaunchKernelGGL(ctc_grad, dim3((Tp + rows_per_wg - 1) / rows_per_wg, B), dim3(256), lds2, st, lp, targets,
                       in_len, tgt_len, loss, logp, alpha, beta, sort_order, sort_start, grad, d, rows_per_wg, is_logits,
                       grad_scale);
    return launch_status();
}
}  // namespace

namespace w2l {
// w2l_ctc_fwd_bwd for the train step: in_len counts input frames before the network's total stride `len_div`
int ctc_fwd_bwd_strided(const float* input, int is_logits, const int* targets, const int* in_len, const int* tgt_len,
                        float* loss, float* grad, int B, int Tp, int C, int Lmax, int blank, float grad_scale,
                        void* workspace, size_t ws_bytes, void* stream, int len_div)
{
    const int rc = ctc_check_args(input, targets, in_len, tgt_len, loss, grad, B, Tp, C, Lmax, blank);
    if (rc) return rc;
    if (len_div < 1) return W2L_ERR_SHAPE;
    if (!workspace || ws_bytes < ws_layout(B, Tp, C, Lmax).total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return W2L_ERR_WORKSPACE;
    return ctc_run(input, is_logits, targets, in_len, tgt_len, loss, grad, B, Tp, C, Lmax, blank, grad_scale, workspace,
                   stream, len_div);
}
}  // namespace w2l

extern "C" int w2l_ctc_fwd_bwd(const float* input, int is_logits, const int* targets, const int* in_len,
                               const int* tgt_len, float* loss, float* grad, int B, int Tp, int C, int Lmax,
                               int blank, float grad_scale, void* workspace, size_t ws_bytes, void* stream)
{
    const int rc = ctc_check_args(input, targets, in_len, tgt_len, loss, grad, B, Tp, C, Lmax, blank);
    if (rc) return rc;
    if (!workspace || ws_bytes < ws_layout(B, Tp, C, Lmax).total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return W2L_ERR_WORKSPACE;
    return ctc_run(input, is_logits, targets, in_len, tgt_len, loss, grad, B, Tp, C, Lmax, blank, grad_scale, workspace,
                   stream);
}

// ---- the same criterion for callers that cannot allocate device memory ---------------------
// The workspace is a file-scope device array.  In host code the array's name is only a handle:
// its device address comes from hipGetSymbolAddress, looked up once per device (each device
// holds its own copy of the array at its own address) and kept.
namespace {
static __device__ __align__(256) unsigned char scratch[W2L_CTC_NOALLOC_SCRATCH_BYTES];

struct ScratchAddr {
    void* ptr = nullptr;
    bool tried = false;
    hipError_t err = hipSuccess;
};
// device address of `scratch` on the current device; nullptr (and the HIP error noted) if the lookup failed
void* scratch_ptr()
{
    static std::mutex mu;
    static ScratchAddr per_device[64];
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64) {
        note_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    ScratchAddr& a = per_device[dev];
    if (!a.tried) {
        a.tried = true;
        void* p = nullptr;
        a.err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        a.ptr = (a.err == hipSuccess) ? p : nullptr;
    }
    if (!a.ptr) note_hip_error(a.err != hipSuccess ? a.err : hipErrorInvalidSymbol);
    return a.ptr;
}
}  // namespace

extern "C" int w2l_ctc_fwd_bwd_noalloc(const float* input, int is_logits, const int* targets, const int* in_len,
                                       const int* tgt_len, float* loss, float* grad, int B, int Tp, int C, int Lmax,
                                       int blank, float grad_scale, void* stream)
{
    const int rc = ctc_check_args(input, targets, in_len, tgt_len, loss, grad, B, Tp, C, Lmax, blank);
    if (rc) return rc;
    if (ws_layout(B, Tp, C, Lmax).total > (size_t)W2L_CTC_NOALLOC_SCRATCH_BYTES) return W2L_ERR_WORKSPACE;
    void* ws = scratch_ptr();
    if (!ws) return W2L_ERR_LAUNCH;
    // Every launch writes what it later reads (score rows, both lattices, the target's sort, log P):
    // nothing in the array has to start at zero, so what the previous call left there is harmless.
    return ctc_run(input, is_logits, targets, in_len, tgt_len, loss, grad, B, Tp, C, Lmax, blank, grad_scale, ws, stream);
}
